"""Temperature sampling of the target and its use in tree verification (oracle; test
infrastructure only).

The paper evaluates at temperature 0 and 1 (section 4.1, Tables 1 and 2) and says no more about
verification at temperature 1 than that a rejection-sampling step keeps the output distribution
that of the target (section 2.1).  Reading taken here: the draft tree is built exactly as at
temperature 0 (its k children per node are a fixed candidate set, not samples), and at every
node the walk visits the target's next token is DRAWN from softmax(logits / T); the walk
descends if a child carries that token, otherwise the drawn token is the bonus token.  Every
committed token is then an exact sample of the target given its prefix, whatever the tree
holds, which is the lossless property; a child c of node v is accepted with probability
p(c | v).  Drawing "the token, then look for it among the children" has the same distribution
as testing the children one after the other with renormalisation in between.

Random numbers are inputs: one uniform number in [0, 1) per sequence position, U[p] deciding the
token at position p.  The draw is by inverse CDF in vocabulary order, so a run is reproducible
and the speculative stream can be compared token for token with vanilla sampling that uses the
same numbers.
"""
import numpy as np

from .model import target_full


def softmax_t(logits, temperature):
    """softmax(logits / temperature) in float64."""
    z = np.asarray(logits, dtype=np.float64) / float(temperature)
    z = z - z.max()
    e = np.exp(z)
    return e / e.sum()


def sample_token(logits, temperature, u):
    """Inverse CDF in vocabulary order: the first id whose cumulative probability exceeds u."""
    cdf = np.cumsum(softmax_t(logits, temperature))
    i = int(np.searchsorted(cdf, u, side="right"))
    return min(i, len(cdf) - 1)


def cdf_interval(logits, temperature, token):
    """[lo, hi): the values of u for which sample_token returns `token`."""
    cdf = np.cumsum(softmax_t(logits, temperature))
    return (float(cdf[token - 1]) if token > 0 else 0.0), float(cdf[token])


def sample_decode(W, cfg, prompt, n_new, temperature, U, act=None):
    """Vanilla autoregressive sampling with full recompute: the token at position p is drawn with
    U[p].  The plain definition the speculative path at temperature > 0 is checked against."""
    seq = [int(t) for t in prompt]
    for _ in range(n_new):
        _, logits = target_full(W, cfg, seq, act)
        seq.append(sample_token(logits[-1], temperature, U[len(seq)]))
    return seq
