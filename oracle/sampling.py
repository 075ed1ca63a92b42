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

Second reading, for the rejection-sampling rule proper ("sampled children"): the k children of an
expanded node are DRAWN from the drafter's distribution q = softmax(drafter logits / T), one after
the other without replacement; verification tests them in the order drawn: candidate c is accepted
with probability min(1, p(c) / q(c)); after a rejection the target distribution is replaced by the
normalised positive part of p - q and the drafter distribution by q without c, renormalised; if no
candidate is accepted the token is drawn from the last residual.  The accepted or drawn token is
distributed exactly as p (speculative sampling extended to several candidates drawn without
replacement, the recursive form of the rule cited in section 2.1), so the committed stream keeps the
target's distribution; here the speculative stream is NOT the vanilla stream of the same numbers,
only equal in distribution.  Uniform numbers are again inputs: one per draw, one per test, one per
residual draw.
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


# ------------------------------------------------------------------ sampled children, rejection rule
def draw_from(p, u, margins=None):
    """Inverse CDF in vocabulary order over a vector of non-negative masses (need not sum to 1): the first id
    whose cumulative mass exceeds u * total; never an id of zero mass.  `margins`, if a list, receives how far
    (as a fraction of the total) u * total is from the nearer end of the chosen id's interval."""
    p = np.asarray(p, dtype=np.float64)
    cdf = np.cumsum(p)
    target = u * cdf[-1]
    i = int(np.searchsorted(cdf, target, side="right"))
    if i >= len(p) or p[i] <= 0.0:                    # rounding pushed the target past the total
        i = int(np.nonzero(p > 0)[0][-1])
    if margins is not None:
        margins.append(float(min(target - (cdf[i - 1] if i > 0 else 0.0), cdf[i] - target) / cdf[-1]))
    return i


def sample_children(logits, temperature, us, margins=None):
    """len(us) distinct ids drawn one after the other from softmax(logits / T), each from what the earlier draws
    left (inverse CDF in vocabulary order, us[i] for draw i).  Returns (ids in draw order, q, the full
    distribution they were drawn from)."""
    q = softmax_t(logits, temperature)
    left = q.copy()
    ids = []
    for u in us:
        c = draw_from(left, u, margins)
        ids.append(c)
        left[c] = 0.0
    return ids, q


def reject_or_accept(p, q, candidates, us, margins=None):
    """The candidates (distinct ids, in the order they were drawn from q without replacement) are tested one
    after the other with us[i]: candidate c passes if us[i] < min(1, p(c) / q(c)) for the CURRENT p and q.
    After a rejection p becomes the normalised positive part of p - q and q loses c and is renormalised.
    Returns (index of the accepted candidate or -1, the p to draw from if none was accepted)."""
    p = np.asarray(p, dtype=np.float64).copy()
    q = np.asarray(q, dtype=np.float64).copy()
    for i, c in enumerate(candidates):
        a = min(1.0, p[c] / q[c])
        if margins is not None and a < 1.0:
            margins.append(abs(float(us[i]) - a))
        if us[i] < a:
            return i, None
        p = np.maximum(p - q, 0.0)
        p /= p.sum()
        q[c] = 0.0
        q /= q.sum()
    return -1, p
