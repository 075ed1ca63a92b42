"""Vanilla autoregressive greedy decoding of the target (oracle; test infrastructure only).

Under greedy verification speculative decoding must reproduce exactly this
stream (section 2.1: draft tokens are kept only where they agree with the
target).  It is the plain definition the speculative path is checked against,
so it is written without any cache: every new token re-runs the target over
the whole sequence.
"""
import numpy as np

from .model import target_full


def argmax_lowest(row):
    """Index of the maximum; the lowest index wins ties."""
    return int(np.argmax(row))       # numpy returns the first occurrence


def greedy_decode(W, cfg, prompt, n_new, act=None, margins=None):
    """Return prompt + n_new greedy tokens.  `margins` (list) receives top1-top2 logit gaps."""
    seq = [int(t) for t in prompt]
    for _ in range(n_new):
        _, logits = target_full(W, cfg, seq, act)
        last = logits[-1]
        nxt = argmax_lowest(last)
        if margins is not None:
            top2 = np.partition(last, -2)[-2:]
            margins.append(float(top2[1] - top2[0]))
        seq.append(nxt)
    return seq
