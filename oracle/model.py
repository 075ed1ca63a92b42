"""Target model rows and one position-specialist pass (oracle; test infrastructure only).

Target: a Llama-style decoder whose last-layer hidden state (before the final
norm) is the "feature" f^(T) of section 2.2, with Head(f) = lm_head . RMSNorm_final(f)
(Eq. 6).  Specialist: fc over [token embedding ; feature] followed by one
decoder layer of the target's shape, sharing the target's embedding and Head
(section 2.2, Eq. 1/2; section 3.2, Eq. 7/9; section 3.3 "same structure").
"""
import numpy as np

from .numerics import (decode_storage, round_storage, rmsnorm, rope, attention, silu)


class Weights:
    """float64 view of a dict of storage-format tensors (decoded on demand)."""

    def __init__(self, cfg, storage, cache=True):
        self.cfg, self.storage, self._cache, self._keep = cfg, storage, {}, cache

    def __call__(self, name):
        if name in self._cache:
            return self._cache[name]
        w = decode_storage(self.storage[name], self.cfg.dtype)
        if self._keep:
            self._cache[name] = w
        return w


def decoder_layer(W, prefix, cfg, h, pos, k_ctx, v_ctx, allowed, act=None, q_rows=None):
    """One pre-norm decoder layer on `rows` new positions.

    h: [rows, d] residual stream; pos: [rows]; k_ctx/v_ctx: [ctx, Hkv, dh] keys and
    values of earlier positions (already rotated); allowed: [len(q_rows), ctx + rows]
    visibility.  All `rows` produce keys/values; only q_rows (default: all) are
    carried through attention and the MLP.  Returns (h_out[q_rows], k_new, v_new).
    """
    Q = lambda x: round_storage(x, act)
    rows = h.shape[0]
    hq, hkv, dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    u = Q(rmsnorm(h, W(prefix + "attn_norm"), cfg.rms_eps))
    k = Q(rope((u @ W(prefix + "wk").T).reshape(rows, hkv, dh), pos, cfg.rope_theta))
    v = Q((u @ W(prefix + "wv").T).reshape(rows, hkv, dh))
    if q_rows is None:
        q_rows = np.arange(rows)
    q_rows = np.asarray(q_rows, dtype=np.int64)
    nq = len(q_rows)
    q = Q(rope((u[q_rows] @ W(prefix + "wq").T).reshape(nq, hq, dh), np.asarray(pos)[q_rows],
               cfg.rope_theta))
    keys = np.concatenate([k_ctx, k], axis=0) if len(k_ctx) else k
    vals = np.concatenate([v_ctx, v], axis=0) if len(v_ctx) else v
    o = Q(attention(q, keys, vals, allowed).reshape(nq, hq * dh))
    h1 = h[q_rows] + o @ W(prefix + "wo").T
    u2 = Q(rmsnorm(h1, W(prefix + "mlp_norm"), cfg.rms_eps))
    a = Q(silu(u2 @ W(prefix + "w_gate").T) * (u2 @ W(prefix + "w_up").T))
    h2 = h1 + a @ W(prefix + "w_down").T
    return h2, k, v


def empty_kv(cfg):
    z = np.zeros((0, cfg.n_kv_heads, cfg.head_dim))
    return [(z, z) for _ in range(cfg.n_layers)]


def target_rows(W, cfg, tokens, pos, kv_ctx, allowed, act=None, taps=None):
    """Target forward over `rows` tokens given per-layer context keys/values.

    Returns (features [rows, d], [(k_new, v_new)] per layer).  `taps`, if a list,
    receives the residual stream entering each layer and the final one.
    """
    h = W("embed")[np.asarray(tokens, dtype=np.int64)]
    new_kv = []
    for l in range(cfg.n_layers):
        if taps is not None:
            taps.append(h.copy())
        kc, vc = kv_ctx[l]
        h, k, v = decoder_layer(W, f"layer{l}.", cfg, h, pos, kc, vc, allowed, act)
        new_kv.append((k, v))
    if taps is not None:
        taps.append(h.copy())
    return h, new_kv


def head(W, cfg, feats, act=None):
    """Head(f) = lm_head . RMSNorm_final(f): logits [rows, vocab]  (Eq. 6)."""
    u = round_storage(rmsnorm(feats, W("final_norm"), cfg.rms_eps), act)
    return u @ W("lm_head").T


def causal_allowed(n_ctx, rows):
    """Row i sees all n_ctx context keys and new keys 0..i."""
    a = np.ones((rows, n_ctx + rows), dtype=bool)
    a[:, n_ctx:] = np.tril(np.ones((rows, rows), dtype=bool))
    return a


def target_full(W, cfg, tokens, act=None):
    """Plain causal forward over a whole sequence: (features, logits)."""
    n = len(tokens)
    f, _ = target_rows(W, cfg, tokens, np.arange(n), empty_kv(cfg), causal_allowed(0, n), act)
    return f, head(W, cfg, f, act)


def specialist_index(position, n, n_specialists):
    """0-based specialist for 0-based draft position i: ceil((i+1)/n), Eq. 7;
    positions beyond S*n stay with the last specialist (a reading: the paper runs
    depths 8-9 on every variant without saying which layer serves them)."""
    return min(position // n, n_specialists - 1)


def specialist_pass(W, cfg, s, tokens, feats, pos, allowed, q_rows, act=None):
    """Specialist s applied to a sequence of [x ; f] pairs (Eq. 2 / Eq. 9 right-hand side).

    tokens [n], feats [n, d] (the feature paired with each token: that of the
    previous sequence position), pos [n].  Every row contributes a key/value computed
    with THIS specialist's weights (no cache is shared between specialists, section
    3.3); q_rows are the rows whose output features are wanted; allowed
    [len(q_rows), n].  Returns drafted features [len(q_rows), d].
    """
    Q = lambda x: round_storage(x, act)
    p = f"spec{s}."
    x = np.concatenate([W("embed")[np.asarray(tokens, dtype=np.int64)], Q(np.asarray(feats))], axis=1)
    h0 = x @ W(p + "fc_w").T
    if cfg.fc_bias:                      # the draft model's fc layer has a bias in the paper's configuration (appendix B)
        h0 = h0 + W(p + "fc_b")
    z = np.zeros((0, cfg.n_kv_heads, cfg.head_dim))
    out, _, _ = decoder_layer(W, p, cfg, h0, np.asarray(pos), z, z, allowed, act, q_rows=q_rows)
    return out


def specialist_kv(W, cfg, s, tokens, feats, pos, act=None):
    """Keys (rotated) and values specialist s holds for a sequence of [x ; f] pairs: what its own,
    unshared cache must contain (section 3.3).  Returns (k, v) of shape [n, Hkv, dh]."""
    Q = lambda x: round_storage(x, act)
    p = f"spec{s}."
    n = len(tokens)
    x = np.concatenate([W("embed")[np.asarray(tokens, dtype=np.int64)], Q(np.asarray(feats))], axis=1)
    h0 = x @ W(p + "fc_w").T
    if cfg.fc_bias:                      # the draft model's fc layer has a bias in the paper's configuration (appendix B)
        h0 = h0 + W(p + "fc_b")
    u = Q(rmsnorm(h0, W(p + "attn_norm"), cfg.rms_eps))
    k = Q(rope((u @ W(p + "wk").T).reshape(n, cfg.n_kv_heads, cfg.head_dim), np.asarray(pos), cfg.rope_theta))
    v = Q((u @ W(p + "wv").T).reshape(n, cfg.n_kv_heads, cfg.head_dim))
    return k, v
