"""Full size, end to end against the oracle (Llama-3-8B shape, the benchmark's launch configuration).

1. The committed stream of speculative rounds, one of them with an injected tree that accepts drafted
   tokens, is fed teacher-forced through the oracle's target in ONE plain causal pass (mixed-precision
   model, float64 accumulation): every committed token must be the oracle's greedy token of its prefix,
   or lie within the stated end-to-end margin of it, and the library's logits of every committed
   position are compared with the oracle's.  The measured end-to-end error is printed.
2. One draft pass of depth 1 and one of depth 2 (fc + specialist layer + Head + log-softmax + top-k) are
   recomputed by the oracle from the library's own inputs: the library's feature of the last committed
   position, the specialist's own key/value cache, the tree's tokens.  With six specialists of one
   position each the depth-2 pass runs another specialist than the depth-1 pass, on a cache that was
   filled by catch-up rows.
"""
import time

import numpy as np
import pytest

from gpu_util import have_gpu, E2E_LOGIT_TOL

pytestmark = pytest.mark.gpu

if have_gpu():
    import torch
    import paper_2506_03566_amd as P
    from synth import get_config, make_prompt
    from synth.gpu import make_weights_on_device
    from oracle.model import Weights, decoder_layer, head, causal_allowed, specialist_index
    from oracle.numerics import decode_storage, round_storage, log_softmax



def _say(msg):
    print(msg, flush=True)


def test_committed_stream_teacher_forced_through_the_oracle():
    name = "c1_llama3_8b_3x2"
    cfg = get_config(name)
    t0 = time.time()
    _say(f"generating weights of {name} (host copy of the target kept)")
    dev, host = make_weights_on_device(cfg, keep_host=["embed", "lm_head", "final_norm", "layer"])
    ctx = P.Poss(cfg, dev)
    del dev
    torch.cuda.empty_cache()
    W = Weights(cfg, host, cache=False)
    prompt = make_prompt(cfg)
    n_p = len(prompt)
    first = ctx.prefill(prompt)
    # ---- the library's own vanilla continuation: what an injected tree has to contain to be accepted
    root = P.TreeArrays.from_lists([0], [-1])
    y = [first]
    for _ in range(4):
        ctx.verify_tree(root, want_argmax=False)
        y.append(ctx.accept_and_commit()[2][0])
    ctx.reset()
    assert ctx.prefill(prompt) == first
    # ---- rounds: one injected tree (chain of three true tokens, decoys beside and below it), then drafted trees
    logits = torch.zeros(cfg.total_tokens + 1, cfg.vocab, device="cuda")
    wrong = lambda tok: (tok + 7) % cfg.vocab
    tok = [0, wrong(y[1]), y[1], y[2], wrong(y[2]), y[3], wrong(y[4])]
    par = [-1, 0, 0, 2, 2, 3, 5]
    committed, rows = [], []           # committed tokens after x_P; the library's logits row each was chosen from
    g = ctx.verify_tree(P.TreeArrays.from_lists(tok, par), logits_out=logits)
    path, m, toks = ctx.accept_and_commit()
    _say(f"  injected tree: accepted {m} drafted tokens, path {path}")
    # the chain is the library's own vanilla continuation: it is accepted as far as the tree pass, which reads
    # the accepted rows' keys from scattered tree slots (another summation order), agrees with the vanilla
    # pass; every token committed here is judged against the oracle below, whatever the vanilla run chose
    assert m >= 1 and path == [0, 2, 3, 5][:m + 1] and toks[:m] == y[1:m + 1]
    rows.append(logits[path].cpu().numpy()); committed += toks
    ms = [m]
    for rnd in range(8):
        tr = ctx.draft_tree()
        ctx.verify_tree(None, logits_out=logits)
        path, m, toks = ctx.accept_and_commit()
        rows.append(logits[path].cpu().numpy()); committed += toks
        ms.append(m)
    lib_logits = np.concatenate(rows, axis=0).astype(np.float64)
    stream = list(prompt) + [first] + committed
    assert ctx.tokens() == stream and len(lib_logits) == len(committed)
    _say(f"  {len(ms)} rounds, accepted {ms}; {len(committed)} committed tokens after x_P; set-up {time.time() - t0:.1f} s")
    ctx.close()
    torch.cuda.empty_cache()
    # ---- the oracle: one causal pass over the stream without its last token, Head on the rows that chose a token
    t1 = time.time()
    n = len(stream) - 1
    # (target_rows' own loop over the layers, written out so that progress can be reported)
    h = decode_storage(host["embed"][np.asarray(stream[:n], dtype=np.int64)], cfg.dtype)
    z = np.zeros((0, cfg.n_kv_heads, cfg.head_dim))
    for l in range(cfg.n_layers):
        h, _, _ = decoder_layer(W, f"layer{l}.", cfg, h, np.arange(n), z, z, causal_allowed(0, n), cfg.dtype)
        if l % 4 == 3:
            _say(f"    oracle layer {l + 1}/{cfg.n_layers} at {time.time() - t1:.0f} s")
    feats = h
    o_logits = head(W, cfg, feats[n_p - 1:], cfg.dtype)                 # row j predicts stream[n_p + j]
    _say(f"  oracle: causal pass over {n} tokens in {time.time() - t1:.1f} s")
    assert int(np.argmax(o_logits[0])) == first or o_logits[0].max() - o_logits[0, first] <= 2 * E2E_LOGIT_TOL
    err = np.abs(o_logits[1:] - lib_logits).max(axis=1)
    near = 0
    for j, tok_j in enumerate(committed):
        row = o_logits[1 + j]
        if int(np.argmax(row)) != tok_j:
            near += 1
            gap = row.max() - row[tok_j]
            assert gap <= 2 * E2E_LOGIT_TOL, f"committed token {j} is {gap:.3f} below the oracle's greedy token"
    top2 = np.sort(o_logits, axis=1)[:, -2:]
    _say(f"  end-to-end max|dlogit| = {err.max():.4f} (median over positions {np.median(err):.4f}; logit std {o_logits.std():.2f}); "
         f"{near} of {len(committed)} committed tokens differ from the oracle's greedy token (smallest top-2 gap {np.min(top2[:, 1] - top2[:, 0]):.3f})")
    assert err.max() <= E2E_LOGIT_TOL


@pytest.mark.parametrize("name", ["c1_llama3_8b_3x2", "c2_llama3_8b_6x1"])
def test_full_size_draft_passes_sampled_against_the_oracle(name):
    cfg = get_config(name, n_prompt=200)
    tol = 2e-2
    s1, s2 = (specialist_index(d, cfg.positions_per_specialist, cfg.n_specialists) for d in (0, 1))
    _say(f"generating weights of {name} (host copy of specialists {sorted({s1, s2})}, embedding and Head kept)")
    dev, host = make_weights_on_device(cfg, keep_host=["embed", "lm_head", "final_norm"] + [f"spec{s}." for s in {s1, s2}])
    ctx = P.Poss(cfg, dev)
    del dev
    torch.cuda.empty_cache()
    W = Weights(cfg, host, cache=False)
    Q = lambda x: round_storage(x, cfg.dtype)
    emb = lambda tok: decode_storage(host["embed"][int(tok)], cfg.dtype)
    prompt = make_prompt(cfg)
    ctx.prefill(prompt)
    # one vanilla step hands over the library's own feature of the last committed position
    feats = torch.zeros(cfg.total_tokens + 1, cfg.d_model, device="cuda")
    ctx.verify_tree(P.TreeArrays.from_lists([0], [-1]), feat_out=feats)
    ctx.accept_and_commit()
    toks = ctx.tokens()
    t = len(toks) - 1                                   # x_t is the root; its pair [x_t ; f_{t-1}] has drafter index t-1
    f_prev = feats[0].cpu().numpy().astype(np.float64)
    d = ctx.draft_tree().as_dict()
    kids = lambda v: [i for i in range(1, d["n"]) if d["parent"][i] == v]

    def fc(s, token, feat):
        x = np.concatenate([emb(token), Q(feat)])
        return W(f"spec{s}.fc_w") @ x + W(f"spec{s}.fc_b")

    def check_children(v, lp, what):
        ch = kids(v)
        assert ch, what
        kth = np.sort(lp)[-cfg.top_k]
        e = 0.0
        for c in ch:
            step = float(d["score"][c]) - float(d["score"][v])
            e = max(e, abs(step - lp[d["token"][c]]))
            assert lp[d["token"][c]] >= kth - 2 * tol, (what, c)
        return e, len(ch)

    # ---- depth 1: specialist s1 on the root pair over its cache of committed pairs
    kc, vc = ctx.debug_read_kv(s1, 0, 0, t)
    h0 = fc(s1, toks[t], f_prev)[None]
    f_root, k_new, v_new = decoder_layer(W, f"spec{s1}.", cfg, h0, np.array([t - 1]), kc[:t - 1].astype(np.float64),
                                         vc[:t - 1].astype(np.float64), np.ones((1, t), bool), act=cfg.dtype)
    assert np.abs(kc[t - 1] - k_new[0]).max() <= tol and np.abs(vc[t - 1] - v_new[0]).max() <= tol
    lp1 = log_softmax(head(W, cfg, f_root, cfg.dtype))[0]
    e1, n1 = check_children(0, lp1, "depth 1")
    _say(f"  depth 1 (specialist {s1}): {n1} children, max|dlogp| = {e1:.3e}")
    assert e1 <= tol
    # ---- depth 2: specialist s2 on the pair [token(v) ; drafted feature of the root] of an expanded child v
    v = next(i for i in kids(0) if kids(i))
    kc2, vc2 = ctx.debug_read_kv(s2, 0, 0, t - 1)                       # committed pairs only: the root row is recomputed
    h2 = np.stack([fc(s2, toks[t], f_prev), fc(s2, d["token"][v], f_root[0])])
    allowed = np.ones((1, t + 1), bool)
    f_v, _, _ = decoder_layer(W, f"spec{s2}.", cfg, h2, np.array([t - 1, t]), kc2.astype(np.float64), vc2.astype(np.float64),
                              allowed, act=cfg.dtype, q_rows=[1])
    lp2 = log_softmax(head(W, cfg, f_v, cfg.dtype))[0]
    e2, n2 = check_children(v, lp2, "depth 2")
    _say(f"  depth 2 (specialist {s2}, node {v}): {n2} children, max|dlogp| = {e2:.3e}")
    assert e2 <= 2 * tol                                 # its input feature is the oracle's, not the library's: two passes of error
    ctx.close()
