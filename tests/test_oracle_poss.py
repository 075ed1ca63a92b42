"""The oracle's speculative round against the plain definition (vanilla greedy decoding),
Eq. 6, and the special cases where the outcome is known in advance."""
import numpy as np
import pytest

from synth import get_config, make_weights, make_prompt
from synth.gen import to_storage
from oracle.model import (Weights, target_full, target_rows, empty_kv, head, specialist_pass, specialist_index,
                          causal_allowed)
from oracle.numerics import log_softmax
from oracle.greedy import greedy_decode
from oracle.poss import PossOracle, topk_lowest_id
from oracle.tree import accept_bruteforce, Tree


def _setup(name, **kw):
    cfg = get_config(name, **kw)
    return cfg, Weights(cfg, make_weights(cfg))


@pytest.mark.parametrize("name,n_prompt,n_new", [("c0_tiny_f32", 64, 32), ("t_tiny_f32_6x1", 33, 12)])
def test_lossless_against_vanilla_greedy(name, n_prompt, n_new):
    cfg, W = _setup(name)
    prompt = make_prompt(cfg, n=n_prompt)
    ref = greedy_decode(W, cfg, prompt, n_new)
    o = PossOracle(W, cfg)
    rec = []
    out = o.generate(prompt, n_new, record=rec)
    assert out == ref
    # every round: walk == brute force, accepted set is a root path, bookkeeping adds up
    for r in rec:
        tr = r["tree"]
        assert accept_bruteforce(tr.token, tr.parent, r["g"])[0] == r["path"]
        assert tr.n == cfg.total_tokens + 1 and max(tr.depth) <= cfg.depth
    assert o.stats.rounds == len(rec)
    assert o.stats.committed == len(o.tokens) - n_prompt - 1
    assert len(o.feats) == o.t == len(o.kv[0][0])


def test_lossless_with_injected_trees_of_every_accept_length():
    """Trees that contain the true continuation to depth m must accept exactly m."""
    cfg, W = _setup("c0_tiny_f32")
    prompt = make_prompt(cfg, n=20)
    L = cfg.depth
    ref = greedy_decode(W, cfg, prompt, L + 3)
    y = ref[len(prompt):]                      # y[0] is the token prefill emits
    for m in range(L + 1):
        o = PossOracle(W, cfg)
        assert o.prefill(prompt) == y[0]
        # chain of the m true tokens, a wrong token after it, plus a decoy branch at the root
        wrong = lambda tok: (tok + 1) % cfg.vocab
        token, parent = [y[0]], [-1]
        token.append((y[1] + 2) % cfg.vocab); parent.append(0)
        for j in range(1, m + 1):
            token.append(y[j]); parent.append(0 if j == 1 else len(token) - 2)
        last = len(token) - 1 if m else 0
        token.append(wrong(y[m + 1])); parent.append(last)
        g, logits, F = o.verify_tree(Tree(token, parent))
        path, mm, bonus = o.accept_and_commit()
        assert mm == m and bonus == y[m + 1]
        assert [token[p] for p in path[1:]] == y[1:m + 1]
        assert o.tokens == list(prompt) + y[:m + 2]
        # Eq. 6: Head of the target feature of a committed position is the target's own
        # next-token distribution: compare with a plain causal pass over the committed text
        f_full, logits_full = target_full(W, cfg, o.tokens[:-1])
        assert np.allclose(np.stack(o.feats), f_full, rtol=1e-9, atol=1e-11)
        assert np.allclose(logits[path], logits_full[len(prompt):], rtol=1e-9, atol=1e-11)
        # and the committed keys / values are those of that plain pass (the accepted rows, which are
        # not the first rows of the tree: node 1 is the decoy)
        n_c = len(o.tokens) - 1
        _, kv_full = target_rows(W, cfg, o.tokens[:-1], np.arange(n_c), empty_kv(cfg), causal_allowed(0, n_c))
        for (k_o, v_o), (k_f, v_f) in zip(o.kv, kv_full):
            assert k_o.shape == k_f.shape and np.allclose(k_o, k_f, rtol=1e-9, atol=1e-11)
            assert np.allclose(v_o, v_f, rtol=1e-9, atol=1e-11)


def test_depth_one_uses_target_features_only():
    """Eq. 2 at k = 1 is Eq. 1: the first draft distribution is Head of specialist 1 applied to
    the committed [x_j ; f^(T)_{j-1}] pairs, and the root's children are its top-k."""
    cfg, W = _setup("c0_tiny_f32")
    prompt = make_prompt(cfg, n=17)
    o = PossOracle(W, cfg)
    o.prefill(prompt)
    tree = o.draft_tree()
    t = o.t
    out = specialist_pass(W, cfg, 0, o.tokens[1:t + 1], np.stack(o.feats[:t]), np.arange(t),
                          np.ones((1, t), bool), [t - 1])
    logits = head(W, cfg, out)[0]
    want = topk_lowest_id(logits.astype(np.float32), cfg.top_k).tolist()
    tb = o.last["builder"]
    assert tb.token[:cfg.top_k] == want
    kids = [tree.token[i] for i in range(1, tree.n) if tree.parent[i] == 0]
    assert set(kids) <= set(want)


@pytest.mark.parametrize("name", ["c0_tiny_f32", "t_tiny_f32_6x1"])
def test_a_root_path_of_the_tree_is_the_plain_pair_sequence(name):
    """Eq. 2 / Eq. 9 on one path, written out without any tree bookkeeping: the committed pairs
    [x_j ; f_{j-1}] followed by the drafted pairs [token(v_i) ; drafted feature of v_{i-1}] of a
    root path form an ordinary sequence - consecutive positions, plain causal attention - and the
    specialist of depth d, applied to that sequence, gives at its last row the distribution the
    children of v_{d-1} were scored with.  Pins what the batched tree drafting must reproduce with
    its masks and position ids (a drafted row sits right behind the committed pairs plus its
    ancestors, and sees nothing else)."""
    cfg, W = _setup(name)
    o = PossOracle(W, cfg)
    o.prefill(make_prompt(cfg, n=19))
    tree = o.draft_tree()
    t = o.t
    deepest = max(range(tree.n), key=lambda i: (tree.depth[i], tree.score[i]))
    assert tree.depth[deepest] >= 3
    path = [deepest]
    while path[-1] != 0:
        path.append(tree.parent[path[-1]])
    path.reverse()
    tok, feat = list(o.tokens[1:t + 1]), list(o.feats[:t])
    for d, node in enumerate(path[1:], start=1):
        s = specialist_index(d - 1, cfg.positions_per_specialist, cfg.n_specialists)
        rows = len(tok)
        out = specialist_pass(W, cfg, s, tok, np.stack(feat), np.arange(rows), causal_allowed(0, rows)[-1:], [rows - 1])
        lp = log_softmax(head(W, cfg, out))[0]
        step = float(tree.score[node]) - float(tree.score[tree.parent[node]])
        assert abs(step - lp[tree.token[node]]) < 1e-4, (d, step, lp[tree.token[node]])
        tok.append(tree.token[node])
        feat.append(out[0])


def test_a_drafter_that_passes_the_feature_through_predicts_the_token_it_is_paired_with():
    """Closed form for the pairing of Eq. 1: the root row is [x_t ; f_{t-1}], and f_{t-1} is the
    feature the target chose x_t from.  A drafter whose fc keeps only the feature half and whose
    layer adds nothing hands Head that very feature, so its best guess for the token after x_t is
    x_t again, its k guesses are the target's top-k at position t-1, and (the drafted feature never
    changing) every expanded node gets the same k children."""
    cfg = get_config("c0_tiny_f32")
    st = make_weights(cfg)
    d = cfg.d_model
    for s in range(cfg.n_specialists):
        fc = np.zeros((d, 2 * d)); fc[:, d:] = np.eye(d)            # the feature half of [x ; f]
        st[f"spec{s}.fc_w"] = to_storage(fc, cfg.dtype)
        st[f"spec{s}.fc_b"] = to_storage(np.zeros(d), cfg.dtype)
        for nm in ("wo", "w_down"):
            st[f"spec{s}.{nm}"] = to_storage(np.zeros(st[f"spec{s}.{nm}"].shape), cfg.dtype)
    W = Weights(cfg, st)
    o = PossOracle(W, cfg)
    o.prefill(make_prompt(cfg, n=23))
    o.draft_tree()
    t, k = o.t, cfg.top_k
    want = topk_lowest_id(head(W, cfg, o.feats[t - 1][None])[0].astype(np.float32), k).tolist()
    assert want[0] == o.tokens[t]
    tb = o.last["builder"]
    assert tb.token[:k] == want
    assert all(tb.token[i:i + k] == want for i in range(0, len(tb.token), k))


def _perfect_drafter_weights(cfg):
    """Target reduced to a per-token map and every specialist made a copy of it.  The head is
    scaled up so that the next-token distributions are peaked: then the greedy chain has the
    highest cumulative score at every depth and cannot fall out of the width-k frontier."""
    from synth.gen import to_float64
    st = make_weights(cfg)
    st["lm_head"] = to_storage(100.0 * to_float64(st["lm_head"], cfg.dtype), cfg.dtype)
    z = lambda a: to_storage(np.zeros(a.shape), cfg.dtype)
    d = cfg.d_model
    for l in range(cfg.n_layers):
        st[f"layer{l}.wo"] = z(st[f"layer{l}.wo"])                  # attention adds nothing
        if l > 0:
            st[f"layer{l}.w_down"] = z(st[f"layer{l}.w_down"])      # later layers are the identity
    for s in range(cfg.n_specialists):
        fc = np.zeros((d, 2 * d)); fc[:, :d] = np.eye(d)            # picks the embedding half of [x ; f]
        st[f"spec{s}.fc_w"] = to_storage(fc, cfg.dtype)
        st[f"spec{s}.fc_b"] = z(st[f"spec{s}.fc_b"])
        for nm in ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down"):
            st[f"spec{s}.{nm}"] = st[f"layer0.{nm}"].copy()
    return st


def test_perfect_drafter_accepts_full_depth():
    cfg = get_config("c0_tiny_f32")
    W = Weights(cfg, _perfect_drafter_weights(cfg))
    prompt = make_prompt(cfg, n=16)
    o = PossOracle(W, cfg)
    rec = []
    out = o.generate(prompt, 3 * (cfg.depth + 1), record=rec)
    assert out == greedy_decode(W, cfg, prompt, 3 * (cfg.depth + 1))
    assert [r["m"] for r in rec] == [cfg.depth] * 3
    assert o.stats.tau_acc == cfg.depth and o.stats.tau_gen == cfg.depth + 1
    assert all(o.stats.pos_acc(i) == 1.0 for i in range(2, cfg.depth + 1))
    assert o.stats.p_accept(1) == 1.0


def test_random_drafter_accepts_almost_nothing():
    cfg, W = _setup("c0_tiny_f32")
    o = PossOracle(W, cfg)
    o.generate(make_prompt(cfg, n=32), 12)
    assert o.stats.tau_acc < 0.5 and 1.0 <= o.stats.tau_gen < 1.5


def test_identical_specialists_equal_single_draft_model():
    """A single draft model is the limit n -> infinity (appendix D): S copies of one specialist
    must draft exactly what S = 1 drafts."""
    cfg3 = get_config("c0_tiny_f32")
    st = make_weights(cfg3)
    for s in (1, 2):
        for k in list(st):
            if k.startswith("spec0."):
                st[k.replace("spec0.", f"spec{s}.")] = st[k].copy()
    cfg1 = cfg3.with_(n_specialists=1, positions_per_specialist=cfg3.depth)
    prompt = make_prompt(cfg3, n=25)
    a, b = PossOracle(Weights(cfg3, st), cfg3), PossOracle(Weights(cfg1, st), cfg1)
    a.prefill(prompt); b.prefill(prompt)
    ta, tb = a.draft_tree(), b.draft_tree()
    assert ta.token == tb.token and ta.parent == tb.parent
    assert np.array_equal(np.array(ta.score), np.array(tb.score))
    # and distinct specialists really are dispatched by depth: different weights, different tree
    c = PossOracle(Weights(cfg3, make_weights(cfg3)), cfg3)
    c.prefill(prompt)
    tc = c.draft_tree()
    assert [tc.token[i] for i in range(1, tc.n) if tc.depth[i] == 1] == \
           [ta.token[i] for i in range(1, ta.n) if ta.depth[i] == 1]      # specialist 1 is shared
    assert tc.token != ta.token                                            # deeper levels differ


def test_mixed_precision_mode_is_lossless_too():
    cfg = get_config("c0_tiny_f32", dtype=1)
    W = Weights(cfg, make_weights(cfg))
    prompt = make_prompt(cfg, n=24)
    ref = greedy_decode(W, cfg, prompt, 10, act=1)
    assert PossOracle(W, cfg, act=1).generate(prompt, 10) == ref
    # rounding the activations moves the logits by about the bf16 step, not more
    _, exact = target_full(W, cfg, prompt)
    _, mixed = target_full(W, cfg, prompt, act=1)
    assert 1e-5 < np.abs(exact - mixed).max() < 2e-2


def test_specialist_kv_of_a_copied_target_layer_is_that_layer_s_cache():
    """Pin of specialist_kv that does not go through the specialist code: a specialist whose fc keeps the
    embedding half of [x ; f] and whose layer is a copy of target layer 0 (with a bias of zero) turns the
    pairs [x_j ; .] into target layer 0's own keys and values of the tokens x_j, provided it is given the
    target's positions.  The target side is pinned against Hugging Face's Llama.  A swapped wk / wv, a
    missing norm or rotation, or the feature half leaking in fail this."""
    from oracle.model import specialist_kv
    cfg = get_config("c0_tiny_f32")
    W = Weights(cfg, _perfect_drafter_weights(cfg))
    tokens = make_prompt(cfg, n=18)
    n = len(tokens)
    feats, kv = target_rows(W, cfg, tokens, np.arange(n), empty_kv(cfg), causal_allowed(0, n))
    junk = np.random.default_rng(3).normal(size=(n - 1, cfg.d_model))        # the feature half must not matter
    for s in range(cfg.n_specialists):
        k, v = specialist_kv(W, cfg, s, tokens[1:], junk, np.arange(1, n))
        assert np.allclose(k, kv[0][0][1:], rtol=1e-10, atol=1e-12), s
        assert np.allclose(v, kv[0][1][1:], rtol=1e-10, atol=1e-12), s
    assert np.abs(kv[0][0][1:] - kv[0][1][1:]).max() > 1e-3                      # keys and values do differ


def test_specialist_kv_is_what_the_pass_attends_to():
    """With ordinary random specialists (fc bias included): giving the decoder layer specialist_kv's keys
    and values as context for the last pair reproduces specialist_pass over the whole pair sequence."""
    from oracle.model import specialist_kv, decoder_layer
    cfg, W = _setup("t_tiny_f32_6x1")
    assert cfg.fc_bias and np.abs(W("spec2.fc_b")).max() > 0
    o = PossOracle(W, cfg)
    o.prefill(make_prompt(cfg, n=21))
    t = o.t
    toks, feats, pos = o.tokens[1:t + 1], np.stack(o.feats[:t]), np.arange(t)
    for s in (0, 2, 5):
        want = specialist_pass(W, cfg, s, toks, feats, pos, np.ones((1, t), bool), [t - 1])
        k, v = specialist_kv(W, cfg, s, toks, feats, pos)
        x_last = np.concatenate([W("embed")[toks[-1]], feats[-1]])
        h_last = (W(f"spec{s}.fc_w") @ x_last + W(f"spec{s}.fc_b"))[None]
        got, k_last, v_last = decoder_layer(W, f"spec{s}.", cfg, h_last, pos[-1:], k[:-1], v[:-1], np.ones((1, t), bool))
        assert np.allclose(got, want, rtol=1e-9, atol=1e-11), s
        assert np.allclose(k_last[0], k[-1], atol=1e-12) and np.allclose(v_last[0], v[-1], atol=1e-12)
        # the context matters: the same row alone gives another feature
        alone, _, _ = decoder_layer(W, f"spec{s}.", cfg, h_last, pos[-1:], k[:0], v[:0], np.ones((1, 1), bool))
        assert np.abs(alone - want).max() > 1e-4


def test_fc_bias_alone_drives_the_draft_when_everything_else_is_switched_off():
    """Closed form for the bias of the fc layer (appendix B: the draft model's configuration has one).
    With fc_w = 0 and the layer's two output projections zero, every drafted feature is the bias itself,
    so every expanded node's children are the top-k of Head(bias) with the log-probabilities of
    log_softmax(Head(bias)); without the bias the feature would be zero and the children ids 0..k-1."""
    cfg = get_config("c0_tiny_f32")
    st = make_weights(cfg)
    rng = np.random.default_rng(11)
    d, k = cfg.d_model, cfg.top_k
    for s in range(cfg.n_specialists):
        st[f"spec{s}.fc_w"] = to_storage(np.zeros((d, 2 * d)), cfg.dtype)
        st[f"spec{s}.fc_b"] = to_storage(rng.normal(size=d) * (1 + s), cfg.dtype)      # a different bias per specialist
        for nm in ("wo", "w_down"):
            st[f"spec{s}.{nm}"] = to_storage(np.zeros(st[f"spec{s}.{nm}"].shape), cfg.dtype)
    W = Weights(cfg, st)
    o = PossOracle(W, cfg)
    o.prefill(make_prompt(cfg, n=14))
    o.draft_tree()
    tb = o.last["builder"]
    pool_depth = [1] * k + [dd for dd in range(2, cfg.depth + 1) for _ in range(k * k)]
    for i0 in range(0, len(tb.token), k):
        s = specialist_index(pool_depth[i0] - 1, cfg.positions_per_specialist, cfg.n_specialists)
        logits = head(W, cfg, W(f"spec{s}.fc_b")[None])[0]
        want = topk_lowest_id(logits.astype(np.float32), k)
        assert tb.token[i0:i0 + k] == want.tolist(), (i0, s)
        lp = log_softmax(logits)[want]
        parent_score = 0.0 if tb.parent[i0] < 0 else float(tb.score[tb.parent[i0]])
        assert np.allclose(np.array(tb.score[i0:i0 + k], dtype=np.float64) - parent_score, lp, atol=1e-4)
    assert tb.token[:k] != list(range(k))


def test_score_tree_and_specialist_kv_agree_with_the_draft():
    """Helpers used by the GPU lock-step tests: re-scoring the oracle's own tree reproduces its
    scores; specialist_kv's keys are rotated by the position they are given."""
    from oracle.model import specialist_kv
    cfg, W = _setup("t_tiny_f32_6x1")
    o = PossOracle(W, cfg)
    o.prefill(make_prompt(cfg, n=21))
    tree = o.draft_tree()
    score, rows = o.score_tree(tree)
    assert np.abs(score - np.array(tree.score, dtype=np.float64)).max() < 1e-5
    assert 0 in rows and abs(np.exp(rows[0]).sum() - 1.0) < 1e-12
    t = o.t
    k, v = specialist_kv(W, cfg, 0, o.tokens[1:t + 1], np.stack(o.feats[:t]), np.arange(t))
    assert k.shape == (t, cfg.n_kv_heads, cfg.head_dim) and v.shape == k.shape
    # keys are rotated: un-rotating position p by -p must give the position-0 key of the same input
    from oracle.numerics import rope
    k0, _ = specialist_kv(W, cfg, 0, o.tokens[1:t + 1], np.stack(o.feats[:t]), np.zeros(t, dtype=int))
    assert np.allclose(rope(k, -np.arange(t), cfg.rope_theta), k0, atol=1e-12)
