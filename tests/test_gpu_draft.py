"""Draft path of the HIP library against the oracle: per-specialist caches and catch-up passes,
perfect-drafter and identical-specialist special cases, lock-step rounds in 16-bit storage."""
import numpy as np
import pytest

from gpu_util import have_gpu, Pair, tol_for, tree_from_gpu

pytestmark = pytest.mark.gpu

if have_gpu():
    import torch
    import paper_2506_03566_amd as P
    from synth import get_config, make_prompt, make_weights
    from synth.gen import to_float64, to_storage
    from oracle.tree import Tree, accept_walk, ancestor_masks, validate_tree
    from oracle.model import specialist_kv, specialist_index


def _say(msg):
    print(msg, flush=True)


def _perfect_drafter_storage(cfg):
    """Same construction as the oracle's CPU test: the target is a per-token map, every specialist
    a copy of it, the head sharpened so that the greedy chain always stays in the frontier."""
    st = make_weights(cfg)
    z = lambda a: to_storage(np.zeros(a.shape), cfg.dtype)
    d = cfg.d_model
    st["lm_head"] = to_storage(100.0 * to_float64(st["lm_head"], cfg.dtype), cfg.dtype)
    for l in range(cfg.n_layers):
        st[f"layer{l}.wo"] = z(st[f"layer{l}.wo"])
        if l > 0:
            st[f"layer{l}.w_down"] = z(st[f"layer{l}.w_down"])
    for s in range(cfg.n_specialists):
        fc = np.zeros((d, 2 * d)); fc[:, :d] = np.eye(d)
        st[f"spec{s}.fc_w"] = to_storage(fc, cfg.dtype)
        st[f"spec{s}.fc_b"] = z(st[f"spec{s}.fc_b"])
        for nm in ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down"):
            st[f"spec{s}.{nm}"] = st[f"layer0.{nm}"].copy()
    return st


@pytest.mark.parametrize("name", ["c0_tiny_f32", "t_tiny_f32_6x1"])
def test_perfect_drafter_accepts_full_depth_and_keeps_caches_right(name):
    cfg = get_config(name)
    pair = Pair(name, storage=_perfect_drafter_storage(cfg))
    ctx, o = pair.ctx, pair.oracle()
    _say(f"perfect drafter {name}")
    prompt = make_prompt(cfg, n=16)
    n_new = 3 * (cfg.depth + 1)
    want = o.generate(prompt, n_new)
    ctx.prefill(prompt)
    ms = []
    for _ in range(3):
        ctx.draft_tree()
        ctx.verify_tree()
        path, m, toks = ctx.accept_and_commit()
        ms.append(m)
        assert len(path) == m + 1
    assert ms == [cfg.depth] * 3                       # every round accepts the full depth
    assert ctx.tokens()[:len(want)] == want
    st = ctx.stats()
    assert st.rounds == 3 and st.committed_tokens == 3 * (cfg.depth + 1)
    assert list(st.c)[1:cfg.depth + 1] == [3] * cfg.depth      # pos-acc_i = c[i]/c[i-1] = 1, tau_acc = L
    # Each round commits depth+1 pairs, so every specialist has to catch up on that many rows (plus
    # the drafted rows of earlier depths) before it runs.  After one more draft, every specialist's
    # own cache must hold exactly the keys/values the oracle computes with that specialist's weights.
    ctx.draft_tree()
    toks = ctx.tokens()
    t = len(toks) - 1
    feats, _ = __import__("oracle.model", fromlist=["target_full"]).target_full(pair.W, cfg, toks[:t])
    for s in range(cfg.n_specialists):
        k, v = specialist_kv(pair.W, cfg, s, toks[1:t + 1], feats, np.arange(t))
        gk, gv = ctx.debug_read_kv(s, 0, 0, t)
        assert np.abs(gk - k).max() < 1e-4 and np.abs(gv - v).max() < 1e-4, f"specialist {s}"
    pair.close()


def test_identical_specialists_equal_single_draft_model_on_gpu():
    """S copies of one specialist must draft bit-for-bit what S = 1 drafts (a single draft model
    is the limit n -> infinity, appendix D): a direct test of the catch-up passes."""
    cfg3 = get_config("c0_tiny_f32")
    st = _perfect_drafter_storage(cfg3)                # long accepted paths => many catch-up rows
    rng = np.random.default_rng(5)
    # disturb the copies a little (still identical to each other): acceptance lengths then vary
    noise = to_storage(rng.normal(size=st["spec0.w_down"].shape) * 0.004, cfg3.dtype)
    for s in range(cfg3.n_specialists):
        st[f"spec{s}.w_down"] = (st[f"spec{s}.w_down"] + noise).astype(st["spec0.w_down"].dtype)
    cfg1 = cfg3.with_(n_specialists=1, positions_per_specialist=cfg3.depth)
    a = Pair("c0_tiny_f32", storage=st)
    b = Pair("c0_tiny_f32", storage=st, n_specialists=1, positions_per_specialist=cfg3.depth)
    prompt = make_prompt(cfg3, n=30)
    assert a.ctx.prefill(prompt) == b.ctx.prefill(prompt)
    ms = []
    for rnd in range(5):
        ta, tb = a.ctx.draft_tree().as_dict(), b.ctx.draft_tree().as_dict()
        assert ta["token"] == tb["token"] and ta["parent"] == tb["parent"], f"round {rnd}"
        assert np.array_equal(ta["score"], tb["score"])
        ga, gb = a.ctx.verify_tree(), b.ctx.verify_tree()
        assert np.array_equal(ga, gb)
        ra, rb = a.ctx.accept_and_commit(), b.ctx.accept_and_commit()
        assert ra == rb
        ms.append(ra[1])
    _say(f"accepted per round: {ms}")
    assert len(set(ms)) > 1 or ms[0] > 0               # the comparison covered non-trivial commits
    a.close(); b.close()


@pytest.mark.parametrize("name", ["t_mid_bf16", "t_mid_f16"])
def test_lockstep_rounds_16bit(name):
    """16-bit storage: free-running streams fork at near-ties, so every call is checked on the
    library's own state.  Tree: structure exact (parents, depths, positions, masks), scores
    within tolerance of the oracle's re-scoring, every kept node at least as good as the oracle's
    worst kept node up to tolerance.  Verification: greedy tokens equal where the oracle's top-2
    gap exceeds twice the tolerance; walk equals brute force on the library's own argmax."""
    pair = Pair(name)
    cfg, ctx = pair.cfg, pair.ctx
    tol = tol_for(cfg)
    o = pair.oracle()
    prompt = make_prompt(cfg)
    first = ctx.prefill(prompt)
    ofirst = o.prefill(prompt)
    if first != ofirst:
        o.tokens[-1] = first
    near_ties = 0
    for rnd in range(4):
        tr = ctx.draft_tree()
        otree, d = tree_from_gpu(tr)
        t = o.t
        assert d["n"] == cfg.total_tokens + 1 and validate_tree(d["token"], d["parent"])
        otree.finish(t)
        assert d["depth"] == otree.depth and d["pos"] == otree.pos and d["mask"] == otree.mask
        assert d["token"][0] == o.tokens[-1]
        score, rows = o.score_tree(otree)
        serr = np.abs(score - d["score"].astype(np.float64)).max()
        _say(f"  round {rnd}: max|dscore| {serr:.2e}")
        assert serr <= 2 * tol                            # a score sums up to `depth` log-probabilities; measured 1e-2
        own = o.draft_tree()                              # the oracle's own tree on the same state
        worst_kept = min(float(s) for s in own.score[1:])
        assert score[1:].min() >= worst_kept - 2 * tol
        # children of an expanded node are among the oracle's best-k of that node, up to tolerance
        for v, lp in rows.items():
            kth = np.sort(lp)[-cfg.top_k]
            for c in range(1, d["n"]):
                if d["parent"][c] == v:
                    assert lp[d["token"][c]] >= kth - 2 * tol
        logits = torch.zeros(d["n"], cfg.vocab, device="cuda")
        g = ctx.verify_tree(None, logits_out=logits)[:d["n"]]
        og, ologits, _ = o.verify_tree(otree)
        err = np.abs(logits.cpu().numpy() - ologits).max()
        assert err <= tol, err
        for i in range(d["n"]):
            top2 = np.partition(ologits[i], -2)[-2:]
            if top2[1] - top2[0] > 2 * tol:
                assert g[i] == og[i]
            elif g[i] != og[i]:
                near_ties += 1
                assert ologits[i].max() - ologits[i, g[i]] <= 2 * tol
        path, m, toks = ctx.accept_and_commit()
        wpath, wbonus = accept_walk(d["token"], d["parent"], g.tolist())
        assert path == wpath and toks[-1] == wbonus and toks[:-1] == [d["token"][p] for p in path[1:]]
        o.accept_and_commit(path=path, bonus=toks[-1])    # adopt the library's decision
        assert ctx.tokens() == o.tokens
    _say(f"  near-ties resolved differently: {near_ties}")
    pair.close()


def test_verify_after_caller_trees_then_draft_catches_up():
    """Rounds driven by caller-supplied trees leave the specialists behind by many pairs; the
    next draft must first bring their caches up to date (chunked catch-up)."""
    pair = Pair("c0_tiny_f32")
    cfg, ctx = pair.cfg, pair.ctx
    o = pair.oracle()
    prompt = make_prompt(cfg, n=24)
    ctx.prefill(prompt); o.prefill(prompt)
    for _ in range(cfg.depth + 4):                       # more root-only rounds than one pass can absorb
        ctx.verify_tree(P.TreeArrays.from_lists([0], [-1]))
        path, m, toks = ctx.accept_and_commit()
        o.verify_tree(Tree([o.tokens[-1]], [-1]))
        o.accept_and_commit()
    assert ctx.tokens() == o.tokens
    d = ctx.draft_tree().as_dict()
    ot = o.draft_tree()
    if min(o.margins) > 2e-5:
        assert d["token"] == ot.token and d["parent"] == ot.parent
    assert np.abs(d["score"] - np.array(ot.score, dtype=np.float32)).max() < 1e-4 or min(o.margins) <= 2e-5
    pair.close()


def test_all_equal_logits_pick_lowest_ids():
    """A zero LM head makes every logit equal: top-k must return tokens 0..k-1 with log-probability
    -log(V) at every expanded node (ties to the lower id, then to the earlier candidate), exactly
    the oracle's tree.  On the GPU this is the case where the threshold selection finds more
    candidates than it keeps and falls back to selection in rounds."""
    cfg = get_config("c0_tiny_f32")
    st = make_weights(cfg)
    st["lm_head"] = to_storage(np.zeros(st["lm_head"].shape), cfg.dtype)
    pair = Pair("c0_tiny_f32", storage=st)
    ctx, o = pair.ctx, pair.oracle()
    prompt = make_prompt(cfg, n=12)
    assert ctx.prefill(prompt) == o.prefill(prompt) == 0          # argmax of equal logits: id 0
    d = ctx.draft_tree().as_dict()
    ot = o.draft_tree()
    assert d["token"] == ot.token and d["parent"] == ot.parent
    k = cfg.top_k
    for i in range(1, d["n"]):
        assert d["token"][i] < k
        assert abs(d["score"][i] + d["depth"][i] * np.log(cfg.vocab)) < 1e-4
    g = ctx.verify_tree()[:d["n"]]
    assert list(g) == [0] * d["n"]
    path, m, toks = ctx.accept_and_commit()
    og, _, _ = o.verify_tree(ot)
    assert (path, m, toks[-1]) == o.accept_and_commit()
    pair.close()


def test_duplicated_head_rows_order_equal_logits_by_id():
    """LM-head rows 2i and 2i+1 made identical: their logits are bitwise equal, so wherever the
    odd token appears among a node's children the even one must be there too, ranked just before
    it (same parent, the even one earlier among the siblings)."""
    cfg = get_config("c0_tiny_f32")
    st = make_weights(cfg)
    head = st["lm_head"].copy()
    head[1::2] = head[0::2]
    st["lm_head"] = head
    pair = Pair("c0_tiny_f32", storage=st)
    ctx = pair.ctx
    ctx.prefill(make_prompt(cfg, n=20))
    pairs_seen = 0
    for _ in range(3):
        d = ctx.draft_tree().as_dict()
        kids = {}
        for i in range(1, d["n"]):
            kids.setdefault(d["parent"][i], []).append((i, d["token"][i], d["score"][i]))
        for p, ch in kids.items():
            toks = {t: (i, s) for i, t, s in ch}
            for t, (i, s) in toks.items():
                if t % 2 == 1 and t - 1 in toks:
                    pairs_seen += 1
                    assert toks[t - 1][0] < i and toks[t - 1][1] == s     # earlier node, bit-equal score
        ctx.verify_tree()
        ctx.accept_and_commit()
    assert pairs_seen > 0
    pair.close()


def test_fc_bias_flag_off_ignores_the_bias_tensor():
    """fc_bias = 0: both sides must leave the bias tensor out even when it holds values."""
    cfg = get_config("c0_tiny_f32", fc_bias=0)
    st = make_weights(get_config("c0_tiny_f32"))             # generated WITH non-zero biases
    assert np.abs(to_float64(st["spec0.fc_b"], cfg.dtype)).max() > 0
    pair = Pair("c0_tiny_f32", storage=st, fc_bias=0)
    with_bias = Pair("c0_tiny_f32", storage=st)
    prompt = make_prompt(cfg, n=18)
    o = pair.oracle()
    assert pair.ctx.prefill(prompt) == o.prefill(prompt) == with_bias.ctx.prefill(prompt)
    d, ot = pair.ctx.draft_tree().as_dict(), o.draft_tree()
    db = with_bias.ctx.draft_tree().as_dict()
    assert np.abs(d["score"] - np.array(ot.score, dtype=np.float32)).max() < 1e-4
    if min(o.margins) > 2e-5:
        assert d["token"] == ot.token and d["parent"] == ot.parent
    assert not np.array_equal(d["score"], db["score"])        # the bias does change the draft
    pair.close(); with_bias.close()


@pytest.mark.parametrize("name", ["c0_tiny_f32", "t_mid_bf16"])
def test_fc_bias_alone_drives_the_draft_when_everything_else_is_switched_off(name):
    """Closed form for the fc bias (the oracle's CPU pin of the same name): fc_w = 0 and zero output
    projections make every drafted feature the specialist's bias, so a node of depth d carries a token of
    the top-k of Head(bias of the specialist serving depth d) and adds that token's log-probability."""
    from oracle.model import head
    from oracle.numerics import log_softmax
    cfg = get_config(name)
    st = make_weights(cfg)
    rng = np.random.default_rng(11)
    d_model, k = cfg.d_model, cfg.top_k
    for s in range(cfg.n_specialists):
        st[f"spec{s}.fc_w"] = to_storage(np.zeros((d_model, 2 * d_model)), cfg.dtype)
        st[f"spec{s}.fc_b"] = to_storage(rng.normal(size=d_model) * (1 + s), cfg.dtype)
        for nm in ("wo", "w_down"):
            st[f"spec{s}.{nm}"] = to_storage(np.zeros(st[f"spec{s}.{nm}"].shape), cfg.dtype)
    pair = Pair(name, storage=st)
    tol = tol_for(cfg)
    pair.ctx.prefill(make_prompt(cfg, n=14))
    tr = pair.ctx.draft_tree().as_dict()
    lp_of = {}
    for s in range(cfg.n_specialists):
        logits = head(pair.W, cfg, pair.W(f"spec{s}.fc_b")[None], pair.act)[0]
        lp_of[s] = (log_softmax(logits), np.sort(logits)[-k])
    assert tr["n"] == cfg.total_tokens + 1
    for i in range(1, tr["n"]):
        s = specialist_index(tr["depth"][i] - 1, cfg.positions_per_specialist, cfg.n_specialists)
        lp, kth = lp_of[s]
        step = float(tr["score"][i]) - float(tr["score"][tr["parent"][i]])
        assert abs(step - lp[tr["token"][i]]) <= 2 * tol, (i, step, lp[tr["token"][i]])
        assert lp[tr["token"][i]] >= np.sort(lp)[-k] - 2 * tol
    pair.close()


@pytest.mark.parametrize("over,n_prompt", [
    (dict(top_k=1, depth=1, total_tokens=1), 1),               # smallest everything: one-token prompt, one draft token
    (dict(top_k=1, depth=6, total_tokens=6), 2),               # a chain
    (dict(top_k=2, depth=2, total_tokens=6), 5),               # the tree keeps the whole candidate pool
    (dict(top_k=16, depth=5, total_tokens=127), 40),           # 128 rows in verification, widest top-k, pool of 1040
    (dict(top_k=6, depth=16, total_tokens=100, n_specialists=3, positions_per_specialist=2), 33),   # deepest tree; depth > S*n
])
def test_degenerate_and_maximal_tree_shapes(over, n_prompt):
    """Smallest and largest tree parameters the library accepts, in float32, lock-step with the
    oracle (large candidate pools always hold a pair of scores closer than float32 resolves):
    structure exact as a function of the library's parents, scores within 1e-4 of the oracle's
    re-scoring, identical tree whenever every decision margin is clear, kept set as good as the
    oracle's otherwise; greedy tokens equal where the margin is clear; walk and stream equal."""
    pair = Pair("c0_tiny_f32", **over)
    cfg, ctx, o = pair.cfg, pair.ctx, pair.oracle()
    prompt = make_prompt(cfg, n=n_prompt)
    assert ctx.prefill(prompt) == o.prefill(prompt)
    identical = 0
    for rnd in range(3):
        otree, d = tree_from_gpu(ctx.draft_tree())
        t = o.t
        assert d["n"] == cfg.total_tokens + 1 and validate_tree(d["token"], d["parent"])
        otree.finish(t)
        assert d["depth"] == otree.depth and d["pos"] == otree.pos and d["mask"] == otree.mask
        score, _ = o.score_tree(otree)
        assert np.abs(score - d["score"].astype(np.float64)).max() < 1e-4
        n_marg = len(o.margins)
        own = o.draft_tree()
        if min(o.margins[n_marg:]) > 2e-5:
            assert d["token"] == own.token and d["parent"] == own.parent, f"round {rnd}"
            identical += 1
        else:
            assert score[1:].min() >= min(float(x) for x in own.score[1:]) - 1e-4
        g = ctx.verify_tree()[:d["n"]]
        og, ologits, _ = o.verify_tree(otree)
        for i in range(otree.n):
            top2 = np.partition(ologits[i], -2)[-2:]
            if top2[1] - top2[0] > 2e-5:
                assert g[i] == og[i]
        path, m, toks = ctx.accept_and_commit()
        wpath, wbonus = accept_walk(d["token"], d["parent"], g.tolist())
        assert path == wpath and toks[-1] == wbonus
        o.accept_and_commit(path=path, bonus=toks[-1])
        assert ctx.tokens() == o.tokens
    _say(f"  {over}: {identical}/3 rounds with an identical tree")
    pair.close()


def _imperfect_drafter_storage(cfg, noise):
    """The perfect drafter with the feature half of every fc matrix filled with noise: drafts are
    right often but not always, so rounds accept anything between nothing and the full depth."""
    st = _perfect_drafter_storage(cfg)
    rng = np.random.default_rng(77)
    d = cfg.d_model
    for s in range(cfg.n_specialists):
        fc = to_float64(st[f"spec{s}.fc_w"], cfg.dtype)
        fc[:, d:] = noise * rng.normal(size=(d, d)) / np.sqrt(d)
        st[f"spec{s}.fc_w"] = to_storage(fc, cfg.dtype)
    return st


@pytest.mark.parametrize("name", ["c0_tiny_f32", "t_tiny_f32_6x1"])
def test_long_run_with_mixed_acceptance_is_lossless(name):
    """Float32 storage, a drafter that is right only some of the time, many rounds: accepted lengths
    of every size occur, the caches are compacted and caught up in every combination, pages are
    crossed - and the committed stream stays exactly the stream of one-token-at-a-time decoding
    through the same library (section 2.1: verification does not change the target's output)."""
    cfg = get_config(name)
    pair = Pair(name, storage=_imperfect_drafter_storage(cfg, 0.1))
    ctx = pair.ctx
    prompt = make_prompt(cfg, n=21)
    ctx.prefill(prompt)
    ms = []
    while len(ctx.tokens()) < len(prompt) + 260:
        ctx.draft_tree(want_tree=False)
        ctx.verify_tree(want_argmax=False)
        _, m, _ = ctx.accept_and_commit()
        ms.append(m)
    spec = ctx.tokens()
    _say(f"  {name}: {len(ms)} rounds, accepted lengths {sorted(set(ms))}, mean {np.mean(ms):.2f}")
    assert len(set(ms)) >= 4 and 0 in ms and max(ms) >= cfg.depth - 1      # the drafter is neither useless nor perfect
    st = ctx.stats()
    assert st.rounds == len(ms) and st.committed_tokens == sum(ms) + len(ms)
    c = list(st.c)
    assert c[1:cfg.depth + 1] == [sum(1 for m in ms if m >= i) for i in range(1, cfg.depth + 1)]   # Eq. 3 counters
    ctx.reset()
    ctx.prefill(prompt)
    root = P.TreeArrays.from_lists([0], [-1])
    while len(ctx.tokens()) < len(spec):
        ctx.verify_tree(root, want_argmax=False)
        ctx.accept_and_commit()
    assert ctx.tokens() == spec
    # and the oracle, free-running, agrees on the first stretch (float32 against float64: until a near-tie)
    want = pair.oracle().generate(prompt, 40)
    assert spec[:len(want)] == want
    pair.close()
