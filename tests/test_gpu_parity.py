"""Parity of the HIP library (through the C ABI) against the CPU oracle.

Bars: bit-exact for committed tokens, accepted-path indices, tree structure, position ids and
masks; max-abs error 1e-4 (float32 storage) / 2e-2 (16-bit storage) for logits.
"""
import numpy as np
import pytest

from gpu_util import have_gpu, Pair, tol_for, tree_from_gpu

pytestmark = pytest.mark.gpu

if have_gpu():
    import torch
    import paper_2506_03566_amd as P
    from synth import get_config, make_prompt, make_weights
    from synth.gen import to_float64, to_storage
    from synth.gpu import to_device
    from oracle.tree import Tree, TreeBuilder, accept_bruteforce, ancestor_masks
    from oracle.poss import PossOracle
    from oracle.model import Weights


def _say(msg):
    print(msg, flush=True)


# --------------------------------------------------------------------------- GEMM
@pytest.mark.parametrize("dtype,M,N,K,twg", [
    (1, 61, 1000, 1408, 0), (2, 10, 520, 512, 0), (1, 81, 256, 768, 0), (1, 128, 384, 256, 0),
    (0, 25, 688, 256, 0), (1, 1, 128, 256, 0), (2, 33, 128, 1024, 0), (1, 61, 6144, 4096, 512),
    (1, 16, 4096, 14336, 1024), (2, 96, 2000, 5120, 300), (1, 17, 130, 8, 0),
    (1, 129, 384, 512, 0), (2, 200, 1000, 1408, 0), (1, 256, 6144, 4096, 512), (1, 244, 4096, 14336, 1024),
    (2, 177, 130, 8, 0), (0, 150, 688, 256, 0)])
def test_gemm_against_float64_matmul(dtype, M, N, K, twg):
    _say(f"gemm dtype={dtype} M={M} N={N} K={K} twg={twg}")
    rng = np.random.default_rng(M * 7 + N)
    x = to_storage(rng.normal(size=(M, K)), dtype)
    w = to_storage(rng.normal(size=(N, K)) * 0.02, dtype)
    y, _ = P.debug_gemm(dtype, to_device(x, dtype), to_device(w, dtype), twg)
    ref = to_float64(x, dtype) @ to_float64(w, dtype).T
    err = np.abs(y.cpu().numpy().astype(np.float64) - ref).max()
    assert err < 2e-5 * np.sqrt(K / 256.0), err          # float32 accumulation of exact products


@pytest.mark.parametrize("dtype,N,K,twg", [(1, 1000, 1408, 0), (2, 4096, 4096, 256), (1, 512, 14336, 0)])
def test_a_gemm_row_does_not_depend_on_the_rows_around_it(dtype, N, K, twg):
    """The same activation row in launches of 1, 10, 61, 122, 183 and 244 rows (every row-tile instantiation, the staged
    chunks of 8 and of 4 k-steps): bit for bit the same result, which is what lets sequences share a launch."""
    rng = np.random.default_rng(N + K)
    x = to_storage(rng.normal(size=(244, K)), dtype)
    w = to_device(to_storage(rng.normal(size=(N, K)) * 0.02, dtype), dtype)
    full, _ = P.debug_gemm(dtype, to_device(x, dtype), w, twg)
    full = full.cpu().numpy()
    for M in (1, 10, 61, 122, 183):
        _say(f"gemm rows dtype={dtype} M={M} N={N} K={K}")
        y, _ = P.debug_gemm(dtype, to_device(x[:M], dtype), w, twg)
        assert np.array_equal(y.cpu().numpy(), full[:M]), M


# --------------------------------------------------------------------------- whole path, float32, strict
def _screened_prompt(pair, n_prompt, n_new, min_margin, max_tries=40):
    """First prompt seed on which every decision the oracle takes (greedy argmax, top-k order,
    frontier, rerank) has a gap of at least min_margin, so that float32 and float64 must agree."""
    for seed in range(max_tries):
        prompt = make_prompt(pair.cfg, n=n_prompt, seed=1000 + seed)
        o = pair.oracle()
        rec = []
        out = o.generate(prompt, n_new, record=rec)
        if min(o.margins) >= min_margin:
            return prompt, o, rec, out
    pytest.fail("no prompt seed with clear decision margins found")


@pytest.mark.parametrize("name", ["c0_tiny_f32", "t_tiny_f32_6x1"])
def test_float32_free_running_is_bit_identical(name):
    pair = Pair(name)
    cfg = pair.cfg
    _say(f"free-running {name}")
    prompt, o, rec, want = _screened_prompt(pair, cfg.n_prompt, cfg.n_new, 2e-5)
    ctx = pair.ctx
    first = ctx.prefill(prompt)
    assert first == want[len(prompt)]
    for i, r in enumerate(rec):
        tr = ctx.draft_tree()
        d = tr.as_dict()
        ot = r["tree"]
        assert d["token"] == ot.token and d["parent"] == ot.parent, f"round {i}"
        assert d["depth"] == ot.depth and d["pos"] == ot.pos and d["mask"] == ot.mask
        assert np.abs(d["score"] - np.array(ot.score, dtype=np.float32)).max() < 1e-4
        g = ctx.verify_tree()
        assert g[:tr.n].tolist() == r["g"]
        path, m, toks = ctx.accept_and_commit()
        assert path == r["path"] and m == r["m"] and toks[-1] == r["bonus"]
    assert ctx.tokens()[:len(want)] == want
    st = ctx.stats()
    assert st.rounds == o.stats.rounds and st.committed_tokens == o.stats.committed
    assert list(st.c)[:cfg.depth + 1] == o.stats.c
    pair.close()


# --------------------------------------------------------------------------- per-call numerics
def _verify_both(pair, prompt, tree_lists=None):
    cfg, ctx = pair.cfg, pair.ctx
    o = pair.oracle()
    o.prefill(prompt)
    first = ctx.prefill(prompt)
    if tree_lists is None:
        tr = ctx.draft_tree()
        otree, _ = tree_from_gpu(tr)
        gtree = None
    else:
        otree = Tree(*tree_lists)
        gtree = P.TreeArrays.from_lists(*tree_lists)
        tr = gtree
    n = otree.n
    logits = torch.zeros(n, cfg.vocab, device="cuda")
    feats = torch.zeros(n, cfg.d_model, device="cuda")
    g = ctx.verify_tree(gtree, logits_out=logits, feat_out=feats)
    og, ologits, ofeats = o.verify_tree(otree)
    return o, first, tr, g[:n], logits.cpu().numpy().astype(np.float64), feats.cpu().numpy().astype(np.float64), og, ologits, ofeats


@pytest.mark.parametrize("name", ["c0_tiny_f32", "t_tiny_f32_6x1", "t_mid_bf16", "t_mid_f16"])
def test_verify_logits_features_and_cache(name):
    pair = Pair(name)
    cfg = pair.cfg
    _say(f"verify numerics {name}")
    prompt = make_prompt(cfg)
    o, first, tr, g, logits, feats, og, ologits, ofeats = _verify_both(pair, prompt)
    assert first == o.tokens[-1] or name.startswith("t_mid")     # 16-bit: near-ties may differ
    tol = tol_for(cfg)
    err = np.abs(logits - ologits).max()
    _say(f"  max|dlogit| = {err:.3e} (tol {tol})  max|dfeat| = {np.abs(feats - ofeats).max():.3e}")
    assert err <= tol
    # features are the residual stream itself (no final norm): the logit bound, scaled by the norm's factor, the root
    # mean square of the row (1 .. 3 at these shapes)
    assert np.abs(feats - ofeats).max() <= tol * max(1.0, np.sqrt((ofeats ** 2).mean(axis=1)).max())
    # greedy tokens agree wherever the oracle's top-2 gap exceeds twice the tolerance
    for i in range(len(og)):
        top2 = np.partition(ologits[i], -2)[-2:]
        if top2[1] - top2[0] > 2 * tol:
            assert g[i] == og[i]
    # target cache rows written by prefill, and the tree rows of this pass, layer 0 and last
    P_ = len(prompt)
    new_kv = o.last["new_kv"]
    for layer in (0, cfg.n_layers - 1):
        k, v = pair.ctx.debug_read_kv(-1, layer, 0, P_)
        assert np.abs(k - o.kv[layer][0]).max() <= tol and np.abs(v - o.kv[layer][1]).max() <= tol
        k, v = pair.ctx.debug_read_kv(-1, layer, P_, len(og))
        assert np.abs(k - new_kv[layer][0]).max() <= tol and np.abs(v - new_kv[layer][1]).max() <= tol
    pair.close()


@pytest.mark.parametrize("gemm_wgs,attn_keys", [(32, 64), (1024, 64), (64, 1024), (2048, 96)])
def test_verify_parity_with_other_launch_shapes(gemm_wgs, attn_keys):
    """Other K-split counts (down to unsplit, up to the cap of two chunks per split) and other
    attention splits (many small ones with a merge, a single unsplit walk): same tolerance."""
    pair = Pair("t_mid_bf16")
    cfg = pair.cfg
    pair.ctx.set_tuning(gemm_wgs, attn_keys)
    o, first, tr, g, logits, feats, og, ologits, ofeats = _verify_both(pair, make_prompt(cfg))
    tol = tol_for(cfg)
    err = np.abs(logits - ologits).max()
    _say(f"  target workgroups {gemm_wgs}, keys per split {attn_keys}: max|dlogit| = {err:.3e}")
    assert err <= tol
    pair.close()


@pytest.mark.parametrize("name,layers,attn_keys", [("t_mid_bf16", 1, 0), ("t_mid_bf16", 1, 1024), ("t_mid_bf16", 3, 0),
                                                   ("t_mid_bf16", 3, 1024), ("t_mid_f16", 2, 0), ("t_mid_f16", 2, 64)])
def test_verify_parity_with_a_wide_score_range(name, layers, attn_keys):
    """Query / key projections of the first `layers` layers scaled by 16 / 2: attention scores spread over
    tens of binary orders instead of a fraction of one, so the running reference of the online softmax is
    overtaken from block to block, by little (kept) and by much (accumulators rescaled), within a split
    and across the merge of splits.  400 committed tokens: several key blocks per split.
    Such attention is close to one-hot, and a model built of it is badly conditioned in 16-bit storage: a
    query or key element that rounds to the other neighbour moves a score by a tenth and a probability by
    ten percent.  The bound is therefore the usual tolerance or, if larger, twice what the oracle's OWN
    logits move when its queries and keys are disturbed by one part in a million before they are rounded
    (what float32 instead of float64 sums do to them): with one bfloat16 layer or both float16 layers
    scaled that is below the usual tolerance, with all three bfloat16 layers scaled it is 0.03-0.07.
    (The kernel carries bfloat16 probabilities into the P V product as a sum of two bfloat16 numbers;
    single ones added another 0.08 here and 2e-2 per layer at the 8B shape.)"""
    from unittest import mock
    import oracle.model
    cfg = get_config(name)
    storage = make_weights(cfg)
    for l in range(layers):
        for key, f in ((f"layer{l}.wq", 16.0), (f"layer{l}.wk", 2.0)):
            storage[key] = to_storage(to_float64(storage[key], cfg.dtype) * f, cfg.dtype)   # powers of two: exact
    pair = Pair(name, storage=storage)
    if attn_keys:
        pair.ctx.set_tuning(0, attn_keys)
    prompt = make_prompt(cfg, n=400)
    o, first, tr, g, logits, feats, og, ologits, ofeats = _verify_both(pair, prompt)
    # conditioning: the oracle once more on the same tokens and tree, queries and keys disturbed before rounding
    rng = np.random.default_rng(1)
    plain_rope = oracle.model.rope
    with mock.patch.object(oracle.model, "rope", lambda x, pos, theta: plain_rope(x, pos, theta) * (1 + 1e-6 * rng.normal(size=x.shape))):
        o2 = pair.oracle()
        o2.prefill(prompt)
        o2.tokens[-1] = o.tokens[-1]
        _, dlogits, _ = o2.verify_tree(Tree(o.last["tree"].token, o.last["tree"].parent))
    cond = np.abs(dlogits - ologits).max()
    tol = max(tol_for(cfg), 2 * cond)
    err = np.abs(logits - ologits).max()
    _say(f"  {name}, {layers} layers scaled, keys per split {attn_keys or 'default'}: max|dlogit| = {err:.3e} "
         f"(oracle moved by {cond:.3e} under 1e-6 noise; bound {tol:.3e})")
    assert err <= tol
    if layers == 1 or cfg.dtype == 2:
        assert err <= tol_for(cfg)
    pair.close()


def test_verify_is_bitwise_repeatable_and_layout_independent():
    name = "t_mid_bf16"
    cfg = get_config(name)
    prompt = make_prompt(cfg)
    outs = []
    for order, page in ((0, 64), (0, 64), (1, 64), (0, 32), (1, 128)):
        pair = Pair(name, kv_page_order=order, kv_page_tokens=page)
        pair.ctx.prefill(prompt)
        tr = pair.ctx.draft_tree()
        logits = torch.zeros(tr.n, cfg.vocab, device="cuda")
        g = pair.ctx.verify_tree(None, logits_out=logits)
        outs.append((tr.as_dict(), g[:tr.n].copy(), logits.cpu().numpy()))
        pair.close()
    for a in outs[1:]:
        assert a[0]["token"] == outs[0][0]["token"] and a[0]["parent"] == outs[0][0]["parent"]
        assert np.array_equal(a[1], outs[0][1])
        assert np.array_equal(a[2], outs[0][2])          # same bits, also with reversed physical pages and other page sizes


# --------------------------------------------------------------------------- acceptance with injected trees
@pytest.mark.parametrize("name", ["c0_tiny_f32", "t_mid_bf16"])
def test_injected_trees_accept_every_length(name):
    pair = Pair(name)
    cfg, ctx = pair.cfg, pair.ctx
    _say(f"injected trees {name}")
    prompt = make_prompt(cfg, n=40)
    L = cfg.depth
    # the true continuation, from the library's own root-only rounds (vanilla greedy steps)
    y = [ctx.prefill(prompt)]
    for _ in range(L + 2):
        ctx.verify_tree(P.TreeArrays.from_lists([0], [-1]))
        path, m, toks = ctx.accept_and_commit()
        assert path == [0] and m == 0 and len(toks) == 1
        y.append(toks[0])
    # ... which the oracle must confirm (teacher-forced; near-ties tolerated in 16-bit mode)
    o = pair.oracle()
    o.prefill(prompt)
    from oracle.model import target_full
    _, lg = target_full(pair.W, cfg, list(prompt) + y[:-1], pair.act)
    for j, tok in enumerate(y):
        row = lg[len(prompt) - 1 + j]
        assert tok == int(np.argmax(row)) or row.max() - row[tok] <= 2 * tol_for(cfg)
    wrong = lambda tok: (tok + 1) % cfg.vocab
    for m_want in range(L + 1):
        ctx.reset()
        assert ctx.prefill(prompt) == y[0]
        token, parent = [y[0], (y[1] + 2) % cfg.vocab], [-1, 0]        # root plus a decoy child
        for j in range(1, m_want + 1):
            token.append(y[j]); parent.append(0 if j == 1 else len(token) - 2)
        last = len(token) - 1 if m_want else 0
        if m_want < L:                       # a wrong continuation where the depth allows one
            token.append(wrong(y[m_want + 1])); parent.append(last)
        g = ctx.verify_tree(P.TreeArrays.from_lists(token, parent))
        path, m, toks = ctx.accept_and_commit()
        bpath, bbonus = accept_bruteforce(token, parent, g[:len(token)].tolist())
        assert path == bpath and toks[-1] == bbonus
        assert m == m_want and toks == y[1:m_want + 2]
        assert ctx.tokens() == list(prompt) + y[:m_want + 2]
        # the compacted cache continues correctly: one more vanilla step gives the next true token
        ctx.verify_tree(P.TreeArrays.from_lists([0], [-1]))
        _, _, nxt = ctx.accept_and_commit()
        if m_want + 2 < len(y):
            assert nxt == [y[m_want + 2]]
    st = ctx.stats()
    assert st.rounds == 2
    pair.close()


# --------------------------------------------------------------------------- tree builder with injected top-k
@pytest.mark.parametrize("name,ties", [("c0_tiny_f32", False), ("c0_tiny_f32", True), ("t_mid_bf16", False),
                                       ("t_mid_bf16", True), ("t_mid_f16", True)])
def test_tree_builder_bit_exact(name, ties):
    pair = Pair(name)
    cfg, ctx = pair.cfg, pair.ctx
    k, L = cfg.top_k, cfg.depth
    prompt = make_prompt(cfg, n=20)
    ctx.prefill(prompt)
    rng = np.random.default_rng(11 + ties)
    for trial in range(4):
        ids = np.zeros((L, k, k), np.int32)
        lp = np.zeros((L, k, k), np.float32)
        for d in range(L):
            for r in range(k):
                ids[d, r] = rng.choice(cfg.vocab, size=k, replace=False)
                if ties:
                    lp[d, r] = -np.sort(rng.integers(1, 4, size=k)).astype(np.float32) * 0.5
                else:
                    lp[d, r] = -np.sort(rng.exponential(2.0, size=k)).astype(np.float32)
        tb = TreeBuilder(k, L, cfg.total_tokens)
        for d in range(L):
            rows = len(tb.frontier())
            tb.push(ids[d, :rows], lp[d, :rows])
        ot = tb.finalize(len(prompt))
        d_ = ctx.debug_build_tree(ids, lp).as_dict()
        assert d_["token"][1:] == ot.token[1:] and d_["parent"] == ot.parent
        assert d_["depth"] == ot.depth and d_["pos"] == ot.pos and d_["mask"] == ot.mask
        assert np.array_equal(d_["score"], np.array(ot.score, dtype=np.float32))
        assert d_["mask"] == ancestor_masks(d_["parent"])
    pair.close()


def test_two_contexts_on_their_own_streams_give_the_default_stream_result():
    """The library queues everything on the stream given at load.  Two contexts on two streams,
    driven in turn, must each reproduce bit for bit what a context on the default stream gives."""
    name = "t_mid_bf16"
    cfg = get_config(name)
    prompt = make_prompt(cfg)

    def run(pairs):
        outs = []
        for p in pairs:
            p.ctx.prefill(prompt)
        trees = [p.ctx.draft_tree() for p in pairs]
        bufs = [torch.zeros(tr.n, cfg.vocab, device="cuda") for tr in trees]
        torch.cuda.synchronize()                              # torch filled the buffers on its own stream
        gs = [p.ctx.verify_tree(None, logits_out=b) for p, b in zip(pairs, bufs)]
        res = [p.ctx.accept_and_commit() for p in pairs]
        torch.cuda.synchronize()
        for tr, g, b, r in zip(trees, gs, bufs, res):
            outs.append((tr.as_dict()["token"], g[:tr.n].tolist(), b.cpu().numpy(), r))
        return outs

    ref_pair = Pair(name)
    ref = run([ref_pair])[0]
    ref_pair.close()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    a, b = Pair(name, lib_over=dict(stream=s1)), Pair(name, lib_over=dict(stream=s2))
    torch.cuda.synchronize()
    for got in run([a, b]):
        assert got[0] == ref[0] and got[1] == ref[1] and got[3] == ref[3]
        assert np.array_equal(got[2], ref[2])
    a.close(); b.close()
