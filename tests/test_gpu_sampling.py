"""Verification at temperature > 0 on the GPU against the oracle: the sampler is an inverse CDF
of the library's own logits, drawn tokens drive the acceptance walk, and with one uniform number
per position the speculative stream equals vanilla sampling token for token."""
import numpy as np
import pytest

from gpu_util import have_gpu, Pair

pytestmark = pytest.mark.gpu

if have_gpu():
    import torch
    import paper_2506_03566_amd as P
    from synth import get_config, make_prompt
    from oracle.sampling import sample_token, cdf_interval, sample_decode
    from oracle.tree import accept_walk

EPS_U = 3e-5       # float32 sums over the vocabulary against the oracle's float64 CDF


def _say(msg):
    print(msg, flush=True)


def _u_for(U, t, depth):
    """The uniform numbers of one round: U[t + j + 1] decides the token after a node of depth j."""
    return np.asarray(U[t + 1:t + depth + 2], dtype=np.float32)


@pytest.mark.parametrize("name,T", [("c0_tiny_f32", 1.0), ("c0_tiny_f32", 0.7), ("t_mid_bf16", 1.0), ("t_mid_f16", 1.3)])
def test_drawn_tokens_are_the_inverse_cdf_of_the_librarys_logits(name, T):
    pair = Pair(name)
    cfg, ctx = pair.cfg, pair.ctx
    rng = np.random.default_rng(17)
    ctx.prefill(make_prompt(cfg))
    exact = total = 0
    for rnd in range(3):
        d = ctx.draft_tree().as_dict()
        u = rng.random(cfg.depth + 1).astype(np.float32)
        ctx.set_sampling(T, u)
        logits = torch.zeros(d["n"], cfg.vocab, device="cuda")
        g = ctx.verify_tree(None, logits_out=logits)[:d["n"]]
        lg = logits.cpu().numpy().astype(np.float64)
        for i in range(d["n"]):
            ui = float(u[d["depth"][i]])
            lo, hi = cdf_interval(lg[i], T, int(g[i]))
            assert lo - EPS_U <= ui < hi + EPS_U, (rnd, i, int(g[i]), ui, lo, hi)
            exact += int(g[i]) == sample_token(lg[i], T, ui)
            total += 1
        path, m, toks = ctx.accept_and_commit()
        wpath, wbonus = accept_walk(d["token"], d["parent"], g.tolist())
        assert path == wpath and toks[-1] == wbonus
    _say(f"  {name} T={T}: {exact}/{total} draws identical to the float64 inverse CDF")
    assert exact >= total - 2
    pair.close()


def test_tiny_temperature_draws_the_argmax():
    pair = Pair("c0_tiny_f32")
    cfg, ctx = pair.cfg, pair.ctx
    ctx.prefill(make_prompt(cfg))
    d = ctx.draft_tree().as_dict()
    logits = torch.zeros(d["n"], cfg.vocab, device="cuda")
    ctx.set_sampling(1e-3, np.full(cfg.depth + 1, 0.37, np.float32))
    g = ctx.verify_tree(None, logits_out=logits)[:d["n"]]
    assert g.tolist() == logits.argmax(dim=1).cpu().tolist()
    ctx.accept_and_commit()
    ctx.set_sampling(0.0)                                    # back to greedy
    ctx.draft_tree()
    g2 = ctx.verify_tree(None, logits_out=logits)[:d["n"]]
    assert g2.tolist() == logits.argmax(dim=1).cpu().tolist()
    pair.close()


@pytest.mark.parametrize("name,T", [("c0_tiny_f32", 1.0), ("c0_tiny_f32", 0.6), ("t_mid_bf16", 1.0)])
def test_speculative_stream_equals_vanilla_sampling_with_the_same_numbers(name, T):
    """Section 2.1 (verification keeps the target's distribution) in its exact form.  The vanilla
    stream comes from the library's own root-only rounds; in float32 it is also the oracle's
    sample_decode (full recompute in float64)."""
    pair = Pair(name)
    cfg, ctx = pair.cfg, pair.ctx
    prompt = make_prompt(cfg, n=24)
    n_new = 18
    U = np.random.default_rng(23).random(len(prompt) + n_new + cfg.depth + 4).astype(np.float32)
    # vanilla: one token per round, the root's draw
    ctx.set_sampling(T, [U[len(prompt)]])
    ar = [ctx.prefill(prompt)]
    root = P.TreeArrays.from_lists([0], [-1])
    while len(ar) < n_new:
        t = len(prompt) + len(ar) - 1
        ctx.set_sampling(T, _u_for(U, t, 0))
        ctx.verify_tree(root, want_argmax=False)
        ar += ctx.accept_and_commit()[2]
    # speculative
    ctx.reset()
    ctx.set_sampling(T, [U[len(prompt)]])
    spec = [ctx.prefill(prompt)]
    ms = []
    while len(spec) < n_new:
        t = len(prompt) + len(spec) - 1
        ctx.set_sampling(T, _u_for(U, t, cfg.depth))
        ctx.draft_tree(want_tree=False)
        ctx.verify_tree(want_argmax=False)
        _, m, toks = ctx.accept_and_commit()
        spec += toks
        ms.append(m)
    _say(f"  {name} T={T}: accepted per round {ms}")
    assert spec[:n_new] == ar[:n_new]
    if cfg.dtype == 0:
        want = sample_decode(pair.W, cfg, prompt, n_new, T, U.astype(np.float64))
        assert [int(x) for x in prompt] + spec[:n_new] == want
    pair.close()


def test_a_drawn_child_is_accepted_and_the_bonus_is_drawn_after_it():
    pair = Pair("c0_tiny_f32")
    cfg, ctx = pair.cfg, pair.ctx
    prompt = make_prompt(cfg, n=20)
    T = 1.0
    root = P.TreeArrays.from_lists([0], [-1])
    ctx.prefill(prompt)
    l0 = torch.zeros(1, cfg.vocab, device="cuda")
    ctx.verify_tree(root, logits_out=l0)                     # the root's logits; nothing committed yet
    ctx.accept_and_commit()
    ctx.reset()
    ctx.prefill(prompt)                                      # same state again
    lg0 = l0[0].cpu().numpy().astype(np.float64)
    child = int(np.argsort(lg0)[-3])                         # some token with a decent probability
    lo, hi = cdf_interval(lg0, T, child)
    u0 = np.float32((lo + hi) / 2)
    decoy = (child + 5) % cfg.vocab
    tree = P.TreeArrays.from_lists([0, decoy, child, (child + 1) % cfg.vocab], [-1, 0, 0, 2])
    u1 = np.float32(0.4321)
    ctx.set_sampling(T, [u0, u1, 0.9])
    logits = torch.zeros(4, cfg.vocab, device="cuda")
    g = ctx.verify_tree(tree, logits_out=logits)[:4]
    assert int(g[0]) == child
    path, m, toks = ctx.accept_and_commit()
    lg = logits.cpu().numpy().astype(np.float64)
    assert path[:2] == [0, 2] and m >= 1 and toks[0] == child
    lo1, hi1 = cdf_interval(lg[2], T, int(g[2]))
    assert lo1 - EPS_U <= float(u1) < hi1 + EPS_U             # depth-1 node: drawn with u[1]
    if m == 1:
        assert toks[1] == int(g[2])
    pair.close()


def test_sampling_arguments_are_checked():
    pair = Pair("c0_tiny_f32")
    ctx = pair.ctx
    with pytest.raises(P.PossError):
        ctx.set_sampling(-1.0, [0.5])
    with pytest.raises(P.PossError):
        ctx.set_sampling(1.0, [1.0])
    with pytest.raises(P.PossError):
        ctx.set_sampling(1.0, None)
    with pytest.raises(P.PossError):
        ctx.set_sampling(1.0, [0.5] * 40)
    pair.close()


# ---------------------------------------------------------------------- drawn children, rejection rule
def _numbers(cfg, seed):
    rng = np.random.default_rng(seed)
    return (rng.random((cfg.depth, cfg.top_k, cfg.top_k)).astype(np.float32),
            rng.random((cfg.depth + 1, cfg.top_k + 1)).astype(np.float32))


@pytest.mark.parametrize("T", [1.0, 0.6])
def test_drawn_children_and_rejection_walk_equal_the_oracle(T):
    """The second reading of verification at a temperature, round by round against the oracle with the same uniform
    numbers.  A vocabulary of 96 tokens keeps every draw's interval wide: numbers are screened by the oracle so that
    every draw and every accept test has a margin of 2e-4 (float32 sums here, float64 there), and then the drawn
    children, the tree, the accepted path and the last token must be identical."""
    pair = Pair("c0_tiny_f32", vocab=96)
    cfg, ctx = pair.cfg, pair.ctx
    o = pair.oracle()
    prompt = make_prompt(cfg, n=24)
    assert ctx.prefill(prompt) == o.prefill(prompt)
    ctx.set_sampling(T, np.zeros(cfg.depth + 1, np.float32))
    seed, rounds, lengths, kinds = 0, 0, [], set()
    while rounds < 8 and seed < 400:
        seed += 1
        UD, UA = _numbers(cfg, seed)
        snap = (list(o.tokens), list(o.feats), list(o.kv), o.stats.rounds)
        otree = o.draft_tree(sampling=(T, UD))
        opath, olast = o.verify_tree_sampled(otree, T, UA)
        if min(o.draw_margins) < 2e-4 or (o.accept_margins and min(o.accept_margins) < 2e-4):
            continue                                          # too close to call in float32: other numbers
        _say(f"  T={T}: numbers {seed} pass the screen, round {rounds} on the GPU")
        ctx.set_draft_sampling(UD, UA)
        d = ctx.draft_tree().as_dict()
        assert d["token"][1:] == otree.token[1:] and d["parent"] == otree.parent, f"seed {seed}"
        assert np.abs(d["score"] - np.array(otree.score, dtype=np.float32)).max() < 1e-4
        g = ctx.verify_tree()
        path, m, toks = ctx.accept_and_commit()
        assert path == opath and toks[-1] == olast and toks[:-1] == [otree.token[p] for p in opath[1:]], f"seed {seed}"
        assert all(g[a] == otree.token[b] for a, b in zip(path, path[1:])) and g[path[-1]] == olast
        o.accept_and_commit(path=opath, bonus=olast)
        assert ctx.tokens() == o.tokens
        rounds += 1
        lengths.append(m)
        tb = o.last["builder"]
        pv = otree.pool_index[opath[-1]]
        kinds.add("leaf" if pv not in tb.expanded else ("dropped child" if olast in [tb.token[c] for c in tb.expanded[pv]] else "residual"))
    _say(f"  T={T}: {rounds} rounds compared ({seed} sets of numbers tried), accepted lengths {lengths}, walks ended by {sorted(kinds)}")
    assert rounds == 8 and max(lengths) >= 1
    # back to the deterministic tree: the coupling rule again
    ctx.set_draft_sampling(None)
    ctx.set_sampling(0.0)
    tr = ctx.draft_tree().as_dict()
    kids = [tr["token"][i] for i in range(1, tr["n"]) if tr["parent"][i] == 0]
    assert len(set(kids)) == len(kids)
    pair.close()


@pytest.mark.parametrize("name", ["t_mid_bf16", "t_mid_f16"])
def test_drawn_children_at_16_bit_shapes_give_valid_rounds(name):
    """16-bit storage, vocabularies of thousands: draws fall too close to interval ends for a token-by-token comparison,
    so the rounds are checked for what must hold whatever the numbers: distinct children under every node, scores that
    are sums of log-probabilities (non-positive steps), a path that is a root path, a last token that is not a kept child
    of the last node, a consistent token stream."""
    pair = Pair(name)
    cfg, ctx = pair.cfg, pair.ctx
    ctx.prefill(make_prompt(cfg))
    ctx.set_sampling(1.0, np.zeros(cfg.depth + 1, np.float32))
    n_before = len(ctx.tokens())
    total = 0
    for rnd in range(5):
        UD, UA = _numbers(cfg, 100 + rnd)
        ctx.set_draft_sampling(UD, UA)
        d = ctx.draft_tree().as_dict()
        assert d["n"] == cfg.total_tokens + 1
        kids = {}
        for i in range(1, d["n"]):
            kids.setdefault(d["parent"][i], []).append(d["token"][i])
            assert d["score"][i] <= d["score"][d["parent"][i]] + 1e-6
        assert all(len(set(v)) == len(v) for v in kids.values())
        ctx.verify_tree()
        path, m, toks = ctx.accept_and_commit()
        assert path[0] == 0 and all(d["parent"][b] == a for a, b in zip(path, path[1:]))
        assert toks[:-1] == [d["token"][p] for p in path[1:]] and toks[-1] not in kids.get(path[-1], [])
        total += len(toks)
    assert len(ctx.tokens()) == n_before + total
    pair.close()


def test_drawn_children_arguments_and_call_order_are_checked():
    pair = Pair("c0_tiny_f32")
    cfg, ctx = pair.cfg, pair.ctx
    UD, UA = _numbers(cfg, 1)
    bad = UD.copy(); bad[0, 0, 0] = 1.0
    with pytest.raises(P.PossError):
        ctx.set_draft_sampling(bad, UA)
    ctx.prefill(make_prompt(cfg, n=12))
    ctx.set_draft_sampling(UD, UA)
    with pytest.raises(P.PossError) as ei:                    # no temperature set
        ctx.draft_tree()
    assert ei.value.code == P.E_BAD_STATE
    ctx.set_sampling(1.0, np.zeros(cfg.depth + 1, np.float32))
    ctx.draft_tree()
    with pytest.raises(P.PossError) as ei:                    # a caller's tree has no draft distributions
        ctx.verify_tree(P.TreeArrays.from_lists([0], [-1]))
    assert ei.value.code == P.E_BAD_STATE
    ctx.verify_tree()
    ctx.accept_and_commit()
    pair.close()
    two = Pair("c0_tiny_f32", lib_over=dict(batch=2))
    with pytest.raises(P.PossError) as ei:
        two.ctx.set_draft_sampling(UD, UA)
    assert ei.value.code == P.E_INVALID_ARG
    two.close()
