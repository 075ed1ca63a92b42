"""Several sequences per round: a batched context must give every sequence exactly what it gets
alone (same tokens, trees, accepted paths: a row's arithmetic does not depend on which other rows
share its launches), and through that what the oracle computes for it."""
import numpy as np
import pytest

from gpu_util import have_gpu, Pair, tree_from_gpu

pytestmark = pytest.mark.gpu

if have_gpu():
    import paper_2506_03566_amd as P
    from synth import get_config, make_prompt
    from test_gpu_draft import _perfect_drafter_storage


def _say(msg):
    print(msg, flush=True)


def _prompts(cfg, lengths):
    # different prompts of different lengths: sequences sit at different positions in every round
    return [[int(x) for x in make_prompt(cfg.with_(prompt_seed=cfg.prompt_seed + 17 * i), n=n)] for i, n in enumerate(lengths)]


def _rounds_alone(pair, prompt, n_rounds):
    """One sequence in a context of its own (the batch-1 path): per round (tree, path, m, tokens)."""
    ctx = P.Poss(pair.cfg, pair.dev_weights)
    first = ctx.prefill(prompt)
    out = []
    for _ in range(n_rounds):
        tr = ctx.draft_tree().as_dict()
        ctx.verify_tree(want_argmax=False)
        path, m, toks = ctx.accept_and_commit()
        out.append((tr, path, m, toks))
    tokens = ctx.tokens()
    ctx.close()
    return first, out, tokens


def _same_tree(a, b):
    return (a["n"] == b["n"] and a["token"] == b["token"] and a["parent"] == b["parent"] and a["depth"] == b["depth"]
            and a["pos"] == b["pos"] and a["mask"] == b["mask"] and np.array_equal(a["score"], b["score"]))


@pytest.mark.parametrize("name,batch,lengths,perfect,n_rounds", [
    ("c0_tiny_f32", 3, (16, 23, 40), False, 4),          # random drafter: every round commits the bonus token only
    ("c0_tiny_f32", 3, (16, 23, 40), True, 3),           # perfect drafter: full depth accepted, long catch-up rows
    ("t_tiny_f32_6x1", 2, (70, 33), True, 3),            # six specialists, one position each
    ("t_mid_bf16", 2, (150, 97), False, 4),              # 16-bit storage, 2 x 61 rows in the verification pass
    ("t_mid_f16", 1, (131,), False, 2),                  # batch field set to 1: the single-sequence path
    ("c0_tiny_f32", 7, (16, 23, 40, 12, 31, 18, 27), True, 3),   # 7 x 25 rows in one launch (float32 kernels)
    ("t_mid_bf16", 3, (150, 97, 120), False, 3),         # 3 x 61 rows: the 12-row-tile instantiations
    ("t_mid_bf16", 4, (150, 97, 120, 33), False, 3),     # 4 x 61 rows: one launch of 244 rows (16 row tiles)
    ("t_mid_f16", 5, (150, 97, 120, 33, 64), False, 2),  # more rows than a launch carries: a group of four sequences and one of one
])
def test_batched_rounds_equal_sequences_alone(name, batch, lengths, perfect, n_rounds):
    cfg = get_config(name)
    pair = Pair(name, storage=_perfect_drafter_storage(cfg) if perfect else None, lib_over={"batch": batch})
    ctx = pair.ctx
    prompts = _prompts(cfg, lengths)
    _say(f"batch {batch} of {name}, prompts {lengths}, perfect drafter {perfect}")
    alone = [_rounds_alone(pair, p, n_rounds) for p in prompts]
    firsts = [ctx.prefill(p, seq=b) for b, p in enumerate(prompts)]
    assert firsts == [a[0] for a in alone]
    for rnd in range(n_rounds):
        tr0 = ctx.draft_tree()
        trees = [ctx.get_tree(b).as_dict() for b in range(batch)]
        assert _same_tree(tr0.as_dict(), trees[0])
        ctx.verify_tree(want_argmax=False)
        path0, m0, toks0 = ctx.accept_and_commit()
        for b in range(batch):
            atr, apath, am, atoks = alone[b][1][rnd]
            assert _same_tree(trees[b], atr), f"round {rnd}, sequence {b}: tree differs"
            path, m, toks = ctx.commit_result(b)
            assert (path, m, toks) == (apath, am, atoks), f"round {rnd}, sequence {b}"
            if b == 0:
                assert (path0, m0, toks0) == (path, m, toks)
        _say(f"  round {rnd}: accepted {[ctx.commit_result(b)[1] for b in range(batch)]}")
    for b in range(batch):
        assert ctx.tokens(b) == alone[b][2]
    st = ctx.stats()
    assert st.rounds == batch * n_rounds                               # one round per sequence and call
    assert st.committed_tokens == sum(len(alone[b][2]) - len(prompts[b]) - 1 for b in range(batch))
    if perfect:
        assert [ctx.commit_result(b)[1] for b in range(batch)] == [cfg.depth] * batch
    if cfg.dtype == 0:
        # float32 storage: the free-running oracle gives the same stream
        for b in range(batch):
            o = pair.oracle()
            want = o.generate(prompts[b], len(ctx.tokens(b)) - len(prompts[b]))
            assert ctx.tokens(b)[:len(want)] == want[:len(ctx.tokens(b))]
    pair.close()


def test_batched_context_refuses_what_it_cannot_do():
    cfg = get_config("c0_tiny_f32")
    pair = Pair("c0_tiny_f32", lib_over={"batch": 2})
    ctx = pair.ctx
    p0, p1 = _prompts(cfg, (12, 20))
    with pytest.raises(P.PossError):
        ctx.prefill(p0, seq=2)                                         # no such sequence
    ctx.prefill(p0, seq=0)
    with pytest.raises(P.PossError):
        ctx.draft_tree()                                               # sequence 1 has no prompt yet
    with pytest.raises(P.PossError):
        ctx.prefill(p0, seq=0)                                         # already started
    ctx.prefill(p1, seq=1)
    with pytest.raises(P.PossError):
        ctx.set_uniforms(2, [0.5])                                     # no such sequence
    with pytest.raises(P.PossError):
        ctx.set_uniforms(1, [1.0])                                     # not in [0, 1)
    ctx.draft_tree(want_tree=False)
    tree = ctx.get_tree(1)
    with pytest.raises(ValueError):
        ctx.verify_tree(tree)                                          # one tree per sequence
    bad = P.TreeArrays.from_lists([0, 1, 1], [-1, 0, 0])               # two siblings with the same token
    with pytest.raises(P.PossError):
        ctx.verify_tree([tree, bad])
    ctx.verify_tree(want_argmax=False)
    ctx.accept_and_commit()
    with pytest.raises(P.PossError):
        ctx.commit_result(5)
    assert len(ctx.tokens(0)) >= len(p0) + 2 and len(ctx.tokens(1)) >= len(p1) + 2
    ctx.reset()
    with pytest.raises(P.PossError):
        ctx.draft_tree()
    pair.close()
    # more than eight sequences are rejected at load (six, whose stacked rows exceed one launch, run in groups)
    with pytest.raises(P.PossError):
        P.Poss(cfg, pair.dev_weights, batch=9)


@pytest.mark.parametrize("lengths", [(512, 300), (512, 300, 411, 77)])
def test_full_size_batch_equals_each_sequence_alone(lengths):
    """The benchmark shape with two sequences per round (2 x 61 rows in the verification pass, the
    128-row GEMM instantiations) and with four (244 rows in one launch, 16 row tiles): trees, accepted
    paths and tokens of each sequence are the ones a context of its own produces."""
    import torch
    from synth.gpu import make_weights_on_device
    cfg = get_config("c1_llama3_8b_3x2")
    _say("generating weights of c1_llama3_8b_3x2")
    dev = make_weights_on_device(cfg)
    prompts = _prompts(cfg, lengths)
    n_rounds, B = 3, len(lengths)
    ctx = P.Poss(cfg, dev, batch=B)
    for b, p in enumerate(prompts):
        ctx.prefill(p, seq=b)
    got = []
    for rnd in range(n_rounds):
        ctx.draft_tree(want_tree=False)
        trees = [ctx.get_tree(b).as_dict() for b in range(B)]
        ctx.verify_tree(want_argmax=False)
        ctx.accept_and_commit()
        got.append([(trees[b],) + ctx.commit_result(b) for b in range(B)])
    tokens = [ctx.tokens(b) for b in range(B)]
    ctx.close()
    torch.cuda.empty_cache()
    for b, p in enumerate(prompts):
        one = P.Poss(cfg, dev)
        one.prefill(p)
        for rnd in range(n_rounds):
            tr = one.draft_tree().as_dict()
            one.verify_tree(want_argmax=False)
            path, m, toks = one.accept_and_commit()
            assert _same_tree(got[rnd][b][0], tr), f"round {rnd}, sequence {b}: tree differs"
            assert got[rnd][b][1:] == (path, m, toks), f"round {rnd}, sequence {b}"
        assert one.tokens() == tokens[b]
        one.close()
        torch.cuda.empty_cache()
        _say(f"  sequence {b}: {n_rounds} rounds identical")


@pytest.mark.parametrize("name,batch,lengths", [("c0_tiny_f32", 3, (16, 23, 40)), ("t_mid_bf16", 2, (150, 97)),
                                                ("t_mid_bf16", 4, (150, 97, 120, 33)),       # 244 rows: the tall kernel writes the logits
                                                ("c0_tiny_f32", 6, (16, 23, 40, 12, 31, 18))])               # groups of 4 and 2
def test_batched_sampling_equals_sequences_alone(name, batch, lengths):
    """Verification at a temperature with a set of uniform numbers per sequence: every sequence of the
    batch commits the tokens it commits alone with the same numbers (and, in float32 storage, the
    tokens of the oracle's sampler)."""
    cfg = get_config(name)
    pair = Pair(name, lib_over={"batch": batch})
    ctx = pair.ctx
    prompts = _prompts(cfg, lengths)
    n_rounds, T = 4, 0.8
    rng = np.random.default_rng(11)
    # U[b][position]: one number per absolute sequence position, as the oracle indexes them
    U = [rng.random(max(lengths) + n_rounds * (cfg.depth + 1) + 2).astype(np.float32) for _ in range(batch)]
    alone = []
    for b, p in enumerate(prompts):
        one = P.Poss(cfg, pair.dev_weights)
        one.set_sampling(T, [U[b][len(p)]])
        one.prefill(p)
        for _ in range(n_rounds):
            t = len(one.tokens()) - 1
            one.set_sampling(T, U[b][t + 1:t + cfg.depth + 2])
            one.draft_tree(want_tree=False)
            one.verify_tree(want_argmax=False)
            one.accept_and_commit()
        alone.append(one.tokens())
        one.close()
    ctx.set_sampling(T, [0.0])
    for b, p in enumerate(prompts):
        ctx.set_uniforms(b, [U[b][len(p)]])
        ctx.prefill(p, seq=b)
    for _ in range(n_rounds):
        for b in range(batch):
            t = len(ctx.tokens(b)) - 1
            ctx.set_uniforms(b, U[b][t + 1:t + cfg.depth + 2])
        ctx.draft_tree(want_tree=False)
        ctx.verify_tree(want_argmax=False)
        ctx.accept_and_commit()
    for b in range(batch):
        assert ctx.tokens(b) == alone[b], f"sequence {b}"
    if cfg.dtype == 0:
        for b in range(batch):
            o = pair.oracle()
            n_new = len(alone[b]) - len(prompts[b])
            want = o.generate(prompts[b], n_new, temperature=T, U=U[b].astype(np.float64))
            assert alone[b][:len(want)] == want[:len(alone[b])], f"sequence {b} against the oracle"
    pair.close()


@pytest.mark.parametrize("name,batch,lengths", [("c0_tiny_f32", 3, (16, 23, 40)), ("t_mid_bf16", 2, (150, 97)),
                                                ("t_mid_bf16", 4, (150, 97, 120, 33)),       # 244 rows: the tall kernel writes the logits
                                                ("c0_tiny_f32", 8, (16, 23, 40, 12, 31, 18, 27, 21))])      # two groups
def test_batched_caller_trees_equal_sequences_alone(name, batch, lengths):
    """Trees handed in by the caller, one per sequence and of different sizes (root-only rounds are
    vanilla decoding): the batch commits what each sequence commits alone, and a draft after such
    rounds catches the specialists up for every sequence."""
    cfg = get_config(name)
    pair = Pair(name, lib_over={"batch": batch})
    ctx = pair.ctx
    prompts = _prompts(cfg, lengths)
    rng = np.random.default_rng(5)

    def some_tree(b, rnd):
        if rnd % 2 == 0:
            return P.TreeArrays.from_lists([0], [-1])                   # root only
        n = 2 + (b + rnd) % 3                                           # a short chain under the root
        toks = [0] + [int(x) for x in rng.integers(0, cfg.vocab, n - 1)]
        return P.TreeArrays.from_lists(toks, [-1] + list(range(n - 1)))

    n_rounds = 4
    trees = [[some_tree(b, r) for b in range(batch)] for r in range(n_rounds)]
    alone = []
    for b, p in enumerate(prompts):
        one = P.Poss(cfg, pair.dev_weights)
        one.prefill(p)
        res = []
        for r in range(n_rounds):
            one.verify_tree(trees[r][b], want_argmax=False)
            res.append(one.accept_and_commit())
        tr = one.draft_tree().as_dict()
        alone.append((res, one.tokens(), tr))
        one.close()
    for b, p in enumerate(prompts):
        ctx.prefill(p, seq=b)
    for r in range(n_rounds):
        ctx.verify_tree(trees[r], want_argmax=False)
        ctx.accept_and_commit()
        for b in range(batch):
            assert ctx.commit_result(b) == alone[b][0][r], f"round {r}, sequence {b}"
    ctx.draft_tree(want_tree=False)
    for b in range(batch):
        assert ctx.tokens(b) == alone[b][1]
        assert _same_tree(ctx.get_tree(b).as_dict(), alone[b][2]), f"sequence {b}: tree after caller-tree rounds"
    pair.close()


def test_a_finished_sequence_is_replaced_while_the_others_go_on():
    """Continuous batching: one sequence of the batch is reset and given a new prompt between
    rounds; every sequence, old and new, commits what it commits alone."""
    name, batch, n_rounds = "t_mid_bf16", 2, 3
    cfg = get_config(name)
    pair = Pair(name, lib_over={"batch": batch})
    ctx = pair.ctx
    p0, p1, p2 = _prompts(cfg, (150, 97, 61))
    a0 = _rounds_alone(pair, p0, 2 * n_rounds)            # runs through both phases
    a1 = _rounds_alone(pair, p1, n_rounds)                # finishes after the first phase
    a2 = _rounds_alone(pair, p2, n_rounds)                # takes its place
    ctx.prefill(p0, seq=0); ctx.prefill(p1, seq=1)

    def rounds(n):
        for _ in range(n):
            ctx.draft_tree(want_tree=False)
            ctx.verify_tree(want_argmax=False)
            ctx.accept_and_commit()

    rounds(n_rounds)
    assert ctx.tokens(1) == a1[2]
    ctx.reset(seq=1)
    with pytest.raises(P.PossError):
        ctx.draft_tree()                                  # sequence 1 has no prompt
    assert ctx.prefill(p2, seq=1) == a2[0]
    rounds(n_rounds)
    assert ctx.tokens(0) == a0[2] and ctx.tokens(1) == a2[2]
    assert ctx.stats().rounds == batch * 2 * n_rounds      # the statistics run on
    pair.close()


def test_rounds_go_on_without_a_sequence_that_was_set_aside():
    """A batch of three: the middle sequence stops after two rounds, the others go on alone (their rows
    move up), then it comes back; every sequence commits what it commits alone over its own rounds."""
    name, batch = "c0_tiny_f32", 3
    cfg = get_config(name)
    pair = Pair(name, storage=_perfect_drafter_storage(cfg), lib_over={"batch": batch})
    ctx = pair.ctx
    prompts = _prompts(cfg, (16, 23, 40))
    alone = [_rounds_alone(pair, prompts[0], 6), _rounds_alone(pair, prompts[1], 4), _rounds_alone(pair, prompts[2], 6)]

    def rounds(n):
        for _ in range(n):
            ctx.draft_tree(want_tree=False)
            ctx.verify_tree(want_argmax=False)
            ctx.accept_and_commit()

    for b, p in enumerate(prompts):
        ctx.prefill(p, seq=b)
    rounds(2)
    ctx.set_active(1, False)
    kept = ctx.tokens(1)
    rounds(2)                                             # sequences 0 and 2 only
    assert ctx.tokens(1) == kept and ctx.stats().rounds == 3 * 2 + 2 * 2
    tr = ctx.draft_tree()                                 # the tree handed back is the first active sequence's
    assert _same_tree(tr.as_dict(), ctx.get_tree(0).as_dict())
    ctx.set_active(1, True)                               # (drops the drafted trees)
    with pytest.raises(P.PossError):
        ctx.verify_tree(want_argmax=False)
    rounds(2)
    for b in range(batch):
        assert ctx.tokens(b) == alone[b][2], f"sequence {b}"
    ctx.set_active(0, False); ctx.set_active(2, False)
    with pytest.raises(P.PossError):
        ctx.set_active(1, False)                          # someone has to stay
    ctx.draft_tree(want_tree=False)
    ctx.verify_tree(want_argmax=False)
    path, m, toks = ctx.accept_and_commit()               # outputs: the first active sequence, here sequence 1
    assert (path, m, toks) == ctx.commit_result(1)
    pair.close()


def test_a_sequence_set_aside_in_a_batch_that_runs_in_groups():
    """Six sequences whose verification rows need two passes (6 x 61 > 256): one of the first group is
    set aside after two rounds, so the groups are made up differently from then on; every sequence
    still commits what it commits alone."""
    name, batch = "t_mid_bf16", 6
    cfg = get_config(name)
    pair = Pair(name, lib_over={"batch": batch})
    ctx = pair.ctx
    prompts = _prompts(cfg, (150, 97, 120, 33, 64, 141))
    n_rounds = [5, 2, 5, 5, 5, 5]
    alone = [_rounds_alone(pair, p, n) for p, n in zip(prompts, n_rounds)]
    for b, p in enumerate(prompts):
        ctx.prefill(p, seq=b)
    for rnd in range(5):
        if rnd == 2:
            ctx.set_active(1, False)
        ctx.draft_tree(want_tree=False)
        ctx.verify_tree(want_argmax=False)
        ctx.accept_and_commit()
    for b in range(batch):
        assert ctx.tokens(b) == alone[b][2], f"sequence {b}"
    assert ctx.stats().rounds == 6 * 2 + 5 * 3
    pair.close()


def test_the_rows_a_launch_carries_do_not_change_any_sequence():
    """Four sequences of a 16-bit shape with launches of at most 256 rows (one verification pass of 244 rows,
    the tall kernel) and of at most 128 rows (two groups of two, the stream kernel): the same trees, paths and
    tokens, which are those of every sequence alone."""
    name, batch, lengths, n_rounds = "t_mid_f16", 4, (131, 64, 150, 97), 3
    cfg = get_config(name)
    pair = Pair(name, lib_over={"batch": batch})
    prompts = _prompts(cfg, lengths)
    alone = [_rounds_alone(pair, p, n_rounds) for p in prompts]
    with pytest.raises(P.PossError):
        pair.ctx.set_launch_rows(64)
    with pytest.raises(P.PossError):
        pair.ctx.set_launch_rows(257)
    for rows in (256, 128):
        ctx = pair.ctx if rows == 256 else P.Poss(cfg, pair.dev_weights, batch=batch)
        ctx.set_launch_rows(rows)
        firsts = [ctx.prefill(p, seq=b) for b, p in enumerate(prompts)]
        assert firsts == [a[0] for a in alone]
        for rnd in range(n_rounds):
            ctx.draft_tree(want_tree=False)
            trees = [ctx.get_tree(b).as_dict() for b in range(batch)]
            ctx.verify_tree(want_argmax=False)
            ctx.accept_and_commit()
            for b in range(batch):
                atr, apath, am, atoks = alone[b][1][rnd]
                assert _same_tree(trees[b], atr), f"launch rows {rows}, round {rnd}, sequence {b}: tree differs"
                assert ctx.commit_result(b) == (apath, am, atoks), f"launch rows {rows}, round {rnd}, sequence {b}"
        for b in range(batch):
            assert ctx.tokens(b) == alone[b][2]
        if rows != 256:
            ctx.close()
    pair.close()


def test_two_maximal_trees_fill_a_launch():
    """Two sequences whose trees have the largest size a sequence can carry (127 draft tokens + root = 128 rows):
    their verification pass is one launch of exactly 256 rows, no ragged tile anywhere; every sequence still
    drafts, verifies and commits what it does alone."""
    name, batch, lengths, n_rounds = "t_mid_bf16", 2, (150, 97), 3
    cfg = get_config(name, total_tokens=127)
    pair = Pair(name, lib_over={"batch": batch}, total_tokens=127)
    ctx = pair.ctx
    prompts = _prompts(cfg, lengths)
    alone = [_rounds_alone(pair, p, n_rounds) for p in prompts]
    for b, p in enumerate(prompts):
        ctx.prefill(p, seq=b)
    for rnd in range(n_rounds):
        ctx.draft_tree(want_tree=False)
        trees = [ctx.get_tree(b).as_dict() for b in range(batch)]
        assert all(t["n"] == 128 for t in trees)
        ctx.verify_tree(want_argmax=False)
        ctx.accept_and_commit()
        for b in range(batch):
            atr, apath, am, atoks = alone[b][1][rnd]
            assert _same_tree(trees[b], atr), f"round {rnd}, sequence {b}: tree differs"
            assert ctx.commit_result(b) == (apath, am, atoks), f"round {rnd}, sequence {b}"
    for b in range(batch):
        assert ctx.tokens(b) == alone[b][2]
    pair.close()
