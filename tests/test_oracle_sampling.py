"""Pins of the oracle's temperature sampling and of verification at temperature > 0: closed
forms, the temperature limits, frequencies against the softmax, and the lossless property in its
strongest form: with the same random numbers the speculative stream equals vanilla sampling."""
import numpy as np

from synth import get_config, make_prompt, make_weights
from oracle.model import Weights
from oracle.poss import PossOracle
from oracle.sampling import sample_token, softmax_t, cdf_interval, sample_decode
from oracle.tree import accept_walk


def test_two_token_closed_form():
    logits = np.array([0.0, np.log(3.0)])            # p = (1/4, 3/4)
    assert [sample_token(logits, 1.0, u) for u in (0.0, 0.2499, 0.25, 0.9999)] == [0, 0, 1, 1]
    # temperature 2 turns odds 1:3 into 1:sqrt(3)
    p0 = 1.0 / (1.0 + np.sqrt(3.0))
    assert np.allclose(softmax_t(logits, 2.0), [p0, 1 - p0])
    assert sample_token(logits, 2.0, p0 - 1e-9) == 0 and sample_token(logits, 2.0, p0 + 1e-9) == 1
    assert cdf_interval(logits, 1.0, 1) == (0.25, 1.0)


def test_inverse_cdf_is_in_vocabulary_order_and_skips_zero_mass():
    logits = np.array([-np.inf, 1.0, -np.inf, 1.0, 0.0])
    e = np.e
    z = 2 * e + 1
    assert sample_token(logits, 1.0, 0.0) == 1                      # id 0 has no mass
    assert sample_token(logits, 1.0, e / z - 1e-12) == 1
    assert sample_token(logits, 1.0, e / z + 1e-12) == 3            # id 2 has no mass either
    assert sample_token(logits, 1.0, 1.0 - 1e-12) == 4


def test_low_temperature_is_argmax_and_high_temperature_is_uniform():
    rng = np.random.default_rng(3)
    logits = rng.normal(size=50)
    assert all(sample_token(logits, 1e-3, u) == int(np.argmax(logits)) for u in rng.random(20))
    us = (np.arange(50) + 0.5) / 50
    assert [sample_token(logits, 1e6, u) for u in us] == list(range(50))


def test_frequencies_follow_the_softmax():
    rng = np.random.default_rng(11)
    logits = rng.normal(size=12) * 1.5
    for T in (1.0, 0.7):
        p = softmax_t(logits, T)
        n = 40000
        counts = np.bincount([sample_token(logits, T, u) for u in rng.random(n)], minlength=12)
        sigma = np.sqrt(n * p * (1 - p))
        assert np.all(np.abs(counts - n * p) < 5 * sigma + 1)


def test_speculative_sampling_equals_vanilla_sampling_with_the_same_numbers():
    """Section 2.1: verification must leave the target's output distribution untouched.  With one
    uniform number per position the statement becomes exact: the committed stream is the vanilla
    sampled stream, whatever the drafter proposes."""
    cfg = get_config("c0_tiny_f32")
    W = Weights(cfg, make_weights(cfg))
    prompt = make_prompt(cfg, n=16)
    rng = np.random.default_rng(5)
    U = rng.random(len(prompt) + 64)
    for T in (1.0, 0.6):
        want = sample_decode(W, cfg, prompt, 14, T, U)
        o = PossOracle(W, cfg)
        rec = []
        got = o.generate(prompt, 14, record=rec, temperature=T, U=U)
        assert got == want
        assert len(rec) >= 2


def test_acceptance_probability_of_a_child_is_its_target_probability():
    """A child c of the root is accepted exactly when the drawn token is c: over many draws the
    acceptance frequency of the first tree level is the total target probability of the root's
    children (here: logits given directly, tree given directly)."""
    rng = np.random.default_rng(2)
    logits_root = rng.normal(size=30) * 2
    token = [7, 3, 11, 29]                     # root (token irrelevant) and three children
    parent = [-1, 0, 0, 0]
    p = softmax_t(logits_root, 1.0)
    n, acc = 30000, 0
    for u in rng.random(n):
        g = [sample_token(logits_root, 1.0, u), 0, 0, 0]
        path, bonus = accept_walk(token, parent, g)
        acc += len(path) - 1
        if len(path) == 1:
            assert bonus == g[0] and bonus not in token[1:]
    want = p[3] + p[11] + p[29]
    assert abs(acc / n - want) < 5 * np.sqrt(want * (1 - want) / n)


# ---------------------------------------------------------------------- sampled children, rejection rule
from oracle.sampling import draw_from, sample_children, reject_or_accept


def test_children_are_drawn_without_replacement_in_proportion_to_what_is_left():
    rng = np.random.default_rng(4)
    logits = rng.normal(size=9) * 1.3
    q = softmax_t(logits, 0.8)
    n = 30000
    first = np.zeros(9)
    second_given_first = np.zeros((9, 9))
    for _ in range(n):
        ids, qq = sample_children(logits, 0.8, rng.random(4))
        assert len(set(ids)) == 4 and np.allclose(qq, q)
        first[ids[0]] += 1
        second_given_first[ids[0], ids[1]] += 1
    assert np.all(np.abs(first - n * q) < 5 * np.sqrt(n * q * (1 - q)) + 1)
    a = int(np.argmax(q))                              # condition on the most frequent first draw
    cond = q.copy(); cond[a] = 0; cond /= cond.sum()
    na = second_given_first[a].sum()
    assert second_given_first[a, a] == 0
    assert np.all(np.abs(second_given_first[a] - na * cond) < 5 * np.sqrt(na * cond * (1 - cond)) + 1)
    # closed form: equal logits, u in the j-th of the remaining equal intervals picks the j-th remaining id
    ids, _ = sample_children(np.zeros(5), 1.0, [0.5, 0.5, 0.99, 0.0])
    assert ids == [2, 3, 4, 0]
    assert draw_from([0.0, 2.0, 0.0, 2.0], 0.5) == 3 and draw_from([0.0, 2.0, 0.0, 2.0], 0.4999) == 1


def test_rejection_rule_closed_forms():
    # one candidate, two tokens: accepted with probability min(1, p/q); the residual is the positive part of p - q
    p, q = np.array([0.3, 0.7]), np.array([0.6, 0.4])
    assert reject_or_accept(p, q, [0], [0.4999]) == (0, None)         # p/q = 0.5
    i, r = reject_or_accept(p, q, [0], [0.5])
    assert i == -1 and np.allclose(r, [0.0, 1.0])                      # max(p - q, 0) = (0, 0.3) -> (0, 1)
    assert reject_or_accept(p, q, [1], [0.999999])[0] == 0             # p/q > 1: always accepted
    # p == q: whatever was drawn is accepted
    assert reject_or_accept(p, p, [0], [0.999999])[0] == 0
    # two candidates: after rejecting 0, q' = (0, 1) and p' = (0, 1): candidate 1 is accepted whatever its number
    assert reject_or_accept(p, q, [0, 1], [0.9, 0.999999])[0] == 1
    # acceptance probability of the first candidate over its own draw: sum_x min(p, q)
    rng = np.random.default_rng(8)
    n, acc = 40000, 0
    for _ in range(n):
        c = draw_from(q, rng.random())
        acc += reject_or_accept(p, q, [c], [rng.random()])[0] == 0
    want = np.minimum(p, q).sum()
    assert abs(acc / n - want) < 5 * np.sqrt(want * (1 - want) / n)


def test_rejection_rule_keeps_the_target_distribution():
    """Whatever the drafter's distribution and however many candidates are drawn from it, the token that comes
    out - an accepted candidate, else a draw from the last residual - is distributed as the target says."""
    rng = np.random.default_rng(21)
    for k, T in ((1, 1.0), (3, 1.0), (4, 0.7)):
        lp, lq = rng.normal(size=7) * 1.5, rng.normal(size=7) * 1.5
        lq[2] = -np.inf                                        # a token the drafter never proposes
        p = softmax_t(lp, T)
        n = 40000
        counts = np.zeros(7)
        accepted = 0
        for _ in range(n):
            cands, q = sample_children(lq, T, rng.random(k))
            i, resid = reject_or_accept(p, q, cands, rng.random(k))
            tok = cands[i] if i >= 0 else draw_from(resid, rng.random())
            accepted += i >= 0
            counts[tok] += 1
        assert np.all(np.abs(counts - n * p) < 5 * np.sqrt(n * p * (1 - p)) + 1), (k, T)
        assert counts[2] > 0 and 0 < accepted < n


def test_sampled_round_on_the_tiny_model():
    """The round with drawn children: the accepted path is a root path of the tree, every child set is distinct,
    numbers of 0 accept every candidate with target mass (the walk then follows the first-drawn kept children),
    the same numbers give the same round, and committing leaves the state consistent."""
    cfg = get_config("c0_tiny_f32")
    W = Weights(cfg, make_weights(cfg))
    prompt = make_prompt(cfg, n=16)
    rng = np.random.default_rng(6)
    UD = rng.random((cfg.depth, cfg.top_k, cfg.top_k))
    UA = rng.random((cfg.depth + 1, cfg.top_k + 1))
    outs = []
    for rep in range(2):
        o = PossOracle(W, cfg)
        o.prefill(prompt)
        tree = o.draft_tree(sampling=(1.0, UD))
        tb = o.last["builder"]
        for v, kids in tb.expanded.items():
            assert len({tb.token[c] for c in kids}) == cfg.top_k
            assert abs(o.last["draft_q"][v].sum() - 1.0) < 1e-12
        path, last = o.verify_tree_sampled(tree, 1.0, UA)
        assert path[0] == 0 and all(tree.parent[b] == a for a, b in zip(path, path[1:]))
        outs.append((tree.token, tree.parent, path, last))
        o.accept_and_commit(path=path, bonus=last)
        assert o.tokens[-1] == last and len(o.feats) == o.t == len(o.kv[0][0])
    assert outs[0] == outs[1]
    o = PossOracle(W, cfg)
    o.prefill(prompt)
    tree = o.draft_tree(sampling=(1.0, UD))
    path, last = o.verify_tree_sampled(tree, 1.0, np.zeros_like(UA))
    tb = o.last["builder"]
    first_kids = tb.expanded[-1]
    if tree.pool_index[1] == first_kids[0]:
        assert path[:2] == [0, 1]                            # the first-drawn child of the root was kept and is accepted
