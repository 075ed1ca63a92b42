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
