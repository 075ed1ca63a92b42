"""Input generators: C and NumPy versions agree; streams are order-independent."""
import numpy as np
import pytest

from synth import get_config, make_weights, make_prompt, tensor_specs
from synth import gen


def test_native_matches_numpy():
    if gen._native() is None:
        pytest.skip("libsynthgen.so not built")
    for dtype in (0, 1, 2):
        a = gen.fill_normal((37, 129), dtype, 7, "x.y", use_native=True)
        b = gen.fill_normal((37, 129), dtype, 7, "x.y", use_native=False)
        assert a.dtype == b.dtype and np.array_equal(a, b)
    assert np.array_equal(gen.fill_tokens(1000, 4096, 3, use_native=True),
                          gen.fill_tokens(1000, 4096, 3, use_native=False))


def test_distribution_and_independence():
    x = gen.to_float64(gen.fill_normal((1 << 18,), 1, 2506, "layer0.wq"), 1)
    assert abs(x.mean()) < 2e-4 and abs(x.std() - 0.02) < 2e-4
    y = gen.to_float64(gen.fill_normal((1 << 18,), 1, 2506, "layer1.wq"), 1)
    assert abs(np.corrcoef(x, y)[0, 1]) < 0.01
    p = gen.fill_tokens(1 << 16, 1000, 3566)
    assert p.min() >= 0 and p.max() < 1000 and len(np.unique(p)) == 1000


def test_inventory_and_subset():
    cfg = get_config("c0_tiny_f32")
    specs = tensor_specs(cfg)
    assert len(specs) == 3 + 9 * cfg.n_layers + 11 * cfg.n_specialists
    w = make_weights(cfg)
    sub = make_weights(cfg, names=["layer1.", "lm_head"])
    assert set(sub) == {n for n, _, _ in specs if n.startswith("layer1.") or n == "lm_head"}
    for k in sub:
        assert np.array_equal(sub[k], w[k])
    assert np.all(w["final_norm"] == 1.0)          # gains are exactly 1 in the benchmark recipe
    assert w["spec2.fc_w"].shape == (cfg.d_model, 2 * cfg.d_model)
    assert len(make_prompt(cfg)) == cfg.n_prompt
