"""Oracle building blocks against closed forms, invariants and library routines."""
import numpy as np
import torch

from oracle import numerics as N


def test_round_storage_matches_torch_casts():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.normal(size=4000), rng.normal(size=100) * 1e-3,
                        [0.0, 1.0, -1.0, 1.00390625, 1.01171875, 3.0e38]])
    t = torch.from_numpy(x)
    assert np.array_equal(N.round_storage(x, N.BF16), t.float().bfloat16().double().numpy())
    assert np.array_equal(N.round_storage(x[:-1], N.F16), t[:-1].half().double().numpy())
    assert np.array_equal(N.round_storage(x, N.F32), t.float().double().numpy())
    assert N.round_storage(x, None) is x
    # ties to even on the 8-bit mantissa: 1 + 2^-8 -> 1, 1 + 3*2^-8 -> 1 + 2^-6
    assert N.round_storage(np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8]), N.BF16).tolist() == [1.0, 1 + 2.0 ** -6]


def test_decode_storage_bf16_roundtrip():
    x = torch.randn(1000, dtype=torch.float32).bfloat16()
    bits = x.view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(N.decode_storage(bits, N.BF16), x.double().numpy())


def test_rmsnorm():
    rng = np.random.default_rng(1)
    x, g = rng.normal(size=(5, 64)), rng.normal(size=64)
    y = N.rmsnorm(x, np.ones(64), 0.0)
    assert np.allclose(np.sqrt((y * y).mean(-1)), 1.0)                    # unit RMS
    assert np.allclose(N.rmsnorm(3.7 * x, g, 0.0), N.rmsnorm(x, g, 0.0))  # scale invariance at eps=0
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), 1e-5).numpy()
    assert np.allclose(N.rmsnorm(x, g, 1e-5), ref, rtol=1e-13, atol=1e-13)
    # closed form: x = (3, 4) -> mean square 12.5
    assert np.allclose(N.rmsnorm(np.array([[3.0, 4.0]]), np.array([1.0, 2.0]), 0.0),
                       [[3 / np.sqrt(12.5), 8 / np.sqrt(12.5)]])


def test_rope_closed_form_and_relativity():
    rng = np.random.default_rng(2)
    dh, theta = 8, 10000.0
    x = rng.normal(size=(3, 2, dh))
    assert np.allclose(N.rope(x, [0, 0, 0], theta), x)                    # position 0 is the identity
    y = N.rope(x, [5, 9, 123], theta)
    assert np.allclose((y * y).sum(-1), (x * x).sum(-1))                  # rotations keep the norm
    # pair (0, dh/2) turns by pos * theta^0 = pos radians; pair (1, 1+dh/2) by pos * theta^(-2/dh)
    e = np.zeros((1, 1, dh)); e[0, 0, 0] = 1.0
    r = N.rope(e, [2], theta)[0, 0]
    assert np.allclose([r[0], r[dh // 2]], [np.cos(2.0), np.sin(2.0)])
    e = np.zeros((1, 1, dh)); e[0, 0, 1] = 1.0
    r = N.rope(e, [3], theta)[0, 0]
    a = 3 * theta ** (-2.0 / dh)
    assert np.allclose([r[1], r[1 + dh // 2]], [np.cos(a), np.sin(a)])
    # relativity: <rope(q, p), rope(k, p')> depends on p - p' only
    q, k = rng.normal(size=(1, 1, dh)), rng.normal(size=(1, 1, dh))
    d1 = (N.rope(q, [17], theta) * N.rope(k, [11], theta)).sum()
    d2 = (N.rope(q, [1006], theta) * N.rope(k, [1000], theta)).sum()
    assert np.allclose(d1, d2)
    d3 = (N.rope(q, [11], theta) * N.rope(k, [17], theta)).sum()
    assert not np.allclose(d1, d3)                                         # and on its sign


def test_attention_special_cases_and_library():
    rng = np.random.default_rng(3)
    rows, keys, hq, hkv, dh = 5, 9, 6, 2, 16
    q, k, v = rng.normal(size=(rows, hq, dh)), rng.normal(size=(keys, hkv, dh)), rng.normal(size=(keys, hkv, dh))
    allowed = rng.random((rows, keys)) < 0.6
    allowed[:, 0] = True
    out = N.attention(q, k, v, allowed)
    # library routine: torch SDPA with an explicit boolean mask and repeated KV heads
    g = hq // hkv
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(k, g, axis=1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(v, g, axis=1)).permute(1, 0, 2)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=torch.from_numpy(allowed)[None, None])
    assert np.allclose(out, ref[0].permute(1, 0, 2).numpy(), rtol=1e-12, atol=1e-12)
    # one visible key => its value; q = 0 => mean of visible values
    one = np.zeros((rows, keys), bool); one[:, 4] = True
    assert np.allclose(N.attention(q, k, v, one), np.repeat(v[4], g, axis=0)[None].repeat(rows, 0))
    z = N.attention(np.zeros_like(q), k, v, allowed)
    for i in range(rows):
        assert np.allclose(z[i, 0], v[allowed[i], 0].mean(0))
        assert np.allclose(z[i, hq - 1], v[allowed[i], hkv - 1].mean(0))


def test_silu_logsoftmax_library():
    from scipy.special import log_softmax as sp_ls
    x = np.random.default_rng(4).normal(size=(4, 50)) * 5
    assert np.allclose(N.silu(x), torch.nn.functional.silu(torch.from_numpy(x)).numpy(), rtol=1e-13)
    assert np.allclose(N.log_softmax(x), sp_ls(x, axis=-1), rtol=1e-13, atol=1e-13)
