"""The entry point that allocates nothing (poss_gemm_static) against the entry point it is a variant of
(poss_debug_gemm, caller-supplied scratch): same kernels, so the results must be bit-identical; both are
also held to the float32-accumulation bound against a float64 product.  Two calls in a row share the
library's static scratch array, the second with a smaller input."""
import numpy as np
import pytest

from gpu_util import have_gpu

pytestmark = pytest.mark.gpu

if have_gpu():
    import torch
    import paper_2506_03566_amd as P
    from synth.gen import to_float64, to_storage
    from synth.gpu import to_device


def _case(dtype, M, N, K, seed):
    rng = np.random.default_rng(seed)
    x = to_storage(rng.normal(size=(M, K)), dtype)
    w = to_storage(rng.normal(size=(N, K)) * 0.02, dtype)
    return x, w, to_float64(x, dtype) @ to_float64(w, dtype).T


@pytest.mark.parametrize("dtype", [1, 2, 0])
def test_static_scratch_gemm_matches_the_scratch_argument_gemm_twice_in_a_row(dtype):
    # first a shape that spans several column tiles, K splits and a ragged tail; then a smaller one
    shapes = [(61, 1000, 1408), (10, 200, 264)]
    for i, (M, N, K) in enumerate(shapes):
        print(f"gemm_static dtype={dtype} call {i}: M={M} N={N} K={K}", flush=True)
        x, w, ref = _case(dtype, M, N, K, 100 + i)
        xd, wd = to_device(x, dtype), to_device(w, dtype)
        want, _ = P.debug_gemm(dtype, xd, wd)
        y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        P.gemm_static(dtype, xd, wd, y)
        torch.cuda.synchronize()
        assert torch.equal(y, want), f"call {i}: differs from poss_debug_gemm"
        err = np.abs(y.cpu().numpy().astype(np.float64) - ref).max()
        assert err < 2e-5 * np.sqrt(max(K, 256) / 256.0), err


def test_static_scratch_gemm_refuses_what_does_not_fit():
    lib = P.load_library()
    x = torch.zeros(8, 8192, dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(4096, 8192, dtype=torch.bfloat16, device="cuda")     # 64 MiB packed: beyond the 32 MiB array
    y = torch.zeros(8, 4096, dtype=torch.float32, device="cuda")
    with pytest.raises(P.PossError) as ei:
        P.gemm_static(1, x, w, y)
    assert ei.value.code == P.E_CAPACITY and "static buffer" in str(ei.value)
    assert lib.poss_gemm_static(1, None, None, None, 8, 8, 8, 0, None) == P.E_INVALID_ARG
    assert lib.poss_gemm_static(1, 1, 1, 1, 129, 8, 8, 0, None) == P.E_INVALID_ARG
