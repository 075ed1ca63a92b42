"""Reproducible synthetic weights and prompts.

Weights are i.i.d. N(0, 0.02) (RMSNorm gains 1, optionally jittered), prompts
are token ids uniform over the vocabulary: random-initialised stand-ins for the
trained checkpoints and evaluation prompts of the paper (section 4.1), which
reproduce shapes and dtypes only.

Each element is a pure function of (seed, tensor name, element index), see
gen.c.  The C routine is used when its shared object has been built, else the
NumPy version below (same bits, slower).
"""
import ctypes
import os
import zlib

import numpy as np

from .configs import DTYPE_F32, DTYPE_BF16, DTYPE_F16

STORAGE_NP = {DTYPE_F32: np.float32, DTYPE_BF16: np.uint16, DTYPE_F16: np.float16}
WEIGHT_STD = 0.02

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsynthgen.so")
_lib = None

LAYER_TENSORS = ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down")


def build_native(verbose=False):
    """Compile gen.c into libsynthgen.so (gcc + OpenMP)."""
    import subprocess
    cmd = ["gcc", "-O3", "-fopenmp", "-shared", "-fPIC", os.path.join(_HERE, "gen.c"),
           "-o", _LIB_PATH]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)


def _native():
    global _lib
    if _lib is None and os.path.exists(_LIB_PATH):
        lib = ctypes.CDLL(_LIB_PATH)
        u64, u32, vp = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p
        lib.synth_fill_table_u16.argtypes = [vp, u64, u64, u32, vp]
        lib.synth_fill_table_u32.argtypes = [vp, u64, u64, u32, vp]
        lib.synth_fill_tokens.argtypes = [vp, u64, u64, u32, u32]
        for f in (lib.synth_fill_table_u16, lib.synth_fill_table_u32, lib.synth_fill_tokens):
            f.restype = None
        _lib = lib
    return _lib


# ---------------------------------------------------------------- hashing
def _mix32_scalar(x):
    x &= 0xFFFFFFFF
    x ^= x >> 16
    x = (x * 0x7feb352d) & 0xFFFFFFFF
    x ^= x >> 15
    x = (x * 0x846ca68b) & 0xFFFFFFFF
    x ^= x >> 16
    return x


def _mix32_np(x):
    x = x.astype(np.uint32, copy=True)
    x ^= x >> np.uint32(16)
    x *= np.uint32(0x7feb352d)
    x ^= x >> np.uint32(15)
    x *= np.uint32(0x846ca68b)
    x ^= x >> np.uint32(16)
    return x


def tensor_key(seed, name):
    """32-bit stream key of one tensor: independent of generation order."""
    return _mix32_scalar((seed * 0x9E3779B1 + zlib.crc32(name.encode())) & 0xFFFFFFFF)


# ---------------------------------------------------------------- storage formats
def _f32_to_bf16_bits(x32):
    """float32 -> bfloat16 bit pattern, round-to-nearest-even."""
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    r = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (r >> np.uint32(16)).astype(np.uint16)


def to_storage(x64, dtype):
    if dtype == DTYPE_F32:
        return np.asarray(x64, dtype=np.float32)
    if dtype == DTYPE_F16:
        return np.asarray(x64, dtype=np.float16)
    return _f32_to_bf16_bits(np.asarray(x64, dtype=np.float32))


def to_float64(arr, dtype):
    """Decode a storage array (as produced here) into float64."""
    if dtype == DTYPE_BF16:
        return (arr.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return arr.astype(np.float64)


_TABLE_CACHE = {}


def _quantile_table(dtype, mean, std):
    """65536 Gaussian quantiles, scaled, in storage format."""
    k = (dtype, float(mean), float(std))
    if k not in _TABLE_CACHE:
        from scipy.special import ndtri
        q = ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0)
        _TABLE_CACHE[k] = np.ascontiguousarray(to_storage(mean + std * q, dtype))
    return _TABLE_CACHE[k]


# ---------------------------------------------------------------- fills
def fill_normal(shape, dtype, seed, name, mean=0.0, std=WEIGHT_STD, out=None, use_native=True):
    """Tensor `name` filled with N(mean, std) in storage format (flat index order = C order)."""
    n = int(np.prod(shape))
    table = _quantile_table(dtype, mean, std)
    key = tensor_key(seed, name)
    if out is None:
        out = np.empty(n, dtype=STORAGE_NP[dtype])
    flat = out.reshape(-1)
    assert flat.size == n and flat.dtype == STORAGE_NP[dtype] and flat.flags.c_contiguous
    lib = _native() if use_native else None
    if lib is not None:
        fn = lib.synth_fill_table_u32 if flat.itemsize == 4 else lib.synth_fill_table_u16
        fn(flat.ctypes.data, n, 0, key, table.ctypes.data)
    else:
        step = 1 << 22
        for s in range(0, n, step):
            e = min(n, s + step)
            idx = (np.arange(s, e, dtype=np.uint64) + np.uint64(key)).astype(np.uint32)
            flat[s:e] = table[_mix32_np(idx) >> np.uint32(16)]
    return out.reshape(shape)


def fill_tokens(n, vocab, seed, name="prompt", use_native=True):
    key = tensor_key(seed, name)
    out = np.empty(n, dtype=np.int32)
    lib = _native() if use_native else None
    if lib is not None:
        lib.synth_fill_tokens(out.ctypes.data, n, 0, key, vocab)
    else:
        idx = (np.arange(n, dtype=np.uint64) + np.uint64(key)).astype(np.uint32)
        out[:] = (_mix32_np(idx) % np.uint32(vocab)).astype(np.int32)
    return out


def make_prompt(cfg, n=None, seed=None):
    return fill_tokens(cfg.n_prompt if n is None else n, cfg.vocab,
                       cfg.prompt_seed if seed is None else seed)


# ---------------------------------------------------------------- tensor inventory
def _layer_specs(cfg, prefix):
    d, qd, kd, f = cfg.d_model, cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim, cfg.d_ffn
    return [(prefix + "attn_norm", (d,), "gain"), (prefix + "wq", (qd, d), "w"),
            (prefix + "wk", (kd, d), "w"), (prefix + "wv", (kd, d), "w"),
            (prefix + "wo", (d, qd), "w"), (prefix + "mlp_norm", (d,), "gain"),
            (prefix + "w_gate", (f, d), "w"), (prefix + "w_up", (f, d), "w"),
            (prefix + "w_down", (d, f), "w")]


def tensor_specs(cfg):
    """[(name, shape, kind)] of every tensor of target + drafter; all are row-major [out, in]."""
    d, v = cfg.d_model, cfg.vocab
    specs = [("embed", (v, d), "w"), ("lm_head", (v, d), "w"), ("final_norm", (d,), "gain")]
    for l in range(cfg.n_layers):
        specs += _layer_specs(cfg, f"layer{l}.")
    for s in range(cfg.n_specialists):
        specs += [(f"spec{s}.fc_w", (d, 2 * d), "w"), (f"spec{s}.fc_b", (d,), "bias")]
        specs += _layer_specs(cfg, f"spec{s}.")
    return specs


def make_tensor(cfg, name, shape, kind, out=None):
    if kind == "gain":
        if cfg.norm_gain_jitter == 0.0:
            arr = to_storage(np.ones(shape), cfg.dtype)
            if out is not None:
                out.reshape(shape)[...] = arr
                return out.reshape(shape)
            return arr
        return fill_normal(shape, cfg.dtype, cfg.weight_seed, name, 1.0, cfg.norm_gain_jitter, out)
    if kind == "bias" and not cfg.fc_bias:
        arr = to_storage(np.zeros(shape), cfg.dtype)
        if out is not None:
            out.reshape(shape)[...] = arr
            return out.reshape(shape)
        return arr
    return fill_normal(shape, cfg.dtype, cfg.weight_seed, name, 0.0, WEIGHT_STD, out)


def make_weights(cfg, names=None):
    """dict name -> storage array.  `names` restricts generation (prefix match allowed)."""
    out = {}
    for name, shape, kind in tensor_specs(cfg):
        if names is not None and not any(name == n or name.startswith(n) for n in names):
            continue
        out[name] = make_tensor(cfg, name, shape, kind)
    return out
