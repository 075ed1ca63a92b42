"""Float64 building blocks of a Llama-style decoder (oracle; test infrastructure only).

The paper fixes none of these beyond "Llama-3-8B-Instruct / Llama-2-13B-chat"
(section 4.1 "Target Models"); the definitions below are the published Llama
architecture: RMSNorm, rotate-half rotary embedding, scaled dot-product
attention with grouped KV heads, SwiGLU.
"""
import numpy as np

F32, BF16, F16 = 0, 1, 2      # storage dtype codes (same numbering as the config field)


# ------------------------------------------------------------------ storage precision
def decode_storage(arr, dtype):
    """Storage array (float32 / bfloat16 bit patterns in uint16 / float16) -> float64."""
    if dtype == BF16:
        return (np.asarray(arr).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return np.asarray(arr).astype(np.float64)


def round_storage(x, dtype):
    """Round float64 values to the storage dtype and return them as float64.

    dtype None: identity (the exact-arithmetic model).  The mixed-precision model
    (weights and every GEMM operand held in a 16-bit type, everything else wide)
    rounds activations exactly where they become GEMM operands or cache entries.
    """
    if dtype is None:
        return x
    x = np.asarray(x, dtype=np.float64)
    if dtype == F32:
        return x.astype(np.float32).astype(np.float64)
    if dtype == F16:
        return x.astype(np.float16).astype(np.float64)
    # bfloat16: round-to-nearest-even on the float32 bit pattern
    u = x.astype(np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(np.float64)


# ------------------------------------------------------------------ layers
def rmsnorm(x, gain, eps):
    """x / sqrt(mean(x^2) + eps) * gain, row-wise over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(x, pos, theta):
    """Rotary position embedding, rotate-half pairing (i, i + dh/2).

    x: [rows, heads, dh]; pos: [rows] integer positions.
    Pair i is rotated by angle pos * theta**(-2i/dh).
    """
    rows, heads, dh = x.shape
    half = dh // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / dh)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]      # [rows, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def attention(q, k, v, allowed):
    """softmax(q k^T / sqrt(dh)) v with an explicit boolean visibility matrix.

    q: [rows, Hq, dh]; k, v: [keys, Hkv, dh]; allowed: [rows, keys] bool.
    Query head h reads KV head h // (Hq // Hkv).  Returns [rows, Hq, dh].
    """
    rows, hq, dh = q.shape
    hkv = k.shape[1]
    group = hq // hkv
    out = np.zeros_like(q)
    scale = 1.0 / np.sqrt(dh)
    for h in range(hq):
        kh, vh = k[:, h // group, :], v[:, h // group, :]
        s = (q[:, h, :] @ kh.T) * scale                     # [rows, keys]
        s = np.where(allowed, s, -np.inf)
        s = s - s.max(axis=-1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=-1, keepdims=True)
        out[:, h, :] = p @ vh
    return out


def silu(x):
    return x / (1.0 + np.exp(-x))


def log_softmax(x):
    m = x.max(axis=-1, keepdims=True)
    return x - (m + np.log(np.exp(x - m).sum(axis=-1, keepdims=True)))
