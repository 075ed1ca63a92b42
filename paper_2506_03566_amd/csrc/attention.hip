// Tree-masked attention over a paged KV cache.
//
// Every row of a pass sees the `n_prefix` committed cache slots and, of the `region_len` slots
// that follow them (the rows of this round: tree nodes in verification, drafted ancestors in a
// specialist pass, the chunk itself in prefill), those whose bit is set in the row's mask.
//
// 16-bit types: one wave per (16 query rows, KV head, key split), on v_mfma_f32_16x16x32.
// Query rows of the G = Hq/Hkv heads that share a KV head are stacked (rho = m*G + g) so a wave's
// 16 rows reuse every key it loads.  Scores are formed transposed, S^T = K Q^T (keys as MFMA rows):
// a lane then holds 8 scores of ONE query row per 32-key block, which is already the B-operand
// layout of O^T = V^T P^T as long as the keys of a block are contracted in the order the score
// tiles deliver them; V is cached transposed ([dh][token]) so that order costs two 8-byte loads.
// Softmax is online (running max / sum per query row, float32); partial (max, sum, O) per split
// are merged by a second kernel in fixed order.
#include "device_utils.h"

namespace poss {

typedef float  f32x4 __attribute__((ext_vector_type(4)));
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef f16_t  f16x8 __attribute__((ext_vector_type(8)));

template <typename T> struct Vec8;
template <> struct Vec8<bf16_t> {
    typedef bf16x8 type;
    static __device__ __forceinline__ f32x4 mfma(bf16x8 a, bf16x8 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
};
template <> struct Vec8<f16_t> {
    typedef f16x8 type;
    static __device__ __forceinline__ f32x4 mfma(f16x8 a, f16x8 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
    }
};

__device__ __forceinline__ bool slot_visible(int slot, int n_prefix, int region_len, uint64_t m0, uint64_t m1) {
    if (slot < n_prefix) return true;
    const int j = slot - n_prefix;
    if (j >= region_len) return false;
    return ((j < 64 ? m0 >> j : m1 >> (j - 64)) & 1ull) != 0;
}

template <typename T, int DH>
__global__ __launch_bounds__(64) void attn_mfma_kernel(
    const T *__restrict__ q, int rows, int hq, int hkv, const uint64_t *__restrict__ mask, int n_prefix,
    int region_len, KVCache kv, int blocks_per_split, float scale, float *__restrict__ o_part,
    float *__restrict__ ml_part, int rho_pad) {
    typedef typename Vec8<T>::type V8;
    constexpr int KS = DH / 32, DT = DH / 16;
    const int lane = threadIdx.x, lr = lane & 15, lg = lane >> 4;
    const int G = hq / hkv, kvh = blockIdx.y, split = blockIdx.z;
    const int rho = blockIdx.x * 16 + lr;
    const bool valid = rho < rows * G;
    const int m = valid ? rho / G : 0, qh = kvh * G + (valid ? rho % G : 0);

    V8 qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        u32x4 v = u32x4{0u, 0u, 0u, 0u};
        if (valid) v = *reinterpret_cast<const u32x4 *>(q + ((size_t)m * hq + qh) * DH + ks * 32 + lg * 8);
        qf[ks] = __builtin_bit_cast(V8, v);
    }
    const uint64_t m0 = valid ? mask[(size_t)m * MASK_WORDS] : 0ull;
    const uint64_t m1 = valid ? mask[(size_t)m * MASK_WORDS + 1] : 0ull;

    const int total = n_prefix + region_len;
    const int n_blocks = (total + 31) >> 5;
    const int b0 = split * blocks_per_split, b1 = min(n_blocks, b0 + blocks_per_split);
    const int P = 1 << kv.page_shift;
    const T *kc = static_cast<const T *>(kv.k), *vc = static_cast<const T *>(kv.vt);

    f32x4 acc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY, l_run = 0.f;

    // Key and value fragments of one 32-slot block: K rows slot0 + tt*16 + lr (A operand of S^T),
    // V^T rows dt*16 + lr at keys {slot0 + 4lg..+3} and {slot0 + 16 + 4lg..+3} (A operand of O^T).
    // Both are requested together, one block ahead of the arithmetic.
    u32x4 kf[2][2][KS];
    u32x2 vf[2][DT][2];
    auto load_block = [&](int b, int buf) {
        const int slot0 = b << 5;
        const int pg = kv.page_table[slot0 >> kv.page_shift], off = slot0 & (P - 1);
        const size_t head_base = (size_t)(pg * hkv + kvh);
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            const T *krow = kc + (head_base * P + off + tt * 16 + lr) * DH + lg * 8;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kf[buf][tt][ks] = *reinterpret_cast<const u32x4 *>(krow + ks * 32);
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const T *vrow = vc + (head_base * DH + dt * 16 + lr) * P + off + 4 * lg;
            vf[buf][dt][0] = *reinterpret_cast<const u32x2 *>(vrow);
            vf[buf][dt][1] = *reinterpret_cast<const u32x2 *>(vrow + 16);
        }
    };
    auto compute_block = [&](int b, int buf) {
        const int slot0 = b << 5;
        f32x4 s[2];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            s[tt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                s[tt] = Vec8<T>::mfma(__builtin_bit_cast(V8, kf[buf][tt][ks]), qf[ks], s[tt]);
        }
        // lane holds keys slot0 + tt*16 + 4*lg + r of query row lr
        float sv[8], bm = -INFINITY;
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int slot = slot0 + tt * 16 + 4 * lg + r;
                const float x = slot_visible(slot, n_prefix, region_len, m0, m1) ? s[tt][r] * scale : -INFINITY;
                sv[tt * 4 + r] = x;
                bm = fmaxf(bm, x);
            }
        bm = fmaxf(bm, __shfl_xor(bm, 16, 64));
        bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
        const float m_new = fmaxf(m_run, bm);
        float alpha = 1.f, psum = 0.f;
        V8 pf;
        if (m_new == -INFINITY) {
#pragma unroll
            for (int j = 0; j < 8; ++j) pf[j] = (T)0.f;
        } else {
            alpha = expf(m_run - m_new);             // exp(-inf) = 0 on the first visible block
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float p = expf(sv[j] - m_new);
                const T pt = from_f<T>(p);
                pf[j] = pt;
                psum += to_f(pt);                    // normalise by what is actually multiplied into V
            }
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            acc[dt] *= alpha;
            const u32x2 lo = vf[buf][dt][0], hi = vf[buf][dt][1];
            acc[dt] = Vec8<T>::mfma(__builtin_bit_cast(V8, (u32x4{lo.x, lo.y, hi.x, hi.y})), pf, acc[dt]);
        }
    };
    if (b0 < b1) load_block(b0, 0);
    for (int b = b0; b < b1; b += 2) {               // two blocks per trip so the buffer index is static
        if (b + 1 < b1) load_block(b + 1, 1);
        compute_block(b, 0);
        if (b + 1 < b1) {
            if (b + 2 < b1) load_block(b + 2, 0);
            compute_block(b + 1, 1);
        }
    }
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);

    // O^T tile dt: lane -> query row lr, register r -> dh index dt*16 + 4*lg + r
    const size_t prow = ((size_t)split * hkv + kvh) * rho_pad + blockIdx.x * 16 + lr;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
        *reinterpret_cast<f32x4 *>(o_part + prow * DH + dt * 16 + 4 * lg) = acc[dt];
    if (lg == 0) {
        ml_part[prow * 2] = m_run;
        ml_part[prow * 2 + 1] = l_run;
    }
}

// out[m][qh][:] = sum_s e^{m_s - M} O_s / sum_s e^{m_s - M} l_s
template <typename T>
__global__ void attn_merge_kernel(const float *__restrict__ o_part, const float *__restrict__ ml_part, int n_splits,
                                  int hq, int hkv, int dh, int rho_pad, T *__restrict__ out) {
    const int m = blockIdx.x, qh = blockIdx.y, G = hq / hkv;
    const int kvh = qh / G, rho = m * G + qh % G;
    float M = -INFINITY;
    for (int s = 0; s < n_splits; ++s) M = fmaxf(M, ml_part[(((size_t)s * hkv + kvh) * rho_pad + rho) * 2]);
    for (int i = threadIdx.x; i < dh; i += blockDim.x) {
        float num = 0.f, den = 0.f;
        for (int s = 0; s < n_splits; ++s) {
            const size_t prow = ((size_t)s * hkv + kvh) * rho_pad + rho;
            const float ms = ml_part[prow * 2];
            if (ms == -INFINITY) continue;
            const float w = expf(ms - M);
            num += w * o_part[prow * dh + i];
            den += w * ml_part[prow * 2 + 1];
        }
        out[((size_t)m * hq + qh) * dh + i] = from_f<T>(num / den);
    }
}

// float32 storage: one wave per (row, query head); exact two-pass softmax.
__global__ __launch_bounds__(64) void attn_f32_kernel(const float *__restrict__ q, int hq, int hkv, int dh,
                                                      const uint64_t *__restrict__ mask, int n_prefix, int region_len,
                                                      KVCache kv, float scale, float *__restrict__ out) {
    extern __shared__ float sc[];
    const int m = blockIdx.x, qh = blockIdx.y, kvh = qh / (hq / hkv), lane = threadIdx.x;
    const float *qr = q + ((size_t)m * hq + qh) * dh;
    const uint64_t m0 = mask[(size_t)m * MASK_WORDS], m1 = mask[(size_t)m * MASK_WORDS + 1];
    const int total = n_prefix + region_len;
    const float *kc = static_cast<const float *>(kv.k), *vc = static_cast<const float *>(kv.vt);
    float mx = -INFINITY;
    for (int sl = lane; sl < total; sl += 64) {
        float x = -INFINITY;
        if (slot_visible(sl, n_prefix, region_len, m0, m1)) {
            const float *kr = kc + k_offset(kv, sl, kvh, hkv, dh);
            float a = 0.f;
            for (int i = 0; i < dh; ++i) a = fmaf(qr[i], kr[i], a);
            x = a * scale;
        }
        sc[sl] = x;
        mx = fmaxf(mx, x);
    }
    mx = wave_max(mx);
    float sum = 0.f;
    for (int sl = lane; sl < total; sl += 64) {
        const float p = expf(sc[sl] - mx);
        sc[sl] = p;
        sum += p;
    }
    sum = wave_sum(sum);
    __syncthreads();
    for (int i = lane; i < dh; i += 64) {
        float a = 0.f;
        for (int sl = 0; sl < total; ++sl) a = fmaf(sc[sl], vc[vt_offset(kv, sl, kvh, hkv, dh, i)], a);
        out[((size_t)m * hq + qh) * dh + i] = a / sum;
    }
}

template <typename T>
static void launch_attention_t(const ModelDims &md, const void *q, int rows, const RowMeta &rm, int n_prefix,
                               int region_len, const KVCache &kv, int keys_per_split, const AttnScratch &sc,
                               void *out, hipStream_t st) {
    const int G = md.hq / md.hkv;
    const int tiles = (rows * G + 15) / 16, rho_pad = tiles * 16;
    const int n_blocks = (n_prefix + region_len + 31) / 32;
    int bps = keys_per_split / 32; if (bps < 1) bps = 1;
    const int n_splits = (n_blocks + bps - 1) / bps;
    const float scale = 1.0f / sqrtf((float)md.dh);
    dim3 grid(tiles, md.hkv, n_splits);
    if (md.dh == 128)
        hipLaunchKernelGGL((attn_mfma_kernel<T, 128>), grid, dim3(64), 0, st, static_cast<const T *>(q), rows, md.hq,
                           md.hkv, rm.mask, n_prefix, region_len, kv, bps, scale, sc.o, sc.ml, rho_pad);
    else
        hipLaunchKernelGGL((attn_mfma_kernel<T, 64>), grid, dim3(64), 0, st, static_cast<const T *>(q), rows, md.hq,
                           md.hkv, rm.mask, n_prefix, region_len, kv, bps, scale, sc.o, sc.ml, rho_pad);
    hipLaunchKernelGGL((attn_merge_kernel<T>), dim3(rows, md.hq), dim3(md.dh < 64 ? 64 : md.dh), 0, st, sc.o, sc.ml,
                       n_splits, md.hq, md.hkv, md.dh, rho_pad, static_cast<T *>(out));
}

int attention_splits(int total_keys, int keys_per_split) {
    int bps = keys_per_split / 32; if (bps < 1) bps = 1;
    return ((total_keys + 31) / 32 + bps - 1) / bps;
}

void launch_attention(const ModelDims &md, const void *q, int rows, const RowMeta &rm, int n_prefix,
                      int region_len, const KVCache &kv, int keys_per_split, const AttnScratch &sc,
                      void *out, hipStream_t st) {
    if (md.dt == DT_F32) {
        const size_t lds = (size_t)(n_prefix + region_len) * sizeof(float);
        hipLaunchKernelGGL(attn_f32_kernel, dim3(rows, md.hq), dim3(64), lds, st, static_cast<const float *>(q),
                           md.hq, md.hkv, md.dh, rm.mask, n_prefix, region_len, kv, 1.0f / sqrtf((float)md.dh),
                           static_cast<float *>(out));
    } else if (md.dt == DT_BF16) {
        launch_attention_t<bf16_t>(md, q, rows, rm, n_prefix, region_len, kv, keys_per_split, sc, out, st);
    } else {
        launch_attention_t<f16_t>(md, q, rows, rm, n_prefix, region_len, kv, keys_per_split, sc, out, st);
    }
}

}  // namespace poss
