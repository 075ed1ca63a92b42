// Consumers of the GEMM's split-K partial sums, fused with what follows each projection in a
// Llama decoder layer: rotary embedding + KV-cache write, residual add + RMSNorm, SiLU * up,
// plus embedding gather, argmax and row copies.  All arithmetic in float32; values become the
// storage type only where they are the next GEMM's operand or a cache entry.
#include "device_utils.h"

namespace poss {

#define POSS_DISPATCH(dt, ...)                                               \
    switch (dt) {                                                            \
        case DT_F32:  { using T = float;  __VA_ARGS__; } break;              \
        case DT_BF16: { using T = bf16_t; __VA_ARGS__; } break;              \
        default:      { using T = f16_t;  __VA_ARGS__; } break;              \
    }

__device__ __forceinline__ float sum_parts(const float *part, size_t plane, int S, size_t idx) {
    float a = part[idx];
    for (int s = 1; s < S; ++s) a += part[(size_t)s * plane + idx];
    return a;
}

// ------------------------------------------------------------------ h = emb[token]; u = T(rmsnorm(h) g)
template <typename T>
__global__ __launch_bounds__(256) void embed_norm_kernel(const T *__restrict__ embed, const int32_t *__restrict__ tokens,
                                                         int d, float eps, const T *__restrict__ gain,
                                                         float *__restrict__ h, T *__restrict__ u) {
    __shared__ float red[17];
    const int row = blockIdx.x;
    const T *e = embed + (size_t)tokens[row] * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += blockDim.x) {
        const float v = to_f(e[i]);
        h[(size_t)row * d + i] = v;
        ss += v * v;
    }
    ss = block_sum(ss, red);
    const float rs = 1.0f / sqrtf(ss / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += blockDim.x)
        u[(size_t)row * d + i] = from_f<T>(to_f(e[i]) * rs * to_f(gain[i]));
}

void launch_embed_norm(const ModelDims &md, const void *embed, const int32_t *tokens, int rows,
                       const void *gain, float *h, void *u, hipStream_t st) {
    POSS_DISPATCH(md.dt, hipLaunchKernelGGL((embed_norm_kernel<T>), dim3(rows), dim3(256), 0, st,
                                            static_cast<const T *>(embed), tokens, md.d, md.eps,
                                            static_cast<const T *>(gain), h, static_cast<T *>(u)));
}

// ------------------------------------------------------------------ QKV partials -> rotated q, cache writes
// Rotary embedding pairs element i with i + dh/2 and turns pair i by pos * theta^(-2i/dh); the
// angle is formed in float64 so that positions in the thousands keep float32-accurate sines.
template <typename T>
__global__ __launch_bounds__(256) void reduce_rope_kv_kernel(
    const float *__restrict__ part, size_t plane, int S, int Npad, int rows_q, const int32_t *__restrict__ pos,
    const int32_t *__restrict__ slot, const double *__restrict__ inv_freq, int hq, int hkv, int dh,
    T *__restrict__ q, KVCache kv) {
    __shared__ float cs[128][2];
    const int m = blockIdx.x, half = dh >> 1;
    if ((int)threadIdx.x < half) {
        double s, c;
        sincos((double)pos[m] * inv_freq[threadIdx.x], &s, &c);
        cs[threadIdx.x][0] = (float)c;
        cs[threadIdx.x][1] = (float)s;
    }
    __syncthreads();
    const size_t row0 = (size_t)m * Npad;
    if (m < rows_q) {
        for (int p = threadIdx.x; p < hq * half; p += blockDim.x) {
            const int h = p / half, i = p % half;
            const float x1 = sum_parts(part, plane, S, row0 + h * dh + i);
            const float x2 = sum_parts(part, plane, S, row0 + h * dh + i + half);
            const float c = cs[i][0], s = cs[i][1];
            T *dst = q + ((size_t)m * hq + h) * dh;
            dst[i] = from_f<T>(x1 * c - x2 * s);
            dst[i + half] = from_f<T>(x2 * c + x1 * s);
        }
    }
    const int sl = slot[m];
    T *kc = static_cast<T *>(kv.k), *vc = static_cast<T *>(kv.vt);
    for (int p = threadIdx.x; p < hkv * half; p += blockDim.x) {
        const int h = p / half, i = p % half;
        const size_t col = (size_t)hq * dh + h * dh + i;
        const float x1 = sum_parts(part, plane, S, row0 + col);
        const float x2 = sum_parts(part, plane, S, row0 + col + half);
        const float c = cs[i][0], s = cs[i][1];
        T *dst = kc + k_offset(kv, sl, h, hkv, dh);
        dst[i] = from_f<T>(x1 * c - x2 * s);
        dst[i + half] = from_f<T>(x2 * c + x1 * s);
    }
    for (int p = threadIdx.x; p < hkv * dh; p += blockDim.x) {
        const int h = p / dh, i = p % dh;
        const float x = sum_parts(part, plane, S, row0 + (size_t)(hq + hkv) * dh + p);
        vc[vt_offset(kv, sl, h, hkv, dh, i)] = from_f<T>(x);
    }
}

void launch_reduce_rope_kv(const ModelDims &md, const GemmShape &g, const float *part, int rows,
                           int rows_q, const RowMeta &rm, const double *inv_freq, void *q,
                           const KVCache &kv, hipStream_t st) {
    const size_t plane = (size_t)g.Mpad * g.Npad;
    POSS_DISPATCH(md.dt, hipLaunchKernelGGL((reduce_rope_kv_kernel<T>), dim3(rows), dim3(256), 0, st, part, plane,
                                            g.S, g.Npad, rows_q, rm.pos, rm.slot, inv_freq, md.hq, md.hkv,
                                            md.dh, static_cast<T *>(q), kv));
}

// ------------------------------------------------------------------ h (+)= sum(part) + bias ; u = T(rmsnorm(h) g)
template <typename T>
__global__ __launch_bounds__(256) void reduce_res_norm_kernel(
    const float *__restrict__ part, size_t plane, int S, int Npad, int d, float eps, int residual,
    const T *__restrict__ bias, const T *__restrict__ gain, float *__restrict__ h, T *__restrict__ u,
    float *__restrict__ h_copy) {
    __shared__ float red[17];
    const int m = blockIdx.x;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += blockDim.x) {
        float v = sum_parts(part, plane, S, (size_t)m * Npad + i);
        if (bias) v += to_f(bias[i]);
        if (residual) v += h[(size_t)m * d + i];
        h[(size_t)m * d + i] = v;
        if (h_copy) h_copy[(size_t)m * d + i] = v;
        ss += v * v;
    }
    if (!gain) return;
    ss = block_sum(ss, red);
    const float rs = 1.0f / sqrtf(ss / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += blockDim.x)
        u[(size_t)m * d + i] = from_f<T>(h[(size_t)m * d + i] * rs * to_f(gain[i]));
}

void launch_reduce_res_norm(const ModelDims &md, const GemmShape &g, const float *part, int rows,
                            bool residual, const void *bias, const void *gain, float *h, void *u,
                            float *h_copy, hipStream_t st) {
    const size_t plane = (size_t)g.Mpad * g.Npad;
    POSS_DISPATCH(md.dt, hipLaunchKernelGGL((reduce_res_norm_kernel<T>), dim3(rows), dim3(256), 0, st, part, plane,
                                            g.S, g.Npad, md.d, md.eps, residual ? 1 : 0,
                                            static_cast<const T *>(bias), static_cast<const T *>(gain), h,
                                            static_cast<T *>(u), h_copy));
}

// ------------------------------------------------------------------ act = T(silu(gate) * up)
template <typename T>
__global__ __launch_bounds__(256) void reduce_silu_kernel(const float *__restrict__ part, size_t plane, int S,
                                                          int Npad, int F, T *__restrict__ act) {
    const int f = blockIdx.x * blockDim.x + threadIdx.x, m = blockIdx.y;
    if (f >= F) return;
    const float g = sum_parts(part, plane, S, (size_t)m * Npad + f);
    const float up = sum_parts(part, plane, S, (size_t)m * Npad + F + f);
    act[(size_t)m * F + f] = from_f<T>(g / (1.0f + expf(-g)) * up);
}

void launch_reduce_silu(const ModelDims &md, const GemmShape &g, const float *part, int rows, void *act,
                        hipStream_t st) {
    const size_t plane = (size_t)g.Mpad * g.Npad;
    POSS_DISPATCH(md.dt, hipLaunchKernelGGL((reduce_silu_kernel<T>), dim3((md.ffn + 255) / 256, rows), dim3(256), 0,
                                            st, part, plane, g.S, g.Npad, md.ffn, static_cast<T *>(act)));
}

// ------------------------------------------------------------------ argmax per row (lowest index on ties)
__global__ __launch_bounds__(1024) void argmax_kernel(const float *__restrict__ logits, int ld, int vocab,
                                                      int32_t *__restrict__ out) {
    __shared__ float red_v[17];
    __shared__ int red_i[17];
    const float *row = logits + (size_t)blockIdx.x * ld;
    float bv = -INFINITY; int bi = 0x7fffffff;
    for (int i = threadIdx.x; i < vocab; i += blockDim.x) {
        const float v = row[i];
        if (better(v, i, bv, bi)) { bv = v; bi = i; }
    }
    block_argmax(bv, bi, red_v, red_i);
    if (threadIdx.x == 0) out[blockIdx.x] = bi;
}

void launch_argmax(const float *logits, int ld, int rows, int vocab, int32_t *out, hipStream_t st) {
    hipLaunchKernelGGL(argmax_kernel, dim3(rows), dim3(1024), 0, st, logits, ld, vocab, out);
}

__global__ void copy_rows_f32_kernel(const float *__restrict__ src, int ld_src, float *__restrict__ dst, int ld_dst,
                                     int cols) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c < cols) dst[(size_t)blockIdx.y * ld_dst + c] = src[(size_t)blockIdx.y * ld_src + c];
}

void launch_copy_rows_f32(const float *src, int ld_src, float *dst, int ld_dst, int rows, int cols,
                          hipStream_t st) {
    hipLaunchKernelGGL(copy_rows_f32_kernel, dim3((cols + 255) / 256, rows), dim3(256), 0, st, src, ld_src, dst,
                       ld_dst, cols);
}

__global__ void fill_u32_kernel(uint32_t *p, size_t n, uint32_t v) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

void launch_fill_u32(uint32_t *p, size_t n, uint32_t v, hipStream_t st) {
    if (n == 0) return;
    size_t blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p, n, v);
}

// ------------------------------------------------------------------ debug: cache slots -> float arrays
template <typename T>
__global__ void read_kv_kernel(KVCache kv, int hkv, int dh, int slot0, float *__restrict__ k_out,
                               float *__restrict__ v_out) {
    const int j = blockIdx.x, sl = slot0 + j;
    const T *kc = static_cast<const T *>(kv.k), *vc = static_cast<const T *>(kv.vt);
    for (int p = threadIdx.x; p < hkv * dh; p += blockDim.x) {
        const int h = p / dh, i = p % dh;
        k_out[(size_t)j * hkv * dh + p] = to_f(kc[k_offset(kv, sl, h, hkv, dh) + i]);
        v_out[(size_t)j * hkv * dh + p] = to_f(vc[vt_offset(kv, sl, h, hkv, dh, i)]);
    }
}

void launch_read_kv(const ModelDims &md, const KVCache &kv, int slot0, int n, float *k_out, float *v_out,
                    hipStream_t st) {
    POSS_DISPATCH(md.dt, hipLaunchKernelGGL((read_kv_kernel<T>), dim3(n), dim3(256), 0, st, kv, md.hkv, md.dh,
                                            slot0, k_out, v_out));
}

}  // namespace poss
