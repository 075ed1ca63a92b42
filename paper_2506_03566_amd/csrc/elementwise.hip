// Small kernels around the GEMMs: embedding gather + first RMSNorm, rotary table, argmax, row copies.  All arithmetic in
// float32; values become the storage type only where they are the next GEMM's operand.
#include "device_utils.h"

namespace poss {

#define POSS_DISPATCH(dt, ...)                                               \
    switch (dt) {                                                            \
        case DT_F32:  { using T = float;  __VA_ARGS__; } break;              \
        case DT_BF16: { using T = bf16_t; __VA_ARGS__; } break;              \
        default:      { using T = f16_t;  __VA_ARGS__; } break;              \
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

// ------------------------------------------------------------------ rotary table of one pass
// cs[m][i] = (cos, sin)(pos[m] * theta^(-2i/dh)).  The angle is formed in float64 so positions in
// the thousands keep float32-accurate sines; one table serves every layer of the pass.
__global__ void rope_table_kernel(const int32_t *__restrict__ pos, const double *__restrict__ inv_freq, int half,
                                  float2 *__restrict__ cs) {
    const int m = blockIdx.x, i = threadIdx.x;
    if (i >= half) return;
    double s, c;
    sincos((double)pos[m] * inv_freq[i], &s, &c);
    cs[m * half + i] = make_float2((float)c, (float)s);
}

void launch_rope_table(const int32_t *pos, const double *inv_freq, int half, int rows, float2 *cs, hipStream_t st) {
    hipLaunchKernelGGL(rope_table_kernel, dim3(rows), dim3(half < 64 ? 64 : half), 0, st, pos, inv_freq, half, cs);
}

// ------------------------------------------------------------------ argmax per row (lowest index on ties)
// Two stages so that a 128K-entry row is not one workgroup's serial scan: (segment, row) partial
// winners, then one small workgroup per row over the partials.
constexpr int ARGMAX_SEG = 4096;
__global__ __launch_bounds__(256) void argmax_seg_kernel(const float *__restrict__ logits, int ld, int vocab, int n_seg,
                                                         float *__restrict__ pv, int *__restrict__ pi) {
    __shared__ float red_v[17];
    __shared__ int red_i[17];
    const int seg = blockIdx.x, rowi = blockIdx.y;
    const float *row = logits + (size_t)rowi * ld;
    float bv = -INFINITY; int bi = 0x7fffffff;
    const int end = min(vocab, (seg + 1) * ARGMAX_SEG);
    for (int i = seg * ARGMAX_SEG + threadIdx.x; i < end; i += blockDim.x) {
        const float v = row[i];
        if (better(v, i, bv, bi)) { bv = v; bi = i; }
    }
    block_argmax(bv, bi, red_v, red_i);
    if (threadIdx.x == 0) { pv[rowi * n_seg + seg] = bv; pi[rowi * n_seg + seg] = bi; }
}

__global__ __launch_bounds__(64) void argmax_merge_kernel(const float *__restrict__ pv, const int *__restrict__ pi, int n_seg,
                                                          int32_t *__restrict__ out) {
    const int rowi = blockIdx.x;
    float bv = -INFINITY; int bi = 0x7fffffff;
    for (int s = threadIdx.x; s < n_seg; s += 64) {
        const float v = pv[rowi * n_seg + s]; const int i = pi[rowi * n_seg + s];
        if (better(v, i, bv, bi)) { bv = v; bi = i; }
    }
    wave_argmax(bv, bi);
    if (threadIdx.x == 0) out[rowi] = bi;
}

size_t argmax_scratch_floats(int rows, int vocab) { return (size_t)2 * rows * ((vocab + ARGMAX_SEG - 1) / ARGMAX_SEG); }

void launch_argmax(const float *logits, int ld, int rows, int vocab, float *scratch, int32_t *out, hipStream_t st) {
    const int n_seg = (vocab + ARGMAX_SEG - 1) / ARGMAX_SEG;
    float *pv = scratch;
    int *pi = reinterpret_cast<int *>(scratch + (size_t)rows * n_seg);
    hipLaunchKernelGGL(argmax_seg_kernel, dim3(n_seg, rows), dim3(256), 0, st, logits, ld, vocab, n_seg, pv, pi);
    hipLaunchKernelGGL(argmax_merge_kernel, dim3(rows), dim3(64), 0, st, pv, pi, n_seg, out);
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
