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
// (and the row's rotary table, which every layer of the pass uses)
template <typename T>
__global__ __launch_bounds__(256) void embed_norm_kernel(const T *__restrict__ embed, const int32_t *__restrict__ tokens,
                                                         int d, float eps, const T *__restrict__ gain,
                                                         float *__restrict__ h, T *__restrict__ u,
                                                         const int32_t *__restrict__ pos,
                                                         const double *__restrict__ inv_freq, int half,
                                                         float2 *__restrict__ cs) {
    __shared__ float red[17];
    const int row = blockIdx.x;
    // the rotary table by the last wave, so that the first ones start on the embedding row at once
    rope_table_row(pos[row], inv_freq, half, cs + (size_t)row * half, half <= 64 && blockDim.x >= 128 ? (int)blockDim.x - 64 : 0);
    const T *e = embed + (size_t)tokens[row] * d;
    constexpr int VE = 16 / (int)sizeof(T);               // elements per 16-byte access
    constexpr int MAXV = 4;                                // 16-byte pieces a thread keeps (d <= 4 * 256 * VE)
    if (d % VE == 0 && d <= MAXV * 256 * VE && blockDim.x == 256) {
        // one trip to memory: the row and the gains are loaded in 16-byte pieces and kept in registers
        union Piece { uint4 q; T t[VE]; };
        Piece ev[MAXV], gv[MAXV];
        const int nv = d / VE;
#pragma unroll
        for (int j = 0; j < MAXV; ++j) {
            const int p = threadIdx.x + j * 256;
            if (p < nv) {
                ev[j].q = reinterpret_cast<const uint4 *>(e)[p];
                gv[j].q = reinterpret_cast<const uint4 *>(gain)[p];
            }
        }
        float ss = 0.f;                                    // fixed order: a thread's pieces one after the other, element by element
#pragma unroll
        for (int j = 0; j < MAXV; ++j) {
            const int p = threadIdx.x + j * 256;
            if (p < nv) {
#pragma unroll
                for (int x = 0; x < VE; ++x) {
                    const float v = to_f(ev[j].t[x]);
                    h[(size_t)row * d + (size_t)p * VE + x] = v;
                    ss += v * v;
                }
            }
        }
        ss = block_sum(ss, red);
        const float rs = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
        for (int j = 0; j < MAXV; ++j) {
            const int p = threadIdx.x + j * 256;
            if (p < nv) {
                Piece o;
#pragma unroll
                for (int x = 0; x < VE; ++x) o.t[x] = from_f<T>(to_f(ev[j].t[x]) * rs * to_f(gv[j].t[x]));
                reinterpret_cast<uint4 *>(u + (size_t)row * d)[p] = o.q;
            }
        }
        return;
    }
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
                       const void *gain, float *h, void *u, const int32_t *pos, const double *inv_freq,
                       float2 *cs, hipStream_t st) {
    POSS_DISPATCH(md.dt, hipLaunchKernelGGL((embed_norm_kernel<T>), dim3(rows), dim3(256), 0, st,
                                            static_cast<const T *>(embed), tokens, md.d, md.eps,
                                            static_cast<const T *>(gain), h, static_cast<T *>(u), pos, inv_freq,
                                            md.dh / 2, cs));
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

size_t argmax_scratch_floats(int rows, int vocab) { return (size_t)2 * rows * head_segments_max(vocab); }   // finest segmentation: the Head GEMM's tiles

void launch_argmax_merge(const float *pv, const int *pi, int n_seg, int rows, int32_t *out, hipStream_t st) {
    hipLaunchKernelGGL(argmax_merge_kernel, dim3(rows), dim3(64), 0, st, pv, pi, n_seg, out);
}

void launch_argmax(const float *logits, int ld, int rows, int vocab, float *scratch, int32_t *out, hipStream_t st) {
    const int n_seg = (vocab + ARGMAX_SEG - 1) / ARGMAX_SEG;
    float *pv = scratch;
    int *pi = reinterpret_cast<int *>(scratch + (size_t)rows * n_seg);
    hipLaunchKernelGGL(argmax_seg_kernel, dim3(n_seg, rows), dim3(256), 0, st, logits, ld, vocab, n_seg, pv, pi);
    launch_argmax_merge(pv, pi, n_seg, rows, out, st);
}

// ------------------------------------------------------------------ temperature sampling per row
// The token after a row is drawn from softmax(logits / T) by inverse CDF in vocabulary order: the first
// id whose cumulative probability exceeds u.  Stage 1: per (segment, row) the maximum and the sum of
// exp((l - max) / T).  Stage 2: one workgroup per row picks the segment in which u * Z falls, then the
// id inside it.  All sums run in a fixed order: the same inputs give the same token on every run.
constexpr int SAMPLE_SEG = 4096, SAMPLE_PER_THREAD = SAMPLE_SEG / 256;
constexpr int SAMPLE_MAX_SEGS = 1024;

__global__ __launch_bounds__(256) void sample_seg_kernel(const float *__restrict__ logits, int ld, int vocab, int n_seg,
                                                         float inv_t, float *__restrict__ pm, float *__restrict__ pe) {
    __shared__ float red[17];
    const int seg = blockIdx.x, rowi = blockIdx.y;
    const float *row = logits + (size_t)rowi * ld;
    const int i0 = seg * SAMPLE_SEG + threadIdx.x * SAMPLE_PER_THREAD;       // a contiguous run per thread
    float v[SAMPLE_PER_THREAD], mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < SAMPLE_PER_THREAD; ++j) {
        v[j] = i0 + j < vocab ? row[i0 + j] : -INFINITY;
        mx = fmaxf(mx, v[j]);
    }
    mx = wave_max(mx);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float se = 0.f;
#pragma unroll
    for (int j = 0; j < SAMPLE_PER_THREAD; ++j) se += v[j] > -INFINITY ? expf((v[j] - mx) * inv_t) : 0.f;
    se = block_sum(se, red);
    if (threadIdx.x == 0) { pm[rowi * n_seg + seg] = mx; pe[rowi * n_seg + seg] = se; }
}

__global__ __launch_bounds__(256) void sample_pick_kernel(const float *__restrict__ logits, int ld, int vocab, int n_seg,
                                                          float inv_t, const float *__restrict__ pm,
                                                          const float *__restrict__ pe, const float *__restrict__ u_by_depth,
                                                          const int32_t *__restrict__ depth, int32_t *__restrict__ out) {
    __shared__ float w[SAMPLE_MAX_SEGS];
    __shared__ float tsum[256];
    __shared__ float red[17];
    __shared__ int s_seg, s_first, s_last;
    __shared__ float s_rest;
    const int rowi = blockIdx.x, tid = threadIdx.x;
    const float u = u_by_depth[depth ? depth[rowi] : 0];
    float mx = -INFINITY;
    for (int s = tid; s < n_seg; s += 256) mx = fmaxf(mx, pm[rowi * n_seg + s]);
    mx = wave_max(mx);
    if ((tid & 63) == 0) red[tid >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    for (int s = tid; s < n_seg; s += 256) {
        const float m = pm[rowi * n_seg + s];
        w[s] = m > -INFINITY ? pe[rowi * n_seg + s] * expf((m - mx) * inv_t) : 0.f;
    }
    __syncthreads();
    if (tid == 0) {                                       // at most a few dozen segments: one thread, fixed order
        float z = 0.f;
        for (int s = 0; s < n_seg; ++s) z += w[s];
        const float target = u * z;
        float cum = 0.f;
        int pick = -1, last = 0;
        for (int s = 0; s < n_seg; ++s) {
            if (w[s] > 0.f) last = s;
            if (pick < 0 && cum + w[s] > target) { pick = s; s_rest = target - cum; }
            if (pick < 0) cum += w[s];
        }
        if (pick < 0) { pick = last; s_rest = INFINITY; }  // rounding pushed u * Z past the total: last id with mass
        s_seg = pick; s_first = 0x7fffffff; s_last = -1;
    }
    __syncthreads();
    const int seg = s_seg;
    const float rest = s_rest;
    const float *row = logits + (size_t)rowi * ld;
    const int i0 = seg * SAMPLE_SEG + tid * SAMPLE_PER_THREAD;
    float x[SAMPLE_PER_THREAD], ts = 0.f;
#pragma unroll
    for (int j = 0; j < SAMPLE_PER_THREAD; ++j) {
        x[j] = i0 + j < vocab ? expf((row[i0 + j] - mx) * inv_t) : 0.f;
        ts += x[j];
    }
    tsum[tid] = ts;
    __syncthreads();
    float before = 0.f;                                   // mass of the threads before this one, summed in order
    for (int t = 0; t < tid; ++t) before += tsum[t];
    int mine = 0x7fffffff, last_mass = -1;
    float cum = before;
#pragma unroll
    for (int j = 0; j < SAMPLE_PER_THREAD; ++j) {
        if (x[j] > 0.f) last_mass = i0 + j;
        cum += x[j];
        if (mine == 0x7fffffff && cum > rest) mine = i0 + j;
    }
    if (mine != 0x7fffffff) atomicMin(&s_first, mine);
    if (last_mass >= 0) atomicMax(&s_last, last_mass);
    __syncthreads();
    // nothing crossed (rounding pushed the target past the segment's mass): the last id with mass in the segment
    if (tid == 0) out[rowi] = s_first != 0x7fffffff ? s_first : (s_last >= 0 ? s_last : 0);
}

size_t sample_scratch_floats(int rows, int vocab) { return (size_t)2 * rows * ((vocab + SAMPLE_SEG - 1) / SAMPLE_SEG); }

bool launch_sample(const float *logits, int ld, int rows, int vocab, float temperature, const float *u_by_depth,
                   const int32_t *depth, float *scratch, int32_t *out, hipStream_t st) {
    const int n_seg = (vocab + SAMPLE_SEG - 1) / SAMPLE_SEG;
    if (n_seg > SAMPLE_MAX_SEGS || !(temperature > 0.f)) return false;
    float *pm = scratch, *pe = scratch + (size_t)rows * n_seg;
    const float inv_t = 1.0f / temperature;
    hipLaunchKernelGGL(sample_seg_kernel, dim3(n_seg, rows), dim3(256), 0, st, logits, ld, vocab, n_seg, inv_t, pm, pe);
    hipLaunchKernelGGL(sample_pick_kernel, dim3(rows), dim3(256), 0, st, logits, ld, vocab, n_seg, inv_t, pm, pe, u_by_depth,
                       depth, out);
    return true;
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
