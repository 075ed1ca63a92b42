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
                                                         int vocab, int d, float eps, const T *__restrict__ gain,
                                                         float *__restrict__ h, T *__restrict__ u,
                                                         const int32_t *__restrict__ pos,
                                                         const double *__restrict__ inv_freq, int half,
                                                         float2 *__restrict__ cs) {
    __shared__ float red[17];
    const int row = blockIdx.x;
    // the rotary table by the last wave, so that the first ones start on the embedding row at once
    rope_table_row(pos[row], inv_freq, half, cs + (size_t)row * half, half <= 64 && blockDim.x >= 128 ? (int)blockDim.x - 64 : 0);
    const T *e = embed + (size_t)embedding_row(tokens[row], vocab) * d;
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
                                            static_cast<const T *>(embed), tokens, md.vocab, md.d, md.eps,
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
    if (threadIdx.x == 0) out[rowi] = bi == 0x7fffffff ? 0 : bi;        // no logit of the row compared (all NaN): token 0, not an id outside the vocabulary
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

// ------------------------------------------------------------------ drawn children and the rejection rule
// Both kernels cut the vocabulary into blocks of 256 ids (one float4 per lane of a wave: coalesced) and find "the first id
// whose cumulative mass exceeds the target" in two steps: the block (a scan over the block sums), then the id inside it (a
// scan over the lanes of one wave).  Every sum is formed in one fixed order, so a run is repeatable.
constexpr int DRAW_THREADS = 1024, DRAW_BLOCK = 256, DRAW_MAX_BLOCKS = 8192;
typedef float f32x4e __attribute__((ext_vector_type(4)));

struct DrawLds {
    float bsum[DRAW_MAX_BLOCKS];       // mass of every block
    float cum[DRAW_THREADS];           // inclusive scan over the threads' shares of bsum
    float red[17];
    float wave_off[17];
    float f[4]; int i[4];
    int removed[16];
};

// Inclusive scan of one value per thread over the workgroup, in a fixed order: inside a wave by shuffles, the 16 wave
// totals by thread 0.  Returns the inclusive value; *total = the sum of all.
__device__ __forceinline__ float block_scan(float v, DrawLds &L, float *total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const float t = __shfl_up(v, o, 64);
        if (lane >= o) v += t;
    }
    __syncthreads();
    if (lane == 63) L.red[wave] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        float a = 0.f;
        for (int w = 0; w < DRAW_THREADS / 64; ++w) { L.wave_off[w] = a; a += L.red[w]; }
        L.wave_off[16] = a;
    }
    __syncthreads();
    *total = L.wave_off[16];
    return v + L.wave_off[wave];
}

// The block that holds u * (total mass): the first whose inclusive cumulative sum exceeds it; blocks without mass are never
// chosen; if rounding pushed the target past the total, the last block with mass (*before = -inf then).  Every thread
// gets the result.
__device__ __forceinline__ int find_block(DrawLds &L, int nblk, float u, float *before, float *total_out) {
    const int tid = threadIdx.x, per = (nblk + DRAW_THREADS - 1) / DRAW_THREADS, b0 = tid * per, b1 = min(nblk, b0 + per);
    float s = 0.f;
    int last_mass = -1;
    for (int b = b0; b < b1; ++b) { s += L.bsum[b]; if (L.bsum[b] > 0.f) last_mass = b; }
    float total;
    const float incl = block_scan(s, L, &total);
    L.cum[tid] = incl;
    if (tid == 0) { L.i[0] = -1; L.i[1] = -1; }
    __syncthreads();
    const float target = u * total, prev = tid ? L.cum[tid - 1] : 0.f;
    if (last_mass >= 0) atomicMax(&L.i[1], last_mass);
    if (s > 0.f && prev <= target && target < incl) {
        // (prev + the shares one by one may round differently from incl: the last share with mass takes what is left)
        float cumb = prev;
        for (int b = b0; b < b1; ++b) {
            const float w = L.bsum[b];
            if (w > 0.f && (cumb + w > target || b == last_mass)) { L.i[0] = b; L.f[0] = cumb; break; }
            cumb += w;
        }
    }
    __syncthreads();
    *total_out = total;
    if (L.i[0] >= 0) { *before = L.f[0]; return L.i[0]; }
    *before = -INFINITY;
    return L.i[1] < 0 ? 0 : L.i[1];
}

// By wave 0: the id inside block b at which the cumulative mass (mass(id), in id order) exceeds `rest`; with rest = +inf or
// nothing crossing, the last id with mass.  The result goes to L.i[2] (every thread reads it after the barrier that follows).
template <class Mass>
__device__ __forceinline__ void pick_in_block(DrawLds &L, int b, float rest, bool take_last, Mass mass) {
    if (threadIdx.x >= 64) return;
    const int lane = threadIdx.x;
    const f32x4e m = mass(b, lane);
    const float ls = ((m[0] + m[1]) + m[2]) + m[3];
    float incl = ls;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const float t = __shfl_up(incl, o, 64);
        if (lane >= o) incl += t;
    }
    const float prev = incl - ls;                         // (exclusive prefix of this lane)
    int last = -1;
#pragma unroll
    for (int j = 0; j < 4; ++j) if (m[j] > 0.f) last = b * DRAW_BLOCK + lane * 4 + j;
    int mine = -1;
    if (!take_last && ls > 0.f && incl > rest) {          // the crossing falls into this lane's four ids
        float c = prev;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            c += m[j];
            if (mine < 0 && m[j] > 0.f && c > rest) mine = b * DRAW_BLOCK + lane * 4 + j;
        }
        if (mine < 0) mine = last;                        // (prev + the four masses rounded below incl)
    }
    // first crossing lane wins; otherwise the last id with mass
    const unsigned long long crossed = __ballot(mine >= 0);
    int pick;
    if (crossed) {
        const int src = __ffsll((long long)crossed) - 1;
        pick = __shfl(mine, src, 64);
    } else {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) last = max(last, __shfl_xor(last, o, 64));
        pick = last;
    }
    if (lane == 0) L.i[2] = pick;
}

// the four values row[id] of lane's ids in block b (0 where the row ends)
__device__ __forceinline__ f32x4e load_ids(const float *row, int ld, int b, int lane) {
    const int id0 = b * DRAW_BLOCK + lane * 4;
    f32x4e v = f32x4e{0.f, 0.f, 0.f, 0.f};
    if (id0 + 3 < ld) v = *reinterpret_cast<const f32x4e *>(row + id0);
    return v;
}
// their masses exp((l - mx) * inv_t) (0 beyond the vocabulary)
__device__ __forceinline__ f32x4e masses_of(f32x4e v, int vocab, int b, int lane, float mx, float inv_t) {
    const int id0 = b * DRAW_BLOCK + lane * 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = id0 + j < vocab ? expf((v[j] - mx) * inv_t) : 0.f;
    return v;
}
// the four masses exp((row[id] - mx) * inv_t) of lane's ids in block b
__device__ __forceinline__ f32x4e exp_masses(const float *row, int ld, int vocab, int b, int lane, float mx, float inv_t) {
    return masses_of(load_ids(row, ld, b, lane), vocab, b, lane, mx, inv_t);
}
// A wave walks the blocks wave, wave + 16, ...: DRAW_UNROLL of them at a time, their loads asked for together (one block
// after the other, each load waited for, the walk over a 128K-entry row is 31 trips to memory in a row).
constexpr int DRAW_UNROLL = 4, DRAW_WAVES = DRAW_THREADS / 64;

__device__ __forceinline__ float draw_block_max(float v, DrawLds &L) {
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) L.red[threadIdx.x >> 6] = v;
    __syncthreads();
    float m = L.red[0];
    for (int w = 1; w < DRAW_THREADS / 64; ++w) m = fmaxf(m, L.red[w]);
    return m;
}

// the largest of row[0 .. vocab)
__device__ __forceinline__ float row_max(const float *row, int ld, int vocab, int nblk, DrawLds &L) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    float mx = -INFINITY;
    for (int b0 = wave; b0 < nblk; b0 += DRAW_WAVES * DRAW_UNROLL) {
        f32x4e v[DRAW_UNROLL];
#pragma unroll
        for (int u = 0; u < DRAW_UNROLL; ++u) v[u] = load_ids(row, ld, min(b0 + u * DRAW_WAVES, nblk - 1), lane);
#pragma unroll
        for (int u = 0; u < DRAW_UNROLL; ++u) {
            const int b = b0 + u * DRAW_WAVES, id0 = b * DRAW_BLOCK + lane * 4;
            if (b < nblk && id0 + 3 < ld) {
#pragma unroll
                for (int j = 0; j < 4; ++j) if (id0 + j < vocab) mx = fmaxf(mx, v[u][j]);
            }
        }
    }
    return draw_block_max(mx, L);
}

__global__ __launch_bounds__(DRAW_THREADS) void sample_children_kernel(const float *__restrict__ logits, int ld, int vocab, int k,
                                                                       float inv_t, const float *__restrict__ u,
                                                                       int32_t *__restrict__ out_id, float *__restrict__ out_logp) {
    __shared__ DrawLds L;
    const int rowi = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const float *row = logits + (size_t)rowi * ld;
    const int nblk = (vocab + DRAW_BLOCK - 1) / DRAW_BLOCK;
    const float mx = row_max(row, ld, vocab, nblk, L);
    // masses of a block without the ids already drawn (n_removed of them)
    auto masses = [&](int b, int ln, int n_removed) {
        f32x4e m = exp_masses(row, ld, vocab, b, ln, mx, inv_t);
        const int id0 = b * DRAW_BLOCK + ln * 4;
        for (int j = 0; j < n_removed; ++j) {
            const int r = L.removed[j] - id0;
            if (r >= 0 && r < 4) m[r] = 0.f;
        }
        return m;
    };
    for (int b0 = wave; b0 < nblk; b0 += DRAW_WAVES * DRAW_UNROLL) {
        f32x4e v[DRAW_UNROLL];
#pragma unroll
        for (int u = 0; u < DRAW_UNROLL; ++u) v[u] = load_ids(row, ld, min(b0 + u * DRAW_WAVES, nblk - 1), lane);
#pragma unroll
        for (int u = 0; u < DRAW_UNROLL; ++u) {
            const int b = b0 + u * DRAW_WAVES;
            if (b >= nblk) break;                         // wave-uniform
            const f32x4e m = masses_of(v[u], vocab, b, lane, mx, inv_t);
            const float s = wave_sum(((m[0] + m[1]) + m[2]) + m[3]);
            if (lane == 0) L.bsum[b] = s;
        }
    }
    __syncthreads();
    float log_z = 0.f;
    for (int d = 0; d < k; ++d) {
        float before, total;
        const int b = find_block(L, nblk, u[rowi * k + d], &before, &total);
        if (d == 0) log_z = logf(total);                  // the normaliser of the full distribution
        const float target = u[rowi * k + d] * total;
        pick_in_block(L, b, target - before, before == -INFINITY, [&](int bb, int ln) { return masses(bb, ln, d); });
        __syncthreads();
        const int c = L.i[2];
        if (tid == 0) {
            L.removed[d] = c;
            out_id[rowi * k + d] = c;
            out_logp[rowi * k + d] = (row[c] - mx) * inv_t - log_z;
        }
        __syncthreads();
        if (wave == 0) {                                  // the block's mass without the id just drawn, formed afresh
            const f32x4e m = masses(b, lane, d + 1);
            const float s = wave_sum(((m[0] + m[1]) + m[2]) + m[3]);
            if (lane == 0) L.bsum[b] = s;
        }
        __syncthreads();
    }
}

void launch_sample_children(const float *logits, int ld, int rows, int vocab, int k, float temperature, const float *u,
                            int32_t *out_id, float *out_logp, hipStream_t st) {
    hipLaunchKernelGGL(sample_children_kernel, dim3(rows), dim3(DRAW_THREADS), 0, st, logits, ld, vocab, k, 1.0f / temperature, u,
                       out_id, out_logp);
}

__global__ __launch_bounds__(DRAW_THREADS) void rejection_walk_kernel(TreeDev td, int k, int L_depth, int vocab,
                                                                      const float *__restrict__ target_logits,
                                                                      const float *__restrict__ draft_logits, int ld, float inv_t,
                                                                      const float *__restrict__ ua, float *__restrict__ resid,
                                                                      int32_t *__restrict__ g) {
    __shared__ DrawLds L;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int nblk = (vocab + DRAW_BLOCK - 1) / DRAW_BLOCK;
    auto resid_masses = [&](int b, int ln) {
        const int id0 = b * DRAW_BLOCK + ln * 4;
        f32x4e v = f32x4e{0.f, 0.f, 0.f, 0.f};
        if (id0 + 3 < ld) v = *reinterpret_cast<const f32x4e *>(resid + id0);
#pragma unroll
        for (int j = 0; j < 4; ++j) if (id0 + j >= vocab) v[j] = 0.f;
        return v;
    };
    const int n_nodes = td.n_nodes[0];
    for (int i = tid; i < n_nodes; i += DRAW_THREADS) g[i] = -1;
    int cur = 0;
    for (int step = 0; step <= L_depth; ++step) {         // at most L accepted children, then the last token
        const int d = td.depth[cur];
        const float *prow = target_logits + (size_t)cur * ld;
        const float mp = row_max(prow, ld, vocab, nblk, L);
        // which drafter row expanded this node, and where its drawn children sit in the pool
        int e = -1, cbase = 0;
        if (cur == 0) { e = 0; cbase = 0; }
        else if (d < L_depth) {
            const int pv = td.node_pool[cur];
            for (int r = 0; r < k; ++r)
                if (td.fr_pool[d * k + r] == pv) { e = 1 + (d - 1) * k + r; cbase = k + (d - 1) * k * k + r * k; }
        }
        // block sums of the target's masses P = exp((l - max) / T); zp = their total (p = P / zp)
        for (int b0 = wave; b0 < nblk; b0 += DRAW_WAVES * DRAW_UNROLL) {
            f32x4e v[DRAW_UNROLL];
#pragma unroll
            for (int u = 0; u < DRAW_UNROLL; ++u) v[u] = load_ids(prow, ld, min(b0 + u * DRAW_WAVES, nblk - 1), lane);
#pragma unroll
            for (int u = 0; u < DRAW_UNROLL; ++u) {
                const int b = b0 + u * DRAW_WAVES;
                if (b >= nblk) break;                     // wave-uniform
                const f32x4e m = masses_of(v[u], vocab, b, lane, mp, inv_t);
                const float s = wave_sum(((m[0] + m[1]) + m[2]) + m[3]);
                if (lane == 0) L.bsum[b] = s;
            }
        }
        __syncthreads();
        if (e < 0) {                                      // no drawn children: the target's own token ends the walk
            float before, total;
            const float un = ua[d * (k + 1) + k];
            const int b = find_block(L, nblk, un, &before, &total);
            pick_in_block(L, b, un * total - before, before == -INFINITY,
                          [&](int bb, int ln) { return exp_masses(prow, ld, vocab, bb, ln, mp, inv_t); });
            __syncthreads();
            if (tid == 0) g[cur] = L.i[2];
            return;
        }
        float before_unused, zp;
        (void)find_block(L, nblk, 0.f, &before_unused, &zp);
        const float *qrow = draft_logits + (size_t)e * ld;
        const float mq = row_max(qrow, ld, vocab, nblk, L);
        float sq = 0.f;                                   // zq: total of the drafter's masses, same block order
        for (int b0 = wave; b0 < nblk; b0 += DRAW_WAVES * DRAW_UNROLL) {
            f32x4e v[DRAW_UNROLL];
#pragma unroll
            for (int u = 0; u < DRAW_UNROLL; ++u) v[u] = load_ids(qrow, ld, min(b0 + u * DRAW_WAVES, nblk - 1), lane);
#pragma unroll
            for (int u = 0; u < DRAW_UNROLL; ++u) {
                const int b = b0 + u * DRAW_WAVES;
                if (b >= nblk) break;                     // wave-uniform
                const f32x4e m = masses_of(v[u], vocab, b, lane, mq, inv_t);
                sq += ((m[0] + m[1]) + m[2]) + m[3];
            }
        }
        float zq = block_sum(sq, L.red);
        bool have_resid = false;
        int next = -1, last_tok = -1;
        for (int i = 0; i < k; ++i) {
            const int c = td.pool_token[cbase + i];
            const float pc = (have_resid ? resid[c] : expf((prow[c] - mp) * inv_t)) / zp;
            const float ec = expf((qrow[c] - mq) * inv_t), qc = ec / zq;
            const float a = fminf(1.f, pc / qc);
            if (ua[d * (k + 1) + i] < a) {                // accepted (every thread takes the same decision)
                const int node = td.pool_node[cbase + i];
                if (tid == 0) g[cur] = c;
                if (node >= 0) next = node; else last_tok = c;
                break;
            }
            // rejected: P <- max(P / zp - Q / zq, 0) with its block sums, zp <- their total; the candidate leaves q
            __syncthreads();                              // resid[c] has been read by every thread
            for (int b0 = wave; b0 < nblk; b0 += DRAW_WAVES * DRAW_UNROLL) {
                f32x4e pv[DRAW_UNROLL], qv[DRAW_UNROLL];
#pragma unroll
                for (int u = 0; u < DRAW_UNROLL; ++u) {
                    const int b = min(b0 + u * DRAW_WAVES, nblk - 1);
                    pv[u] = load_ids(have_resid ? resid : prow, ld, b, lane);
                    qv[u] = load_ids(qrow, ld, b, lane);
                }
#pragma unroll
                for (int u = 0; u < DRAW_UNROLL; ++u) {
                    const int b = b0 + u * DRAW_WAVES;
                    if (b >= nblk) break;                 // wave-uniform
                    const int id0 = b * DRAW_BLOCK + lane * 4;
                    f32x4e pm = pv[u];
                    if (have_resid) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) if (id0 + j >= vocab) pm[j] = 0.f;
                    } else {
                        pm = masses_of(pm, vocab, b, lane, mp, inv_t);
                    }
                    f32x4e qm = masses_of(qv[u], vocab, b, lane, mq, inv_t);
                    for (int j = 0; j < i; ++j) {
                        const int r = L.removed[j] - id0;
                        if (r >= 0 && r < 4) qm[r] = 0.f;
                    }
                    f32x4e r4;
#pragma unroll
                    for (int j = 0; j < 4; ++j) r4[j] = fmaxf(pm[j] / zp - qm[j] / zq, 0.f);
                    if (id0 + 3 < ld) *reinterpret_cast<f32x4e *>(resid + id0) = r4;
                    const float s = wave_sum(((r4[0] + r4[1]) + r4[2]) + r4[3]);
                    if (lane == 0) L.bsum[b] = s;
                }
            }
            if (tid == 0) L.removed[i] = c;
            __syncthreads();
            (void)find_block(L, nblk, 0.f, &before_unused, &zp);   // (its barriers also publish resid[])
            zq -= ec;
            have_resid = true;
        }
        if (next >= 0) { cur = next; continue; }
        if (last_tok < 0) {                               // every candidate rejected: draw from the last residual
            float before, total;
            const float un = ua[d * (k + 1) + k];
            const int b = find_block(L, nblk, un, &before, &total);
            pick_in_block(L, b, un * total - before, before == -INFINITY, resid_masses);
            __syncthreads();
            if (tid == 0) g[cur] = L.i[2];
        }
        return;
    }
}

void launch_rejection_walk(const TreeDev &td, int k, int L, int vocab, const float *target_logits, const float *draft_logits,
                           int ld, float temperature, const float *ua, float *resid, int32_t *g, hipStream_t st) {
    hipLaunchKernelGGL(rejection_walk_kernel, dim3(1), dim3(DRAW_THREADS), 0, st, td, k, L, vocab, target_logits, draft_logits, ld,
                       1.0f / temperature, ua, resid, g);
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
