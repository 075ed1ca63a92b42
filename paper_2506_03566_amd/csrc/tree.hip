// Draft-tree kernels: log-softmax + top-k of the drafter's logits, level-by-level expansion with a
// width-k frontier, final top-N rerank and tree emission (tree drafting with width / depth / total
// tokens, section 4.1 "Implementations" of the paper), assembly of the [embedding ; feature] rows a
// specialist consumes (Eq. 2 / Eq. 9), greedy acceptance walk and commit (section 2.1, 3.1).
//
// Ordering rules, identical everywhere: larger value first; ties to the lower token id (children of
// one node) or the earlier candidate (anything else).  Candidate order = (depth, rank of the parent
// in its frontier, rank of the child among its siblings).  Scores are float32 running sums of
// log-probabilities.  All selection is by rank counting, so results do not depend on thread timing.
#include "device_utils.h"

namespace poss {

// ------------------------------------------------------------------ top-k + log-sum-exp
// Selection of the k best (value, index) pairs held NV per thread by a 256-thread workgroup.
// block_topk_rounds: every wave extracts its own k best with shuffles only (no workgroup barrier
// inside the k rounds), then wave 0 picks the k best of the 4k survivors.
// block_topk: threshold first.  The k-th largest of any 64 of the per-thread maxima (one wave's) is a
// lower bound of the k-th largest element; the largest of the four waves' bounds is used, so every
// winner is among the elements >= it: a few dozen, ranked by counting.  No chain of dependent
// shuffles; the rounds remain as the fallback for inputs with more than TOPK_CAND elements above
// the bound (long runs of equal values).
// Either way thread r < k ends up with the r-th best, (-inf, 0x7fffffff...) where fewer than k exist.
constexpr int TOPK_SEG = 2048;
constexpr int TOPK_CAND = 256;
struct __attribute__((aligned(16))) TopkLds {
    float tmax[256];
    float cand_v[TOPK_CAND]; int cand_i[TOPK_CAND];
    float out_v[TOPK_MAXK]; int out_i[TOPK_MAXK];
    float rounds_v[4 * TOPK_MAXK]; int rounds_i[4 * TOPK_MAXK];
    float thr_w[4]; int cnt;
};

template <int NV>
__device__ __forceinline__ void block_topk_rounds(float (&v)[NV], int (&id)[NV], int k, float *s_val, int *s_id,
                                                  float &out_v, int &out_i) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int r = 0; r < k; ++r) {
        float bv = -INFINITY; int bi = 0x7fffffff;
#pragma unroll
        for (int j = 0; j < NV; ++j)
            if (better(v[j], id[j], bv, bi)) { bv = v[j]; bi = id[j]; }
        wave_argmax(bv, bi);
        if (lane == 0) { s_val[wave * TOPK_MAXK + r] = bv; s_id[wave * TOPK_MAXK + r] = bi; }
#pragma unroll
        for (int j = 0; j < NV; ++j)
            if (id[j] == bi) v[j] = -INFINITY;           // indices are unique: removes exactly the winner
    }
    __syncthreads();
    out_v = -INFINITY; out_i = 0x7fffffff;
    if (wave == 0) {
        const int w = lane / TOPK_MAXK, r = lane % TOPK_MAXK;
        float cv = -INFINITY; int ci = 0x7fffffff;
        if (w < (int)(blockDim.x >> 6) && r < k) { cv = s_val[w * TOPK_MAXK + r]; ci = s_id[w * TOPK_MAXK + r]; }
        for (int r2 = 0; r2 < k; ++r2) {
            float bv = cv; int bi = ci;
            wave_argmax(bv, bi);
            if (lane == r2) { out_v = bv; out_i = bi; }
            if (ci == bi) cv = -INFINITY;
        }
    }
}

template <int NV>
__device__ __forceinline__ void block_topk(float (&v)[NV], int (&id)[NV], int k, TopkLds &L, float &out_v, int &out_i) {
    const int tid = threadIdx.x;                          // blockDim.x == 256
    float tm = -INFINITY;
#pragma unroll
    for (int j = 0; j < NV; ++j) tm = fmaxf(tm, v[j]);
    const int lane = tid & 63, wave = tid >> 6;
    L.tmax[tid] = tm;
    if (tid == 0) L.cnt = 0;
    if (tid < 4) L.thr_w[tid] = -INFINITY;
    if (tid < TOPK_MAXK) { L.out_v[tid] = -INFINITY; L.out_i[tid] = 0x7fffffff; }
    __syncthreads();
    int rank = 0;                                         // of this thread's maximum within its wave, ties to the lower lane
    for (int j = 0; j < 64; j += 4) {
        const float4 o = *reinterpret_cast<const float4 *>(&L.tmax[wave * 64 + j]);
        rank += (o.x > tm) || (o.x == tm && j < lane);
        rank += (o.y > tm) || (o.y == tm && j + 1 < lane);
        rank += (o.z > tm) || (o.z == tm && j + 2 < lane);
        rank += (o.w > tm) || (o.w == tm && j + 3 < lane);
    }
    if (rank == k - 1) L.thr_w[wave] = tm;                // exactly one lane per wave (k <= 16 < 64)
    __syncthreads();
    const float thr = fmaxf(fmaxf(L.thr_w[0], L.thr_w[1]), fmaxf(L.thr_w[2], L.thr_w[3]));
#pragma unroll
    for (int j = 0; j < NV; ++j)
        if (v[j] > -INFINITY && v[j] >= thr) {
            const int p = atomicAdd(&L.cnt, 1);           // arrival order does not matter: ranks are by (value, index)
            if (p < TOPK_CAND) { L.cand_v[p] = v[j]; L.cand_i[p] = id[j]; }
        }
    __syncthreads();
    const int cnt = L.cnt;
    if (cnt > TOPK_CAND) {                                // workgroup-uniform
        block_topk_rounds<NV>(v, id, k, L.rounds_v, L.rounds_i, out_v, out_i);
        return;
    }
    if (tid < cnt) {
        const float cv = L.cand_v[tid]; const int ci = L.cand_i[tid];
        int r = 0;
        for (int j = 0; j < cnt; ++j) r += better(L.cand_v[j], L.cand_i[j], cv, ci);
        if (r < k) { L.out_v[r] = cv; L.out_i[r] = ci; }
    }
    __syncthreads();
    out_v = -INFINITY; out_i = 0x7fffffff;
    if (tid < k) { out_v = L.out_v[tid]; out_i = L.out_i[tid]; }
}

// stage 1: one workgroup per (segment of <= TOPK_SEG logits, row): segment maximum, sum of
// exp(l - max) and the segment's k best.  record: [max, sumexp, k values, k indices (as bits)]
__global__ __launch_bounds__(256) void topk_seg_kernel(const float *__restrict__ logits, int ld, int vocab, int k,
                                                       int n_seg, float *__restrict__ seg_out) {
    constexpr int NV = TOPK_SEG / 256;
    __shared__ TopkLds lds;
    __shared__ float red[17];
    const int seg = blockIdx.x, row = blockIdx.y;
    const int base = seg * TOPK_SEG;
    const float *src = logits + (size_t)row * ld;
    float v[NV]; int id[NV];
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int i = base + threadIdx.x + j * 256;
        const bool ok = i < vocab;
        v[j] = ok ? src[i] : -INFINITY;
        id[j] = ok ? i : 0x7fffffff - j;                  // distinct dummies keep "indices are unique" true
        mx = fmaxf(mx, v[j]);
    }
    mx = wave_max(mx);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float se = 0.f;
#pragma unroll
    for (int j = 0; j < NV; ++j) se += v[j] > -INFINITY ? expf(v[j] - mx) : 0.f;
    se = block_sum(se, red);
    float *rec = seg_out + ((size_t)row * n_seg + seg) * (2 + 2 * TOPK_MAXK);
    if (threadIdx.x == 0) { rec[0] = mx; rec[1] = se; }
    float ov; int oi;
    block_topk<NV>(v, id, k, lds, ov, oi);
    if ((int)threadIdx.x < k) {
        rec[2 + threadIdx.x] = ov;
        reinterpret_cast<int *>(rec)[2 + TOPK_MAXK + threadIdx.x] = ov > -INFINITY ? oi : 0x7fffffff;
    }
}

// The merge in two trips, tried first: a segment's values are sorted, so its first value decides whether anything of it
// can be among the k best.  Trip 1 fetches (max, sum of exponentials, best value) of every segment, up to NT per thread;
// the threshold is formed as in block_topk, from the threads' best values; trip 2 fetches the k values of the few
// segments whose best value reaches it.  Returns false, with nothing written, when more than TOPK_CAND candidates sit at
// the threshold (long runs of equal values): the caller then merges in full.  *lse_out: the row's log-sum-exp.
template <int NT>
__device__ __forceinline__ bool topk_merge_heads(const float *__restrict__ recs, int n_seg, int k, TopkLds &L, float *red,
                                                 float &ov, int &oi, float &lse_out) {
    constexpr int REC = TOPK_REC;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float m_s[NT], z_s[NT], v0[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {                        // unconditional loads: a segment that does not exist reads segment 0
        const int sg = tid + j * 256;
        const float *r = recs + (sg < n_seg ? (size_t)sg * REC : 0);
        m_s[j] = r[0]; z_s[j] = r[1]; v0[j] = r[2];
        const int i0 = reinterpret_cast<const int *>(r)[2 + TOPK_MAXK];
        if (sg >= n_seg) { m_s[j] = -INFINITY; z_s[j] = 0.f; v0[j] = -INFINITY; }
        else if (i0 == 0x7fffffff) v0[j] = -INFINITY;     // a segment without a valid entry
    }
    float mx = -INFINITY, tm = -INFINITY;
#pragma unroll
    for (int j = 0; j < NT; ++j) { mx = fmaxf(mx, m_s[j]); tm = fmaxf(tm, v0[j]); }
    mx = wave_max(mx);
    L.tmax[tid] = tm;
    if (tid == 0) L.cnt = 0;
    if (tid < 4) L.thr_w[tid] = -INFINITY;
    if (tid < TOPK_MAXK) { L.out_v[tid] = -INFINITY; L.out_i[tid] = 0x7fffffff; }
    if (lane == 0) red[wave] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float se = 0.f;
#pragma unroll
    for (int j = 0; j < NT; ++j) se += m_s[j] > -INFINITY ? z_s[j] * expf(m_s[j] - mx) : 0.f;
    int rank = 0;                                         // of this thread's best value within its wave, ties to the lower lane
    for (int j = 0; j < 64; j += 4) {
        const float4 o = *reinterpret_cast<const float4 *>(&L.tmax[wave * 64 + j]);
        rank += (o.x > tm) || (o.x == tm && j < lane);
        rank += (o.y > tm) || (o.y == tm && j + 1 < lane);
        rank += (o.z > tm) || (o.z == tm && j + 2 < lane);
        rank += (o.w > tm) || (o.w == tm && j + 3 < lane);
    }
    if (rank == k - 1) L.thr_w[wave] = tm;
    se = block_sum(se, red);                              // (its barriers also publish thr_w)
    lse_out = mx + logf(se);
    const float thr = fmaxf(fmaxf(L.thr_w[0], L.thr_w[1]), fmaxf(L.thr_w[2], L.thr_w[3]));
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        if (!(v0[j] > -INFINITY && v0[j] >= thr)) continue;
        const float *r = recs + (size_t)(tid + j * 256) * REC;
        float cv[TOPK_MAXK]; int ci[TOPK_MAXK];           // the whole record at once: one more trip, not k
#pragma unroll
        for (int q = 0; q < TOPK_MAXK; ++q) { cv[q] = r[2 + q]; ci[q] = reinterpret_cast<const int *>(r)[2 + TOPK_MAXK + q]; }
#pragma unroll
        for (int q = 0; q < TOPK_MAXK; ++q) {
            if (q < k && cv[q] >= thr && ci[q] != 0x7fffffff) {
                const int p = atomicAdd(&L.cnt, 1);       // arrival order does not matter: ranks are by (value, index)
                if (p < TOPK_CAND) { L.cand_v[p] = cv[q]; L.cand_i[p] = ci[q]; }
            }
        }
    }
    __syncthreads();
    const int cnt = L.cnt;
    if (cnt > TOPK_CAND) { __syncthreads(); return false; }   // (workgroup-uniform; L is reused by the full merge)
    if (tid < cnt) {
        const float cv = L.cand_v[tid]; const int ci = L.cand_i[tid];
        int r = 0;
        for (int j = 0; j < cnt; ++j) r += better(L.cand_v[j], L.cand_i[j], cv, ci);
        if (r < k) { L.out_v[r] = cv; L.out_i[r] = ci; }
    }
    __syncthreads();
    ov = -INFINITY; oi = 0x7fffffff;
    if (tid < k) { ov = L.out_v[tid]; oi = L.out_i[tid]; }
    return true;
}

// stage 2: one workgroup per row merges the segments: lse over the segment records, then the k
// best of the n_seg * k candidates; writes token ids and log-probabilities (value - lse).
// NV candidates per thread: 8 (up to 2048: the records of topk_seg_kernel), 32 or 64 (the records of a Head GEMM,
// one per column tile: up to 1002 x 16)
template <int TOPK_MERGE_NV>
__global__ __launch_bounds__(256) void topk_merge_kernel(const float *__restrict__ seg_out, int n_seg, int k,
                                                         int32_t *__restrict__ out_id, float *__restrict__ out_logp) {
    __shared__ TopkLds lds;
    __shared__ float red[17];
    const int row = blockIdx.x, nc = n_seg * k;
    constexpr int REC = TOPK_REC;
    const float *recs = seg_out + (size_t)row * n_seg * REC;
    if (n_seg <= 4 * 256) {                               // (workgroup-uniform) the short way first
        float hv, hl; int hi;
        if (topk_merge_heads<4>(recs, n_seg, k, lds, red, hv, hi, hl)) {
            if ((int)threadIdx.x < k) {
                out_id[row * k + threadIdx.x] = hi;
                out_logp[row * k + threadIdx.x] = hv - hl;
            }
            return;
        }
    }
    // The full merge.  Every load is issued before the first reduction, unconditionally (an entry that does not exist
    // reads slot 0 of segment 0 and is discarded afterwards): one trip to memory, not one per step.
    float v[TOPK_MERGE_NV]; int id[TOPK_MERGE_NV];
#pragma unroll
    for (int j = 0; j < TOPK_MERGE_NV; ++j) {
        const int c = threadIdx.x + j * 256;
        const bool exists = c < nc;
        const float *r = recs + (exists ? (size_t)(c / k) * REC + c % k : 0);
        const float cv = r[2];
        const int ci = reinterpret_cast<const int *>(r)[2 + TOPK_MAXK];
        const bool ok = exists && ci != 0x7fffffff;
        v[j] = ok ? cv : -INFINITY; id[j] = ok ? ci : 0x7fffffff - j;
    }
    const bool own = (int)threadIdx.x < n_seg;            // this thread's segment record (more than 256 segments: the loops)
    const float m0 = recs[own ? (size_t)threadIdx.x * REC : 0], z0 = recs[(own ? (size_t)threadIdx.x * REC : 0) + 1];
    float mx = own ? m0 : -INFINITY;
    for (int s = threadIdx.x + 256; s < n_seg; s += 256) mx = fmaxf(mx, recs[(size_t)s * REC]);
    mx = wave_max(mx);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float se = own ? z0 * expf(m0 - mx) : 0.f;
    for (int s = threadIdx.x + 256; s < n_seg; s += 256) {
        const float *r = recs + (size_t)s * REC;
        se += r[1] * expf(r[0] - mx);
    }
    se = block_sum(se, red);
    const float lse = mx + logf(se);
    float ov; int oi;
    block_topk<TOPK_MERGE_NV>(v, id, k, lds, ov, oi);
    if ((int)threadIdx.x < k) {
        out_id[row * k + threadIdx.x] = oi;
        out_logp[row * k + threadIdx.x] = ov - lse;
    }
}

void launch_topk_merge(const float *seg_records, int n_seg, int rows, int k, int32_t *out_id, float *out_logp, hipStream_t st) {
    const int nc = n_seg * k;
    if (nc <= 8 * 256)
        hipLaunchKernelGGL((topk_merge_kernel<8>), dim3(rows), dim3(256), 0, st, seg_records, n_seg, k, out_id, out_logp);
    else if (nc <= 32 * 256)
        hipLaunchKernelGGL((topk_merge_kernel<32>), dim3(rows), dim3(256), 0, st, seg_records, n_seg, k, out_id, out_logp);
    else                                                   // nc <= 64 * 256: checked when the context is configured
        hipLaunchKernelGGL((topk_merge_kernel<64>), dim3(rows), dim3(256), 0, st, seg_records, n_seg, k, out_id, out_logp);
}

void launch_topk_logsoftmax(const float *logits, int ld, int rows, int vocab, int k, float *seg_scratch,
                            int32_t *out_id, float *out_logp, hipStream_t st) {
    const int n_seg = (vocab + TOPK_SEG - 1) / TOPK_SEG;
    hipLaunchKernelGGL(topk_seg_kernel, dim3(n_seg, rows), dim3(256), 0, st, logits, ld, vocab, k, n_seg, seg_scratch);
    launch_topk_merge(seg_scratch, n_seg, rows, k, out_id, out_logp, st);
}

size_t topk_scratch_floats(int rows, int vocab) {      // the Head GEMM's column tiles are the finer segmentation
    return (size_t)rows * head_segments_max(vocab) * TOPK_REC;
}

// ------------------------------------------------------------------ expansion of one depth
// Children of the frontier of depth d-1 (the root for d = 1) join the candidate pool; unless d = L,
// the k best of them become the frontier of depth d.  A frontier node's drafter row lives in temp
// slot (d-1)*k + rank; fr_mask collects the temp slots of the node and its drafted ancestors.
// One workgroup per sequence of the batch.
struct TreeBatch {
    TreeDev td[TREE_BATCH_MAX];
    int t[TREE_BATCH_MAX];
    const int32_t *tokens_dev[TREE_BATCH_MAX];
    int32_t *slot_out[TREE_BATCH_MAX];
};

__global__ __launch_bounds__(256) void tree_expand_kernel(TreeBatch tb, int d, int k, int L, int rows, int vocab) {
    __shared__ float sc[256];
    const TreeDev &td = tb.td[blockIdx.x];
    const int n_child = rows * k;
    const int base = d == 1 ? 0 : k + (d - 2) * k * k;
    const int tid = threadIdx.x;
    uint64_t pw0 = 0ull, pw1 = 0ull;                      // the parent's ancestor mask, asked for with the rest
    if (tid < n_child) {
        const int r = tid / k;
        const float ps = d == 1 ? 0.f : td.fr_score[(d - 1) * k + r];
        if (d > 1 && d < L) { pw0 = td.fr_mask[((d - 1) * k + r) * MASK_WORDS]; pw1 = td.fr_mask[((d - 1) * k + r) * MASK_WORDS + 1]; }
        // A score that is not a number (a drafter fed NaN) would compare false with everything: every child would rank
        // first here and every candidate be kept by the final ranking, beyond the tree's arrays.  It counts as -inf
        // (ties go by index), and an id that is no vocabulary entry as token 0.
        float s = ps + td.topk_logp[tid];
        if (!(s == s)) s = -INFINITY;
        sc[tid] = s;
        const int tok = embedding_row(td.topk_id[tid], vocab);
        td.pool_token[base + tid] = tok;
        td.pool_parent[base + tid] = d == 1 ? -1 : td.fr_pool[(d - 1) * k + r];
        td.pool_depth[base + tid] = d;
        td.pool_score[base + tid] = s;
    }
    __syncthreads();
    if (d < L && tid < n_child) {
        const float s = sc[tid];
        int rank = 0;
        for (int j = 0; j < n_child; ++j) rank += (sc[j] > s) || (sc[j] == s && j < tid);
        if (rank < k) {
            const int r = tid / k, o = d * k + rank;
            td.fr_pool[o] = base + tid;
            td.fr_token[o] = embedding_row(td.topk_id[tid], vocab);
            td.fr_parent_rank[o] = r;
            td.fr_score[o] = s;
            const int bit = (d - 1) * k + rank;
            uint64_t w0 = pw0, w1 = pw1;
            if (bit < 64) w0 |= 1ull << bit; else w1 |= 1ull << (bit - 64);
            td.fr_mask[o * MASK_WORDS] = w0;
            td.fr_mask[o * MASK_WORDS + 1] = w1;
        }
    }
}

void launch_tree_expand(const TreeDev *tds, int n_seq, int d, int k, int L, int rows, int vocab, hipStream_t st) {
    if (n_seq < 1 || n_seq > TREE_BATCH_MAX) return;
    TreeBatch tb{};
    for (int i = 0; i < n_seq; ++i) tb.td[i] = tds[i];
    hipLaunchKernelGGL(tree_expand_kernel, dim3(n_seq), dim3(256), 0, st, tb, d, k, L, rows, vocab);
}

// ------------------------------------------------------------------ rerank + emit
// Keep the n_keep best candidates; order them as candidates are ordered (parents first); node 0 is
// the root x_t.  pos = t + depth; mask = node and its ancestors; slot = t + node index.
constexpr int POOL_MAX = 2048;
constexpr int POSS_TREE_MAX_DEPTH = 16;              // the deepest tree a context can be configured for
__global__ __launch_bounds__(1024) void tree_finalize_kernel(TreeBatch tb, int pool_n, int n_keep) {
    const TreeDev &td = tb.td[blockIdx.x];
    const int t = tb.t[blockIdx.x];
    const int32_t *__restrict__ tokens_dev = tb.tokens_dev[blockIdx.x];
    int32_t *__restrict__ slot_out = tb.slot_out[blockIdx.x];
    __shared__ __attribute__((aligned(16))) float sc[POOL_MAX];
    __shared__ int16_t par[POOL_MAX];                 // candidate -> parent candidate (-1: the root)
    __shared__ int16_t new_idx[POOL_MAX];             // candidate -> node index in the tree, -1 if dropped
    __shared__ int wave_cnt[2 * 16];                  // kept candidates per (pass, wave)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int my_token[2], my_depth[2];                     // of candidates tid and tid + 1024: asked for with the scores
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int i = tid + p * 1024;
        my_token[p] = 0; my_depth[p] = 0;
        if (i < pool_n) {
            sc[i] = td.pool_score[i]; par[i] = (int16_t)td.pool_parent[i];
            my_token[p] = td.pool_token[i]; my_depth[p] = td.pool_depth[i];
        } else if (i < ((pool_n + 3) & ~3)) {
            sc[i] = -INFINITY;                        // the ranking reads the scores four at a time
        }
    }
    __syncthreads();
    // rank by counting; node index = 1 + number of kept candidates before this one (candidate order is
    // kept, so parents come first), from wave ballots instead of a serial scan
    bool keep[2];
    int before[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int i = tid + p * 1024;
        keep[p] = false;
        if (i < pool_n) {
            const float s = sc[i];
            int rank = 0;
            for (int j = 0; j < pool_n; j += 4) {
                const float4 o = *reinterpret_cast<const float4 *>(&sc[j]);
                rank += (o.x > s) || (o.x == s && j < i);
                rank += (o.y > s) || (o.y == s && j + 1 < i);
                rank += (o.z > s) || (o.z == s && j + 2 < i);
                rank += (o.w > s) || (o.w == s && j + 3 < i);
            }
            keep[p] = rank < n_keep;
        }
        const unsigned long long b = __ballot(keep[p]);
        before[p] = __popcll(b & ((1ull << lane) - 1ull));
        if (lane == 0) wave_cnt[p * 16 + wave] = __popcll(b);
    }
    __syncthreads();
    int total = 0;
    for (int w = 0; w < 32; ++w) total += wave_cnt[w];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int i = tid + p * 1024;
        int off = 0;
        for (int w = 0; w < p * 16 + wave; ++w) off += wave_cnt[w];
        if (i < pool_n) {
            new_idx[i] = keep[p] ? (int16_t)(off + before[p] + 1) : (int16_t)-1;
            td.pool_node[i] = new_idx[i];
            if (keep[p]) td.node_pool[new_idx[i]] = i;
        }
    }
    if (tid == 0) {
        td.n_nodes[0] = total + 1;
        td.token[0] = tokens_dev[t]; td.parent[0] = -1; td.depth[0] = 0; td.pos[0] = t; td.score[0] = 0.f;
        td.mask[0] = 1ull; td.mask[1] = 0ull;
        td.node_pool[0] = -1;
        slot_out[0] = t;
    }
    __syncthreads();
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int i = tid + p * 1024;
        if (i >= pool_n) continue;
        const int ni = new_idx[i];
        if (ni < 0) continue;
        const int pp = par[i], dep = my_depth[p];
        td.token[ni] = my_token[p];
        td.parent[ni] = pp < 0 ? 0 : new_idx[pp];
        td.depth[ni] = dep;
        td.pos[ni] = t + dep;
        slot_out[ni] = t + ni;
        td.score[ni] = sc[i];
        uint64_t w0 = 1ull, w1 = 0ull;               // the root
        for (int u = i, hops = 0; u >= 0 && hops <= POSS_TREE_MAX_DEPTH; u = par[u], ++hops) {   // (bounded: a node has at most depth ancestors)
            const int bit = new_idx[u];
            if (bit < 64) w0 |= 1ull << bit; else w1 |= 1ull << (bit - 64);
        }
        td.mask[ni * MASK_WORDS] = w0;
        td.mask[ni * MASK_WORDS + 1] = w1;
    }
}

void launch_tree_finalize(const TreeDev *tds, int n_seq, int k, int L, int n_keep, const int *t,
                          const int32_t *const *tokens_dev, int32_t *const *slot_out, hipStream_t st) {
    if (n_seq < 1 || n_seq > TREE_BATCH_MAX) return;
    const int pool_n = k + (L - 1) * k * k;
    TreeBatch tb{};
    for (int i = 0; i < n_seq; ++i) { tb.td[i] = tds[i]; tb.t[i] = t[i]; tb.tokens_dev[i] = tokens_dev[i]; tb.slot_out[i] = slot_out[i]; }
    hipLaunchKernelGGL(tree_finalize_kernel, dim3(n_seq), dim3(1024), 0, st, tb, pool_n, n_keep < pool_n ? n_keep : pool_n);
}

// ------------------------------------------------------------------ rows of one specialist pass
template <typename T>
__global__ __launch_bounds__(256) void draft_assemble_kernel(
    DraftRowPlan plan, int depth_index, int k, int d_model, int vocab, const T *__restrict__ embed,
    const int32_t *__restrict__ tokens_dev, const T *__restrict__ feat_stash, TreeDev td,
    const float *__restrict__ fhat_prev, T *__restrict__ xin_tmp, T *__restrict__ x_out,
    int32_t *__restrict__ pos_out, int32_t *__restrict__ slot_out, uint64_t *__restrict__ mask_out,
    const double *__restrict__ inv_freq, int half, float2 *__restrict__ cs) {
    const int prow = blockIdx.x, kind = plan.kind[prow], idx = plan.idx[prow], row = plan.dst[prow];
    // the pass's rotary table, row by row; by the last wave, which has the least copying to do
    rope_table_row(plan.pos[prow], inv_freq, half, cs + (size_t)row * half, half <= 64 ? (int)blockDim.x - 64 : 0);
    T *dst = x_out + (size_t)row * 2 * d_model;
    uint64_t w0 = plan.mask0[0], w1 = plan.mask0[1];
    constexpr int VE = 16 / (int)sizeof(T);              // elements per 16-byte access
    const bool vec = d_model % VE == 0;
    const int nv = d_model / VE;
    if (kind == 0) {                    // committed pair [x_{i+1} ; f_i]
        const T *e = embed + (size_t)embedding_row(tokens_dev[idx + 1], vocab) * d_model, *f = feat_stash + (size_t)idx * d_model;
        if (vec) {
            const uint4 *e4 = reinterpret_cast<const uint4 *>(e), *f4 = reinterpret_cast<const uint4 *>(f);
            uint4 *d4 = reinterpret_cast<uint4 *>(dst);
            for (int i = threadIdx.x; i < nv; i += blockDim.x) { d4[i] = e4[i]; d4[nv + i] = f4[i]; }
        } else {
            for (int i = threadIdx.x; i < d_model; i += blockDim.x) { dst[i] = e[i]; dst[d_model + i] = f[i]; }
        }
    } else if (kind == 1) {             // a frontier row of an earlier depth, as assembled then
        const T *src = xin_tmp + (size_t)idx * 2 * d_model;
        if (vec) {
            const uint4 *s4 = reinterpret_cast<const uint4 *>(src);
            uint4 *d4 = reinterpret_cast<uint4 *>(dst);
            for (int i = threadIdx.x; i < 2 * nv; i += blockDim.x) d4[i] = s4[i];
        } else {
            for (int i = threadIdx.x; i < 2 * d_model; i += blockDim.x) dst[i] = src[i];
        }
    } else {                            // new frontier row: [emb(token_v) ; drafted feature of parent(v)]
        const int o = depth_index * k + idx;
        const T *e = embed + (size_t)embedding_row(td.fr_token[o], vocab) * d_model;
        const float *f = fhat_prev + (size_t)td.fr_parent_rank[o] * d_model;
        T *keep = xin_tmp + (size_t)((depth_index - 1) * k + idx) * 2 * d_model;
        if (vec) {
            const uint4 *e4 = reinterpret_cast<const uint4 *>(e);
            uint4 *d4 = reinterpret_cast<uint4 *>(dst), *k4 = reinterpret_cast<uint4 *>(keep);
            for (int i = threadIdx.x; i < nv; i += blockDim.x) {
                const uint4 ev = e4[i];
                union { uint4 q; T t[VE]; } fv;
#pragma unroll
                for (int j = 0; j < VE; j += 4) {
                    const float4 x = *reinterpret_cast<const float4 *>(f + (size_t)i * VE + j);
                    fv.t[j] = from_f<T>(x.x); fv.t[j + 1] = from_f<T>(x.y); fv.t[j + 2] = from_f<T>(x.z); fv.t[j + 3] = from_f<T>(x.w);
                }
                d4[i] = ev; d4[nv + i] = fv.q;
                k4[i] = ev; k4[nv + i] = fv.q;
            }
        } else {
            for (int i = threadIdx.x; i < d_model; i += blockDim.x) {
                const T ev = e[i], fv = from_f<T>(f[i]);
                dst[i] = ev; dst[d_model + i] = fv;
                keep[i] = ev; keep[d_model + i] = fv;
            }
        }
        w0 = td.fr_mask[o * MASK_WORDS]; w1 = td.fr_mask[o * MASK_WORDS + 1];
    }
    if (threadIdx.x == 0) {
        pos_out[row] = plan.pos[prow];
        slot_out[row] = plan.slot[prow];
        mask_out[row * MASK_WORDS] = w0;
        mask_out[row * MASK_WORDS + 1] = w1;
    }
}

void launch_draft_assemble(const ModelDims &md, const DraftRowPlan &plan, int depth_index, int k,
                           const void *embed, const int32_t *tokens_dev, const void *feat_stash,
                           const TreeDev &td, const float *fhat_prev, void *xin_tmp, void *x_out,
                           int32_t *pos_out, int32_t *slot_out, uint64_t *mask_out, const double *inv_freq,
                           float2 *cs, hipStream_t st) {
#define POSS_ASM(T)                                                                                          \
    hipLaunchKernelGGL((draft_assemble_kernel<T>), dim3(plan.n_rows), dim3(256), 0, st, plan, depth_index, k,   \
                       md.d, md.vocab, static_cast<const T *>(embed), tokens_dev, static_cast<const T *>(feat_stash), td, \
                       fhat_prev, static_cast<T *>(xin_tmp), static_cast<T *>(x_out), pos_out, slot_out, mask_out, \
                       inv_freq, md.dh / 2, cs)
    if (md.dt == DT_F32) POSS_ASM(float); else if (md.dt == DT_BF16) POSS_ASM(bf16_t); else POSS_ASM(f16_t);
#undef POSS_ASM
}

// ------------------------------------------------------------------ caller-supplied tree -> depth/pos/slot/mask
__global__ void tree_upload_finish_kernel(int n, int t, const int32_t *__restrict__ parent, int32_t *__restrict__ depth,
                                          int32_t *__restrict__ pos, int32_t *__restrict__ slot,
                                          uint64_t *__restrict__ mask) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint64_t w0 = 0ull, w1 = 0ull;
    int dep = -1;
    for (int u = i; u >= 0; u = parent[u]) {
        if (u < 64) w0 |= 1ull << u; else w1 |= 1ull << (u - 64);
        ++dep;
    }
    depth[i] = dep; pos[i] = t + dep; slot[i] = t + i;
    mask[i * MASK_WORDS] = w0; mask[i * MASK_WORDS + 1] = w1;
}

void launch_tree_upload_finish(int n, int t, const int32_t *token, const int32_t *parent, int32_t *depth,
                               int32_t *pos, int32_t *slot, uint64_t *mask, hipStream_t st) {
    (void)token;
    hipLaunchKernelGGL(tree_upload_finish_kernel, dim3(1), dim3(128), 0, st, n, t, parent, depth, pos, slot, mask);
}

// ------------------------------------------------------------------ greedy acceptance walk + commit
// The walk (Eq. 4 with the tree's nodes as candidates): from the root, follow the child whose token
// is the target's choice g at the current node, lowest node index first, until none matches.
// walk[0] = m (accepted draft tokens), walk[1] = bonus token, walk[2..2+m] = node indices of the path.
// Run by the first wave of a workgroup into its own LDS copy: 60 nodes and at most max_path steps
// cost less than a dependent launch, so every workgroup of the commit repeats it.
__device__ __forceinline__ void accept_walk_wave(const int32_t *__restrict__ token, const int32_t *__restrict__ parent,
                                                 const int32_t *__restrict__ g, int n, int max_path, int32_t *walk) {
    const int lane = threadIdx.x;
    int cur = 0, m = 0;
    if (lane == 0) walk[2] = 0;
    while (m < max_path) {
        const int want = g[cur];
        int found = 0x7fffffff;
        for (int i = 1 + lane; i < n; i += 64)
            if (parent[i] == cur && token[i] == want) found = min(found, i);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) found = min(found, __shfl_xor(found, o, 64));
        if (found == 0x7fffffff) break;
        cur = found; ++m;
        if (lane == 0) walk[2 + m] = cur;
    }
    if (lane == 0) { walk[0] = m; walk[1] = g[cur]; }
}

// One launch commits a round.  Workgroups [0, n_layers * hkv): keys/values of the accepted rows of
// one (layer, KV head) move from slot t + path[j] to slot t + j; a destination may be another
// move's source, so the workgroup gathers everything, synchronises, scatters.  Workgroups after
// those, one per path position j <= m: the feature of the accepted row becomes f_{t+j}, the accepted
// token (the bonus token for j = m) joins the stream; they also write the result the host reads:
// result[0..2+m] = the walk, result[32 + j] = committed token j.  `result` is host memory the device
// can write, so no copy follows the kernel.
template <typename T>
__global__ __launch_bounds__(256) void commit_kernel(const KVCache *__restrict__ caches, int n_kv_wgs, int hkv, int dh,
                                                     const int32_t *__restrict__ tree_token,
                                                     const int32_t *__restrict__ tree_parent,
                                                     const int32_t *__restrict__ g, const int32_t *__restrict__ n_nodes,
                                                     int max_path, int t, int d_model, const float *__restrict__ feats,
                                                     T *__restrict__ feat_stash, int32_t *__restrict__ tokens_dev,
                                                     int32_t *__restrict__ walk_dev, int32_t *__restrict__ result) {
    extern __shared__ unsigned char smem[];
    __shared__ int32_t walk[32];                      // 3 + the longest path (depth <= 16)
    if (threadIdx.x < 64) accept_walk_wave(tree_token, tree_parent, g, n_nodes[0], max_path, walk);
    __syncthreads();
    const int m = walk[0];
    if ((int)blockIdx.x < n_kv_wgs) {
        T *kbuf = reinterpret_cast<T *>(smem);
        const int n = (m + 1) * dh;
        T *vbuf = kbuf + n;
        const KVCache kv = caches[blockIdx.x / hkv];
        const int head = blockIdx.x % hkv;
        T *kc = static_cast<T *>(kv.k), *vc = static_cast<T *>(kv.vt);
        for (int e = threadIdx.x; e < n; e += blockDim.x) {
            const int j = e / dh, i = e % dh, src = t + walk[2 + j];
            kbuf[e] = kc[k_offset(kv, src, head, hkv, dh) + i];
            vbuf[e] = vc[vt_offset(kv, src, head, hkv, dh, i)];
        }
        __syncthreads();
        for (int e = threadIdx.x; e < n; e += blockDim.x) {
            const int j = e / dh, i = e % dh, dst = t + j;
            kc[k_offset(kv, dst, head, hkv, dh) + i] = kbuf[e];
            vc[vt_offset(kv, dst, head, hkv, dh, i)] = vbuf[e];
        }
        return;
    }
    const int j = blockIdx.x - n_kv_wgs;
    if (j > m) return;
    const float *src = feats + (size_t)walk[2 + j] * d_model;
    T *dst = feat_stash + (size_t)(t + j) * d_model;
    for (int i = threadIdx.x; i < d_model; i += blockDim.x) dst[i] = from_f<T>(src[i]);
    if (threadIdx.x == 0) {
        const int32_t tok = j < m ? tree_token[walk[2 + j + 1]] : walk[1];
        tokens_dev[t + 1 + j] = tok;
        result[32 + j] = tok;
    }
    if (j == 0 && (int)threadIdx.x < m + 3) {
        walk_dev[threadIdx.x] = walk[threadIdx.x];
        result[threadIdx.x] = walk[threadIdx.x];
    }
}

void launch_commit(const ModelDims &md, int n_layers, const KVCache *caches_dev, const int32_t *tree_token,
                   const int32_t *tree_parent, const int32_t *g, const int32_t *n_nodes, int max_path, int t,
                   const float *feats, void *feat_stash, int32_t *tokens_dev, int32_t *walk_dev, int32_t *result,
                   hipStream_t st) {
    const size_t lds = (size_t)2 * (max_path + 1) * md.dh * dtype_size(md.dt);
    const int n_kv_wgs = n_layers * md.hkv;
#define POSS_COMMIT(T)                                                                                             \
    hipLaunchKernelGGL((commit_kernel<T>), dim3(n_kv_wgs + max_path + 1), dim3(256), lds, st, caches_dev, n_kv_wgs,   \
                       md.hkv, md.dh, tree_token, tree_parent, g, n_nodes, max_path, t, md.d, feats,               \
                       static_cast<T *>(feat_stash), tokens_dev, walk_dev, result)
    if (md.dt == DT_F32) { POSS_COMMIT(float); } else if (md.dt == DT_BF16) { POSS_COMMIT(bf16_t); } else { POSS_COMMIT(f16_t); }
#undef POSS_COMMIT
}

}  // namespace poss
