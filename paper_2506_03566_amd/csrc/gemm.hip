// Weight-streaming GEMM for M <= 256 activation rows:  Y[m][n] = sum_k X[m][k] W[n][k], with the
// operation that follows it in a Llama decoder layer fused into its epilogue.
//
// The round is bound by reading every weight once (the verify pass reads the whole target, each
// draft pass one specialist and the shared LM head; sections 3.3 and 6.2 of the paper discuss the
// cost of switching specialist parameters, which is exactly this stream).  Design:
//   * weights pre-packed in MFMA B-operand order: each lane issues 16-byte loads, a wave reads
//     GEMM_NT KiB contiguous per k-step straight into registers (no LDS hop for the big operand);
//   * a ring of PF k-steps of weight loads stays in flight per wave across LDS chunk boundaries;
//   * the (small, L2-resident) activation slice is staged in LDS in A-operand order, double
//     buffered, its global loads issued one chunk ahead so they are older than the weight loads
//     they overlap and never force the weight ring to drain;
//   * K is split across workgroups (as many splits as keep the launch at one workgroup per CU) into
//     partial planes; an epilogue kernel sums them in split order and applies the fused operation:
//     rotary embedding + KV-cache write (tile-parallel), or residual add followed by the RMSNorm
//     that feeds the next GEMM (one workgroup per row).  Bitwise repeatable, and a row's result
//     does not depend on how many rows the launch carries.  (Reducing inside the GEMM by the last
//     workgroup to arrive at a tile was measured 3.5x slower: agent-scope fences write back and
//     invalidate the per-XCD L2s.)
//   * the gate/up projection is not split: gate and up rows are interleaved so that one lane holds
//     both factors, and the kernel writes SiLU(gate) * up in the storage type itself;
//   * three kernels share the packed weights, the split rule and the order of every sum, so a row gets bit for bit
//     the same result from each: the stream kernel (up to 128 rows, bound by the weight stream), the tall kernel
//     (129..256 rows: several sequences in one stream, prefill; bound by what the L2s hand to the CUs, every
//     workgroup reading all rows of the activations) and the QKV kernel with its epilogue inside (up to 32 rows).
#include "device_utils.h"

#include <hip/hip_ext.h>

#include <type_traits>

namespace poss {

typedef float  f32x4 __attribute__((ext_vector_type(4)));
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef f16_t  f16x8 __attribute__((ext_vector_type(8)));

template <typename T> struct Mfma;
template <> struct Mfma<bf16_t> {
    static __device__ __forceinline__ f32x4 run(u32x4 a, u32x4 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mfma<f16_t> {
    static __device__ __forceinline__ f32x4 run(u32x4 a, u32x4 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                      __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};

// Rotation of one rotary pair, spelt out operation by operation (two products, two fused multiply-adds): the two kernels
// that apply it must round alike, so nothing is left to the compiler's choice of what to contract.
__device__ __forceinline__ void rope_pair(float x1, float x2, float2 cs, float &o1, float &o2) {
#pragma clang fp contract(off)
    const float p = x2 * cs.y, q = x1 * cs.y;
    o1 = __builtin_fmaf(x1, cs.x, -p);
    o2 = __builtin_fmaf(x2, cs.x, q);
}

constexpr int KCS = GEMM_KCHUNK / GEMM_KSTEP;   // k-steps per LDS chunk (8)
// PF = weight k-steps in flight per wave (template parameter of the stream kernel): 4, or 8 for launches
// with fewer workgroups than CUs, where each CU has to keep more bytes in flight to fill the memory system.

// ------------------------------------------------------------------------------------------
// Epilogue of one output tile (columns [tile*128, tile*128+128)) for rows [r_begin, r_end), run by
// 256 threads.  Split-K planes are added in split order; loads are issued eight at a time.
constexpr int EPI_ROWS_PLAIN = 16;  // rows per epilogue workgroup: plain sums sweep 8 rows at a time,
constexpr int EPI_ROWS_PAIR = 4;    // rotary / SiLU epilogues give every 64-thread group one row

__device__ __forceinline__ float sum_planes(const float *part, size_t plane, int S, size_t idx) {
    float a = 0.f;
    int s = 0;
    for (; s + 8 <= S; s += 8) {
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = part[(size_t)(s + j) * plane + idx];
#pragma unroll
        for (int j = 0; j < 8; ++j) a += v[j];
    }
    for (; s + 2 <= S; s += 2) {
        const float v0 = part[(size_t)s * plane + idx], v1 = part[(size_t)(s + 1) * plane + idx];
        a = (a + v0) + v1;
    }
    for (; s < S; ++s) a += part[(size_t)s * plane + idx];
    return a;
}

__device__ __forceinline__ f32x4 sum_planes4(const float *part, size_t plane, int S, size_t idx) {
    f32x4 a = f32x4{0.f, 0.f, 0.f, 0.f};
    int s = 0;
    for (; s + 8 <= S; s += 8) {
        f32x4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = *reinterpret_cast<const f32x4 *>(part + (size_t)(s + j) * plane + idx);
#pragma unroll
        for (int j = 0; j < 8; ++j) a += v[j];
    }
    for (; s + 2 <= S; s += 2) {
        const f32x4 v0 = *reinterpret_cast<const f32x4 *>(part + (size_t)s * plane + idx);
        const f32x4 v1 = *reinterpret_cast<const f32x4 *>(part + (size_t)(s + 1) * plane + idx);
        a = (a + v0) + v1;
    }
    for (; s < S; ++s) a += *reinterpret_cast<const f32x4 *>(part + (size_t)s * plane + idx);
    return a;
}

template <typename T, int EPI>
__device__ __forceinline__ void tile_epilogue(const float *__restrict__ part, size_t plane, int S, int Npad,
                                              int N, int r_begin, int r_end, int tile, const EpiArgs &e) {
    const int t = threadIdx.x, n0 = tile * GEMM_BLOCK_N;
    if constexpr (EPI == EPI_ROPE_KV) {
        // thread -> rotary pair i of one head inside the tile; pairs are (i, i + dh/2)
        const int half = e.dh >> 1, c = t & 63;
        const int hb = n0 + (c / half) * e.dh, i = c % half, gh = hb / e.dh;
        if (gh >= e.hq + 2 * e.hkv) return;
        // columns of the pair: natural order (i, i + dh/2), or the packed order of PackSrc::rope_dh, in which a 32-column
        // group holds dims [16j, 16j+16) followed by their partners
        const int c1 = e.rope_packed ? hb + (i >> 4) * 32 + (i & 15) : hb + i, c2 = e.rope_packed ? c1 + 16 : c1 + half;
        T *kc = static_cast<T *>(e.kv.k), *vc = static_cast<T *>(e.kv.vt), *q = static_cast<T *>(e.q);
        for (int r = r_begin + (t >> 6); r < r_end; r += 4) {
            if (gh < e.hq && r >= e.rows_q) continue;
            const float2 cs = e.cs[r * half + i];          // requested together with the planes
            const int sl = e.slot[r];
            const float x1 = sum_planes(part, plane, S, (size_t)r * Npad + c1);
            const float x2 = sum_planes(part, plane, S, (size_t)r * Npad + c2);
            float o1, o2;
            rope_pair(x1, x2, cs, o1, o2);
            if (gh < e.hq) {
                T *dst = q + ((size_t)r * e.hq + gh) * e.dh;
                dst[i] = from_f<T>(o1);
                dst[i + half] = from_f<T>(o2);
            } else if (gh < e.hq + e.hkv) {
                T *dst = kc + k_offset(e.kv, sl, gh - e.hq, e.hkv, e.dh);
                dst[i] = from_f<T>(o1);
                dst[i + half] = from_f<T>(o2);
            } else {
                const int vh = gh - e.hq - e.hkv;
                vc[vt_offset(e.kv, sl, vh, e.hkv, e.dh, i)] = from_f<T>(x1);
                vc[vt_offset(e.kv, sl, vh, e.hkv, e.dh, i + half)] = from_f<T>(x2);
            }
        }
    } else if constexpr (EPI == EPI_SILU) {
        const int c = t & 63, f = tile * 64 + c, cg = n0 + (c >> 4) * 32 + (c & 15);   // gate column; up is 16 further
        if (f >= e.F) return;
        T *act = static_cast<T *>(e.act);
        for (int r = r_begin + (t >> 6); r < r_end; r += 4) {
            const float g = sum_planes(part, plane, S, (size_t)r * Npad + cg);
            const float up = sum_planes(part, plane, S, (size_t)r * Npad + cg + 16);
            act[(size_t)r * e.F + f] = from_f<T>(g / (1.0f + expf(-g)) * up);
        }
    } else {    // EPI_PLAIN: 32 threads x 4 columns per row, 8 rows per sweep
        const int c4 = (t & 31) * 4, n = n0 + c4;
        for (int rb = r_begin; rb < r_end; rb += 8) {
            const int r = rb + (t >> 5);
            if (r < r_end && n < N) {
                const f32x4 v = sum_planes4(part, plane, S, (size_t)r * Npad + n);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (n + j < N) e.out[(size_t)r * e.ld_out + n + j] = v[j];
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// WPB waves per workgroup: 4 (one 128-column tile) or 8 (two tiles sharing one staged activation
// slice: halves the L2 traffic per weight byte; used where N alone fills the GPU).
// FUSE_SILU (K not split, gate/up interleaved per wave tile): the kernel applies SiLU(gate) * up to its
// accumulators and writes the activation act[M][F] itself; no partial plane, no epilogue kernel.
// HEAD (K not split, columns = vocabulary): the workgroup reduces its column tile per row in its own epilogue - the
// best (value, index) for greedy verification, or maximum, sum of exponentials and the k best for the drafter's
// log-softmax + top-k - so that no kernel has to read the logits back; they are written only on request.
struct HeadEpi { int mode, k, vocab, write_logits; float *seg_out; float *pv; int *pi; };

// (value, index) reductions over the 32 lanes of a half wave
__device__ __forceinline__ void half_argmax(float &v, int &i) {
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) {
        const float ov = __shfl_xor(v, o, 32);
        const int oi = __shfl_xor(i, o, 32);
        if (better(ov, oi, v, i)) { v = ov; i = oi; }
    }
}


// ---- epilogues on a finished output tile, shared by the stream kernel and the tall kernel --------------------------
// SiLU(gate) * up of a workgroup's rows x TW activation columns, collected in LDS (row stride TW + 8 elements: the four
// row groups of a wave hit different banks) and written out so that a row leaves as one contiguous piece in 16-byte
// stores instead of 16-column fragments of two bytes per lane.
template <typename T, int ROWS, int TW, int NTHREADS>
__device__ __forceinline__ void silu_tile_store(const T *tile, T *__restrict__ act, int M, int F, int f0, int tid) {
    constexpr int TWP = TW + 8, EPV = 16 / (int)sizeof(T), PPR = TW / EPV;   // elements per 16-byte store, pieces per row
    for (int p = tid; p < ROWS * PPR; p += NTHREADS) {
        const int m = p / PPR, f = f0 + (p % PPR) * EPV;
        if (m < M && f + EPV <= F)                       // F is a multiple of 8: a piece is inside or outside as a whole
            *reinterpret_cast<u32x4 *>(act + (size_t)m * F + f) = *reinterpret_cast<const u32x4 *>(tile + m * TWP + (p % PPR) * EPV);
    }
}

// The Head's reduction of a tile of logits in LDS, tile[row][TW] = columns [col0, col0 + TW): one half wave per row (NHW
// of them; shuffles stay inside a half).  HEAD_ARGMAX: the best (value, index) of the row's segment; HEAD_TOPK: maximum,
// sum of exp(l - max) in a fixed order, and the k best by k rounds of (argmax, remove).
template <int TW, int NHW>
__device__ __forceinline__ void head_tile_reduce(const float *tile, int M, const HeadEpi &he, int seg, int n_seg, int tid) {
    constexpr int NVH = TW / 32;
    const int hw = tid >> 5, hl = tid & 31, col0 = seg * TW;
    for (int row = hw; row < M; row += NHW) {
        float v[NVH]; int id[NVH];
        float bv = -INFINITY; int bi = 0x7fffffff;
#pragma unroll
        for (int j = 0; j < NVH; ++j) {
            const int c = hl + 32 * j, n = col0 + c;
            const bool ok = n < he.vocab;
            v[j] = ok ? tile[row * TW + c] : -INFINITY;
            id[j] = ok ? n : 0x7fffffff - j;         // dummies stay below every real entry
            if (better(v[j], id[j], bv, bi)) { bv = v[j]; bi = id[j]; }
        }
        if (he.mode == HEAD_ARGMAX) {
            half_argmax(bv, bi);
            if (hl == 0) { he.pv[(size_t)row * n_seg + seg] = bv; he.pi[(size_t)row * n_seg + seg] = bi; }
            continue;
        }
        float mx = bv;
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 32));
        float se = 0.f;
#pragma unroll
        for (int j = 0; j < NVH; ++j) se += v[j] > -INFINITY ? expf(v[j] - mx) : 0.f;
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) se += __shfl_xor(se, o, 32);
        float *rec = he.seg_out + ((size_t)row * n_seg + seg) * TOPK_REC;
        if (hl == 0) { rec[0] = mx; rec[1] = se; }
        float my_v = -INFINITY; int my_i = 0x7fffffff;
        for (int r = 0; r < he.k; ++r) {
            float wv = -INFINITY; int wi = 0x7fffffff;
#pragma unroll
            for (int j = 0; j < NVH; ++j)
                if (better(v[j], id[j], wv, wi)) { wv = v[j]; wi = id[j]; }
            half_argmax(wv, wi);
            if (hl == r) { my_v = wv; my_i = wi; }
#pragma unroll
            for (int j = 0; j < NVH; ++j)
                if (id[j] == wi) v[j] = -INFINITY;   // real indices are unique: removes exactly the winner
        }
        if (hl < he.k) {
            rec[2 + hl] = my_v;
            reinterpret_cast<int *>(rec)[2 + TOPK_MAXK + hl] = my_v > -INFINITY ? my_i : 0x7fffffff;
        }
    }
}

__device__ __forceinline__ int xs_swizzle(int g) { return (0xea40 >> (4 * g)) & 15; }   // f(g) = 0, 4, 10, 14

template <typename T, int MT, int WPB, bool FUSE_SILU, int PF, bool HEAD = false>
__global__ __launch_bounds__(WPB * 64) void gemm_stream_kernel(
    const u32x4 *__restrict__ Wp, const T *__restrict__ X, int ldx, float *__restrict__ part,
    int M, int K, int Npad, int ksteps_total, T *__restrict__ act, int F, HeadEpi he) {
    static_assert(KCS % PF == 0, "ring index must be static");
    constexpr int XUNITS = KCS * MT * 64;                 // 16-byte units of one staged chunk
    // units per thread; where 64 * WPB does not divide the units the last threads stage the last unit again
    constexpr int XPT    = (XUNITS + WPB * 64 - 1) / (WPB * 64);
    __shared__ u32x4 xs[2][XUNITS];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    // split y of gridDim.y owns chunks [y * n / S, (y + 1) * n / S): sizes differ by at most one chunk
    const int n_chunks_total = ksteps_total / KCS;
    const int chunk0 = (int)blockIdx.y * n_chunks_total / (int)gridDim.y;
    const int chunk1 = ((int)blockIdx.y + 1) * n_chunks_total / (int)gridDim.y;
    const int ngroup = blockIdx.x * WPB + wave;
    const u32x4 *wp = Wp + ((size_t)ngroup * ksteps_total + (size_t)chunk0 * KCS) * (GEMM_NT * 64) + lane;

    // Global->LDS staging map: a wave instruction covers one A-operand block [k_step][m_tile] (64 units of 16
    // bytes): four consecutive lanes take the four 8-element groups of one row's k-step (64 contiguous bytes in
    // global memory), consecutive quads take consecutive rows.  In LDS the block is stored in operand order with the
    // row index swizzled by the k-group, unit g * 16 + (m ^ f(g)), f = {0, 4, 10, 14}: the four units a quad stores
    // (same row, g = 0..3) would otherwise lie 256 bytes apart, in the same banks; with f the 8 and the 16 lanes that
    // the LDS takes together always store to 8 and 16 different 16-byte columns, and a read (16 lanes of one g, all rows)
    // still covers one contiguous 256 bytes.
    // Loads are never predicated (a predicated load becomes a branch, and the compiler then waits
    // for every outstanding load at it): out-of-range units read a clamped, valid address and are
    // zeroed by a select.
    const T *x_src[XPT];
    int x_k[XPT], x_dst[XPT];
    bool x_row_ok[XPT];
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
        const int u = min(tid + i * (WPB * 64), XUNITS - 1);
        const int blk = u >> 6, ln = u & 63;
        const int m = (blk % MT) * 16 + (ln >> 2), k8 = (blk / MT) * 4 + (ln & 3);
        x_row_ok[i] = m < M;
        x_src[i] = X + (size_t)(m < M ? m : M - 1) * ldx;
        x_k[i] = k8 * 8;
        x_dst[i] = blk * 64 + ((ln & 3) << 4) + ((ln >> 2) ^ xs_swizzle(ln & 3));
    }
    auto load_x = [&](int chunk, u32x4 (&xr)[XPT]) {
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            const int k = chunk * GEMM_KCHUNK + x_k[i];
            xr[i] = *reinterpret_cast<const u32x4 *>(x_src[i] + (k < K ? k : K - 8));
        }
    };
    auto store_x = [&](int chunk, int b, const u32x4 (&xr)[XPT]) {   // the select happens here, not at the load
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            const bool ok = x_row_ok[i] && chunk * GEMM_KCHUNK + x_k[i] < K;
            xs[b][x_dst[i]] = ok ? xr[i] : u32x4{0u, 0u, 0u, 0u};
        }
    };

    f32x4 acc[MT][GEMM_NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < GEMM_NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    u32x4 xr[XPT];
    load_x(chunk0, xr);
    u32x4 wr[PF][GEMM_NT];
#pragma unroll
    for (int p = 0; p < PF; ++p) {                   // a workgroup owns at least one chunk (KCS >= PF steps)
#pragma unroll
        for (int nt = 0; nt < GEMM_NT; ++nt) wr[p][nt] = __builtin_nontemporal_load(wp + nt * 64);
        wp += GEMM_NT * 64;
    }
    store_x(chunk0, 0, xr);
    __syncthreads();

    // One chunk of KCS k-steps.  MORE (another chunk follows) is a compile-time flag so that the
    // body is straight-line code: the weight ring is refilled PF steps ahead, across the chunk
    // boundary when MORE, and the next chunk's activations are requested before any of it.
    int buf = 0;
    const int lane_sw = (lane & 48) + ((lane & 15) ^ xs_swizzle(lane >> 4));   // this lane's A fragment inside a block
    auto chunk_body = [&](auto more_tag, int chunk) {
        constexpr bool MORE = decltype(more_tag)::value;
        if constexpr (MORE) load_x(chunk + 1, xr);
        __builtin_amdgcn_sched_barrier(0);           // keep these loads older than the weight loads below
        // A fragments of k-step i + 1 are requested from LDS before the MFMAs of k-step i are issued
        u32x4 a[2][MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) a[0][mt] = xs[buf][mt * 64 + lane_sw];
#pragma unroll
        for (int i = 0; i < KCS; ++i) {
            if (i + 1 < KCS) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) a[(i + 1) & 1][mt] = xs[buf][((i + 1) * MT + mt) * 64 + lane_sw];
            }
            // The MFMAs read the ring slot itself and the slot is refilled after them: with a copy taken first (so that
            // the refill could be issued ahead of the MFMAs) the compiler gathers the copies of all slots at the top of
            // the chunk and waits there for the whole ring, which empties the memory pipeline once per chunk.
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < GEMM_NT; ++nt) acc[mt][nt] = Mfma<T>::run(a[i & 1][mt], wr[i % PF][nt], acc[mt][nt]);
            if (MORE || i + PF < KCS) {
#pragma unroll
                for (int nt = 0; nt < GEMM_NT; ++nt) wr[i % PF][nt] = __builtin_nontemporal_load(wp + nt * 64);
                wp += GEMM_NT * 64;
            }
            __builtin_amdgcn_sched_barrier(0);       // one k-step at a time: loads stay in ring order
        }
        if constexpr (MORE) {
            store_x(chunk + 1, buf ^ 1, xr);
            __syncthreads();
            buf ^= 1;
        }
    };
    for (int chunk = chunk0; chunk + 1 < chunk1; ++chunk) chunk_body(std::true_type{}, chunk);
    chunk_body(std::false_type{}, chunk1 - 1);

    // D tile: lane -> column n = lane % 16, register r -> row m = 4 * (lane / 16) + r
    if constexpr (FUSE_SILU) {
        static_assert(GEMM_NT == 2, "gate and up are the two column tiles of a wave");
        // The waves of the workgroup own WPB * 16 consecutive columns of act.  The tile is collected in LDS (the
        // staging memory, free after a barrier) so that a row leaves as one contiguous piece in 16-byte stores
        // instead of 16-column fragments written two bytes per lane.
        constexpr int TW = WPB * 16, TWP = TW + 8;       // padded row: the four row groups of a wave hit different banks
        static_assert((size_t)MT * 16 * TWP * sizeof(T) <= sizeof(xs), "the tile fits the staging memory");
        T *tile = reinterpret_cast<T *>(&xs[0][0]);
        __syncthreads();                                 // every wave has read its last operand fragments
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float g = acc[mt][0][r], up = acc[mt][1][r];
                tile[(mt * 16 + 4 * (lane >> 4) + r) * TWP + wave * 16 + (lane & 15)] = from_f<T>(g / (1.0f + expf(-g)) * up);
            }
        __syncthreads();
        silu_tile_store<T, MT * 16, TW, WPB * 64>(tile, act, M, F, blockIdx.x * TW, tid);
        return;
    }
    if constexpr (HEAD) {
        constexpr int TW = WPB * GEMM_NT * 16;           // columns of the workgroup's tile = one segment
        static_assert((size_t)MT * 16 * TW * sizeof(float) <= sizeof(xs), "the tile fits the staging memory");
        if (he.write_logits) {
            const int nl = ngroup * (GEMM_NT * 16) + (lane & 15);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < GEMM_NT; ++nt)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        part[(size_t)(mt * 16 + 4 * (lane >> 4) + r) * Npad + nl + nt * 16] = acc[mt][nt][r];
        }
        float *tile = reinterpret_cast<float *>(&xs[0][0]);
        __syncthreads();                                 // every wave has read its last operand fragments
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < GEMM_NT; ++nt)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    tile[(mt * 16 + 4 * (lane >> 4) + r) * TW + wave * (GEMM_NT * 16) + nt * 16 + (lane & 15)] = acc[mt][nt][r];
        __syncthreads();
        head_tile_reduce<TW, WPB * 2>(tile, M, he, blockIdx.x, gridDim.x, tid);
        return;
    }
    float *out = part + (size_t)blockIdx.y * (MT * 16) * Npad;
    const int n0 = ngroup * (GEMM_NT * 16) + (lane & 15);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < GEMM_NT; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = mt * 16 + 4 * (lane >> 4) + r;
                out[(size_t)m * Npad + n0 + nt * 16] = acc[mt][nt][r];
            }
}

// ------------------------------------------------------------------------------------------
// The same product for 129..256 rows (several sequences verified in one weight stream, prefill).  At that height a
// workgroup's 256 x 128 tile needs 16 KB of activations and 8 KB of weights per k-step and every workgroup re-reads the
// whole activation matrix.  Counters and timestamps of earlier versions of this kernel: with operands fetched by the
// waves that multiply (weights into registers, activations through registers into LDS) the matrix pipe was busy 29 % of
// the time, the waves waiting for loads 53 %, and 963 MB went through the L1s for 235 MB of weights, because the two
// waves that share a column group each fetched its weights; with both operands staged in LDS by LDS-direct loads, each
// fetched once, a wave still sat 450 - 1300 cycles of a 2600-cycle stage in the ISSUE of its six loads (the CU's vector
// memory pipe takes in about 64 bytes a cycle, and a wave issues in order: while it waits to issue a load it issues no
// MFMA), wherever in the stage the loads were put.  So the work is split by wave:
//   eight consumer waves, two per SIMD: wave (wm, wn) owns the rows [128 wm, 128 wm + 128) of the 32 columns wn of the
//       tile, reads its operand fragments from LDS and issues MFMAs, nothing else;
//   eight producer waves, two per SIMD, issue the loads, three stages of two k-steps (48 KB each) deep, and wait for
//       them (four of them were slower: a wave issues an LDS-direct load only every 100 - 250 cycles).
// Staging, by 16-byte LDS-direct loads (no staging registers, no masks):
//   activations: a stage holds 256 rows x 64 k, a row's 128 bytes (both k-steps) contiguous, its eight 16-byte units
//       xor-swizzled by a function of the row - eight consecutive lanes fetch one row's 128 bytes, a whole line of the
//       L2 (four lanes and 64 bytes, one k-step, made twice the requests), and an operand read (lane % 16 the row,
//       lane / 16 the k-group) runs at the full LDS rate;
//   weights: the packed layout is already the B-operand image, 1 KB per (k-step, column tile), copied as it is.
// Rows >= M and k >= K are not zeroed: such a lane fetches a valid element of the matrix instead (row M - 1, k = 0);
// the rows are never read back and the packed weights are zero beyond K.
// Splits own whole groups of 8 k-steps as in the stream kernel and a wave adds its k-steps in ascending order, so a
// row's sums are bit for bit those of the stream kernel.
constexpr int TALL_KCL = 2, TALL_NST = 3, TALL_THREADS = 1024;   // (row tiles per workgroup, MT: 16, or 12 for up to 192 rows)

// position of 16-byte unit u of row r (of a 16-row tile) inside the row's 128 bytes: u ^ tall_x_swizzle(r)
__device__ __forceinline__ int tall_x_swizzle(int r) { return (((r >> 1) & 1) << 2) | ((r >> 1) & 3); }

template <typename T, int MT, bool FUSE_SILU, bool HEAD>
__global__ __launch_bounds__(TALL_THREADS) void gemm_tall_kernel(
    const u32x4 *__restrict__ Wp, const T *__restrict__ X, int ldx, float *__restrict__ part,
    int M, int K, int Npad, int ksteps_total, T *__restrict__ act, int F, HeadEpi he) {
    typedef __attribute__((address_space(3))) void *LdsPtr;
    constexpr int KCL = TALL_KCL, NST = TALL_NST, MTW = MT / 2;
    static_assert(KCS % KCL == 0, "a split's k-steps are whole stages");
    static_assert(KCL == 2 && GEMM_NT == 2 && (MT == 16 || MT == 12), "the schedules below are written for these");
    constexpr int XBLKS = KCL * MT, WBLKS = KCL * 4 * GEMM_NT;           // 1 KB blocks of a stage: activations, weights
    constexpr int XPP = XBLKS / 8;                                       // activation blocks per producer wave
    constexpr int STAGE_UNITS = (XBLKS + WBLKS) * 64;
    constexpr int LPS = (XBLKS + WBLKS) / 8;                             // loads of a producer wave per stage
    __shared__ __attribute__((aligned(1024))) u32x4 xs[NST * STAGE_UNITS];
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const bool producer = wave >= 8;                      // wave-uniform
    const int wn = wave & 3, wm = (wave >> 2) & 1;
    const int n_chunks_total = ksteps_total / KCS;
    const int chunk0 = ((int)blockIdx.y * n_chunks_total / (int)gridDim.y) * (KCS / KCL);          // in stages
    const int chunk1 = (((int)blockIdx.y + 1) * n_chunks_total / (int)gridDim.y) * (KCS / KCL);
    const int ngroup = blockIdx.x * 4 + wn;

    f32x4 acc[MTW][GEMM_NT];
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
        for (int nt = 0; nt < GEMM_NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (producer) {
        // Producer p = wave - 8 brings the blocks p, p + 8, p + 16 (, p + 24) of the stage's activations (block b = rows
        // 8 b .. 8 b + 7, eight lanes per row: the unit that belongs at the lane's position under the swizzle) and the two
        // column tiles of (k-step p / 4, column group p % 4).
        const int pw = wave - 8;
        const int f_row = lane >> 3;
        const T *x_row[XPP];
        int f_k[XPP];
#pragma unroll
        for (int j = 0; j < XPP; ++j) {
            const int m = (pw + 8 * j) * 8 + f_row;
            x_row[j] = X + (size_t)(m < M ? m : M - 1) * ldx;
            f_k[j] = ((lane & 7) ^ tall_x_swizzle(m & 15)) * 8;
        }
        const u32x4 *w_src = Wp + ((size_t)(blockIdx.x * 4 + (pw & 3)) * ksteps_total + (pw >> 2)) * (GEMM_NT * 64) + lane;
        const unsigned lds0 = (unsigned)(uintptr_t)(LdsPtr)&xs[0];
        auto fetch = [&](int chunk, int st) {             // stage st <- k-steps chunk KCL .. + KCL - 1
            const unsigned base = lds0 + (unsigned)(st * STAGE_UNITS * 16);
#pragma unroll
            for (int j = 0; j < XPP; ++j) {
                const int k = chunk * (KCL * GEMM_KSTEP) + f_k[j];
                lds_dma16(base + (unsigned)((pw + 8 * j) * 1024), x_row[j] + (k < K ? k : 0));
            }
#pragma unroll
            for (int nt = 0; nt < GEMM_NT; ++nt)
                lds_dma16(base + (unsigned)((XBLKS + ((pw >> 2) * 4 + (pw & 3)) * GEMM_NT + nt) * 1024),
                          w_src + (size_t)chunk * KCL * (GEMM_NT * 64) + nt * 64);
        };
        static_assert(LPS == XPP + GEMM_NT && XBLKS == 8 * XPP, "the fetch above brings exactly one stage");
        fetch(chunk0, 0);
        if (chunk0 + 1 < chunk1) { fetch(chunk0 + 1, 1); dma_wait<LPS>(); } else dma_wait<0>();
        __syncthreads();
        int st = 0;
        for (int chunk = chunk0; chunk < chunk1; ++chunk) {
            // stage (st + 2) % 3 was read last in the iteration before this one: every wave is past that barrier;
            // the next stage has landed once only the loads just issued are outstanding
            if (chunk + 2 < chunk1) { fetch(chunk + 2, st == 0 ? 2 : st - 1); dma_wait<LPS>(); } else dma_wait<0>();
            __syncthreads();
            st = st == NST - 1 ? 0 : st + 1;
        }
    } else {
        // operand reads of this wave inside a stage, in 16-byte units
        const int a_row = (wm * MTW) * 128 + (lane & 15) * 8, a_swz = tall_x_swizzle(lane & 15), lg = lane >> 4;
        const int b_unit = XBLKS * 64 + wn * GEMM_NT * 64 + lane;
        __syncthreads();
        int st = 0;
        for (int chunk = chunk0; chunk < chunk1; ++chunk) {
            // The fragments of the stage's first k-step are asked for at once - the only LDS wait of the stage; those of the
            // second follow one by one behind the first k-step's MFMAs.  (The order is given to the scheduler as it stands:
            // left alone it puts every read next to its use and waits for it there.)
            const u32x4 *xa = &xs[st * STAGE_UNITS + a_row], *wb = &xs[st * STAGE_UNITS + b_unit];
            u32x4 w[KCL][GEMM_NT], a[KCL][MTW];
#pragma unroll
            for (int ks = 0; ks < KCL; ++ks) {
#pragma unroll
                for (int nt = 0; nt < GEMM_NT; ++nt) w[ks][nt] = wb[(ks * 4 * GEMM_NT + nt) * 64];
#pragma unroll
                for (int mt = 0; mt < MTW; ++mt) a[ks][mt] = xa[mt * 128 + ((ks * 4 + lg) ^ a_swz)];
            }
#pragma unroll
            for (int ks = 0; ks < KCL; ++ks)
#pragma unroll
                for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
                    for (int nt = 0; nt < GEMM_NT; ++nt) acc[mt][nt] = Mfma<T>::run(a[ks][mt], w[ks][nt], acc[mt][nt]);
            constexpr int FR = GEMM_NT + MTW, MF = MTW * GEMM_NT;          // fragments and MFMAs of a k-step
            static_assert(MF >= FR && MF <= 2 * FR, "one or two MFMAs of the first k-step ahead of every read of the second");
            __builtin_amdgcn_sched_group_barrier(0x100, FR, 0);
#pragma unroll
            for (int i = 0; i < MF - FR; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
#pragma unroll
            for (int i = 0; i < 2 * FR - MF; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, MTW * GEMM_NT, 0);
            __syncthreads();
            st = st == NST - 1 ? 0 : st + 1;
        }
    }

    // D tile: lane -> column n = lane % 16, register r -> row m = 4 * (lane / 16) + r of row tile wm * MTW + mt.
    // (The producer waves take part in the barriers below and in nothing else.)
    const int row0 = wm * (MTW * 16) + 4 * (lane >> 4);
    if constexpr (FUSE_SILU) {
        constexpr int TW = 4 * 16, TWP = TW + 8;
        static_assert((size_t)MT * 16 * TWP * sizeof(T) <= sizeof(xs), "the tile fits the staging memory");
        T *tile = reinterpret_cast<T *>(&xs[0]);
        __syncthreads();                                 // every wave has read its last operand fragments
        if (!producer) {
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float g = acc[mt][0][r], up = acc[mt][1][r];
                    tile[(row0 + mt * 16 + r) * TWP + wn * 16 + (lane & 15)] = from_f<T>(g / (1.0f + expf(-g)) * up);
                }
        }
        __syncthreads();
        if (!producer) silu_tile_store<T, MT * 16, TW, 512>(tile, act, M, F, blockIdx.x * TW, tid);
        return;
    }
    if constexpr (HEAD) {
        constexpr int TW = 4 * GEMM_NT * 16;
        static_assert((size_t)MT * 16 * TW * sizeof(float) <= sizeof(xs), "the tile fits the staging memory");
        if (he.write_logits && !producer) {
            const int nl = ngroup * (GEMM_NT * 16) + (lane & 15);
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
                for (int nt = 0; nt < GEMM_NT; ++nt)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        part[(size_t)(row0 + mt * 16 + r) * Npad + nl + nt * 16] = acc[mt][nt][r];
        }
        float *tile = reinterpret_cast<float *>(&xs[0]);
        __syncthreads();
        if (!producer) {
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
                for (int nt = 0; nt < GEMM_NT; ++nt)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        tile[(row0 + mt * 16 + r) * TW + wn * (GEMM_NT * 16) + nt * 16 + (lane & 15)] = acc[mt][nt][r];
        }
        __syncthreads();
        if (!producer) head_tile_reduce<TW, 16>(tile, M, he, blockIdx.x, gridDim.x, tid);
        return;
    }
    if (producer) return;
    float *out = part + (size_t)blockIdx.y * (MT * 16) * Npad;
    const int n0 = ngroup * (GEMM_NT * 16) + (lane & 15);
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
        for (int nt = 0; nt < GEMM_NT; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) out[(size_t)(row0 + mt * 16 + r) * Npad + n0 + nt * 16] = acc[mt][nt][r];
}

// ------------------------------------------------------------------------------------------
// The QKV projection with its epilogue inside: K split INSIDE the workgroup.  One 32-column tile per workgroup, the
// k-steps dealt to its four waves in contiguous quarters; a wave loads its own operands straight into registers (an A
// fragment of v_mfma 16x16x32 is 16 contiguous bytes of one activation row, and with K split among the waves no two of
// them want the same fragment: no LDS hop, no barrier in the loop).  The four partial tiles meet in LDS and are added
// in wave order, so the workgroup holds finished sums and applies the rotary embedding and writes queries, keys and
// values itself: no partial planes, no epilogue kernel.  The weight rows are packed so that the two 16-column tiles
// of a wave are dims [16j, 16j+16) and [16j + dh/2, ..) of one head: a lane owns both members of a rotary pair.
// Bitwise repeatable; a row's result does not depend on the rows around it.
struct QkvEpi { const float2 *cs; const int32_t *slot; void *q; int hq, hkv, dh; RopeRanges rr; };

template <typename T, int MT, int PF>
__global__ __launch_bounds__(256) void gemm_qkv_rope_kernel(const u32x4 *__restrict__ Wp, const T *__restrict__ X, int ldx,
                                                           int M, int K, int ksteps_total, QkvEpi e) {
    constexpr int NTILE = MT * GEMM_NT;
    __shared__ f32x4 red[4][NTILE][64];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, tile = blockIdx.x;
    const int w0 = wave * ksteps_total / 4, w1 = (wave + 1) * ksteps_total / 4, n_w = w1 - w0;
    const u32x4 *wp = Wp + ((size_t)tile * ksteps_total + w0) * (GEMM_NT * 64) + lane;      // this wave's first k-step
    const T *xp[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + (lane & 15);
        xp[mt] = X + (size_t)(m < M ? m : M - 1) * ldx + (size_t)w0 * GEMM_KSTEP + (lane >> 4) * 8;   // rows beyond M repeat the last row
    }
    f32x4 acc[MT][GEMM_NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < GEMM_NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    int done = 0;
    if (w1 * GEMM_KSTEP <= K && n_w >= PF) {             // no k-step of this wave reaches beyond K: loads need no mask
        u32x4 wr[PF][GEMM_NT], ar[PF][MT];
        auto load_step = [&](int p, int i) {             // k-step w0 + i into ring slot p (p static after unrolling)
#pragma unroll
            for (int nt = 0; nt < GEMM_NT; ++nt) wr[p][nt] = __builtin_nontemporal_load(wp + (size_t)i * (GEMM_NT * 64) + nt * 64);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) ar[p][mt] = *reinterpret_cast<const u32x4 *>(xp[mt] + (size_t)i * GEMM_KSTEP);
        };
#pragma unroll
        for (int p = 0; p < PF; ++p) load_step(p, p);
        const int groups = n_w / PF;
        auto group = [&](auto more_tag, int g) {
            constexpr bool MORE = decltype(more_tag)::value;
#pragma unroll
            for (int p = 0; p < PF; ++p) {
                u32x4 w[GEMM_NT], a[MT];
#pragma unroll
                for (int nt = 0; nt < GEMM_NT; ++nt) w[nt] = wr[p][nt];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) a[mt] = ar[p][mt];
                if constexpr (MORE) load_step(p, (g + 1) * PF + p);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int nt = 0; nt < GEMM_NT; ++nt) acc[mt][nt] = Mfma<T>::run(a[mt], w[nt], acc[mt][nt]);
                __builtin_amdgcn_sched_barrier(0);       // one k-step at a time: loads stay in ring order
            }
        };
        for (int g = 0; g + 1 < groups; ++g) group(std::true_type{}, g);
        group(std::false_type{}, groups - 1);
        done = groups * PF;
    }
    for (int i = done; i < n_w; ++i) {                   // what the ring did not cover; fragments beyond K are zero
        const bool ok = (w0 + i) * GEMM_KSTEP + (lane >> 4) * 8 < K;
        u32x4 w[GEMM_NT], a[MT];
#pragma unroll
        for (int nt = 0; nt < GEMM_NT; ++nt) w[nt] = wp[(size_t)i * (GEMM_NT * 64) + nt * 64];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const u32x4 v = *reinterpret_cast<const u32x4 *>(ok ? xp[mt] + (size_t)i * GEMM_KSTEP : xp[mt] - (size_t)w0 * GEMM_KSTEP - (lane >> 4) * 8);
            a[mt] = ok ? v : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < GEMM_NT; ++nt) acc[mt][nt] = Mfma<T>::run(a[mt], w[nt], acc[mt][nt]);
    }

#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < GEMM_NT; ++nt) red[wave][mt * GEMM_NT + nt][lane] = acc[mt][nt];
    __syncthreads();
    // D tile: lane -> column c = lane % 16, register r -> row 4 * (lane / 16) + r.  Wave w finishes row tiles w, w + 4.
    const int half = e.dh >> 1, tph = half >> 4;          // 32-column tiles per head
    const int gh = tile / tph, i = (tile % tph) * 16 + (lane & 15);
    if (gh >= e.hq + 2 * e.hkv) return;                   // padding columns
    T *q = static_cast<T *>(e.q);
    for (int mt = wave; mt < MT; mt += 4) {
        const f32x4 x1 = ((red[0][mt * GEMM_NT][lane] + red[1][mt * GEMM_NT][lane]) + red[2][mt * GEMM_NT][lane]) + red[3][mt * GEMM_NT][lane];
        const f32x4 x2 = ((red[0][mt * GEMM_NT + 1][lane] + red[1][mt * GEMM_NT + 1][lane]) + red[2][mt * GEMM_NT + 1][lane]) + red[3][mt * GEMM_NT + 1][lane];
        for (int qi = 0; qi < e.rr.n; ++qi) {             // (workgroup-uniform) the sequences that share this launch
            const int r0 = e.rr.r0[qi], r1 = e.rr.r1[qi], rows_q = e.rr.rows_q[qi];
            const KVCache kv = e.rr.kv[qi];
            T *kc = static_cast<T *>(kv.k), *vc = static_cast<T *>(kv.vt);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = mt * 16 + 4 * (lane >> 4) + r;
                if (m < r0 || m >= r1 || m >= M) continue;
                const float a = x1[r], b = x2[r];
                if (gh < e.hq) {
                    if (m >= rows_q) continue;
                    float o1, o2;
                    rope_pair(a, b, e.cs[m * half + i], o1, o2);
                    T *dst = q + ((size_t)m * e.hq + gh) * e.dh;
                    dst[i] = from_f<T>(o1);
                    dst[i + half] = from_f<T>(o2);
                } else if (gh < e.hq + e.hkv) {
                    float o1, o2;
                    rope_pair(a, b, e.cs[m * half + i], o1, o2);
                    T *dst = kc + k_offset(kv, e.slot[m], gh - e.hq, e.hkv, e.dh);
                    dst[i] = from_f<T>(o1);
                    dst[i + half] = from_f<T>(o2);
                } else {
                    const int vh = gh - e.hq - e.hkv, sl = e.slot[m];
                    vc[vt_offset(kv, sl, vh, e.hkv, e.dh, i)] = from_f<T>(a);
                    vc[vt_offset(kv, sl, vh, e.hkv, e.dh, i + half)] = from_f<T>(b);
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Residual epilogue, one workgroup per row: h = sum of planes (+ bias) (+ h); then, because the
// whole row is in this workgroup, the RMSNorm that feeds the next GEMM right away:
// u = T(h / sqrt(mean(h^2) + eps) * gain).  Saves a kernel per norm.
template <typename T>
__global__ __launch_bounds__(1024) void epilogue_residual_norm_kernel(const float *__restrict__ part, size_t plane, int S,
                                                                      int Npad, int N, float eps, EpiArgs e) {
    __shared__ float red[17];
    constexpr int MAXIT = 4;                               // N <= 4 * 4 * 1024
    const int m = blockIdx.x;
    const T *bias = static_cast<const T *>(e.bias), *gain = static_cast<const T *>(e.gain);
    T *u = static_cast<T *>(e.u);
    float *h = e.h + (size_t)m * N, *h_copy = e.h_copy ? e.h_copy + (size_t)m * N : nullptr;
    f32x4 x[MAXIT], gn[MAXIT];
    float ss = 0.f;
#pragma unroll
    for (int it = 0; it < MAXIT; ++it) {
        const int n = (it * (int)blockDim.x + (int)threadIdx.x) * 4;
        x[it] = f32x4{0.f, 0.f, 0.f, 0.f};
        gn[it] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (n < N) {
            // every operand is requested before the first use: one memory round trip, not four
            f32x4 add = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (n + j >= N) continue;
                if (e.residual) add[j] = h[n + j];
                if (bias) add[j] += to_f(bias[n + j]);
                if (gain) gn[it][j] = to_f(gain[n + j]);
            }
            f32x4 v = sum_planes4(part, plane, S, (size_t)m * Npad + n);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (n + j >= N) { v[j] = 0.f; continue; }
                v[j] += add[j];
                h[n + j] = v[j];
                if (h_copy) h_copy[n + j] = v[j];
                ss += v[j] * v[j];
            }
            x[it] = v;
        }
    }
    if (!gain) return;
    ss = block_sum(ss, red);
    const float rs = 1.0f / sqrtf(ss / (float)N + eps);
#pragma unroll
    for (int it = 0; it < MAXIT; ++it) {
        const int n = (it * (int)blockDim.x + (int)threadIdx.x) * 4;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (n + j < N) u[(size_t)m * N + n + j] = from_f<T>(x[it][j] * rs * gn[it][j]);
    }
}

// ------------------------------------------------------------------------------------------
// float32 storage (reference-precision mode of the small test shape): plain FMA loop, weights
// kept row-major, one thread per output element, k ascending.
__global__ void gemm_f32_kernel(const float *__restrict__ W, const float *__restrict__ X, int ldx,
                                float *__restrict__ part, int M, int N, int Npad, int K) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    const int m = blockIdx.y;
    if (n >= Npad) return;
    float acc = 0.f;
    if (n < N && m < M) {
        const float *w = W + (size_t)n * K, *x = X + (size_t)m * ldx;
        for (int k = 0; k < K; ++k) acc = fmaf(x[k], w[k], acc);
    }
    part[(size_t)m * Npad + n] = acc;
}

// The epilogue of every (128-column tile, 16-row block), one workgroup each: sums the split-K planes in split
// order (bitwise repeatable) and applies the fused operation.
template <typename T, int EPI>
__global__ __launch_bounds__(256) void epilogue_kernel(const float *__restrict__ part, size_t plane, int S, int Npad,
                                                       int N, int row0, int M, EpiArgs epi) {   // rows [row0, M)
    constexpr int ROWS = EPI == EPI_PLAIN ? EPI_ROWS_PLAIN : EPI_ROWS_PAIR;
    const int r0 = row0 + blockIdx.y * ROWS;
    tile_epilogue<T, EPI>(part, plane, S, Npad, N, r0, min(M, r0 + ROWS), blockIdx.x, epi);
}

// The RoPE + KV-write epilogue over several row ranges in one launch, each range into its own cache
// (sequences batched into one GEMM); blockIdx.y runs over the 4-row blocks of all ranges.
template <typename T>
__global__ __launch_bounds__(256) void epilogue_rope_ranges_kernel(const float *__restrict__ part, size_t plane, int S, int Npad,
                                                                   int N, RopeRanges rr, EpiArgs epi) {
    int j = 0;
    for (int i = 1; i < rr.n; ++i)
        if ((int)blockIdx.y >= rr.blk0[i]) j = i;
    const int r0 = rr.r0[j] + ((int)blockIdx.y - rr.blk0[j]) * EPI_ROWS_PAIR;
    epi.kv = rr.kv[j];
    epi.rows_q = rr.rows_q[j];
    tile_epilogue<T, EPI_ROPE_KV>(part, plane, S, Npad, N, r0, min(rr.r1[j], r0 + EPI_ROWS_PAIR), blockIdx.x, epi);
}

// ------------------------------------------------------------------------------------------
// Row count of a partial plane as the kernel instantiation writes it.
static int gemm_rows_written(int mpad) {
    const int mt = mpad / 16;
    return (mt <= 2 ? mt : mt <= 4 ? 4 : mt <= 6 ? 6 : mt <= 8 ? 8 : mt <= 12 ? 12 : 16) * 16;
}

GemmShape gemm_plan(int dt, int M, int N, int K, int target_wgs) {
    GemmShape g;
    g.M = M; g.N = N; g.K = K;
    g.Npad = gemm_npad(N);
    g.Kpad = gemm_kpad(dt, K);
    g.Mpad = round_up(M < 1 ? 1 : M, 16);
    if (dt == DT_F32) { g.S = 1; return g; }
    g.Mpad = gemm_rows_written(g.Mpad);       // the kernels are instantiated for 1, 2, 4, 6, 8 or (tall kernel) 12, 16 row tiles
    const int n_blocks = g.Npad / GEMM_BLOCK_N;
    const int n_chunks = g.Kpad / GEMM_KCHUNK;
    // One workgroup per CU (256) at most, as many as fit, chunks dealt out evenly: in every sweep more
    // splits were slower (partial-plane traffic grows, two workgroups on a CU share its LDS and barriers)
    // and fewer leave CUs without a stream.
    if (target_wgs <= 0) target_wgs = 256;
    int S = target_wgs / n_blocks;
    int max_s = n_chunks / 2; if (max_s < 1) max_s = 1;          // at least 512 of K per split
    if (S > max_s) S = max_s;
    if (S < 1) S = 1;
    // The longest stream sets the time: take the fewest splits that keep it (16 chunks over 5 splits
    // is 4 chunks on the busiest; 4 splits do the same with one partial plane less).
    const int longest = (n_chunks + S - 1) / S;
    S = (n_chunks + longest - 1) / longest;
    g.S = S;
    return g;
}

// Two 128-column tiles per workgroup (8 waves sharing one staged activation slice) when the column count alone
// gives every CU work and K is not split.
static bool gemm_wide(const GemmShape &g) {
    return g.S == 1 && g.Mpad <= 96 && g.Npad % (2 * GEMM_BLOCK_N) == 0 && g.Npad / (2 * GEMM_BLOCK_N) >= 256;
}

int gemm_head_segments(const GemmShape &g) { return g.Npad / (GEMM_BLOCK_N * (gemm_wide(g) ? 2 : 1)); }

template <typename T>
static void launch_epilogue_t(const GemmShape &g, const float *part, const EpiArgs &epi, float eps, bool silu_done,
                              hipStream_t st) {
    const size_t plane = (size_t)g.Mpad * g.Npad;
    const int tiles = g.Npad / GEMM_BLOCK_N;
    dim3 pair_grid(tiles, (g.M + EPI_ROWS_PAIR - 1) / EPI_ROWS_PAIR), plain_grid(tiles, (g.M + EPI_ROWS_PLAIN - 1) / EPI_ROWS_PLAIN);
    dim3 eb(256);
    switch (epi.mode) {
        case EPI_ROPE_KV:
            hipLaunchKernelGGL((epilogue_kernel<T, EPI_ROPE_KV>), pair_grid, eb, 0, st, part, plane, g.S, g.Npad, g.N, 0, g.M, epi);
            break;
        case EPI_RESIDUAL: {
            int threads = round_up((g.N + 3) / 4, 64);
            if (threads > 1024) threads = 1024;
            hipLaunchKernelGGL((epilogue_residual_norm_kernel<T>), dim3(g.M), dim3(threads), 0, st, part, plane, g.S, g.Npad,
                               g.N, eps, epi);
            break;
        }
        case EPI_HEAD: break;           // reduced inside the stream kernel
        case EPI_SILU:
            if (silu_done) break;       // applied inside the stream kernel
            hipLaunchKernelGGL((epilogue_kernel<T, EPI_SILU>), pair_grid, eb, 0, st, part, plane, g.S, g.Npad, g.N, 0, g.M, epi);
            break;
        default:
            if (g.S > 1 || epi.out)     // S == 1 without an output buffer: plane 0 is the result
                hipLaunchKernelGGL((epilogue_kernel<T, EPI_PLAIN>), plain_grid, eb, 0, st, part, plane, g.S, g.Npad, g.N, 0, g.M, epi);
            break;
    }
}

// The QKV projection of 16-bit types: one kernel, rotary embedding and cache writes included.
template <typename T>
static void launch_qkv_rope_t(const GemmShape &g, const void *Wp, const void *X, int ldx, const EpiArgs &epi, const RopeRanges &rr,
                              hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
    QkvEpi qe{epi.cs, epi.slot, epi.q, epi.hq, epi.hkv, epi.dh, rr};
    dim3 grid(g.Npad / (GEMM_NT * 16)), block(256);
    const int ksteps = g.Kpad / GEMM_KSTEP;
    const u32x4 *w = static_cast<const u32x4 *>(Wp);
    const T *x = static_cast<const T *>(X);
#define POSS_QKV_LAUNCH(MT, PFV)                                                                              \
    do {                                                                                                      \
        if (ev_start && ev_stop)                                                                              \
            hipExtLaunchKernelGGL((gemm_qkv_rope_kernel<T, MT, PFV>), grid, block, 0, st, ev_start, ev_stop, 0, w, x, ldx, g.M, g.K, ksteps, qe); \
        else                                                                                                  \
            hipLaunchKernelGGL((gemm_qkv_rope_kernel<T, MT, PFV>), grid, block, 0, st, w, x, ldx, g.M, g.K, ksteps, qe); \
    } while (0)
    switch (g.Mpad / 16) {
        case 1: POSS_QKV_LAUNCH(1, 8); break;
        case 2: POSS_QKV_LAUNCH(2, 8); break;
        case 4: POSS_QKV_LAUNCH(4, 8); break;
        case 6: POSS_QKV_LAUNCH(6, 4); break;
        default: POSS_QKV_LAUNCH(8, 4); break;
    }
#undef POSS_QKV_LAUNCH
}

template <typename T>
static void launch_gemm_t(const GemmShape &g, const void *Wp, const void *X, int ldx, float *part,
                          const EpiArgs &epi, float eps, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop, const RopeRanges *rr) {
    // The QKV projection of at most 32 rows (draft passes, plain decoding) runs as one kernel with the K split inside the
    // workgroup; with more rows that kernel's activation traffic (every workgroup reads every row over the whole K)
    // outweighs the partial planes and the epilogue kernel it saves: 25 us against 13.6 + 4.9 us at 61 rows of the 8B shape.
    // It is used only where its four waves own exactly the four splits the streaming kernel would take (four splits, chunk
    // count a multiple of four) and adds them in the same order: a row then gets bit for bit the same sums from either
    // kernel, whatever the number of rows that share its launch.
    if (epi.mode == EPI_ROPE_KV && g.Mpad <= 32 && g.S == 4 && (g.Kpad / GEMM_KCHUNK) % 4 == 0) {
        launch_qkv_rope_t<T>(g, Wp, X, ldx, epi, *rr, st, ev_start, ev_stop);
        return;
    }
    const bool fuse_silu = epi.mode == EPI_SILU && g.S == 1;
    const bool head = epi.mode == EPI_HEAD;
    if (g.Mpad > 128) {                                  // the tall kernel: one 128-column tile of 192 or 256 rows
        HeadEpi he{};
        if (head) he = HeadEpi{epi.head_mode, epi.head_k, g.N, epi.write_logits, epi.seg_out, epi.pv, epi.pi};
        dim3 grid(g.Npad / GEMM_BLOCK_N, g.S), block(TALL_THREADS);
        const int ksteps = g.Kpad / GEMM_KSTEP;
        const u32x4 *w = static_cast<const u32x4 *>(Wp);
        const T *x = static_cast<const T *>(X);
        T *act = static_cast<T *>(epi.act);
#define POSS_TALL_LAUNCH_MT(MT, FUSE, HD, FARG)                                                               \
    do {                                                                                                      \
        if (ev_start && ev_stop)                                                                              \
            hipExtLaunchKernelGGL((gemm_tall_kernel<T, MT, FUSE, HD>), grid, block, 0, st, ev_start, ev_stop, 0, w, x, ldx, part, \
                                  g.M, g.K, g.Npad, ksteps, act, FARG, he);                                   \
        else                                                                                                  \
            hipLaunchKernelGGL((gemm_tall_kernel<T, MT, FUSE, HD>), grid, block, 0, st, w, x, ldx, part, g.M, g.K, g.Npad, \
                               ksteps, act, FARG, he);                                                        \
    } while (0)
#define POSS_TALL_LAUNCH(FUSE, HD, FARG)                                                                      \
    do { if (g.Mpad <= 192) POSS_TALL_LAUNCH_MT(12, FUSE, HD, FARG); else POSS_TALL_LAUNCH_MT(16, FUSE, HD, FARG); } while (0)
        if (fuse_silu) POSS_TALL_LAUNCH(true, false, epi.F);
        else if (head) POSS_TALL_LAUNCH(false, true, 0);
        else POSS_TALL_LAUNCH(false, false, 0);
#undef POSS_TALL_LAUNCH_MT
#undef POSS_TALL_LAUNCH
        if (epi.mode == EPI_ROPE_KV) {
            EpiArgs pe = epi;
            pe.rope_packed = 1;
            const size_t plane = (size_t)g.Mpad * g.Npad;
            const int blocks = rr->blk0[rr->n - 1] + (rr->r1[rr->n - 1] - rr->r0[rr->n - 1] + EPI_ROWS_PAIR - 1) / EPI_ROWS_PAIR;
            hipLaunchKernelGGL((epilogue_rope_ranges_kernel<T>), dim3(g.Npad / GEMM_BLOCK_N, blocks), dim3(256), 0, st, part, plane, g.S,
                               g.Npad, g.N, *rr, pe);
            return;
        }
        launch_epilogue_t<T>(g, part, epi, eps, fuse_silu, st);
        return;
    }
    // Two tiles per workgroup when the column count alone gives every CU work and K is not split.
    const bool wide = !fuse_silu && gemm_wide(g);
    const int wpb = wide ? 8 : 4;
    HeadEpi he{};
    if (head) he = HeadEpi{epi.head_mode, epi.head_k, g.N, epi.write_logits, epi.seg_out, epi.pv, epi.pi};
    dim3 grid(g.Npad / (GEMM_NT * 16 * wpb), g.S), block(wpb * 64);
    const int ksteps = g.Kpad / GEMM_KSTEP;
    const u32x4 *w = static_cast<const u32x4 *>(Wp);
    const T *x = static_cast<const T *>(X);
    T *act = static_cast<T *>(epi.act);
    const bool deep = !wide && (int)(grid.x * grid.y) < 256;     // fewer workgroups than CUs: deeper weight ring
    // With a pair of events the launch itself carries them: they take the kernel's own begin and end
    // timestamps (what a profiler reports), not the time of extra packets around it.
    const bool timed = ev_start && ev_stop;
#define POSS_GEMM_LAUNCH(MT, W, FUSE, PFV, HD, FARG)                                                          \
    do {                                                                                                      \
        if (timed)                                                                                            \
            hipExtLaunchKernelGGL((gemm_stream_kernel<T, MT, W, FUSE, PFV, HD>), grid, block, 0, st, ev_start, \
                                  ev_stop, 0, w, x, ldx, part, g.M, g.K, g.Npad, ksteps, act, FARG, he);      \
        else                                                                                                  \
            hipLaunchKernelGGL((gemm_stream_kernel<T, MT, W, FUSE, PFV, HD>), grid, block, 0, st, w, x, ldx, part, \
                               g.M, g.K, g.Npad, ksteps, act, FARG, he);                                      \
    } while (0)
#define POSS_GEMM_CASE(MT)                                                                                    \
    do {                                                                                                      \
        if (fuse_silu) { if (deep) POSS_GEMM_LAUNCH(MT, 4, true, 8, false, epi.F); else POSS_GEMM_LAUNCH(MT, 4, true, 4, false, epi.F); } \
        else if (head) { if (wide) POSS_GEMM_LAUNCH(MT, 8, false, 4, true, 0); else POSS_GEMM_LAUNCH(MT, 4, false, 4, true, 0); } \
        else if (wide) POSS_GEMM_LAUNCH(MT, 8, false, 4, false, 0);                                           \
        else if (deep) POSS_GEMM_LAUNCH(MT, 4, false, 8, false, 0);                                           \
        else POSS_GEMM_LAUNCH(MT, 4, false, 4, false, 0);                                                     \
    } while (0)
    switch (g.Mpad / 16) {
        case 1: POSS_GEMM_CASE(1); break;
        case 2: POSS_GEMM_CASE(2); break;
        case 4: POSS_GEMM_CASE(4); break;
        case 6: POSS_GEMM_CASE(6); break;
        default: POSS_GEMM_CASE(8); break;
    }
#undef POSS_GEMM_CASE
#undef POSS_GEMM_LAUNCH
    if (epi.mode == EPI_ROPE_KV) {                       // rotary + cache writes per row range, one launch
        EpiArgs pe = epi;
        pe.rope_packed = 1;
        const size_t plane = (size_t)g.Mpad * g.Npad;
        const int blocks = rr->blk0[rr->n - 1] + (rr->r1[rr->n - 1] - rr->r0[rr->n - 1] + EPI_ROWS_PAIR - 1) / EPI_ROWS_PAIR;
        hipLaunchKernelGGL((epilogue_rope_ranges_kernel<T>), dim3(g.Npad / GEMM_BLOCK_N, blocks), dim3(256), 0, st, part, plane, g.S,
                           g.Npad, g.N, *rr, pe);
        return;
    }
    launch_epilogue_t<T>(g, part, epi, eps, fuse_silu, st);
}

// Refuse, on the host, argument sets that would make a kernel write through a null pointer.
static bool gemm_args_ok(const GemmShape &g, const void *Wp, const void *X, const float *part, const EpiArgs &e) {
    if (!Wp || !X || !part || g.M < 1 || g.M > LAUNCH_ROWS || g.S < 1) return false;
    switch (e.mode) {
        case EPI_PLAIN: return e.out || g.S == 1;          // unsplit: plane 0 is the result
        case EPI_ROPE_KV: return e.q && e.cs && e.slot && (e.dh == 64 || e.dh == 128 || !e.dh);   // caches: checked per range
        case EPI_RESIDUAL: return e.h && (!e.gain || e.u);
        case EPI_SILU: return e.act != nullptr;
        case EPI_HEAD:
            if (g.S != 1 || g.N < 1) return false;
            if (e.head_mode == HEAD_ARGMAX) return e.pv && e.pi;
            return e.head_mode == HEAD_TOPK && e.seg_out && e.head_k >= 1 && e.head_k <= TOPK_MAXK;
        default: return false;
    }
}

static bool ranges_ok(const GemmShape &g, const EpiArgs &epi, RopeRanges &rr) {
    if (rr.n < 1 || rr.n > ROPE_MAX_RANGES) return false;
    int blocks = 0;
    for (int i = 0; i < rr.n; ++i) {
        if (rr.r0[i] < 0 || rr.r1[i] > g.M || rr.r0[i] >= rr.r1[i]) return false;
        if (!rr.kv[i].k || !rr.kv[i].vt || !rr.kv[i].page_table) return false;
        rr.blk0[i] = blocks;
        blocks += (rr.r1[i] - rr.r0[i] + EPI_ROWS_PAIR - 1) / EPI_ROWS_PAIR;
    }
    (void)epi;
    return true;
}

bool launch_gemm(int dt, const GemmShape &g, const void *Wp, const void *X, int ldx, float *part,
                 const EpiArgs &epi, float eps, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop, const RopeRanges *ranges) {
    if (!gemm_args_ok(g, Wp, X, part, epi)) return false;
    if (ranges && epi.mode != EPI_ROPE_KV) return false;               // only that epilogue works by row range
    RopeRanges rr;
    if (epi.mode == EPI_ROPE_KV) {
        if (ranges) rr = *ranges;
        else { rr.n = 1; rr.r0[0] = 0; rr.r1[0] = g.M; rr.rows_q[0] = epi.rows_q; rr.kv[0] = epi.kv; }
        if (!ranges_ok(g, epi, rr)) return false;
    }
    if (dt == DT_F32) {
        if (epi.mode == EPI_HEAD) return false;          // float32 storage reduces its logits with the two-stage kernels
        if (!part) return false;
        dim3 grid((g.Npad + 127) / 128, g.Mpad), block(128);
        if (ev_start && ev_stop)
            hipExtLaunchKernelGGL(gemm_f32_kernel, grid, block, 0, st, ev_start, ev_stop, 0, static_cast<const float *>(Wp),
                                  static_cast<const float *>(X), ldx, part, g.M, g.N, g.Npad, g.K);
        else
            hipLaunchKernelGGL(gemm_f32_kernel, grid, block, 0, st, static_cast<const float *>(Wp),
                               static_cast<const float *>(X), ldx, part, g.M, g.N, g.Npad, g.K);
        if (epi.mode == EPI_ROPE_KV) {                   // rotary + cache writes per row range, one launch
            const size_t plane = (size_t)g.Mpad * g.Npad;
            int blocks = rr.blk0[rr.n - 1] + (rr.r1[rr.n - 1] - rr.r0[rr.n - 1] + EPI_ROWS_PAIR - 1) / EPI_ROWS_PAIR;
            dim3 egrid(g.Npad / GEMM_BLOCK_N, blocks), eb(256);
            hipLaunchKernelGGL((epilogue_rope_ranges_kernel<float>), egrid, eb, 0, st, part, plane, g.S, g.Npad, g.N, rr, epi);
        } else {
            launch_epilogue_t<float>(g, part, epi, eps, false, st);
        }
    } else if (dt == DT_BF16) {
        launch_gemm_t<bf16_t>(g, Wp, X, ldx, part, epi, eps, st, ev_start, ev_stop, epi.mode == EPI_ROPE_KV ? &rr : nullptr);
    } else {
        launch_gemm_t<f16_t>(g, Wp, X, ldx, part, epi, eps, st, ev_start, ev_stop, epi.mode == EPI_ROPE_KV ? &rr : nullptr);
    }
    return true;
}

// ------------------------------------------------------------------------------------------
// Repack row-major [rows_i, K] matrices, stacked along N (or gate/up interleaved in groups of 16
// rows), into B-operand order.
__device__ __forceinline__ bool pack_source_row(const PackSrc &src, int n, int &which, int &row) {
    if (src.interleave16) {          // 32 rows = 16 rows of matrix 0, then the same 16 rows of matrix 1
        const int w = n & 31;
        which = w >> 4; row = (n >> 5) * 16 + (w & 15);
        return row < src.rows[which];
    }
    if (src.rope_dh > 0) {           // packed column p of a head -> dim (p / 32) * 16 + p % 16 + (p / 16 % 2) * dh / 2
        const int dh = src.rope_dh, p = n % dh;
        n = n - p + (p >> 5) * 16 + (p & 15) + ((p >> 4) & 1) * (dh >> 1);
    }
    for (which = 0; which < 3; ++which) {
        if (n < src.rows[which]) { row = n; return true; }
        n -= src.rows[which];
    }
    return false;
}

__global__ void pack16_kernel(PackSrc src, int K, int Kpad, int Npad, u32x4 *__restrict__ dst) {
    const size_t unit = (size_t)blockIdx.x * blockDim.x + threadIdx.x;     // one 16-byte unit of dst
    const size_t total = (size_t)Npad * Kpad / 8;
    if (unit >= total) return;
    const int ksteps = Kpad / GEMM_KSTEP;
    const int lane = unit & 63;
    size_t r = unit >> 6;
    const int nt = r % GEMM_NT; r /= GEMM_NT;
    const int ks = r % ksteps;
    const int ngroup = r / ksteps;
    const int n = (ngroup * GEMM_NT + nt) * 16 + (lane & 15);
    const int k = ks * GEMM_KSTEP + (lane >> 4) * 8;
    u32x4 v = u32x4{0u, 0u, 0u, 0u};
    int which, row;
    if (k < K && pack_source_row(src, n, which, row))
        v = *reinterpret_cast<const u32x4 *>(static_cast<const uint16_t *>(src.ptr[which]) + (size_t)row * K + k);
    dst[unit] = v;
}

__global__ void pack32_kernel(PackSrc src, int K, int Npad, float *__restrict__ dst) {
    const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (size_t)Npad * K) return;
    const int n = e / K, k = e % K;
    int which, row;
    dst[e] = pack_source_row(src, n, which, row) ? static_cast<const float *>(src.ptr[which])[(size_t)row * K + k] : 0.f;
}

void launch_pack(int dt, const PackSrc &src, int K, void *dst, hipStream_t st) {
    const int N = src.interleave16 ? gate_up_rows(src.rows[0]) : src.rows[0] + src.rows[1] + src.rows[2];
    const int Npad = gemm_npad(N), Kpad = gemm_kpad(dt, K);
    if (dt == DT_F32) {
        const size_t total = (size_t)Npad * K;
        hipLaunchKernelGGL(pack32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, src, K, Npad,
                           static_cast<float *>(dst));
    } else {
        const size_t total = (size_t)Npad * Kpad / 8;
        hipLaunchKernelGGL(pack16_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, src, K, Kpad,
                           Npad, static_cast<u32x4 *>(dst));
    }
}

}  // namespace poss
