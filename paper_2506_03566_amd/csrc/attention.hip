// Tree-masked attention over a paged KV cache.
//
// Every row of a pass sees the `n_prefix` committed cache slots and, of the `region_len` slots
// that follow them (the rows of this round: tree nodes in verification, drafted ancestors in a
// specialist pass, the chunk itself in prefill), those whose bit is set in the row's mask.
//
// 16-bit types: one wave per 16 query rows, four waves (one KV head) per workgroup sharing the
// key/value blocks through LDS, on v_mfma_f32_16x16x32.
// Query rows of the G = Hq/Hkv heads that share a KV head are stacked (rho = m*G + g) so a wave's
// 16 rows reuse every key it loads.  Scores are formed transposed, S^T = K Q^T (keys as MFMA rows):
// a lane then holds 8 scores of ONE query row per 32-key block, which is already the B-operand
// layout of O^T = V^T P^T as long as the keys of a block are contracted in the order the score
// tiles deliver them; V is cached transposed ([dh][token]) so that order costs two 8-byte loads.
// Softmax is online (running max / sum per query row, float32); partial (max, sum, O) per split
// are merged by a second kernel in fixed order.
#include "device_utils.h"

#include <type_traits>

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
    // straight-line: a lane's eight slots would otherwise each cost a divergent branch
    const int j = slot - n_prefix;
    const uint64_t word = j < 64 ? m0 : m1;
    const bool bit = ((word >> (j & 63)) & 1ull) != 0;
    return (j < 0) | (((unsigned)j < (unsigned)region_len) & bit);
}

// One workgroup = 4 waves x RT tiles of 16 query rows of ONE KV head (times KW key-ways), over the key
// blocks of one split.  RT = 2 halves the LDS operand reads per MFMA (every key / value fragment
// feeds two row tiles): long contexts are bound by exactly those reads.  Key / value blocks (32 slots) go global -> registers -> LDS one block ahead of the
// arithmetic and are shared by the four waves.  LDS layouts: K rows padded to DH+8 elements (row
// stride 272 B: conflict-free 16-byte operand reads); V^T rows hold their 32 keys permuted so that
// the 8 keys a lane contracts (4 of each 16-key half) are one 16-byte chunk.
// With a single split the result is normalised and written in the storage type directly;
// otherwise (max, sum, O) partials go to the merge kernel.
template <typename T, int DH, int KW, int RT>
__device__ __forceinline__ void attn_mfma_body(
    const int wg_id, const T *__restrict__ q, int rows, int hq, int hkv, const uint64_t *__restrict__ mask, int n_prefix,
    int region_len, KVCache kv, int blocks_per_split, int n_splits, int n_row_groups, float scale,
    float *__restrict__ o_part, float *__restrict__ ml_part, int rho_pad, T *__restrict__ out_direct) {
    typedef typename Vec8<T>::type V8;
    constexpr int KS = DH / 32, DT = DH / 16;
    constexpr int KROW = DH + 8;                          // padded K row, elements
    constexpr int K_UNITS = 32 * DH / 8;                  // 16-byte units of one K block
    constexpr int KPT = K_UNITS / 256, VPT = K_UNITS / 256;
    constexpr int VROW = 32 + 8;                          // padded V^T row (80 B stride: conflict-free operand reads)
    constexpr int KBLK = 32 * KROW, VBLK = DH * VROW;     // elements of one staged K / V^T block
    // [2 buffers][KW blocks]; after the last block the same memory carries the KW-way merge
    __shared__ __attribute__((aligned(16))) T lds_all[2 * KW * (KBLK + VBLK)];
    T *ks_lds = lds_all, *vs_lds = lds_all + 2 * KW * KBLK;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lr = lane & 15, lg = lane >> 4;
    // staging: 256 threads per block; the block index is wave-uniform, and said to be, so that the
    // page-table reads become scalar loads that do not queue behind the key/value loads in flight
    const int stage_blk = __builtin_amdgcn_readfirstlane(tid >> 8), stid = tid & 255;
    const int kway = stage_blk;                           // which of the KW blocks of an iteration this wave takes (wave / 4): branches on it are scalar
    // Workgroup id -> (row group, KV head, split).  Consecutive ids go to the 8 XCDs in turn, each with an
    // L2 of its own, so the row groups that read the same keys and values (same head and split) are given
    // ids that are equal modulo 8: the block is fetched from memory once and then found in that L2.
    const int n_pairs = hkv * n_splits;
    const int xcd = wg_id & 7, qid = wg_id >> 3;
    const int row_group = qid % n_row_groups, pair = (qid / n_row_groups) * 8 + xcd;
    if (pair >= n_pairs) return;                          // padding of the last round of eight
    const int G = hq / hkv, kvh = pair % hkv, split = pair / hkv;
    const int tile0 = (row_group * 4 + (wave & 3)) * RT;  // this wave's tiles: tile0 .. tile0 + RT - 1
    bool valid[RT];
    int m[RT], qh[RT];
    V8 qf[RT][KS];
    uint64_t m0[RT], m1[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const int rho = (tile0 + rt) * 16 + lr;
        valid[rt] = rho < rows * G;
        m[rt] = valid[rt] ? rho / G : 0;
        qh[rt] = kvh * G + (valid[rt] ? rho % G : 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const u32x4 v = *reinterpret_cast<const u32x4 *>(q + ((size_t)m[rt] * hq + qh[rt]) * DH + ks * 32 + lg * 8);
            qf[rt][ks] = __builtin_bit_cast(V8, valid[rt] ? v : u32x4{0u, 0u, 0u, 0u});
        }
        m0[rt] = valid[rt] ? mask[(size_t)m[rt] * MASK_WORDS] : 0ull;
        m1[rt] = valid[rt] ? mask[(size_t)m[rt] * MASK_WORDS + 1] : 0ull;
    }

    const int total = n_prefix + region_len;
    const int n_blocks = (total + 31) >> 5;
    const int b0 = split * blocks_per_split, b1 = min(n_blocks, b0 + blocks_per_split);
    const int P = 1 << kv.page_shift;
    const T *kc = static_cast<const T *>(kv.k), *vc = static_cast<const T *>(kv.vt);

    // staging: K block = 32 consecutive token rows = 32*DH contiguous elements; V^T block = DH rows
    // of 32 keys (64 bytes each, row stride P elements).
    // Key and value blocks travel global -> registers -> LDS in two rings of their own, two iterations deep (an
    // iteration's arithmetic is much shorter than the latency of its loads).  Keys run one iteration AHEAD of values:
    // the score MFMAs of iteration it + 1 are issued before the softmax of iteration it, so that the matrix pipe works
    // while the vector ALU exponentiates (waves of a workgroup move in step from barrier to barrier: without this
    // every wave of a SIMD would sit in its softmax at the same time, the matrix pipe idle).
    u32x4 kr[2][KPT], vr[2][VPT];
    // The page-table entry of a block is fetched one call ahead of the block itself: read where it is
    // used, it would put a dependent trip to memory (and a wait for every load in flight) into each
    // iteration.  Calls go up in steps of KW blocks.
    // (The table is read through the constant address space: nothing writes it while a kernel runs,
    // and a wave-uniform read from there is a scalar load, outside the vector-memory queue.)
    typedef const __attribute__((address_space(4))) int32_t *ConstTable;
    const ConstTable page_table_c = (ConstTable)(uintptr_t)kv.page_table;
    auto page_of = [&](int bfirst) {
        const int b = min(bfirst + stage_blk, b1 - 1);
        return page_table_c[(b << 5) >> kv.page_shift];
    };
    int pgk_next = page_of(b0), pgv_next = pgk_next;
    // this thread's share of the keys / values of block bfirst + stage_blk; pg_after: the entry for the call that follows
    auto load_k = [&](auto slot_tag, int bfirst, int pg_after) {
        constexpr int SLOT = decltype(slot_tag)::value;
        int b = bfirst + stage_blk;
        if (b >= b1) b = b1 - 1;                          // never predicated: reload a valid block, it is ignored
        const int off = (b << 5) & (P - 1);
        const T *kb = kc + ((size_t)(pgk_next * hkv + kvh) * P + off) * DH;
        pgk_next = pg_after;
#pragma unroll
        for (int i = 0; i < KPT; ++i) kr[SLOT][i] = *reinterpret_cast<const u32x4 *>(kb + (size_t)(stid + i * 256) * 8);
    };
    auto load_v = [&](auto slot_tag, int bfirst, int pg_after) {
        constexpr int SLOT = decltype(slot_tag)::value;
        int b = bfirst + stage_blk;
        if (b >= b1) b = b1 - 1;
        const int off = (b << 5) & (P - 1);
        const T *vb = vc + (size_t)(pgv_next * hkv + kvh) * DH * P + off;
        pgv_next = pg_after;
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const int u = stid + i * 256;                 // unit: dh row u / 4, keys (u % 4) * 8 .. +8
            vr[SLOT][i] = *reinterpret_cast<const u32x4 *>(vb + (size_t)(u >> 2) * P + (u & 3) * 8);
        }
    };
    auto store_k = [&](auto slot_tag, int buf) {
        constexpr int SLOT = decltype(slot_tag)::value;
#pragma unroll
        for (int i = 0; i < KPT; ++i) {
            const int u = stid + i * 256, row = u / (DH / 8), c8 = u % (DH / 8);
            *reinterpret_cast<u32x4 *>(&ks_lds[(buf * KW + stage_blk) * KBLK + row * KROW + c8 * 8]) = kr[SLOT][i];
        }
    };
    auto store_v = [&](auto slot_tag, int buf) {
        constexpr int SLOT = decltype(slot_tag)::value;
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            // keys k0 = (u%4)*8 .. k0+7: key k sits at element (k%16)/4*8 + (k/16)*4 + k%4 of its row
            const int u = stid + i * 256, row = u >> 2, k0 = (u & 3) * 8;
            const int half = k0 >> 4, g0 = (k0 & 15) >> 2;                 // k0..k0+3 -> group g0, k0+4..k0+7 -> g0+1
            T *dst = &vs_lds[(buf * KW + stage_blk) * VBLK + row * VROW];
            *reinterpret_cast<u32x2 *>(dst + g0 * 8 + half * 4) = u32x2{vr[SLOT][i].x, vr[SLOT][i].y};
            *reinterpret_cast<u32x2 *>(dst + (g0 + 1) * 8 + half * 4) = u32x2{vr[SLOT][i].z, vr[SLOT][i].w};
        }
    };

    f32x4 acc[RT][DT];
    float m_run[RT], l_run[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        m_run[rt] = -INFINITY; l_run[rt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) acc[rt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // S^T tiles of one block for this wave's row tiles: rows = keys slot0 + tt*16 + (0..15), columns = query rows.
    // Every key fragment of the block is requested before the first MFMA.
    auto scores = [&](int buf, f32x4 (&s)[RT][2]) {
        const T *kbuf = &ks_lds[(buf * KW + kway) * KBLK];
        u32x4 kf[2][KS];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                kf[tt][ks] = *reinterpret_cast<const u32x4 *>(&kbuf[(tt * 16 + lr) * KROW + ks * 32 + lg * 8]);
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) s[rt][tt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
                    s[rt][tt] = Vec8<T>::mfma(__builtin_bit_cast(V8, kf[tt][ks]), qf[rt][ks], s[rt][tt]);
        }
    };

    typedef std::integral_constant<int, 0> S0;
    typedef std::integral_constant<int, 1> S1;
    // prologue: keys of iterations 0 and 1 and values of iteration 0 into LDS, the scores of iteration 0 formed,
    // both rings refilled (keys up to iteration 3, values up to iteration 2)
    load_k(S0{}, b0, page_of(b0 + KW));
    load_k(S1{}, b0 + KW, page_of(b0 + 2 * KW));
    load_v(S0{}, b0, page_of(b0 + KW));
    load_v(S1{}, b0 + KW, page_of(b0 + 2 * KW));
    store_k(S0{}, 0);
    load_k(S0{}, b0 + 2 * KW, page_of(b0 + 3 * KW));
    __syncthreads();
    f32x4 s_cur[RT][2];
    if (b0 + kway < b1) scores(0, s_cur);
    store_k(S1{}, 1);
    load_k(S1{}, b0 + 3 * KW, page_of(b0 + 4 * KW));
    store_v(S0{}, 0);
    load_v(S0{}, b0 + 2 * KW, page_of(b0 + 3 * KW));
    __syncthreads();
    // iteration `it` (blocks bi .. bi+KW-1, PAR = it % 2): scores of it + 1 (keys in LDS buffer PAR ^ 1), softmax of it,
    // P V of it (values in buffer PAR); then keys of it + 2 go into key buffer PAR (last read by the scores of `it`, an
    // iteration ago) and values of it + 1 into value buffer PAR ^ 1, and the two ring slots are refilled at once with
    // iterations it + 4 (keys) and it + 3 (values).  A slot is reloaded right behind the LDS stores that read it: its
    // registers are never free in between, and the wait for a block's loads comes after an iteration's arithmetic.
    auto iteration = [&](auto par_tag, int bi) {
        constexpr int PAR = decltype(par_tag)::value;
        // requested here, used by this iteration's refills: at the foot of the iteration the wait for the
        // LDS stores ahead of the barrier would wait for these scalar loads as well
        const int pgk_ahead = page_of(bi + 5 * KW), pgv_ahead = page_of(bi + 4 * KW);
        const int b = bi + kway;
        f32x4 s_next[RT][2];
        if (b + KW < b1) scores(PAR ^ 1, s_next);         // wave-uniform
        if (b < b1) {                                     // wave-uniform
        const int slot0 = b << 5;
        const T *vbuf = &vs_lds[(PAR * KW + kway) * VBLK];
        u32x4 vf[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) vf[dt] = *reinterpret_cast<const u32x4 *>(&vbuf[(dt * 16 + lr) * VROW + lg * 8]);
        // lane holds keys slot0 + tt*16 + 4*lg + r of query row lr.  Scores are kept in the log2
        // domain (scale * log2 e folded into one factor) so that the exponentials are single
        // v_exp_f32 instructions; the softmax is VALU-bound, not MFMA-bound, at these sizes.
        // bf16 keeps 8 significant bits: probabilities rounded to it moved a layer's output by 2e-2 at the 8B
        // shape (the mean of hundreds of values loses its low bits), ten times everything else.  They go into the
        // P V product as a sum of two bf16 numbers, p = hi + lo, 16 significant bits, at the price of a second
        // MFMA per value fragment.  fp16 (11 bits) stays single.
        constexpr bool SPLIT_P = std::is_same<T, bf16_t>::value;
        V8 pf[RT], pf_lo[RT];
        float alpha[RT];
        bool rescale = false;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            // raw scores; the factor (positive: the maximum commutes with it) goes into the exponent's fma
            float sv[8], bm = -INFINITY;
            if (slot0 + 32 <= n_prefix) {                // whole block inside the committed prefix
#pragma unroll
                for (int j = 0; j < 8; ++j) { sv[j] = s_cur[rt][j >> 2][j & 3]; bm = fmaxf(bm, sv[j]); }
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int slot = slot0 + (j >> 2) * 16 + 4 * lg + (j & 3);
                    sv[j] = slot_visible(slot, n_prefix, region_len, m0[rt], m1[rt]) ? s_cur[rt][j >> 2][j & 3] : -INFINITY;
                    bm = fmaxf(bm, sv[j]);
                }
            }
            bm = rows_max(bm) * scale;
            // The reference point of the exponentials only moves when the block's maximum is more than
            // 2^8 above it (any reference gives the same quotient; the probabilities then go up to 256
            // instead of 1, exact in float32 and in the 16-bit operand alike): without the slack nearly
            // every block moves some row's maximum a little and all accumulators are rescaled.
            const float m_new = bm > m_run[rt] + 8.f ? bm : m_run[rt];
            float psum = 0.f;
            alpha[rt] = 1.f;
            if (m_new == -INFINITY) {
#pragma unroll
                for (int j = 0; j < 8; ++j) { pf[rt][j] = (T)0.f; pf_lo[rt][j] = (T)0.f; }
            } else {
                alpha[rt] = __builtin_amdgcn_exp2f(m_run[rt] - m_new);   // 2^(-inf) = 0 on the first visible block
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float pe = __builtin_amdgcn_exp2f(fmaf(sv[j], scale, -m_new));
                    pf[rt][j] = from_f<T>(pe);
                    if constexpr (SPLIT_P) pf_lo[rt][j] = from_f<T>(pe - to_f(pf[rt][j]));
                    psum += pe;
                }
            }
            l_run[rt] = l_run[rt] * alpha[rt] + psum;
            m_run[rt] = m_new;
            rescale = rescale || __builtin_amdgcn_ballot_w64(alpha[rt] != 1.f) != 0;   // rare once the maximum has settled
        }
        if (rescale) {                                   // wave-uniform: a real branch, taken rarely
            asm volatile("" ::: "memory");               // (keeps the compiler from turning it into 64 selects)
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) acc[rt][dt] *= alpha[rt];
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
                acc[rt][dt] = Vec8<T>::mfma(__builtin_bit_cast(V8, vf[dt]), pf[rt], acc[rt][dt]);
        if constexpr (SPLIT_P) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
                    acc[rt][dt] = Vec8<T>::mfma(__builtin_bit_cast(V8, vf[dt]), pf_lo[rt], acc[rt][dt]);
        }
        }
        store_k(std::integral_constant<int, PAR>{}, PAR);
        load_k(std::integral_constant<int, PAR>{}, bi + 4 * KW, pgk_ahead);
        store_v(std::integral_constant<int, PAR ^ 1>{}, PAR ^ 1);
        load_v(std::integral_constant<int, PAR ^ 1>{}, bi + 3 * KW, pgv_ahead);
        __syncthreads();
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) { s_cur[rt][0] = s_next[rt][0]; s_cur[rt][1] = s_next[rt][1]; }
    };
    for (int bi = b0; bi < b1; bi += 2 * KW) {            // unrolled by two so that ring slots and buffers are static
        iteration(S0{}, bi);
        if (bi + KW < b1) iteration(S1{}, bi + KW);
    }
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        l_run[rt] += __shfl_xor(l_run[rt], 16, 64);
        l_run[rt] += __shfl_xor(l_run[rt], 32, 64);
    }

    if constexpr (KW > 1) {
        // Merge the KW partial (max, sum, O) of each row tile in key-way order: ways 1.. park theirs
        // in LDS (the staging buffers are free after the loop's final barrier), way 0 folds them in;
        // one tile of each wave at a time, so that the records fit the staging memory.
        float *xch = reinterpret_cast<float *>(lds_all);  // per (way-1, wave): 64 lanes x (DT*4 + 2) floats
        constexpr int REC = DT * 4 + 2;
        static_assert((size_t)(KW - 1) * 4 * 64 * REC * sizeof(float) <= sizeof(lds_all), "merge records must fit");
        float *mine = xch + ((size_t)((kway - 1) * 4 + (wave & 3)) * 64 + lane) * REC;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            if (rt > 0) __syncthreads();                  // way 0 has read the previous tile's records
            if (kway > 0) {
                mine[0] = m_run[rt]; mine[1] = l_run[rt];
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) mine[2 + dt * 4 + r] = acc[rt][dt][r];
            }
            __syncthreads();
            if (kway == 0) {
#pragma unroll
                for (int w = 1; w < KW; ++w) {
                    const float *o = xch + ((size_t)((w - 1) * 4 + (wave & 3)) * 64 + lane) * REC;
                    const float mo = o[0], lo = o[1];
                    const float mn = fmaxf(m_run[rt], mo);
                    if (mn == -INFINITY) continue;
                    const float a0 = __builtin_amdgcn_exp2f(m_run[rt] - mn), a1 = __builtin_amdgcn_exp2f(mo - mn);
                    l_run[rt] = l_run[rt] * a0 + lo * a1;
                    m_run[rt] = mn;
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[rt][dt][r] = acc[rt][dt][r] * a0 + o[2 + dt * 4 + r] * a1;
                }
            }
        }
        if (kway > 0) return;
    }

    // O^T tile dt: lane -> query row lr, register r -> dh index dt*16 + 4*lg + r
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        if (out_direct) {
            if (valid[rt]) {
                const float inv = 1.0f / l_run[rt];
                T *dst = out_direct + ((size_t)m[rt] * hq + qh[rt]) * DH + 4 * lg;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) dst[dt * 16 + r] = from_f<T>(acc[rt][dt][r] * inv);
            }
            continue;
        }
        const int tile = tile0 + rt;
        const size_t prow = ((size_t)split * hkv + kvh) * rho_pad + tile * 16 + lr;
        if (tile * 16 < rho_pad) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
                *reinterpret_cast<f32x4 *>(o_part + prow * DH + dt * 16 + 4 * lg) = acc[rt][dt];
            if (lg == 0) {
                ml_part[prow * 2] = m_run[rt];
                ml_part[prow * 2 + 1] = l_run[rt];
            }
        }
    }
}

template <typename T, int DH, int KW, int RT>
__global__ __launch_bounds__(256 * KW) void attn_mfma_kernel(
    const T *__restrict__ q, int rows, int hq, int hkv, const uint64_t *__restrict__ mask, int n_prefix,
    int region_len, KVCache kv, int blocks_per_split, int n_splits, int n_row_groups, float scale,
    float *__restrict__ o_part, float *__restrict__ ml_part, int rho_pad, T *__restrict__ out_direct) {
    attn_mfma_body<T, DH, KW, RT>(blockIdx.x, q, rows, hq, hkv, mask, n_prefix, region_len, kv, blocks_per_split, n_splits,
                                  n_row_groups, scale, o_part, ml_part, rho_pad, out_direct);
}

// Several sequences in one launch: every sequence has its own rows, cache, prefix, split count and slice of the
// partial buffers; a workgroup finds its sequence from the first workgroup id of each, then does exactly what it does
// in a launch of its own.
constexpr int ATTN_MAX_SEQ = 8;
struct AttnSeq {
    const void *q; const uint64_t *mask; void *out_direct; float *o_part, *ml_part;
    KVCache kv;
    int rows, n_prefix, region_len, blocks_per_split, n_splits, n_row_groups, rho_pad, wg0, row0;
};
struct AttnSeqs { int n; AttnSeq s[ATTN_MAX_SEQ]; };

template <typename T, int DH, int KW, int RT>
__global__ __launch_bounds__(256 * KW) void attn_mfma_batch_kernel(AttnSeqs seqs, int hq, int hkv, float scale) {
    int i = 0;
    for (int j = 1; j < seqs.n; ++j)
        if ((int)blockIdx.x >= seqs.s[j].wg0) i = j;
    const AttnSeq &a = seqs.s[i];
    attn_mfma_body<T, DH, KW, RT>(blockIdx.x - a.wg0, static_cast<const T *>(a.q), a.rows, hq, hkv, a.mask, a.n_prefix, a.region_len,
                                  a.kv, a.blocks_per_split, a.n_splits, a.n_row_groups, scale, a.o_part, a.ml_part, a.rho_pad,
                                  static_cast<T *>(a.out_direct));
}

// out[m][qh][:] = sum_s e^{m_s - M} O_s / sum_s e^{m_s - M} l_s, splits in order.  The (max, sum) pairs of
// all splits are fetched in one go and turned into weights once; the partial outputs are then read
// four splits at a time so that their latencies overlap.
constexpr int ATTN_MAX_SPLITS = 256;
template <typename T>
__device__ __forceinline__ void attn_merge_body(const int m, const float *__restrict__ o_part, const float *__restrict__ ml_part,
                                                int n_splits, int hq, int hkv, int dh, int rho_pad, T *__restrict__ out) {
    __shared__ float w_lds[ATTN_MAX_SPLITS];
    __shared__ float den_lds;
    const int qh = blockIdx.y, G = hq / hkv;
    const int kvh = qh / G, rho = m * G + qh % G;
    const size_t stride = (size_t)hkv * rho_pad;          // rows between consecutive splits
    const size_t row0 = (size_t)kvh * rho_pad + rho;
    // Up to 12 splits (the usual case): everything in registers and every load requested before the first use - one
    // trip to memory, no barrier.  Each thread forms the weights itself (the (max, sum) pairs are the same addresses
    // for the whole workgroup); sums run in split order, as in the general path.  Slots beyond n_splits re-read the
    // last split and are not used.
    auto in_registers = [&](auto nr_tag) {
        constexpr int NR = decltype(nr_tag)::value;
        const int i = (int)threadIdx.x < dh ? (int)threadIdx.x : dh - 1;
        const float *src = o_part + row0 * dh + i;
        float ms[NR], ls[NR], v[NR];
#pragma unroll
        for (int s0 = 0; s0 < NR; ++s0) {
            const int sc = s0 < n_splits ? s0 : n_splits - 1;
            const float2 ml = *reinterpret_cast<const float2 *>(ml_part + (row0 + sc * stride) * 2);
            ms[s0] = ml.x; ls[s0] = ml.y;
            v[s0] = src[(size_t)sc * stride * dh];
        }
        float M = -INFINITY;
#pragma unroll
        for (int s0 = 0; s0 < NR; ++s0) if (s0 < n_splits) M = fmaxf(M, ms[s0]);
        float den = 0.f, num = 0.f;
#pragma unroll
        for (int s0 = 0; s0 < NR; ++s0)
            if (s0 < n_splits) {
                const float w = ms[s0] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ms[s0] - M);   // maxima are in the log2 domain
                den += w * ls[s0];
                num += w * v[s0];                         // a split without visible keys has weight 0 and O = 0
            }
        if ((int)threadIdx.x < dh) out[((size_t)m * hq + qh) * dh + i] = from_f<T>(num / den);
    };
    if (n_splits <= 4) { in_registers(std::integral_constant<int, 4>{}); return; }     // (workgroup-uniform)
    if (n_splits <= 8) { in_registers(std::integral_constant<int, 8>{}); return; }
    if (n_splits <= 12) { in_registers(std::integral_constant<int, 12>{}); return; }
    for (int s0 = threadIdx.x; s0 < n_splits; s0 += blockDim.x) w_lds[s0] = ml_part[(row0 + s0 * stride) * 2];
    __syncthreads();
    float M = -INFINITY;
    for (int s0 = 0; s0 < n_splits; ++s0) M = fmaxf(M, w_lds[s0]);
    __syncthreads();
    if (threadIdx.x == 0) {                               // one thread: the order of the sum is fixed
        float den = 0.f;
        for (int s0 = 0; s0 < n_splits; ++s0) {
            const float ms = w_lds[s0];
            const float w = ms == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ms - M);   // maxima are in the log2 domain
            w_lds[s0] = w;
            den += w * ml_part[(row0 + s0 * stride) * 2 + 1];
        }
        den_lds = den;
    }
    __syncthreads();
    const float den = den_lds;
    for (int i = threadIdx.x; i < dh; i += blockDim.x) {
        const float *src = o_part + row0 * dh + i;
        float num = 0.f;
        int s0 = 0;
        for (; s0 + 4 <= n_splits; s0 += 4) {
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = src[(size_t)(s0 + j) * stride * dh];
#pragma unroll
            for (int j = 0; j < 4; ++j) num += w_lds[s0 + j] * v[j];    // a split without visible keys has weight 0 and O = 0
        }
        for (; s0 < n_splits; ++s0) num += w_lds[s0] * src[(size_t)s0 * stride * dh];
        out[((size_t)m * hq + qh) * dh + i] = from_f<T>(num / den);
    }
}

template <typename T>
__global__ void attn_merge_kernel(const float *__restrict__ o_part, const float *__restrict__ ml_part, int n_splits,
                                  int hq, int hkv, int dh, int rho_pad, T *__restrict__ out) {
    attn_merge_body<T>(blockIdx.x, o_part, ml_part, n_splits, hq, hkv, dh, rho_pad, out);
}

// The merge of several sequences' rows in one launch (blockIdx.x = row of the pass); sequences whose keys fit one
// split wrote their rows directly and are skipped.
template <typename T>
__global__ void attn_merge_batch_kernel(AttnSeqs seqs, int hq, int hkv, int dh, T *__restrict__ out) {
    int i = 0;
    for (int j = 1; j < seqs.n; ++j)
        if ((int)blockIdx.x >= seqs.s[j].row0) i = j;
    const AttnSeq &a = seqs.s[i];
    const int m = blockIdx.x - a.row0;
    if (m >= a.rows || a.n_splits == 1) return;          // (workgroup-uniform)
    attn_merge_body<T>(m, a.o_part, a.ml_part, a.n_splits, hq, hkv, dh, a.rho_pad, out + (size_t)a.row0 * hq * dh);
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

// Blocks of 32 keys per split.  A workgroup walks its blocks one after the other, each a dependent trip
// to memory, so a short context is still cut into about four pieces of >= 4 blocks (the merge kernel
// costs less than the serial walk it replaces); long contexts walk 32 blocks per workgroup.  The rule looks at the committed
// prefix only, never at the number of rows or the size of the tree region: a row's arithmetic (which keys
// meet in which split, in which order) is then the same whether it is verified alone or among 60 others,
// which is what makes the speculative stream reproduce the one-token-at-a-time stream bit for bit as long
// as only bonus tokens are committed.  keys_per_split > 0 overrides.
// keys_per_split < 0: the rule above with splits of at most -keys_per_split keys (the specialists' passes carry few
// rows, so that only a few dozen workgroups exist per split level: at long contexts they want shorter walks than the
// target's passes; the drafter's caches are its own, so its rule need not match the target's).
static int blocks_per_split(int n_prefix, int keys_per_split) {
    if (keys_per_split > 0) return keys_per_split >= 32 ? keys_per_split / 32 : 1;
    const int prefix_blocks = (n_prefix + 31) / 32;
    int bps = (prefix_blocks + 3) / 4;
    if (bps < 4) bps = 4;
    const int cap = keys_per_split < 0 && -keys_per_split >= 128 ? -keys_per_split / 32 : 32;
    if (bps > cap) bps = cap;
    return bps;
}

template <typename T>
static void launch_attention_t(const ModelDims &md, const void *q, int rows, const RowMeta &rm, int n_prefix,
                               int region_len, const KVCache &kv, int keys_per_split, const AttnScratch &sc,
                               void *out, hipStream_t st) {
    const int G = md.hq / md.hkv;
    const int tiles = (rows * G + 15) / 16, rho_pad = tiles * 16;
    const int n_blocks = (n_prefix + region_len + 31) / 32;
    int bps = blocks_per_split(n_prefix, keys_per_split);
    while ((n_blocks + bps - 1) / bps > ATTN_MAX_SPLITS) bps *= 2;     // only with a tiny split override on a very long context
    const int n_splits = (n_blocks + bps - 1) / bps;
    const float scale = 1.4426950408889634f / sqrtf((float)md.dh);     // log2(e) / sqrt(dh): scores in the log2 domain
    T *direct = n_splits == 1 ? static_cast<T *>(out) : nullptr;
    // Key-ways follow the split size (so, like it, the committed prefix only); the number of row tiles per
    // wave may follow the row count: it does not change any row's arithmetic.
    const int kw = bps >= 4 ? 2 : 1;
    const int rt = tiles > 4 && bps >= 8 ? 2 : 1;         // pays only where the walk is long
    const int n_row_groups = (tiles + 4 * rt - 1) / (4 * rt), n_pairs = md.hkv * n_splits;
    dim3 grid(8 * n_row_groups * ((n_pairs + 7) / 8));
#define POSS_ATTN(DH, KW, RT)                                                                                    \
    hipLaunchKernelGGL((attn_mfma_kernel<T, DH, KW, RT>), grid, dim3(256 * KW), 0, st, static_cast<const T *>(q),   \
                       rows, md.hq, md.hkv, rm.mask, n_prefix, region_len, kv, bps, n_splits, n_row_groups, scale,  \
                       sc.o, sc.ml, rho_pad, direct)
#define POSS_ATTN_DH(DH)                                                                                         \
    do {                                                                                                         \
        if (kw == 2) { if (rt == 2) POSS_ATTN(DH, 2, 2); else POSS_ATTN(DH, 2, 1); }                             \
        else         { if (rt == 2) POSS_ATTN(DH, 1, 2); else POSS_ATTN(DH, 1, 1); }                             \
    } while (0)
    if (md.dh == 128) POSS_ATTN_DH(128); else POSS_ATTN_DH(64);
#undef POSS_ATTN_DH
#undef POSS_ATTN
    if (n_splits > 1)
        hipLaunchKernelGGL((attn_merge_kernel<T>), dim3(rows, md.hq), dim3(md.dh < 64 ? 64 : md.dh), 0, st, sc.o, sc.ml,
                           n_splits, md.hq, md.hkv, md.dh, rho_pad, static_cast<T *>(out));
}

// Launch shape of one sequence's attention: the split rule, key-ways and row tiles per wave (see above).
struct AttnShape { int bps, n_splits, kw, rt, n_row_groups, rho_pad, n_wgs; };
static AttnShape attention_shape(const ModelDims &md, int rows, int n_prefix, int region_len, int keys_per_split) {
    AttnShape a;
    const int G = md.hq / md.hkv;
    const int tiles = (rows * G + 15) / 16;
    a.rho_pad = tiles * 16;
    const int n_blocks = (n_prefix + region_len + 31) / 32;
    a.bps = blocks_per_split(n_prefix, keys_per_split);
    while ((n_blocks + a.bps - 1) / a.bps > ATTN_MAX_SPLITS) a.bps *= 2;
    a.n_splits = (n_blocks + a.bps - 1) / a.bps;
    a.kw = a.bps >= 4 ? 2 : 1;
    a.rt = tiles > 4 && a.bps >= 8 ? 2 : 1;
    a.n_row_groups = (tiles + 4 * a.rt - 1) / (4 * a.rt);
    a.n_wgs = 8 * a.n_row_groups * ((md.hkv * a.n_splits + 7) / 8);
    return a;
}

template <typename T>
static void launch_attention_batch_t(const ModelDims &md, const void *q, const RowMeta &rm, const AttnSeg *segs, int n,
                                     int keys_per_split, const AttnScratch &sc, void *out, hipStream_t st) {
    const float scale = 1.4426950408889634f / sqrtf((float)md.dh);
    const size_t qd = (size_t)md.hq * md.dh;
    AttnShape shp[ATTN_MAX_SEQ];
    AttnSeq all[ATTN_MAX_SEQ];
    size_t o_off = 0, ml_off = 0;
    bool any_split = false;
    for (int i = 0; i < n; ++i) {
        const AttnSeg &g = segs[i];
        shp[i] = attention_shape(md, g.rows, g.n_prefix, g.region_len, keys_per_split);
        AttnSeq &a = all[i];
        a.q = static_cast<const T *>(q) + g.row0 * qd;
        a.mask = rm.mask + (size_t)g.row0 * MASK_WORDS;
        a.out_direct = shp[i].n_splits == 1 ? static_cast<T *>(out) + g.row0 * qd : nullptr;
        a.o_part = sc.o + o_off; a.ml_part = sc.ml + ml_off;
        o_off += (size_t)shp[i].n_splits * md.hkv * shp[i].rho_pad * md.dh;
        ml_off += (size_t)shp[i].n_splits * md.hkv * shp[i].rho_pad * 2;
        a.kv = *g.kv;
        a.rows = g.rows; a.n_prefix = g.n_prefix; a.region_len = g.region_len;
        a.blocks_per_split = shp[i].bps; a.n_splits = shp[i].n_splits; a.n_row_groups = shp[i].n_row_groups;
        a.rho_pad = shp[i].rho_pad; a.wg0 = 0; a.row0 = g.row0;
        any_split = any_split || shp[i].n_splits > 1;
    }
    // one launch per (key-ways, row tiles) instantiation that occurs: as a rule one
    for (int kw = 1; kw <= 2; ++kw)
        for (int rt = 1; rt <= 2; ++rt) {
            AttnSeqs grp;
            grp.n = 0;
            int wgs = 0;
            for (int i = 0; i < n; ++i)
                if (shp[i].kw == kw && shp[i].rt == rt) {
                    grp.s[grp.n] = all[i];
                    grp.s[grp.n].wg0 = wgs;
                    wgs += shp[i].n_wgs;
                    ++grp.n;
                }
            if (grp.n == 0) continue;
#define POSS_ATTNB(DH, KW, RT)                                                                                   \
    hipLaunchKernelGGL((attn_mfma_batch_kernel<T, DH, KW, RT>), dim3(wgs), dim3(256 * KW), 0, st, grp, md.hq, md.hkv, scale)
#define POSS_ATTNB_DH(DH)                                                                                        \
    do {                                                                                                         \
        if (kw == 2) { if (rt == 2) POSS_ATTNB(DH, 2, 2); else POSS_ATTNB(DH, 2, 1); }                           \
        else         { if (rt == 2) POSS_ATTNB(DH, 1, 2); else POSS_ATTNB(DH, 1, 1); }                           \
    } while (0)
            if (md.dh == 128) POSS_ATTNB_DH(128); else POSS_ATTNB_DH(64);
#undef POSS_ATTNB_DH
#undef POSS_ATTNB
        }
    if (any_split) {
        AttnSeqs grp;
        grp.n = n;
        for (int i = 0; i < n; ++i) grp.s[i] = all[i];
        const int rows_span = segs[n - 1].row0 + segs[n - 1].rows;       // sequences are in row order
        hipLaunchKernelGGL((attn_merge_batch_kernel<T>), dim3(rows_span, md.hq), dim3(md.dh < 64 ? 64 : md.dh), 0, st, grp,
                           md.hq, md.hkv, md.dh, static_cast<T *>(out));
    }
}

void launch_attention_batch(const ModelDims &md, const void *q, const RowMeta &rm, const AttnSeg *segs, int n,
                            int keys_per_split, const AttnScratch &sc, void *out, hipStream_t st) {
    if (n == 1 || md.dt == DT_F32 || n > ATTN_MAX_SEQ) {       // one sequence: the launch of its own; float32: the exact kernel
        const size_t row_bytes = (size_t)md.hq * md.dh * dtype_size(md.dt);
        for (int i = 0; i < n; ++i) {
            const AttnSeg &g = segs[i];
            const RowMeta srm{rm.pos + g.row0, rm.slot + g.row0, rm.mask + (size_t)g.row0 * MASK_WORDS};
            launch_attention(md, static_cast<const char *>(q) + g.row0 * row_bytes, g.rows, srm, g.n_prefix, g.region_len, *g.kv,
                             keys_per_split, sc, static_cast<char *>(out) + g.row0 * row_bytes, st);
        }
        return;
    }
    if (md.dt == DT_BF16) launch_attention_batch_t<bf16_t>(md, q, rm, segs, n, keys_per_split, sc, out, st);
    else launch_attention_batch_t<f16_t>(md, q, rm, segs, n, keys_per_split, sc, out, st);
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
