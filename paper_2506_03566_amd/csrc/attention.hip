// Tree-masked attention over a paged KV cache.
//
// Every row of a pass sees the `n_prefix` committed cache slots and, of the `region_len` slots
// that follow them (the rows of this round: tree nodes in verification, drafted ancestors in a
// specialist pass, the chunk itself in prefill), those whose bit is set in the row's mask.
//
// 16-bit types: one wave per 16 (or 32) query rows, four waves (one KV head) per key-way and workgroup
// sharing the key/value blocks through LDS, on v_mfma_f32_16x16x32.
// Query rows of the G = Hq/Hkv heads that share a KV head are stacked (rho = m*G + g) so a wave's
// 16 rows reuse every key it loads.  Scores are formed transposed, S^T = K Q^T (keys as MFMA rows):
// a lane then holds 8 scores of ONE query row per 32-key block, which is already the B-operand
// layout of O^T = V^T P^T as long as the keys of a block are contracted in the order the score
// tiles deliver them; the key rows are dealt to the two score tiles so that this order is the
// natural one of V^T, which is cached transposed ([dh][token]).  Blocks go from memory straight
// into LDS (LDS-direct loads), swizzled so that operand reads run at the full LDS rate.
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

// Swizzles of the staged blocks.  A block reaches LDS through 16-byte LDS-direct loads: lane l of a wave
// writes base + 16 l, so a row cannot be padded; instead the 16-byte chunk c of row r is kept at position
// c ^ swz(r) of the row (the loading lane simply fetches the chunk that belongs at its position).
// An operand read has its 64 lanes read one row each (lane % 16 picks the row, lane / 16 the chunk).  Measured
// on this GPU with every wave of a CU reading: these two patterns run at 4.0 cycles per ds_read_b128 (256 bytes
// per cycle, the same as consecutive addresses), rows padded by 16 bytes instead (272- or 80-byte strides), a
// three-bit key swizzle, or a value swizzle that also folds in row bit 3, at 8.2 - 8.9 cycles.
// Keys: row kappa of a block (bits 0, 1 and 3, 4 vary over the lanes of a read; bit 2 is the score tile).
template <int DH>
__device__ __forceinline__ int key_swizzle(int kappa) {
    const int l0 = kappa & 1, l1 = (kappa >> 1) & 1, l2 = (kappa >> 3) & 1, l3 = (kappa >> 4) & 1;
    if (DH >= 128) return l0 | (l1 << 1) | (l2 << 2) | (l3 << 3);     // 16 chunks per row: the reading lane's row number
    return l1 | (l2 << 1) | (l3 << 2);                                // 8 chunks per row, two rows per 256 bytes: half of it
}
// Values: row rho of V^T (a dh index; 4 chunks of 8 keys per row, four rows per 256 bytes).
__device__ __forceinline__ int value_swizzle(int rho) { return (rho >> 1) & 3; }

// One workgroup = 4 waves x RT tiles of 16 query rows of ONE KV head (times KW key-ways), over the key
// blocks of one split.  RT = 2 halves the LDS operand reads per MFMA (every key / value fragment
// feeds two row tiles): long contexts are bound by exactly those reads.
// Key / value blocks (32 slots) go from memory straight into LDS (no registers, no LDS stores), four stages
// deep, shared by the four waves of a key-way.  The 16 key rows of score tile tt are rows 8(i/4) + 4tt + i%4
// of the block, so that the 8 scores a lane holds of a query row belong to 8 CONSECUTIVE keys
// (8 lg .. 8 lg + 7): its slice of P^T then pairs with one natural 16-byte chunk of a V^T row.
// With a single split the result is normalised and written in the storage type directly;
// otherwise (max, sum, O) partials go to the merge kernel.
template <typename T, int DH, int KW, int RT>
__device__ __forceinline__ void attn_mfma_body(
    const int wg_id, const T *__restrict__ q, int rows, int hq, int hkv, const uint64_t *__restrict__ mask, int n_prefix,
    int region_len, KVCache kv, int blocks_per_split, int n_splits, int n_row_groups, float scale,
    float *__restrict__ o_part, float *__restrict__ ml_part, int rho_pad, T *__restrict__ out_direct) {
    typedef typename Vec8<T>::type V8;
    typedef __attribute__((address_space(3))) void *LdsPtr;
    constexpr int KS = DH / 32, DT = DH / 16;
    constexpr int CPR = DH / 8;                           // 16-byte chunks of a key row
    constexpr int UNITS = 32 * CPR;                       // 16-byte units of a key block (and of a value block)
    constexpr int WPW = 4;                                // waves per key-way
    constexpr int STG = 64 * WPW;                         // threads of a key-way: they load its blocks
    constexpr int UPT = UNITS / STG;                      // loads per thread and block
    static_assert(UPT >= 1, "a block must give every thread of its key-way a load");
    constexpr int BLK = 32 * DH;                          // elements of a staged block
    constexpr int NST = 4;                                // stages
    // [stage][key-way] blocks of keys, then of values; after the last block the same memory carries the KW-way merge
    __shared__ __attribute__((aligned(1024))) T lds_all[2 * NST * KW * BLK];
    T *ks_lds = lds_all, *vs_lds = lds_all + NST * KW * BLK;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lr = lane & 15, lg = lane >> 4;
    // which of the KW blocks of an iteration this wave takes (wave / 4; wave-uniform: branches on it are scalar) and
    // which of the four groups of row tiles.  (Waves w and w + 4, the two key-ways of a tile group, are the pair the
    // text below places on one SIMD; giving the pairs (2w, 2w + 1) the two ways instead measured the same.)
    const int kway = __builtin_amdgcn_readfirstlane(tid / STG), wq = wave % WPW;
    const int stid = tid % STG;
    // Workgroup id -> (row group, KV head, split).  Consecutive ids go to the 8 XCDs in turn, each with an
    // L2 of its own, so the row groups that read the same keys and values (same head and split) are given
    // ids that are equal modulo 8: the block is fetched from memory once and then found in that L2.
    const int n_pairs = hkv * n_splits;
    const int xcd = wg_id & 7, qid = wg_id >> 3;
    const int row_group = qid % n_row_groups, pair = (qid / n_row_groups) * 8 + xcd;
    if (pair >= n_pairs) return;                          // padding of the last round of eight
    const int G = hq / hkv, kvh = pair % hkv, split = pair / hkv;
    const int tile0 = (row_group * WPW + wq) * RT;        // this wave's tiles: tile0 .. tile0 + RT - 1
    // query row of lane lr in row tile rt: (valid, row of the pass, query head).  Recomputed where it is needed
    // (the masked blocks at the end of the keys, the final stores) rather than kept in registers over the loop.
    auto row_of = [&](int rt, bool &valid, int &m, int &qh) {
        const int rho = (tile0 + rt) * 16 + lr;
        valid = rho < rows * G;
        m = valid ? rho / G : 0;
        qh = kvh * G + (valid ? rho % G : 0);
    };
    V8 qf[RT][KS];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        bool valid; int m, qh;
        row_of(rt, valid, m, qh);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const u32x4 v = *reinterpret_cast<const u32x4 *>(q + ((size_t)m * hq + qh) * DH + ks * 32 + lg * 8);
            qf[rt][ks] = __builtin_bit_cast(V8, valid ? v : u32x4{0u, 0u, 0u, 0u});
        }
    }

    const int total = n_prefix + region_len;
    const int n_blocks = (total + 31) >> 5;
    const int b0 = split * blocks_per_split, b1 = min(n_blocks, b0 + blocks_per_split);
    const int n_it = (b1 - b0 + KW - 1) / KW;             // iteration `it` takes blocks b0 + it KW .. + KW - 1, one per key-way
    const int P = 1 << kv.page_shift;
    const T *kc = static_cast<const T *>(kv.k), *vc = static_cast<const T *>(kv.vt);

    // Staging.  K block = 32 consecutive token rows = 32*DH contiguous elements; V^T block = DH rows of 32 keys
    // (64 bytes each, row stride P elements).  Thread stid of a block's 256 owns LDS units stid + 256 i and fetches
    // the chunk that belongs there under the swizzle.  Stage it % NST holds iteration it's blocks.
    // (Page-table entries: lane j of pg_vec holds the entry of block b0 + j - a split has at most ATTN_MAX_BPS = 64
    // blocks - fetched with one vector load before the loads to LDS start and picked with v_readlane afterwards.  A
    // scalar load per block would sit in the same counter as the LDS reads and, returning out of order, turn every
    // wait for an operand fragment into a wait for a trip to memory; a vector load inside the loop would make the
    // compiler wait for every load in flight.)
    auto block_of = [&](int it) { return min(b0 + it * KW + kway, b1 - 1); };   // never predicated: past the end a valid block is loaded again and ignored
    const int pg_vec = kv.page_table[(min(b0 + lane, b1 - 1) << 5) >> kv.page_shift];
    auto page_of_block = [&](int b) { return __builtin_amdgcn_readlane(pg_vec, (b - b0) & 63); };   // b wave-uniform
    int k_goff[UPT], v_goff[UPT];                         // element offsets of this thread's chunks inside a block
#pragma unroll
    for (int i = 0; i < UPT; ++i) {
        const int u = stid + i * STG;
        const int krow = u / CPR, kpos = u % CPR;
        k_goff[i] = krow * DH + (kpos ^ key_swizzle<DH>(krow)) * 8;
        const int vrow = u >> 2, vpos = u & 3;
        v_goff[i] = vrow * P + (vpos ^ value_swizzle(vrow)) * 8;
    }
    const unsigned lds_k0 = (unsigned)(uintptr_t)(LdsPtr)ks_lds, lds_v0 = (unsigned)(uintptr_t)(LdsPtr)vs_lds;
    // byte offset of this wave's 64 units of load 0 inside a stage, wave-uniform
    const unsigned wave_units = __builtin_amdgcn_readfirstlane(kway * BLK * (int)sizeof(T) + wq * 1024);
    auto issue_k = [&](int it) {
        const int b = block_of(it), off = (b << 5) & (P - 1);
        const T *kb = kc + ((size_t)(page_of_block(b) * hkv + kvh) * P + off) * DH;
        const unsigned base = lds_k0 + (unsigned)((it & (NST - 1)) * KW * BLK * (int)sizeof(T)) + wave_units;
#pragma unroll
        for (int i = 0; i < UPT; ++i) lds_dma16(base + i * STG * 16, kb + k_goff[i]);
    };
    auto issue_v = [&](int it) {
        const int b = block_of(it), off = (b << 5) & (P - 1);
        const T *vb = vc + (size_t)(page_of_block(b) * hkv + kvh) * DH * P + off;
        const unsigned base = lds_v0 + (unsigned)((it & (NST - 1)) * KW * BLK * (int)sizeof(T)) + wave_units;
#pragma unroll
        for (int i = 0; i < UPT; ++i) lds_dma16(base + i * STG * 16, vb + v_goff[i]);
    };

    f32x4 acc[RT][DT];
    float m_run[RT], l_run[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        m_run[rt] = -INFINITY; l_run[rt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) acc[rt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // operand reads: element offsets of this lane inside a staged block
    const int kappa0 = 8 * (lr >> 2) + (lr & 3), kswz = key_swizzle<DH>(kappa0);
    int k_rd[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) k_rd[ks] = kappa0 * DH + ((ks * 4 + lg) ^ kswz) * 8;
    const int v_rd = lr * 32 + (lg ^ value_swizzle(lr)) * 8;

    // S^T tiles of iteration it's block for this wave's row tiles: rows = keys 8(i/4) + 4tt + i%4, columns = query rows.
    // Every key fragment of the block is requested before the first MFMA.
    auto key_fragments = [&](int it, u32x4 (&kf)[2][KS]) {
        const T *kbuf = &ks_lds[((it & (NST - 1)) * KW + kway) * BLK];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kf[tt][ks] = *reinterpret_cast<const u32x4 *>(&kbuf[tt * 4 * DH + k_rd[ks]]);
    };
    auto scores_of = [&](const u32x4 (&kf)[2][KS], f32x4 (&s)[RT][2]) {
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
    auto scores = [&](int it, f32x4 (&s)[RT][2]) {
        u32x4 kf[2][KS];
        key_fragments(it, kf);
        scores_of(kf, s);
    };
    // bf16 keeps 8 significant bits: probabilities rounded to it moved a layer's output by 2e-2 at the 8B
    // shape (the mean of hundreds of values loses its low bits), ten times everything else.  They go into the
    // P V product as a sum of two bf16 numbers, p = hi + lo, 16 significant bits, at the price of a second
    // MFMA per value fragment.  fp16 (11 bits) stays single.
    constexpr bool SPLIT_P = std::is_same<T, bf16_t>::value;
    // acc += V^T P^T of iteration it's block, in two halves of the value fragments (h = 0, 1) so that only half of them
    // need registers at a time
    auto pv_half = [&](int it, auto h_tag, const V8 (&p_hi)[RT], const V8 (&p_lo)[RT]) {
        constexpr int HD = DT / 2, H = decltype(h_tag)::value;
        const T *vbuf = &vs_lds[((it & (NST - 1)) * KW + kway) * BLK];
        u32x4 vf[HD];
#pragma unroll
        for (int d = 0; d < HD; ++d) vf[d] = *reinterpret_cast<const u32x4 *>(&vbuf[(H * HD + d) * 16 * 32 + v_rd]);
#pragma unroll
        for (int d = 0; d < HD; ++d)
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
                acc[rt][H * HD + d] = Vec8<T>::mfma(__builtin_bit_cast(V8, vf[d]), p_hi[rt], acc[rt][H * HD + d]);
        if constexpr (SPLIT_P) {
#pragma unroll
            for (int d = 0; d < HD; ++d)
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
                    acc[rt][H * HD + d] = Vec8<T>::mfma(__builtin_bit_cast(V8, vf[d]), p_lo[rt], acc[rt][H * HD + d]);
        }
    };
    typedef std::integral_constant<int, 0> I0;
    typedef std::integral_constant<int, 1> I1;
    auto pv = [&](int it, const V8 (&p_hi)[RT], const V8 (&p_lo)[RT]) {
        pv_half(it, I0{}, p_hi, p_lo);
        pv_half(it, I1{}, p_hi, p_lo);
    };
    // Online softmax of one block's scores: running maximum and sum updated, the probabilities left in MFMA operand
    // form, alpha = the factor the accumulators are to be multiplied by; returns whether any lane's alpha differs from 1.
    // A lane holds keys slot0 + 8 lg + j (j = 4 tt + r) of query row lr.  Scores are kept in the log2
    // domain (scale * log2 e folded into one factor) so that the exponentials are single v_exp_f32 instructions.
    // INSIDE: the whole block lies in the committed prefix (no mask, and some key is visible to every row).
    auto softmax_tile = [&](auto inside_tag, auto rt_tag, int slot0, const f32x4 (&s)[RT][2], V8 (&p_hi)[RT], V8 (&p_lo)[RT], float (&alpha)[RT]) {
        constexpr bool INSIDE = decltype(inside_tag)::value;
        constexpr int rt = decltype(rt_tag)::value;
        {
            // raw scores; the factor (positive: the maximum commutes with it) goes into the exponent's fma
            float sv[8], bm = -INFINITY;
            if (INSIDE || slot0 + 32 <= n_prefix) {
#pragma unroll
                for (int j = 0; j < 8; ++j) { sv[j] = s[rt][j >> 2][j & 3]; bm = fmaxf(bm, sv[j]); }
            } else {
                // the row's mask words come from memory here: few blocks reach into the region
                bool valid; int m, qh;
                row_of(rt, valid, m, qh);
                const uint64_t m0 = valid ? mask[(size_t)m * MASK_WORDS] : 0ull, m1 = valid ? mask[(size_t)m * MASK_WORDS + 1] : 0ull;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int slot = slot0 + 8 * lg + j;
                    sv[j] = slot_visible(slot, n_prefix, region_len, m0, m1) ? s[rt][j >> 2][j & 3] : -INFINITY;
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
            if (!INSIDE && m_new == -INFINITY) {
#pragma unroll
                for (int j = 0; j < 8; ++j) { p_hi[rt][j] = (T)0.f; p_lo[rt][j] = (T)0.f; }
            } else {
                alpha[rt] = __builtin_amdgcn_exp2f(m_run[rt] - m_new);   // 2^(-inf) = 0 on the first visible block
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float pe = __builtin_amdgcn_exp2f(fmaf(sv[j], scale, -m_new));
                    p_hi[rt][j] = from_f<T>(pe);
                    if constexpr (SPLIT_P) p_lo[rt][j] = from_f<T>(pe - to_f(p_hi[rt][j]));
                    psum += pe;
                }
            }
            l_run[rt] = l_run[rt] * alpha[rt] + psum;
            m_run[rt] = m_new;
            return __builtin_amdgcn_ballot_w64(alpha[rt] != 1.f) != 0;   // rare once the maximum has settled
        }
    };
    auto softmax = [&](auto inside_tag, int slot0, const f32x4 (&s)[RT][2], V8 (&p_hi)[RT], V8 (&p_lo)[RT], float (&alpha)[RT]) {
        bool rescale = softmax_tile(inside_tag, I0{}, slot0, s, p_hi, p_lo, alpha);
        if constexpr (RT > 1) rescale = rescale | softmax_tile(inside_tag, I1{}, slot0, s, p_hi, p_lo, alpha);   // (no short circuit: it would cut the block in two)
        return rescale;
    };
    auto rescale_acc = [&](const float (&alpha)[RT]) {   // behind a wave-uniform branch that is rarely taken
        asm volatile("" ::: "memory");                   // (keeps the compiler from turning it into 64 selects)
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) acc[rt][dt] *= alpha[rt];
    };

    // Schedule.  The loads of an iteration are issued two iterations before the first wave reads them: at the top of
    // iteration `it` go the keys of it + 3 (stage last read by the scores of it - 1, at least one barrier ago) and the
    // values of it + 2 (stage last read by the P V of it - 2, at least one barrier ago); at its foot every wave waits
    // until only those are outstanding, and the barrier then publishes the keys of it + 2 and the values of it + 1.
    // The waves of a workgroup move in step from barrier to barrier, and with two key-ways a SIMD holds one wave of
    // each.  The two key-ways take an iteration in opposite order, so that one wave of a SIMD has vector work while the
    // other has matrix work:
    //   way 0: softmax of it (scores formed an iteration ago), then P V of it and scores of it + 1      vector, matrix
    //   way 1: scores of it + 1 and P V of it (probabilities formed an iteration ago), then softmax of it + 1
    // The accumulators of a key-way see the same operations in the same order either way.  (One key-way: the order of
    // way 0.)  Measured against both ways in way 0's order with the next scores ahead of the softmax: 35.5 against
    // 35.9 us at 8192 tokens - timestamps taken inside the kernel show each wave's own chain (LDS reads, a run of
    // dependent MFMAs, the softmax) at about 3000 of an iteration's 4200 cycles whatever the other wave does.
    // The P V product of an iteration is unconditional (a conditional one made the compiler keep two copies of the
    // accumulators): way 1's block beyond an odd end gets zero probabilities against the valid block staged in its place.
    typedef std::integral_constant<bool, true> Inside;
    typedef std::integral_constant<bool, false> Anywhere;
    const bool matrix_first = KW == 2 && kway == 1;        // wave-uniform
    issue_k(0);
    issue_k(1);
    issue_v(0);
    issue_k(2);
    issue_v(1);
    dma_wait<2 * UPT>();                                  // keys of iterations 0 and 1 and values of iteration 0 have landed
    __syncthreads();
    // softmax of block b's scores -> probabilities; accumulators rescaled
    auto softmax_block = [&](int b, const f32x4 (&s)[RT][2], V8 (&p_hi)[RT], V8 (&p_lo)[RT]) {
        float alpha[RT];
        const bool rescale = (b << 5) + 32 <= n_prefix ? softmax(Inside{}, b << 5, s, p_hi, p_lo, alpha)
                                                       : softmax(Anywhere{}, b << 5, s, p_hi, p_lo, alpha);
        if (rescale) rescale_acc(alpha);
    };
    auto top = [&](int it) {
        if (it + 3 < n_it) issue_k(it + 3);               // workgroup-uniform, like the waits at the foot
        if (it + 2 < n_it) issue_v(it + 2);
    };
    auto foot = [&](int it) {
        if (it + 3 < n_it) dma_wait<2 * UPT>();
        else if (it + 2 < n_it) dma_wait<UPT>();
        else dma_wait<0>();
        __syncthreads();
    };
    // (one loop per order, each with the state of its own order only: scores kept from iteration to iteration in
    // the first, probabilities in the second.  Branches on block indices are wave-uniform.)
    if (!matrix_first) {
        f32x4 s[RT][2];
        scores(0, s);                                     // way 0's block of an iteration always exists
        for (int it = 0; it < n_it; ++it) {
            top(it);
            const int b = b0 + it * KW + kway;
            V8 p_hi[RT], p_lo[RT];
            softmax_block(b, s, p_hi, p_lo);
            __builtin_amdgcn_sched_barrier(0);            // (operand reads hoisted above the softmax would not fit the registers)
            pv(it, p_hi, p_lo);
            if (b + KW < b1) scores(it + 1, s);
            foot(it);
        }
    } else {
        V8 p_hi[RT], p_lo[RT];
        f32x4 s[RT][2];
        auto probabilities = [&](int b) {                 // of block b from its scores in s; zero beyond the end
            if (b < b1) {
                softmax_block(b, s, p_hi, p_lo);
            } else {
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                    for (int j = 0; j < 8; ++j) { p_hi[rt][j] = (T)0.f; p_lo[rt][j] = (T)0.f; }
            }
        };
        if (b0 + kway < b1) scores(0, s);
        probabilities(b0 + kway);
        for (int it = 0; it < n_it; ++it) {
            const int b_next = b0 + (it + 1) * KW + kway;
            // The next block's scores lead the matrix part: by the time the P V products are issued they are complete,
            // and the softmax behind them starts at once (and needs the matrix pipe no more while way 0 fills it).
            top(it);
            if (b_next < b1) scores(it + 1, s);
            pv(it, p_hi, p_lo);
            __builtin_amdgcn_sched_barrier(0);
            probabilities(b_next);
            foot(it);
        }
    }
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        l_run[rt] += __shfl_xor(l_run[rt], 16, 64);
        l_run[rt] += __shfl_xor(l_run[rt], 32, 64);
    }

    if constexpr (KW > 1) {
        // Merge the KW partial (max, sum, O) of each row tile in key-way order: ways 1.. park theirs
        // in LDS (the stages are free once every wave has read its last values), way 0 folds them in;
        // one tile of each wave at a time.
        float *xch = reinterpret_cast<float *>(lds_all);  // per (way-1, wave): 64 lanes x (DT*4 + 2) floats
        constexpr int REC = DT * 4 + 2;
        static_assert((size_t)(KW - 1) * WPW * 64 * REC * sizeof(float) <= sizeof(lds_all), "merge records must fit");
        float *mine = xch + ((size_t)((kway - 1) * WPW + wq) * 64 + lane) * REC;
        __syncthreads();
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
                    const float *o = xch + ((size_t)((w - 1) * WPW + wq) * 64 + lane) * REC;
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
            bool valid; int m, qh;
            row_of(rt, valid, m, qh);
            if (valid) {
                const float inv = 1.0f / l_run[rt];
                T *dst = out_direct + ((size_t)m * hq + qh) * DH + 4 * lg;
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
constexpr int ATTN_MAX_BPS = 64;                         // blocks per split the kernel can address (one page-table entry per lane)
static int blocks_per_split(int n_prefix, int keys_per_split) {
    if (keys_per_split > 0) return keys_per_split >= 32 ? (keys_per_split / 32 < ATTN_MAX_BPS ? keys_per_split / 32 : ATTN_MAX_BPS) : 1;
    const int prefix_blocks = (n_prefix + 31) / 32;
    int bps = (prefix_blocks + 3) / 4;
    if (bps < 4) bps = 4;
    const int cap = keys_per_split < 0 && -keys_per_split >= 128 ? -keys_per_split / 32 : 32;
    if (bps > cap) bps = cap;
    return bps;
}

// Launch shape of one sequence's attention: the split rule, key-ways and row tiles per wave.
// Key-ways follow the split size (so, like it, the committed prefix only); the number of row tiles per wave may follow
// the row count: it does not change any row's arithmetic.  Eight tiles per workgroup where the walk is long (every key /
// value block staged once for eight tiles), as 4 waves x 2 tiles per key-way; 8 waves x 1 tile (sixteen waves per
// workgroup, four per SIMD) measured the same.
struct AttnShape { int bps, n_splits, kw, rt, n_row_groups, rho_pad, n_wgs; };
static AttnShape attention_shape(const ModelDims &md, int rows, int n_prefix, int region_len, int keys_per_split,
                                 bool crowded = false) {
    AttnShape a;
    const int G = md.hq / md.hkv;
    const int tiles = (rows * G + 15) / 16;
    a.rho_pad = tiles * 16;
    const int n_blocks = (n_prefix + region_len + 31) / 32;
    a.bps = blocks_per_split(n_prefix, keys_per_split);
    while ((n_blocks + a.bps - 1) / a.bps > ATTN_MAX_SPLITS) a.bps *= 2;     // only with a tiny split override on a very long context
    a.n_splits = (n_blocks + a.bps - 1) / a.bps;
    a.kw = a.bps >= 4 ? 2 : 1;
    // pays where the walk is long - or where the launch would otherwise hold more workgroups than the chip has CUs
    // (a workgroup fills a CU's LDS: the surplus would run as a second round)
    a.rt = tiles > 4 && (a.bps >= 8 || crowded) ? 2 : 1;
    a.n_row_groups = (tiles + 4 * a.rt - 1) / (4 * a.rt);
    a.n_wgs = 8 * a.n_row_groups * ((md.hkv * a.n_splits + 7) / 8);
    return a;
}

template <typename T>
static void launch_attention_t(const ModelDims &md, const void *q, int rows, const RowMeta &rm, int n_prefix,
                               int region_len, const KVCache &kv, int keys_per_split, const AttnScratch &sc,
                               void *out, hipStream_t st) {
    const AttnShape a = attention_shape(md, rows, n_prefix, region_len, keys_per_split);
    const float scale = 1.4426950408889634f / sqrtf((float)md.dh);     // log2(e) / sqrt(dh): scores in the log2 domain
    T *direct = a.n_splits == 1 ? static_cast<T *>(out) : nullptr;
#define POSS_ATTN(DH, KW, RT)                                                                                     \
    hipLaunchKernelGGL((attn_mfma_kernel<T, DH, KW, RT>), dim3(a.n_wgs), dim3(256 * KW), 0, st,                  \
                       static_cast<const T *>(q), rows, md.hq, md.hkv, rm.mask, n_prefix, region_len, kv, a.bps,  \
                       a.n_splits, a.n_row_groups, scale, sc.o, sc.ml, a.rho_pad, direct)
#define POSS_ATTN_DH(DH)                                                                                         \
    do {                                                                                                         \
        if (a.kw == 2) { if (a.rt == 2) POSS_ATTN(DH, 2, 2); else POSS_ATTN(DH, 2, 1); }                         \
        else           { if (a.rt == 2) POSS_ATTN(DH, 1, 2); else POSS_ATTN(DH, 1, 1); }                         \
    } while (0)
    if (md.dh == 128) POSS_ATTN_DH(128); else POSS_ATTN_DH(64);
#undef POSS_ATTN_DH
#undef POSS_ATTN
    if (a.n_splits > 1)
        hipLaunchKernelGGL((attn_merge_kernel<T>), dim3(rows, md.hq), dim3(md.dh < 64 ? 64 : md.dh), 0, st, sc.o, sc.ml,
                           a.n_splits, md.hq, md.hkv, md.dh, a.rho_pad, static_cast<T *>(out));
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
    int wgs_all = 0;
    for (int i = 0; i < n; ++i)
        wgs_all += attention_shape(md, segs[i].rows, segs[i].n_prefix, segs[i].region_len, keys_per_split).n_wgs;
    const bool crowded = wgs_all > 256;
    for (int i = 0; i < n; ++i) {
        const AttnSeg &g = segs[i];
        shp[i] = attention_shape(md, g.rows, g.n_prefix, g.region_len, keys_per_split, crowded);
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
