// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace poss {

typedef __bf16   bf16_t;
typedef _Float16 f16_t;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte load
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

enum { DT_F32 = 0, DT_BF16 = 1, DT_F16 = 2 };
static inline size_t dtype_size(int dt) { return dt == DT_F32 ? 4 : 2; }

// ---------------------------------------------------------------- GEMM geometry
// Y[M, N] = X[M, K] . W[N, K]^T with M <= 128 rows: the weight matrix is streamed once.
// 16-bit types use v_mfma_f32_16x16x32 with the activations as A (rows m) and the weights
// as B (columns n).  Weights are repacked at load time into B-operand order:
//   Wp[n_group][k_step][nt][lane][8],  n = (n_group*GEMM_NT + nt)*16 + lane%16,
//                                       k = k_step*32 + (lane/16)*8 + j
// so that one wave reads GEMM_NT KiB per k-step, contiguous and in k order.
#ifndef POSS_GEMM_NT
#define POSS_GEMM_NT 2
#endif
#ifndef POSS_GEMM_WPB
#define POSS_GEMM_WPB 4
#endif
constexpr int GEMM_NT      = POSS_GEMM_NT;            // 16-column tiles per wave
constexpr int GEMM_WPB     = POSS_GEMM_WPB;           // waves per workgroup
constexpr int GEMM_BLOCK_N = GEMM_NT * 16 * GEMM_WPB; // 128 columns per workgroup
constexpr int GEMM_KSTEP   = 32;
constexpr int GEMM_KCHUNK  = 256;                     // K is padded to this at pack time
constexpr int MAX_ROWS     = 128;                     // rows of one sequence in a pass (tree masks are 128 bits wide)
constexpr int LAUNCH_ROWS  = 256;                     // rows one weight-streaming launch carries (several sequences, prefill)
constexpr int MASK_WORDS   = 2;

static inline int round_up(int x, int m) { return (x + m - 1) / m * m; }
static inline int gemm_npad(int n) { return round_up(n, GEMM_BLOCK_N); }
static inline int gemm_kpad(int dt, int k) { return dt == DT_F32 ? k : round_up(k, GEMM_KCHUNK); }
static inline size_t packed_elems(int dt, int n, int k) { return (size_t)gemm_npad(n) * gemm_kpad(dt, k); }

struct GemmShape {
    int M;          // real rows
    int N, K;       // logical sizes
    int Npad, Kpad; // padded sizes of the packed weight
    int S;          // K splits (chunks dealt out evenly); partial sums land in part[S][Mpad][Npad]
    int Mpad;       // rows of one partial plane (row stride Npad)
};
GemmShape gemm_plan(int dt, int M, int N, int K, int target_wgs);

struct PackSrc {
    const void *ptr[3]; int rows[3];   // up to three matrices stacked along N
    int interleave16;                  // 1: ptr[0]/ptr[1] alternate in groups of 16 rows (gate | up per 32-column wave tile)
    int rope_dh;                       // > 0 (16-bit types): rows are heads of rope_dh dims; inside each head the columns are permuted so
                                       // that a 32-column wave tile holds dims [16j, 16j+16) and their rotary partners [16j + dh/2, ..)
};
void launch_pack(int dt, const PackSrc &src, int K, void *dst, hipStream_t st);
static inline int gate_up_rows(int F) { return 2 * round_up(F, 16); }

// ---------------------------------------------------------------- KV caches
// K  : [phys_page][Hkv][P][dh]      (row per token)
// Vt : [phys_page][Hkv][dh][P]      (tokens contiguous: the A operand of O^T = V^T P^T)
struct KVCache {
    void *k, *vt;
    const int32_t *page_table;     // device: logical page -> physical page
    int page_shift;                // log2(P)
};

struct ModelDims {
    int d, hq, hkv, dh, ffn, vocab;
    float eps, theta;
    int dt;
};

// Per-row metadata of one pass, all DEVICE arrays.
struct RowMeta {
    const int32_t  *pos;    // rotary position
    const int32_t  *slot;   // cache slot the row's key/value is written to
    const uint64_t *mask;   // [rows][MASK_WORDS] visibility over region slots (bit j = slot region0 + j)
};

// ---------------------------------------------------------------- GEMM with fused epilogue
// The stream kernel writes split-K partial planes; an epilogue kernel with one workgroup per
// 128-column tile sums them in split order and applies the fused operation.
enum { EPI_PLAIN = 0, EPI_ROPE_KV = 1, EPI_RESIDUAL = 2, EPI_SILU = 3, EPI_HEAD = 4 };
// What the Head GEMM reduces in its own epilogue (EPI_HEAD, 16-bit types, K unsplit): every workgroup owns whole
// columns of every row, so it leaves, per row, the winner or the k best of its columns instead of (or besides) logits.
enum { HEAD_ARGMAX = 1, HEAD_TOPK = 2 };
constexpr int TOPK_MAXK = 16;
constexpr int TOPK_REC = 2 + 2 * TOPK_MAXK;    // segment record: [max, sum exp(l - max), k values, k indices (as bits)]
struct EpiArgs {
    int mode;
    // EPI_PLAIN: out[m][n] = sum (with out == nullptr and S == 1 plane 0 is the result, row stride Npad)
    float *out; int ld_out;
    // EPI_ROPE_KV: columns are [q heads | k heads | v heads]; rows < rows_q get a rotated query,
    // every row its rotated key and its value written to cache slot slot[m]
    int rows_q; const float2 *cs; const int32_t *slot; void *q; KVCache kv; int hq, hkv, dh;
    int rope_packed;   // set by the launcher: the columns of a head are in the packed order of PackSrc::rope_dh
    // EPI_RESIDUAL: h[m][n] = sum + bias[n] + (residual ? h[m][n] : 0); h_copy likewise; then, if
    // gain != nullptr, u[m][n] = T(rmsnorm(h[m]) * gain[n]) - the operand of the next GEMM
    float *h; const void *bias; int residual; float *h_copy; const void *gain; void *u;
    // EPI_HEAD (N = vocabulary; the stream kernel's column tile is a "segment"; seg_out / pv, pi must hold
    // gemm_head_segments() entries per row): head_mode HEAD_ARGMAX: pv/pi[row * n_seg + seg] = best (value, index) of the
    // segment, ties to the lower index; HEAD_TOPK: seg_out[(row * n_seg + seg) * TOPK_REC ..] = the segment's record.
    // write_logits != 0: the float32 logits are also written to the partial-plane buffer (row stride Npad).
    int head_mode, head_k, write_logits; float *seg_out; float *pv; int *pi;
    // EPI_SILU: columns [32j, 32j+16) hold gate[16j..16j+15], the next 16 up[16j..16j+15], so one MFMA lane
    // owns both factors of act[m][f] = T(silu(gate) * up); with S == 1 the stream kernel writes act itself
    void *act; int F;
};
// part must hold S * Mpad * Npad floats.  X row-major [M][ldx] of dtype dt.  ev_start / ev_stop, if both
// given, receive the begin and end timestamps of the weight-streaming kernel itself (per-launch timing).
// Returns false, launching nothing, if a pointer the chosen epilogue writes through is null.
// EPI_ROPE_KV (the QKV projection; 16-bit types: one kernel that needs no partial planes, weights packed with
// PackSrc::rope_dh): `ranges`, if given, sends row ranges [r0, r1) each into its own cache with its own query limit
// (rows below rows_q get a rotated query) - several sequences batched into one launch; row indices stay those of the
// launch (epi.cs, epi.slot, epi.q are indexed by them), epi.kv and epi.rows_q are ignored, blk0 is filled in here.
constexpr int ROPE_MAX_RANGES = 16;
struct RopeRanges { int n; int r0[ROPE_MAX_RANGES], r1[ROPE_MAX_RANGES], rows_q[ROPE_MAX_RANGES], blk0[ROPE_MAX_RANGES]; KVCache kv[ROPE_MAX_RANGES]; };
bool launch_gemm(int dt, const GemmShape &g, const void *Wp, const void *X, int ldx, float *part,
                 const EpiArgs &epi, float rms_eps, hipStream_t st, hipEvent_t ev_start = nullptr,
                 hipEvent_t ev_stop = nullptr, const RopeRanges *ranges = nullptr);
// Column tiles ("segments") of an unsplit launch of this shape, i.e. records per row an EPI_HEAD launch writes;
// head_segments_max bounds it for any row count.
int gemm_head_segments(const GemmShape &g);
static inline int head_segments_max(int vocab) { return gemm_npad(vocab) / GEMM_BLOCK_N; }

// ---------------------------------------------------------------- launchers: elementwise
// also writes the rotary table of the rows: cs[m][i] = (cos, sin)(pos[m] * theta^(-2i/dh)), angle formed in float64
void launch_embed_norm(const ModelDims &md, const void *embed, const int32_t *tokens, int rows,
                       const void *gain, float *h, void *u, const int32_t *pos, const double *inv_freq,
                       float2 *cs, hipStream_t st);
size_t argmax_scratch_floats(int rows, int vocab);
void launch_argmax(const float *logits, int ld, int rows, int vocab, float *scratch, int32_t *out, hipStream_t st);
// second stage alone: pv / pi hold n_seg partial winners per row
void launch_argmax_merge(const float *pv, const int *pi, int n_seg, int rows, int32_t *out, hipStream_t st);
// Temperature sampling: out[r] = first id whose cumulative probability under softmax(logits[r] / temperature)
// exceeds u_by_depth[depth ? depth[r] : 0] (DEVICE arrays).  Returns false (nothing launched) for temperature <= 0
// or a vocabulary beyond 4M entries.
size_t sample_scratch_floats(int rows, int vocab);
bool launch_sample(const float *logits, int ld, int rows, int vocab, float temperature, const float *u_by_depth,
                   const int32_t *depth, float *scratch, int32_t *out, hipStream_t st);
void launch_copy_rows_f32(const float *src, int ld_src, float *dst, int ld_dst, int rows, int cols,
                          hipStream_t st);

// ---------------------------------------------------------------- attention
struct AttnScratch { float *o; float *ml; };  // partial outputs [split][Hq][rows][dh], (m, l) pairs
void launch_attention(const ModelDims &md, const void *q, int rows, const RowMeta &rm, int n_prefix,
                      int region_len, const KVCache &kv, int keys_per_split, const AttnScratch &sc,
                      void *out, hipStream_t st);
// The same for several sequences whose rows [row0, row0 + rows) share the q / mask / out buffers (segs in row
// order): one launch for all of them (and one merge), each sequence against its own cache with its own split count.
// The partial buffers must hold every sequence's slices: row tiles padded per sequence.
struct AttnSeg { int row0, rows, n_prefix, region_len; const KVCache *kv; };
void launch_attention_batch(const ModelDims &md, const void *q, const RowMeta &rm, const AttnSeg *segs, int n,
                            int keys_per_split, const AttnScratch &sc, void *out, hipStream_t st);

// ---------------------------------------------------------------- draft-tree kernels
struct TreeDev {            // device-resident tree state of one round
    // candidate pool
    int32_t *pool_token, *pool_parent, *pool_depth; float *pool_score;
    // frontier of each depth: [depth][k]
    int32_t *fr_pool, *fr_token, *fr_parent_rank; float *fr_score; uint64_t *fr_mask;
    // per-pass top-k results [k rows][k]
    int32_t *topk_id; float *topk_logp;
    // final tree
    int32_t *n_nodes, *token, *parent, *depth, *pos; uint64_t *mask; float *score;
    // candidate <-> tree node, written with the final tree: pool_node[candidate] = node index or -1 (dropped),
    // node_pool[node] = candidate index (-1 for the root)
    int32_t *pool_node, *node_pool;
};
// Verification at a temperature with DRAWN children (the rejection-sampling rule).
// Children: for each of `rows` logits rows, k distinct ids drawn one after the other from softmax(logits / temperature),
// each from what the earlier draws left (inverse CDF in vocabulary order), draw i of row r with u[r * k + i]; out_logp is
// the log-probability under the full distribution.  One workgroup per row.
void launch_sample_children(const float *logits, int ld, int rows, int vocab, int k, float temperature, const float *u,
                            int32_t *out_id, float *out_logp, hipStream_t st);
// The walk: from the root, the k drawn children of the current node (candidates cbase .. cbase + k - 1 of the pool, in
// draw order) are tested with ua[depth * (k + 1) + i] against min(1, p / q), p from the target's logits row of the node,
// q from the drafter's logits row that produced the children (draft_logits row 0 for the root, 1 + (depth - 1) * k + rank
// for a frontier node); after a rejection p becomes the positive part of p - q and q loses the candidate.  An accepted child
// that the tree kept becomes the current node; otherwise the walk ends with one more token (an accepted child the tree
// dropped, a draw from the last residual with ua[depth * (k + 1) + k], or at a node without drawn children a draw from
// the target's distribution).  The result is written as the g[] of a greedy walk: g[node] = next token for every
// node of the path, so that the commit kernel reproduces it.  resid: vocab floats of scratch.
void launch_rejection_walk(const TreeDev &td, int k, int L, int vocab, const float *target_logits, const float *draft_logits,
                           int ld, float temperature, const float *ua, float *resid, int32_t *g, hipStream_t st);
size_t topk_scratch_floats(int rows, int vocab);
// second stage alone, over n_seg segment records per row (written by topk_seg_kernel or by an EPI_HEAD launch)
void launch_topk_merge(const float *seg_records, int n_seg, int rows, int k, int32_t *out_id, float *out_logp, hipStream_t st);
void launch_topk_logsoftmax(const float *logits, int ld, int rows, int vocab, int k, float *seg_scratch,
                            int32_t *out_id, float *out_logp, hipStream_t st);
// Both take the trees of n_seq <= TREE_BATCH_MAX sequences (arrays of n_seq entries): one workgroup each.
constexpr int TREE_BATCH_MAX = 8;
void launch_tree_expand(const TreeDev *tds, int n_seq, int d, int k, int L, int rows, int vocab, hipStream_t st);
// also writes the KV slot of every node (slot_out[s][i] = t[s] + i), which the verification pass reads
void launch_tree_finalize(const TreeDev *tds, int n_seq, int k, int L, int n_keep, const int *t,
                          const int32_t *const *tokens_dev, int32_t *const *slot_out, hipStream_t st);
// rows of [embedding ; feature] pairs for one specialist pass
struct DraftRowPlan {
    int n_rows;
    uint64_t mask0[MASK_WORDS];   // region mask given to rows of kind 0 and 1
    int16_t kind[MAX_ROWS];       // 0: committed pair (idx = drafter index i); 1: stored frontier row
                                  // (idx = temp row); 2: new frontier row (idx = rank in this depth)
    int32_t idx[MAX_ROWS];
    int32_t slot[MAX_ROWS];
    int32_t pos[MAX_ROWS];
    int16_t dst[MAX_ROWS];        // row of the pass this plan row is written to (several sequences share a pass)
};
void launch_draft_assemble(const ModelDims &md, const DraftRowPlan &plan, int depth_index, int k,
                           const void *embed, const int32_t *tokens_dev, const void *feat_stash,
                           const TreeDev &td, const float *fhat_prev, void *xin_tmp, void *x_out,
                           int32_t *pos_out, int32_t *slot_out, uint64_t *mask_out, const double *inv_freq,
                           float2 *cs, hipStream_t st);     // also writes the rows' rotary table cs

// ---------------------------------------------------------------- accept + commit
void launch_tree_upload_finish(int n, int t, const int32_t *token, const int32_t *parent, int32_t *depth,
                               int32_t *pos, int32_t *slot, uint64_t *mask, hipStream_t st);
// One launch: the greedy walk over the verified tree, then KV compaction, feature stash and token
// stream.  walk_dev / result: [0] = m, [1] = bonus token, [2..2+m] = node indices of the accepted
// path; result[32 + j] = committed token j.  result must be host memory mapped into the device.
void launch_commit(const ModelDims &md, int n_layers, const KVCache *caches_dev, const int32_t *tree_token,
                   const int32_t *tree_parent, const int32_t *g, const int32_t *n_nodes, int max_path, int t,
                   const float *feats, void *feat_stash, int32_t *tokens_dev, int32_t *walk_dev, int32_t *result,
                   hipStream_t st);

void launch_read_kv(const ModelDims &md, const KVCache &kv, int slot0, int n, float *k_out, float *v_out,
                    hipStream_t st);
void launch_fill_u32(uint32_t *p, size_t n, uint32_t v, hipStream_t st);
int attention_splits(int total_keys, int keys_per_split);

}  // namespace poss
