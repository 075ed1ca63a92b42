// Host side of the C ABI (include/poss.h): context, workspace carving, weight repacking, the pass
// schedules of prefill / draft / verify / accept-and-commit.  No arithmetic of the method happens
// here: every step is a kernel launch on the caller's stream.  A context carries one or several
// sequences; a pass stacks the rows of all of them so that they share the weight streams.
#include "../../include/poss.h"
#include "common.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

using namespace poss;

namespace {

char g_load_error[512] = "";

struct LayerW { const void *attn_norm, *wqkv, *wo, *mlp_norm, *wgu, *wdown; };
struct SpecW  { const void *fc_w, *fc_b; LayerW layer; };

// Bump allocator over the caller's workspace; with base == nullptr it only measures.
struct Arena {
    char *base; size_t off = 0;
    explicit Arena(void *b) : base(static_cast<char *>(b)) {}
    void *take(size_t bytes) {
        off = (off + 255) / 256 * 256;
        void *p = base ? base + off : nullptr;
        off += bytes;
        return p;
    }
    template <typename T> T *take_n(size_t n) { return static_cast<T *>(take(n * sizeof(T))); }
};

enum { ST_LOADED = 0, ST_READY = 1, ST_VERIFIED = 2 };
constexpr int PROFILE_EVENTS = 1024;

}  // namespace

// One sequence of the batch: its caches, its tree, its token stream.  Weights and activation
// buffers are shared; a pass stacks the rows of every sequence into one set of GEMM launches.
struct Seq {
    std::vector<KVCache> target_kv, spec_kv;
    KVCache *target_kv_dev;
    TreeDev td;                        // final-tree arrays are slices of the batch-wide row arrays
    int32_t *tree_slot, *tokens_dev, *walk_dev;
    void *feat_stash, *xin_tmp;
    int32_t *result_pinned, *result_dev;   // the commit kernel's result: host memory and its device address
    int t, tree_ready, tree_n, tree_row0, prefilled;   // tree_row0: first row of its tree in the batch-wide arrays
    int active;                        // takes part in the rounds (poss_set_active)
    std::vector<int32_t> tokens;
    std::vector<int> spec_len, spec_tmp_depth;
    int last_m;                        // the last commit: accepted drafts, path, committed tokens
    int32_t last_path[POSS_MAX_DEPTH + 1], last_tokens[POSS_MAX_DEPTH + 1];
};

struct poss_ctx {
    poss_config cfg;
    ModelDims md;
    hipStream_t st;
    char err[512];
    // weights (workspace)
    const void *embed, *lm_head, *final_norm;
    std::vector<LayerW> layers;
    std::vector<SpecW> specs;
    // caches
    int cache_slots, n_pages;
    int32_t *page_table;
    size_t cache_bytes_each;
    int B;                             // sequences per round
    int rows_all;                      // rows of the batch-wide tree arrays
    std::vector<Seq> seq;
    // activations
    float *h, *part, *logits, *feats, *fhat[2], *topk_scratch, *taps_user;
    float2 *cs;
    void *u, *xin, *q, *attn_out, *act;
    AttnScratch attn_sc;
    int32_t *row_pos, *row_slot;
    uint64_t *row_mask;
    int32_t *tree_token_all, *tree_pos_all, *tree_slot_all, *tree_depth_all, *tree_parent_all;   // rows of the verification pass, all sequences
    uint64_t *tree_mask_all;
    float *tree_score_all;
    int32_t *topk_id_all; float *topk_logp_all;
    int32_t *argmax_dev;
    double *inv_freq;
    // host state
    int state;
    poss_stats stats;
    void *pinned; size_t pinned_bytes;
    int32_t *result_pinned_all;
    hipEvent_t ev[6];                  // begin/end of the draft, verify and commit phases
    bool ev_pending[3];                // phase recorded, elapsed time not yet added to the statistics
    bool launch_refused;               // a GEMM launch was refused on the host (null operand): internal error
    float temperature;                 // 0: greedy verification; > 0: the target's tokens are drawn (poss_set_sampling)
    float *u_pinned, *u_dev;           // per sequence, one uniform number per tree depth: host staging and device copy
    // drawn children (poss_set_draft_sampling): uniform numbers of the draws [depth][k][k] and of the tests [depth + 1][k + 1]
    // (host staging, device copies), the drafter's logits of every expanded node, the residual vector of the walk
    int draft_sampling;
    float *ud_pinned, *ua_pinned, *ud_dev, *ua_dev, *dlogits, *resid;
    int gemm_target_wgs, attn_keys_per_split;
    int launch_rows;                   // rows one launch of a batch's pass carries (POSS_LAUNCH_ROWS unless lowered for a sweep)
    // gemm profiling
    int prof_on, prof_n;
    hipEvent_t prof_ev[2 * PROFILE_EVENTS];
    double prof_bytes;
};

namespace {

int fail(poss_ctx *c, int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(c ? c->err : g_load_error, 512, fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(c, call)                                                                        \
    do {                                                                                        \
        hipError_t e_ = (call);                                                                 \
        if (e_ != hipSuccess) return fail(c, POSS_E_HIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)


const char *check_config(const poss_config &c) {
    if (c.n_layers < 1 || c.d_model < 8 || c.n_q_heads < 1 || c.n_kv_heads < 1 || c.d_ffn < 8 || c.vocab < 2)
        return "non-positive model dimension";
    if (c.dtype < 0 || c.dtype > 2) return "dtype must be 0 (f32), 1 (bf16) or 2 (f16)";
    if (c.d_model > 16384) return "d_model above 16384 is not supported by the residual epilogue";
    if (c.n_q_heads % c.n_kv_heads) return "n_q_heads must be a multiple of n_kv_heads";
    if (c.dtype != POSS_DTYPE_F32 && c.head_dim != 64 && c.head_dim != 128)
        return "16-bit kernels support head_dim 64 or 128";
    if (c.head_dim < 2 || c.head_dim > 256 || (c.head_dim & 1)) return "head_dim must be even and <= 256";
    if (c.dtype != POSS_DTYPE_F32 && ((c.d_model % 8) || (c.d_ffn % 8))) return "16-bit kernels need d_model, d_ffn multiples of 8";
    if (c.n_specialists < 1 || c.positions_per_specialist < 1) return "need at least one specialist and one position each";
    if (c.top_k < 1 || c.top_k > 16 || c.top_k >= c.vocab) return "top_k must be in 1..16 and below vocab";
    if (c.depth < 1 || c.depth > POSS_MAX_DEPTH) return "depth must be in 1..16";
    const int pool = c.top_k + (c.depth - 1) * c.top_k * c.top_k;
    if (c.total_tokens < 1 || c.total_tokens + 1 > POSS_MAX_ROWS) return "total_tokens must be in 1..127";
    if (c.total_tokens > pool) return "total_tokens exceeds the candidate pool k + (depth-1) k^2";
    if (pool > 2048) return "candidate pool too large";
    if ((long long)head_segments_max(c.vocab) * c.top_k > 64 * 256) return "vocab * top_k too large for the top-k merge";
    if ((c.depth - 1) * c.top_k > 64 * POSS_MASK_WORDS) return "(depth-1)*top_k must fit the 128-bit ancestor mask";
    if (c.top_k + (c.depth + 1) + (c.depth - 1) * c.top_k > POSS_MAX_ROWS) return "a specialist pass would exceed 128 rows";
    if (c.kv_page_tokens != 32 && c.kv_page_tokens != 64 && c.kv_page_tokens != 128) return "kv_page_tokens must be 32, 64 or 128";
    if (c.max_seq < 2 || c.max_seq % c.kv_page_tokens) return "max_seq must be a positive multiple of kv_page_tokens";
    // attention cuts the keys into at most 256 splits of at most 64 blocks of 32
    if (c.max_seq > 500000) return "max_seq above 500000 is not supported";
    if (c.kv_page_order < 0 || c.kv_page_order > 1) return "kv_page_order must be 0 or 1";
    if (!(c.rms_eps >= 0.f) || !(c.rope_theta > 0.f)) return "rms_eps / rope_theta out of range";
    if (c.batch < 0 || c.batch > 8) return "batch must be in 0..8 (0 and 1: one sequence)";
    // the float32 attention kernel keeps one score per cache slot in LDS (64 KiB without opting in to more)
    if (c.dtype == POSS_DTYPE_F32 && (size_t)(c.max_seq + POSS_MAX_ROWS + c.kv_page_tokens) * sizeof(float) > 64 * 1024)
        return "float32 storage supports max_seq up to about 16000 (scores of one row are kept in LDS)";
    return nullptr;
}

size_t esize(const poss_config &c) { return dtype_size(c.dtype); }

// Lays every buffer out in the arena (measuring when it has no base) and, if ctx != nullptr,
// records the addresses.  Weight destinations are returned through ctx as well.
struct WeightSlots {
    void *embed, *lm_head, *final_norm;
    std::vector<void *> layer;   // [n_layers][6]: attn_norm, wqkv, wo, mlp_norm, wgu, wdown
    std::vector<void *> spec;    // [S][8]: fc_w, fc_b, then the 6
};

size_t carve(const poss_config &c, Arena &a, poss_ctx *ctx, WeightSlots *ws) {
    const int dt = c.dtype;
    const size_t es = esize(c);
    const int d = c.d_model, qd = c.n_q_heads * c.head_dim, kd = c.n_kv_heads * c.head_dim, F = c.d_ffn, V = c.vocab;
    auto layer_slots = [&](std::vector<void *> &out) {
        out.push_back(a.take(d * es));
        out.push_back(a.take(packed_elems(dt, qd + 2 * kd, d) * es));
        out.push_back(a.take(packed_elems(dt, d, qd) * es));
        out.push_back(a.take(d * es));
        out.push_back(a.take(packed_elems(dt, gate_up_rows(F), d) * es));
        out.push_back(a.take(packed_elems(dt, d, F) * es));
    };
    WeightSlots local;
    WeightSlots &w = ws ? *ws : local;
    w.embed = a.take((size_t)V * d * es);
    w.lm_head = a.take(packed_elems(dt, V, d) * es);
    w.final_norm = a.take(d * es);
    for (int l = 0; l < c.n_layers; ++l) layer_slots(w.layer);
    for (int s = 0; s < c.n_specialists; ++s) {
        w.spec.push_back(a.take(packed_elems(dt, d, 2 * d) * es));
        w.spec.push_back(a.take(d * es));
        layer_slots(w.spec);
    }
    // caches: every sequence has its own storage and shares the page table
    const int B = c.batch > 1 ? c.batch : 1;
    const int P = c.kv_page_tokens;
    const int slots = round_up(c.max_seq + MAX_ROWS, P), pages = slots / P;
    const size_t cache_each = (size_t)pages * c.n_kv_heads * P * c.head_dim * es;
    int32_t *pt = a.take_n<int32_t>(pages);
    std::vector<void *> kvp;
    for (int i = 0; i < B * 2 * (c.n_layers + c.n_specialists); ++i) kvp.push_back(a.take(cache_each));
    KVCache *kv_dev = a.take_n<KVCache>((size_t)B * c.n_layers);
    // activations
    const int R = LAUNCH_ROWS;
    const int RA = B * (c.total_tokens + 1) > R ? B * (c.total_tokens + 1) : R;   // tree rows of all sequences (several groups)
    size_t part_floats = 0;
    const int shapes[6][2] = {{qd + 2 * kd, d}, {d, qd}, {gate_up_rows(F), d}, {d, F}, {d, 2 * d}, {V, d}};
    for (int i = 0; i < 5; ++i) {
        // split count does not depend on M; planes are at most R rows
        GemmShape g = gemm_plan(dt, R, shapes[i][0], shapes[i][1], 4096);   // upper bound on splits
        const size_t f = (size_t)g.S * R * g.Npad;
        if (f > part_floats) part_floats = f;
    }
    const int QR = B * 16 < R ? B * 16 : R;                  // full rows of a draft pass: at most k <= 16 per sequence
    float *h = a.take_n<float>((size_t)R * d);
    float2 *cs = a.take_n<float2>((size_t)R * (c.head_dim / 2));
    float *part = a.take_n<float>(part_floats);
    float *logits = a.take_n<float>((size_t)R * gemm_npad(V));
    float *feats = a.take_n<float>((size_t)RA * d);
    float *fhat0 = a.take_n<float>((size_t)QR * d), *fhat1 = a.take_n<float>((size_t)QR * d);
    size_t scr_floats = topk_scratch_floats(QR, V);
    if (argmax_scratch_floats(R, V) > scr_floats) scr_floats = argmax_scratch_floats(R, V);
    if (sample_scratch_floats(R, V) > scr_floats) scr_floats = sample_scratch_floats(R, V);
    float *topk_scr = a.take_n<float>(scr_floats);      // shared by top-k (draft) and argmax (verify)
    void *u = a.take((size_t)R * d * es), *xin = a.take((size_t)R * 2 * d * es);
    void *q = a.take((size_t)R * qd * es), *ao = a.take((size_t)R * qd * es), *act = a.take((size_t)R * F * es);
    const int G = c.n_q_heads / c.n_kv_heads;
    const int rho_pad = round_up(R * G, 16) + 16 * 8;          // every sequence of a batch pads its row tiles
    const int max_splits = attention_splits(slots, 64);
    float *ao_part = a.take_n<float>((size_t)max_splits * c.n_kv_heads * rho_pad * c.head_dim);
    float *ml_part = a.take_n<float>((size_t)max_splits * c.n_kv_heads * rho_pad * 2);
    int32_t *row_pos = a.take_n<int32_t>(R), *row_slot = a.take_n<int32_t>(R);
    uint64_t *row_mask = a.take_n<uint64_t>((size_t)R * MASK_WORDS);
    // rows of the verification pass (sequence b owns rows [b * (total_tokens + 1), ...)) and of the top-k
    int32_t *token_all = a.take_n<int32_t>(RA), *pos_all = a.take_n<int32_t>(RA), *slot_all = a.take_n<int32_t>(RA);
    int32_t *depth_all = a.take_n<int32_t>(RA), *parent_all = a.take_n<int32_t>(RA);
    uint64_t *mask_all = a.take_n<uint64_t>((size_t)RA * MASK_WORDS);
    float *score_all = a.take_n<float>(RA);
    int32_t *topk_id_all = a.take_n<int32_t>((size_t)QR * 16); float *topk_logp_all = a.take_n<float>((size_t)QR * 16);
    int32_t *argmax_dev = a.take_n<int32_t>(RA);
    double *inv_freq = a.take_n<double>(c.head_dim / 2);
    float *u_dev = a.take_n<float>((size_t)B * (POSS_MAX_DEPTH + 1));
    float *ud_dev = a.take_n<float>((size_t)c.depth * c.top_k * c.top_k), *ua_dev = a.take_n<float>((size_t)(c.depth + 1) * (c.top_k + 1));
    // one row per expanded node; a pass's Head launch writes whole 16-row tiles, so the last pass needs room beyond its rows
    float *dlogits = a.take_n<float>((size_t)(1 + (c.depth - 1) * c.top_k + 16) * gemm_npad(V));
    float *resid = a.take_n<float>(gemm_npad(V));
    // per sequence: tree state, token stream, feature stash, stored frontier rows
    const int k = c.top_k, L = c.depth, pool = k + (L - 1) * k * k, stride = c.total_tokens + 1;
    std::vector<Seq> seqs(B);
    for (int b = 0; b < B; ++b) {
        Seq &sq = seqs[b];
        TreeDev &td = sq.td;
        td.pool_token = a.take_n<int32_t>(pool); td.pool_parent = a.take_n<int32_t>(pool);
        td.pool_depth = a.take_n<int32_t>(pool); td.pool_score = a.take_n<float>(pool);
        td.fr_pool = a.take_n<int32_t>((L + 1) * k); td.fr_token = a.take_n<int32_t>((L + 1) * k);
        td.fr_parent_rank = a.take_n<int32_t>((L + 1) * k); td.fr_score = a.take_n<float>((L + 1) * k);
        td.fr_mask = a.take_n<uint64_t>((size_t)(L + 1) * k * MASK_WORDS);
        td.topk_id = topk_id_all; td.topk_logp = topk_logp_all;          // re-pointed at the sequence's rows per pass
        td.n_nodes = a.take_n<int32_t>(4);
        td.pool_node = a.take_n<int32_t>(pool); td.node_pool = a.take_n<int32_t>(c.total_tokens + 1);
        td.token = token_all + b * stride; td.parent = parent_all + b * stride;
        td.depth = depth_all + b * stride; td.pos = pos_all + b * stride;
        td.mask = mask_all + (size_t)b * stride * MASK_WORDS; td.score = score_all + b * stride;
        sq.tree_slot = slot_all + b * stride;
        sq.tokens_dev = a.take_n<int32_t>(slots + 8);
        sq.walk_dev = a.take_n<int32_t>(POSS_MAX_DEPTH + 4);
        sq.feat_stash = a.take((size_t)slots * d * es);
        sq.xin_tmp = a.take((size_t)MAX_ROWS * 2 * d * es);
        sq.target_kv_dev = kv_dev + (size_t)b * c.n_layers;
        const int shift = P == 32 ? 5 : P == 64 ? 6 : 7;
        const size_t base = (size_t)b * 2 * (c.n_layers + c.n_specialists);
        for (int l = 0; l < c.n_layers; ++l) sq.target_kv.push_back(KVCache{kvp[base + 2 * l], kvp[base + 2 * l + 1], pt, shift});
        for (int s2 = 0; s2 < c.n_specialists; ++s2)
            sq.spec_kv.push_back(KVCache{kvp[base + 2 * (c.n_layers + s2)], kvp[base + 2 * (c.n_layers + s2) + 1], pt, shift});
    }
    if (ctx) {
        ctx->B = B; ctx->rows_all = RA;
        ctx->cache_slots = slots; ctx->n_pages = pages; ctx->page_table = pt; ctx->cache_bytes_each = cache_each;
        ctx->seq = seqs;
        ctx->cs = cs;
        ctx->h = h; ctx->part = part; ctx->logits = logits; ctx->feats = feats; ctx->fhat[0] = fhat0; ctx->fhat[1] = fhat1;
        ctx->topk_scratch = topk_scr; ctx->u = u; ctx->xin = xin; ctx->q = q; ctx->attn_out = ao; ctx->act = act;
        ctx->attn_sc = AttnScratch{ao_part, ml_part};
        ctx->row_pos = row_pos; ctx->row_slot = row_slot; ctx->row_mask = row_mask;
        ctx->tree_token_all = token_all; ctx->tree_pos_all = pos_all; ctx->tree_slot_all = slot_all;
        ctx->tree_depth_all = depth_all; ctx->tree_mask_all = mask_all; ctx->tree_parent_all = parent_all; ctx->tree_score_all = score_all;
        ctx->topk_id_all = topk_id_all; ctx->topk_logp_all = topk_logp_all;
        ctx->argmax_dev = argmax_dev;
        ctx->inv_freq = inv_freq; ctx->u_dev = u_dev;
        ctx->ud_dev = ud_dev; ctx->ua_dev = ua_dev; ctx->dlogits = dlogits; ctx->resid = resid;
    }
    return a.off + 256;
}

// ------------------------------------------------------------------------------------------ GEMM wrapper
GemmShape run_gemm(poss_ctx *c, const void *Wp, int N, int K, const void *X, int ldx, int M, float *part,
                   bool single_split, EpiArgs epi, const RopeRanges *ranges = nullptr) {
    GemmShape g = gemm_plan(c->md.dt, M, N, K, single_split ? 1 : c->gemm_target_wgs);
    const bool prof = c->prof_on && c->prof_n < PROFILE_EVENTS;
    if (!launch_gemm(c->md.dt, g, Wp, X, ldx, part, epi, c->md.eps, c->st, prof ? c->prof_ev[2 * c->prof_n] : nullptr,
                     prof ? c->prof_ev[2 * c->prof_n + 1] : nullptr, ranges))
        c->launch_refused = true;                   // reported by the next call that waits for the stream
    if (prof) {
        ++c->prof_n;
        c->prof_bytes += (double)N * K * dtype_size(c->md.dt);
    }
    return g;
}

// h (+)= GEMM (+ bias), then u = T(rmsnorm(h) * gain) for the next GEMM
EpiArgs epi_residual(poss_ctx *c, bool residual, const void *bias, float *h_copy, const void *gain) {
    EpiArgs e{};
    e.mode = EPI_RESIDUAL; e.h = c->h; e.bias = bias; e.residual = residual ? 1 : 0; e.h_copy = h_copy;
    e.gain = gain; e.u = c->u;
    return e;
}

// The rows of one sequence inside a pass: full rows [q0, q0 + nq) (query, attention, MLP) and
// key/value-only rows [x0, x0 + nx); its cache, committed prefix and region length.
struct Seg { int b; const KVCache *kv; int q0, nq, x0, nx, n_prefix, region_len; };

// One decoder layer on rows_all rows (all produce K/V) of which the first rows_q go through
// attention and the MLP; the full rows of every sequence come first, each sequence attends to its
// own cache.  On entry c->u holds T(rmsnorm(h) * attn_norm) and c->cs the rotary table of the rows;
// on exit c->h is updated and c->u holds T(rmsnorm(h) * next_gain).
void run_layer(poss_ctx *c, const LayerW &w, const std::vector<Seg> &segs, int rows_all, int rows_q, const RowMeta &rm,
               const void *next_gain, float *h_copy, bool drafter = false) {
    const ModelDims &md = c->md;
    const int qd = md.hq * md.dh, kd = md.hkv * md.dh;
    EpiArgs e{};
    e.mode = EPI_ROPE_KV; e.rows_q = rows_q; e.cs = c->cs; e.slot = rm.slot; e.q = c->q; e.kv = *segs[0].kv;
    e.hq = md.hq; e.hkv = md.hkv; e.dh = md.dh;
    const bool one = segs.size() == 1 && segs[0].q0 == 0 && segs[0].x0 == segs[0].nq;
    if (one) {
        run_gemm(c, w.wqkv, qd + 2 * kd, md.d, c->u, md.d, rows_all, c->part, false, e);
    } else {
        // one weight stream for every sequence, each sequence's rows into its own cache
        RopeRanges rr;
        rr.n = 0;
        for (const Seg &sg : segs) {
            if (sg.nq > 0) { rr.r0[rr.n] = sg.q0; rr.r1[rr.n] = sg.q0 + sg.nq; rr.rows_q[rr.n] = sg.q0 + sg.nq; rr.kv[rr.n] = *sg.kv; ++rr.n; }
            if (sg.nx > 0) { rr.r0[rr.n] = sg.x0; rr.r1[rr.n] = sg.x0 + sg.nx; rr.rows_q[rr.n] = 0; rr.kv[rr.n] = *sg.kv; ++rr.n; }
        }
        run_gemm(c, w.wqkv, qd + 2 * kd, md.d, c->u, md.d, rows_all, c->part, false, e, &rr);
    }
    if (rows_q == 0) return;
    {
        AttnSeg as[8];
        int na = 0;
        for (const Seg &sg : segs)
            if (sg.nq > 0) as[na++] = AttnSeg{sg.q0, sg.nq, sg.n_prefix, sg.region_len, sg.kv};
        // a specialist's pass: splits of at most 512 keys (few rows, its own cache); a tuning override applies to both
        const int kps = c->attn_keys_per_split ? c->attn_keys_per_split : (drafter ? -512 : 0);
        launch_attention_batch(md, c->q, rm, as, na, kps, c->attn_sc, c->attn_out, c->st);
    }
    run_gemm(c, w.wo, md.d, qd, c->attn_out, qd, rows_q, c->part, false, epi_residual(c, true, nullptr, nullptr, w.mlp_norm));
    EpiArgs es{};
    es.mode = EPI_SILU; es.act = c->act; es.F = md.ffn;
    // K unsplit: the stream kernel then applies SiLU * up itself (one tile per workgroup already fills most CUs)
    run_gemm(c, w.wgu, gate_up_rows(md.ffn), md.d, c->u, md.d, rows_q, c->part, true, es);
    run_gemm(c, w.wdown, md.d, md.ffn, c->act, md.ffn, rows_q, c->part, false, epi_residual(c, true, nullptr, h_copy, next_gain));
}

// Target pass over `rows` rows (all of them full rows; segs says which belong to which sequence)
// whose tokens / metadata are on the device.  Leaves features in c->feats and
// T(rmsnorm_final(features)) in c->u.
void target_forward(poss_ctx *c, int rows, const int32_t *tokens_dev, const RowMeta &rm, std::vector<Seg> segs, float *feats_out) {
    const ModelDims &md = c->md;
    launch_embed_norm(md, c->embed, tokens_dev, rows, c->layers[0].attn_norm, c->h, c->u, rm.pos, c->inv_freq, c->cs, c->st);
    const int nl = c->cfg.n_layers;
    for (int l = 0; l < nl; ++l) {
        if (c->taps_user)
            launch_copy_rows_f32(c->h, md.d, c->taps_user + (size_t)l * rows * md.d, md.d, rows, md.d, c->st);
        const void *next_gain = l + 1 < nl ? c->layers[l + 1].attn_norm : c->final_norm;
        for (Seg &sg : segs) sg.kv = &c->seq[sg.b].target_kv[l];
        run_layer(c, c->layers[l], segs, rows, rows, rm, next_gain, l + 1 == nl ? feats_out : nullptr);
    }
    if (c->taps_user)
        launch_copy_rows_f32(c->h, md.d, c->taps_user + (size_t)nl * rows * md.d, md.d, rows, md.d, c->st);
}

// Head(features) for the rows whose final-normed activations start at x (default: c->u).  head_mode 0: the logits,
// c->logits[rows][Npad].  HEAD_ARGMAX / HEAD_TOPK (16-bit storage): the GEMM reduces its own column tiles into
// c->topk_scratch - per row and tile the best (value, index), or the record of the k best with the tile's maximum and
// sum of exponentials - and writes the logits only if asked; *n_seg_out receives the number of tiles.  Float32
// storage has no such epilogue: it always writes logits and reports 0 tiles.
GemmShape run_head(poss_ctx *c, int rows, int head_mode, bool write_logits, int *n_seg_out, const void *x = nullptr,
                   float *logits_dst = nullptr) {
    EpiArgs e{};
    e.mode = EPI_PLAIN;
    if (n_seg_out) *n_seg_out = 0;
    if (head_mode && c->md.dt != DT_F32) {
        const GemmShape g0 = gemm_plan(c->md.dt, rows, c->md.vocab, c->md.d, 1);
        const int n_seg = gemm_head_segments(g0);
        e.mode = EPI_HEAD; e.head_mode = head_mode; e.head_k = c->cfg.top_k; e.write_logits = write_logits ? 1 : 0;
        e.seg_out = c->topk_scratch;
        e.pv = c->topk_scratch; e.pi = reinterpret_cast<int *>(c->topk_scratch + (size_t)rows * n_seg);
        if (n_seg_out) *n_seg_out = n_seg;
    }
    return run_gemm(c, c->lm_head, c->md.vocab, c->md.d, x ? x : c->u, c->md.d, rows, logits_dst ? logits_dst : c->logits, true, e);
}

// The drafter's k best next tokens and their log-probabilities for `rows` rows of final-normed activations in c->u.
void run_head_topk(poss_ctx *c, int rows, int depth) {
    if (c->draft_sampling) {
        // drawn children: the logits of the pass's rows are kept (the walk needs the distribution each child came from),
        // k children per row drawn without replacement with the caller's numbers
        const int k = c->cfg.top_k;
        float *dst = c->dlogits + (size_t)(depth == 1 ? 0 : 1 + (depth - 2) * k) * gemm_npad(c->cfg.vocab);
        const GemmShape g = run_head(c, rows, 0, true, nullptr, nullptr, dst);
        launch_sample_children(dst, g.Npad, rows, c->cfg.vocab, k, c->temperature, c->ud_dev + (size_t)(depth - 1) * k * k,
                               c->topk_id_all, c->topk_logp_all, c->st);
        return;
    }
    int n_seg = 0;
    const GemmShape g = run_head(c, rows, HEAD_TOPK, false, &n_seg);
    if (n_seg)
        launch_topk_merge(c->topk_scratch, n_seg, rows, c->cfg.top_k, c->topk_id_all, c->topk_logp_all, c->st);
    else
        launch_topk_logsoftmax(c->logits, g.Npad, rows, c->cfg.vocab, c->cfg.top_k, c->topk_scratch, c->topk_id_all, c->topk_logp_all, c->st);
}

__global__ void causal_meta_kernel(int n, int c0, int32_t *pos, int32_t *slot, uint64_t *mask) {
    const int i = threadIdx.x;
    if (i >= n) return;
    pos[i] = c0 + i; slot[i] = c0 + i;
    const int bits = i % MAX_ROWS + 1;                     // within the row's range of MAX_ROWS rows
    mask[i * MASK_WORDS] = bits >= 64 ? ~0ull : ((1ull << bits) - 1);
    mask[i * MASK_WORDS + 1] = bits <= 64 ? 0ull : (bits >= 128 ? ~0ull : ((1ull << (bits - 64)) - 1));
}

template <typename T>
__global__ void stash_rows_kernel(const float *__restrict__ feats, int d, T *__restrict__ stash, int row0) {
    const int r = blockIdx.x;
    for (int i = threadIdx.x; i < d; i += blockDim.x) stash[(size_t)(row0 + r) * d + i] = (T)feats[(size_t)r * d + i];
}

void stash_rows(poss_ctx *c, Seq &sq, int rows, int row0) {
    if (c->md.dt == DT_F32)
        hipLaunchKernelGGL((stash_rows_kernel<float>), dim3(rows), dim3(256), 0, c->st, c->feats, c->md.d, (float *)sq.feat_stash, row0);
    else if (c->md.dt == DT_BF16)
        hipLaunchKernelGGL((stash_rows_kernel<bf16_t>), dim3(rows), dim3(256), 0, c->st, c->feats, c->md.d, (bf16_t *)sq.feat_stash, row0);
    else
        hipLaunchKernelGGL((stash_rows_kernel<f16_t>), dim3(rows), dim3(256), 0, c->st, c->feats, c->md.d, (f16_t *)sq.feat_stash, row0);
}

uint64_t ones(int bits) { return bits <= 0 ? 0ull : bits >= 64 ? ~0ull : ((1ull << bits) - 1); }

// Rows of sequence b in one specialist pass: plan rows [0, nq) are its full rows, the rest produce
// keys and values only.
struct SeqPlan { int b; DraftRowPlan plan; int nq, n_prefix, region_len; };

// One pass of specialist s over the rows of every plan.  Full rows of all sequences first (sequence
// order), then the key/value-only rows: the GEMMs after attention run on the leading rows.
// fhat_prev / fhat_out hold one row per full row of the previous / this pass.
// Returns the first full row of each sequence through q0_out.
void spec_pass(poss_ctx *c, int s, std::vector<SeqPlan> &plans, int depth_index, const float *fhat_prev, int prev_rows_each,
               float *fhat_out, std::vector<int> *q0_out) {
    const ModelDims &md = c->md;
    const SpecW &w = c->specs[s];
    int rows_q = 0, rows_all = 0;
    for (const SeqPlan &p : plans) { rows_q += p.nq; rows_all += p.plan.n_rows; }
    std::vector<Seg> segs;
    int q0 = 0, x0 = rows_q;
    for (size_t i = 0; i < plans.size(); ++i) {
        SeqPlan &p = plans[i];
        Seq &sq = c->seq[p.b];
        const int nx = p.plan.n_rows - p.nq;
        for (int r = 0; r < p.nq; ++r) p.plan.dst[r] = (int16_t)(q0 + r);
        for (int r = 0; r < nx; ++r) p.plan.dst[p.nq + r] = (int16_t)(x0 + r);
        launch_draft_assemble(md, p.plan, depth_index, c->cfg.top_k, c->embed, sq.tokens_dev, sq.feat_stash, sq.td,
                              fhat_prev ? fhat_prev + (size_t)i * prev_rows_each * md.d : nullptr, sq.xin_tmp, c->xin,
                              c->row_pos, c->row_slot, c->row_mask, c->inv_freq, c->cs, c->st);
        segs.push_back(Seg{p.b, &sq.spec_kv[s], q0, p.nq, x0, nx, p.n_prefix, p.region_len});
        if (q0_out) q0_out->push_back(q0);
        q0 += p.nq; x0 += nx;
    }
    run_gemm(c, w.fc_w, md.d, 2 * md.d, c->xin, 2 * md.d, rows_all, c->part, false,
             epi_residual(c, false, c->cfg.fc_bias ? w.fc_b : nullptr, nullptr, w.layer.attn_norm));
    RowMeta rm{c->row_pos, c->row_slot, c->row_mask};
    run_layer(c, w.layer, segs, rows_all, rows_q, rm, c->final_norm, fhat_out, true);
}

// Keys/values of committed pairs [spec_len[s], upto) of one sequence for specialist s, in chunks of MAX_ROWS rows.
void spec_catchup(poss_ctx *c, int b, int s, int upto) {
    Seq &sq = c->seq[b];
    while (sq.spec_len[s] < upto) {
        const int i0 = sq.spec_len[s], n = upto - i0 < MAX_ROWS ? upto - i0 : MAX_ROWS;
        std::vector<SeqPlan> plans(1);
        SeqPlan &p = plans[0];
        p.b = b; p.nq = 0; p.n_prefix = 0; p.region_len = 0;
        p.plan.n_rows = n; p.plan.mask0[0] = p.plan.mask0[1] = 0;
        for (int r = 0; r < n; ++r) { p.plan.kind[r] = 0; p.plan.idx[r] = i0 + r; p.plan.slot[r] = i0 + r; p.plan.pos[r] = i0 + r; }
        spec_pass(c, s, plans, 0, nullptr, 0, nullptr, nullptr);
        sq.spec_len[s] = i0 + n;
    }
}

int copy_tree_out(poss_ctx *c, Seq &sq, poss_tree *out) {
    const int n = sq.tree_n;
    out->n_nodes = n;
    struct { void *dst; const void *src; size_t b; } cp[] = {
        {out->token, sq.td.token, n * sizeof(int32_t)}, {out->parent, sq.td.parent, n * sizeof(int32_t)},
        {out->depth, sq.td.depth, n * sizeof(int32_t)}, {out->pos, sq.td.pos, n * sizeof(int32_t)},
        {out->mask, sq.td.mask, (size_t)n * MASK_WORDS * sizeof(uint64_t)}, {out->score, sq.td.score, n * sizeof(float)}};
    for (auto &x : cp)
        if (x.dst) HIP_TRY(c, hipMemcpyAsync(x.dst, x.src, x.b, hipMemcpyDeviceToHost, c->st));
    HIP_TRY(c, hipStreamSynchronize(c->st));
    return POSS_OK;
}

void pack_layer(poss_ctx *c, const void *const *src, const std::vector<void *> &dst, size_t base) {
    const poss_config &cf = c->cfg;
    const int dt = cf.dtype, d = cf.d_model, qd = cf.n_q_heads * cf.head_dim, kd = cf.n_kv_heads * cf.head_dim, F = cf.d_ffn;
    const size_t es = esize(cf);
    (void)hipMemcpyAsync(dst[base + 0], src[0], d * es, hipMemcpyDeviceToDevice, c->st);
    launch_pack(dt, PackSrc{{src[1], src[2], src[3]}, {qd, kd, kd}, 0, dt == DT_F32 ? 0 : cf.head_dim}, d, dst[base + 1], c->st);
    launch_pack(dt, PackSrc{{src[4], nullptr, nullptr}, {d, 0, 0}}, qd, dst[base + 2], c->st);
    (void)hipMemcpyAsync(dst[base + 3], src[5], d * es, hipMemcpyDeviceToDevice, c->st);
    launch_pack(dt, PackSrc{{src[6], src[7], nullptr}, {F, F, 0}, 1}, d, dst[base + 4], c->st);
    launch_pack(dt, PackSrc{{src[8], nullptr, nullptr}, {d, 0, 0}}, F, dst[base + 5], c->st);
}

LayerW layer_view(const std::vector<void *> &v, size_t base) {
    return LayerW{v[base], v[base + 1], v[base + 2], v[base + 3], v[base + 4], v[base + 5]};
}

// The final-tree arrays of a sequence are a slice of the batch-wide row arrays: drafted trees sit at a fixed
// stride (total_tokens + 1), caller-supplied ones back to back.
void point_tree(poss_ctx *c, Seq &sq, int row0) {
    sq.tree_row0 = row0;
    sq.td.token = c->tree_token_all + row0; sq.td.parent = c->tree_parent_all + row0;
    sq.td.depth = c->tree_depth_all + row0; sq.td.pos = c->tree_pos_all + row0;
    sq.td.mask = c->tree_mask_all + (size_t)row0 * MASK_WORDS; sq.td.score = c->tree_score_all + row0;
    sq.tree_slot = c->tree_slot_all + row0;
}

void reset_sequence(poss_ctx *c) {
    c->state = ST_LOADED;
    for (Seq &sq : c->seq) {
        sq.t = 0; sq.tree_ready = 0; sq.tree_n = 0; sq.prefilled = 0; sq.last_m = 0; sq.active = 1;
        point_tree(c, sq, (int)(&sq - &c->seq[0]) * (c->cfg.total_tokens + 1));
        sq.tokens.clear();
        sq.spec_len.assign(c->cfg.n_specialists, 0);
        sq.spec_tmp_depth.assign(c->cfg.n_specialists, 0);
    }
    memset(&c->stats, 0, sizeof(c->stats));
}

// The sequences that take part in the rounds, in order; a pass stacks their rows in this order.
std::vector<int> active_seqs(const poss_ctx *c) {
    std::vector<int> a;
    for (int b = 0; b < c->B; ++b)
        if (c->seq[b].active) a.push_back(b);
    return a;
}

// Rounds can run when every active sequence has its prompt.
void update_ready(poss_ctx *c) {
    bool all = true;
    for (const Seq &o : c->seq) all = all && (o.prefilled || !o.active);
    if (c->state == ST_LOADED && all) c->state = ST_READY;
    if (c->state == ST_READY && !all) c->state = ST_LOADED;
}

// Events and pinned host memory of a context (whatever of them exists: a failed poss_load stops half way).
void release_host(poss_ctx *c) {
    for (int i = 0; i < 6; ++i)
        if (c->ev[i]) (void)hipEventDestroy(c->ev[i]);
    for (int i = 0; i < 2 * PROFILE_EVENTS; ++i)
        if (c->prof_ev[i]) (void)hipEventDestroy(c->prof_ev[i]);
    if (c->pinned) (void)hipHostFree(c->pinned);
    if (c->u_pinned) (void)hipHostFree(c->u_pinned);
    if (c->ud_pinned) (void)hipHostFree(c->ud_pinned);
    if (c->ua_pinned) (void)hipHostFree(c->ua_pinned);
    if (c->result_pinned_all) (void)hipHostFree(c->result_pinned_all);
}

}  // namespace

// ============================================================================================ C ABI
extern "C" {

size_t poss_workspace_bytes(const poss_config *cfg) {
    if (!cfg || check_config(*cfg)) return 0;
    Arena a(nullptr);
    return carve(*cfg, a, nullptr, nullptr);
}

int poss_load(const poss_config *cfg, const poss_weights *w, void *workspace, size_t workspace_bytes,
              void *hip_stream, poss_ctx **out) {
    if (!cfg || !w || !workspace || !out) return fail(nullptr, POSS_E_INVALID_ARG, "poss_load: null argument");
    if (const char *why = check_config(*cfg)) return fail(nullptr, POSS_E_INVALID_ARG, "poss_load: %s", why);
    if (!w->embed || !w->lm_head || !w->final_norm || !w->layer || !w->spec)
        return fail(nullptr, POSS_E_INVALID_ARG, "poss_load: null weight pointer");
    for (int i = 0; i < cfg->n_layers * 9; ++i)
        if (!w->layer[i]) return fail(nullptr, POSS_E_INVALID_ARG, "poss_load: null layer tensor %d", i);
    for (int i = 0; i < cfg->n_specialists * 11; ++i)
        if (!w->spec[i]) return fail(nullptr, POSS_E_INVALID_ARG, "poss_load: null specialist tensor %d", i);
    if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(nullptr, POSS_E_INVALID_ARG, "poss_load: workspace not 256-byte aligned");
    const size_t need = poss_workspace_bytes(cfg);
    if (workspace_bytes < need)
        return fail(nullptr, POSS_E_CAPACITY, "poss_load: workspace of %zu bytes, %zu needed", workspace_bytes, need);

    poss_ctx *c = new (std::nothrow) poss_ctx();
    if (!c) return fail(nullptr, POSS_E_INVALID_ARG, "poss_load: out of host memory");
    c->cfg = *cfg;
    c->md = ModelDims{cfg->d_model, cfg->n_q_heads, cfg->n_kv_heads, cfg->head_dim, cfg->d_ffn, cfg->vocab,
                      cfg->rms_eps, cfg->rope_theta, cfg->dtype};
    c->st = static_cast<hipStream_t>(hip_stream);
    c->err[0] = 0;
    c->taps_user = nullptr;
    c->gemm_target_wgs = 0; c->attn_keys_per_split = 0; c->launch_rows = LAUNCH_ROWS;
    c->prof_on = 0; c->prof_n = 0; c->prof_bytes = 0;
    Arena a(workspace);
    WeightSlots ws;
    carve(*cfg, a, c, &ws);

    auto bail = [&](int code) { g_load_error[0] = 0; strncpy(g_load_error, c->err, 511); release_host(c); delete c; return code; };
#define LOAD_TRY(call)                                                                    \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess) { fail(c, POSS_E_HIP, "%s: %s", #call, hipGetErrorString(e_)); return bail(POSS_E_HIP); } \
    } while (0)

    const size_t es = esize(*cfg);
    const int d = cfg->d_model, V = cfg->vocab;
    // weights
    LOAD_TRY(hipMemcpyAsync(ws.embed, w->embed, (size_t)V * d * es, hipMemcpyDeviceToDevice, c->st));
    launch_pack(cfg->dtype, PackSrc{{w->lm_head, nullptr, nullptr}, {V, 0, 0}}, d, ws.lm_head, c->st);
    LOAD_TRY(hipMemcpyAsync(ws.final_norm, w->final_norm, d * es, hipMemcpyDeviceToDevice, c->st));
    c->embed = ws.embed; c->lm_head = ws.lm_head; c->final_norm = ws.final_norm;
    for (int l = 0; l < cfg->n_layers; ++l) {
        pack_layer(c, w->layer + (size_t)l * 9, ws.layer, (size_t)l * 6);
        c->layers.push_back(layer_view(ws.layer, (size_t)l * 6));
    }
    for (int s = 0; s < cfg->n_specialists; ++s) {
        const void *const *src = w->spec + (size_t)s * 11;
        launch_pack(cfg->dtype, PackSrc{{src[0], nullptr, nullptr}, {d, 0, 0}}, 2 * d, ws.spec[(size_t)s * 8], c->st);
        LOAD_TRY(hipMemcpyAsync(ws.spec[(size_t)s * 8 + 1], src[1], d * es, hipMemcpyDeviceToDevice, c->st));
        pack_layer(c, src + 2, ws.spec, (size_t)s * 8 + 2);
        c->specs.push_back(SpecW{ws.spec[(size_t)s * 8], ws.spec[(size_t)s * 8 + 1], layer_view(ws.spec, (size_t)s * 8 + 2)});
    }
    // caches: zero (attention may touch, masked, slots that were never written)
    for (Seq &sq : c->seq) {
        for (auto &kv : sq.target_kv) { launch_fill_u32((uint32_t *)kv.k, c->cache_bytes_each / 4, 0, c->st); launch_fill_u32((uint32_t *)kv.vt, c->cache_bytes_each / 4, 0, c->st); }
        for (auto &kv : sq.spec_kv) { launch_fill_u32((uint32_t *)kv.k, c->cache_bytes_each / 4, 0, c->st); launch_fill_u32((uint32_t *)kv.vt, c->cache_bytes_each / 4, 0, c->st); }
    }
    // small host->device tables
    c->pinned_bytes = 1 << 20;
    LOAD_TRY(hipHostMalloc(&c->pinned, c->pinned_bytes, hipHostMallocDefault));
    LOAD_TRY(hipHostMalloc(reinterpret_cast<void **>(&c->u_pinned), (size_t)c->B * (POSS_MAX_DEPTH + 1) * sizeof(float), hipHostMallocDefault));
    for (int i = 0; i < c->B * (POSS_MAX_DEPTH + 1); ++i) c->u_pinned[i] = 0.f;
    LOAD_TRY(hipHostMalloc(reinterpret_cast<void **>(&c->ud_pinned), (size_t)cfg->depth * cfg->top_k * cfg->top_k * sizeof(float), hipHostMallocDefault));
    LOAD_TRY(hipHostMalloc(reinterpret_cast<void **>(&c->ua_pinned), (size_t)(cfg->depth + 1) * (cfg->top_k + 1) * sizeof(float), hipHostMallocDefault));
    c->draft_sampling = 0;
    LOAD_TRY(hipHostMalloc(reinterpret_cast<void **>(&c->result_pinned_all), (size_t)c->B * 64 * sizeof(int32_t), hipHostMallocDefault));
    {
        int32_t *dev = nullptr;
        LOAD_TRY(hipHostGetDevicePointer(reinterpret_cast<void **>(&dev), c->result_pinned_all, 0));
        for (int b = 0; b < c->B; ++b) { c->seq[b].result_pinned = c->result_pinned_all + b * 64; c->seq[b].result_dev = dev + b * 64; }
    }
    c->temperature = 0.f;
    {
        char *p = static_cast<char *>(c->pinned);
        int32_t *pt = reinterpret_cast<int32_t *>(p);
        for (int i = 0; i < c->n_pages; ++i) pt[i] = cfg->kv_page_order == 1 ? c->n_pages - 1 - i : i;
        LOAD_TRY(hipMemcpyAsync(c->page_table, pt, c->n_pages * sizeof(int32_t), hipMemcpyHostToDevice, c->st));
        p += round_up(c->n_pages * (int)sizeof(int32_t), 256);
        double *fr = reinterpret_cast<double *>(p);
        const int half = cfg->head_dim / 2;
        for (int i = 0; i < half; ++i) fr[i] = pow((double)cfg->rope_theta, -2.0 * i / cfg->head_dim);
        LOAD_TRY(hipMemcpyAsync(c->inv_freq, fr, half * sizeof(double), hipMemcpyHostToDevice, c->st));
        p += round_up(half * (int)sizeof(double), 256);
        KVCache *kvh = reinterpret_cast<KVCache *>(p);
        for (int b = 0; b < c->B; ++b)
            for (int l = 0; l < cfg->n_layers; ++l) kvh[b * cfg->n_layers + l] = c->seq[b].target_kv[l];
        LOAD_TRY(hipMemcpyAsync(c->seq[0].target_kv_dev, kvh, (size_t)c->B * cfg->n_layers * sizeof(KVCache), hipMemcpyHostToDevice, c->st));
    }
    for (int i = 0; i < 6; ++i) LOAD_TRY(hipEventCreate(&c->ev[i]));
    c->ev_pending[0] = c->ev_pending[1] = c->ev_pending[2] = false;
    c->launch_refused = false;
    for (int i = 0; i < 2 * PROFILE_EVENTS; ++i) LOAD_TRY(hipEventCreate(&c->prof_ev[i]));
    LOAD_TRY(hipStreamSynchronize(c->st));
    LOAD_TRY(hipGetLastError());
#undef LOAD_TRY
    reset_sequence(c);
    *out = c;
    return POSS_OK;
}

int poss_reset(poss_ctx *c) {
    if (!c) return POSS_E_INVALID_ARG;
    (void)hipStreamSynchronize(c->st);
    c->ev_pending[0] = c->ev_pending[1] = c->ev_pending[2] = false;
    c->launch_refused = false;
    reset_sequence(c);
    return POSS_OK;
}

static int sync_and_harvest(poss_ctx *c);

int poss_reset_seq(poss_ctx *c, int32_t seq) {
    if (!c) return POSS_E_INVALID_ARG;
    if (seq < 0 || seq >= c->B) return fail(c, POSS_E_INVALID_ARG, "poss_reset_seq: no sequence %d (batch %d)", seq, c->B);
    if (c->state == ST_VERIFIED) return fail(c, POSS_E_BAD_STATE, "poss_reset_seq: a verified round is waiting for poss_accept_and_commit");
    { int rc = sync_and_harvest(c); if (rc) return rc; }
    Seq &sq = c->seq[seq];
    sq.t = 0; sq.tree_ready = 0; sq.tree_n = 0; sq.prefilled = 0; sq.last_m = 0;
    sq.tokens.clear();
    sq.spec_len.assign(c->cfg.n_specialists, 0);
    sq.spec_tmp_depth.assign(c->cfg.n_specialists, 0);
    sq.active = 1;
    for (Seq &o : c->seq) o.tree_ready = 0;               // trees drafted for the old line-up are void
    c->state = ST_LOADED;                                  // rounds resume once the sequence has a prompt again
    update_ready(c);
    return POSS_OK;
}

int poss_set_active(poss_ctx *c, int32_t seq, int32_t active) {
    if (!c) return POSS_E_INVALID_ARG;
    if (seq < 0 || seq >= c->B) return fail(c, POSS_E_INVALID_ARG, "poss_set_active: no sequence %d (batch %d)", seq, c->B);
    if (c->state == ST_VERIFIED) return fail(c, POSS_E_BAD_STATE, "poss_set_active: a verified round is waiting for poss_accept_and_commit");
    Seq &sq = c->seq[seq];
    if (!active) {
        int others = 0;
        for (const Seq &o : c->seq) others += (&o != &sq && o.active);
        if (!others) return fail(c, POSS_E_INVALID_ARG, "poss_set_active: the last active sequence cannot be set aside");
    }
    sq.active = active ? 1 : 0;
    for (Seq &o : c->seq) o.tree_ready = 0;               // the rows of a round are laid out per line-up
    update_ready(c);
    return POSS_OK;
}

void poss_free(poss_ctx *c) {
    if (!c) return;
    (void)hipStreamSynchronize(c->st);
    release_host(c);
    delete c;
}

const char *poss_last_error(poss_ctx *c) { return c ? c->err : g_load_error; }

static int head_and_choose(poss_ctx *c, const void *x, int rows, bool want_logits, const int32_t *depth, const int *seq_ids,
                           int n_seq, const int *row0, const int *n_rows, int base, int *ld_out, bool drafted_tree = false);

int poss_prefill_seq(poss_ctx *c, int32_t seq, const int32_t *prompt, int32_t n_prompt, int32_t *first_token_out) {
    if (!c) return POSS_E_INVALID_ARG;
    if (seq < 0 || seq >= c->B) return fail(c, POSS_E_INVALID_ARG, "poss_prefill: no sequence %d (batch %d)", seq, c->B);
    if (!prompt || n_prompt < 1) return fail(c, POSS_E_INVALID_ARG, "poss_prefill: empty prompt");
    Seq &sq = c->seq[seq];
    if (c->state != ST_LOADED || sq.prefilled) return fail(c, POSS_E_BAD_STATE, "poss_prefill: sequence already started (poss_reset first)");
    if (n_prompt + 1 > c->cfg.max_seq) return fail(c, POSS_E_CAPACITY, "poss_prefill: prompt of %d tokens, max_seq %d", n_prompt, c->cfg.max_seq);
    for (int i = 0; i < n_prompt; ++i)
        if (prompt[i] < 0 || prompt[i] >= c->cfg.vocab) return fail(c, POSS_E_INVALID_ARG, "poss_prefill: token id %d out of range at %d", prompt[i], i);
    const ModelDims &md = c->md;
    int32_t *stage = static_cast<int32_t *>(c->pinned);
    // A launch carries LAUNCH_ROWS prompt tokens as two row ranges of at most MAX_ROWS (the width of a row's mask): the
    // second range finds the keys of the first, written by the same layer's QKV epilogue, in its committed prefix.
    for (int c0 = 0; c0 < n_prompt; c0 += LAUNCH_ROWS) {
        const int rows = n_prompt - c0 < LAUNCH_ROWS ? n_prompt - c0 : LAUNCH_ROWS;
        memcpy(stage, prompt + c0, rows * sizeof(int32_t));
        HIP_TRY(c, hipMemcpyAsync(sq.tokens_dev + c0, stage, rows * sizeof(int32_t), hipMemcpyHostToDevice, c->st));
        hipLaunchKernelGGL(causal_meta_kernel, dim3(1), dim3(LAUNCH_ROWS), 0, c->st, rows, c0, c->row_pos, c->row_slot, c->row_mask);
        RowMeta rm{c->row_pos, c->row_slot, c->row_mask};
        std::vector<Seg> segs;
        const int ra = rows < MAX_ROWS ? rows : MAX_ROWS;
        segs.push_back(Seg{seq, nullptr, 0, ra, rows, 0, c0, ra});
        if (rows > ra) segs.push_back(Seg{seq, nullptr, ra, rows - ra, rows, 0, c0 + ra, rows - ra});
        target_forward(c, rows, sq.tokens_dev + c0, rm, segs, c->feats);
        stash_rows(c, sq, rows, c0);
        if (c0 + rows == n_prompt) {
            // Head on the last row only: its normed activations sit at row rows-1 of c->u
            const char *last = static_cast<const char *>(c->u) + (size_t)(rows - 1) * md.d * dtype_size(md.dt);
            { const int zero = 0, one = 1, id = seq; int rc = head_and_choose(c, last, 1, false, nullptr, &id, 1, &zero, &one, 0, nullptr); if (rc) return rc; }
            HIP_TRY(c, hipMemcpyAsync(sq.tokens_dev + n_prompt, c->argmax_dev, sizeof(int32_t), hipMemcpyDeviceToDevice, c->st));
        }
        HIP_TRY(c, hipStreamSynchronize(c->st));          // the staging buffer is reused by the next chunk
    }
    int32_t first = 0;
    HIP_TRY(c, hipMemcpy(&first, c->argmax_dev, sizeof(int32_t), hipMemcpyDeviceToHost));
    sq.tokens.assign(prompt, prompt + n_prompt);
    sq.tokens.push_back(first);
    sq.t = n_prompt;
    for (int s = 0; s < c->cfg.n_specialists; ++s) spec_catchup(c, seq, s, sq.t - 1);
    HIP_TRY(c, hipStreamSynchronize(c->st));
    HIP_TRY(c, hipGetLastError());
    sq.prefilled = 1; sq.tree_ready = 0;
    sq.active = 1;
    update_ready(c);                                       // rounds start once every active sequence has its prompt
    if (first_token_out) *first_token_out = first;
    return POSS_OK;
}

int poss_prefill(poss_ctx *c, const int32_t *prompt, int32_t n_prompt, int32_t *first_token_out) {
    return poss_prefill_seq(c, 0, prompt, n_prompt, first_token_out);
}

// Head over `rows` rows of final-normed activations at x (nullptr: c->u), then the token the target chooses after
// each: the argmax - reduced per column tile inside the Head GEMM, the logits written only if want_logits - or at
// temperature > 0 a draw by inverse CDF with the uniform number of the row's depth (depth == nullptr: all rows use u[0]).
// Sequence seq_ids[i] owns rows [row0[i], row0[i] + n_rows[i]) and has its own numbers; the rows' depths and results
// sit `base` rows further on in the batch-wide arrays (the rows of earlier groups).  *ld_out: row stride of c->logits.
static int head_and_choose(poss_ctx *c, const void *x, int rows, bool want_logits, const int32_t *depth, const int *seq_ids,
                           int n_seq, const int *row0, const int *n_rows, int base, int *ld_out, bool drafted_tree) {
    if (c->temperature > 0.f && c->draft_sampling && drafted_tree) {
        // drawn children: the rejection walk over the target's and the drafter's logits writes the path as the g[] of a
        // greedy walk (g[node] = next token on the path), which is what the commit kernel follows
        const GemmShape g = run_head(c, rows, 0, true, nullptr, x);
        if (ld_out) *ld_out = g.Npad;
        const poss_config &cf = c->cfg;
        HIP_TRY(c, hipMemcpyAsync(c->ua_dev, c->ua_pinned, (size_t)(cf.depth + 1) * (cf.top_k + 1) * sizeof(float), hipMemcpyHostToDevice, c->st));
        launch_rejection_walk(c->seq[seq_ids[0]].td, cf.top_k, cf.depth, cf.vocab, c->logits, c->dlogits, g.Npad, c->temperature,
                              c->ua_dev, c->resid, c->argmax_dev + base, c->st);
        return POSS_OK;
    }
    if (c->temperature > 0.f) {
        const GemmShape g = run_head(c, rows, 0, true, nullptr, x);
        if (ld_out) *ld_out = g.Npad;
        const int nu = POSS_MAX_DEPTH + 1, ld = g.Npad;
        HIP_TRY(c, hipMemcpyAsync(c->u_dev, c->u_pinned, (size_t)c->B * nu * sizeof(float), hipMemcpyHostToDevice, c->st));
        for (int i = 0; i < n_seq; ++i)
            if (!launch_sample(c->logits + (size_t)row0[i] * ld, ld, n_rows[i], c->cfg.vocab, c->temperature,
                               c->u_dev + (size_t)seq_ids[i] * nu, depth ? depth + base + row0[i] : nullptr, c->topk_scratch,
                               c->argmax_dev + base + row0[i], c->st))
                return fail(c, POSS_E_INVALID_ARG, "sampling: vocabulary too large for the sampler");
        return POSS_OK;
    }
    int n_seg = 0;
    const GemmShape g = run_head(c, rows, HEAD_ARGMAX, want_logits, &n_seg, x);
    if (ld_out) *ld_out = g.Npad;
    if (n_seg)
        launch_argmax_merge(c->topk_scratch, reinterpret_cast<const int *>(c->topk_scratch + (size_t)rows * n_seg), n_seg, rows,
                            c->argmax_dev + base, c->st);
    else
        launch_argmax(c->logits, g.Npad, rows, c->cfg.vocab, c->topk_scratch, c->argmax_dev + base, c->st);
    return POSS_OK;
}

// Wait for the stream; then add the elapsed time of every phase recorded since the last wait to the
// statistics (draft, verify, commit: event pairs 0/1, 2/3, 4/5).
static int sync_and_harvest(poss_ctx *c) {
    HIP_TRY(c, hipStreamSynchronize(c->st));
    HIP_TRY(c, hipGetLastError());
    if (c->launch_refused) return fail(c, POSS_E_HIP, "internal error: a GEMM launch was refused (null operand)");
    double *acc[3] = {&c->stats.ms_draft, &c->stats.ms_verify, &c->stats.ms_commit};
    for (int i = 0; i < 3; ++i) {
        if (!c->ev_pending[i]) continue;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, c->ev[2 * i], c->ev[2 * i + 1]) == hipSuccess) *acc[i] += ms;
        c->ev_pending[i] = false;
    }
    return POSS_OK;
}

int poss_draft_tree(poss_ctx *c, poss_tree *out) {
    if (!c) return POSS_E_INVALID_ARG;
    if (c->state != ST_READY) return fail(c, POSS_E_BAD_STATE, "poss_draft_tree: needs a prefilled context with no pending verification");
    const poss_config &cf = c->cfg;
    const int k = cf.top_k, L = cf.depth;
    const std::vector<int> all = active_seqs(c);
    for (int b : all) {
        const int t = c->seq[b].t;
        if (t + cf.total_tokens + 1 > c->cache_slots || t + L + 1 > cf.max_seq)
            return fail(c, POSS_E_CAPACITY, "poss_draft_tree: %d committed tokens leave no room (max_seq %d)", t, cf.max_seq);
    }
    // Rows of every pass, worked out before anything is launched or any state is touched (a pass that does not fit
    // must not leave a half-drafted round behind): specialist s catches up on the pairs and frontier rows it has not seen.
    for (int b : all) {
        const Seq &sq = c->seq[b];
        std::vector<int> len = sq.spec_len, tmp(cf.n_specialists, 0);
        for (int s = 0; s < cf.n_specialists; ++s)
            if (sq.t - 1 - len[s] > L) len[s] = sq.t - 1;             // brought up to date in chunks of their own first
        for (int d = 1; d <= L; ++d) {
            int s = (d - 1) / cf.positions_per_specialist;
            if (s > cf.n_specialists - 1) s = cf.n_specialists - 1;
            const int n = d == 1 ? sq.t - len[s] : k + (sq.t - len[s]) + k * (d - 2 - tmp[s] > 0 ? d - 2 - tmp[s] : 0);
            if (n > MAX_ROWS) return fail(c, POSS_E_CAPACITY, "poss_draft_tree: the pass at depth %d would carry %d rows for one sequence (limit %d)", d, n, MAX_ROWS);
            len[s] = sq.t; tmp[s] = d - 1;
        }
    }
    if (c->draft_sampling) {
        if (!(c->temperature > 0.f)) return fail(c, POSS_E_BAD_STATE, "poss_draft_tree: drawn children need a temperature (poss_set_sampling)");
        if ((int)all.size() != 1) return fail(c, POSS_E_BAD_STATE, "poss_draft_tree: drawn children are built for one sequence per round");
    }
    if (c->ev_pending[0]) { int rc = sync_and_harvest(c); if (rc) return rc; }   // a re-draft: keep the first one's time
    (void)hipEventRecord(c->ev[0], c->st);
    if (c->draft_sampling)
        HIP_TRY(c, hipMemcpyAsync(c->ud_dev, c->ud_pinned, (size_t)L * k * k * sizeof(float), hipMemcpyHostToDevice, c->st));
    for (int i = 0; i < (int)all.size(); ++i) {
        const int b = all[i];
        Seq &sq = c->seq[b];
        point_tree(c, sq, i * (cf.total_tokens + 1));
        for (int s = 0; s < cf.n_specialists; ++s) {
            sq.spec_tmp_depth[s] = 0;
            if (sq.t - 1 - sq.spec_len[s] > L) spec_catchup(c, b, s, sq.t - 1);      // only after caller-supplied trees
        }
    }
    const std::vector<int> &act = all;
    const int B = (int)act.size();                         // sequences in this round
    for (int d = 1; d <= L; ++d) {
        int s = (d - 1) / cf.positions_per_specialist;
        if (s > cf.n_specialists - 1) s = cf.n_specialists - 1;
        std::vector<SeqPlan> plans(B);
        const int rows_q_each = d == 1 ? 1 : k;
        for (int i = 0; i < B; ++i) {
            const int b = act[i];
            Seq &sq = c->seq[b];
            SeqPlan &sp = plans[i];
            DraftRowPlan &plan = sp.plan;
            const int t = sq.t;
            int n = 0;
            sp.b = b; sp.nq = rows_q_each;
            if (d == 1) {
                // root pair [x_t ; f_{t-1}] first (the only row whose output is used), then the other
                // pairs this specialist has not seen; all of them become committed cache entries
                sp.n_prefix = sq.spec_len[s]; sp.region_len = t - sp.n_prefix;
                plan.mask0[0] = ones(sp.region_len); plan.mask0[1] = ones(sp.region_len - 64);
                plan.kind[n] = 0; plan.idx[n] = t - 1; plan.slot[n] = t - 1; plan.pos[n] = t - 1; ++n;
                for (int j = sp.n_prefix; j < t - 1; ++j) { plan.kind[n] = 0; plan.idx[n] = j; plan.slot[n] = j; plan.pos[n] = j; ++n; }
            } else {
                sp.n_prefix = t; sp.region_len = (d - 1) * k;
                plan.mask0[0] = plan.mask0[1] = 0;
                for (int r = 0; r < k; ++r) { plan.kind[n] = 2; plan.idx[n] = r; plan.slot[n] = t + (d - 2) * k + r; plan.pos[n] = t - 1 + (d - 1); ++n; }
                for (int j = sq.spec_len[s]; j < t; ++j) { plan.kind[n] = 0; plan.idx[n] = j; plan.slot[n] = j; plan.pos[n] = j; ++n; }
                for (int dl = sq.spec_tmp_depth[s] + 1; dl <= d - 2; ++dl)
                    for (int r = 0; r < k; ++r) { plan.kind[n] = 1; plan.idx[n] = (dl - 1) * k + r; plan.slot[n] = t + (dl - 1) * k + r; plan.pos[n] = t - 1 + dl; ++n; }
            }
            plan.n_rows = n;
            if (n > MAX_ROWS) return fail(c, POSS_E_CAPACITY, "poss_draft_tree: a pass of %d rows for one sequence (limit %d)", n, MAX_ROWS);
        }
        // One pass over the rows of as many sequences as a launch carries (all of them unless the batch is
        // large: then group by group, each depth by the rows it brings).  The drafted features of the
        // frontier rows sit at the sequence's place in the batch (i * rows_q_each), whatever the grouping.
        const int prev_each = d - 1 == 1 ? 1 : k;
        for (int i0 = 0; i0 < B;) {
            int i1 = i0, grows = 0;
            while (i1 < B && grows + plans[i1].plan.n_rows <= c->launch_rows) grows += plans[i1++].plan.n_rows;
            std::vector<SeqPlan> gp(plans.begin() + i0, plans.begin() + i1);
            const int nb = i1 - i0;
            std::vector<int> q0;
            spec_pass(c, s, gp, d - 1, c->fhat[(d - 1) & 1] + (size_t)i0 * prev_each * c->md.d, prev_each,
                      c->fhat[d & 1] + (size_t)i0 * rows_q_each * c->md.d, &q0);
            const int rows_q = nb * rows_q_each;
            run_head_topk(c, rows_q, d);
            TreeDev tds[8];
            for (int i = 0; i < nb; ++i) {
                Seq &sq = c->seq[act[i0 + i]];
                tds[i] = sq.td;                              // with this sequence's rows of the top-k
                tds[i].topk_id = c->topk_id_all + (size_t)q0[i] * k; tds[i].topk_logp = c->topk_logp_all + (size_t)q0[i] * k;
                sq.spec_len[s] = sq.t;
                sq.spec_tmp_depth[s] = d - 1;
            }
            launch_tree_expand(tds, nb, d, k, L, rows_q_each, cf.vocab, c->st);   // one launch, a workgroup per sequence
            i0 = i1;
        }
    }
    const int pool = k + (L - 1) * k * k;
    {
        TreeDev tds[8];
        int ts[8];
        const int32_t *toks[8];
        int32_t *slots[8];
        for (int i = 0; i < B; ++i) {
            Seq &sq = c->seq[act[i]];
            tds[i] = sq.td; ts[i] = sq.t; toks[i] = sq.tokens_dev; slots[i] = sq.tree_slot;
            sq.tree_n = (cf.total_tokens < pool ? cf.total_tokens : pool) + 1;
            sq.tree_ready = 1;
        }
        launch_tree_finalize(tds, B, k, L, cf.total_tokens, ts, toks, slots, c->st);
    }
    (void)hipEventRecord(c->ev[1], c->st);
    c->ev_pending[0] = true;
    HIP_TRY(c, hipGetLastError());
    if (!out) return POSS_OK;                    // nothing for the host: the work stays queued
    int rc = copy_tree_out(c, c->seq[all[0]], out);             // the first active sequence's
    if (rc) return rc;
    return sync_and_harvest(c);
}

int poss_get_tree_seq(poss_ctx *c, int32_t seq, poss_tree *out) {
    if (!c || !out) return POSS_E_INVALID_ARG;
    if (seq < 0 || seq >= c->B) return fail(c, POSS_E_INVALID_ARG, "poss_get_tree_seq: no sequence %d (batch %d)", seq, c->B);
    if (!c->seq[seq].tree_ready) return fail(c, POSS_E_BAD_STATE, "poss_get_tree_seq: no drafted tree");
    int rc = copy_tree_out(c, c->seq[seq], out);
    if (rc) return rc;
    return sync_and_harvest(c);
}

int poss_debug_build_tree(poss_ctx *c, const int32_t *ids, const float *logp, poss_tree *out) {
    if (!c) return POSS_E_INVALID_ARG;
    if (!ids || !logp) return fail(c, POSS_E_INVALID_ARG, "poss_debug_build_tree: null argument");
    if (c->state != ST_READY) return fail(c, POSS_E_BAD_STATE, "poss_debug_build_tree: needs a prefilled context");
    const poss_config &cf = c->cfg;
    const int k = cf.top_k, L = cf.depth;
    Seq &sq = c->seq[0];
    int32_t *sid = static_cast<int32_t *>(c->pinned);
    float *slp = reinterpret_cast<float *>(sid + (size_t)L * k * k);
    memcpy(sid, ids, (size_t)L * k * k * sizeof(int32_t));
    memcpy(slp, logp, (size_t)L * k * k * sizeof(float));
    for (int d = 1; d <= L; ++d) {
        const int rows = d == 1 ? 1 : k;
        HIP_TRY(c, hipMemcpyAsync(sq.td.topk_id, sid + (size_t)(d - 1) * k * k, rows * k * sizeof(int32_t), hipMemcpyHostToDevice, c->st));
        HIP_TRY(c, hipMemcpyAsync(sq.td.topk_logp, slp + (size_t)(d - 1) * k * k, rows * k * sizeof(float), hipMemcpyHostToDevice, c->st));
        launch_tree_expand(&sq.td, 1, d, k, L, rows, cf.vocab, c->st);
    }
    {
        const int32_t *toks = sq.tokens_dev;
        launch_tree_finalize(&sq.td, 1, k, L, cf.total_tokens, &sq.t, &toks, &sq.tree_slot, c->st);
    }
    const int pool = k + (L - 1) * k * k;
    sq.tree_n = (cf.total_tokens < pool ? cf.total_tokens : pool) + 1;
    sq.tree_ready = 1;
    if (out) { int rc = copy_tree_out(c, sq, out); if (rc) return rc; }
    HIP_TRY(c, hipStreamSynchronize(c->st));
    HIP_TRY(c, hipGetLastError());
    return POSS_OK;
}

int poss_verify_tree(poss_ctx *c, const poss_tree *tree, int32_t *argmax_out, void *logits_out, void *feat_out) {
    if (!c) return POSS_E_INVALID_ARG;
    if (c->state != ST_READY) return fail(c, POSS_E_BAD_STATE, "poss_verify_tree: needs a prefilled context with no pending verification");
    const poss_config &cf = c->cfg;
    const std::vector<int> act = active_seqs(c);
    const int B = (int)act.size();                         // sequences in this round; i-th active sequence = act[i]
    int row0[8], n_rows[8], rows = 0;                      // a sequence's rows in the batch-wide arrays
    if (tree) {                                            // one tree per sequence: tree[0 .. batch-1], inactive ones ignored
        for (int i = 0; i < B; ++i) {
            const poss_tree &tr = tree[act[i]];
            const int n = tr.n_nodes;
            if (n < 1 || n > cf.total_tokens + 1) return fail(c, POSS_E_BAD_TREE, "poss_verify_tree: %d nodes, capacity %d", n, cf.total_tokens + 1);
            if (!tr.token || !tr.parent) return fail(c, POSS_E_INVALID_ARG, "poss_verify_tree: null tree arrays");
            std::vector<int> depth(n, 0);
            if (tr.parent[0] != -1) return fail(c, POSS_E_BAD_TREE, "poss_verify_tree: parent[0] must be -1");
            for (int v2 = 1; v2 < n; ++v2) {
                const int p = tr.parent[v2];
                if (p < 0 || p >= v2) return fail(c, POSS_E_BAD_TREE, "poss_verify_tree: parent[%d] = %d does not precede the node", v2, p);
                if (tr.token[v2] < 0 || tr.token[v2] >= cf.vocab) return fail(c, POSS_E_BAD_TREE, "poss_verify_tree: token[%d] out of range", v2);
                depth[v2] = depth[p] + 1;
                if (depth[v2] > cf.depth) return fail(c, POSS_E_BAD_TREE, "poss_verify_tree: node %d deeper than depth %d", v2, cf.depth);
                for (int j = 1; j < v2; ++j)
                    if (tr.parent[j] == p && tr.token[j] == tr.token[v2])
                        return fail(c, POSS_E_BAD_TREE, "poss_verify_tree: siblings %d and %d carry the same token", j, v2);
            }
            row0[i] = rows; n_rows[i] = n; rows += n;       // back to back
        }
    } else {
        for (int i = 0; i < B; ++i) {
            const Seq &sq = c->seq[act[i]];
            if (!sq.tree_ready) return fail(c, POSS_E_BAD_STATE, "poss_verify_tree: no drafted tree");
            row0[i] = sq.tree_row0; n_rows[i] = sq.tree_n; rows = row0[i] + n_rows[i];   // fixed stride, no gaps
        }
    }
    for (int i = 0; i < B; ++i) {
        const int t = c->seq[act[i]].t;
        if (t + n_rows[i] > c->cache_slots || t + cf.depth + 1 > cf.max_seq)
            return fail(c, POSS_E_CAPACITY, "poss_verify_tree: %d committed tokens leave no room (max_seq %d)", t, cf.max_seq);
    }
    if (tree && c->draft_sampling && c->temperature > 0.f)
        return fail(c, POSS_E_BAD_STATE, "poss_verify_tree: with drawn children only the drafted tree can be verified (a caller's tree has no draft distributions)");
    (void)hipEventRecord(c->ev[2], c->st);
    if (tree) {
        int32_t *stage = static_cast<int32_t *>(c->pinned);      // [tokens | parents | node counts]
        const int RA = c->rows_all;
        for (int i = 0; i < B; ++i) {
            const int b = act[i];
            Seq &sq = c->seq[b];
            const int n = n_rows[i], t = sq.t;
            point_tree(c, sq, row0[i]);
            memcpy(stage + row0[i], tree[b].token, n * sizeof(int32_t));
            stage[row0[i]] = sq.tokens[t];                        // the root is always x_t
            memcpy(stage + RA + row0[i], tree[b].parent, n * sizeof(int32_t));
            stage[2 * RA + i] = n;
            HIP_TRY(c, hipMemcpyAsync(sq.td.token, stage + row0[i], n * sizeof(int32_t), hipMemcpyHostToDevice, c->st));
            HIP_TRY(c, hipMemcpyAsync(sq.td.parent, stage + RA + row0[i], n * sizeof(int32_t), hipMemcpyHostToDevice, c->st));
            HIP_TRY(c, hipMemcpyAsync(sq.td.n_nodes, stage + 2 * RA + i, sizeof(int32_t), hipMemcpyHostToDevice, c->st));
            launch_tree_upload_finish(n, t, sq.td.token, sq.td.parent, sq.td.depth, sq.td.pos, sq.tree_slot, sq.td.mask, c->st);
            sq.tree_n = n; sq.tree_ready = 1;
        }
    }                                     // (a drafted tree's slots were written when it was finalized)
    // The trees' rows are adjacent slices of the batch-wide arrays: one pass over all of them, or, when they
    // are more than a launch carries, one pass per group of sequences (the rows of a group are adjacent too;
    // as many sequences as fit: eight root-only trees, vanilla decoding of a batch, share one pass).
    const int n = n_rows[0];                               // host and device outputs: the first active sequence's rows
    for (int i0 = 0; i0 < B;) {
        int i1 = i0, grows = 0;
        while (i1 < B && grows + n_rows[i1] <= c->launch_rows) grows += n_rows[i1++];
        const int base = row0[i0];
        RowMeta rm{c->tree_pos_all + base, c->tree_slot_all + base, c->tree_mask_all + (size_t)base * MASK_WORDS};
        std::vector<Seg> segs;
        int rel0[8];
        for (int i = i0; i < i1; ++i) {
            rel0[i - i0] = row0[i] - base;
            segs.push_back(Seg{act[i], nullptr, row0[i] - base, n_rows[i], grows, 0, c->seq[act[i]].t, n_rows[i]});
        }
        target_forward(c, grows, c->tree_token_all + base, rm, segs, c->feats + (size_t)base * cf.d_model);
        int ld = 0;
        { int rc = head_and_choose(c, nullptr, grows, i0 == 0 && logits_out, c->tree_depth_all, act.data() + i0, i1 - i0, rel0, n_rows + i0, base, &ld, tree == nullptr); if (rc) return rc; }
        if (i0 == 0 && logits_out)                         // before the next group overwrites the logits
            launch_copy_rows_f32(c->logits, ld, static_cast<float *>(logits_out), cf.vocab, n, cf.vocab, c->st);
        i0 = i1;
    }
    (void)hipEventRecord(c->ev[3], c->st);
    c->ev_pending[1] = true;
    if (feat_out) launch_copy_rows_f32(c->feats, cf.d_model, static_cast<float *>(feat_out), cf.d_model, n, cf.d_model, c->st);
    HIP_TRY(c, hipGetLastError());
    c->state = ST_VERIFIED;
    // Nothing to hand over: stay queued.  (A caller's tree was staged in pinned memory; the only call
    // allowed next, poss_accept_and_commit, waits for the stream before that memory is touched again.)
    if (!argmax_out && !logits_out && !feat_out) return POSS_OK;
    if (argmax_out) HIP_TRY(c, hipMemcpyAsync(argmax_out, c->argmax_dev, n * sizeof(int32_t), hipMemcpyDeviceToHost, c->st));
    return sync_and_harvest(c);
}

int poss_accept_and_commit(poss_ctx *c, int32_t *path_idx_out, int32_t *n_accepted_out, int32_t *committed_out,
                           int32_t *n_committed_out) {
    if (!c) return POSS_E_INVALID_ARG;
    if (c->state != ST_VERIFIED) return fail(c, POSS_E_BAD_STATE, "poss_accept_and_commit: no verified tree");
    const poss_config &cf = c->cfg;
    const int L = cf.depth;
    const std::vector<int> act = active_seqs(c);
    (void)hipEventRecord(c->ev[4], c->st);
    for (int b : act) {
        Seq &sq = c->seq[b];
        const int row0 = sq.tree_row0;
        launch_commit(c->md, cf.n_layers, sq.target_kv_dev, sq.td.token, sq.td.parent, c->argmax_dev + row0, sq.td.n_nodes, L, sq.t,
                      c->feats + (size_t)row0 * cf.d_model, sq.feat_stash, sq.tokens_dev, sq.walk_dev, sq.result_dev, c->st);
    }
    (void)hipEventRecord(c->ev[5], c->st);
    c->ev_pending[2] = true;
    { int rc = sync_and_harvest(c); if (rc) return rc; }
    for (int b : act) {
        Seq &sq = c->seq[b];
        const int32_t *walk = sq.result_pinned, *toks = walk + 32;     // written by the kernel itself
        const int m = walk[0];
        if (m < 0 || m > L) return fail(c, POSS_E_HIP, "poss_accept_and_commit: walk returned %d accepted tokens", m);
        for (int j = 0; j <= m; ++j) { sq.tokens.push_back(toks[j]); sq.last_tokens[j] = toks[j]; sq.last_path[j] = walk[2 + j]; }
        sq.last_m = m;
        sq.t += m + 1;
        sq.tree_ready = 0;
        c->stats.rounds += 1;
        c->stats.committed_tokens += m + 1;
        for (int i = 1; i <= m; ++i) c->stats.c[i] += 1;
    }
    const Seq &s0 = c->seq[act[0]];                        // the outputs of this call: the first active sequence
    if (path_idx_out) for (int j = 0; j <= s0.last_m; ++j) path_idx_out[j] = s0.last_path[j];
    if (n_accepted_out) *n_accepted_out = s0.last_m;
    if (committed_out) for (int j = 0; j <= s0.last_m; ++j) committed_out[j] = s0.last_tokens[j];
    if (n_committed_out) *n_committed_out = s0.last_m + 1;
    c->state = ST_READY;
    return POSS_OK;
}

int poss_get_commit_seq(poss_ctx *c, int32_t seq, int32_t *path_idx_out, int32_t *n_accepted_out, int32_t *committed_out,
                        int32_t *n_committed_out) {
    if (!c) return POSS_E_INVALID_ARG;
    if (seq < 0 || seq >= c->B) return fail(c, POSS_E_INVALID_ARG, "poss_get_commit_seq: no sequence %d (batch %d)", seq, c->B);
    if (c->state != ST_READY || c->stats.rounds == 0) return fail(c, POSS_E_BAD_STATE, "poss_get_commit_seq: no committed round");
    const Seq &sq = c->seq[seq];
    if (path_idx_out) for (int j = 0; j <= sq.last_m; ++j) path_idx_out[j] = sq.last_path[j];
    if (n_accepted_out) *n_accepted_out = sq.last_m;
    if (committed_out) for (int j = 0; j <= sq.last_m; ++j) committed_out[j] = sq.last_tokens[j];
    if (n_committed_out) *n_committed_out = sq.last_m + 1;
    return POSS_OK;
}

static int check_uniforms(poss_ctx *c, const float *u, int32_t n_u) {
    if (!u || n_u < 1 || n_u > POSS_MAX_DEPTH + 1) return fail(c, POSS_E_INVALID_ARG, "sampling: needs 1..%d uniform numbers", POSS_MAX_DEPTH + 1);
    for (int i = 0; i < n_u; ++i)
        if (!(u[i] >= 0.f && u[i] < 1.f)) return fail(c, POSS_E_INVALID_ARG, "sampling: u[%d] is not in [0, 1)", i);
    return POSS_OK;
}

int poss_set_sampling(poss_ctx *c, float temperature, const float *u, int32_t n_u) {
    if (!c) return POSS_E_INVALID_ARG;
    if (!(temperature >= 0.f)) return fail(c, POSS_E_INVALID_ARG, "poss_set_sampling: temperature must be >= 0");
    if (temperature > 0.f) {
        { int rc = check_uniforms(c, u, n_u); if (rc) return rc; }
        HIP_TRY(c, hipStreamSynchronize(c->st));           // a queued verification may still read the staging array
        for (int b = 0; b < c->B; ++b)                     // every sequence; poss_set_uniforms_seq gives one its own
            for (int i = 0; i <= POSS_MAX_DEPTH; ++i) c->u_pinned[b * (POSS_MAX_DEPTH + 1) + i] = i < n_u ? u[i] : u[n_u - 1];
    }
    c->temperature = temperature;
    return POSS_OK;
}

int poss_set_draft_sampling(poss_ctx *c, int32_t enable, const float *u_draft, const float *u_accept) {
    if (!c) return POSS_E_INVALID_ARG;
    if (!enable) { c->draft_sampling = 0; return POSS_OK; }
    if (c->B != 1) return fail(c, POSS_E_INVALID_ARG, "poss_set_draft_sampling: built for contexts of one sequence");
    if (!u_draft || !u_accept) return fail(c, POSS_E_INVALID_ARG, "poss_set_draft_sampling: null argument");
    if (c->cfg.vocab > 8192 * 256 || c->cfg.top_k > 16)   // the samplers' block sums and list of drawn ids in LDS
        return fail(c, POSS_E_CAPACITY, "poss_set_draft_sampling: vocabulary above 2097152 or k above 16");
    const int k = c->cfg.top_k, L = c->cfg.depth, nd = L * k * k, na = (L + 1) * (k + 1);
    for (int i = 0; i < nd; ++i)
        if (!(u_draft[i] >= 0.f && u_draft[i] < 1.f)) return fail(c, POSS_E_INVALID_ARG, "poss_set_draft_sampling: u_draft[%d] is not in [0, 1)", i);
    for (int i = 0; i < na; ++i)
        if (!(u_accept[i] >= 0.f && u_accept[i] < 1.f)) return fail(c, POSS_E_INVALID_ARG, "poss_set_draft_sampling: u_accept[%d] is not in [0, 1)", i);
    HIP_TRY(c, hipStreamSynchronize(c->st));              // queued work may still read the staging arrays
    memcpy(c->ud_pinned, u_draft, nd * sizeof(float));
    memcpy(c->ua_pinned, u_accept, na * sizeof(float));
    c->draft_sampling = 1;
    return POSS_OK;
}

int poss_set_uniforms_seq(poss_ctx *c, int32_t seq, const float *u, int32_t n_u) {
    if (!c) return POSS_E_INVALID_ARG;
    if (seq < 0 || seq >= c->B) return fail(c, POSS_E_INVALID_ARG, "poss_set_uniforms_seq: no sequence %d (batch %d)", seq, c->B);
    { int rc = check_uniforms(c, u, n_u); if (rc) return rc; }
    HIP_TRY(c, hipStreamSynchronize(c->st));
    for (int i = 0; i <= POSS_MAX_DEPTH; ++i) c->u_pinned[seq * (POSS_MAX_DEPTH + 1) + i] = i < n_u ? u[i] : u[n_u - 1];
    return POSS_OK;
}

int poss_get_stats(poss_ctx *c, poss_stats *out) {
    if (!c || !out) return POSS_E_INVALID_ARG;
    { int rc = sync_and_harvest(c); if (rc) return rc; }
    *out = c->stats;
    return POSS_OK;
}

int poss_get_tokens_seq(poss_ctx *c, int32_t seq, int32_t *tokens_out, int32_t cap, int32_t *n_out) {
    if (!c) return POSS_E_INVALID_ARG;
    if (seq < 0 || seq >= c->B) return fail(c, POSS_E_INVALID_ARG, "poss_get_tokens: no sequence %d (batch %d)", seq, c->B);
    const std::vector<int32_t> &tokens = c->seq[seq].tokens;
    const int n = (int)tokens.size();
    if (n_out) *n_out = n;
    if (tokens_out) {
        if (cap < n) return fail(c, POSS_E_CAPACITY, "poss_get_tokens: %d tokens, capacity %d", n, cap);
        memcpy(tokens_out, tokens.data(), n * sizeof(int32_t));
    }
    return POSS_OK;
}

int poss_get_tokens(poss_ctx *c, int32_t *tokens_out, int32_t cap, int32_t *n_out) {
    return poss_get_tokens_seq(c, 0, tokens_out, cap, n_out);
}

int poss_profile_gemm(poss_ctx *c, int32_t enable) {
    if (!c) return POSS_E_INVALID_ARG;
    c->prof_on = enable ? 1 : 0;
    return POSS_OK;
}

int poss_gemm_profile(poss_ctx *c, int64_t *launches, double *ms, double *weight_bytes) {
    if (!c) return POSS_E_INVALID_ARG;
    HIP_TRY(c, hipStreamSynchronize(c->st));
    double total = 0;
    for (int i = 0; i < c->prof_n; ++i) {
        float e = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&e, c->prof_ev[2 * i], c->prof_ev[2 * i + 1]));
        total += e;
    }
    if (launches) *launches = c->prof_n;
    if (ms) *ms = total;
    if (weight_bytes) *weight_bytes = c->prof_bytes;
    c->prof_n = 0; c->prof_bytes = 0;
    return POSS_OK;
}

int poss_set_tuning(poss_ctx *c, int32_t gemm_target_workgroups, int32_t attn_keys_per_split) {
    if (!c) return POSS_E_INVALID_ARG;
    if (gemm_target_workgroups < 0 || gemm_target_workgroups > 4096) return fail(c, POSS_E_INVALID_ARG, "poss_set_tuning: workgroup target out of range");
    if (attn_keys_per_split && (attn_keys_per_split < 64 || attn_keys_per_split % 32)) return fail(c, POSS_E_INVALID_ARG, "poss_set_tuning: keys per split must be a multiple of 32, >= 64");
    c->gemm_target_wgs = gemm_target_workgroups;
    if (attn_keys_per_split) c->attn_keys_per_split = attn_keys_per_split;
    return POSS_OK;
}

int poss_set_launch_rows(poss_ctx *c, int32_t rows) {
    if (!c) return POSS_E_INVALID_ARG;
    if (rows < MAX_ROWS || rows > LAUNCH_ROWS) return fail(c, POSS_E_INVALID_ARG, "poss_set_launch_rows: %d is outside %d..%d", rows, MAX_ROWS, LAUNCH_ROWS);
    c->launch_rows = rows;
    return POSS_OK;
}

int poss_debug_set_taps(poss_ctx *c, void *taps) {
    if (!c) return POSS_E_INVALID_ARG;
    c->taps_user = static_cast<float *>(taps);
    return POSS_OK;
}

int poss_debug_draft_logits(poss_ctx *c, int32_t row0, int32_t n, float *out) {
    if (!c || !out) return POSS_E_INVALID_ARG;
    const poss_config &cf = c->cfg;
    const int rows = 1 + (cf.depth - 1) * cf.top_k;
    if (!c->draft_sampling || !c->seq[0].tree_ready)
        return fail(c, POSS_E_BAD_STATE, "poss_debug_draft_logits: needs a tree drafted with drawn children");
    if (row0 < 0 || n < 1 || row0 + n > rows) return fail(c, POSS_E_INVALID_ARG, "poss_debug_draft_logits: rows out of range (%d expanded nodes)", rows);
    const int ld = gemm_npad(cf.vocab);
    launch_copy_rows_f32(c->dlogits + (size_t)row0 * ld, ld, out, cf.vocab, n, cf.vocab, c->st);
    return sync_and_harvest(c);
}

int poss_debug_read_kv(poss_ctx *c, int32_t which, int32_t layer, int32_t slot0, int32_t n, float *k_out, float *v_out) {
    if (!c || !k_out || !v_out) return POSS_E_INVALID_ARG;
    if (n < 1 || slot0 < 0 || slot0 + n > c->cache_slots) return fail(c, POSS_E_INVALID_ARG, "poss_debug_read_kv: slots out of range");
    if (which >= c->cfg.n_specialists || (which < 0 && (layer < 0 || layer >= c->cfg.n_layers)))
        return fail(c, POSS_E_INVALID_ARG, "poss_debug_read_kv: no such cache");
    const KVCache &kv = which < 0 ? c->seq[0].target_kv[layer] : c->seq[0].spec_kv[which];
    // stage through the partial-sum buffer (idle between calls)
    const size_t per = (size_t)c->md.hkv * c->md.dh;
    const int chunk = 64;
    for (int i = 0; i < n; i += chunk) {
        const int m = n - i < chunk ? n - i : chunk;
        float *kd = c->part, *vd = c->part + (size_t)chunk * per;
        launch_read_kv(c->md, kv, slot0 + i, m, kd, vd, c->st);
        HIP_TRY(c, hipMemcpyAsync(k_out + (size_t)i * per, kd, m * per * sizeof(float), hipMemcpyDeviceToHost, c->st));
        HIP_TRY(c, hipMemcpyAsync(v_out + (size_t)i * per, vd, m * per * sizeof(float), hipMemcpyDeviceToHost, c->st));
        HIP_TRY(c, hipStreamSynchronize(c->st));
    }
    return POSS_OK;
}

__global__ void sum_planes_kernel(const float *__restrict__ part, int S, size_t plane, int Npad, int N, float *__restrict__ y) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x, m = blockIdx.y;
    if (n >= N) return;
    float a = 0.f;
    for (int s = 0; s < S; ++s) a += part[(size_t)s * plane + (size_t)m * Npad + n];
    y[(size_t)m * N + n] = a;
}

size_t poss_debug_gemm_scratch_bytes(int32_t dtype, int32_t M, int32_t N, int32_t K) {
    if (dtype < 0 || dtype > 2 || M < 1 || M > LAUNCH_ROWS || N < 1 || K < 1) return 0;
    GemmShape g = gemm_plan(dtype, M, N, K, 4096);
    return (packed_elems(dtype, N, K) * dtype_size(dtype) + 255) / 256 * 256 +
           (size_t)g.S * LAUNCH_ROWS * g.Npad * sizeof(float) + (size_t)(g.Npad / GEMM_BLOCK_N) * sizeof(unsigned) + 1024;
}

int poss_debug_gemm(int32_t dtype, const void *x, const void *w, void *y, int32_t M, int32_t N, int32_t K,
                    int32_t target_workgroups, void *scratch, void *hip_stream, int32_t repeats,
                    float *ms_per_launch_out) {
    if (!x || !w || !y || !scratch) return fail(nullptr, POSS_E_INVALID_ARG, "poss_debug_gemm: null argument");
    if (dtype < 0 || dtype > 2 || M < 1 || M > LAUNCH_ROWS || N < 1 || K < 1 || repeats < 1)
        return fail(nullptr, POSS_E_INVALID_ARG, "poss_debug_gemm: bad shape");
    if (dtype != DT_F32 && (K % 8)) return fail(nullptr, POSS_E_INVALID_ARG, "poss_debug_gemm: K must be a multiple of 8");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    GemmShape g = gemm_plan(dtype, M, N, K, target_workgroups);
    char *p = static_cast<char *>(scratch);
    void *wp = p;
    p += (packed_elems(dtype, N, K) * dtype_size(dtype) + 255) / 256 * 256;
    float *part = reinterpret_cast<float *>(p);
    p += ((size_t)g.S * LAUNCH_ROWS * g.Npad * sizeof(float) + 255) / 256 * 256;
    EpiArgs epi{};
    epi.mode = EPI_PLAIN; epi.out = static_cast<float *>(y); epi.ld_out = N;
    launch_pack(dtype, PackSrc{{w, nullptr, nullptr}, {N, 0, 0}}, K, wp, st);
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return fail(nullptr, POSS_E_HIP, "poss_debug_gemm: event creation failed");
    if (!launch_gemm(dtype, g, wp, x, K, part, epi, 0.f, st)) return fail(nullptr, POSS_E_INVALID_ARG, "poss_debug_gemm: launch refused");
    (void)hipEventRecord(e0, st);
    for (int i = 0; i < repeats; ++i) launch_gemm(dtype, g, wp, x, K, part, epi, 0.f, st);
    (void)hipEventRecord(e1, st);
    hipError_t e = hipStreamSynchronize(st);
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    if (e != hipSuccess) return fail(nullptr, POSS_E_HIP, "poss_debug_gemm: %s", hipGetErrorString(e));
    if (ms_per_launch_out) *ms_per_launch_out = ms / repeats;
    return POSS_OK;
}

}  // extern "C"

// ---- the same GEMM path for callers that cannot allocate device memory --------------------------
// Packed weights and split-K planes live in a file-scope device array instead of a caller's buffer.
// In host code the array's name is only a handle: its device address is looked up once per GPU
// (hipGetSymbolAddress, with that GPU current) and that address is what kernels are given.
static __device__ __align__(256) unsigned char scratch[POSS_GEMM_STATIC_BYTES];

namespace {
constexpr int STATIC_MAX_DEVICES = 64;
void *g_scratch_ptr[STATIC_MAX_DEVICES];     // device address of `scratch` on each GPU, nullptr until looked up
std::mutex g_scratch_mutex;

// The address of the current GPU's copy of `scratch`; nullptr (and a message) on failure.
void *static_scratch_address() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) {
        fail(nullptr, POSS_E_HIP, "poss_gemm_static: no current device (or device index above %d)", STATIC_MAX_DEVICES - 1);
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            fail(nullptr, POSS_E_HIP, "poss_gemm_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
            return nullptr;
        }
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

extern "C" int poss_gemm_static(int32_t dtype, const void *x, const void *w, void *y, int32_t M, int32_t N, int32_t K,
                                int32_t target_workgroups, void *hip_stream) {
    if (!x || !w || !y) return fail(nullptr, POSS_E_INVALID_ARG, "poss_gemm_static: null argument");
    if (dtype < 0 || dtype > 2 || M < 1 || M > MAX_ROWS || N < 1 || K < 1)
        return fail(nullptr, POSS_E_INVALID_ARG, "poss_gemm_static: bad shape");
    if (dtype != DT_F32 && (K % 8)) return fail(nullptr, POSS_E_INVALID_ARG, "poss_gemm_static: K must be a multiple of 8");
    if (target_workgroups < 0 || target_workgroups > 4096) return fail(nullptr, POSS_E_INVALID_ARG, "poss_gemm_static: workgroup target out of range");
    // sizes in 64 bits before anything is laid out: the limit is checked on the exact byte count
    const GemmShape g = gemm_plan(dtype, M, N, K, target_workgroups);
    const size_t w_bytes = ((size_t)g.Npad * g.Kpad * dtype_size(dtype) + 255) / 256 * 256;
    const size_t part_bytes = (size_t)g.S * MAX_ROWS * g.Npad * sizeof(float);
    if ((size_t)g.Npad > POSS_GEMM_STATIC_BYTES || (size_t)g.Kpad > POSS_GEMM_STATIC_BYTES || w_bytes + part_bytes > POSS_GEMM_STATIC_BYTES)
        return fail(nullptr, POSS_E_CAPACITY, "poss_gemm_static: M=%d N=%d K=%d needs %zu bytes of scratch, the static buffer holds %zu",
                    M, N, K, w_bytes + part_bytes, (size_t)POSS_GEMM_STATIC_BYTES);
    unsigned char *base = static_cast<unsigned char *>(static_scratch_address());
    if (!base) return POSS_E_HIP;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    void *wp = base;
    float *part = reinterpret_cast<float *>(base + w_bytes);
    EpiArgs epi{};
    epi.mode = EPI_PLAIN; epi.out = static_cast<float *>(y); epi.ld_out = N;
    // every byte the kernels read is written first by this call: the packed matrix including its zero
    // padding by the pack kernel, every row of every plane by the stream kernel
    launch_pack(dtype, PackSrc{{w, nullptr, nullptr}, {N, 0, 0}}, K, wp, st);
    if (!launch_gemm(dtype, g, wp, x, K, part, epi, 0.f, st)) return fail(nullptr, POSS_E_INVALID_ARG, "poss_gemm_static: launch refused");
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(nullptr, POSS_E_HIP, "poss_gemm_static: %s", hipGetErrorString(e));
    return POSS_OK;
}
