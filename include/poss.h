/* poss.h - C ABI of the MI355X (gfx950) PosS draft-and-verify library.
 *
 * One round of position-specialist speculative decoding (arXiv 2506.03566) at
 * batch 1, under greedy verification or, after poss_set_sampling, at a temperature:
 *
 *   poss_load -> poss_prefill -> ( poss_draft_tree -> poss_verify_tree
 *                                  -> poss_accept_and_commit )*
 *
 * With poss_config.batch = B > 1 a context carries B independent sequences:
 * each has its own caches, tree and token stream, every pass stacks their rows into one set of
 * weight-streaming launches (of at most POSS_LAUNCH_ROWS rows: a larger batch runs its passes group by
 * group), and the three round calls advance all of them; poss_prefill_seq,
 * poss_get_tree_seq, poss_get_commit_seq, poss_get_tokens_seq and poss_set_uniforms_seq address one
 * sequence (the calls without _seq address sequence 0); poss_set_active and poss_reset_seq take a
 * sequence out of the rounds or replace it.  A sequence's tokens are the ones it gets at batch 1.
 *
 * Every step runs in hand-written HIP kernels of this library.  All pointers
 * are plain addresses; each argument says whether it is HOST or DEVICE memory.
 * The library never allocates device memory: weights, the workspace and the
 * stream belong to the caller.  Calls enqueue work on the stream given to
 * poss_load and wait for it only to hand back host outputs: a round whose draft and
 * verify calls ask for none waits once, in poss_accept_and_commit.
 *
 * Every function returning int returns POSS_OK (0) or a negative POSS_E_*
 * code; a failing call leaves the context as it was and poss_last_error()
 * describes the failure.  Calls on one context must not overlap.
 *
 * Notation (paper): target model theta_T with last-layer hidden state
 * ("feature") f^(T); S position specialists theta_S^1..S, each serving n draft
 * positions (PosS-n); prediction depth L; tree width k; N draft tokens kept
 * per round; t = index of the last committed token x_t (the tree root).
 */
#ifndef POSS_H
#define POSS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define POSS_OK             0
#define POSS_E_INVALID_ARG -1   /* null pointer, shape the kernels do not support     */
#define POSS_E_BAD_STATE   -2   /* call out of order                                  */
#define POSS_E_CAPACITY    -3   /* sequence, tree or workspace larger than configured */
#define POSS_E_BAD_TREE    -4   /* caller-supplied tree is not a valid draft tree     */
#define POSS_E_HIP         -5   /* a HIP runtime call failed                          */

#define POSS_DTYPE_F32  0
#define POSS_DTYPE_BF16 1
#define POSS_DTYPE_F16  2

#define POSS_MAX_ROWS   128     /* rows of ONE sequence in a pass: tree rows           */
#define POSS_LAUNCH_ROWS 256    /* rows one launch carries: sequences together, prefill */
#define POSS_MASK_WORDS 2       /* 64-bit words of one ancestor mask                  */
#define POSS_MAX_DEPTH  16

typedef struct poss_ctx poss_ctx;           /* opaque; created by poss_load, host memory */

/* Shapes.  Target: Llama-style decoder (section 4.1 "Target Models").  Drafter:
 * n_specialists layers of the target's layer shape, each preceded by an fc
 * projection 2*d_model -> d_model over [token embedding ; feature] (section 2.2,
 * Eq. 1; section 3.2).  Draft position i (0-based) is served by specialist
 * min(i / positions_per_specialist, n_specialists - 1)  (Eq. 7; the clamp is this
 * library's reading for depths beyond S*n).  Tree: section 4.1 "Implementations"
 * (width = top_k, depth, total_tokens = draft nodes kept, root not counted).
 * dtype is the storage type of weights, GEMM operands and KV caches; accumulation,
 * the residual stream, softmax, norms and logits are float32. */
typedef struct poss_config {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float   rms_eps, rope_theta;
    int32_t dtype;                           /* POSS_DTYPE_*                               */
    int32_t n_specialists, positions_per_specialist, fc_bias;
    int32_t top_k, depth, total_tokens;
    int32_t max_seq;                         /* capacity in committed tokens (multiple of kv_page_tokens, at most 500000) */
    int32_t kv_page_tokens;                  /* tokens per KV page: 32, 64 or 128           */
    int32_t kv_page_order;                   /* 0: pages in order; 1: physical pages reversed (layout tests) */
    int32_t batch;                           /* sequences per round: 0 or 1 = one; up to 8.  A pass stacks the rows of as *
                                              * many sequences as fit POSS_LAUNCH_ROWS and runs group by group beyond it */
} poss_config;

/* Weights: DEVICE pointers to row-major [out, in] tensors of `dtype`.
 * layer[l*9 + j], j = attn_norm[d], wq[Hq*dh,d], wk[Hkv*dh,d], wv[Hkv*dh,d], wo[d,Hq*dh],
 *                     mlp_norm[d], w_gate[F,d], w_up[F,d], w_down[d,F].
 * spec[s*11 + j], j = fc_w[d,2d] (input columns ordered [embedding ; feature]), fc_b[d],
 *                     then the 9 layer tensors.  The arrays of pointers are HOST memory.
 * poss_load repacks everything into the workspace; the caller may free its copies after. */
typedef struct poss_weights {
    const void *embed;        /* [vocab, d]  token embedding, shared by target and drafter */
    const void *lm_head;      /* [vocab, d]  shared LM head (section 2.2)                  */
    const void *final_norm;   /* [d]         final RMSNorm gain (part of Head)             */
    const void *const *layer;
    const void *const *spec;
} poss_weights;

/* A draft tree in HOST memory, arrays of capacity >= total_tokens + 1 owned by the caller.
 * Node 0 is the root x_t.  parent[0] = -1, parent[i] < i.  pos[i] = t + depth[i].
 * mask[i*POSS_MASK_WORDS + w]: bit j of the concatenated words is set iff node j is node i
 * or an ancestor of it.  score[i]: sum of drafter log-probabilities on the path (0 for the
 * root).  As input to poss_verify_tree only n_nodes, token[1..] and parent are read. */
typedef struct poss_tree {
    int32_t   n_nodes;
    int32_t  *token, *parent, *depth, *pos;
    uint64_t *mask;
    float    *score;
} poss_tree;

/* Acceptance statistics (section 3.1): c[i] = rounds that accepted at least i draft tokens,
 * so P(A_i) = c[i]/rounds, pos-acc_i = c[i]/c[i-1] (Eq. 3), and the mean number of accepted
 * draft tokens per round is sum_i c[i] / rounds (Eq. 4 summed over k).  With batch > 1 every
 * sequence's round counts (rounds grows by batch per poss_accept_and_commit).  Times are HIP-event
 * milliseconds summed over the calls. */
typedef struct poss_stats {
    int64_t rounds, committed_tokens;
    int64_t c[POSS_MAX_DEPTH + 1];
    double  ms_draft, ms_verify, ms_commit;
} poss_stats;

/* Bytes of DEVICE workspace poss_load needs for this configuration (0 if it is invalid). */
size_t poss_workspace_bytes(const poss_config *cfg);

/* Create a context.  cfg, w: HOST structs (w's tensors DEVICE).  workspace: DEVICE memory of
 * at least poss_workspace_bytes(cfg) bytes, 256-byte aligned, owned by the caller and kept
 * alive until poss_free.  hip_stream: a hipStream_t (NULL = default stream).  *out receives
 * the context.  Repacks the weights into MFMA operand order and zeroes the KV caches. */
int poss_load(const poss_config *cfg, const poss_weights *w, void *workspace,
              size_t workspace_bytes, void *hip_stream, poss_ctx **out);

/* Forget the sequence (back to the state after poss_load); statistics are cleared. */
int poss_reset(poss_ctx *ctx);
/* Forget one sequence of a batch; the others keep their state and the statistics are kept.  Rounds
 * resume once the sequence has been given a new prompt (poss_prefill_seq): a finished sequence is
 * replaced while the rest of the batch goes on.  Not between verify and accept. */
int poss_reset_seq(poss_ctx *ctx, int32_t seq);
/* Set a sequence of a batch aside (active == 0: the rounds go on without it, its tokens stay readable)
 * or take it back in (it must still have its prompt; after poss_reset_seq use poss_prefill_seq, which
 * activates it).  The last active sequence cannot be set aside.  Drafted trees are dropped: the rows
 * of a round are laid out for the sequences that take part.  Not between verify and accept.  The
 * outputs of the round calls that address "sequence 0" address the first active sequence. */
int poss_set_active(poss_ctx *ctx, int32_t seq, int32_t active);

/* Causal target pass over the prompt (HOST int32 ids, 1 <= n_prompt, n_prompt + 1 <= max_seq),
 * then every specialist's keys/values for the pairs [x_j ; f_{j-1}], j = 1..n_prompt-1
 * (section 3.3: specialists do not share a cache).  *first_token_out = x_P, the target's greedy
 * token after the prompt; it becomes the root of the first tree. */
int poss_prefill(poss_ctx *ctx, const int32_t *prompt, int32_t n_prompt, int32_t *first_token_out);
/* The same for sequence seq (0 <= seq < batch).  Rounds can start once every sequence has its prompt. */
int poss_prefill_seq(poss_ctx *ctx, int32_t seq, const int32_t *prompt, int32_t n_prompt, int32_t *first_token_out);

/* Draft phase (section 6.2): `depth` specialist passes expand the tree level by level; the
 * total_tokens best candidates by cumulative log-probability form the tree.  out (HOST, may be
 * NULL) receives it; it also stays on the device for poss_verify_tree(ctx, NULL, ..).  With
 * out == NULL the call returns once the work is queued on the stream (no host wait); a device
 * error then surfaces at the next call that waits. */
int poss_draft_tree(poss_ctx *ctx, poss_tree *out);
/* The tree drafted last for sequence seq (HOST arrays as for poss_draft_tree); waits for the stream. */
int poss_get_tree_seq(poss_ctx *ctx, int32_t seq, poss_tree *out);

/* Verification phase (section 2.1): one target pass over all tree rows with tree position ids
 * and the ancestor mask.  tree: HOST, or NULL for the tree drafted last.  argmax_out (HOST,
 * int32[n_nodes], may be NULL): the target's greedy token after each node, lowest id on ties.
 * logits_out (DEVICE float32 [n_nodes, vocab], may be NULL) and feat_out (DEVICE float32
 * [n_nodes, d_model], may be NULL) receive Head(f) and f of every row (Eq. 6).  With all three
 * outputs NULL the call returns once the work is queued (no host wait), so that a round
 * draft -> verify -> accept waits for the device once, in poss_accept_and_commit; the tree
 * arrays are copied before the call returns.  With batch > 1 all sequences are verified in one pass:
 * tree is NULL (the drafted trees) or points to an array of `batch` trees, one per sequence; the
 * outputs then cover sequence 0's rows. */
int poss_verify_tree(poss_ctx *ctx, const poss_tree *tree, int32_t *argmax_out,
                     void *logits_out, void *feat_out);

/* Greedy acceptance (section 2.1, section 3.1: A_i subset of A_{i-1}) and commit.  Walks from
 * the root to the child whose token equals the target's greedy token, as long as there is one;
 * moves the accepted rows' keys/values to positions t.., keeps their features for the next
 * draft, appends the accepted tokens and the bonus token (the target's choice after the last
 * accepted node).  All outputs HOST, any may be NULL: path_idx_out[depth+1] node indices starting
 * with 0; *n_accepted_out = m; committed_out[depth+1] the m+1 new tokens; *n_committed_out = m+1.
 * With batch > 1 every sequence is committed (one kernel launch each, one wait); the outputs are
 * sequence 0's, poss_get_commit_seq has the others; the statistics count one round per sequence. */
int poss_accept_and_commit(poss_ctx *ctx, int32_t *path_idx_out, int32_t *n_accepted_out,
                           int32_t *committed_out, int32_t *n_committed_out);
/* What the last poss_accept_and_commit did for sequence seq (same outputs; no device work). */
int poss_get_commit_seq(poss_ctx *ctx, int32_t seq, int32_t *path_idx_out, int32_t *n_accepted_out,
                        int32_t *committed_out, int32_t *n_committed_out);

/* Verification at temperature > 0 (the paper evaluates temperature 0 and 1, section 4.1; section 2.1
 * only requires that verification keeps the target's output distribution).  The draft tree is built
 * as at temperature 0; the token the target chooses after a node is DRAWN from
 * softmax(logits / temperature) by inverse CDF in vocabulary order (the first id whose cumulative
 * probability exceeds u), with u[d] for a node of depth d, i.e. one uniform number in [0, 1) per
 * sequence position; poss_prefill draws x_P with u[0].  The walk then descends where a child
 * carries the drawn token, so every committed token is an exact sample of the target given its
 * prefix.  u: HOST, n_u values (1..depth+1; deeper levels reuse the last); copied before the call
 * returns; it stays in force until the next call.  temperature == 0 restores greedy verification
 * (u ignored).  Statistics count accepted draft tokens as before. */
int poss_set_sampling(poss_ctx *ctx, float temperature, const float *u, int32_t n_u);
/* The rejection-sampling rule proper at a temperature (section 2.1 names the step; this is the second reading of
 * it): with enable != 0, and a temperature set by poss_set_sampling, poss_draft_tree DRAWS the top_k children of
 * every expanded node from the drafter's softmax(logits / temperature), one after the other without replacement
 * (inverse CDF in vocabulary order over what is left), child i of the node of frontier rank r at depth d with
 * u_draft[((d - 1) * top_k + r) * top_k + i], and scores them with their log-probability; poss_verify_tree
 * (drafted tree only) tests the children of the current node in the order drawn, child i at a node of depth d
 * with u_accept[d * (top_k + 1) + i] against min(1, p / q) - p the target's, q the drafter's probability,
 * after a rejection p becomes the normalised positive part of p - q and q loses the candidate - and ends the
 * walk with a token drawn from the last residual (u_accept[d * (top_k + 1) + top_k]), with an accepted child that
 * the tree had dropped, or at a node without drawn children with a token drawn from the target's distribution.
 * That last token takes the bonus token's place in poss_accept_and_commit; every committed token is
 * distributed as the target's softmax(logits / temperature) given its prefix.  argmax_out of poss_verify_tree
 * then holds, for the nodes of the accepted path, the token that follows them, and -1 elsewhere.
 * u_draft: HOST float32 [depth][top_k][top_k]; u_accept: HOST float32 [depth + 1][top_k + 1]; all in [0, 1);
 * copied before the call returns, in force until the next call.  One sequence per context.  enable == 0:
 * back to the deterministic tree and the inverse-CDF coupling of poss_set_sampling. */
int poss_set_draft_sampling(poss_ctx *ctx, int32_t enable, const float *u_draft, const float *u_accept);
/* With batch > 1 poss_set_sampling gives every sequence the same numbers; this call gives sequence
 * seq its own (same rules for u and n_u; the temperature is the context's). */
int poss_set_uniforms_seq(poss_ctx *ctx, int32_t seq, const float *u, int32_t n_u);

/* Waits for queued work, then copies the statistics. */
int poss_get_stats(poss_ctx *ctx, poss_stats *out);
/* Number of committed tokens (prompt included); tokens_out (HOST, may be NULL) of capacity cap. */
int poss_get_tokens(poss_ctx *ctx, int32_t *tokens_out, int32_t cap, int32_t *n_out);
int poss_get_tokens_seq(poss_ctx *ctx, int32_t seq, int32_t *tokens_out, int32_t cap, int32_t *n_out);
const char *poss_last_error(poss_ctx *ctx);       /* ctx may be NULL: last poss_load error */
void poss_free(poss_ctx *ctx);

/* ---- instrumentation -------------------------------------------------------------------- */

/* Per-kernel timing of the weight-streaming GEMM (the kernel that carries the round's bytes).
 * enable != 0: every launch carries a pair of HIP events that take the kernel's begin and end
 * timestamps (slows the round slightly: use a pass of its own).  poss_gemm_profile sums the launches since the last call:
 * count, milliseconds, and algorithmic bytes (each launch's weight matrix once, in storage
 * dtype). */
int poss_profile_gemm(poss_ctx *ctx, int32_t enable);
int poss_gemm_profile(poss_ctx *ctx, int64_t *launches, double *ms, double *weight_bytes);

/* Tuning knobs for sweeps: target number of workgroups per GEMM launch (0 = default). */
int poss_set_tuning(poss_ctx *ctx, int32_t gemm_target_workgroups, int32_t attn_keys_per_split);

/* Rows that one launch of a batch's pass carries at most (POSS_MAX_ROWS .. POSS_LAUNCH_ROWS, default the latter): the
 * sequences of a pass are grouped so that a group's rows fit.  A sequence's results do not depend on it; lower values
 * re-stream the weights more often (for sweeps of that cost). */
int poss_set_launch_rows(poss_ctx *ctx, int32_t rows);

/* ---- test hooks (same kernels, inputs injected) ----------------------------------------- */

/* Tree builder alone: ids/logp are HOST arrays [depth][top_k][top_k]: for the pass at depth
 * d (0-based index d-1) and frontier row r, the top_k child tokens in rank order and their
 * float32 log-probabilities (at depth 1 only row 0 is read).  Needs a prefilled context (for
 * t); does not touch the drafter caches. */
int poss_debug_build_tree(poss_ctx *ctx, const int32_t *ids, const float *logp, poss_tree *out);

/* Copy target residual streams of the last target pass: DEVICE float32
 * [n_layers + 1][rows][d_model] (entry l = input of layer l; last = features). */
int poss_debug_set_taps(poss_ctx *ctx, void *taps_dev_or_null);

/* With drawn children (poss_set_draft_sampling), after poss_draft_tree: the drafter's logits of the expanded nodes
 * row0 .. row0+n-1 (row 0: the root; row 1 + (d-1) * top_k + r: the frontier node of rank r at depth d) into out,
 * DEVICE float32 [n][vocab]: the distributions the children were drawn from.  Waits for the stream. */
int poss_debug_draft_logits(poss_ctx *ctx, int32_t row0, int32_t n, float *out);

/* Read keys/values of logical slots [slot0, slot0+n) of one cache into HOST float32 arrays
 * [n][n_kv_heads][head_dim].  which = -1: target layer `layer`; which = s >= 0: specialist s. */
int poss_debug_read_kv(poss_ctx *ctx, int32_t which, int32_t layer, int32_t slot0, int32_t n,
                       float *k_out, float *v_out);

/* Y[M, N] (DEVICE float32) = X[M, K] . W[N, K]^T through the library's GEMM path; X and W DEVICE
 * row-major of `dtype`, M <= POSS_LAUNCH_ROWS (up to 128 rows the stream kernel, above it the tall kernel);
 * scratch DEVICE of at least poss_debug_gemm_scratch_bytes bytes (0 for a shape that is refused). */
size_t poss_debug_gemm_scratch_bytes(int32_t dtype, int32_t M, int32_t N, int32_t K);
int poss_debug_gemm(int32_t dtype, const void *x, const void *w, void *y, int32_t M, int32_t N,
                    int32_t K, int32_t target_workgroups, void *scratch, void *hip_stream,
                    int32_t repeats, float *ms_per_launch_out);

/* ---- for callers that cannot allocate ------------------------------------------------------ */

/* poss_debug_gemm for callers that may not allocate device memory or hand over a scratch buffer:
 * code under HIP graph capture, serving loops and harnesses that forbid hipMalloc.  Same kernels,
 * same result (Y[M, N] DEVICE float32 = X[M, K] . W[N, K]^T, X and W DEVICE row-major of `dtype`,
 * M <= POSS_MAX_ROWS), but the repacked weights and the split-K partial planes live in a
 * POSS_GEMM_STATIC_BYTES array inside the library's device image (each GPU the library runs on holds
 * its own copy until the process ends).  The call allocates nothing, creates no events and does
 * not wait: it enqueues three kernels on hip_stream (NULL = default stream) and returns; Y is valid
 * once the stream has been waited for.  Shapes whose packed matrix
 * (N rounded up to 128) x (K rounded up to 256) x sizeof(dtype) plus planes
 * splits x 128 x (N rounded up to 128) x 4 exceed the array are refused with POSS_E_CAPACITY and
 * nothing is launched.  Every call on a GPU uses that GPU's one array, on whatever stream: calls
 * that overlap on one GPU race, the caller serialises them.  Nothing in the array has to start at
 * zero; a call overwrites all of it that it reads. */
#define POSS_GEMM_STATIC_BYTES (32u << 20)
int poss_gemm_static(int32_t dtype, const void *x, const void *w, void *y, int32_t M, int32_t N,
                     int32_t K, int32_t target_workgroups, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* POSS_H */
