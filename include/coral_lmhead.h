/*
 * coral_lmhead.h -- C ABI of the weight-grouped LM head for a speculative-decoding
 * draft model on AMD MI355X (gfx950).
 *
 * The operation is the "LM head router" of the paper's section 3.3: the LM head
 * weight [V,H] is divided into G groups of vocabulary rows; per draft token a
 * router scores the groups, the g best groups are activated, logits are computed
 * over the rows of those groups only, and the k best candidates per token are
 * handed to tree expansion (appendix "Discussion on LM Head Router", paragraph
 * "Tree decoding").  The dense head (every row a candidate, the "N/A" row of the
 * router ablation, Table 4) is exported beside it for comparison.
 *
 * Conventions for every entry point
 *   - Pointers marked [device] are HIP device memory, [host] ordinary host memory.
 *   - All matrices are row-major and dense (no padding between rows).
 *   - Ownership: the caller owns every buffer.  The library allocates nothing on the
 *     device and frees nothing; inputs are only read.  The only state it keeps between
 *     calls is a per-device cache of two device properties (the number of compute units,
 *     and which kernels have been granted how much dynamic LDS), guarded by a mutex.
 *   - Execution: work is enqueued on `hip_stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and the call returns without
 *     synchronising.  Outputs are valid once the stream reaches that point.
 *   - Errors: every argument check is done on the host before anything is
 *     enqueued; a call that returns an argument error (any status but CORAL_OK and
 *     CORAL_ERR_HIP) has enqueued nothing.  No exceptions cross the boundary.
 *   - Limits (reported as CORAL_ERR_UNSUPPORTED, never silently mishandled):
 *     1 <= M <= 64, 1 <= k <= 64, 1 <= G <= 1024; H a multiple of 8 (bf16) or
 *     of 4 (f32); hidden, gate_W and lm_W 16-byte aligned.
 *   - NaN inputs give unspecified results.
 */
#ifndef CORAL_LMHEAD_H
#define CORAL_LMHEAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CORAL_OK = 0,
    CORAL_ERR_NULL = 1,          /* a required pointer is NULL                       */
    CORAL_ERR_SHAPE = 2,         /* a size is out of range or inconsistent           */
    CORAL_ERR_GROUP_INDEX = 3,   /* the group index is not a partition of 0..V-1     */
    CORAL_ERR_UNSUPPORTED = 4,   /* valid request outside the kernels' stated limits */
    CORAL_ERR_WORKSPACE = 5,     /* workspace missing, misaligned or too small       */
    CORAL_ERR_HIP = 6            /* the HIP runtime refused a launch                 */
} coral_status;

/* Storage type of hidden, gate_W and lm_W (all three share it): fp32, bf16, or IEEE
 * fp16 (the type the appendix paragraph "Backends" measures).  Products are accumulated
 * in fp32 for all; outputs are always fp32 logits and int32 ids. */
typedef enum {
    CORAL_F32 = 0,
    CORAL_BF16 = 1,
    CORAL_F16 = 2
} coral_dtype;

/*
 * Partition of the vocabulary into G groups (section 3.3 divides the LM head into N
 * groups of equal size; here any partition in CSR form, the equal contiguous split
 * being one case).  Group n owns vocabulary rows
 *     group_rows[group_offsets[n] .. group_offsets[n+1])
 * The struct itself is host memory.  The offsets are needed on both sides: the
 * host copy sizes the launch, the device copy is read by the kernels; the two
 * must hold the same values.
 */
typedef struct {
    int32_t G;                          /* number of groups (paper's N)               */
    const int32_t *group_offsets_host;  /* [host]   [G+1], [0] = 0, [G] = V, ascending */
    const int32_t *group_offsets;       /* [device] [G+1], same values                */
    const int32_t *group_rows;          /* [device] [V], a permutation of 0..V-1      */
} coral_group_index;

/* Human-readable name of a status code; never NULL. */
const char *coral_status_string(coral_status st);

/*
 * Host-side check that (offsets, rows) is a partition of 0..V-1 into G groups
 * (section 3.3).  Both arrays are [host].  Off the hot path: O(V) time and V
 * bytes of temporary host memory (the only allocation the library ever makes).
 * Returns CORAL_OK, CORAL_ERR_NULL, CORAL_ERR_SHAPE or CORAL_ERR_GROUP_INDEX.
 */
coral_status coral_group_index_validate(const int32_t *host_offsets,
                                        const int32_t *host_rows, int G, int V);

/*
 * Bytes of device workspace that coral_lmhead_grouped / coral_lmhead_dense need
 * for these sizes (pass G = g = 0 for the dense head).  The bound holds for any
 * partition of V rows into G groups.  Returns 0 if the sizes are invalid.
 */
size_t coral_lmhead_workspace_bytes(int M, int H, int V, int G, int g, int k,
                                    coral_dtype dt);

/*
 * Which kernels a call with these sizes will use (dense != 0: coral_lmhead_dense):
 * 0 = staged general path (one launch per stage), 1 = single-launch path (gate,
 * selection, row streaming and top-k of section 3.3 in one persistent kernel),
 * 2 = matrix-core tile path (bf16, H a multiple of 512, weights below 4 GiB: groups
 * shared by many tokens, the appendix's tree-decoding case, when the hidden vectors do
 * not fit on chip; dense head with 8 or more tokens and at least 65536 rows),
 * -1 = sizes not supported (outside the limits above, or a shape only the staged path
 * could take whose token batch does not fit LDS: rows beyond about 10 000 values with 8 or
 * more tokens).  Host-only, no device work; for tests and benchmark reports.
 */
int coral_lmhead_path(int dense, int M, int H, int V, int G, int g, int k, coral_dtype dt);

/*
 * The same for coral_lmhead_grouped_logprob (Eq. 8's output): 1 = single-launch kernel
 * (at most 64 activated groups, min(M*g, G) <= 64, g <= 16, and its LDS plan fits),
 * 2 = matrix-core tile path (where that path's conditions hold and G <= 64),
 * 0 = staged path, -1 = sizes not supported.  Host-only.
 */
int coral_lmhead_logprob_path(int M, int H, int V, int G, int g, int k, coral_dtype dt);

/*
 * Prepares a freshly allocated workspace: zeroes its control words (a small kernel
 * on hip_stream, no memset node, so it may be captured in a HIP graph).  Required
 * once before the first coral_lmhead_grouped / coral_lmhead_dense call that uses the
 * workspace; every completed call leaves the control words ready for the next one.
 * The control words count the workgroups that have published their partial top-k
 * lists, so that the last one can merge them (the per-token top-k of the appendix's
 * "Tree decoding" paragraph) without a further launch, and hand out blocks of weight
 * rows to the workgroups of the tile path.  A call that fails with CORAL_ERR_HIP may
 * leave them non-zero: prepare the workspace again before reusing it.
 *   workspace [device], 256-byte aligned, at least 256 bytes.
 */
coral_status coral_lmhead_workspace_init(void *workspace, size_t workspace_bytes,
                                         void *hip_stream);

/*
 * Grouped LM head for one draft step (section 3.3, Eq. 7 and Eq. 8; appendix
 * "Tree decoding").  For each token m = 0..M-1:
 *   s[m,n]   = sum_j gate_W[n,j] * hidden[m,j] (+ gate_bias[n])      n = 0..G-1
 *              (the W2 projection of the router; the softmax of Eq. 7 is
 *              monotone, so selection is taken on s)
 *   sel[m,:] = the g groups with the largest s[m,.], best first; equal scores:
 *              lower group id first
 *   z[m,r]   = sum_j lm_W[r,j] * hidden[m,j]   for the rows r of sel[m,:] only
 *   output   = the k largest z[m,.] among those rows, best first; equal logits:
 *              lower vocabulary id first
 * Weight rows of a group selected by several tokens are read once for all of
 * them.  The logits row is never written to memory; on the tile path (see
 * coral_lmhead_path) the logits of the activated rows, for the tokens that
 * selected them, pass through the workspace between that path's kernels.
 *
 *   hidden      [device] [M,H]  draft hidden states
 *   gate_W      [device] [G,H]  router projection (paper's W2)
 *   gate_bias   [device] [G] fp32, or NULL for none
 *   lm_W        [device] [V,H]  LM head weight
 *   gi          [host]   partition, see coral_group_index
 *   M,H,V       sizes; g active groups per token (1..G); k candidates per token
 *               (1..64, and at most g times the smallest group's row count)
 *   topk_ids    [device] out [M,k] int32 vocabulary ids
 *   topk_logits [device] out [M,k] fp32 logits of those ids
 *   sel_groups  [device] out [M,g] int32 selected groups, or NULL if not wanted
 *   workspace   [device] at least coral_lmhead_workspace_bytes(...) bytes,
 *               256-byte aligned, prepared once by coral_lmhead_workspace_init;
 *               two calls in flight at once must not share it
 */
coral_status coral_lmhead_grouped(const void *hidden, const void *gate_W,
                                  const float *gate_bias, const void *lm_W,
                                  const coral_group_index *gi, int M, int H, int V,
                                  int g, int k, coral_dtype dt, int32_t *topk_ids,
                                  float *topk_logits, int32_t *sel_groups,
                                  void *workspace, size_t workspace_bytes,
                                  void *hip_stream);

/*
 * coral_lmhead_grouped for callers that cannot allocate device memory or pass a workspace
 * along: code under HIP graph capture, tight serving loops, harnesses that forbid
 * allocation.  Same operation, arguments, results (bit for bit) and errors as
 * coral_lmhead_grouped, with no workspace argument: the kernels' scratch (published partial
 * lists, arrival counters, the staged path's hand-over arrays) lives in a static device array
 * of CORAL_NOALLOC_SCRATCH_BYTES inside the library, one copy per GPU, held until the
 * process ends.  The call allocates and frees nothing.
 *   - Shapes whose scratch need (coral_lmhead_workspace_bytes for the same sizes, without the
 *     log-probability mode's tables) exceeds CORAL_NOALLOC_SCRATCH_BYTES are refused with
 *     CORAL_ERR_WORKSPACE before anything is enqueued.  Every workload shape of Table 1 with up
 *     to 16 tokens fits.
 *   - All calls on one GPU share that GPU's array: calls that overlap on one GPU (two
 *     streams, two threads) race and give unspecified results; calls on one stream, or
 *     otherwise ordered, are safe.  Each call first clears the array's control words with a
 *     small kernel on hip_stream (no memset node), so it may be captured and replayed.
 *   - The first call on a device looks the array's address up (hipGetSymbolAddress); it may
 *     fail with CORAL_ERR_HIP if no device is current.
 */
#define CORAL_NOALLOC_SCRATCH_BYTES (8u << 20)

coral_status coral_lmhead_grouped_noalloc(const void *hidden, const void *gate_W,
                                          const float *gate_bias, const void *lm_W,
                                          const coral_group_index *gi, int M, int H, int V,
                                          int g, int k, coral_dtype dt, int32_t *topk_ids,
                                          float *topk_logits, int32_t *sel_groups,
                                          void *hip_stream);

/*
 * Grouped LM head with the paper's probability composition (section 3.3, Eq. 7 and
 * Eq. 8).  Selection and logits as in coral_lmhead_grouped; then for each token m and
 * each row x of a selected group n
 *   log p(x) = log p_router(n) + z[m,x] - lse(m,n)
 *   log p_router(n) = s[m,n] - log sum_{n'=0..G-1} exp(s[m,n'])     (softmax over all groups)
 *   lse(m,n)        = log sum_{r in group n} exp(z[m,r])            (softmax inside the group)
 * and the output is the k rows with the largest log p(x) among the token's g groups,
 * best first (equal values: lower vocabulary id first).  The order can differ from
 * coral_lmhead_grouped's, which ranks the raw logits across groups.  Rows outside the
 * selected groups have probability zero (Eq. 8) and are never returned.
 *   topk_logprob [device] out [M,k] fp32 log-probabilities (natural logarithm)
 * All other arguments, limits and errors as for coral_lmhead_grouped.  Runs in the
 * single-launch kernel, on the tile path or on the staged path (coral_lmhead_logprob_path
 * tells which).
 */
coral_status coral_lmhead_grouped_logprob(const void *hidden, const void *gate_W,
                                          const float *gate_bias, const void *lm_W,
                                          const coral_group_index *gi, int M, int H,
                                          int V, int g, int k, coral_dtype dt,
                                          int32_t *topk_ids, float *topk_logprob,
                                          int32_t *sel_groups, void *workspace,
                                          size_t workspace_bytes, void *hip_stream);

/*
 * The router's inner term (section 3.3, Eq. 7): u[m,:] = act(W1 hidden[m,:]) + hidden[m,:]
 * for every token, W1 [H,H] row-major with one row per output feature
 * (y[i] = sum_j W1[i,j] hidden[m,j]).  The paper does not name act; CORAL_ACT_SILU is this
 * library's default reading, the others are there to compare.  Sums in fp32; u is written in
 * the storage type dt (bf16: round to nearest even).
 *   hidden [device] [M,H]; W1 [device] [H,H]; u_out [device] out [M,H], must not overlap
 *   hidden.  All 16-byte aligned; H a multiple of 8 (bf16, fp16) / 4 (fp32), H * element size
 *   at most 160 KB.  Needs no workspace.
 */
typedef enum {
    CORAL_ACT_SILU = 0,
    CORAL_ACT_RELU = 1,
    CORAL_ACT_IDENTITY = 2
} coral_activation;

coral_status coral_router_premix(const void *hidden, const void *W1, int M, int H,
                                 coral_dtype dt, coral_activation act, void *u_out,
                                 void *hip_stream);

/*
 * Grouped LM head whose router sees another vector than the LM head (section 3.3, Eq. 7:
 * p_router = Softmax(W2 (act(W1 h) + h)), while the logits of Eq. 8's p_group come from h):
 *   s[m,n] = sum_j gate_W[n,j] * gate_hidden[m,j] (+ gate_bias[n]),  z from hidden.
 * gate_hidden [device] [M,H] is typically coral_router_premix's output; NULL means hidden.
 * logprob = 0: output as coral_lmhead_grouped (k best logits); logprob != 0: output as
 * coral_lmhead_grouped_logprob (k best log p(x), p_router from the scores above).
 * All other arguments, limits and errors as for those two calls.
 */
coral_status coral_lmhead_grouped_routed(const void *hidden, const void *gate_hidden,
                                         const void *gate_W, const float *gate_bias,
                                         const void *lm_W, const coral_group_index *gi,
                                         int M, int H, int V, int g, int k, coral_dtype dt,
                                         int logprob, int32_t *topk_ids, float *topk_out,
                                         int32_t *sel_groups, void *workspace,
                                         size_t workspace_bytes, void *hip_stream);

/*
 * One level of draft-tree expansion (tree drafting of section 2.1 with the per-level node
 * budget of section 4.1, "Implementation"; the paper takes the rule from the dynamic draft
 * tree it builds on and does not restate it, so this is a reading): node m of the current
 * level carries the cumulative log-probability parent_score[m]; candidate i of node m has
 * score = parent_score[m] + cand_logp[m,i] (one fp32 addition); the n_next best scores of
 * all M*k candidates form the next level, best first; equal scores: lower m, then lower i.
 *   parent_score [device] [M] fp32, or NULL for all zero (the root level)
 *   cand_ids     [device] [M,k] int32 token ids, e.g. coral_lmhead_grouped_logprob's
 *                topk_ids; a negative id marks an empty slot
 *   cand_logp    [device] [M,k] fp32, each row non-increasing (as the heads return it)
 *   next_parent  [device] out [n_next] int32: index m of the parent node
 *   next_token   [device] out [n_next] int32: the candidate's token id
 *   next_score   [device] out [n_next] fp32: its cumulative score
 *   Slots beyond the number of candidates hold (-1, -1, -inf).
 * Limits: 1 <= M <= 64, 1 <= k <= 64, 1 <= n_next <= M*k.  Needs no workspace.
 */
coral_status coral_tree_expand(const float *parent_score, const int32_t *cand_ids,
                               const float *cand_logp, int M, int k, int n_next,
                               int32_t *next_parent, int32_t *next_token,
                               float *next_score, void *hip_stream);

/*
 * One level of tree drafting in one call: the log-probability head of section 3.3 (Eq. 7,
 * Eq. 8; arguments as coral_lmhead_grouped_routed with logprob != 0, gate_hidden may be
 * NULL) for the M nodes of the current level, then coral_tree_expand on its own output
 * (cand_ids = topk_ids, cand_logp = topk_logprob).  Where the head runs in the single-launch
 * kernel (coral_lmhead_logprob_path == 1) the workgroup that writes the head's result also
 * expands the level, so the call is one launch; otherwise the expansion is one more launch
 * behind those of the tile or staged path.  Results are identical to the two calls made one
 * after the other.
 *   parent_score [device] [M] fp32 or NULL, n_next, next_parent / next_token / next_score
 *   [device] out [n_next]: as for coral_tree_expand.  topk_ids, topk_logprob, sel_groups:
 *   as for coral_lmhead_grouped_logprob (they are written as well).
 * Errors as for the two calls.
 */
coral_status coral_lmhead_draft_level(const void *hidden, const void *gate_hidden,
                                      const void *gate_W, const float *gate_bias,
                                      const void *lm_W, const coral_group_index *gi,
                                      int M, int H, int V, int g, int k, coral_dtype dt,
                                      const float *parent_score, int n_next,
                                      int32_t *topk_ids, float *topk_logprob,
                                      int32_t *sel_groups, int32_t *next_parent,
                                      int32_t *next_token, float *next_score,
                                      void *workspace, size_t workspace_bytes,
                                      void *hip_stream);

/*
 * Dense LM head: z[m,r] for every r = 0..V-1, then the k best per token with the
 * same ordering rules (the no-router baseline of Table 4; the head whose latency
 * the appendix paragraph "Backends" measures).  Arguments as above; k <= V.
 */
coral_status coral_lmhead_dense(const void *hidden, const void *lm_W, int M, int H,
                                int V, int k, coral_dtype dt, int32_t *topk_ids,
                                float *topk_logits, void *workspace,
                                size_t workspace_bytes, void *hip_stream);

/*
 * Measurement variants: identical to coral_lmhead_grouped / coral_lmhead_grouped_logprob /
 * coral_lmhead_dense (same operation of section 3.3, same arguments, same results), and in addition
 * bind two caller-created HIP events (hipEvent_t passed as void*, created with
 * timing enabled) to the launch of the kernel that streams the LM-head weight rows,
 * which is where the appendix paragraph "Backends" locates the head's time: ev_before
 * takes the time at which that kernel starts, ev_after the time at which it ends.
 * hipEventElapsedTime(ev_before, ev_after) after synchronisation gives that
 * kernel's duration, as a kernel trace reports it (no dispatch latency, no gap to the
 * neighbouring launches).  Both events are required (CORAL_ERR_NULL otherwise).  Not for
 * use under stream capture.
 */
coral_status coral_lmhead_grouped_profiled(const void *hidden, const void *gate_W,
                                           const float *gate_bias, const void *lm_W,
                                           const coral_group_index *gi, int M, int H,
                                           int V, int g, int k, coral_dtype dt,
                                           int32_t *topk_ids, float *topk_logits,
                                           int32_t *sel_groups, void *workspace,
                                           size_t workspace_bytes, void *hip_stream,
                                           void *ev_before, void *ev_after);

coral_status coral_lmhead_grouped_logprob_profiled(
    const void *hidden, const void *gate_W, const float *gate_bias, const void *lm_W,
    const coral_group_index *gi, int M, int H, int V, int g, int k, coral_dtype dt,
    int32_t *topk_ids, float *topk_logprob, int32_t *sel_groups, void *workspace,
    size_t workspace_bytes, void *hip_stream, void *ev_before, void *ev_after);

coral_status coral_lmhead_dense_profiled(const void *hidden, const void *lm_W, int M,
                                         int H, int V, int k, coral_dtype dt,
                                         int32_t *topk_ids, float *topk_logits,
                                         void *workspace, size_t workspace_bytes,
                                         void *hip_stream, void *ev_before,
                                         void *ev_after);

/*
 * Measurement aid, no part of the method: a kernel that only reads, in the launch shape of
 * the single-launch path (one workgroup per compute unit, `waves` waves of 64 lanes each,
 * 1..16; every wave takes 16 KB pieces of src, dealt round robin, 16 loads of 1 KB in flight
 * per piece, non-temporal like the weight rows).  What it takes for as many bytes as a step
 * of section 3.3 must move is the yardstick the bench line's figures are held against.
 *   src   [device] at least `bytes` bytes, 16-byte aligned; read once, nothing is written
 *   bytes a multiple of 16384
 *   ev_before, ev_after  as for the *_profiled entry points (both required)
 * Returns CORAL_OK, CORAL_ERR_NULL, CORAL_ERR_SHAPE, CORAL_ERR_UNSUPPORTED or CORAL_ERR_HIP.
 */
coral_status coral_probe_read(const void *src, size_t bytes, int waves, void *hip_stream,
                              void *ev_before, void *ev_after);

#ifdef __cplusplus
}
#endif
#endif /* CORAL_LMHEAD_H */
