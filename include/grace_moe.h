/*
 * grace_moe.h - C ABI of the MI355X (gfx950) GRACE-MoE layer hot path.
 *
 * One GPU's share of one Mixture-of-Experts layer as reorganised by GRACE-MoE
 * (arxiv 2509.25041): top-k gating, locality-aware replica selection against an
 * expert placement / replica table, the node-then-GPU dispatch permutation, the
 * grouped SwiGLU expert FFN over the rows routed to this GPU, and the weighted
 * combine back to token order.
 *
 * Conventions
 *  - Every function returns a status: GRACE_OK (0) or a negative error code.
 *    Nothing throws, aborts or prints.  grace_last_error() gives the text of the
 *    calling thread's most recent failure.
 *  - Pointers marked HOST are read during the call and not retained.
 *    Pointers marked DEVICE belong to the caller; the library borrows them until
 *    the work it enqueued on `stream` has completed.  Compute calls are
 *    asynchronous on `stream` (a hipStream_t passed as void*; NULL = the default
 *    stream) and never synchronise the device.
 *  - Shapes and ranges are checked on the host before anything is launched.
 *    Values held in device memory (logits, ids) are the caller's precondition:
 *    logits must be finite, ids in range.  Out-of-range ids never cause an
 *    out-of-bounds access; the affected outputs are unspecified.
 *  - All matrices are dense row-major.  Index arrays are int32.
 *  - Assignment index a = t*k + j (token t, j-th chosen expert).
 *  - An "instance" is one copy of an expert on one rank.  Instance ids are
 *    positions in the dispatch order: all instances sorted by
 *    (node of rank, rank, expert id).  The instances of one rank are therefore
 *    consecutive ids; the position of an instance among its rank's instances is
 *    its "slot", which is also the index of its weights in the stacked weight
 *    arrays passed to grace_expert_ffn.
 */
#ifndef GRACE_MOE_H
#define GRACE_MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    GRACE_OK = 0,
    GRACE_EINVAL = -1, /* null pointer, negative size, value out of range           */
    GRACE_ESHAPE = -2, /* shape not supported (limits below) or not matching table */
    GRACE_ETABLE = -3, /* malformed placement table                                 */
    GRACE_ENOMEM = -4, /* host or device allocation failed                          */
    GRACE_EHIP = -5    /* HIP runtime error (text in grace_last_error)              */
};

typedef enum { GRACE_F32 = 0, GRACE_BF16 = 1 } grace_dtype;

/* Replica selection policy (Section 4.3 of the paper describes both). */
typedef enum {
    GRACE_POLICY_TAR = 0, /* topology-aware routing with locality preference (Algorithm 4)            */
    GRACE_POLICY_WRR = 1  /* weighted round-robin over all instances, no locality (Algorithm 3 alone) */
} grace_policy;

/* Limits checked by the entry points. */
#define GRACE_MAX_EXPERTS 256   /* E                        */
#define GRACE_MAX_TOPK 64       /* k                        */
#define GRACE_MAX_RANKS 1024    /* R                        */
#define GRACE_MAX_INSTANCES 4096 /* I                       */
#define GRACE_MAX_POLL_WEIGHT 65535u
#define GRACE_STATIC_SCRATCH_BYTES (4u << 20) /* scratch of grace_route_permute_static, per GPU */
#define GRACE_SHARE_STATE_INTS 8 /* size of the state of grace_expert_ffn_up_share / _down_share */

typedef struct grace_table grace_table; /* opaque; owns host and device copies */

/* ---- placement / replica table (Sections 4.1-4.3 of the paper) -------------
 * The output of the paper's offline phase, given purely as data: the virtual
 * topology (rank -> node), the per-GPU polling weights of the weighted
 * round-robin (Section 4.3, Algorithm 3: map gpu_id -> weight) and, in CSR form
 * over experts, the ranks holding an instance of each expert (primary group
 * member or replica; Section 4.2 - the routing treats all instances alike).
 *
 * All pointers HOST.
 *   E, R, N      experts, ranks (virtual GPUs), nodes
 *   rank_node    [R]   node of each rank, values in [0, N), non-decreasing
 *   poll_weight  [R]   integer polling weight, 1 .. GRACE_MAX_POLL_WEIGHT
 *   inst_ptr     [E+1] instances of expert e are inst_rank[inst_ptr[e] .. inst_ptr[e+1])
 *   inst_rank    [I]   hosting rank, strictly ascending within one expert
 * Errors: GRACE_EINVAL (null, sizes < 1), GRACE_ESHAPE (over the limits),
 * GRACE_ETABLE (expert without instance, rank out of range, duplicate or
 * unsorted (expert, rank), zero or oversized weight, decreasing rank_node,
 * node id out of range, inst_ptr not starting at 0 or decreasing).
 */
int grace_table_validate(int32_t E, int32_t R, int32_t N, const int32_t *rank_node,
                         const uint32_t *poll_weight, const int32_t *inst_ptr, const int32_t *inst_rank);

/* Validates as above, then builds the table on the current HIP device
 * (device copy made on `stream`, complete on return).  *out is set only on
 * success and must be released with grace_table_destroy. */
int grace_table_create(grace_table **out, int32_t E, int32_t R, int32_t N, const int32_t *rank_node,
                       const uint32_t *poll_weight, const int32_t *inst_ptr, const int32_t *inst_rank,
                       void *stream);
int grace_table_destroy(grace_table *table); /* NULL is accepted */

/* Sizes of a table.  Any output pointer may be NULL. */
int grace_table_info(const grace_table *table, int32_t *E, int32_t *R, int32_t *N, int32_t *I,
                     int32_t *max_local_slots);

/* The dispatch order (Section 5: first by target node, then by target GPU).
 * HOST outputs, any may be NULL: inst_expert [I], inst_rank [I] for each
 * instance id; rank_ptr [R+1]: the instances of rank r are ids
 * rank_ptr[r] .. rank_ptr[r+1]. */
int grace_table_instances(const grace_table *table, int32_t *inst_expert, int32_t *inst_rank, int32_t *rank_ptr);

/* Experts hosted by `rank` in slot order (ascending expert id): tells the
 * caller how to stack the weights for grace_expert_ffn.  HOST outputs;
 * experts_out must hold max_local_slots entries. */
int grace_table_local_experts(const grace_table *table, int32_t rank, int32_t *experts_out, int32_t *n_out);

/* Tuning of one table: where the routing and permutation index kernels of calls made with it switch
 * algorithm.  They turn per-chunk histograms (chunks of 16 or 32 tokens in grace_route, of 512
 * assignments in grace_permute and grace_send_lists) into prefix counts: up to one_level_max
 * histogram loads per column of 64 keys (chunks * ceil(keys / 64)) every block sums the rows before
 * its own chunk; up to two_level_max loads (of super-chunk sums of 64 rows plus the rows of the own
 * super-chunk) it uses those two-level sums, one more launch; beyond that, single-block scan
 * kernels.  Results are identical on every path.  A negative value restores the default (1024,
 * 8192).  Affects calls made with this table afterwards; not to be changed while another thread
 * is inside a call with the same table.  Errors: GRACE_EINVAL (null table). */
int grace_table_set_fold_limits(grace_table *table, int32_t one_level_max, int32_t two_level_max);

/* Bytes of device scratch that any single call below needs for these sizes
 * (the same buffer may be reused by consecutive calls on one stream).
 * f and n_shared may be 0 when the FFN entry points are not used.  Returns 0
 * on invalid arguments.  The buffer must be 256-byte aligned. */
size_t grace_workspace_bytes(int32_t T, int32_t E, int32_t k, int32_t I, int32_t d, int32_t f, int32_t n_shared,
                             grace_dtype dt);

/* ---- grace_route: top-k gating + replica pick -------------------------------
 * Gating (Section 3: every token activates k experts): the k largest logits of
 * a token, in descending order, equal logits to the lower expert id; gate
 * weight = softmax over all E logits, divided by the sum over the k chosen when
 * renorm != 0.  -0.0 equals +0.0; a logit of -infinity masks an expert: it
 * ranks behind every finite logit and its weight is exactly 0 (a token needs
 * at least one finite logit; NaN and +infinity are not defined inputs).
 * Replica pick (Section 4.3; Algorithm 4 with Algorithm 3 inside a tier): all
 * T tokens reside on local_rank.  For each assignment, in order of a, the c-th
 * request for expert e (c starts at rr_in[e]) goes to
 *   the instance on local_rank, if there is one; else
 *   among the instances on local_rank's node, if any; else among all instances,
 * the candidate (ascending rank) whose cumulative polling-weight interval
 * contains c mod W, W = sum of the tier's polling weights (deterministic
 * weighted round-robin: over any W consecutive requests each candidate receives
 * exactly its weight).  With GRACE_POLICY_WRR the candidate set is always "all
 * instances" (the paper's first policy, which balances load but ignores
 * locality); local_rank is then only range-checked.
 *
 * DEVICE: logits [T,E] fp32; rr_in [E] or NULL (= zeros); rr_out [E] or NULL,
 * receives (rr_in[e] + requests of e) mod W_e and must not overlap rr_in (the
 * kernels read rr_in while rr_out is written; GRACE_EINVAL); topk_expert [T,k];
 * topk_weight [T,k] fp32; topk_inst [T,k] instance ids; expert_count [E]
 * requests per expert in this call; ws from grace_workspace_bytes.
 * Limits: 1 <= k <= min(E, GRACE_MAX_TOPK), E == table's E, T*k < 2^31, T >= 0.
 */
int grace_route(const grace_table *table, int32_t local_rank, grace_policy policy, const float *logits, int32_t T, int32_t E, int32_t k,
                int32_t renorm, const uint32_t *rr_in, uint32_t *rr_out, int32_t *topk_expert, float *topk_weight,
                int32_t *topk_inst, int32_t *expert_count, void *ws, void *stream);

/* ---- grace_permute: hierarchical dispatch permutation -----------------------
 * Orders the T*k assignments by instance id, i.e. by (node, rank, slot) - the
 * order in which the two-stage dispatch of Section 5 forwards rows first to the
 * target node and then to the target GPU - keeping assignment order among equal
 * ids (a stable sort), and moves the token rows into that order.
 *
 * DEVICE: topk_inst [T*k]; x [T,d] rows of dtype dt, or NULL to build only the
 * index arrays (then xp is ignored); outputs perm_pos [T*k] (assignment ->
 * buffer position), perm_src [T*k] (buffer position -> assignment),
 * inst_off [I+1], rank_off [R+1], node_off [N+1] (exclusive row offsets of each
 * instance / rank / node; the last entry of each is T*k), xp [T*k,d] with
 * xp[p] = x[perm_src[p] / k].
 * Limits: d >= 1 and d * sizeof(dt) a multiple of 16 when x != NULL.
 */
int grace_permute(const grace_table *table, const int32_t *topk_inst, int32_t T, int32_t k, const void *x, int32_t d,
                  grace_dtype dt, int32_t *perm_pos, int32_t *perm_src, int32_t *inst_off, int32_t *rank_off,
                  int32_t *node_off, void *xp, void *ws, void *stream);

/* The row movement of grace_permute alone (Section 5: rows in dispatch order), for callers that
 * built the index arrays with x == NULL and move the rows later or on another stream:
 *     xp[perm_pos[t*k+j]] = x[t]   for every assignment whose perm_pos is in [0, T*k).
 * DEVICE: x [T,d]; perm_pos [T*k] from grace_permute / grace_route_permute; xp [T*k,d].
 * Limits as for grace_permute with x != NULL. */
int grace_permute_rows(const void *x, const int32_t *perm_pos, int32_t T, int32_t k, int32_t d, grace_dtype dt, void *xp,
                       void *stream);

/* ---- grace_route_permute: grace_route then grace_permute in one call ----------
 * Same arguments, outputs (bit for bit) and errors as grace_route (Section 3,
 * Section 4.3, Algorithms 3 and 4) followed by grace_permute (Section 5) on its
 * topk_inst, with fewer kernel launches.  Decode-sized batches, which are bound
 * by launch latency, are handled by the top-k kernel, one single-workgroup
 * kernel and the row scatter instead of five launches: that path is taken when
 * ceil(T / 16) * k <= 256, E <= 256 and the table has at most 256 instances.
 * For every other size the replica pick also produces the histograms the
 * permutation starts from, which saves one launch.  The workspace holds the
 * routing and the permutation histograms side by side during this call
 * (grace_workspace_bytes covers it).
 */
int grace_route_permute(const grace_table *table, int32_t local_rank, grace_policy policy, const float *logits, int32_t T,
                        int32_t E, int32_t k, int32_t renorm, const uint32_t *rr_in, uint32_t *rr_out,
                        int32_t *topk_expert, float *topk_weight, int32_t *topk_inst, int32_t *expert_count,
                        const void *x, int32_t d, grace_dtype dt, int32_t *perm_pos, int32_t *perm_src,
                        int32_t *inst_off, int32_t *rank_off, int32_t *node_off, void *xp, void *ws, void *stream);

/* ---- grace_route_permute_static: grace_route_permute without a workspace -------
 * For callers that cannot allocate device memory or hand one in: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus ws), outputs (bit
 * for bit) and errors as grace_route_permute; the index kernels' scratch is a static device array of
 * GRACE_STATIC_SCRATCH_BYTES that every GPU the library runs on holds from its first use until
 * the process ends.  The call allocates and frees nothing (no hipMalloc, no hipFree, no allocating
 * library routine); its first use on a device looks the array's address up once.
 * Limit: sizes whose histograms do not fit the array are rejected with GRACE_ESHAPE and a text
 * that says so (needed bytes = 16 * ceil(T / 16) * E + 8 * ceil(T * k / 512) * I, each term rounded
 * up to 256: e.g. T = 32768, E = 64, k = 6, I = 88 needs 2.3 MB; T = 100 000 with E = 128 does not
 * fit) - use grace_route_permute with a workspace then.
 * All calls on one GPU share that GPU's array: two calls that overlap in time on the same GPU (on
 * different streams or from different threads) race on it and must be serialised by the caller;
 * calls on one stream are ordered and safe.  Nothing in the array has to be zero on entry and a
 * call leaves its histograms behind.
 */
int grace_route_permute_static(const grace_table *table, int32_t local_rank, grace_policy policy, const float *logits,
                               int32_t T, int32_t E, int32_t k, int32_t renorm, const uint32_t *rr_in, uint32_t *rr_out,
                               int32_t *topk_expert, float *topk_weight, int32_t *topk_inst, int32_t *expert_count,
                               const void *x, int32_t d, grace_dtype dt, int32_t *perm_pos, int32_t *perm_src,
                               int32_t *inst_off, int32_t *rank_off, int32_t *node_off, void *xp, void *stream);

/* ---- grace_send_lists: de-duplicated hierarchical send lists ------------------
 * Section 5: a token with several experts on one destination crosses the link
 * to that destination a single time.  For the T tokens of local_rank and their instance ids
 * (from grace_route) this builds
 *   rank_send_ptr [R+1], rank_send_tok : for every destination rank the ascending list of
 *       distinct tokens with at least one assignment there (what stage 2 delivers to it);
 *   node_send_ptr [N+1], node_send_tok : the same per destination node (what stage 1 sends);
 *   expand [T*k] : for assignment a, the index of its token inside the send list of its
 *       destination rank, so the receiver can expand the unique rows to one row per
 *       assignment (row of assignment a = received row expand[a]);
 *   traffic [4] (int64, may be NULL) in tokens: [0] cross-node with de-duplication (sum over
 *       other nodes of their distinct tokens), [1] cross-node without (one row per assignment),
 *       [2] intra-node with de-duplication (distinct tokens for the other ranks of the own node,
 *       plus in every other node for the ranks other than the stage-1 peer, i.e. the rank with
 *       local_rank's index inside that node), [3] intra-node rows of a flat dispatch
 *       (assignments to the other ranks of the own node).
 * DEVICE: topk_inst [T*k]; the two token arrays and expand hold T*k entries (at most
 * T*min(k, R) resp. T*min(k, N) are written); ws from grace_workspace_bytes.
 * The dispatch permutation of grace_permute is unaffected (one row per assignment).
 */
int grace_send_lists(const grace_table *table, int32_t local_rank, const int32_t *topk_inst, int32_t T, int32_t k,
                     int32_t *rank_send_ptr, int32_t *rank_send_tok, int32_t *node_send_ptr, int32_t *node_send_tok,
                     int32_t *expand, int64_t *traffic, void *ws, void *stream);

/* ---- grace_expert_ffn: grouped SwiGLU FFN over one rank's rows ---------------
 * The expert computation between dispatch and aggregation (Section 1).  For
 * every instance i hosted by `rank` (slot s, expert e) and every buffer row p
 * in [inst_off[i], inst_off[i+1]):
 *     y[p] = W_down[s] ( silu(W_gate[s] xp[p]) * (W_up[s] xp[p]) ),
 *     silu(g) = g / (1 + exp(-g)),
 * with fp32 accumulation.  For GRACE_BF16 the hidden activation is rounded to
 * bf16 before the down projection and y is stored in bf16; GRACE_F32 stays fp32
 * end to end.  Rows of other ranks are not touched.
 *
 * DEVICE: xp [T*k,d]; inst_off [I+1] as written by grace_permute;
 * w_gate, w_up [S,f,d] and w_down [S,d,f], S = number of local slots, slot
 * order as given by grace_table_local_experts; every weight row holds one
 * output feature, contiguous over the input feature; y [T*k,d].
 * Limits: d and f multiples of 8 for GRACE_BF16.
 * `rank` is an argument (normally local_rank) so that a caller can evaluate
 * every virtual rank on one device.
 */
int grace_expert_ffn(const grace_table *table, int32_t rank, const void *xp, const int32_t *inst_off, int32_t T,
                     int32_t k, int32_t d, int32_t f, grace_dtype dt, const void *w_gate, const void *w_up,
                     const void *w_down, void *y, void *ws, void *stream);

/* The two launches of grace_expert_ffn as separate calls, for callers that
 * interleave other work between them or time them individually:
 * _up writes the hidden activation silu(W_gate xp) * (W_up xp) of the rank's
 * rows to ws ([T*k, f] of dt, row p at the same index as in xp); _down reads it
 * from ws and writes y.  grace_expert_ffn(...) == _up(...) then _down(...) with
 * the same ws.  Arguments and limits as for grace_expert_ffn. */
int grace_expert_ffn_up(const grace_table *table, int32_t rank, const void *xp, const int32_t *inst_off, int32_t T,
                        int32_t k, int32_t d, int32_t f, grace_dtype dt, const void *w_gate, const void *w_up,
                        void *ws, void *stream);
int grace_expert_ffn_down(const grace_table *table, int32_t rank, const int32_t *inst_off, int32_t T, int32_t k,
                          int32_t d, int32_t f, grace_dtype dt, const void *w_down, void *y, void *ws, void *stream);

/* grace_expert_ffn_up / _down that also keep y a rank share from step to step.  On one GPU only
 * the rows of `rank` are computed; the rows of other ranks, which the second all-to-all of
 * Section 1 would deliver, are defined as zero.  The rank's row range [inst_off[first instance of
 * rank], inst_off[last + 1]) moves with the routing, so a y buffer reused across steps would keep
 * results of an earlier range.  Called as a pair, once each per step and in this order on one
 * stream, _up_share records the step's range in `state` and _down_share zeroes, inside its own
 * launch, the rows that the previous step wrote and that lie outside the current range (no extra
 * launch, no memset, no atomics: the step stays capturable).
 * DEVICE: state: GRACE_SHARE_STATE_INTS int32 owned by the caller, all zero before the first step
 * (y zero-filled by the caller at that time), otherwise private to these two functions; one
 * state per y buffer.  Rows are cleared with 16-byte stores: d * sizeof(dt) must be a multiple of
 * 16.  When `rank` hosts no instance nothing is launched and y is never written.  Other arguments
 * as for grace_expert_ffn_up / grace_expert_ffn_down. */
int grace_expert_ffn_up_share(const grace_table *table, int32_t rank, const void *xp, const int32_t *inst_off, int32_t T,
                              int32_t k, int32_t d, int32_t f, grace_dtype dt, const void *w_gate, const void *w_up,
                              int32_t *state, void *ws, void *stream);
int grace_expert_ffn_down_share(const grace_table *table, int32_t rank, const int32_t *inst_off, int32_t T, int32_t k,
                                int32_t d, int32_t f, grace_dtype dt, const void *w_down, void *y, int32_t *state,
                                void *ws, void *stream);

/* Always-on shared experts evaluated on all T token rows and summed:
 *     y_shared[t] = sum_s W_down[s] ( silu(W_gate[s] x[t]) * (W_up[s] x[t]) ).
 * DEVICE: x [T,d]; w_gate, w_up [n_shared,f,d]; w_down [n_shared,d,f];
 * y_shared [T,d].  Same dtype rules and limits as grace_expert_ffn. */
int grace_shared_ffn(const void *x, int32_t T, int32_t d, int32_t f, int32_t n_shared, grace_dtype dt,
                     const void *w_gate, const void *w_up, const void *w_down, void *y_shared, void *ws,
                     void *stream);

/* The two launches of grace_shared_ffn as separate calls (as for grace_expert_ffn): _up writes the
 * hidden activation of all T rows to ws ([T, n_shared*f] of dt), _down reads it and writes
 * y_shared.  grace_shared_ffn(...) == _up(...) then _down(...) with the same ws. */
int grace_shared_ffn_up(const void *x, int32_t T, int32_t d, int32_t f, int32_t n_shared, grace_dtype dt,
                        const void *w_gate, const void *w_up, void *ws, void *stream);
int grace_shared_ffn_down(int32_t T, int32_t d, int32_t f, int32_t n_shared, grace_dtype dt, const void *w_down,
                          void *y_shared, void *ws, void *stream);

/* grace_shared_ffn_up and grace_permute_rows (the row movement of Section 5's dispatch order) as one
 * call: both read only x (and perm_pos), the projection is bound by the matrix cores and the row
 * movement by HBM, so for bf16 rows that are multiples of 1024 bytes the persistent kernel of the
 * projection carries the rows along (every wavefront moves a 1 KB piece of a token row every few K
 * steps) instead of a launch of its own; other shapes run the two launches.  Outputs are those of the
 * two calls, bit for bit: the hidden activation in ws and xp[perm_pos[t*k+j]] = x[t].
 * DEVICE: perm_pos [T*k] from grace_permute / grace_route_permute called with x == NULL; xp [T*k,d];
 * the rest as for grace_shared_ffn_up.  xp must not overlap x or ws. */
int grace_shared_ffn_up_scatter(const void *x, int32_t T, int32_t d, int32_t f, int32_t n_shared, grace_dtype dt,
                                const void *w_gate, const void *w_up, void *ws, const int32_t *perm_pos, int32_t k,
                                void *xp, void *stream);

/* ---- grace_combine: weighted aggregation back to token order ----------------
 * The aggregation step that follows the expert computation (Section 1):
 *     out[t] = sum_{j<k} topk_weight[t,j] * y[perm_pos[t*k+j]]  (+ y_shared[t]),
 * accumulated in fp32 in ascending j and rounded once to dt.
 * DEVICE: y [T*k,d]; perm_pos [T*k]; topk_weight [T,k]; y_shared [T,d] or NULL;
 * out [T,d].  Limits: d * sizeof(dt) a multiple of 16.
 */
int grace_combine(const void *y, const int32_t *perm_pos, const float *topk_weight, int32_t T, int32_t k, int32_t d,
                  grace_dtype dt, const void *y_shared, void *out, void *stream);

/* ---- diagnostics ---------------------------------------------------------------
 * Measures the bf16 MFMA rate the current device sustains with the grouped GEMM's
 * inner instruction mix (v_mfma_f32_16x16x32_bf16, 12 fragment reads per 32 of them)
 * and no global traffic (8 wavefronts per CU, one barrier per 64 MFMAs): constant or pseudo-random operands (a power-limited part runs
 * slower the more operand bits toggle), fragments held in registers or re-read
 * from LDS.  NOT for the hot path and the one exception to the conventions
 * above: it allocates and frees a small device buffer (hipMalloc / hipFree),
 * runs for a few tens of milliseconds on `stream` and synchronises it, so it
 * must not be called under stream capture.  HOST output: TFLOP/s. */
int grace_mfma_sustained(int32_t random_operands, int32_t lds_fed, double *tflops_out, void *stream);

/* Text of the calling thread's most recent error ("" if none).  The pointer
 * stays valid until the thread's next failing call. */
const char *grace_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* GRACE_MOE_H */
