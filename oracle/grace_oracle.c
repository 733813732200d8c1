/*
 * CPU oracle for one GPU's share of a GRACE-MoE layer.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, loop-by-loop statement of what the layer computes, used by the
 * tests, the smoke check and the benchmark's cpu_baseline leg.  It shares no
 * code with the HIP library and the product never calls it.
 *
 * Steps, in the paper's order (one MoE layer, Section 1 / Section 3: top-k
 * routing -> dispatch -> expert FFN -> aggregation; Section 4.3 + Algorithms 3
 * and 4 for the replica pick; Section 5 for the node-then-GPU dispatch order):
 *
 *   O1  top-k gating                      oracle_topk
 *   O2  per-expert request counter        oracle_pick (first half of the loop)
 *   O3  locality-first replica pick       oracle_pick
 *   O4  dispatch order of the instances   oracle_instance_order
 *   O5  stable permutation + offsets      oracle_permute, oracle_gather_rows
 *   O6  SwiGLU expert FFN on given rows   oracle_ffn_rows
 *   O7  weighted combine to token order   oracle_combine
 *
 * Floating point is fp64 throughout (inputs are widened by the caller); the
 * gate weights are rounded to fp32 once, when stored.
 *
 * Readings of points the paper leaves open (each also listed in the design
 * notes):
 *   - gating = softmax over all E logits, top-k on the raw logits, ties to the
 *     lower expert id, optional renormalisation over the k chosen;
 *   - "weighted round-robin" (Section 4.3) is read as classic block WRR per
 *     expert: the c-th request for an expert (counted in token order on the
 *     source GPU) goes to the candidate whose cumulative integer weight
 *     interval contains c mod W.  Algorithm 3's random weighted draw has the
 *     same long-run shares; this reading is deterministic;
 *   - all tokens of a call live on local_rank (Algorithm 4's token_gpu_id);
 *   - dispatch order = (node, rank, expert id), stable in assignment order.
 *
 * Parity pins: see tests/test_oracle_*.py (library argsort / matmul, brute
 * force, closed forms, hand-computed goldens under tests/golden/).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_EINVAL (-1)

/* ------------------------------------------------------------------ O1 --
 * Top-k gating (Section 3: each token activates k experts per layer).
 * For each token: experts ordered by (logit descending, id ascending); the
 * first k are chosen.  Weight = softmax probability over all E logits
 * (max-subtracted, fp64); with renorm the k weights are divided by their sum.
 */
int oracle_topk(const float *logits, int32_t T, int32_t E, int32_t k, int32_t renorm,
                int32_t *topk_expert, float *topk_weight)
{
    if (T < 0 || E < 1 || k < 1 || k > E) return ORACLE_EINVAL;
    char *taken = (char *)malloc((size_t)E);
    double *p = (double *)malloc(sizeof(double) * (size_t)E);
    if (!taken || !p) { free(taken); free(p); return ORACLE_EINVAL; }
    for (int32_t t = 0; t < T; ++t) {
        const float *row = logits + (size_t)t * E;
        float mx = row[0];
        for (int32_t e = 1; e < E; ++e) if (row[e] > mx) mx = row[e];
        double den = 0.0;
        for (int32_t e = 0; e < E; ++e) { p[e] = exp((double)row[e] - (double)mx); den += p[e]; }
        for (int32_t e = 0; e < E; ++e) p[e] /= den;
        memset(taken, 0, (size_t)E);
        double ksum = 0.0;
        for (int32_t j = 0; j < k; ++j) {
            int32_t best = -1;
            for (int32_t e = 0; e < E; ++e) {           /* ascending id: strict > keeps the lower id on ties */
                if (taken[e]) continue;
                if (best < 0 || row[e] > row[best]) best = e;
            }
            taken[best] = 1;
            topk_expert[(size_t)t * k + j] = best;
            ksum += p[best];
        }
        for (int32_t j = 0; j < k; ++j) {
            double w = p[topk_expert[(size_t)t * k + j]];
            if (renorm) w /= ksum;
            topk_weight[(size_t)t * k + j] = (float)w;
        }
    }
    free(taken); free(p);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ O4 --
 * Dispatch order of the expert instances (Section 5: stage 1 forwards to the
 * target node, stage 2 to the target GPU): sort all instances by
 * (node of rank, rank, expert id).  Instance ids used everywhere below are
 * positions in this order.  Inputs are the CSR table: instances of expert e
 * are inst_rank[inst_ptr[e] .. inst_ptr[e+1]).
 * Outputs: csr_to_g[I], g_expert[I], g_rank[I], rank_ptr[R+1] (instances of
 * rank r are ids rank_ptr[r] .. rank_ptr[r+1]; slot = id - rank_ptr[r]).
 */
int oracle_instance_order(int32_t E, int32_t R, const int32_t *rank_node,
                          const int32_t *inst_ptr, const int32_t *inst_rank,
                          int32_t *csr_to_g, int32_t *g_expert, int32_t *g_rank, int32_t *rank_ptr)
{
    int32_t I = inst_ptr[E];
    /* selection sort on the triple key; I is small */
    int32_t *ce = (int32_t *)malloc(sizeof(int32_t) * (size_t)(I > 0 ? I : 1));
    char *done = (char *)calloc((size_t)(I > 0 ? I : 1), 1);
    if (!ce || !done) { free(ce); free(done); return ORACLE_EINVAL; }
    for (int32_t e = 0; e < E; ++e)
        for (int32_t i = inst_ptr[e]; i < inst_ptr[e + 1]; ++i) ce[i] = e;
    for (int32_t g = 0; g < I; ++g) {
        int32_t best = -1;
        for (int32_t i = 0; i < I; ++i) {
            if (done[i]) continue;
            if (best < 0) { best = i; continue; }
            int32_t ni = rank_node[inst_rank[i]], nb = rank_node[inst_rank[best]];
            if (ni != nb) { if (ni < nb) best = i; continue; }
            if (inst_rank[i] != inst_rank[best]) { if (inst_rank[i] < inst_rank[best]) best = i; continue; }
            if (ce[i] < ce[best]) best = i;
        }
        done[best] = 1;
        csr_to_g[best] = g;
        g_expert[g] = ce[best];
        g_rank[g] = inst_rank[best];
    }
    for (int32_t r = 0; r <= R; ++r) rank_ptr[r] = 0;
    for (int32_t g = 0; g < I; ++g) rank_ptr[g_rank[g] + 1] += 1;
    for (int32_t r = 0; r < R; ++r) rank_ptr[r + 1] += rank_ptr[r];
    free(ce); free(done);
    return ORACLE_OK;
}

/* ------------------------------------------------------------- O2 + O3 --
 * Request counter and replica pick, one assignment at a time in (token, j)
 * order.  Candidate tier per Algorithm 4: an instance on the token's GPU; else
 * the instances on the token's node; else all instances.  Inside the tier the
 * c-th request of the expert goes to the candidate (ascending rank) whose
 * cumulative polling-weight interval contains c mod W (Algorithm 3 read as
 * deterministic weighted round-robin).  topk_inst holds dispatch-order ids.
 * rr_in / rr_out: per-expert counter carried across calls (NULL = start at 0);
 * rr_out[e] = (rr_in[e] + requests of e) mod W_e.
 */
int oracle_pick(const int32_t *topk_expert, int32_t T, int32_t k, int32_t E, int32_t R,
                const int32_t *rank_node, const uint32_t *poll_weight,
                const int32_t *inst_ptr, const int32_t *inst_rank, const int32_t *csr_to_g,
                int32_t local_rank, int32_t policy, const uint32_t *rr_in, uint32_t *rr_out,
                int32_t *topk_inst, int32_t *expert_count)
{
    /* policy 0: topology-aware tiers (Algorithm 4); policy 1: all instances are candidates
       (weighted round-robin alone, Section 4.3 first policy) */
    if (policy != 0 && policy != 1) return ORACLE_EINVAL;
    if (local_rank < 0 || local_rank >= R) return ORACLE_EINVAL;
    uint64_t *cnt = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)E);
    int32_t *cand = (int32_t *)malloc(sizeof(int32_t) * (size_t)(R > 0 ? R : 1));
    if (!cnt || !cand) { free(cnt); free(cand); return ORACLE_EINVAL; }
    for (int32_t e = 0; e < E; ++e) { cnt[e] = rr_in ? rr_in[e] : 0; expert_count[e] = 0; }
    const int32_t my_node = rank_node[local_rank];
    for (int64_t a = 0; a < (int64_t)T * k; ++a) {
        const int32_t e = topk_expert[a];
        if (e < 0 || e >= E) { free(cnt); free(cand); return ORACLE_EINVAL; }
        const uint64_t c = cnt[e];                      /* O2 */
        cnt[e] += 1;
        expert_count[e] += 1;
        /* O3: build the tier's candidate list (CSR indices, ascending rank) */
        int32_t nc = 0;
        if (policy == 0) {
            for (int32_t i = inst_ptr[e]; i < inst_ptr[e + 1]; ++i)
                if (inst_rank[i] == local_rank) cand[nc++] = i;
            if (nc == 0)
                for (int32_t i = inst_ptr[e]; i < inst_ptr[e + 1]; ++i)
                    if (rank_node[inst_rank[i]] == my_node) cand[nc++] = i;
        }
        if (nc == 0)
            for (int32_t i = inst_ptr[e]; i < inst_ptr[e + 1]; ++i) cand[nc++] = i;
        if (nc == 0) { free(cnt); free(cand); return ORACLE_EINVAL; }
        uint64_t W = 0;
        for (int32_t s = 0; s < nc; ++s) W += poll_weight[inst_rank[cand[s]]];
        const uint64_t q = c % W;
        uint64_t cum = 0;
        int32_t chosen = -1;
        for (int32_t s = 0; s < nc; ++s) {
            cum += poll_weight[inst_rank[cand[s]]];
            if (cum > q) { chosen = cand[s]; break; }
        }
        topk_inst[a] = csr_to_g[chosen];
    }
    if (rr_out) {
        for (int32_t e = 0; e < E; ++e) {
            /* tier weight sum of expert e as seen from local_rank */
            int32_t nc = 0;
            if (policy == 0) {
                for (int32_t i = inst_ptr[e]; i < inst_ptr[e + 1]; ++i)
                    if (inst_rank[i] == local_rank) cand[nc++] = i;
                if (nc == 0)
                    for (int32_t i = inst_ptr[e]; i < inst_ptr[e + 1]; ++i)
                        if (rank_node[inst_rank[i]] == my_node) cand[nc++] = i;
            }
            if (nc == 0)
                for (int32_t i = inst_ptr[e]; i < inst_ptr[e + 1]; ++i) cand[nc++] = i;
            uint64_t W = 0;
            for (int32_t s = 0; s < nc; ++s) W += poll_weight[inst_rank[cand[s]]];
            rr_out[e] = W ? (uint32_t)(cnt[e] % W) : 0u;
        }
    }
    free(cnt); free(cand);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ O5 --
 * Dispatch permutation: the buffer position of every assignment when the
 * assignments are sorted by instance id (= by node, rank, slot), keeping
 * assignment order among equal ids.  Written as the definition of a stable
 * sort: walk the ids in ascending order and, for each, the assignments in
 * ascending order.  Offsets are exclusive prefix counts; rank_off / node_off
 * are the offsets of the first instance of each rank / node.
 */
int oracle_permute(const int32_t *topk_inst, int32_t T, int32_t k, int32_t I, int32_t R, int32_t N,
                   const int32_t *g_rank, const int32_t *rank_node,
                   int32_t *perm_pos, int32_t *perm_src,
                   int32_t *inst_off, int32_t *rank_off, int32_t *node_off)
{
    const int64_t n = (int64_t)T * k;
    int64_t p = 0;
    for (int32_t g = 0; g < I; ++g) {
        inst_off[g] = (int32_t)p;
        for (int64_t a = 0; a < n; ++a)
            if (topk_inst[a] == g) { perm_src[p] = (int32_t)a; perm_pos[a] = (int32_t)p; ++p; }
    }
    inst_off[I] = (int32_t)p;
    if (p != n) return ORACLE_EINVAL;                   /* some id was outside [0, I) */
    /* rows destined to ranks < r, nodes < m */
    for (int32_t r = 0; r <= R; ++r) {
        int64_t c = 0;
        for (int64_t a = 0; a < n; ++a) if (g_rank[topk_inst[a]] < r) ++c;
        rank_off[r] = (int32_t)c;
    }
    for (int32_t m = 0; m <= N; ++m) {
        int64_t c = 0;
        for (int64_t a = 0; a < n; ++a) if (rank_node[g_rank[topk_inst[a]]] < m) ++c;
        node_off[m] = (int32_t)c;
    }
    return ORACLE_OK;
}

/* xp[p, :] = x[perm_src[p] / k, :] as a byte copy of rows. */
int oracle_gather_rows(const void *x, int64_t row_bytes, const int32_t *perm_src, int64_t n_rows, int32_t k,
                       void *xp)
{
    for (int64_t p = 0; p < n_rows; ++p)
        memcpy((char *)xp + p * row_bytes, (const char *)x + (int64_t)(perm_src[p] / k) * row_bytes,
               (size_t)row_bytes);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ O6 --
 * SwiGLU expert FFN on n_rows rows with one expert's weights, fp64:
 *   g = W_gate x, u = W_up x, h = g / (1 + exp(-g)) * u, y = W_down h.
 * Weight rows are output features: w_gate, w_up are [f, d]; w_down is [d, f].
 * x is [n_rows, d] and y is [n_rows, d], both dense.  accumulate != 0 adds
 * into y (used to sum shared experts).
 */
int oracle_ffn_rows(const double *x, int64_t n_rows, int32_t d, int32_t f,
                    const double *w_gate, const double *w_up, const double *w_down,
                    double *y, int32_t accumulate, int32_t n_threads)
{
    if (n_threads < 1) n_threads = 1;
    int bad = 0;
#pragma omp parallel for num_threads(n_threads) schedule(dynamic, 1)
    for (int64_t r = 0; r < n_rows; ++r) {
        double *h = (double *)malloc(sizeof(double) * (size_t)f);
        if (!h) { bad = 1; continue; }
        const double *xr = x + r * d;
        for (int32_t n = 0; n < f; ++n) {
            double g = 0.0, u = 0.0;
            const double *wg = w_gate + (size_t)n * d, *wu = w_up + (size_t)n * d;
            for (int32_t c = 0; c < d; ++c) { g += xr[c] * wg[c]; u += xr[c] * wu[c]; }
            h[n] = g / (1.0 + exp(-g)) * u;
        }
        double *yr = y + r * d;
        for (int32_t c = 0; c < d; ++c) {
            double acc = 0.0;
            const double *wd = w_down + (size_t)c * f;
            for (int32_t n = 0; n < f; ++n) acc += h[n] * wd[n];
            yr[c] = accumulate ? yr[c] + acc : acc;
        }
        free(h);
    }
    return bad ? ORACLE_EINVAL : ORACLE_OK;
}

/* ------------------------------------------------------------------ O7 --
 * out[t] = sum_j topk_weight[t, j] * y[perm_pos[t*k + j]]  (+ y_shared[t]),
 * fp64, j ascending.  y is [T*k, d] in dispatch order.
 */
int oracle_combine(const double *y, const int32_t *perm_pos, const float *topk_weight,
                   int32_t T, int32_t k, int32_t d, const double *y_shared, double *out)
{
    for (int64_t t = 0; t < T; ++t) {
        double *o = out + t * d;
        for (int32_t c = 0; c < d; ++c) o[c] = 0.0;
        for (int32_t j = 0; j < k; ++j) {
            const double w = (double)topk_weight[t * k + j];
            const double *yr = y + (int64_t)perm_pos[t * k + j] * d;
            for (int32_t c = 0; c < d; ++c) o[c] += w * yr[c];
        }
        if (y_shared)
            for (int32_t c = 0; c < d; ++c) o[c] += y_shared[t * d + c];
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------ send lists --
 * Section 5: a token with several experts on one destination is transmitted
 * once.  For every destination rank (node): the ascending list of tokens that
 * have at least one assignment there.  expand[a] = index of a's token in the
 * list of a's destination rank.  traffic (tokens): [0] cross-node with
 * de-duplication, [1] cross-node one row per assignment, [2] intra-node with
 * de-duplication (other ranks of the own node, plus in every other node the
 * ranks other than the stage-1 peer = the rank with local_rank's index inside
 * that node), [3] intra-node rows of a flat dispatch (assignments to the other
 * ranks of the own node).
 */
int oracle_send_lists(const int32_t *topk_inst, int32_t T, int32_t k, int32_t I, int32_t R, int32_t N,
                      const int32_t *g_rank, const int32_t *rank_node, int32_t local_rank,
                      int32_t *rank_send_ptr, int32_t *rank_send_tok, int32_t *node_send_ptr,
                      int32_t *node_send_tok, int32_t *expand, int64_t *traffic)
{
    if (local_rank < 0 || local_rank >= R) return ORACLE_EINVAL;
    for (int64_t a = 0; a < (int64_t)T * k; ++a)
        if (topk_inst[a] < 0 || topk_inst[a] >= I) return ORACLE_EINVAL;
    int32_t p = 0;
    for (int32_t r = 0; r < R; ++r) {
        rank_send_ptr[r] = p;
        for (int32_t t = 0; t < T; ++t) {
            int hit = 0;
            for (int32_t j = 0; j < k; ++j) if (g_rank[topk_inst[(int64_t)t * k + j]] == r) hit = 1;
            if (hit) {
                for (int32_t j = 0; j < k; ++j)
                    if (g_rank[topk_inst[(int64_t)t * k + j]] == r) expand[(int64_t)t * k + j] = p - rank_send_ptr[r];
                rank_send_tok[p++] = t;
            }
        }
    }
    rank_send_ptr[R] = p;
    p = 0;
    for (int32_t n = 0; n < N; ++n) {
        node_send_ptr[n] = p;
        for (int32_t t = 0; t < T; ++t) {
            int hit = 0;
            for (int32_t j = 0; j < k; ++j) if (rank_node[g_rank[topk_inst[(int64_t)t * k + j]]] == n) hit = 1;
            if (hit) node_send_tok[p++] = t;
        }
    }
    node_send_ptr[N] = p;
    if (traffic) {
        const int32_t my_node = rank_node[local_rank];
        int32_t my_first = 0;
        while (rank_node[my_first] != my_node) ++my_first;
        const int32_t local_idx = local_rank - my_first;
        traffic[0] = traffic[1] = traffic[2] = traffic[3] = 0;
        for (int32_t n = 0; n < N; ++n)
            if (n != my_node) traffic[0] += node_send_ptr[n + 1] - node_send_ptr[n];
        for (int64_t a = 0; a < (int64_t)T * k; ++a) {
            const int32_t r = g_rank[topk_inst[a]];
            if (rank_node[r] != my_node) traffic[1] += 1;
            else if (r != local_rank) traffic[3] += 1;
        }
        for (int32_t r = 0; r < R; ++r) {
            const int32_t nd = rank_node[r];
            const int32_t uniq = rank_send_ptr[r + 1] - rank_send_ptr[r];
            if (nd == my_node) {
                if (r != local_rank) traffic[2] += uniq;
            } else {
                int32_t first = 0, size = 0;
                while (rank_node[first] != nd) ++first;
                while (first + size < R && rank_node[first + size] == nd) ++size;
                if (r != first + local_idx % size) traffic[2] += uniq;
            }
        }
    }
    return ORACLE_OK;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
