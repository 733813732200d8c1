// Placement / replica table: validation, dispatch order, per-rank candidate
// tiers (Algorithm 4 evaluated once per (rank, expert) on the host), device copy.
#include <algorithm>
#include <cstring>
#include <new>
#include <numeric>
#include <string>

#include "common.h"

namespace grace {

static thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}
const char *last_error() { return g_err; }

}  // namespace grace

using grace::fail;

extern "C" const char *grace_last_error(void) { return grace::last_error(); }

extern "C" int grace_table_validate(int32_t E, int32_t R, int32_t N, const int32_t *rank_node,
                                    const uint32_t *poll_weight, const int32_t *inst_ptr,
                                    const int32_t *inst_rank) {
    if (!rank_node || !poll_weight || !inst_ptr || !inst_rank) return fail(GRACE_EINVAL, "table: null pointer");
    if (E < 1 || R < 1 || N < 1) return fail(GRACE_EINVAL, "table: E, R, N must be >= 1 (got %d, %d, %d)", E, R, N);
    if (E > GRACE_MAX_EXPERTS || R > GRACE_MAX_RANKS || N > R)
        return fail(GRACE_ESHAPE, "table: E=%d R=%d N=%d outside limits (E<=%d, R<=%d, N<=R)", E, R, N,
                    GRACE_MAX_EXPERTS, GRACE_MAX_RANKS);
    for (int32_t r = 0; r < R; ++r) {
        if (rank_node[r] < 0 || rank_node[r] >= N)
            return fail(GRACE_ETABLE, "table: rank_node[%d]=%d outside [0,%d)", r, rank_node[r], N);
        if (r > 0 && rank_node[r] < rank_node[r - 1])
            return fail(GRACE_ETABLE, "table: rank_node must be non-decreasing (rank %d)", r);
        if (poll_weight[r] < 1 || poll_weight[r] > GRACE_MAX_POLL_WEIGHT)
            return fail(GRACE_ETABLE, "table: poll_weight[%d]=%u outside [1,%u]", r, poll_weight[r],
                        GRACE_MAX_POLL_WEIGHT);
    }
    if (inst_ptr[0] != 0) return fail(GRACE_ETABLE, "table: inst_ptr[0] must be 0");
    for (int32_t e = 0; e < E; ++e) {
        if (inst_ptr[e + 1] <= inst_ptr[e])
            return fail(GRACE_ETABLE, "table: expert %d has no instance (or inst_ptr decreases)", e);
        if (inst_ptr[e + 1] > GRACE_MAX_INSTANCES)
            return fail(GRACE_ESHAPE, "table: more than %d instances", GRACE_MAX_INSTANCES);
        for (int32_t i = inst_ptr[e]; i < inst_ptr[e + 1]; ++i) {
            if (inst_rank[i] < 0 || inst_rank[i] >= R)
                return fail(GRACE_ETABLE, "table: expert %d instance on rank %d outside [0,%d)", e, inst_rank[i], R);
            if (i > inst_ptr[e] && inst_rank[i] <= inst_rank[i - 1])
                return fail(GRACE_ETABLE, "table: ranks of expert %d must be strictly ascending (duplicate?)", e);
        }
    }
    return GRACE_OK;
}

// Tier of expert e seen from rank lr (Algorithm 4): the instance on lr; else the
// instances on lr's node; else all of them.  Returns CSR indices, ascending rank.
static void tier_of(const grace_table &t, int32_t lr, int32_t e, std::vector<int32_t> &out) {
    out.clear();
    const int32_t b = t.inst_ptr[e], en = t.inst_ptr[e + 1];
    for (int32_t i = b; i < en; ++i)
        if (t.inst_rank_csr[i] == lr) out.push_back(i);
    if (!out.empty()) return;
    for (int32_t i = b; i < en; ++i)
        if (t.rank_node[t.inst_rank_csr[i]] == t.rank_node[lr]) out.push_back(i);
    if (!out.empty()) return;
    for (int32_t i = b; i < en; ++i) out.push_back(i);
}

extern "C" int grace_table_create(grace_table **out, int32_t E, int32_t R, int32_t N, const int32_t *rank_node,
                                  const uint32_t *poll_weight, const int32_t *inst_ptr, const int32_t *inst_rank,
                                  void *stream) {
    if (!out) return fail(GRACE_EINVAL, "table_create: out is null");
    int rc = grace_table_validate(E, R, N, rank_node, poll_weight, inst_ptr, inst_rank);
    if (rc != GRACE_OK) return rc;
    grace_table *t = new (std::nothrow) grace_table();
    if (!t) return fail(GRACE_ENOMEM, "table_create: host allocation failed");
    t->E = E; t->R = R; t->N = N; t->I = inst_ptr[E];
    const int32_t I = t->I;
    t->rank_node.assign(rank_node, rank_node + R);
    t->poll_weight.assign(poll_weight, poll_weight + R);
    t->inst_ptr.assign(inst_ptr, inst_ptr + E + 1);
    t->inst_rank_csr.assign(inst_rank, inst_rank + I);

    // dispatch order: (node, rank, expert).  rank_node is non-decreasing, so (rank, expert) suffices.
    std::vector<int32_t> csr_expert(I);
    for (int32_t e = 0; e < E; ++e)
        for (int32_t i = inst_ptr[e]; i < inst_ptr[e + 1]; ++i) csr_expert[i] = e;
    std::vector<int32_t> ord(I);
    std::iota(ord.begin(), ord.end(), 0);
    std::sort(ord.begin(), ord.end(), [&](int32_t a, int32_t b) {
        if (inst_rank[a] != inst_rank[b]) return inst_rank[a] < inst_rank[b];
        return csr_expert[a] < csr_expert[b];
    });
    t->csr_to_g.resize(I); t->g_expert.resize(I); t->g_rank.resize(I);
    for (int32_t g = 0; g < I; ++g) {
        t->csr_to_g[ord[g]] = g;
        t->g_expert[g] = csr_expert[ord[g]];
        t->g_rank[g] = inst_rank[ord[g]];
    }
    t->rank_ptr.assign(R + 1, 0);
    for (int32_t g = 0; g < I; ++g) t->rank_ptr[t->g_rank[g] + 1] += 1;
    for (int32_t r = 0; r < R; ++r) {
        t->max_local_slots = std::max(t->max_local_slots, t->rank_ptr[r + 1]);
        t->rank_ptr[r + 1] += t->rank_ptr[r];
    }
    // first instance id of every node (ranks are node-major)
    std::vector<int32_t> node_first_inst(N + 1, I);
    {
        int32_t r = 0;
        for (int32_t n = 0; n <= N; ++n) {
            while (r < R && rank_node[r] < n) ++r;
            node_first_inst[n] = (r < R) ? t->rank_ptr[r] : I;
        }
    }

    // candidate tiers for every (local rank, expert)
    // block lr == R: all instances of the expert (policy without locality)
    std::vector<int32_t> cand_ptr((size_t)(R + 1) * E + 1, 0), cand_g;
    std::vector<uint32_t> cand_cum;
    std::vector<int32_t> tier;
    for (int32_t lr = 0; lr <= R; ++lr)
        for (int32_t e = 0; e < E; ++e) {
            if (lr < R) {
                tier_of(*t, lr, e, tier);
            } else {
                tier.clear();
                for (int32_t i = inst_ptr[e]; i < inst_ptr[e + 1]; ++i) tier.push_back(i);
            }
            uint32_t cum = 0;
            for (int32_t i : tier) {
                cum += poll_weight[inst_rank[i]];
                cand_g.push_back(t->csr_to_g[i]);
                cand_cum.push_back(cum);
            }
            cand_ptr[(size_t)lr * E + e + 1] = (int32_t)cand_g.size();
        }

    // one packed device allocation
    auto al = [](size_t v) { return grace::align_up(v, 256); };
    const size_t o_ptr = 0;
    const size_t o_g = o_ptr + al(cand_ptr.size() * 4);
    const size_t o_cum = o_g + al(cand_g.size() * 4);
    const size_t o_rank = o_cum + al(cand_cum.size() * 4);
    const size_t o_node = o_rank + al((size_t)(R + 1) * 4);
    const size_t o_irank = o_node + al((size_t)(N + 1) * 4);
    const size_t o_rnode = o_irank + al((size_t)I * 4);
    const size_t total = o_rnode + al((size_t)R * 4);
    std::vector<char> stage(total, 0);
    memcpy(stage.data() + o_ptr, cand_ptr.data(), cand_ptr.size() * 4);
    t->cand_view.resize((size_t)R + 2);
    for (int v = 0; v <= R + 1; ++v) t->cand_view[v] = cand_ptr[(size_t)v * E];
    memcpy(stage.data() + o_g, cand_g.data(), cand_g.size() * 4);
    memcpy(stage.data() + o_cum, cand_cum.data(), cand_cum.size() * 4);
    memcpy(stage.data() + o_rank, t->rank_ptr.data(), (size_t)(R + 1) * 4);
    memcpy(stage.data() + o_node, node_first_inst.data(), (size_t)(N + 1) * 4);
    memcpy(stage.data() + o_irank, t->g_rank.data(), (size_t)I * 4);
    memcpy(stage.data() + o_rnode, rank_node, (size_t)R * 4);

    hipError_t he = hipGetDevice(&t->device);
    if (he == hipSuccess) he = hipMalloc(&t->d_base, total);
    if (he == hipSuccess) he = hipMemcpyAsync(t->d_base, stage.data(), total, hipMemcpyHostToDevice, (hipStream_t)stream);
    if (he == hipSuccess) he = hipStreamSynchronize((hipStream_t)stream);
    if (he != hipSuccess) {
        if (t->d_base) (void)hipFree(t->d_base);
        delete t;
        return fail(GRACE_EHIP, "table_create: %s", hipGetErrorString(he));
    }
    char *b = (char *)t->d_base;
    t->d_cand_ptr = (const int32_t *)(b + o_ptr);
    t->d_cand_g = (const int32_t *)(b + o_g);
    t->d_cand_cum = (const uint32_t *)(b + o_cum);
    t->d_rank_ptr = (const int32_t *)(b + o_rank);
    t->d_node_first_inst = (const int32_t *)(b + o_node);
    t->d_inst_rank = (const int32_t *)(b + o_irank);
    t->d_rank_node = (const int32_t *)(b + o_rnode);
    *out = t;
    return GRACE_OK;
}

extern "C" int grace_table_destroy(grace_table *t) {
    if (!t) return GRACE_OK;
    int rc = GRACE_OK;
    if (t->d_base) {
        hipError_t he = hipFree(t->d_base);
        if (he != hipSuccess) rc = fail(GRACE_EHIP, "table_destroy: %s", hipGetErrorString(he));
    }
    delete t;
    return rc;
}

extern "C" int grace_table_info(const grace_table *t, int32_t *E, int32_t *R, int32_t *N, int32_t *I,
                                int32_t *max_local_slots) {
    if (!t) return fail(GRACE_EINVAL, "table_info: table is null");
    if (E) *E = t->E;
    if (R) *R = t->R;
    if (N) *N = t->N;
    if (I) *I = t->I;
    if (max_local_slots) *max_local_slots = t->max_local_slots;
    return GRACE_OK;
}

extern "C" int grace_table_instances(const grace_table *t, int32_t *inst_expert, int32_t *inst_rank,
                                     int32_t *rank_ptr) {
    if (!t) return fail(GRACE_EINVAL, "table_instances: table is null");
    if (inst_expert) memcpy(inst_expert, t->g_expert.data(), (size_t)t->I * 4);
    if (inst_rank) memcpy(inst_rank, t->g_rank.data(), (size_t)t->I * 4);
    if (rank_ptr) memcpy(rank_ptr, t->rank_ptr.data(), (size_t)(t->R + 1) * 4);
    return GRACE_OK;
}

extern "C" int grace_table_local_experts(const grace_table *t, int32_t rank, int32_t *experts_out, int32_t *n_out) {
    if (!t || !experts_out || !n_out) return fail(GRACE_EINVAL, "table_local_experts: null pointer");
    if (rank < 0 || rank >= t->R) return fail(GRACE_EINVAL, "table_local_experts: rank %d outside [0,%d)", rank, t->R);
    int32_t n = 0;
    for (int32_t g = t->rank_ptr[rank]; g < t->rank_ptr[rank + 1]; ++g) experts_out[n++] = t->g_expert[g];
    *n_out = n;
    return GRACE_OK;
}

namespace grace {
int fold_mode(const grace_table *table, int nchunks, int nkeys) {
    constexpr int64_t SUPER = 64;  // rows per super-chunk (FOLD_SUPER of the kernels)
    const int64_t kb = (nkeys + 63) / 64;
    if (nchunks < 1) return 0;
    if ((int64_t)nchunks * nkeys >= (int64_t)1 << 31) return 0;  // the folded sums index the histogram with 32 bits
    if (nchunks * kb <= table->fold_one_level) return 1;
    const int64_t nsuper = (nchunks + SUPER - 1) / SUPER;
    return (nsuper + SUPER) * kb <= table->fold_two_level ? 2 : 0;
}

size_t fused_perm_ws_offset(int32_t T, int32_t E) {
    return 2 * align_up((size_t)ceil_div(T, ROUTE_CHUNK_SMALL) * (size_t)E * 4, 256);
}

size_t route_permute_ws_bytes(int32_t T, int32_t E, int32_t k, int32_t I) {
    const size_t chunks_p = (size_t)ceil_div((int64_t)T * k, PERM_CHUNK);
    return fused_perm_ws_offset(T, E) + 2 * align_up(chunks_p * (size_t)I * 4, 256);
}
}  // namespace grace

extern "C" int grace_table_set_fold_limits(grace_table *table, int32_t one_level_max, int32_t two_level_max) {
    if (!table) return fail(GRACE_EINVAL, "table_set_fold_limits: table is null");
    table->fold_one_level = one_level_max < 0 ? grace::FOLD_ONE_LEVEL_DEFAULT : one_level_max;
    table->fold_two_level = two_level_max < 0 ? grace::FOLD_TWO_LEVEL_DEFAULT : two_level_max;
    return GRACE_OK;
}

extern "C" size_t grace_workspace_bytes(int32_t T, int32_t E, int32_t k, int32_t I, int32_t d, int32_t f,
                                        int32_t n_shared, grace_dtype dt) {
    if (T < 0 || E < 1 || k < 1 || I < 1 || d < 0 || f < 0 || n_shared < 0) return 0;
    if (dt != GRACE_F32 && dt != GRACE_BF16) return 0;
    const size_t el = dt == GRACE_F32 ? 4 : 2;
    const size_t n = (size_t)T * (size_t)k;
    const size_t chunks_p = (size_t)grace::ceil_div((int64_t)n, grace::PERM_CHUNK);
    // routing and permutation histograms side by side (grace_route_permute uses both at once)
    size_t need = grace::route_permute_ws_bytes(T, E, k, I);
    need = std::max(need, grace::align_up(n * (size_t)f * el, 256));
    need = std::max(need, grace::align_up((size_t)T * (size_t)n_shared * (size_t)f * el, 256));
    // send lists: five int32 arrays over the assignments + chunk histograms over up to GRACE_MAX_RANKS keys + counters
    need = std::max(need, 5 * grace::align_up(n * 4, 256) + 2 * grace::align_up(chunks_p * (size_t)GRACE_MAX_RANKS * 4, 256) +
                              grace::align_up(((size_t)GRACE_MAX_RANKS + 1) * 4, 256));
    return need + 256;
}
