// grace_send_lists: de-duplicated hierarchical send lists and traffic counters.
//
// The two-stage dispatch of Section 5 forwards a token once per destination even
// when several of its experts live there.  For the tokens of
// local_rank this builds, per destination rank and per destination node, the
// ascending list of distinct tokens that have at least one assignment there, the
// map that lets the receiver expand the unique rows back to one row per
// assignment, and the token counts the paper's traffic metrics are made of.
//
//   1. dedup_keys_kernel  one lane per assignment: its destination rank / node; the
//                         token's first assignment per destination keeps the
//                         destination as its sort key, the others get -1
//   2. stable counting sort by rank key and by node key (stable_sort.h)
//   3. expand_traffic_kernel  expansion map + traffic sums
#include "common.h"
#include "stable_sort.h"

namespace grace {

// One lane per assignment.  The first blocks also clear the counters that expand_traffic_kernel
// accumulates into later in the same call (rows per destination rank, finished-block count).
__global__ __launch_bounds__(256) void dedup_keys_kernel(const int32_t *__restrict__ topk_inst, int64_t n_assign, int k,
                                                         int I, const int32_t *__restrict__ inst_rank,
                                                         const int32_t *__restrict__ rank_node,
                                                         int32_t *__restrict__ rank_key, int32_t *__restrict__ node_key,
                                                         int32_t *__restrict__ first_idx, int32_t *__restrict__ counters,
                                                         int n_counters) {
    const int64_t a = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (a < n_counters) counters[a] = 0;
    if (a >= n_assign) return;
    const int64_t t = a / k;
    const int j = (int)(a - t * k);
    const int32_t *row = topk_inst + t * k;
    const int g = row[j];
    if ((unsigned)g >= (unsigned)I) {  // id outside the table: no destination
        rank_key[a] = -1; node_key[a] = -1; first_idx[a] = -1;
        return;
    }
    const int r = inst_rank[g], nd = rank_node[r];
    int first_r = j;
    bool first_n = true;
    for (int jj = 0; jj < j; ++jj) {
        const int g2 = row[jj];
        if ((unsigned)g2 >= (unsigned)I) continue;
        const int r2 = inst_rank[g2];
        if (r2 == r && first_r == j) first_r = jj;
        if (rank_node[r2] == nd) first_n = false;
    }
    rank_key[a] = (first_r == j) ? r : -1;
    node_key[a] = first_n ? nd : -1;
    first_idx[a] = (int32_t)(t * k + first_r);
}

// expand[a] = index of a's token in the send list of a's destination rank.
// traffic[0] cross-node tokens with de-duplication: sum over other nodes of their distinct tokens
// traffic[1] cross-node rows without (one per assignment)
// traffic[2] intra-node tokens with de-duplication: distinct tokens for the other ranks of the own
//            node plus, in every other node, for the ranks other than the peer that received stage 1
// traffic[3] intra-node rows of a flat dispatch: assignments to the other ranks of the own node
// counters: [0, R) rows per destination rank (all blocks add their share: integer sums, exact in any
// order), [R] number of blocks that have added; the block that finishes last turns them into traffic[].
__global__ __launch_bounds__(256) void expand_traffic_kernel(const int32_t *__restrict__ topk_inst, int64_t n_assign, int I,
                                                             int R, int N, int local_rank,
                                                             const int32_t *__restrict__ inst_rank,
                                                             const int32_t *__restrict__ rank_node,
                                                             const int32_t *__restrict__ first_idx,
                                                             const int32_t *__restrict__ send_pos,
                                                             const int32_t *__restrict__ rank_send_ptr,
                                                             const int32_t *__restrict__ node_send_ptr,
                                                             int32_t *__restrict__ expand, int64_t *__restrict__ traffic,
                                                             int32_t *__restrict__ counters) {
    __shared__ int32_t naive_rank[GRACE_MAX_RANKS];
    __shared__ unsigned long long acc[4];
    __shared__ int last_block;
    const int64_t a = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (traffic)
        for (int r = (int)threadIdx.x; r < R; r += 256) naive_rank[r] = 0;
    __syncthreads();
    if (a < n_assign) {
        const int g = topk_inst[a];
        int32_t e = -1;
        if ((unsigned)g < (unsigned)I) {
            const int r = inst_rank[g];
            e = send_pos[first_idx[a]] - rank_send_ptr[r];
            if (traffic) atomicAdd(&naive_rank[r], 1);
        }
        expand[a] = e;
    }
    if (!traffic) return;
    __syncthreads();
    for (int r = (int)threadIdx.x; r < R; r += 256)
        if (naive_rank[r]) atomicAdd(&counters[r], naive_rank[r]);
    __threadfence();  // this block's sums are visible before it counts itself as finished
    __syncthreads();
    if (threadIdx.x == 0) last_block = atomicAdd(&counters[R], 1) == (int)gridDim.x - 1;
    __syncthreads();
    if (!last_block) return;
    __threadfence();
    if (threadIdx.x < 4) acc[threadIdx.x] = 0ull;
    __syncthreads();
    const int my_node = rank_node[local_rank];
    int my_first = 0;  // first rank of the own node (ranks are node-major)
    while (my_first < R && rank_node[my_first] != my_node) ++my_first;
    const int local_idx = local_rank - my_first;
    for (int r = (int)threadIdx.x; r < R; r += 256) {
        const int nd = rank_node[r];
        const unsigned long long uniq = (unsigned long long)(rank_send_ptr[r + 1] - rank_send_ptr[r]);
        const unsigned long long rows = (unsigned long long)atomicAdd(&counters[r], 0);  // read at the L2, past this CU's cache
        if (nd != my_node) {
            atomicAdd(&acc[1], rows);
            // the peer of local_rank in node nd: same index inside the node (modulo the node's size)
            int first = r, size = 0;
            while (first > 0 && rank_node[first - 1] == nd) --first;
            while (first + size < R && rank_node[first + size] == nd) ++size;
            const int peer = first + local_idx % size;
            if (r != peer) atomicAdd(&acc[2], uniq);
        } else if (r != local_rank) {
            atomicAdd(&acc[2], uniq);
            atomicAdd(&acc[3], rows);
        }
    }
    for (int n = (int)threadIdx.x; n < N; n += 256)
        if (n != my_node) atomicAdd(&acc[0], (unsigned long long)(node_send_ptr[n + 1] - node_send_ptr[n]));
    __syncthreads();
    if (threadIdx.x < 4) traffic[threadIdx.x] = (int64_t)acc[threadIdx.x];
}

static int sort_by_key(const grace_table *table, const int32_t *keys, int64_t n, int k, int nkeys, int32_t *hist, int32_t *base, int32_t *off,
                       int32_t *pos, int32_t *tok, hipStream_t st) {
    const char *failed = stable_sort_launch(table, keys, n, nkeys, k, hist, base, 0, 0, nullptr, nullptr, off, nullptr, nullptr,
                                            pos, tok, st);
    if (failed) return fail(GRACE_EHIP, "send_lists: launch of %s failed", failed);
    return GRACE_OK;
}

}  // namespace grace

using namespace grace;

extern "C" int grace_send_lists(const grace_table *table, int32_t local_rank, const int32_t *topk_inst, int32_t T,
                                int32_t k, int32_t *rank_send_ptr, int32_t *rank_send_tok, int32_t *node_send_ptr,
                                int32_t *node_send_tok, int32_t *expand, int64_t *traffic, void *ws, void *stream) {
    if (!table) return fail(GRACE_EINVAL, "send_lists: table is null");
    if (local_rank < 0 || local_rank >= table->R)
        return fail(GRACE_EINVAL, "send_lists: local_rank=%d outside [0,%d)", local_rank, table->R);
    if (T < 0 || k < 1) return fail(GRACE_EINVAL, "send_lists: T=%d, k=%d invalid", T, k);
    if ((int64_t)T * k > INT32_MAX) return fail(GRACE_ESHAPE, "send_lists: T*k exceeds 2^31-1");
    if (!rank_send_ptr || !node_send_ptr || !ws) return fail(GRACE_EINVAL, "send_lists: null offset or ws pointer");
    if (T > 0 && (!topk_inst || !rank_send_tok || !node_send_tok || !expand))
        return fail(GRACE_EINVAL, "send_lists: null device pointer");
    hipStream_t st = (hipStream_t)stream;
    const int64_t n = (int64_t)T * k;
    const int R = table->R, N = table->N, I = table->I;
    const size_t seg = align_up((size_t)n * 4, 256);
    char *w = (char *)ws;
    int32_t *rank_key = (int32_t *)w, *node_key = (int32_t *)(w + seg), *first_idx = (int32_t *)(w + 2 * seg);
    int32_t *pos_r = (int32_t *)(w + 3 * seg), *pos_n = (int32_t *)(w + 4 * seg);
    const size_t nchunks = (size_t)ceil_div(n, PERM_CHUNK);
    int32_t *hist = (int32_t *)(w + 5 * seg);
    int32_t *base = (int32_t *)(w + 5 * seg + align_up(nchunks * (size_t)GRACE_MAX_RANKS * 4, 256));
    // R per-rank row counters + 1 finished-block counter, behind the chunk histograms
    int32_t *counters = (int32_t *)(w + 5 * seg + 2 * align_up(nchunks * (size_t)GRACE_MAX_RANKS * 4, 256));
    {
        const int64_t lanes = std::max<int64_t>(n, R + 1);
        dedup_keys_kernel<<<(unsigned)ceil_div(lanes, 256), 256, 0, st>>>(topk_inst, n, k, I, table->d_inst_rank,
                                                                         table->d_rank_node, rank_key, node_key, first_idx,
                                                                         counters, R + 1);
        GRACE_LAUNCH_CHECK("dedup_keys_kernel");
    }
    int rc = sort_by_key(table, rank_key, n, k, R, hist, base, rank_send_ptr, pos_r, rank_send_tok, st);
    if (rc != GRACE_OK) return rc;
    rc = sort_by_key(table, node_key, n, k, N, hist, base, node_send_ptr, pos_n, node_send_tok, st);
    if (rc != GRACE_OK) return rc;
    if (n > 0 || traffic) {
        expand_traffic_kernel<<<(unsigned)std::max<int64_t>(1, ceil_div(n, 256)), 256, 0, st>>>(
            topk_inst, n, I, R, N, local_rank, table->d_inst_rank, table->d_rank_node, first_idx, pos_r, rank_send_ptr,
            node_send_ptr, expand, traffic, counters);
        GRACE_LAUNCH_CHECK("expand_traffic_kernel");
    }
    return GRACE_OK;
}
