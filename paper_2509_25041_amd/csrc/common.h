// Internal declarations shared by the translation units of libgrace_moe.so.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "grace_moe.h"

struct grace_table;

namespace grace {

// Thread-local error text behind grace_last_error().
int fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
const char *last_error();

#define GRACE_HIP(expr)                                                                          \
    do {                                                                                         \
        hipError_t e_ = (expr);                                                                  \
        if (e_ != hipSuccess)                                                                    \
            return ::grace::fail(GRACE_EHIP, "%s: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, \
                                 __LINE__);                                                      \
    } while (0)

#define GRACE_LAUNCH_CHECK(name)                                                                   \
    do {                                                                                           \
        hipError_t e_ = hipGetLastError();                                                         \
        if (e_ != hipSuccess)                                                                      \
            return ::grace::fail(GRACE_EHIP, "launch of %s: %s", name, hipGetErrorString(e_));     \
    } while (0)

constexpr int WAVE = 64;

// Assignments are ranked in chunks; one wavefront owns one chunk.
// route: the top-k kernel writes one histogram row per chunk of 16 tokens (small batches: more
// workgroups), 32 or 64 tokens (large batches: fewer histogram rows to sum); the workspace is sized
// for the smallest one
constexpr int ROUTE_CHUNK_SMALL = 16, ROUTE_CHUNK_LARGE = 32, ROUTE_CHUNK_HUGE = 64;
constexpr int ROUTE_SMALL_CHUNK_MAX_T = 8192, ROUTE_LARGE_CHUNK_MAX_T = 16384;
inline int route_chunk_tokens(int T) {
    return T <= ROUTE_SMALL_CHUNK_MAX_T ? ROUTE_CHUNK_SMALL : T <= ROUTE_LARGE_CHUNK_MAX_T ? ROUTE_CHUNK_LARGE : ROUTE_CHUNK_HUGE;
}
constexpr int PERM_CHUNK = 512;              // permute: chunk = 512 assignments

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// How the index kernels turn chunk histograms into prefix counts (grace_table_set_fold_limits moves
// a table's switch points).  0: separate single-block scan kernels; 1: every block sums the rows before its
// chunk; 2: two-level sums (super-chunks of 64 rows, one extra launch).
constexpr int FOLD_ONE_LEVEL_DEFAULT = 1024;  // histogram loads per key column a block may spend on a one-level sum
constexpr int FOLD_TWO_LEVEL_DEFAULT = 8192;  // the same for the super rows + chunk rows of a two-level sum
int fold_mode(const grace_table *table, int nchunks, int nkeys);
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace grace

struct grace_table;

namespace grace {

// Host-side argument checks of grace_route / grace_permute (shared with the fused call) and the
// launch of the row scatter.
int check_route_args(const grace_table *table, int32_t local_rank, grace_policy policy, const float *logits, int32_t T,
                     int32_t E, int32_t k, const uint32_t *rr_in, const uint32_t *rr_out, const int32_t *topk_expert,
                     const float *topk_weight, const int32_t *topk_inst, const int32_t *expert_count, const void *ws);
int check_permute_args(const grace_table *table, const int32_t *topk_inst, int32_t T, int32_t k, const void *x, int32_t d,
                       grace_dtype dt, const int32_t *perm_pos, const int32_t *perm_src, const int32_t *inst_off,
                       const int32_t *rank_off, const int32_t *node_off, const void *xp, const void *ws);
int launch_topk(const float *logits, int T, int E, int k, int renorm, int32_t *topk_expert, float *topk_weight,
                int32_t *chunk_hist, int32_t *clear, int n_clear, hipStream_t st);
int launch_route(const grace_table *table, int32_t local_rank, grace_policy policy, const float *logits, int32_t T,
                 int32_t E, int32_t k, int32_t renorm, const uint32_t *rr_in, uint32_t *rr_out, int32_t *topk_expert,
                 float *topk_weight, int32_t *topk_inst, int32_t *expert_count, void *ws, int32_t *inst_hist,
                 hipStream_t st);
// Byte offset, inside the workspace, of the permutation's histograms when routing and permutation
// share one call (the routing histograms of the same call lie below it).
size_t fused_perm_ws_offset(int32_t T, int32_t E);
// Workspace bytes of routing + permutation as one call (both sets of histograms and their prefix sums).
size_t route_permute_ws_bytes(int32_t T, int32_t E, int32_t k, int32_t I);
int launch_scatter_rows(const void *x, int T, int k, int d, grace_dtype dt, const int32_t *perm_pos, void *xp,
                        hipStream_t st);

}  // namespace grace

// The opaque table.  Host vectors describe the topology; one device allocation
// holds the arrays the kernels read.
struct grace_table {
    int32_t E = 0, R = 0, N = 0, I = 0, max_local_slots = 0;
    int device = -1;
    // CSR as given
    std::vector<int32_t> rank_node, inst_ptr, inst_rank_csr;
    std::vector<uint32_t> poll_weight;
    // dispatch order (node, rank, expert)
    std::vector<int32_t> csr_to_g, g_expert, g_rank, rank_ptr, node_first_rank;
    // device side
    void *d_base = nullptr;
    // per (local_rank, expert): candidates of the tier Algorithm 4 selects
    const int32_t *d_cand_ptr = nullptr;   // [(R+1)*E + 1]; block R = all instances (no locality)
    std::vector<int32_t> cand_view;        // host: cand_ptr[v * E] for v = 0 .. R+1 (first candidate of each view)
    const int32_t *d_cand_g = nullptr;     // instance id of each candidate, ascending rank
    const uint32_t *d_cand_cum = nullptr;  // inclusive cumulative polling weight inside the tier
    const int32_t *d_rank_ptr = nullptr;   // [R+1]
    const int32_t *d_node_first_inst = nullptr;  // [N+1] first instance id of each node (I at the end)
    const int32_t *d_inst_rank = nullptr;        // [I] hosting rank of each instance id
    const int32_t *d_rank_node = nullptr;        // [R]
    // switch points of the index kernels' prefix-count algorithms for calls with this table
    int fold_one_level = grace::FOLD_ONE_LEVEL_DEFAULT, fold_two_level = grace::FOLD_TWO_LEVEL_DEFAULT;
};
