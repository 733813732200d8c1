// Internal declarations shared by the translation units of libgrace_moe.so.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "grace_moe.h"

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
constexpr int ROUTE_TOKENS_PER_CHUNK = 32;   // route: chunk = 32 tokens = 32*k assignments
constexpr int PERM_CHUNK = 512;              // permute: chunk = 512 assignments

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

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
    const int32_t *d_cand_g = nullptr;     // instance id of each candidate, ascending rank
    const uint32_t *d_cand_cum = nullptr;  // inclusive cumulative polling weight inside the tier
    const int32_t *d_rank_ptr = nullptr;   // [R+1]
    const int32_t *d_node_first_inst = nullptr;  // [N+1] first instance id of each node (I at the end)
    const int32_t *d_inst_rank = nullptr;        // [I] hosting rank of each instance id
    const int32_t *d_rank_node = nullptr;        // [R]
};
