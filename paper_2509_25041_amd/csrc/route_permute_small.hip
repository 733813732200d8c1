// grace_route_permute: grace_route followed by grace_permute as one call.
//
// Any batch: the replica pick also counts its choices per permutation chunk and
// instance (into counters the top-k kernel cleared), so the permutation's own
// histogram launch is dropped: top-k, pick, positions, row scatter.
//
// Decode-sized batches (a few hundred tokens) are bound by launch latency: the
// two calls need five launches of kernels that each run a few microseconds.  When
// the batch is small enough, the top-k gate (one wavefront per token, spread over
// the device) is followed by ONE single-workgroup kernel that does all the index
// work, every wavefront owning a contiguous range of assignments:
//   1. request counters    scan of the per-wavefront expert counts (Section 4.3)
//   2. replica pick        Algorithm 4 tier + weighted round-robin, per wavefront in order
//   3. offsets             per instance / rank / node, scan of the per-wavefront instance counts
//   4. positions           stable rank of every assignment in (node, rank, slot) order (Section 5)
// and by the row scatter: three launches.
// Outputs are identical either way (all integer work is exact and order-independent).
#include <mutex>

#include "common.h"
#include "route_device.h"
#include "stable_sort.h"
#include "wave_utils.h"

namespace grace {

constexpr int SMALL_THREADS = 1024, SMALL_WAVES = SMALL_THREADS / 64;
constexpr int SMALL_MAX_KEYS = 256;      // experts and instances the LDS tables hold
constexpr int SMALL_MAX_PER_WAVE = 256;  // assignments one wavefront walks

inline bool small_batch(int T, int k, int E, int I) {
    return T >= 1 && E <= SMALL_MAX_KEYS && I <= SMALL_MAX_KEYS &&
           ceil_div(T, SMALL_WAVES) * k <= SMALL_MAX_PER_WAVE;
}

__global__ __launch_bounds__(SMALL_THREADS) void dispatch_small_kernel(
    int T, int E, int k, const uint32_t *__restrict__ rr_in, uint32_t *__restrict__ rr_out,
    const int32_t *__restrict__ cand_ptr, const int32_t *__restrict__ cand_g, const uint32_t *__restrict__ cand_cum, int I,
    int R, int N, const int32_t *__restrict__ rank_ptr, const int32_t *__restrict__ node_first_inst,
    const int32_t *__restrict__ topk_expert, int32_t *__restrict__ topk_inst, int32_t *__restrict__ expert_count,
    int32_t *__restrict__ perm_pos, int32_t *__restrict__ perm_src, int32_t *__restrict__ inst_off,
    int32_t *__restrict__ rank_off, int32_t *__restrict__ node_off) {
    __shared__ int32_t ecnt[SMALL_WAVES][SMALL_MAX_KEYS];  // requests per expert of a wavefront, then before it
    __shared__ int32_t icnt[SMALL_WAVES][SMALL_MAX_KEYS];  // rows per instance of a wavefront, then before it
    __shared__ int32_t asg[SMALL_WAVES][SMALL_MAX_PER_WAVE];  // expert, then instance, of the wavefront's assignments
    __shared__ int32_t ioff[SMALL_MAX_KEYS + 1];
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tpw = (T + SMALL_WAVES - 1) / SMALL_WAVES;  // tokens per wavefront
    const int t0 = min(T, wave * tpw), t1 = min(T, t0 + tpw);
    const int n_w = (t1 - t0) * k;                         // assignments of this wavefront, in order
    const int64_t a0 = (int64_t)t0 * k;
    for (int i = lane; i < SMALL_MAX_KEYS; i += 64) {
        ecnt[wave][i] = 0;
        icnt[wave][i] = 0;
    }
    int ebits = 0, ibits = 0;
    while ((1 << ebits) < E) ++ebits;
    while ((1 << ibits) < I) ++ibits;
    const uint64_t lt = lanemask_lt();
    // The LDS operations of one wavefront execute in program order, so a counter updated by the last
    // lane of a match set is seen by the next group of 64 assignments.
    // ---- 0. this wavefront's experts and their counts ---------------------------------------------
    for (int b = 0; b < n_w; b += 64) {
        const int j = b + lane;
        bool valid = j < n_w;
        int e = valid ? topk_expert[a0 + j] : 0;
        valid = valid && (unsigned)e < (unsigned)E;
        if (j < n_w) asg[wave][j] = valid ? e : -1;
        const uint64_t same = wave_match((uint32_t)e, valid, ebits);
        if (valid && is_last_of(same)) wave_ctr_add(&ecnt[wave][e], (int32_t)__popcll(same));
        wave_ctr_fence();
    }
    __syncthreads();
    // ---- 1. requests of each expert before each wavefront; totals -----------------------------
    if (tid < E) {
        int32_t run = 0;
#pragma unroll
        for (int w = 0; w < SMALL_WAVES; ++w) {
            const int32_t c = ecnt[w][tid];
            ecnt[w][tid] = run;
            run += c;
        }
        expert_count[tid] = run;
        if (rr_out) rr_out[tid] = next_rr(rr_in, tid, run, cand_ptr, cand_cum);
    }
    __syncthreads();
    // ---- 2. replica pick, in assignment order; instance counts ---------------------------------
    for (int b = 0; b < n_w; b += 64) {
        const int j = b + lane;
        const int e_in = j < n_w ? asg[wave][j] : -1;
        const bool valid = e_in >= 0;
        const int e = valid ? e_in : 0;
        const uint64_t same = wave_match((uint32_t)e, valid, ebits);
        int g = 0;
        if (valid) {
            const uint64_t c = (uint64_t)(uint32_t)wave_ctr_load(&ecnt[wave][e]) + (uint32_t)__popcll(same & lt) +
                               (uint64_t)(rr_in ? rr_in[e] : 0u);
            g = pick_candidate(c, e, cand_ptr, cand_g, cand_cum);
            topk_inst[a0 + j] = g;
        }
        if (j < n_w) asg[wave][j] = valid ? g : -1;
        if (valid && is_last_of(same)) wave_ctr_add(&ecnt[wave][e], (int32_t)__popcll(same));
        const uint64_t same_g = wave_match((uint32_t)g, valid, ibits);
        if (valid && is_last_of(same_g)) wave_ctr_add(&icnt[wave][g], (int32_t)__popcll(same_g));
        wave_ctr_fence();
    }
    __syncthreads();
    // ---- 3. rows of each instance before each wavefront; offsets --------------------------------
    int32_t total = 0;
    if (tid < I) {
#pragma unroll
        for (int w = 0; w < SMALL_WAVES; ++w) {
            const int32_t c = icnt[w][tid];
            icnt[w][tid] = total;
            total += c;
        }
    }
    if (tid < SMALL_MAX_KEYS) ioff[tid] = total;  // totals, scanned below (zero for ids >= I)
    __syncthreads();
    if (wave == 0) {
        // exclusive scan over the ids: each lane owns four consecutive ids
        int32_t c[4], s = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            c[q] = ioff[lane * 4 + q];
            s += c[q];
        }
        int32_t incl = s;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int32_t v = __shfl_up(incl, o, 64);
            if (lane >= o) incl += v;
        }
        int32_t run = incl - s;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            ioff[lane * 4 + q] = run;
            run += c[q];
        }
        if (lane == 63) ioff[SMALL_MAX_KEYS] = incl;  // grand total = offset of every id >= I
    }
    __syncthreads();
    for (int i = tid; i <= I; i += SMALL_THREADS) inst_off[i] = ioff[i];
    for (int r = tid; r <= R; r += SMALL_THREADS) rank_off[r] = ioff[rank_ptr[r]];
    for (int n = tid; n <= N; n += SMALL_THREADS) node_off[n] = ioff[node_first_inst[n]];
    // ---- 4. positions ---------------------------------------------------------------------------
    for (int b = 0; b < n_w; b += 64) {
        const int j = b + lane;
        const int g_in = j < n_w ? asg[wave][j] : -1;
        const bool valid = g_in >= 0;
        const int g = valid ? g_in : 0;
        const uint64_t same = wave_match((uint32_t)g, valid, ibits);
        if (valid) {
            const int32_t pos = ioff[g] + wave_ctr_load(&icnt[wave][g]) + (int32_t)__popcll(same & lt);
            perm_pos[a0 + j] = pos;
            perm_src[pos] = (int32_t)(a0 + j);
        } else if (j < n_w) {
            perm_pos[a0 + j] = -1;  // expert id outside the table: no row
        }
        if (valid && is_last_of(same)) wave_ctr_add(&icnt[wave][g], (int32_t)__popcll(same));
        wave_ctr_fence();
    }
}

}  // namespace grace

using namespace grace;

static int route_permute_impl(const grace_table *table, int32_t local_rank, grace_policy policy, const float *logits,
                             int32_t T, int32_t E, int32_t k, int32_t renorm, const uint32_t *rr_in, uint32_t *rr_out,
                             int32_t *topk_expert, float *topk_weight, int32_t *topk_inst, int32_t *expert_count,
                             const void *x, int32_t d, grace_dtype dt, int32_t *perm_pos, int32_t *perm_src,
                             int32_t *inst_off, int32_t *rank_off, int32_t *node_off, void *xp, void *ws, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    int rc;
    // the shared-histogram path counts with 32-bit indices; sizes beyond that take the two calls
    const bool hist_fits = ceil_div((int64_t)T * k, PERM_CHUNK) * table->I <= (int64_t)1 << 30;
    if (T == 0 || !hist_fits) {
        rc = grace_route(table, local_rank, policy, logits, T, E, k, renorm, rr_in, rr_out, topk_expert, topk_weight,
                         topk_inst, expert_count, ws, stream);
        if (rc != GRACE_OK) return rc;
        return grace_permute(table, topk_inst, T, k, x, d, dt, perm_pos, perm_src, inst_off, rank_off, node_off, xp, ws,
                             stream);
    }
    if (!small_batch(T, k, E, table->I)) {
        const int I = table->I;
        const int64_t n = (int64_t)T * k;
        const int nchunks = (int)ceil_div(n, PERM_CHUNK);
        int32_t *phist = (int32_t *)((char *)ws + fused_perm_ws_offset(T, E));
        int32_t *pbase = (int32_t *)((char *)phist + align_up((size_t)nchunks * I * 4, 256));
        rc = launch_route(table, local_rank, policy, logits, T, E, k, renorm, rr_in, rr_out, topk_expert, topk_weight,
                          topk_inst, expert_count, ws, phist, st);
        if (rc != GRACE_OK) return rc;
        const char *failed = stable_sort_launch(table, topk_inst, n, I, 1, phist, pbase, table->R, table->N, table->d_rank_ptr,
                                                table->d_node_first_inst, inst_off, rank_off, node_off, perm_pos, perm_src,
                                                st, /*hist_ready=*/true);
        if (failed) return fail(GRACE_EHIP, "route_permute: launch of %s failed", failed);
        if (x) return launch_scatter_rows(x, T, k, d, dt, perm_pos, xp, st);
        return GRACE_OK;
    }
    const int32_t *cand_ptr = table->d_cand_ptr + (size_t)(policy == GRACE_POLICY_WRR ? table->R : local_rank) * E;
    rc = launch_topk(logits, T, E, k, renorm, topk_expert, topk_weight, (int32_t *)ws, nullptr, 0, st);
    if (rc != GRACE_OK) return rc;
    dispatch_small_kernel<<<1, SMALL_THREADS, 0, st>>>(T, E, k, rr_in, rr_out, cand_ptr, table->d_cand_g, table->d_cand_cum,
                                                      table->I, table->R, table->N, table->d_rank_ptr,
                                                      table->d_node_first_inst, topk_expert, topk_inst, expert_count,
                                                      perm_pos, perm_src, inst_off, rank_off, node_off);
    GRACE_LAUNCH_CHECK("dispatch_small_kernel");
    if (x) return launch_scatter_rows(x, T, k, d, dt, perm_pos, xp, st);
    return GRACE_OK;
}

extern "C" int grace_route_permute(const grace_table *table, int32_t local_rank, grace_policy policy, const float *logits,
                                   int32_t T, int32_t E, int32_t k, int32_t renorm, const uint32_t *rr_in,
                                   uint32_t *rr_out, int32_t *topk_expert, float *topk_weight, int32_t *topk_inst,
                                   int32_t *expert_count, const void *x, int32_t d, grace_dtype dt, int32_t *perm_pos,
                                   int32_t *perm_src, int32_t *inst_off, int32_t *rank_off, int32_t *node_off, void *xp,
                                   void *ws, void *stream) {
    int rc = check_route_args(table, local_rank, policy, logits, T, E, k, rr_in, rr_out, topk_expert, topk_weight, topk_inst,
                              expert_count, ws);
    if (rc != GRACE_OK) return rc;
    rc = check_permute_args(table, topk_inst, T, k, x, d, dt, perm_pos, perm_src, inst_off, rank_off, node_off, xp, ws);
    if (rc != GRACE_OK) return rc;
    return route_permute_impl(table, local_rank, policy, logits, T, E, k, renorm, rr_in, rr_out, topk_expert, topk_weight,
                              topk_inst, expert_count, x, d, dt, perm_pos, perm_src, inst_off, rank_off, node_off, xp, ws,
                              stream);
}

// ---- the same call for callers that cannot allocate ------------------------------------------------
// The index kernels' scratch (chunk histograms and their prefix sums) lives in a file-scope device
// array instead of a caller-provided workspace.  Every GPU the library runs on holds its own copy of
// the array at its own address until the process ends; the address is looked up once per device, with
// that device current, and from then on only that pointer is used on the host side (kernel arguments):
// the array's name itself is no device address in host code.
static __device__ __align__(256) unsigned char scratch[GRACE_STATIC_SCRATCH_BYTES];

static int static_scratch(void **out) {
    constexpr int MAX_DEVICES = 64;
    static std::mutex mu;
    static void *ptr[MAX_DEVICES] = {nullptr};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(GRACE_EHIP, "route_permute_static: hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(GRACE_EHIP, "route_permute_static: device %d not supported", dev);
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(GRACE_EHIP, "route_permute_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return GRACE_OK;
}

extern "C" int grace_route_permute_static(const grace_table *table, int32_t local_rank, grace_policy policy,
                                          const float *logits, int32_t T, int32_t E, int32_t k, int32_t renorm,
                                          const uint32_t *rr_in, uint32_t *rr_out, int32_t *topk_expert, float *topk_weight,
                                          int32_t *topk_inst, int32_t *expert_count, const void *x, int32_t d,
                                          grace_dtype dt, int32_t *perm_pos, int32_t *perm_src, int32_t *inst_off,
                                          int32_t *rank_off, int32_t *node_off, void *xp, void *stream) {
    if (!table) return fail(GRACE_EINVAL, "route_permute_static: table is null");
    void *ws = nullptr;
    int rc = static_scratch(&ws);
    if (rc != GRACE_OK) return rc;
    rc = check_route_args(table, local_rank, policy, logits, T, E, k, rr_in, rr_out, topk_expert, topk_weight, topk_inst,
                          expert_count, ws);
    if (rc != GRACE_OK) return rc;
    rc = check_permute_args(table, topk_inst, T, k, x, d, dt, perm_pos, perm_src, inst_off, rank_off, node_off, xp, ws);
    if (rc != GRACE_OK) return rc;
    const size_t need = route_permute_ws_bytes(T, E, k, table->I);
    if (need > (size_t)GRACE_STATIC_SCRATCH_BYTES)
        return fail(GRACE_ESHAPE,
                    "route_permute_static: T=%d, E=%d, k=%d, I=%d need %zu bytes of scratch, the static buffer holds %zu; "
                    "use grace_route_permute with a workspace",
                    T, E, k, table->I, need, (size_t)GRACE_STATIC_SCRATCH_BYTES);
    // nothing in the scratch has to start at zero: every kernel of the call writes the histogram
    // rows and counters it later reads (the top-k kernel clears the permutation's counters)
    return route_permute_impl(table, local_rank, policy, logits, T, E, k, renorm, rr_in, rr_out, topk_expert, topk_weight,
                              topk_inst, expert_count, x, d, dt, perm_pos, perm_src, inst_off, rank_off, node_off, xp, ws,
                              stream);
}
