// grace_permute: stable counting sort of the assignments by instance id
// (= node, rank, slot: the two-stage dispatch order of Section 5) and the row
// movement into that order.
//
//   1. inst_hist_kernel   histogram of instance ids per chunk of 512 assignments
//   2. perm_scan_kernel   per-id exclusive scan over chunks, exclusive scan over
//                         ids -> inst_off / rank_off / node_off
//   3. perm_pos_kernel    one wavefront per chunk: stable rank of each assignment
//                         among equal ids (ballot matching) -> perm_pos, perm_src
//   4. scatter_rows_kernel one block per token: read the token row once, write it
//                         to its k buffer positions with 16-byte accesses
#include "bf16.h"
#include "common.h"
#include "wave_utils.h"

namespace grace {

__global__ __launch_bounds__(64) void inst_hist_kernel(const int32_t *__restrict__ topk_inst, int64_t n_assign, int I,
                                                       int32_t *__restrict__ chunk_hist) {
    __shared__ int32_t hist[GRACE_MAX_INSTANCES];
    const int lane = (int)threadIdx.x;
    const int chunk = (int)blockIdx.x;
    for (int i = lane; i < I; i += 64) hist[i] = 0;
    __syncthreads();
    const int64_t a0 = (int64_t)chunk * PERM_CHUNK;
    const int64_t a1 = min(n_assign, a0 + PERM_CHUNK);
    for (int64_t a = a0 + lane; a < a1; a += 64) {
        const int g = topk_inst[a];
        if ((unsigned)g < (unsigned)I) atomicAdd(&hist[g], 1);
    }
    __syncthreads();
    for (int i = lane; i < I; i += 64) chunk_hist[(size_t)chunk * I + i] = hist[i];
}

__global__ __launch_bounds__(SCAN_THREADS) void perm_scan_kernel(const int32_t *__restrict__ hist,
                                                                 int32_t *__restrict__ base, int nchunks, int I, int R,
                                                                 int N, const int32_t *__restrict__ rank_ptr,
                                                                 const int32_t *__restrict__ node_first_inst,
                                                                 int32_t *__restrict__ inst_off,
                                                                 int32_t *__restrict__ rank_off,
                                                                 int32_t *__restrict__ node_off) {
    __shared__ int32_t totals[GRACE_MAX_INSTANCES + 1];
    __shared__ int32_t part_sums[SCAN_THREADS];
    const int tid = (int)threadIdx.x;
    for (int i = tid; i <= I; i += SCAN_THREADS) totals[i] = 0;
    __syncthreads();
    block_scan_chunks(hist, base, nchunks, I, totals, part_sums);
    __syncthreads();
    // exclusive scan over ids by the first wavefront: each lane owns a contiguous run
    if (tid < 64) {
        const int per = (I + 63) / 64;
        const int lo = min(I, tid * per), hi = min(I, lo + per);
        int32_t s = 0;
        for (int i = lo; i < hi; ++i) s += totals[i];
        int32_t incl = s;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int32_t v = __shfl_up(incl, o, 64);
            if (tid >= o) incl += v;
        }
        int32_t run = incl - s;
        for (int i = lo; i < hi; ++i) {
            const int32_t c = totals[i];
            totals[i] = run;
            run += c;
        }
        if (tid == 63) totals[I] = incl;  // lane 63 holds the grand total
    }
    __syncthreads();
    for (int i = tid; i <= I; i += SCAN_THREADS) inst_off[i] = totals[i];
    for (int r = tid; r <= R; r += SCAN_THREADS) rank_off[r] = totals[rank_ptr[r]];
    for (int n = tid; n <= N; n += SCAN_THREADS) node_off[n] = totals[node_first_inst[n]];
}

__global__ __launch_bounds__(64) void perm_pos_kernel(const int32_t *__restrict__ topk_inst, int64_t n_assign, int I,
                                                      const int32_t *__restrict__ chunk_base,
                                                      const int32_t *__restrict__ inst_off,
                                                      int32_t *__restrict__ perm_pos, int32_t *__restrict__ perm_src,
                                                      int nbits) {
    __shared__ int32_t cnt[GRACE_MAX_INSTANCES];
    const int lane = (int)threadIdx.x;
    const int chunk = (int)blockIdx.x;
    for (int i = lane; i < I; i += 64) cnt[i] = inst_off[i] + chunk_base[(size_t)chunk * I + i];
    __syncthreads();
    const int64_t a0 = (int64_t)chunk * PERM_CHUNK;
    const int64_t a1 = min(n_assign, a0 + PERM_CHUNK);
    const uint64_t lt = lanemask_lt();
    for (int64_t b = a0; b < a1; b += 64) {
        const int64_t a = b + lane;
        const bool in = a < a1;
        const int g = in ? topk_inst[a] : 0;
        const bool valid = in && (unsigned)g < (unsigned)I;
        const uint64_t same = wave_match((uint32_t)g, valid, nbits);
        if (valid) {
            const int32_t pos = cnt[g] + (int32_t)__popcll(same & lt);
            perm_pos[a] = pos;
            perm_src[pos] = (int32_t)a;
        } else if (in) {
            perm_pos[a] = -1;  // id outside the table: no row
        }
        __syncthreads();
        if (valid && is_last_of(same)) cnt[g] += (int32_t)__popcll(same);
        __syncthreads();
    }
}

// One block per token: the row is read once and written k times.
__global__ __launch_bounds__(256) void scatter_rows_kernel(const uint4 *__restrict__ x, int k, int row_vec,
                                                           int64_t n_assign, const int32_t *__restrict__ perm_pos,
                                                           uint4 *__restrict__ xp) {
    const int64_t t = blockIdx.x;
    const uint4 *src = x + t * row_vec;
    for (int c = (int)threadIdx.x; c < row_vec; c += 256) {
        const uint4 v = src[c];
        for (int j = 0; j < k; ++j) {
            const int32_t p = perm_pos[t * k + j];
            if (p >= 0 && p < n_assign) nt_store16(v, &xp[(int64_t)p * row_vec + c]);
        }
    }
}

}  // namespace grace

using namespace grace;

extern "C" int grace_permute(const grace_table *table, const int32_t *topk_inst, int32_t T, int32_t k, const void *x,
                             int32_t d, grace_dtype dt, int32_t *perm_pos, int32_t *perm_src, int32_t *inst_off,
                             int32_t *rank_off, int32_t *node_off, void *xp, void *ws, void *stream) {
    if (!table) return fail(GRACE_EINVAL, "permute: table is null");
    if (T < 0 || k < 1) return fail(GRACE_EINVAL, "permute: T=%d, k=%d invalid", T, k);
    if ((int64_t)T * k > INT32_MAX) return fail(GRACE_ESHAPE, "permute: T*k exceeds 2^31-1");
    if (dt != GRACE_F32 && dt != GRACE_BF16) return fail(GRACE_EINVAL, "permute: unknown dtype %d", (int)dt);
    if (!inst_off || !rank_off || !node_off || !ws) return fail(GRACE_EINVAL, "permute: null offset or ws pointer");
    if (T > 0 && (!topk_inst || !perm_pos || !perm_src)) return fail(GRACE_EINVAL, "permute: null device pointer");
    const size_t el = dt == GRACE_F32 ? 4 : 2;
    if (x) {
        if (d < 1) return fail(GRACE_EINVAL, "permute: d=%d invalid", d);
        if (((size_t)d * el) % 16 != 0) return fail(GRACE_ESHAPE, "permute: row of %zu bytes is not a multiple of 16", (size_t)d * el);
        if (T > 0 && !xp) return fail(GRACE_EINVAL, "permute: xp is null");
        if ((((uintptr_t)x) | ((uintptr_t)xp)) & 15) return fail(GRACE_EINVAL, "permute: x and xp must be 16-byte aligned");
    }
    hipStream_t st = (hipStream_t)stream;
    const int I = table->I;
    const int64_t n = (int64_t)T * k;
    const int nchunks = (int)ceil_div(n, PERM_CHUNK);
    int32_t *hist = (int32_t *)ws;
    int32_t *base = (int32_t *)((char *)ws + align_up((size_t)nchunks * I * 4, 256));
    int nbits = 0;
    while ((1 << nbits) < I) ++nbits;
    if (nchunks > 0) {
        inst_hist_kernel<<<nchunks, 64, 0, st>>>(topk_inst, n, I, hist);
        GRACE_LAUNCH_CHECK("inst_hist_kernel");
    }
    perm_scan_kernel<<<1, SCAN_THREADS, 0, st>>>(hist, base, nchunks, I, table->R, table->N, table->d_rank_ptr,
                                                 table->d_node_first_inst, inst_off, rank_off, node_off);
    GRACE_LAUNCH_CHECK("perm_scan_kernel");
    if (nchunks > 0) {
        perm_pos_kernel<<<nchunks, 64, 0, st>>>(topk_inst, n, I, base, inst_off, perm_pos, perm_src, nbits);
        GRACE_LAUNCH_CHECK("perm_pos_kernel");
        if (x) {
            scatter_rows_kernel<<<T, 256, 0, st>>>((const uint4 *)x, k, (int)((size_t)d * el / 16), n, perm_pos,
                                                   (uint4 *)xp);
            GRACE_LAUNCH_CHECK("scatter_rows_kernel");
        }
    }
    return GRACE_OK;
}
