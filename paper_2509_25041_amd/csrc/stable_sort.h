// Stable counting sort of small integer keys over chunks of assignments: the
// building block of the dispatch permutation and of the per-destination send lists.
//   key_hist_kernel   histogram of keys per chunk of PERM_CHUNK items
//   key_scan_kernel   per-key exclusive scan over chunks, exclusive scan over keys
//   key_pos_kernel    one wavefront per chunk: stable rank of each item among equal
//                     keys (ballot matching) -> position of every item and its inverse
// Keys outside [0, nkeys) are skipped (position -1).  No atomics that affect order.
#pragma once
#include "common.h"
#include "wave_utils.h"

namespace grace {


static __global__ __launch_bounds__(64) void key_hist_kernel(const int32_t *__restrict__ topk_inst, int64_t n_assign, int I,
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

static __global__ __launch_bounds__(SCAN_THREADS) void key_scan_kernel(const int32_t *__restrict__ hist,
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
    if (rank_off)
        for (int r = tid; r <= R; r += SCAN_THREADS) rank_off[r] = totals[rank_ptr[r]];
    if (node_off)
        for (int n = tid; n <= N; n += SCAN_THREADS) node_off[n] = totals[node_first_inst[n]];
}

static __global__ __launch_bounds__(64) void key_pos_kernel(const int32_t *__restrict__ topk_inst, int64_t n_assign, int I,
                                                      const int32_t *__restrict__ chunk_base,
                                                      const int32_t *__restrict__ inst_off,
                                                      int32_t *__restrict__ perm_pos, int32_t *__restrict__ perm_src,
                                                      int nbits, int src_div) {
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
            perm_src[pos] = (int32_t)(a / src_div);  // src_div = 1: the item itself; k: its token
        } else if (in) {
            perm_pos[a] = -1;  // id outside the table: no row
        }
        __syncthreads();
        if (valid && is_last_of(same)) cnt[g] += (int32_t)__popcll(same);
        __syncthreads();
    }
}


}  // namespace grace
