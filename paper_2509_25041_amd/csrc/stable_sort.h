// Stable counting sort of small integer keys over chunks of assignments: the
// building block of the dispatch permutation and of the per-destination send lists.
//   key_hist_kernel   histogram of keys per chunk of PERM_CHUNK items
//   key_scan_kernel   per-key exclusive scan over chunks, exclusive scan over keys
//   key_pos_kernel    one wavefront per chunk: stable rank of each item among equal
//                     keys (ballot matching) -> position of every item and its inverse
//   key_pos_fold_kernel  the last two in one launch when there are few chunks
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

// One wavefront ranks the items of its chunk in order: cnt[key] (LDS) holds the position of the
// next item with that key; equal keys inside a group of 64 items are ranked by ballot matching.
// The LDS operations of one wavefront execute in program order, so a counter updated by the last
// lane of a match set is seen by the next group of 64 items without a barrier.
// The chunk's keys are fetched up front (load_chunk_keys, before the counters are prepared), so
// the ranking rounds do not each wait for a load.
constexpr int CHUNK_ROUNDS = PERM_CHUNK / 64;

__device__ __forceinline__ void load_chunk_keys(const int32_t *__restrict__ keys, int64_t n_items, int chunk, int lane,
                                                int (&g)[CHUNK_ROUNDS]) {
    const int64_t a0 = (int64_t)chunk * PERM_CHUNK;
#pragma unroll
    for (int q = 0; q < CHUNK_ROUNDS; ++q) {
        const int64_t a = a0 + q * 64 + lane;
        g[q] = a < n_items ? keys[a] : -1;
    }
}

__device__ __forceinline__ void rank_chunk(const int (&g_in)[CHUNK_ROUNDS], int64_t n_items, int nkeys, int32_t *cnt,
                                           int32_t *__restrict__ perm_pos, int32_t *__restrict__ perm_src, int nbits,
                                           int src_div, int chunk, int lane) {
    const int64_t a0 = (int64_t)chunk * PERM_CHUNK;
    const int64_t a1 = min(n_items, a0 + PERM_CHUNK);
    const uint64_t lt = lanemask_lt();
#pragma unroll
    for (int q = 0; q < CHUNK_ROUNDS; ++q) {
        const int64_t a = a0 + q * 64 + lane;
        if (a0 + q * 64 >= a1) break;  // uniform
        const bool in = a < a1;
        const int g = in ? g_in[q] : 0;
        const bool valid = in && (unsigned)g < (unsigned)nkeys;
        const uint64_t same = wave_match((uint32_t)g, valid, nbits);
        if (valid) {
            const int32_t pos = wave_ctr_load(&cnt[g]) + (int32_t)__popcll(same & lt);
            perm_pos[a] = pos;
            perm_src[pos] = (int32_t)(a / src_div);  // src_div = 1: the item itself; k: its token
        } else if (in) {
            perm_pos[a] = -1;  // key outside the table: no row
        }
        if (valid && is_last_of(same)) wave_ctr_add(&cnt[g], (int32_t)__popcll(same));
        wave_ctr_fence();
    }
}

static __global__ __launch_bounds__(64) void key_pos_kernel(const int32_t *__restrict__ topk_inst, int64_t n_assign, int I,
                                                      const int32_t *__restrict__ chunk_base,
                                                      const int32_t *__restrict__ inst_off,
                                                      int32_t *__restrict__ perm_pos, int32_t *__restrict__ perm_src,
                                                      int nbits, int src_div) {
    __shared__ int32_t cnt[GRACE_MAX_INSTANCES];
    const int lane = (int)threadIdx.x;
    const int chunk = (int)blockIdx.x;
    int g[CHUNK_ROUNDS];
    load_chunk_keys(topk_inst, n_assign, chunk, lane, g);
    for (int i = lane; i < I; i += 64) cnt[i] = inst_off[i] + chunk_base[(size_t)chunk * I + i];
    __syncthreads();
    rank_chunk(g, n_assign, I, cnt, perm_pos, perm_src, nbits, src_div, chunk, lane);
}

// The scan folded into the position kernel: every block derives its offsets from the chunk
// histograms itself (totals over all chunks -> exclusive scan over keys, plus the counts of the
// chunks before its own), which saves the single-block scan launch; block 0 also writes the offset
// outputs.  With super_tot (column sums per FOLD_SUPER chunk rows) the block reads the super rows
// and the chunk rows of its own super-chunk instead of every row.
// Ranking: with at most POS_PAR_KEYS keys every wavefront ranks 64 of the chunk's items at once
// (match sets by ballot, their sizes in the wavefront's row of wcnt, an exclusive scan over the
// eight rows on top of the chunk's start positions); with more keys wavefront 0 walks the chunk.
constexpr int POS_FOLD_THREADS = 512, POS_WAVES = POS_FOLD_THREADS / 64;
constexpr int POS_PAR_KEYS = 512;
static_assert(PERM_CHUNK == POS_FOLD_THREADS, "one item per thread when all wavefronts rank");

static __global__ __launch_bounds__(POS_FOLD_THREADS) void key_pos_fold_kernel(
    const int32_t *__restrict__ keys, int64_t n_items, int I, const int32_t *__restrict__ chunk_hist, int nchunks, int R,
    int N, const int32_t *__restrict__ rank_ptr, const int32_t *__restrict__ node_first_inst,
    int32_t *__restrict__ inst_off, int32_t *__restrict__ rank_off, int32_t *__restrict__ node_off,
    int32_t *__restrict__ perm_pos, int32_t *__restrict__ perm_src, int nbits, int src_div,
    const int32_t *__restrict__ super_tot) {
    __shared__ int32_t cnt[GRACE_MAX_INSTANCES];      // items of each key in the chunks before this one, then positions
    __shared__ int32_t off[GRACE_MAX_INSTANCES + 1];  // items of each key in all chunks, then exclusive offsets
    __shared__ int32_t wcnt[POS_WAVES][POS_PAR_KEYS];
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = (int)blockIdx.x;
    const bool par = I <= POS_PAR_KEYS;  // uniform
    int g[CHUNK_ROUNDS];
    int g_one = -1;
    const int64_t a_one = (int64_t)chunk * PERM_CHUNK + tid;
    if (par) g_one = a_one < n_items ? keys[a_one] : -1;          // in flight while the histograms are summed
    else if (wave == 0) load_chunk_keys(keys, n_items, chunk, lane, g);
    for (int i = tid; i < I; i += POS_FOLD_THREADS) {
        cnt[i] = 0;
        off[i] = 0;
    }
    __syncthreads();
    if (super_tot) {
        const int s = chunk / FOLD_SUPER, nsuper = (nchunks + FOLD_SUPER - 1) / FOLD_SUPER;
        block_add_rows<POS_FOLD_THREADS>(super_tot, 0, nsuper, I, off, tid, cnt, s);
        block_add_rows<POS_FOLD_THREADS>(chunk_hist, s * FOLD_SUPER, chunk, I, cnt, tid);
    } else {
        // one pass over all rows gives both sums
        block_add_rows<POS_FOLD_THREADS>(chunk_hist, 0, nchunks, I, off, tid, cnt, chunk);
    }
    __syncthreads();
    if (wave == 0) {
        int32_t carry = 0;
        for (int k0 = 0; k0 < I; k0 += 64) {
            const int key = k0 + lane;
            const int32_t tot = key < I ? off[key] : 0;
            int32_t incl = tot;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int32_t v = __shfl_up(incl, o, 64);
                if (lane >= o) incl += v;
            }
            if (key < I) {
                off[key] = carry + incl - tot;
                cnt[key] += carry + incl - tot;
            }
            carry += __shfl(incl, 63, 64);
        }
        if (lane == 0) off[I] = carry;
        if (chunk == 0) {
            for (int i = lane; i <= I; i += 64) inst_off[i] = off[i];
            if (rank_off)
                for (int r = lane; r <= R; r += 64) rank_off[r] = off[rank_ptr[r]];
            if (node_off)
                for (int n = lane; n <= N; n += 64) node_off[n] = off[node_first_inst[n]];
        }
        if (!par) rank_chunk(g, n_items, I, cnt, perm_pos, perm_src, nbits, src_div, chunk, lane);
    }
    if (!par) return;
    // every wavefront ranks its 64 items: cnt[key] is the position of the chunk's first item with that key
    const bool in = a_one < n_items;
    const bool valid = in && (unsigned)g_one < (unsigned)I;
    const int key = valid ? g_one : 0;
    for (int i = lane; i < I; i += 64) wcnt[wave][i] = 0;  // this wavefront's row; its LDS operations execute in order
    const uint64_t same = wave_match((uint32_t)key, valid, nbits);
    if (valid && is_last_of(same)) wcnt[wave][key] = (int32_t)__popcll(same);
    __syncthreads();  // also: wavefront 0 has finished cnt
    for (int i = tid; i < I; i += POS_FOLD_THREADS) {
        int32_t run = cnt[i];
#pragma unroll
        for (int w = 0; w < POS_WAVES; ++w) {
            const int32_t c = wcnt[w][i];
            wcnt[w][i] = run;
            run += c;
        }
    }
    __syncthreads();
    if (valid) {
        const int32_t pos = wcnt[wave][key] + (int32_t)__popcll(same & lanemask_lt());
        perm_pos[a_one] = pos;
        perm_src[pos] = (int32_t)(a_one / src_div);  // src_div = 1: the item itself; k: its token
    } else if (in) {
        perm_pos[a_one] = -1;  // key outside the table: no row
    }
}

// Host side: the launches of one stable counting sort.  hist / base: workspace of nchunks * nkeys
// ints each.  rank_ptr .. node_off may be null (plain sort: only `off` is produced).
// hist_ready: an earlier kernel on the stream already wrote the chunk histograms into `hist`.
static inline const char *stable_sort_launch(const grace_table *table, const int32_t *keys, int64_t n, int nkeys, int src_div, int32_t *hist,
                                             int32_t *base, int R, int N, const int32_t *rank_ptr,
                                             const int32_t *node_first_inst, int32_t *off, int32_t *rank_off,
                                             int32_t *node_off, int32_t *pos, int32_t *src, hipStream_t st,
                                             bool hist_ready = false) {
    const int nchunks = (int)ceil_div(n, PERM_CHUNK);
    int nbits = 0;
    while ((1 << nbits) < nkeys) ++nbits;
    if (nchunks > 0 && !hist_ready) {
        key_hist_kernel<<<nchunks, 64, 0, st>>>(keys, n, nkeys, hist);
        if (hipGetLastError() != hipSuccess) return "key_hist_kernel";
    }
    const int mode = fold_mode(table, nchunks, nkeys);
    if (mode != 0) {
        const int32_t *super_tot = nullptr;
        if (mode == 2) {  // column sums per super-chunk of rows, into the (otherwise unused) scan buffer
            super_sum_kernel<<<(unsigned)ceil_div(nchunks, FOLD_SUPER), SUPER_THREADS, 0, st>>>(hist, nchunks, nkeys, base);
            if (hipGetLastError() != hipSuccess) return "super_sum_kernel";
            super_tot = base;
        }
        key_pos_fold_kernel<<<nchunks, POS_FOLD_THREADS, 0, st>>>(keys, n, nkeys, hist, nchunks, R, N, rank_ptr, node_first_inst, off,
                                                    rank_off, node_off, pos, src, nbits, src_div, super_tot);
        if (hipGetLastError() != hipSuccess) return "key_pos_fold_kernel";
        return nullptr;
    }
    key_scan_kernel<<<1, SCAN_THREADS, 0, st>>>(hist, base, nchunks, nkeys, R, N, rank_ptr, node_first_inst, off, rank_off,
                                                 node_off);
    if (hipGetLastError() != hipSuccess) return "key_scan_kernel";
    if (nchunks > 0) {
        key_pos_kernel<<<nchunks, 64, 0, st>>>(keys, n, nkeys, base, off, pos, src, nbits, src_div);
        if (hipGetLastError() != hipSuccess) return "key_pos_kernel";
    }
    return nullptr;
}


}  // namespace grace
