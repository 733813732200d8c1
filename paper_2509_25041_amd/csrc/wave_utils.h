// Wavefront-level (64 lanes) helpers used by the routing and permutation kernels.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

namespace grace {

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63u); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)v, o, 64);
        uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(v >> 32), o, 64);
        uint64_t w = ((uint64_t)hi << 32) | lo;
        v = w > v ? w : v;
    }
    return v;
}

// Lanes holding the same key as this lane (among lanes with valid == true).
// nbits = number of significant key bits.  The result is meaningless for
// lanes with valid == false.
__device__ __forceinline__ uint64_t wave_match(uint32_t key, bool valid, int nbits) {
    uint64_t m = __ballot(valid);
    for (int b = 0; b < nbits; ++b) {
        const bool bit = (key >> b) & 1u;
        const uint64_t bal = __ballot(bit);
        m &= bit ? bal : ~bal;
    }
    return m;
}
__device__ __forceinline__ uint64_t lanemask_lt() { return (1ull << lane_id()) - 1ull; }
// true for the highest lane of a match set
__device__ __forceinline__ bool is_last_of(uint64_t same) {
    const int l = lane_id();
    const uint64_t above = (l == 63) ? 0ull : (same >> (l + 1));
    return above == 0ull;
}
// LDS counters that one wavefront updates in one round of a loop and reads in the next (the highest
// lane of a match set adds the set's size; other lanes read the counter a round later).  LDS
// operations of one wavefront execute in program order; relaxed atomic accesses (plain ds_read /
// ds_write on this target) with a wavefront-scope fence between the rounds make that hand-over
// defined for the compiler as well.
template <typename T>
__device__ __forceinline__ T wave_ctr_load(const T *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
}
template <typename T>
__device__ __forceinline__ void wave_ctr_add(T *p, T v) {
    __hip_atomic_store(p, (T)(__hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT) + v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_WAVEFRONT);
}
__device__ __forceinline__ void wave_ctr_fence() { __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); }

__device__ __forceinline__ int bits_for(int nkeys) {
    int b = 0;
    while ((1 << b) < nkeys) ++b;
    return b;
}

// Column sums of rows [r0, r1) of a row-major [rows][nkeys] int32 matrix, added into acc[nkeys] (LDS,
// initialised by the caller, who also synchronises before reading it) by a block of NT threads.
// With `acc_lt` the rows below r_lt are also summed into acc_lt[nkeys].
// The rows are read as a flat array in groups of whole rows of at most 4 * NT elements: a thread
// reads four consecutive elements of every group (one 16-byte load where the alignment allows it),
// always of the same four columns, so it sums in registers and adds to LDS once at the end; all
// lanes are busy whatever nkeys is.  Integer sums: exact in any order.  `m` must be 16-byte aligned.
template <int NT>
__device__ __forceinline__ void block_add_rows(const int32_t *__restrict__ m, int r0, int r1, int nkeys, int32_t *acc, int tid,
                                               int32_t *acc_lt = nullptr, int r_lt = 0) {
    if (r1 <= r0) return;
    const int rg = (4 * NT) / nkeys;  // rows per group
    if (rg == 0) {
        // rows longer than a group: a thread owns columns tid, tid + NT, ... and walks the rows
        for (int key = tid; key < nkeys; key += NT) {
            int32_t tot = 0, lt = 0;
#pragma unroll 8
            for (int r = r0; r < r1; ++r) {
                const int32_t v = m[(size_t)r * nkeys + key];
                tot += v;
                lt += (r < r_lt) ? v : 0;
            }
            if (tot) atomicAdd(&acc[key], tot);
            if (acc_lt && lt) atomicAdd(&acc_lt[key], lt);
        }
        return;
    }
    const int gs = rg * nkeys;        // elements per group, <= 4 * NT
    const int o = 4 * tid;            // this thread's elements of a group: o .. o + 3
    if (o >= gs) return;
    int key[4], row[4];
    bool on[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        on[q] = o + q < gs;
        row[q] = (o + q) / nkeys;
        key[q] = (o + q) - row[q] * nkeys;
    }
    const int64_t s0 = (int64_t)r0 * nkeys, s1 = (int64_t)r1 * nkeys;
    const bool vec = (s0 % 4 == 0) && (gs % 4 == 0);  // then every group start and o are multiples of four elements
    const int ngroups = (r1 - r0 + rg - 1) / rg;
    int32_t tot[4] = {0, 0, 0, 0}, lt[4] = {0, 0, 0, 0};
    auto add = [&](const int32_t (&v)[4], int grp) {
        const int rbase = r0 + grp * rg;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            tot[q] += v[q];
            lt[q] += (rbase + row[q] < r_lt) ? v[q] : 0;
        }
    };
    // every group but the last lies wholly below s1: batches of 8 and 4 unguarded 16-byte loads, all of a
    // batch in flight before the first is used
    auto batch = [&](int grp, auto nb) {
        constexpr int NB = decltype(nb)::value;
        uint4 x[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) x[b] = *(const uint4 *)(m + s0 + (int64_t)(grp + b) * gs + o);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int32_t v[4] = {(int32_t)x[b].x, (int32_t)x[b].y, (int32_t)x[b].z, (int32_t)x[b].w};
            add(v, grp + b);
        }
    };
    int grp = 0;
    if (vec) {
        for (; grp + 8 < ngroups; grp += 8) batch(grp, std::integral_constant<int, 8>{});
        if (grp + 4 < ngroups) {
            batch(grp, std::integral_constant<int, 4>{});
            grp += 4;
        }
    }
#pragma unroll 4
    for (; grp < ngroups; ++grp) {
        const int64_t f = s0 + (int64_t)grp * gs + o;  // flat index of this thread's first element
        int32_t v[4] = {0, 0, 0, 0};
        if (vec && f + 3 < s1) {
            const uint4 x = *(const uint4 *)(m + f);
            v[0] = (int32_t)x.x; v[1] = (int32_t)x.y; v[2] = (int32_t)x.z; v[3] = (int32_t)x.w;
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (on[q] && f + q < s1) v[q] = m[f + q];
        }
        add(v, grp);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (on[q] && tot[q]) atomicAdd(&acc[key[q]], tot[q]);
        if (acc_lt && on[q] && lt[q]) atomicAdd(&acc_lt[key[q]], lt[q]);
    }
}

// Two-level histogram sums: the chunk rows are grouped into super-chunks of FOLD_SUPER rows whose
// column sums super_sum_kernel writes; a block then needs the super rows before its super-chunk and
// the chunk rows inside it instead of every row before its chunk.
constexpr int FOLD_SUPER = 64;
constexpr int SUPER_THREADS = 512;
static __global__ __launch_bounds__(SUPER_THREADS) void super_sum_kernel(const int32_t *__restrict__ hist, int nchunks,
                                                                        int nkeys, int32_t *__restrict__ super_tot) {
    __shared__ int32_t acc[4096];  // the largest key count of any caller (instances)
    const int tid = (int)threadIdx.x, s = (int)blockIdx.x;
    for (int i = tid; i < nkeys; i += SUPER_THREADS) acc[i] = 0;
    __syncthreads();
    block_add_rows<SUPER_THREADS>(hist, s * FOLD_SUPER, min(nchunks, (s + 1) * FOLD_SUPER), nkeys, acc, tid);
    __syncthreads();
    for (int i = tid; i < nkeys; i += SUPER_THREADS) super_tot[(size_t)s * nkeys + i] = acc[i];
}

// Exclusive scan over chunks of a [nchunks][nkeys] histogram, per key:
// base[c][key] = sum_{c' < c} hist[c'][key]; totals[key] = column sum (LDS or
// global array of nkeys entries).  Must be called by a whole block of
// SCAN_THREADS threads; `part_sums` is LDS of SCAN_PARTS * SCAN_KW ints.
constexpr int SCAN_THREADS = 1024;
constexpr int SCAN_KW = 64;
constexpr int SCAN_PARTS = SCAN_THREADS / SCAN_KW;

__device__ inline void block_scan_chunks(const int32_t *__restrict__ hist, int32_t *__restrict__ base, int nchunks,
                                         int nkeys, int32_t *totals, int32_t *part_sums) {
    const int tid = (int)threadIdx.x;
    const int kl = tid % SCAN_KW, part = tid / SCAN_KW;
    const int per = (nchunks + SCAN_PARTS - 1) / SCAN_PARTS;
    const int c_lo = min(nchunks, part * per), c_hi = min(nchunks, c_lo + per);
    for (int k0 = 0; k0 < nkeys; k0 += SCAN_KW) {
        const int key = k0 + kl;
        int32_t sum = 0;
        if (key < nkeys)
            for (int c = c_lo; c < c_hi; ++c) sum += hist[(size_t)c * nkeys + key];
        part_sums[part * SCAN_KW + kl] = sum;
        __syncthreads();
        int32_t run = 0;
        for (int p = 0; p < part; ++p) run += part_sums[p * SCAN_KW + kl];
        if (key < nkeys) {
            if (part == SCAN_PARTS - 1) totals[key] = run + sum;
            for (int c = c_lo; c < c_hi; ++c) {
                const size_t i = (size_t)c * nkeys + key;
                base[i] = run;
                run += hist[i];
            }
        }
        __syncthreads();
    }
}

}  // namespace grace
