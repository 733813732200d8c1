// Device routines shared by the routing kernels: the per-token top-k gate of one
// wavefront and the weighted round-robin candidate pick (Section 4.3, Algorithms 3 and 4).
#pragma once
#include "common.h"
#include "wave_utils.h"

namespace grace {

__device__ __forceinline__ uint32_t ordered_bits(float v) {
    const uint32_t u = __float_as_uint(v);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Maximum of v over the 64 lanes, as a uniform value: four butterfly steps inside each row of 16
// lanes with DPP operands (quad swaps, half-row mirror, row mirror), then the four row maxima
// through scalar registers.  All 64 lanes must be active.
template <int DPP_CTRL>
__device__ __forceinline__ uint32_t dpp_max_step(uint32_t v) {
    const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, DPP_CTRL, 0xF, 0xF, false);
    return max(v, o);
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
    v = dpp_max_step<0xB1>(v);   // quad_perm [1,0,3,2]
    v = dpp_max_step<0x4E>(v);   // quad_perm [2,3,0,1]
    v = dpp_max_step<0x141>(v);  // row_half_mirror
    v = dpp_max_step<0x140>(v);  // row_mirror
    const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 0), r1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
    const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 32), r3 = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
    return max(max(r0, r1), max(r2, r3));
}

// Sum of v over the 64 lanes, the same bits in every lane: the same butterfly with additions.
template <int DPP_CTRL>
__device__ __forceinline__ float dpp_add_step(float v) {
    const int o = __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, v), __builtin_bit_cast(int, v), DPP_CTRL, 0xF, 0xF, false);
    return v + __builtin_bit_cast(float, o);
}
__device__ __forceinline__ float wave_sum_f32(float v) {
    v = dpp_add_step<0xB1>(v);
    v = dpp_add_step<0x4E>(v);
    v = dpp_add_step<0x141>(v);
    v = dpp_add_step<0x140>(v);  // every lane of a row now holds the row's sum, added in the same order
    const int b = __builtin_bit_cast(int, v);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0)), r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32)), r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
    return (r0 + r1) + (r2 + r3);
}

// Top-k gate of one token by one wavefront, VPL experts per lane (expert e = lane + 64 v).
// Order: logit descending, equal logits by ascending expert id.  Two ways to find the k choices,
// picked by their instruction counts (the kernel is bound by vector ALU work):
//  * k rounds of arg-max: wavefront maximum of the remaining logits (as order-preserving
//    integers), the lowest expert id holding it is choice j and leaves the pool;
//  * rank by broadcast: each lane's key is broadcast through a scalar register (v_readlane) and
//    compared against the local keys, so after E broadcasts rank = number of larger keys.  Keys are
//    distinct (they include the expert id), so ranks are a permutation.
// Out: rank[v] of every local expert (any value >= k when it is not chosen) and, for ranks < k,
// its gate weight (softmax over all E logits, divided by the sum over the k chosen when renorm != 0).
template <int VPL>
__device__ __forceinline__ void token_topk(const float (&raw)[VPL], int lane, int E, int k, int renorm, int (&rank)[VPL],
                                           float (&weight)[VPL]) {
    float val[VPL];
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
        float x = raw[v];
        if (x == 0.0f) x = 0.0f;  // -0.0 and +0.0 compare equal: make them the same bits
        val[v] = x;
    }
    if (k * (18 + 8 * VPL) < 64 * VPL * (2 + 5 * VPL)) {  // uniform
        // finite logits map to integers >= 0x007FFFFF; 0 marks "no expert here" and "already chosen"
        uint32_t pool[VPL];
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
            pool[v] = (lane + 64 * v < E) ? ordered_bits(val[v]) : 0u;
            rank[v] = k;
        }
        for (int j = 0; j < k; ++j) {
            uint32_t m = pool[0];
#pragma unroll
            for (int v = 1; v < VPL; ++v) m = max(m, pool[v]);
            const uint32_t mx = wave_max_u32(m);
            bool found = false;  // uniform
#pragma unroll
            for (int v = 0; v < VPL; ++v) {
                const uint64_t hit = __ballot(pool[v] == mx);  // lowest v, then lowest lane = lowest expert id
                if (!found && hit) {
                    found = true;
                    if (lane == (int)__builtin_ctzll(hit)) {
                        rank[v] = j;
                        pool[v] = 0u;
                    }
                }
            }
        }
    } else {
        uint64_t key[VPL];
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
            const int e = lane + 64 * v;
            // larger key wins: value first, then the lower expert id
            key[v] = (e < E) ? (((uint64_t)ordered_bits(val[v]) << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)e)) : 0ull;
            rank[v] = 0;
        }
        // Lanes without an expert hold key 0, which beats nothing, so all 64 lanes of every
        // register are broadcast unconditionally and the loop unrolls with constant lane ids.
#pragma unroll
        for (int u = 0; u < VPL; ++u) {
#pragma unroll
            for (int src = 0; src < 64; ++src) {
                const uint32_t ohi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(key[u] >> 32), src);
                const uint32_t olo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)key[u], src);
                const uint64_t other = ((uint64_t)ohi << 32) | olo;
#pragma unroll
                for (int v = 0; v < VPL; ++v) rank[v] += (other > key[v]) ? 1 : 0;
            }
        }
    }
    // the maximum logit belongs to the expert of rank 0
    float mx = 0.0f;
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
        const uint64_t first = __ballot(rank[v] == 0 && lane + 64 * v < E);
        if (first) mx = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, val[v]), (int)__builtin_ctzll(first)));
    }
    float ex[VPL], den = 0.0f, sel = 0.0f;
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
        ex[v] = (lane + 64 * v < E) ? expf(val[v] - mx) : 0.0f;
        den += ex[v];
        sel += (rank[v] < k) ? ex[v] : 0.0f;
    }
    const float norm = renorm ? wave_sum_f32(sel) : wave_sum_f32(den);
#pragma unroll
    for (int v = 0; v < VPL; ++v) weight[v] = ex[v] / norm;
}

// W of Section 4.3's round-robin for expert e: the weight sum of its candidate tier.
__device__ __forceinline__ uint32_t next_rr(const uint32_t *rr_in, int e, int32_t n, const int32_t *cand_ptr,
                                            const uint32_t *cand_cum) {
    const uint32_t W = cand_cum[cand_ptr[e + 1] - 1];
    const uint64_t c = (uint64_t)(rr_in ? rr_in[e] : 0u) + (uint64_t)(uint32_t)n;
    return (uint32_t)(c % W);
}

// Request number c of expert e -> instance: the candidate of e's tier (ascending rank) whose
// cumulative polling-weight interval contains c mod W.
__device__ __forceinline__ int32_t pick_candidate(uint64_t c, int e, const int32_t *__restrict__ cand_ptr,
                                                  const int32_t *__restrict__ cand_g,
                                                  const uint32_t *__restrict__ cand_cum) {
    const int cb = cand_ptr[e], ce = cand_ptr[e + 1];
    const uint32_t W = cand_cum[ce - 1];
    const uint32_t q = (c >> 32) ? (uint32_t)(c % W) : ((uint32_t)c % W);
    int s = cb;
    while (s < ce - 1 && cand_cum[s] <= q) ++s;
    return cand_g[s];
}

}  // namespace grace
