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

// Top-k gate of one token by one wavefront, VPL experts per lane (expert e = lane + 64 v).
// Instead of k rounds of arg-max, every lane learns the rank of its own logits: each lane's key is
// broadcast through a scalar register (v_readlane) and compared against the local keys, so after
// E broadcasts rank = number of larger keys.  Keys are distinct (they include the expert id), so
// ranks are a permutation and the expert with rank j < k is the token's j-th choice.
// Out: rank[v] of every local expert and, for ranks < k, its gate weight (softmax over all E
// logits, divided by the sum over the k chosen when renorm != 0).
template <int VPL>
__device__ __forceinline__ void token_topk(const float (&raw)[VPL], int lane, int E, int k, int renorm, int (&rank)[VPL],
                                           float (&weight)[VPL]) {
    float val[VPL];
    uint64_t key[VPL];
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
        const int e = lane + 64 * v;
        float x = raw[v];
        if (x == 0.0f) x = 0.0f;  // -0.0 and +0.0 compare equal: make them the same bits
        val[v] = x;
        // larger key wins: value first, then the lower expert id
        key[v] = (e < E) ? (((uint64_t)ordered_bits(x) << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)e)) : 0ull;
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
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        den += __shfl_xor(den, o, 64);
        sel += __shfl_xor(sel, o, 64);
    }
    const float norm = renorm ? sel : den;
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
