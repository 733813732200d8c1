// Arguments and tile location shared by the grouped GEMM kernels.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace grace {

struct GemmArgs {
    const void *A;          // activations, row p at A + p * lda
    int64_t lda;
    const void *B0;         // weights [S][N][ldb...]; B1 = second matrix of the fused up projection
    const void *B1;
    int64_t b_slot_stride;  // elements between the weights of consecutive slots
    int64_t ldb;            // elements between weight rows
    int N, K;
    int kseg_len;           // weight K axis split in segments of this length ...
    int64_t kseg_stride;    // ... that lie this many elements apart (shared experts' down projection)
    void *out;              // output rows, row p at out + p * ldo
    int64_t ldo;
    const int32_t *seg_off; // device: S+1 row offsets of the local slots, or null
    int S;
    int M_single;           // rows of the single segment when seg_off is null
};

// Which (slot, row range) does m-tile `mt` fall into?  Returns false for surplus tiles.
template <int BM>
__device__ __forceinline__ bool locate_tile(const GemmArgs &g, int mt, int &slot, int &m0, int &m_end) {
    if (!g.seg_off) {
        slot = 0;
        m0 = mt * BM;
        m_end = g.M_single;
        return m0 < m_end;
    }
    int acc = 0;
    for (int s = 0; s < g.S; ++s) {
        const int lo = g.seg_off[s], hi = g.seg_off[s + 1];
        const int tiles = (hi - lo + BM - 1) / BM;
        if (mt < acc + tiles) {
            slot = s;
            m0 = lo + (mt - acc) * BM;
            m_end = hi;
            return true;
        }
        acc += tiles;
    }
    return false;
}

// Row segments (one per local expert slot) cut into m-tiles of BM rows, held in registers by every
// wavefront: lane l keeps segments SPL * l .. SPL * l + SPL - 1 (so at most 64 * SPL segments) and
// the index of their first m-tile.  A tile's segment is found with a ballot; no table in memory.
struct Tile {
    int slot, m0, m_end;  // segment, first row, end of the segment
};

template <int BM, int SPL>
struct SegTable {
    int lo[SPL], hi[SPL], base[SPL];
    int total;  // m-tiles over all segments (scalar)

    __device__ __forceinline__ void init(const GemmArgs &g, int lane) {
        int lane_tiles = 0;
#pragma unroll
        for (int q = 0; q < SPL; ++q) {
            const int s = lane * SPL + q;
            int l = 0, h = 0;
            if (g.seg_off) {
                if (s < g.S) { l = g.seg_off[s]; h = max(l, g.seg_off[s + 1]); }
            } else if (s == 0) {
                h = g.M_single;
            }
            lo[q] = l;
            hi[q] = h;
            base[q] = lane_tiles;                 // made global below
            lane_tiles += (h - l + BM - 1) / BM;  // h >= l
        }
        int incl = lane_tiles;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int up = __shfl_up(incl, o, 64);
            if (lane >= o) incl += up;
        }
        const int lane_base = incl - lane_tiles;
#pragma unroll
        for (int q = 0; q < SPL; ++q) base[q] += lane_base;
        total = __builtin_amdgcn_readlane(incl, 63);
    }

    // (slot, first row, segment end) of m-tile mt < total, as scalars
    __device__ __forceinline__ Tile lookup(int mt, int lane) const {
        int slot = 0, m0 = 0, m_end = 0;
        bool hit = false;
#pragma unroll
        for (int q = 0; q < SPL; ++q) {
            const int rel = mt - base[q];
            const int tiles = (hi[q] - lo[q] + BM - 1) / BM;
            if (rel >= 0 && rel < tiles) {
                hit = true;
                slot = lane * SPL + q;
                m0 = lo[q] + rel * BM;
                m_end = hi[q];
            }
        }
        const unsigned long long owners = __ballot(hit);
        const int src = owners ? __builtin_ctzll(owners) : 0;
        Tile t;
        t.slot = __builtin_amdgcn_readlane(slot, src);
        t.m0 = __builtin_amdgcn_readlane(m0, src);
        t.m_end = __builtin_amdgcn_readlane(m_end, src);
        return t;
    }
};

__device__ __forceinline__ int64_t koff(const GemmArgs &g, int kk) {
    return (int64_t)(kk / g.kseg_len) * g.kseg_stride + (kk % g.kseg_len);
}

}  // namespace grace
