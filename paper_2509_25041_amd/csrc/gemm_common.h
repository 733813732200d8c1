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

__device__ __forceinline__ int64_t koff(const GemmArgs &g, int kk) {
    return (int64_t)(kk / g.kseg_len) * g.kseg_stride + (kk % g.kseg_len);
}

}  // namespace grace
