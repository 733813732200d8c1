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
    // Rank-share upkeep of the down projection's output buffer (null: off).  share_state: [0], [1] =
    // first and end row that the previous step wrote, [4], [5] = the same for the current step.  The up
    // projection's launch keeps the record, the down projection's launch (a later kernel on the same
    // stream) only reads it: no kernel reads what another workgroup of the same launch writes.
    int32_t *share_state;
    int64_t share_rows;     // rows of the whole output buffer
    int share_row_vec;      // 16-byte vectors per output row
    // Row scatter carried along by the launch (null: none): xp[pos[t*k+j]] = x[t], rows of sc_row_bytes
    // bytes (a multiple of 1024).  Independent of the GEMM's own operands and outputs.
    const void *sc_x;
    void *sc_xp;
    const int32_t *sc_pos;
    int sc_T, sc_k, sc_row_bytes;
};
constexpr int SHARE_STATE_INTS = 8;

// Up projection, first thread of the grid: what was the current range becomes the previous one, the
// segments of this step the current one.
__device__ __forceinline__ void share_record(const GemmArgs &g) {
    if (!g.share_state || blockIdx.x != 0 || threadIdx.x != 0) return;
    const int32_t p0 = g.share_state[4], p1 = g.share_state[5];
    g.share_state[0] = p0;
    g.share_state[1] = p1;
    g.share_state[4] = g.seg_off[0];
    g.share_state[5] = g.seg_off[g.S];
}

// Down projection: rows of the output that the previous step wrote for this rank and the current
// segments no longer cover would keep old results; every workgroup zeroes its part of them before
// it does anything else (they lie outside the rows this launch writes).
__device__ __forceinline__ void share_clear_stale(const GemmArgs &g) {
    if (!g.share_state) return;
    const int64_t n = g.share_rows;
    const int64_t pl = max((int64_t)0, min(n, (int64_t)g.share_state[0]));
    const int64_t ph = max(pl, min(n, (int64_t)g.share_state[1]));
    const int64_t nl = max((int64_t)0, min(n, (int64_t)g.seg_off[0]));
    const int64_t nh = max(nl, min(n, (int64_t)g.seg_off[g.S]));
    // stale rows: [pl, min(ph, nl)) and [max(pl, nh), ph)
    const int64_t a_end = max(pl, min(ph, nl)), b_begin = min(ph, max(pl, nh));
    const int64_t n_a = (a_end - pl) * g.share_row_vec, n_b = (ph - b_begin) * g.share_row_vec;
    uint4 *y = (uint4 *)g.out;
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_a + n_b; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t v = i < n_a ? pl * g.share_row_vec + i : b_begin * g.share_row_vec + (i - n_a);
        y[v] = zero;
    }
}

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

// Row segments (one per local expert slot) cut into m-tiles of bm rows, held in registers by every
// wavefront: lane l keeps segments SPL * l .. SPL * l + SPL - 1 (so at most 64 * SPL segments) and
// the index of their first m-tile.  A tile's segment is found with a ballot; no table in memory.
struct Tile {
    int slot, m0, m_end;  // segment, first row, end of the tile's rows (the segment's end for its last tile)
};

template <int SPL>
struct SegTable {
    int lo[SPL], hi[SPL], base[SPL];
    int total;  // m-tiles over all segments (scalar)
    int bm;     // rows per m-tile (scalar)

    // first: the segments' bounds, read once
    __device__ __forceinline__ void load(const GemmArgs &g, int lane) {
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
        }
    }

    // m-tiles of `rows_per_tile` rows over all segments (scalar); changes nothing
    __device__ __forceinline__ int count(int rows_per_tile) const {
        int lane_tiles = 0;
#pragma unroll
        for (int q = 0; q < SPL; ++q) lane_tiles += (hi[q] - lo[q] + rows_per_tile - 1) / rows_per_tile;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) lane_tiles += __shfl_xor(lane_tiles, o, 64);
        return __builtin_amdgcn_readfirstlane(lane_tiles);
    }

    // then: cut into m-tiles of `rows_per_tile` rows
    __device__ __forceinline__ void cut(int lane, int rows_per_tile) {
        bm = rows_per_tile;
        int lane_tiles = 0;
#pragma unroll
        for (int q = 0; q < SPL; ++q) {
            base[q] = lane_tiles;                         // made global below
            lane_tiles += (hi[q] - lo[q] + bm - 1) / bm;  // hi >= lo
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

    // (slot, first row, end of the tile's rows) of m-tile mt < total, as scalars
    __device__ __forceinline__ Tile lookup(int mt, int lane) const {
        int slot = 0, m0 = 0, m_end = 0;
        bool hit = false;
#pragma unroll
        for (int q = 0; q < SPL; ++q) {
            const int rel = mt - base[q];
            const int tiles = (hi[q] - lo[q] + bm - 1) / bm;
            if (rel >= 0 && rel < tiles) {
                hit = true;
                slot = lane * SPL + q;
                m0 = lo[q] + rel * bm;
                m_end = min(hi[q], m0 + bm);
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
