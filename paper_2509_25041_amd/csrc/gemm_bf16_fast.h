// bf16 MFMA grouped GEMM for gfx950, large tiles.
//
// Block tile 256 activation rows x 256 weight rows, K in steps of 64, 8
// wavefronts (2 along M x 4 along N, 128 x 64 outputs each, 32x32x16 MFMA).
// Both operands are K-contiguous in HBM.  Tiles are copied HBM -> LDS with
// direct-to-LDS 16-byte loads (no staging registers); the 16-byte chunk c of
// tile row r is kept at chunk position c ^ (r & 7), which is applied on the
// global address side because a direct load writes consecutive lanes to
// consecutive LDS addresses.  Two LDS stages: the loads of step kt+1 are in
// flight while step kt is multiplied; one barrier per step.
//
// Ragged row segments: rows past the end of a segment are clamped to its last
// row when loading (their products are never stored) and 32-row MFMA sub-tiles
// that lie entirely past the end are skipped.  Weight rows past N are clamped
// likewise.  Precondition: K is a multiple of 64 (no K tail).
//
// Block -> tile mapping is XCD-aware: workgroups are dealt round-robin to the
// 8 XCDs, so block b runs on XCD b % 8; each XCD is given a contiguous range of
// m-tiles and walks all n-tiles of an m-tile consecutively, so the blocks
// resident on one XCD share activation rows and (within a segment) weights in
// that XCD's L2.
#pragma once
#include "bf16.h"
#include "gemm_common.h"

namespace grace {
namespace fast {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int BM = 256, BROWS = 256, BK = 64, THREADS = 512;
constexpr int A_BYTES = BM * BK * 2, B_BYTES = BROWS * BK * 2;
constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
constexpr int LDS_BYTES = 2 * STAGE_BYTES;
constexpr int N_XCD = 8;

typedef __attribute__((address_space(3))) void lds_void_t;
typedef const __attribute__((address_space(1))) void global_void_t;

__device__ __forceinline__ void load16_to_lds(const void *gptr, char *lds_wave_base) {
    __builtin_amdgcn_global_load_lds((global_void_t *)gptr, (lds_void_t *)lds_wave_base, 16, 0, 0);
}

template <bool FUSED_UP>
__global__ __launch_bounds__(THREADS, 1) void gemm_bf16_fast_kernel(const GemmArgs g, int n_tiles_n) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    constexpr int BN = FUSED_UP ? 128 : 256;  // output columns per block
    const int tid = (int)threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar
    const int wm = wave >> 2, wn = wave & 3;

    // ---- tile of this block -------------------------------------------------
    int total_mt = 0;
    if (g.seg_off) {
        for (int s = 0; s < g.S; ++s) total_mt += (g.seg_off[s + 1] - g.seg_off[s] + BM - 1) / BM;
    } else {
        total_mt = (g.M_single + BM - 1) / BM;
    }
    const int per_xcd = (total_mt + N_XCD - 1) / N_XCD;
    const int xcd = (int)blockIdx.x % N_XCD, j = (int)blockIdx.x / N_XCD;
    const int mt_local = j / n_tiles_n, nt = j % n_tiles_n;
    if (mt_local >= per_xcd) return;
    const int mt = xcd * per_xcd + mt_local;
    int slot, m0, m_end;
    if (!locate_tile<BM>(g, mt, slot, m0, m_end)) return;
    const int n0 = nt * BN;

    const uint16_t *A = (const uint16_t *)g.A;
    const uint16_t *B0 = (const uint16_t *)g.B0 + (int64_t)slot * g.b_slot_stride;
    const uint16_t *B1 = FUSED_UP ? (const uint16_t *)g.B1 + (int64_t)slot * g.b_slot_stride : nullptr;

    // ---- this lane's 4 + 4 load sources (fixed rows, advancing along K) -------
    const int lrow = lane >> 3;                 // row inside a group of 8 rows (= row & 7)
    const int gchunk = (lane & 7) ^ lrow;       // global chunk that lands at LDS chunk position lane & 7
    const uint16_t *a_src[4], *b_src[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int tr = (i * 8 + wave) * 8 + lrow;  // tile row
        const int m = min(m0 + tr, m_end - 1);
        a_src[i] = A + (int64_t)m * g.lda + gchunk * 8;
        int n;
        const uint16_t *Bm;
        if (FUSED_UP) { n = n0 + (tr & 127); Bm = (tr >> 7) ? B1 : B0; }
        else { n = n0 + tr; Bm = B0; }
        n = min(n, g.N - 1);
        b_src[i] = Bm + (int64_t)n * g.ldb + gchunk * 8;
    }
    // weight K offset of the step being loaded; jumps at segment ends (a step never straddles one)
    int64_t kb = 0;
    int kpos = 0;
    auto issue_loads = [&](int stage, int k0) {
        char *sa = smem + stage * STAGE_BYTES + wave * 1024;
        char *sb = sa + A_BYTES;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            load16_to_lds(a_src[i] + k0, sa + i * 8192);
            load16_to_lds(b_src[i] + kb, sb + i * 8192);
        }
        kb += BK;
        kpos += BK;
        if (kpos == g.kseg_len) { kpos = 0; kb += g.kseg_stride - g.kseg_len; }
    };

    f32x16_t acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jj][v] = 0.0f;

    // 32-row sub-tiles of this wavefront that hold at least one valid row (scalar)
    const int n_valid = max(0, min(4, (m_end - (m0 + wm * 128) + 31) / 32));

    // fragment addresses: row r = base + (lane & 31), chunk c = 2*ks + (lane >> 5) stored at c ^ (r & 7)
    const int frow = lane & 31, fhalf = lane >> 5, fx = lane & 7;
    int a_off[4], b_off[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) a_off[i] = (wm * 128 + i * 32 + frow) * 128;
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
        b_off[jj] = A_BYTES + ((FUSED_UP ? jj * 128 + wn * 32 : wn * 64 + jj * 32) + frow) * 128;
    int pc[BK / 16];
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) pc[ks] = ((ks * 2 + fhalf) ^ fx) * 16;

    const int nk = g.K / BK;
    issue_loads(0, 0);
    if (n_valid == 4) {
        for (int kt = 0; kt < nk; ++kt) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (kt + 1 < nk) issue_loads((kt + 1) & 1, (kt + 1) * BK);
            const char *st = smem + (kt & 1) * STAGE_BYTES;
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks) {
                bf16x8_t fb[2], fa[4];
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) fb[jj] = *(const bf16x8_t *)(st + b_off[jj] + pc[ks]);
#pragma unroll
                for (int i = 0; i < 4; ++i) fa[i] = *(const bf16x8_t *)(st + a_off[i] + pc[ks]);
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj)
                        acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[jj], acc[i][jj], 0, 0, 0);
            }
        }
    } else {
        for (int kt = 0; kt < nk; ++kt) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (kt + 1 < nk) issue_loads((kt + 1) & 1, (kt + 1) * BK);
            const char *st = smem + (kt & 1) * STAGE_BYTES;
            if (n_valid > 0) {
#pragma unroll
                for (int ks = 0; ks < BK / 16; ++ks) {
                    bf16x8_t fb[2];
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj) fb[jj] = *(const bf16x8_t *)(st + b_off[jj] + pc[ks]);
#pragma unroll
                    for (int i = 0; i < 3; ++i) {
                        if (i < n_valid) {
                            const bf16x8_t fa = *(const bf16x8_t *)(st + a_off[i] + pc[ks]);
#pragma unroll
                            for (int jj = 0; jj < 2; ++jj)
                                acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb[jj], acc[i][jj], 0, 0, 0);
                        }
                    }
                }
            }
        }
    }

    // ---- epilogue: acc[i][jj][v] is (row 8*(v/4) + 4*(lane/32) + v%4, col lane%32) of a 32x32 tile ----
    uint16_t *out = (uint16_t *)g.out;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (i >= n_valid) continue;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = m0 + wm * 128 + i * 32 + 8 * (v >> 2) + 4 * fhalf + (v & 3);
            if (row >= m_end) continue;
            if (FUSED_UP) {
                const int n = n0 + wn * 32 + frow;
                if (n < g.N) {
                    const float gt = acc[i][0][v], up = acc[i][1][v];
                    const float h = gt * __frcp_rn(1.0f + __expf(-gt)) * up;
                    out[(int64_t)row * g.ldo + n] = (uint16_t)f32_to_bf16_bits(h);
                }
            } else {
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    const int n = n0 + wn * 64 + jj * 32 + frow;
                    if (n < g.N) out[(int64_t)row * g.ldo + n] = (uint16_t)f32_to_bf16_bits(acc[i][jj][v]);
                }
            }
        }
    }
}

// Grid size for an upper bound `mt_bound` on the number of m-tiles.
inline int64_t grid_blocks(int64_t mt_bound, int n_tiles_n) {
    const int64_t per_xcd = (mt_bound + N_XCD - 1) / N_XCD;
    return per_xcd * N_XCD * n_tiles_n;
}

}  // namespace fast
}  // namespace grace
