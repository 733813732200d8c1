// fp32 grouped GEMM on the vector ALUs.
#pragma once
#include "gemm_common.h"

namespace grace {

// ---------------------------------------------------------------- fp32 FMA path --
// Plain fp32 tiles (no reduced-precision matrix formats): 64x64 outputs per block,
// 4x4 per thread, K in steps of 16 through LDS.
constexpr int FBM = 64, FBN = 64, FBK = 16;

template <bool FUSED_UP>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const GemmArgs g, int n_tiles_n) {
    __shared__ float sA[FBK][FBM + 4];
    __shared__ float sB0[FBK][FBN + 4];
    __shared__ float sB1[FUSED_UP ? FBK : 1][FBN + 4];
    const int tid = (int)threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int nt = (int)blockIdx.x % n_tiles_n, mt = (int)blockIdx.x / n_tiles_n;
    int slot, m0, m_end;
    if (FUSED_UP) share_record(g); else share_clear_stale(g);
    if (!locate_tile<FBM>(g, mt, slot, m0, m_end)) return;
    const int n0 = nt * FBN;
    const float *A = (const float *)g.A;
    const float *B0 = (const float *)g.B0 + (int64_t)slot * g.b_slot_stride;
    const float *B1 = FUSED_UP ? (const float *)g.B1 + (int64_t)slot * g.b_slot_stride : nullptr;
    float acc0[4][4], acc1[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc0[i][j] = acc1[i][j] = 0.0f;

    for (int k0 = 0; k0 < g.K; k0 += FBK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + 256 * i;
            const int row = idx >> 4, kk = idx & 15;
            const bool kin = (k0 + kk) < g.K;
            const int m = m0 + row, n = n0 + row;
            sA[kk][row] = (m < m_end && kin) ? A[(int64_t)m * g.lda + k0 + kk] : 0.0f;
            const int64_t bo = (int64_t)n * g.ldb + (kin ? koff(g, k0 + kk) : 0);
            sB0[kk][row] = (n < g.N && kin) ? B0[bo] : 0.0f;
            if (FUSED_UP) sB1[kk][row] = (n < g.N && kin) ? B1[bo] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < FBK; ++kk) {
            float a[4], b0[4], b1[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = sA[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                b0[j] = sB0[kk][tx * 4 + j];
                b1[j] = FUSED_UP ? sB1[kk][tx * 4 + j] : 0.0f;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc0[i][j] = fmaf(a[i], b0[j], acc0[i][j]);
                    if (FUSED_UP) acc1[i][j] = fmaf(a[i], b1[j], acc1[i][j]);
                }
        }
        __syncthreads();
    }
    float *out = (float *)g.out;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= m_end) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= g.N) continue;
            float v = acc0[i][j];
            if (FUSED_UP) v = v / (1.0f + expf(-v)) * acc1[i][j];
            out[(int64_t)m * g.ldo + n] = v;
        }
    }
}

}  // namespace grace
