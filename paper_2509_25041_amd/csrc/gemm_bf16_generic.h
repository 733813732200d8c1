// Generic bf16 MFMA grouped GEMM: 128x128 block tiles, register-staged loads
// with zero fill, any K and N that are multiples of 8.  Used when the fast
// kernel's preconditions do not hold.
#pragma once
#include "bf16.h"
#include "gemm_common.h"

namespace grace {

// ------------------------------------------------------------------ bf16 MFMA --
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int BM = 128, BK = 64;
constexpr int TILE_VECS = 128 * (BK / 8);      // 16-byte vectors per operand tile

__device__ __forceinline__ int swz(int row, int c) { return row * (BK / 8) + (c ^ (row & 7)); }

// FUSED_UP: B tile = 64 rows of W_gate + the same 64 rows of W_up, epilogue silu(g)*u.
template <bool FUSED_UP>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const GemmArgs g, int n_tiles_n) {
    __shared__ uint4 sA[2][TILE_VECS];
    __shared__ uint4 sB[2][TILE_VECS];
    constexpr int BN = FUSED_UP ? 64 : 128;
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int nt = (int)blockIdx.x % n_tiles_n, mt = (int)blockIdx.x / n_tiles_n;
    int slot, m0, m_end;
    if (FUSED_UP) share_record(g); else share_clear_stale(g);
    if (!locate_tile<BM>(g, mt, slot, m0, m_end)) return;
    const int n0 = nt * BN;
    const uint16_t *A = (const uint16_t *)g.A;
    const uint16_t *B0 = (const uint16_t *)g.B0 + (int64_t)slot * g.b_slot_stride;
    const uint16_t *B1 = FUSED_UP ? (const uint16_t *)g.B1 + (int64_t)slot * g.b_slot_stride : nullptr;

    // this thread's 4 + 4 vectors of every tile
    int a_row[4], a_c[4];
    const uint16_t *a_ptr[4], *b_ptr[4];
    bool a_ok[4], b_ok[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = tid + 256 * i;
        const int row = idx >> 3, c = idx & 7;
        a_row[i] = row; a_c[i] = c;
        a_ok[i] = (m0 + row) < m_end;
        a_ptr[i] = A + (int64_t)(m0 + row) * g.lda + c * 8;
        int n;
        const uint16_t *Bm;
        if (FUSED_UP) { n = n0 + (row & 63); Bm = (row >> 6) ? B1 : B0; }
        else { n = n0 + row; Bm = B0; }
        b_ok[i] = n < g.N;
        b_ptr[i] = Bm + (int64_t)n * g.ldb;
    }
    f32x16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const uint4 zero = make_uint4(0, 0, 0, 0);
    uint4 ra[4], rb[4];
    auto load_tile = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int kk = k0 + a_c[i] * 8;
            const bool kin = kk < g.K;
            ra[i] = (a_ok[i] && kin) ? *(const uint4 *)(a_ptr[i] + k0) : zero;
            rb[i] = (b_ok[i] && kin) ? *(const uint4 *)(b_ptr[i] + koff(g, kk)) : zero;
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            sA[buf][swz(a_row[i], a_c[i])] = ra[i];
            sB[buf][swz(a_row[i], a_c[i])] = rb[i];
        }
    };

    const int nk = (g.K + BK - 1) / BK;
    load_tile(0);
    store_tile(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_tile((kt + 1) * BK);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int c = ks * 2 + (lane >> 5);
            bf16x8_t fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int row = wm * 64 + i * 32 + (lane & 31);
                const uint4 v = sA[buf][swz(row, c)];
                fa[i] = __builtin_bit_cast(bf16x8_t, v);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int row = (FUSED_UP ? j * 64 + wn * 32 : wn * 64 + j * 32) + (lane & 31);
                const uint4 v = sB[buf][swz(row, c)];
                fb[j] = __builtin_bit_cast(bf16x8_t, v);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) store_tile(buf ^ 1);
        __syncthreads();
    }

    // epilogue.  acc[i][j][v] is element (row, col) of a 32x32 tile with
    // row = 8*(v/4) + 4*(lane/32) + v%4, col = lane%32.
    uint16_t *out = (uint16_t *)g.out;
    const int col_l = lane & 31;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = m0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            if (row >= m_end) continue;
            if (FUSED_UP) {
                const int n = n0 + wn * 32 + col_l;
                if (n < g.N) {
                    const float gt = acc[i][0][v], up = acc[i][1][v];
                    const float h = gt * __frcp_rn(1.0f + __expf(-gt)) * up;
                    out[(int64_t)row * g.ldo + n] = (uint16_t)f32_to_bf16_bits(h);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int n = n0 + wn * 64 + j * 32 + col_l;
                    if (n < g.N) out[(int64_t)row * g.ldo + n] = (uint16_t)f32_to_bf16_bits(acc[i][j][v]);
                }
            }
        }
}

}  // namespace grace
