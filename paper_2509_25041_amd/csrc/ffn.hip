// grace_expert_ffn / grace_shared_ffn: grouped SwiGLU FFN.
//
// Two grouped GEMM launches per call.  Operands are K-contiguous on both sides
// (activations [rows, K]; weights [N, K], one output feature per row), which is
// the layout the MFMA units consume directly:
//   up:   h[p, n]  = silu(sum_c xp[p,c] Wg[n,c]) * (sum_c xp[p,c] Wu[n,c])   K = d, N = f
//   down: y[p, m]  = sum_n h[p,n] Wd[m,n]                                     K = f, N = d
// Rows are grouped by instance: the rows of one rank are a contiguous range of
// the dispatch buffer, subdivided per local slot by inst_off (read on the
// device; there is no host synchronisation).  The grid is sized from an upper
// bound of the tile count and surplus blocks exit at once.
#include "bf16.h"
#include "common.h"

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

// ------------------------------------------------------------------ bf16 MFMA --
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int BM = 128, BK = 64, BROWS = 128;  // BROWS = weight rows staged per tile
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

template <bool FUSED_UP>
static int launch_gemm(const GemmArgs &g, grace_dtype dt, int64_t m_bound, hipStream_t st, const char *what) {
    if (m_bound <= 0 || g.N <= 0 || g.K <= 0) return GRACE_OK;
    if (dt == GRACE_BF16) {
        constexpr int BN = FUSED_UP ? 64 : 128;
        const int64_t mt = m_bound / BM + (g.seg_off ? g.S : 1);
        const int ntn = (g.N + BN - 1) / BN;
        if (mt * ntn > INT32_MAX) return fail(GRACE_ESHAPE, "%s: grid too large", what);
        gemm_bf16_kernel<FUSED_UP><<<(unsigned)(mt * ntn), 256, 0, st>>>(g, ntn);
    } else {
        const int64_t mt = m_bound / FBM + (g.seg_off ? g.S : 1);
        const int ntn = (g.N + FBN - 1) / FBN;
        if (mt * ntn > INT32_MAX) return fail(GRACE_ESHAPE, "%s: grid too large", what);
        gemm_f32_kernel<FUSED_UP><<<(unsigned)(mt * ntn), 256, 0, st>>>(g, ntn);
    }
    GRACE_LAUNCH_CHECK(what);
    return GRACE_OK;
}

static int check_ffn_shapes(const char *who, int32_t d, int32_t f, grace_dtype dt) {
    if (dt != GRACE_F32 && dt != GRACE_BF16) return fail(GRACE_EINVAL, "%s: unknown dtype %d", who, (int)dt);
    if (d < 1 || f < 1) return fail(GRACE_EINVAL, "%s: d=%d, f=%d invalid", who, d, f);
    if (dt == GRACE_BF16 && ((d % 8) || (f % 8)))
        return fail(GRACE_ESHAPE, "%s: bf16 needs d and f to be multiples of 8 (d=%d, f=%d)", who, d, f);
    return GRACE_OK;
}

}  // namespace grace

using namespace grace;

static int expert_ffn_common(const char *who, const grace_table *table, int32_t rank, int32_t T, int32_t k, int32_t d,
                             int32_t f, grace_dtype dt, int &g0, int &S) {
    if (!table) return fail(GRACE_EINVAL, "%s: table is null", who);
    if (rank < 0 || rank >= table->R) return fail(GRACE_EINVAL, "%s: rank=%d outside [0,%d)", who, rank, table->R);
    if (T < 0 || k < 1) return fail(GRACE_EINVAL, "%s: T=%d, k=%d invalid", who, T, k);
    if ((int64_t)T * k > INT32_MAX) return fail(GRACE_ESHAPE, "%s: T*k exceeds 2^31-1", who);
    int rc = check_ffn_shapes(who, d, f, dt);
    if (rc != GRACE_OK) return rc;
    g0 = table->rank_ptr[rank];
    S = table->rank_ptr[rank + 1] - g0;
    return GRACE_OK;
}

extern "C" int grace_expert_ffn_up(const grace_table *table, int32_t rank, const void *xp, const int32_t *inst_off,
                                   int32_t T, int32_t k, int32_t d, int32_t f, grace_dtype dt, const void *w_gate,
                                   const void *w_up, void *ws, void *stream) {
    int g0, S;
    int rc = expert_ffn_common("expert_ffn_up", table, rank, T, k, d, f, dt, g0, S);
    if (rc != GRACE_OK) return rc;
    if (S == 0 || T == 0) return GRACE_OK;
    if (!xp || !inst_off || !w_gate || !w_up || !ws) return fail(GRACE_EINVAL, "expert_ffn_up: null device pointer");
    if ((((uintptr_t)xp) | ((uintptr_t)w_gate) | ((uintptr_t)w_up) | ((uintptr_t)ws)) & 15)
        return fail(GRACE_EINVAL, "expert_ffn_up: device pointers must be 16-byte aligned");
    GemmArgs up{};
    up.A = xp; up.lda = d;
    up.B0 = w_gate; up.B1 = w_up; up.b_slot_stride = (int64_t)d * f; up.ldb = d;
    up.N = f; up.K = d; up.kseg_len = d; up.kseg_stride = 0;
    up.out = ws; up.ldo = f;
    up.seg_off = inst_off + g0; up.S = S; up.M_single = 0;
    return launch_gemm<true>(up, dt, (int64_t)T * k, (hipStream_t)stream, "expert_ffn up projection");
}

extern "C" int grace_expert_ffn_down(const grace_table *table, int32_t rank, const int32_t *inst_off, int32_t T,
                                     int32_t k, int32_t d, int32_t f, grace_dtype dt, const void *w_down, void *y,
                                     void *ws, void *stream) {
    int g0, S;
    int rc = expert_ffn_common("expert_ffn_down", table, rank, T, k, d, f, dt, g0, S);
    if (rc != GRACE_OK) return rc;
    if (S == 0 || T == 0) return GRACE_OK;
    if (!inst_off || !w_down || !y || !ws) return fail(GRACE_EINVAL, "expert_ffn_down: null device pointer");
    if ((((uintptr_t)w_down) | ((uintptr_t)y) | ((uintptr_t)ws)) & 15)
        return fail(GRACE_EINVAL, "expert_ffn_down: device pointers must be 16-byte aligned");
    GemmArgs dn{};
    dn.A = ws; dn.lda = f;
    dn.B0 = w_down; dn.B1 = nullptr; dn.b_slot_stride = (int64_t)d * f; dn.ldb = f;
    dn.N = d; dn.K = f; dn.kseg_len = f; dn.kseg_stride = 0;
    dn.out = y; dn.ldo = d;
    dn.seg_off = inst_off + g0; dn.S = S; dn.M_single = 0;
    return launch_gemm<false>(dn, dt, (int64_t)T * k, (hipStream_t)stream, "expert_ffn down projection");
}

extern "C" int grace_expert_ffn(const grace_table *table, int32_t rank, const void *xp, const int32_t *inst_off,
                                int32_t T, int32_t k, int32_t d, int32_t f, grace_dtype dt, const void *w_gate,
                                const void *w_up, const void *w_down, void *y, void *ws, void *stream) {
    int rc = grace_expert_ffn_up(table, rank, xp, inst_off, T, k, d, f, dt, w_gate, w_up, ws, stream);
    if (rc != GRACE_OK) return rc;
    return grace_expert_ffn_down(table, rank, inst_off, T, k, d, f, dt, w_down, y, ws, stream);
}

extern "C" int grace_shared_ffn(const void *x, int32_t T, int32_t d, int32_t f, int32_t n_shared, grace_dtype dt,
                                const void *w_gate, const void *w_up, const void *w_down, void *y_shared, void *ws,
                                void *stream) {
    if (T < 0 || n_shared < 1) return fail(GRACE_EINVAL, "shared_ffn: T=%d, n_shared=%d invalid", T, n_shared);
    int rc = check_ffn_shapes("shared_ffn", d, f, dt);
    if (rc != GRACE_OK) return rc;
    if ((int64_t)n_shared * f > INT32_MAX) return fail(GRACE_ESHAPE, "shared_ffn: n_shared*f too large");
    if (T == 0) return GRACE_OK;
    if (!x || !w_gate || !w_up || !w_down || !y_shared || !ws) return fail(GRACE_EINVAL, "shared_ffn: null device pointer");
    if ((((uintptr_t)x) | ((uintptr_t)w_gate) | ((uintptr_t)w_up) | ((uintptr_t)w_down) | ((uintptr_t)y_shared) |
         ((uintptr_t)ws)) & 15)
        return fail(GRACE_EINVAL, "shared_ffn: device pointers must be 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    const int F = n_shared * f;  // the shared experts act as one expert of width n_shared * f
    GemmArgs up{};
    up.A = x; up.lda = d;
    up.B0 = w_gate; up.B1 = w_up; up.b_slot_stride = 0; up.ldb = d;   // [n_shared, f, d] viewed as [F, d]
    up.N = F; up.K = d; up.kseg_len = d; up.kseg_stride = 0;
    up.out = ws; up.ldo = F;
    up.seg_off = nullptr; up.S = 1; up.M_single = T;
    rc = launch_gemm<true>(up, dt, T, st, "shared_ffn up projection");
    if (rc != GRACE_OK) return rc;
    GemmArgs dn{};
    dn.A = ws; dn.lda = F;
    dn.B0 = w_down; dn.B1 = nullptr; dn.b_slot_stride = 0; dn.ldb = f;
    dn.N = d; dn.K = F; dn.kseg_len = f; dn.kseg_stride = (int64_t)d * f;  // K segment s lives in w_down[s]
    dn.out = y_shared; dn.ldo = d;
    dn.seg_off = nullptr; dn.S = 1; dn.M_single = T;
    return launch_gemm<false>(dn, dt, T, st, "shared_ffn down projection");
}
