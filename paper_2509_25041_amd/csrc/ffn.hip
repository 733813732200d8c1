// grace_expert_ffn / grace_shared_ffn: grouped SwiGLU FFN.
//
// Two grouped GEMM launches per call.  Operands are K-contiguous on both sides
// (activations [rows, K]; weights [N, K], one output feature per row), which is
// the layout the MFMA units consume directly:
//   up:   h[p, n]  = silu(sum_c xp[p,c] Wg[n,c]) * (sum_c xp[p,c] Wu[n,c])   K = d, N = f
//   down: y[p, m]  = sum_n h[p,n] Wd[m,n]                                     K = f, N = d
// Rows are grouped by instance: the rows of one rank are a contiguous range of
// the dispatch buffer, subdivided per local slot by inst_off (read on the
// device; there is no host synchronisation).  The bf16 kernel is persistent (one
// workgroup per compute unit walks the tiles); the fallback kernels size their
// grid from an upper bound of the tile count and surplus blocks exit at once.
#include <mutex>

#include "bf16.h"
#include "common.h"
#include "gemm_bf16_generic.h"
#include "gemm_bf16_persist.h"
#include "gemm_common.h"
#include "gemm_f32.h"

namespace grace {

// Compute units of the current device (cached per device).
static int compute_units() {
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return -1;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return -1;
        cached[dev] = n;
    }
    return cached[dev];
}

// The persistent kernel needs the 160 KB of dynamic LDS opted in, once per kernel and device.
static bool allow_full_lds(const void *kernel, const char *what) {
    constexpr int MAX_KERNELS = 8, MAX_DEVICES = 64;
    static std::mutex mu;
    static const void *known[MAX_KERNELS] = {nullptr};
    static bool done[MAX_KERNELS][MAX_DEVICES] = {{false}};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        fail(GRACE_EHIP, "%s: cannot query the device", what);
        return false;
    }
    std::lock_guard<std::mutex> lock(mu);
    int slot = 0;
    while (slot < MAX_KERNELS && known[slot] && known[slot] != kernel) ++slot;
    if (slot == MAX_KERNELS) {
        fail(GRACE_EHIP, "%s: kernel table full", what);
        return false;
    }
    known[slot] = kernel;
    if (!done[slot][dev]) {
        const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, pers::LDS_BYTES);
        if (e != hipSuccess) {
            fail(GRACE_EHIP, "%s: cannot reserve LDS: %s", what, hipGetErrorString(e));
            return false;
        }
        done[slot][dev] = true;
    }
    return true;
}

template <bool FUSED_UP, pers::Who WHO>
static int launch_gemm(const GemmArgs &g, grace_dtype dt, int64_t m_bound, hipStream_t st, const char *what) {
    if (m_bound <= 0 || g.N <= 0 || g.K <= 0) return GRACE_OK;
    const int n_seg = g.seg_off ? g.S : 1;
    const bool k_ok = g.K % pers::BK == 0 && g.kseg_len % pers::BK == 0 && g.K >= pers::MIN_K_STEPS * pers::BK &&
                      n_seg <= pers::MAX_SEGMENTS;
    if (dt == GRACE_BF16 && k_ok) {
        const int n_cu = compute_units();
        if (n_cu <= 0) return fail(GRACE_EHIP, "%s: cannot query the device", what);
        // persistent large-tile kernel: one workgroup per compute unit, 160 KB of dynamic LDS
        using SH = pers::Shape<FUSED_UP>;
        const int ntn = (g.N + SH::BN - 1) / SH::BN;
        const int grid = pers::grid_blocks(n_cu);
        if ((m_bound / 160 + n_seg) * (int64_t)ntn > INT32_MAX) return fail(GRACE_ESHAPE, "%s: too many tiles", what);   // the lowest m-tile has 160 rows
        if (n_seg <= 64) {
            if (!allow_full_lds((const void *)pers::gemm_bf16_persist_kernel<FUSED_UP, 1, WHO>, what)) return GRACE_EHIP;
            pers::gemm_bf16_persist_kernel<FUSED_UP, 1, WHO><<<grid, pers::THREADS, pers::LDS_BYTES, st>>>(g, ntn);
        } else if constexpr (WHO == pers::EXPERTS) {  // the shared experts are a single row segment
            if (!allow_full_lds((const void *)pers::gemm_bf16_persist_kernel<FUSED_UP, 4, WHO>, what)) return GRACE_EHIP;
            pers::gemm_bf16_persist_kernel<FUSED_UP, 4, WHO><<<grid, pers::THREADS, pers::LDS_BYTES, st>>>(g, ntn);
        }
    } else if (dt == GRACE_BF16) {
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

static int expert_ffn_up(const char *who, const grace_table *table, int32_t rank, const void *xp, const int32_t *inst_off,
                         int32_t T, int32_t k, int32_t d, int32_t f, grace_dtype dt, const void *w_gate, const void *w_up,
                         int32_t *state, void *ws, void *stream) {
    int g0, S;
    int rc = expert_ffn_common(who, table, rank, T, k, d, f, dt, g0, S);
    if (rc != GRACE_OK) return rc;
    if (S == 0 || T == 0) return GRACE_OK;
    if (!xp || !inst_off || !w_gate || !w_up || !ws) return fail(GRACE_EINVAL, "%s: null device pointer", who);
    if ((((uintptr_t)xp) | ((uintptr_t)w_gate) | ((uintptr_t)w_up) | ((uintptr_t)ws)) & 15)
        return fail(GRACE_EINVAL, "%s: device pointers must be 16-byte aligned", who);
    GemmArgs up{};
    up.A = xp; up.lda = d;
    up.B0 = w_gate; up.B1 = w_up; up.b_slot_stride = (int64_t)d * f; up.ldb = d;
    up.N = f; up.K = d; up.kseg_len = d; up.kseg_stride = 0;
    up.out = ws; up.ldo = f;
    up.seg_off = inst_off + g0; up.S = S; up.M_single = 0;
    up.share_state = state;
    return launch_gemm<true, pers::EXPERTS>(up, dt, (int64_t)T * k, (hipStream_t)stream, who);
}

extern "C" int grace_expert_ffn_up(const grace_table *table, int32_t rank, const void *xp, const int32_t *inst_off,
                                   int32_t T, int32_t k, int32_t d, int32_t f, grace_dtype dt, const void *w_gate,
                                   const void *w_up, void *ws, void *stream) {
    return expert_ffn_up("expert_ffn_up", table, rank, xp, inst_off, T, k, d, f, dt, w_gate, w_up, nullptr, ws, stream);
}

extern "C" int grace_expert_ffn_up_share(const grace_table *table, int32_t rank, const void *xp, const int32_t *inst_off,
                                         int32_t T, int32_t k, int32_t d, int32_t f, grace_dtype dt, const void *w_gate,
                                         const void *w_up, int32_t *state, void *ws, void *stream) {
    if (!state) return fail(GRACE_EINVAL, "expert_ffn_up_share: state is null");
    return expert_ffn_up("expert_ffn_up_share", table, rank, xp, inst_off, T, k, d, f, dt, w_gate, w_up, state, ws, stream);
}

static_assert(SHARE_STATE_INTS == GRACE_SHARE_STATE_INTS, "header and kernels must agree on the state size");

static int expert_ffn_down(const char *who, const grace_table *table, int32_t rank, const int32_t *inst_off, int32_t T,
                           int32_t k, int32_t d, int32_t f, grace_dtype dt, const void *w_down, void *y, int32_t *state,
                           void *ws, void *stream) {
    int g0, S;
    int rc = expert_ffn_common(who, table, rank, T, k, d, f, dt, g0, S);
    if (rc != GRACE_OK) return rc;
    if (S == 0 || T == 0) return GRACE_OK;
    if (!inst_off || !w_down || !y || !ws) return fail(GRACE_EINVAL, "%s: null device pointer", who);
    if ((((uintptr_t)w_down) | ((uintptr_t)y) | ((uintptr_t)ws)) & 15)
        return fail(GRACE_EINVAL, "%s: device pointers must be 16-byte aligned", who);
    const size_t el = dt == GRACE_F32 ? 4 : 2;
    if (state && ((size_t)d * el) % 16 != 0)
        return fail(GRACE_ESHAPE, "%s: row of %zu bytes is not a multiple of 16", who, (size_t)d * el);
    GemmArgs dn{};
    dn.A = ws; dn.lda = f;
    dn.B0 = w_down; dn.B1 = nullptr; dn.b_slot_stride = (int64_t)d * f; dn.ldb = f;
    dn.N = d; dn.K = f; dn.kseg_len = f; dn.kseg_stride = 0;
    dn.out = y; dn.ldo = d;
    dn.seg_off = inst_off + g0; dn.S = S; dn.M_single = 0;
    dn.share_state = state; dn.share_rows = (int64_t)T * k; dn.share_row_vec = (int)((size_t)d * el / 16);
    return launch_gemm<false, pers::EXPERTS>(dn, dt, (int64_t)T * k, (hipStream_t)stream, who);
}

extern "C" int grace_expert_ffn_down(const grace_table *table, int32_t rank, const int32_t *inst_off, int32_t T,
                                     int32_t k, int32_t d, int32_t f, grace_dtype dt, const void *w_down, void *y,
                                     void *ws, void *stream) {
    return expert_ffn_down("expert_ffn_down", table, rank, inst_off, T, k, d, f, dt, w_down, y, nullptr, ws, stream);
}

extern "C" int grace_expert_ffn_down_share(const grace_table *table, int32_t rank, const int32_t *inst_off, int32_t T,
                                           int32_t k, int32_t d, int32_t f, grace_dtype dt, const void *w_down, void *y,
                                           int32_t *state, void *ws, void *stream) {
    if (!state) return fail(GRACE_EINVAL, "expert_ffn_down_share: state is null");
    return expert_ffn_down("expert_ffn_down_share", table, rank, inst_off, T, k, d, f, dt, w_down, y, state, ws, stream);
}

extern "C" int grace_expert_ffn(const grace_table *table, int32_t rank, const void *xp, const int32_t *inst_off,
                                int32_t T, int32_t k, int32_t d, int32_t f, grace_dtype dt, const void *w_gate,
                                const void *w_up, const void *w_down, void *y, void *ws, void *stream) {
    int rc = grace_expert_ffn_up(table, rank, xp, inst_off, T, k, d, f, dt, w_gate, w_up, ws, stream);
    if (rc != GRACE_OK) return rc;
    return grace_expert_ffn_down(table, rank, inst_off, T, k, d, f, dt, w_down, y, ws, stream);
}

static int shared_ffn_common(const char *who, int32_t T, int32_t d, int32_t f, int32_t n_shared, grace_dtype dt) {
    if (T < 0 || n_shared < 1) return fail(GRACE_EINVAL, "%s: T=%d, n_shared=%d invalid", who, T, n_shared);
    int rc = check_ffn_shapes(who, d, f, dt);
    if (rc != GRACE_OK) return rc;
    if ((int64_t)n_shared * f > INT32_MAX) return fail(GRACE_ESHAPE, "%s: n_shared*f too large", who);
    return GRACE_OK;
}

// The shared experts act as one expert of width F = n_shared * f: gate and up weights [n_shared, f, d]
// are one [F, d] matrix each; the down weights [n_shared, d, f] are F input features in n_shared
// K segments of length f that lie d * f elements apart.
static int shared_ffn_up(const char *who, const void *x, int32_t T, int32_t d, int32_t f, int32_t n_shared, grace_dtype dt,
                         const void *w_gate, const void *w_up, void *ws, const int32_t *perm_pos, int32_t k, void *xp,
                         void *stream) {
    int rc = shared_ffn_common(who, T, d, f, n_shared, dt);
    if (rc != GRACE_OK) return rc;
    if (T == 0) return GRACE_OK;
    if (!x || !w_gate || !w_up || !ws) return fail(GRACE_EINVAL, "%s: null device pointer", who);
    if ((((uintptr_t)x) | ((uintptr_t)w_gate) | ((uintptr_t)w_up) | ((uintptr_t)ws)) & 15)
        return fail(GRACE_EINVAL, "%s: device pointers must be 16-byte aligned", who);
    const int F = n_shared * f;
    GemmArgs up{};
    up.A = x; up.lda = d;
    up.B0 = w_gate; up.B1 = w_up; up.b_slot_stride = 0; up.ldb = d;
    up.N = F; up.K = d; up.kseg_len = d; up.kseg_stride = 0;
    up.out = ws; up.ldo = F;
    up.seg_off = nullptr; up.S = 1; up.M_single = T;
    if (perm_pos) {
        // the row scatter rides on the persistent bf16 kernel when rows are whole 1 KB pieces; otherwise it
        // is a launch of its own ahead of the projection
        const size_t row_bytes = (size_t)d * (dt == GRACE_F32 ? 4 : 2);
        const bool persistent = dt == GRACE_BF16 && d % pers::BK == 0 && d >= pers::MIN_K_STEPS * pers::BK;
        if (persistent && row_bytes % 1024 == 0 && (int64_t)T * k < ((int64_t)1 << 29) && row_bytes <= (size_t)INT32_MAX) {
            up.sc_x = x; up.sc_xp = xp; up.sc_pos = perm_pos; up.sc_T = T; up.sc_k = k; up.sc_row_bytes = (int)row_bytes;
        } else {
            rc = grace_permute_rows(x, perm_pos, T, k, d, dt, xp, stream);
            if (rc != GRACE_OK) return rc;
        }
    }
    return launch_gemm<true, pers::SHARED>(up, dt, T, (hipStream_t)stream, who);
}

extern "C" int grace_shared_ffn_up(const void *x, int32_t T, int32_t d, int32_t f, int32_t n_shared, grace_dtype dt,
                                   const void *w_gate, const void *w_up, void *ws, void *stream) {
    return shared_ffn_up("shared_ffn_up", x, T, d, f, n_shared, dt, w_gate, w_up, ws, nullptr, 0, nullptr, stream);
}

extern "C" int grace_shared_ffn_up_scatter(const void *x, int32_t T, int32_t d, int32_t f, int32_t n_shared, grace_dtype dt,
                                           const void *w_gate, const void *w_up, void *ws, const int32_t *perm_pos,
                                           int32_t k, void *xp, void *stream) {
    if (k < 1) return fail(GRACE_EINVAL, "shared_ffn_up_scatter: k=%d invalid", k);
    if (T > 0 && (!perm_pos || !xp)) return fail(GRACE_EINVAL, "shared_ffn_up_scatter: null device pointer");
    if (((uintptr_t)xp) & 15) return fail(GRACE_EINVAL, "shared_ffn_up_scatter: xp must be 16-byte aligned");
    if ((int64_t)T * k > INT32_MAX) return fail(GRACE_ESHAPE, "shared_ffn_up_scatter: T*k exceeds 2^31-1");
    return shared_ffn_up("shared_ffn_up_scatter", x, T, d, f, n_shared, dt, w_gate, w_up, ws, perm_pos, k, xp, stream);
}

extern "C" int grace_shared_ffn_down(int32_t T, int32_t d, int32_t f, int32_t n_shared, grace_dtype dt,
                                     const void *w_down, void *y_shared, void *ws, void *stream) {
    int rc = shared_ffn_common("shared_ffn_down", T, d, f, n_shared, dt);
    if (rc != GRACE_OK) return rc;
    if (T == 0) return GRACE_OK;
    if (!w_down || !y_shared || !ws) return fail(GRACE_EINVAL, "shared_ffn_down: null device pointer");
    if ((((uintptr_t)w_down) | ((uintptr_t)y_shared) | ((uintptr_t)ws)) & 15)
        return fail(GRACE_EINVAL, "shared_ffn_down: device pointers must be 16-byte aligned");
    const int F = n_shared * f;
    GemmArgs dn{};
    dn.A = ws; dn.lda = F;
    dn.B0 = w_down; dn.B1 = nullptr; dn.b_slot_stride = 0; dn.ldb = f;
    dn.N = d; dn.K = F; dn.kseg_len = f; dn.kseg_stride = (int64_t)d * f;  // K segment s lives in w_down[s]
    dn.out = y_shared; dn.ldo = d;
    dn.seg_off = nullptr; dn.S = 1; dn.M_single = T;
    return launch_gemm<false, pers::SHARED>(dn, dt, T, (hipStream_t)stream, "shared_ffn down projection");
}

extern "C" int grace_shared_ffn(const void *x, int32_t T, int32_t d, int32_t f, int32_t n_shared, grace_dtype dt,
                                const void *w_gate, const void *w_up, const void *w_down, void *y_shared, void *ws,
                                void *stream) {
    int rc = shared_ffn_common("shared_ffn", T, d, f, n_shared, dt);
    if (rc != GRACE_OK) return rc;
    if (T == 0) return GRACE_OK;
    if (!w_down || !y_shared) return fail(GRACE_EINVAL, "shared_ffn: null device pointer");
    rc = grace_shared_ffn_up(x, T, d, f, n_shared, dt, w_gate, w_up, ws, stream);
    if (rc != GRACE_OK) return rc;
    return grace_shared_ffn_down(T, d, f, n_shared, dt, w_down, y_shared, ws, stream);
}
