// grace_permute: stable counting sort of the assignments by instance id
// (= node, rank, slot: the two-stage dispatch order of Section 5) and the row
// movement into that order.
//
//   1-3. key_hist / key_scan / key_pos kernels (stable_sort.h): histogram of
//        instance ids per chunk of 512 assignments, exclusive scans -> inst_off /
//        rank_off / node_off, stable rank of each assignment -> perm_pos, perm_src
//        (scan and rank share one launch when there are few chunks)
//   4. scatter_rows_kernel one block per token: read the token row once, write it
//                         to its k buffer positions with 16-byte accesses
#include "bf16.h"
#include "common.h"
#include "stable_sort.h"
#include "wave_utils.h"

namespace grace {

// One block per token: the row is read once and written k times.
__global__ __launch_bounds__(256) void scatter_rows_kernel(const uint4 *__restrict__ x, int k, int row_vec,
                                                           int64_t n_assign, const int32_t *__restrict__ perm_pos,
                                                           uint4 *__restrict__ xp) {
    const int64_t t = blockIdx.x;
    const uint4 *src = x + t * row_vec;
    for (int c = (int)threadIdx.x; c < row_vec; c += 256) {
        const uint4 v = src[c];
        for (int j = 0; j < k; ++j) {
            const int32_t p = perm_pos[t * k + j];
            if (p >= 0 && p < n_assign) nt_store16(v, &xp[(int64_t)p * row_vec + c]);
        }
    }
}

}  // namespace grace

namespace grace {

int check_permute_args(const grace_table *table, const int32_t *topk_inst, int32_t T, int32_t k, const void *x, int32_t d,
                       grace_dtype dt, const int32_t *perm_pos, const int32_t *perm_src, const int32_t *inst_off,
                       const int32_t *rank_off, const int32_t *node_off, const void *xp, const void *ws) {
    if (!table) return fail(GRACE_EINVAL, "permute: table is null");
    if (T < 0 || k < 1) return fail(GRACE_EINVAL, "permute: T=%d, k=%d invalid", T, k);
    if ((int64_t)T * k > INT32_MAX) return fail(GRACE_ESHAPE, "permute: T*k exceeds 2^31-1");
    if (dt != GRACE_F32 && dt != GRACE_BF16) return fail(GRACE_EINVAL, "permute: unknown dtype %d", (int)dt);
    if (!inst_off || !rank_off || !node_off || !ws) return fail(GRACE_EINVAL, "permute: null offset or ws pointer");
    if (T > 0 && (!topk_inst || !perm_pos || !perm_src)) return fail(GRACE_EINVAL, "permute: null device pointer");
    const size_t el = dt == GRACE_F32 ? 4 : 2;
    if (x) {
        if (d < 1) return fail(GRACE_EINVAL, "permute: d=%d invalid", d);
        if (((size_t)d * el) % 16 != 0) return fail(GRACE_ESHAPE, "permute: row of %zu bytes is not a multiple of 16", (size_t)d * el);
        if (T > 0 && !xp) return fail(GRACE_EINVAL, "permute: xp is null");
        if ((((uintptr_t)x) | ((uintptr_t)xp)) & 15) return fail(GRACE_EINVAL, "permute: x and xp must be 16-byte aligned");
    }
    return GRACE_OK;
}

int launch_scatter_rows(const void *x, int T, int k, int d, grace_dtype dt, const int32_t *perm_pos, void *xp,
                        hipStream_t st) {
    const size_t el = dt == GRACE_F32 ? 4 : 2;
    scatter_rows_kernel<<<T, 256, 0, st>>>((const uint4 *)x, k, (int)((size_t)d * el / 16), (int64_t)T * k, perm_pos,
                                           (uint4 *)xp);
    GRACE_LAUNCH_CHECK("scatter_rows_kernel");
    return GRACE_OK;
}

}  // namespace grace

using namespace grace;

extern "C" int grace_permute_rows(const void *x, const int32_t *perm_pos, int32_t T, int32_t k, int32_t d, grace_dtype dt,
                                  void *xp, void *stream) {
    if (T < 0 || k < 1 || d < 1) return fail(GRACE_EINVAL, "permute_rows: T=%d, k=%d, d=%d invalid", T, k, d);
    if (dt != GRACE_F32 && dt != GRACE_BF16) return fail(GRACE_EINVAL, "permute_rows: unknown dtype %d", (int)dt);
    if ((int64_t)T * k > INT32_MAX) return fail(GRACE_ESHAPE, "permute_rows: T*k exceeds 2^31-1");
    const size_t el = dt == GRACE_F32 ? 4 : 2;
    if (((size_t)d * el) % 16 != 0)
        return fail(GRACE_ESHAPE, "permute_rows: row of %zu bytes is not a multiple of 16", (size_t)d * el);
    if (T == 0) return GRACE_OK;
    if (!x || !perm_pos || !xp) return fail(GRACE_EINVAL, "permute_rows: null device pointer");
    if ((((uintptr_t)x) | ((uintptr_t)xp)) & 15) return fail(GRACE_EINVAL, "permute_rows: x and xp must be 16-byte aligned");
    return launch_scatter_rows(x, T, k, d, dt, perm_pos, xp, (hipStream_t)stream);
}

extern "C" int grace_permute(const grace_table *table, const int32_t *topk_inst, int32_t T, int32_t k, const void *x,
                             int32_t d, grace_dtype dt, int32_t *perm_pos, int32_t *perm_src, int32_t *inst_off,
                             int32_t *rank_off, int32_t *node_off, void *xp, void *ws, void *stream) {
    const int rc = check_permute_args(table, topk_inst, T, k, x, d, dt, perm_pos, perm_src, inst_off, rank_off, node_off,
                                      xp, ws);
    if (rc != GRACE_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    const int I = table->I;
    const int64_t n = (int64_t)T * k;
    const int nchunks = (int)ceil_div(n, PERM_CHUNK);
    int32_t *hist = (int32_t *)ws;
    int32_t *base = (int32_t *)((char *)ws + align_up((size_t)nchunks * I * 4, 256));
    const char *failed = stable_sort_launch(table, topk_inst, n, I, 1, hist, base, table->R, table->N, table->d_rank_ptr,
                                            table->d_node_first_inst, inst_off, rank_off, node_off, perm_pos, perm_src, st);
    if (failed) return fail(GRACE_EHIP, "permute: launch of %s failed", failed);
    if (nchunks > 0 && x) return launch_scatter_rows(x, T, k, d, dt, perm_pos, xp, st);
    return GRACE_OK;
}
