// grace_combine: weighted gather of the k expert outputs of every token back to
// token order (the aggregation step after the expert computation, Section 1),
// fp32 accumulation in ascending j, one rounding.
#include "bf16.h"
#include "common.h"

namespace grace {

template <bool BF16>
__global__ __launch_bounds__(256) void combine_kernel(const uint4 *__restrict__ y, const int32_t *__restrict__ perm_pos,
                                                      const float *__restrict__ topk_weight, int k, int row_vec,
                                                      int64_t n_rows, const uint4 *__restrict__ y_shared,
                                                      uint4 *__restrict__ out) {
    constexpr int NV = BF16 ? 8 : 4;  // values per 16-byte vector
    const int64_t t = blockIdx.x;
    for (int c = (int)threadIdx.x; c < row_vec; c += 256) {
        float acc[NV];
#pragma unroll
        for (int i = 0; i < NV; ++i) acc[i] = 0.0f;
        for (int j = 0; j < k; ++j) {
            const int32_t p = perm_pos[t * k + j];
            if (p < 0 || p >= n_rows) continue;
            const float w = topk_weight[t * k + j];
            const uint4 v = nt_load16(&y[(int64_t)p * row_vec + c]);
            float f[NV];
            if constexpr (BF16) unpack_bf16x8(v, f); else unpack_f32x4(v, f);
#pragma unroll
            for (int i = 0; i < NV; ++i) acc[i] = fmaf(w, f[i], acc[i]);
        }
        if (y_shared) {
            const uint4 v = y_shared[t * row_vec + c];
            float f[NV];
            if constexpr (BF16) unpack_bf16x8(v, f); else unpack_f32x4(v, f);
#pragma unroll
            for (int i = 0; i < NV; ++i) acc[i] += f[i];
        }
        uint4 o;
        if constexpr (BF16) o = pack_bf16x8(acc); else o = pack_f32x4(acc);
        out[t * row_vec + c] = o;
    }
}

}  // namespace grace

using namespace grace;

extern "C" int grace_combine(const void *y, const int32_t *perm_pos, const float *topk_weight, int32_t T, int32_t k,
                             int32_t d, grace_dtype dt, const void *y_shared, void *out, void *stream) {
    if (T < 0 || k < 1 || d < 1) return fail(GRACE_EINVAL, "combine: T=%d, k=%d, d=%d invalid", T, k, d);
    if (dt != GRACE_F32 && dt != GRACE_BF16) return fail(GRACE_EINVAL, "combine: unknown dtype %d", (int)dt);
    const size_t el = dt == GRACE_F32 ? 4 : 2;
    if (((size_t)d * el) % 16 != 0) return fail(GRACE_ESHAPE, "combine: row of %zu bytes is not a multiple of 16", (size_t)d * el);
    if ((int64_t)T * k > INT32_MAX) return fail(GRACE_ESHAPE, "combine: T*k exceeds 2^31-1");
    if (T == 0) return GRACE_OK;
    if (!y || !perm_pos || !topk_weight || !out) return fail(GRACE_EINVAL, "combine: null device pointer");
    if ((((uintptr_t)y) | ((uintptr_t)out) | ((uintptr_t)y_shared)) & 15)
        return fail(GRACE_EINVAL, "combine: y, y_shared and out must be 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    const int row_vec = (int)((size_t)d * el / 16);
    const int64_t n = (int64_t)T * k;
    if (dt == GRACE_BF16)
        combine_kernel<true><<<T, 256, 0, st>>>((const uint4 *)y, perm_pos, topk_weight, k, row_vec, n,
                                                (const uint4 *)y_shared, (uint4 *)out);
    else
        combine_kernel<false><<<T, 256, 0, st>>>((const uint4 *)y, perm_pos, topk_weight, k, row_vec, n,
                                                 (const uint4 *)y_shared, (uint4 *)out);
    GRACE_LAUNCH_CHECK("combine_kernel");
    return GRACE_OK;
}
