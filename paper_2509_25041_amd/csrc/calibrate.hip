// grace_mfma_sustained: what bf16 MFMA rate this device sustains.
//
// The MFMA rate of a power-limited part depends on how many operand bits
// toggle, so the nominal peak is not what a GEMM on real data can reach.  This
// kernel issues the grouped GEMM's inner instruction mix with no global
// traffic: per K group 32 x v_mfma_f32_16x16x32_bf16 (eight activation
// fragments x four weight fragments, in the GEMM's two passes) and (optionally)
// 12 16-byte fragment reads from LDS for the next group, 8 wavefronts per CU,
// one barrier per 64 MFMAs, with constant or pseudo-random bf16 operands.
#include "common.h"

namespace grace {

typedef __attribute__((ext_vector_type(8))) __bf16 cal_bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float cal_f32x4_t;

template <bool LDS_FED>
__global__ __launch_bounds__(512) void mfma_sustained_kernel(float *out, int iters, int random_operands) {
    __shared__ __attribute__((aligned(1024))) char smem[65536];
    const int lane = (int)threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    for (int i = (int)threadIdx.x; i < 65536 / 4; i += 512) {
        unsigned h = (unsigned)(i + (int)blockIdx.x * 7919) * 2654435761u;
        h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
        // two bf16 values in +-[0.5, 1): random sign and mantissa
        const unsigned lo = 0x3F00u | (h & 0x80FFu), hi = 0x3F00u | ((h >> 16) & 0x80FFu);
        ((unsigned *)smem)[i] = random_operands ? (lo | (hi << 16)) : 0x3C003C00u;
    }
    __syncthreads();
    cal_f32x4_t acc[8][4];
    for (int i = 0; i < 8; ++i)
        for (int j = 0; j < 4; ++j)
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
    // the grouped GEMM's fragment addressing: 128-byte rows, 16 rows per fragment, chunk ^ ((row >> 1) & 7)
    const int row = lane & 15, quarter = lane >> 4;
    const int base = (wave & 3) * 8192 + row * 128;
    int pc[2];
    for (int gk = 0; gk < 2; ++gk) pc[gk] = ((gk * 4 + quarter) ^ ((row >> 1) & 7)) * 16;
    cal_bf16x8_t f[2][12];  // per K group: fragments 0..3 weights, 4..11 activations
    for (int b = 0; b < 2; ++b)
        for (int r = 0; r < 12; ++r) f[b][r] = *(const cal_bf16x8_t *)(smem + ((base + r * 2048 + pc[b]) & 0xFFFF));
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int grp = 0; grp < 2; ++grp) {
            const int cur = grp, nxt = grp ^ 1;
            if (LDS_FED) {
#pragma unroll
                for (int r = 0; r < 12; ++r)
                    f[nxt][r] = *(const cal_bf16x8_t *)(smem + ((base + r * 2048 + pc[nxt] + (it & 1) * 32768) & 0xFFFF));
            }
#pragma unroll
            for (int pass = 0; pass < 2; ++pass)
#pragma unroll
                for (int i = 0; i < 8; ++i)
#pragma unroll
                    for (int jl = 0; jl < 2; ++jl) {
                        const int j = pass * 2 + jl;
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[cur][j], f[cur][4 + i], acc[i][j], 0, 0, 0);
                    }
            if (LDS_FED) {
#pragma unroll
                for (int m = 0; m < 32; ++m) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    if (m >= 16 && m < 28) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        asm volatile("s_barrier" ::: "memory");
    }
    float s = 0;
    for (int i = 0; i < 8; ++i)
        for (int j = 0; j < 4; ++j)
            for (int v = 0; v < 4; ++v) s += acc[i][j][v];
    out[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

}  // namespace grace

using namespace grace;

extern "C" int grace_mfma_sustained(int32_t random_operands, int32_t lds_fed, double *tflops_out, void *stream) {
    if (!tflops_out) return fail(GRACE_EINVAL, "mfma_sustained: tflops_out is null");
    hipStream_t st = (hipStream_t)stream;
    int dev = 0, cus = 0;
    GRACE_HIP(hipGetDevice(&dev));
    GRACE_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const int blocks = cus > 0 ? cus : 256;
    float *out = nullptr;
    GRACE_HIP(hipMalloc(&out, (size_t)blocks * 512 * sizeof(float)));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t he = hipEventCreate(&e0);
    if (he == hipSuccess) he = hipEventCreate(&e1);
    const int iters = 8000;  // about 10 ms: long enough for the power management to settle
    float best = 0.f;
    for (int rep = 0; rep < 3 && he == hipSuccess; ++rep) {
        he = hipEventRecord(e0, st);
        if (he != hipSuccess) break;
        if (lds_fed) mfma_sustained_kernel<true><<<blocks, 512, 0, st>>>(out, iters, random_operands);
        else mfma_sustained_kernel<false><<<blocks, 512, 0, st>>>(out, iters, random_operands);
        he = hipGetLastError();
        if (he == hipSuccess) he = hipEventRecord(e1, st);
        if (he == hipSuccess) he = hipEventSynchronize(e1);
        float ms = 0.f;
        if (he == hipSuccess) he = hipEventElapsedTime(&ms, e0, e1);
        if (he == hipSuccess && rep > 0 && (best == 0.f || ms > best)) best = ms;  // slowest of the warm runs
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(out);
    if (he != hipSuccess) return fail(GRACE_EHIP, "mfma_sustained: %s", hipGetErrorString(he));
    const double flops = (double)blocks * 8 * iters * 64 * 16384.0;   // 64 MFMAs of 16 x 16 x 32 x 2 FLOP per iteration
    *tflops_out = flops / (best * 1e-3) / 1e12;
    return GRACE_OK;
}
