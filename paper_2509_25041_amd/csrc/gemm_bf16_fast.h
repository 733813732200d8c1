// bf16 MFMA grouped GEMM for gfx950, large tiles.
//
// Block tile 256 activation rows x 256 weight rows, K in steps of 64, 8
// wavefronts (2 along M x 4 along N, 128 x 64 outputs each, 32x32x16 MFMA).
// Both operands are K-contiguous in HBM.  Tiles are copied HBM -> LDS with
// direct-to-LDS 16-byte loads (no staging registers); the 16-byte chunk c of
// tile row r is kept at chunk position c ^ ((r >> 1) & 7), which is applied on
// the global address side because a direct load writes consecutive lanes to
// consecutive LDS addresses.  Two LDS stages: the loads of step kt+1 are in
// flight while step kt is multiplied; one barrier per step.
//
// Ragged row segments: rows past the end of a segment are clamped to its last
// row when loading (their products are never stored) and 32-row MFMA sub-tiles
// that lie entirely past the end are skipped.  Weight rows past N are clamped
// likewise.  Precondition: K is a multiple of 64 (no K tail).
//
// Block -> tile mapping is XCD-aware: workgroups are dealt round-robin to the
// 8 XCDs, so block b runs on XCD b % 8 (checked with HW_REG_XCC_ID); each XCD
// is given a contiguous range of m-tiles and walks all n-tiles of an m-tile
// consecutively, so the blocks resident on one XCD share activation rows and
// (within a segment) weights in that XCD's L2.  Dealing groups of m-tiles
// round-robin over the XCDs instead balances them better on paper but was
// not faster in interleaved repeated timings on the Zipf-skewed workload.
#pragma once
#include <type_traits>

#include "bf16.h"
#include "gemm_common.h"

namespace grace {
namespace fast {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int BM = 256, BROWS = 256, THREADS = 512;
constexpr int N_XCD = 8;

// Tile geometry for a K step of BK elements and NSTAGE LDS stages.
template <int BK_, int NSTAGE_, int KEY_SHIFT_ = (BK_ == 64 ? 1 : 2)>
struct Geo {
    static constexpr int BK = BK_, NSTAGE = NSTAGE_;
    static constexpr int ROW_BYTES = BK * 2;                 // one tile row in LDS
    static constexpr int CPR = BK / 8;                       // 16-byte chunks per row
    static constexpr int ROWS_PER_LOAD = 1024 / ROW_BYTES;   // rows covered by one wavefront-wide 16-byte load
    static constexpr int LOADS = BM / (8 * ROWS_PER_LOAD);   // loads per lane per operand per stage
    static constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BROWS * ROW_BYTES;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    // operand stages, or the epilogue's 8 x 128 rows x 128 bytes of output staging, whichever is larger
    static constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES > 131072 ? NSTAGE * STAGE_BYTES : 131072;
    // swizzle key of a tile row: chunk c is stored at c ^ key(row)
    static constexpr int KEY_SHIFT = KEY_SHIFT_;
    __device__ static __forceinline__ int key(int row) { return (row >> KEY_SHIFT) & (CPR - 1); }
};

// K step 64, two stages, swizzle key (row >> 1) & 7: no LDS bank conflicts on the fragment reads.
using DefaultGeo = Geo<64, 2, 1>;

typedef __attribute__((address_space(3))) void lds_void_t;
typedef const __attribute__((address_space(1))) void global_void_t;

__device__ __forceinline__ void load16_to_lds(const void *gptr, char *lds_wave_base) {
    __builtin_amdgcn_global_load_lds((global_void_t *)gptr, (lds_void_t *)lds_wave_base, 16, 0, 0);
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    if constexpr (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else if constexpr (N == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
    else if constexpr (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else if constexpr (N == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else if constexpr (N == 12) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
    else if constexpr (N == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    else if constexpr (N == 24) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
    else static_assert(N == 0, "unsupported vmcnt");
}

template <bool FUSED_UP, typename G>
__global__ __launch_bounds__(THREADS, 1) void gemm_bf16_fast_kernel(const GemmArgs g, int n_tiles_n) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    constexpr int BK = G::BK, NSTAGE = G::NSTAGE, LOADS = G::LOADS;
    constexpr int BN = FUSED_UP ? 128 : 256;  // output columns per block
    const int tid = (int)threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar
    const int wm = wave >> 2, wn = wave & 3;

    // ---- tile of this block -------------------------------------------------
    // XCD x owns the contiguous m-tile range [x * per_xcd, (x + 1) * per_xcd) and walks it in
    // (m-tile, n-tile) order, so the 32 blocks resident on an XCD cover a few consecutive
    // m-tiles x all n-tiles and share their operands in that XCD's L2.
    int total_mt = 0;
    if (g.seg_off) {
        for (int s = 0; s < g.S; ++s) total_mt += (g.seg_off[s + 1] - g.seg_off[s] + BM - 1) / BM;
    } else {
        total_mt = (g.M_single + BM - 1) / BM;
    }
    const int per_xcd = (total_mt + N_XCD - 1) / N_XCD;
    const int xcd = (int)blockIdx.x % N_XCD, j = (int)blockIdx.x / N_XCD;
    const int mt_idx = j / n_tiles_n, nt = j % n_tiles_n;
    if (mt_idx >= per_xcd) return;
    int slot, m0, m_end;
    if (!locate_tile<BM>(g, xcd * per_xcd + mt_idx, slot, m0, m_end)) return;
    const int n0 = nt * BN;

    const uint16_t *A = (const uint16_t *)g.A;
    const uint16_t *B0 = (const uint16_t *)g.B0 + (int64_t)slot * g.b_slot_stride;
    const uint16_t *B1 = FUSED_UP ? (const uint16_t *)g.B1 + (int64_t)slot * g.b_slot_stride : nullptr;

    // ---- this lane's load sources (fixed rows, advancing along K) -------------
    // One wavefront-wide load fills 1 KB of LDS = ROWS_PER_LOAD consecutive tile
    // rows; lane l lands at row l / CPR, chunk position l % CPR.
    const int lrow = lane / G::CPR, lpos = lane % G::CPR;
    const uint16_t *a_src[LOADS], *b_src[LOADS];
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
        const int tr = (i * 8 + wave) * G::ROWS_PER_LOAD + lrow;  // tile row
        const int gchunk = lpos ^ G::key(tr);                      // global chunk that lands at position lpos
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
    const int nk = g.K / BK;
    int64_t kb = 0;
    int kpos = 0, k_issue = 0, stage_issue = 0;
    auto issue_loads = [&]() {
        char *sa = smem + stage_issue * G::STAGE_BYTES + wave * 1024;
        char *sb = sa + G::A_BYTES;
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            load16_to_lds(a_src[i] + k_issue, sa + i * 8192);
            load16_to_lds(b_src[i] + kb, sb + i * 8192);
        }
        k_issue += BK;
        kb += BK;
        kpos += BK;
        if (kpos == g.kseg_len) { kpos = 0; kb += g.kseg_stride - g.kseg_len; }
        stage_issue = (stage_issue + 1 == NSTAGE) ? 0 : stage_issue + 1;
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

    // fragment addresses: row r = base + (lane & 31), chunk c = 2*ks + (lane >> 5) stored at c ^ key(r)
    const int frow = lane & 31, fhalf = lane >> 5, fkey = G::key(frow);  // bases are multiples of 32
    int a_off[4], b_off[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) a_off[i] = (wm * 128 + i * 32 + frow) * G::ROW_BYTES;
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
        b_off[jj] = G::A_BYTES + ((FUSED_UP ? jj * 128 + wn * 32 : wn * 64 + jj * 32) + frow) * G::ROW_BYTES;
    int pc[BK / 16];
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) pc[ks] = ((ks * 2 + fhalf) ^ fkey) * 16;

    // ---- main loop -------------------------------------------------------------
    // All NSTAGE buffers are filled up front.  In step kt, before the MFMAs of its
    // last 16-wide K group, the block synchronises once: by then every wavefront
    // has read all of stage kt (fragments are fetched one group ahead), so its
    // buffer is handed to the loads of stage kt + NSTAGE, and stage kt + 1 is known
    // to have landed, so the first fragments of the next step can be fetched while
    // the last MFMAs of this step run.
    constexpr int KS = BK / 16;
#pragma unroll
    for (int s = 0; s < NSTAGE; ++s)
        if (s < nk) issue_loads();
    // Loads complete in issue order: a stage has landed once at most the 2 * LOADS loads of
    // each younger stage are outstanding.
    auto wait_younger = [&](int younger) {
        if (NSTAGE > 3 && younger >= 3) wait_vmcnt<6 * LOADS>();
        else if (NSTAGE > 2 && younger == 2) wait_vmcnt<4 * LOADS>();
        else if (younger == 1) wait_vmcnt<2 * LOADS>();
        else wait_vmcnt<0>();
    };
    wait_younger(min(NSTAGE - 1, nk - 1));  // stages 1 .. NSTAGE-1 may still be in flight
    asm volatile("s_barrier" ::: "memory");

    int stage_c = 0;
    if (n_valid == 4) {
        bf16x8_t fa[2][4], fb[2][2];
        auto fetch = [&](int buf, const char *st, int ks) {
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) fb[buf][jj] = *(const bf16x8_t *)(st + b_off[jj] + pc[ks]);
#pragma unroll
            for (int i = 0; i < 4; ++i) fa[buf][i] = *(const bf16x8_t *)(st + a_off[i] + pc[ks]);
        };
        fetch(0, smem, 0);
        // One K step.  HAS_NEXT: another step follows (synchronise, fetch its first fragments).
        // HAS_LOADS: the stage freed at the barrier is refilled; its loads sit in the same basic
        // block as the last group's MFMAs so that they can be issued one per MFMA.
        auto step = [&](auto has_loads, auto has_next, int kt) {
            constexpr bool HAS_LOADS = decltype(has_loads)::value, HAS_NEXT = decltype(has_next)::value;
            const char *st = smem + stage_c * G::STAGE_BYTES;
            stage_c = (stage_c + 1 == NSTAGE) ? 0 : stage_c + 1;
            const char *st_next = smem + stage_c * G::STAGE_BYTES;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int cur = ks & 1, nxt = cur ^ 1;  // KS is even: parity restarts every step
                const bool last = ks == KS - 1;
                if (last) {
                    if (HAS_NEXT) {
                        wait_younger(min(NSTAGE - 2, nk - 2 - kt));  // in flight: stages kt+2 .. kt+NSTAGE-1
                        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                        asm volatile("s_barrier" ::: "memory");
                        if (HAS_LOADS) issue_loads();
                        fetch(nxt, st_next, 0);
                    }
                } else {
                    fetch(nxt, st, ks + 1);
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj)
                        acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[cur][jj], fa[cur][i], acc[i][jj], 0, 0, 0);
                // issue order inside a group: the 6 fragment reads of the next group (and, after the
                // barrier, the 2 * LOADS direct-to-LDS loads) are spread between the 8 MFMAs
                if (last && HAS_NEXT && HAS_LOADS) {
#pragma unroll
                    for (int r = 0; r < 8; ++r) {
                        if (r < 2 * LOADS) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);  // 1 VMEM
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                      // 1 MFMA
                        if (r < 6) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);           // 1 LDS read
                    }
                } else if (!last || HAS_NEXT) {
#pragma unroll
                    for (int r = 0; r < 6; ++r) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // 1 MFMA
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // 1 LDS read
                    }
                    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        using T_ = std::integral_constant<bool, true>;
        using F_ = std::integral_constant<bool, false>;
        int kt = 0;
        for (; kt + NSTAGE < nk; ++kt) step(T_{}, T_{}, kt);
        for (; kt + 1 < nk; ++kt) step(F_{}, T_{}, kt);
        step(F_{}, F_{}, kt);
    } else {
        for (int kt = 0; kt < nk; ++kt) {
            const char *st = smem + stage_c * G::STAGE_BYTES;
            stage_c = (stage_c + 1 == NSTAGE) ? 0 : stage_c + 1;
            if (n_valid > 0) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    bf16x8_t fb[2];
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj) fb[jj] = *(const bf16x8_t *)(st + b_off[jj] + pc[ks]);
#pragma unroll
                    for (int i = 0; i < 3; ++i) {
                        if (i < n_valid) {
                            const bf16x8_t fa = *(const bf16x8_t *)(st + a_off[i] + pc[ks]);
#pragma unroll
                            for (int jj = 0; jj < 2; ++jj)
                                acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[jj], fa, acc[i][jj], 0, 0, 0);
                        }
                    }
                }
            }
            if (kt + 1 < nk) {
                wait_younger(min(NSTAGE - 2, nk - 2 - kt));
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                asm volatile("s_barrier" ::: "memory");
                if (kt + NSTAGE < nk) issue_loads();
            }
        }
    }

    // ---- epilogue -------------------------------------------------------------------
    // The weight fragment is the MFMA's first operand, so acc[i][jj] holds a transposed 32x32
    // tile: element v of lane l is (n = 8*(v/4) + 4*(l/32) + v%4, m = l%32), i.e. four
    // consecutive output columns of one row per group of four values.  Each wavefront packs
    // them to bf16, transposes its 128 x BNW tile through its own LDS region (16-byte chunks
    // XOR-swizzled by row) and writes whole rows with 16-byte stores.
    constexpr int BNW = FUSED_UP ? 32 : 64;     // output columns per wavefront
    constexpr int ROWB = BNW * 2;               // bytes per staged row
    constexpr int CH = ROWB / 16;               // 16-byte chunks per staged row
    constexpr int KSH = (ROWB == 128) ? 1 : 2;  // rows per 256 bytes of LDS = 1 << KSH
    static_assert(8 * 128 * ROWB <= G::LDS_BYTES, "epilogue staging exceeds the LDS allocation");
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    asm volatile("s_barrier" ::: "memory");     // every wavefront is done reading the operand stages
    char *stg = smem + wave * (128 * ROWB);
    const int fhalf8 = fhalf * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (i >= n_valid) continue;
        const int ml = i * 32 + frow;
        const int key = (ml >> KSH) & (CH - 1);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (FUSED_UP) {
                float h[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float gt = acc[i][0][q * 4 + r], up = acc[i][1][q * 4 + r];
                    h[r] = gt * __frcp_rn(1.0f + __expf(-gt)) * up;
                }
                uint2 pk = make_uint2(pack_bf16x2(h[0], h[1]), pack_bf16x2(h[2], h[3]));
                *(uint2 *)(stg + ml * ROWB + ((q ^ key) * 16) + fhalf8) = pk;
            } else {
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    uint2 pk = make_uint2(pack_bf16x2(acc[i][jj][q * 4 + 0], acc[i][jj][q * 4 + 1]),
                                          pack_bf16x2(acc[i][jj][q * 4 + 2], acc[i][jj][q * 4 + 3]));
                    *(uint2 *)(stg + ml * ROWB + (((jj * 4 + q) ^ key) * 16) + fhalf8) = pk;
                }
            }
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // this wavefront's own writes, read back below
    {
        uint16_t *out = (uint16_t *)g.out;
        constexpr int ROWS_PER_IT = 64 / CH;
        const int rr = lane / CH, cc = lane % CH;
        const int ncol = n0 + wn * BNW + cc * 8;
#pragma unroll
        for (int it = 0; it < 128 / ROWS_PER_IT; ++it) {
            const int ml = it * ROWS_PER_IT + rr;
            const int row = m0 + wm * 128 + ml;
            if (row < m_end && ncol < g.N) {
                const int key = (ml >> KSH) & (CH - 1);
                const uint4 v = *(const uint4 *)(stg + ml * ROWB + ((cc ^ key) * 16));
                *(uint4 *)(out + (int64_t)row * g.ldo + ncol) = v;
            }
        }
    }
}

// Grid size for `m_bound` rows in at most `n_seg` segments.
inline int64_t grid_blocks(int64_t m_bound, int n_seg, int n_tiles_n) {
    const int64_t tiles = m_bound / BM + n_seg;  // >= sum of ceil(M_s / BM)
    return (tiles + N_XCD - 1) / N_XCD * N_XCD * n_tiles_n;
}

}  // namespace fast
}  // namespace grace
