// bf16 MFMA grouped GEMM for gfx950: persistent workgroups, large tiles.
//
// One workgroup per compute unit walks a list of output tiles.  Tile = 256
// activation rows x 256 weight rows, K in steps of 64, 8 wavefronts (2 along M
// x 4 along N, 128 x 64 outputs each, v_mfma_f32_16x16x32_bf16: on this part,
// whose MFMA rate is set by the power limit, it sustains about a tenth more
// than the 32x32x16 form at the same operand traffic, having a quarter of the
// accumulator values per instruction for half the arithmetic).  Both operands are
// K-contiguous in HBM and are copied HBM -> LDS with direct-to-LDS 16-byte
// loads (no staging registers); the 16-byte chunk c of tile row r is kept at
// chunk position c ^ ((r >> 1) & 7) (conflict-free fragment reads), applied on
// the global address side because a direct load writes consecutive lanes to
// consecutive LDS addresses.
//
// All 160 KB of LDS hold operand buffers: two for the activation tile and
// three for the weight tile (32 KB each).  The K loop is flattened over the
// workgroup's tiles.  Step g issues the weight loads of step g + 2 during its
// first 32-wide K group (their buffer was read in step g - 1) and, after the one
// barrier of the step, once every wavefront has read the buffers of step g, the
// activation loads of step g + 2 during its second K group; whether step g + 2
// is in the same tile or the next one.  A batch of loads needs longer than one
// step to land, which a plain double buffer cannot hide; with this split the
// weight batch has more than a step and a half, the activation batch is half as
// large, and the loads are spread over the step instead of issued in one burst.
// The pipeline never drains between tiles: the first steps of the next tile are
// in flight while the current tile's accumulators are converted and written out
// (a workgroup's last tile loads its own first steps again instead: valid
// addresses that nobody reads, so that every step is the same straight code).
// The epilogue stages through the weight buffer that was read last (each
// wavefront uses exactly the bytes its own next weight loads will overwrite),
// so it needs no workgroup barrier.
//
// Ragged row segments (one per local expert slot): rows past the end of a
// segment are clamped to its last row when loading and never stored; a
// wavefront whose 128 rows all lie past the end skips its MFMAs.  Weight rows
// past N are clamped likewise.  Every wavefront keeps the segment table in
// registers (1 or 4 segments per lane, so at most 256 segments) and finds a
// tile's segment with a ballot; there is no tile table in memory.
// Preconditions (checked by the launcher): K and the K segment length are
// multiples of 64, K >= 128, at most 256 segments, grid a multiple of 8.
//
// Tiles are dealt to the grid in whole rounds, so a tile count just above a
// multiple of the grid wastes most of a round.  The experts' down projection
// therefore exists for m-tiles of 256, 224, 192 and 160 rows (8, 7, 6, 5
// activation fragments per wavefront; the weight tile stays 256 rows) and picks
// the height on the device, from the segment lengths of the launch
// (tile_height).
//
// Tile order is XCD-aware: workgroups are dealt round-robin to the 8 XCDs, so
// block b runs on XCD b % 8 (checked with HW_REG_XCC_ID).  Each XCD owns a
// contiguous range of m-tiles and its workgroups take consecutive (m-tile,
// n-tile) pairs, so at any time an XCD works on a few m-tiles x all n-tiles
// and shares their operands in its own L2.  When whole m-tiles cannot be dealt
// evenly (few m-tiles, many n-tiles) the pairs are instead numbered with the
// shorter axis fastest and cut into eight equal ranges.
#pragma once
#include <type_traits>

#include "bf16.h"
#include "gemm_common.h"

namespace grace {
namespace pers {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

constexpr int BM = 256, BROWS = 256, THREADS = 512, N_XCD = 8;
constexpr int BK = 64;
constexpr int NBUF_A = 2, NBUF_B = 3;          // LDS buffers per operand
constexpr int MIN_K_STEPS = 2;
constexpr int ROW_BYTES = BK * 2;              // one tile row in LDS
constexpr int CPR = BK / 8;                    // 16-byte chunks per row
constexpr int ROWS_PER_LOAD = 1024 / ROW_BYTES;  // rows covered by one wavefront-wide 16-byte load
constexpr int LOADS = BM / (8 * ROWS_PER_LOAD);  // loads per lane per operand per stage
constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BROWS * ROW_BYTES;
constexpr int B_BASE = NBUF_A * A_BYTES;       // weight buffers follow the activation buffers
constexpr int LDS_BYTES = NBUF_A * A_BYTES + NBUF_B * B_BYTES;
constexpr int MAX_SEG_PER_LANE = 4, MAX_SEGMENTS = 64 * MAX_SEG_PER_LANE;

template <bool FUSED_UP>
struct Shape {
    static constexpr int BN = FUSED_UP ? 128 : 256;   // output columns per tile
    static constexpr int BNW = FUSED_UP ? 32 : 64;    // output columns per wavefront
    static constexpr int ROWB = BNW * 2;              // bytes per staged output row
};
static_assert(LOADS == 4 && 32 * 128 <= LOADS * 1024, "a wavefront's share of a weight buffer must hold one staged 32-row sub-tile");

__device__ __forceinline__ int swizzle_key(int row) { return (row >> 1) & (CPR - 1); }

// Direct-to-LDS load of 16 bytes per lane: lane l reads base + voff and its data lands at
// lds_wave_base + 16 * l.  `base` and `lds_wave_base` are uniform.  Issued as inline assembly
// (the instruction the compiler's own builtin emits, LDS address in M0): the compiler then does
// not count the load against the LDS counter, and the fragment reads around it keep their exact
// per-read waits instead of "wait for everything".  The waits for these loads are explicit
// s_waitcnt vmcnt(N) in the K loop.  M0 is written here only: nothing else in these kernels
// needs it (LDS instructions do not on this target).  The compiler does not see inside the assembly and
// cannot keep the hardware's wait states for it: s_nop 0 is the one between the write of M0 and its
// use; the five wait states between a VECTOR instruction writing `base` (a v_readlane that reloads
// a spilled pointer) and the load reading it are not padded here (three more idle cycles per load cost
// 0.5-1 % of the kernel): `base` is kept by scalar instructions, and asm_hazards.py / its test verify on
// the compiled ISA that no such write comes closer than that to any assembly block.
__device__ __forceinline__ void load16_to_lds(const char *base, uint32_t voff, char *lds_wave_base) {
    const uint32_t lds_addr = (uint32_t)(size_t)(__attribute__((address_space(3))) char *)lds_wave_base;
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0" ::"s"(base), "v"(voff), "s"(lds_addr) : "memory");
}

enum Who { EXPERTS = 0, SHARED = 1 };

// HF: activation fragments (of 16 rows) per wavefront, i.e. the m-tile holds 32 * HF rows, HF * 16 for each
// of the two wavefront rows.  8 is the full tile; 7, 6, 5 make tiles of 224, 192, 160 rows whose K loop
// has proportionally fewer MFMAs (the weight tile and the loads stay the same).  The kernel picks, from
// the row segments it finds on the device, the height whose tile count fills whole rounds of the grid
// best (tile_height below).
template <bool FUSED_UP, int SEG_PER_LANE, Who WHO, int HF>
__device__ __forceinline__ void persist_body(const GemmArgs g, int n_tiles_n, SegTable<SEG_PER_LANE> &segs) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    static_assert(HF >= 5 && HF <= 8, "schedule positions below assume 5 to 8 fragments");
    using SH = Shape<FUSED_UP>;
    constexpr int BN = SH::BN;
    constexpr int HALF_ROWS = HF * 16, TILE_ROWS = 2 * HALF_ROWS;
    const int tid = (int)threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar
    const int wm = wave >> 2, wn = wave & 3;

    segs.cut(lane, TILE_ROWS);
    const int total_mt = segs.total;
    auto lookup = [&](int mt) { return segs.lookup(mt, lane); };

    // ---- this workgroup's tiles ------------------------------------------------------------
    // Two ways to split the (m-tile, n-tile) pairs over the XCDs; the workgroups of an XCD take
    // consecutive pairs of its share.
    //  * by m-tile: an XCD owns a contiguous range of m-tiles with all their n-tiles (shares end on
    //    m-tile boundaries, so a row block is read by one L2 only);
    //  * flat: the pairs, numbered with the shorter axis running fastest, are cut into eight equal
    //    contiguous ranges.  Taken when it needs fewer rounds of tiles, i.e. when whole m-tiles
    //    cannot be dealt evenly (few m-tiles with many n-tiles).
    const int nblk = (int)gridDim.x / N_XCD;                          // workgroups per XCD
    const int xcd = (int)blockIdx.x % N_XCD, bslot = (int)blockIdx.x / N_XCD;
    const int mt_each = total_mt / N_XCD, mt_rem = total_mt % N_XCD;  // first mt_rem XCDs take one more
    const int mt_first = xcd * mt_each + min(xcd, mt_rem);
    const int n_pairs = total_mt * n_tiles_n;                         // < 2^31 (checked by the launcher)
    const int j_each = n_pairs / N_XCD, j_rem = n_pairs % N_XCD;      // first j_rem XCDs take one more
    const int j_first = xcd * j_each + min(xcd, j_rem);
    const int rounds_m = ((mt_each + (mt_rem ? 1 : 0)) * n_tiles_n + nblk - 1) / nblk;
    const int rounds_f = (j_each + (j_rem ? 1 : 0) + nblk - 1) / nblk;
    const bool flat = rounds_f < rounds_m;                            // uniform
    const bool m_fastest = n_tiles_n > total_mt;
    const int njobs = flat ? j_each + (xcd < j_rem ? 1 : 0) : (mt_each + (xcd < mt_rem ? 1 : 0)) * n_tiles_n;  // >= 0
    // By m-tile, the XCD's tiles are walked in panels of PANEL_M m-tiles x PANEL_N n-tiles (m running
    // fastest inside a panel, then the panels of one group of m-tiles side by side): the workgroups of
    // an XCD, which take consecutive jobs, then share PANEL_M activation tiles and PANEL_N weight tiles
    // at any time, and the XCD's L2 is filled with PANEL_M + PANEL_N tiles per round of tiles instead
    // of about one activation tile plus every weight tile of the row.
    const int my_mt = mt_each + (xcd < mt_rem ? 1 : 0);
    const int PANEL_N = min(n_tiles_n, 4), PANEL_M = max(1, nblk / PANEL_N);
    auto job_tile = [&](int job, int &mt, int &n0) {
        if (flat) {
            const int q = j_first + job;
            mt = m_fastest ? q % total_mt : q / n_tiles_n;
            n0 = (m_fastest ? q / total_mt : q % n_tiles_n) * BN;
        } else {
            const int per_group = PANEL_M * n_tiles_n;
            const int mg = job / per_group, r = job - mg * per_group;
            const int gm = min(PANEL_M, my_mt - mg * PANEL_M);   // m-tiles of this group (the last may be short)
            const int ng = r / (gm * PANEL_N), r2 = r - ng * gm * PANEL_N;
            mt = mt_first + mg * PANEL_M + r2 % gm;
            n0 = (ng * PANEL_N + r2 / gm) * BN;
        }
    };
    // rank-share upkeep of the expert down projection's output (no-op unless the launcher asks for it)
    if (WHO == EXPERTS) {
        if (FUSED_UP) share_record(g); else share_clear_stale(g);
    }
    // Lane-dependent values that are only needed at tile boundaries are recomputed there from an
    // opaque copy of the lane id: kept live across the K loop they would be spilled to scratch.
    auto opaque_lane = [&]() {
        int l = lane;
        asm volatile("" : "+v"(l));
        return l;
    };
    // ---- row scatter carried along (shared experts' gate+up projection only) ---------------------
    // The kernel is bound by the matrix cores and leaves most of the HBM bandwidth unused, the row
    // scatter of the dispatch permutation is bound by HBM and leaves the matrix cores idle, and the
    // two are independent.  Every wavefront therefore moves SC_NU 1 KB pieces of token rows every
    // sc_period-th K step: the pieces and their tokens' k positions are loaded just before a K step (so they are
    // older than the step's four weight loads and have landed when the step's wait has passed) and
    // stored to the k rows right behind that wait and the barrier, in the middle of the step: vmcnt counts
    // stores too, so the next step's wait has to see them acknowledged, and from there they have a whole
    // step for it (issued after the step they had half of one, which cost 15-20 us more on the same
    // workload).  Pieces are dealt round-robin to all wavefronts of the grid;
    // whatever is left when a wavefront runs out of K steps is moved at the end, so the scatter is
    // complete whatever the tile count.
    constexpr bool COPY = FUSED_UP && WHO == SHARED;
    const bool copy_on = COPY && g.sc_x != nullptr;                       // uniform
    const int sc_cpr = copy_on ? g.sc_row_bytes / 1024 : 1;                // 1 KB pieces per row
    const int sc_units = copy_on ? g.sc_T * sc_cpr : 0;
    const int sc_stride = (int)gridDim.x * (THREADS / 64);
    int sc_u = (int)blockIdx.x * (THREADS / 64) + wave;                    // this wavefront's next piece
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    // Measured on the 32768-token workload (k = 6) with the first version (stores after the step, a piece every
    // 4th step): +83 us on the 577 us projection for a 188 us scatter; four pieces every 16th step cost 30 us more
    // than that, the wavefronts taking turns (some wavefront storing in every step) 40 us more, plain instead of
    // non-temporal stores 20 us more.
    constexpr int SC_NU = 1;                                               // pieces per copy event
    int sc_period = 1, sc_countdown = 0;                                   // K steps between copy events (set below), steps to the next
    u32x4_t sc_data[SC_NU];
    int sc_pos_v[SC_NU], sc_q[SC_NU];
    int sc_pending = 0;                                                    // pieces loaded and not yet stored (uniform)
#pragma unroll
    for (int n = 0; n < SC_NU; ++n) {
        sc_data[n] = u32x4_t{0u, 0u, 0u, 0u};
        sc_pos_v[n] = 0;
        sc_q[n] = 0;
    }
    auto copy_issue = [&]() {
        if (!copy_on) return;
        const int ll = opaque_lane();
#pragma unroll
        for (int n = 0; n < SC_NU; ++n) {
            if (sc_u >= sc_units) break;
            const int t = sc_u / sc_cpr;
            sc_q[n] = sc_u - t * sc_cpr;
            const uint32_t poff = (uint32_t)(t * g.sc_k + min(ll, g.sc_k - 1)) * 4u;   // T*k < 2^29 here (launcher)
            const char *src = (const char *)g.sc_x + (int64_t)t * g.sc_row_bytes + sc_q[n] * 1024;
            // s_nop 4: the compiler does not see inside inline assembly, so it cannot keep the five wait
            // states between a vector instruction that wrote one of these scalar registers (a v_readlane
            // that reloads a spilled pointer, say) and the memory instruction that reads it
            asm volatile("s_nop 4\n\tglobal_load_dword %0, %2, %3\n\tglobal_load_dwordx4 %1, %4, %5"
                         : "=&v"(sc_pos_v[n]), "=&v"(sc_data[n])
                         : "v"(poff), "s"(g.sc_pos), "v"((uint32_t)ll * 16u), "s"(src)
                         : "memory");
            sc_pending = n + 1;
            sc_u += sc_stride;
        }
    };
    auto copy_store = [&]() {   // only after a wait that covers the loads of copy_issue
        if (sc_pending == 0) return;
        const uint32_t voff = (uint32_t)opaque_lane() * 16u;
        const int64_t n_rows = (int64_t)g.sc_T * g.sc_k;
#pragma unroll
        for (int n = 0; n < SC_NU; ++n) {
            if (n >= sc_pending) break;
            for (int j = 0; j < g.sc_k; ++j) {
                const int p = __builtin_amdgcn_readlane(sc_pos_v[n], j);
                if (p < 0 || p >= n_rows) continue;
                char *dst = (char *)g.sc_xp + (int64_t)p * g.sc_row_bytes + sc_q[n] * 1024;
                asm volatile("s_nop 4\n\tglobal_store_dwordx4 %0, %1, %2 nt" ::"v"(voff), "v"(sc_data[n]), "s"(dst) : "memory");
            }
        }
        sc_pending = 0;
    };
    auto copy_rest = [&]() {
        while (copy_on && sc_u < sc_units) {
            copy_issue();
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            copy_store();
        }
    };
    int job = bslot;
    if (job >= njobs) {
        if (COPY) copy_rest();
        return;
    }

    const int nk = g.K / BK;
    // The pieces of this wavefront are spread evenly over the K steps it will run (every tile's steps but the
    // last two), so that the scatter ends with the kernel instead of crowding its first part: measured on
    // the 32768-token workload, a piece every 5th step (what this gives there) against every 4th 660 -> 645 us,
    // every 3rd 680 us, every 2nd 687 us; every 6th would leave pieces for after the tile loop.
    if (COPY && copy_on) {
        const int my_tiles = (njobs - bslot + nblk - 1) / nblk;                           // > 0 here
        const int my_pieces = sc_u < sc_units ? (sc_units - sc_u + sc_stride - 1) / sc_stride : 0;
        sc_period = max(1, my_tiles * max(nk - 2, 0) / max(my_pieces, 1));
    }

    // ---- load sources: a scalar base per operand (advancing along K) + a 32-bit byte offset per lane ----
    // One wavefront-wide load fills 1 KB of LDS = ROWS_PER_LOAD consecutive tile rows; lane l
    // lands at row l / CPR, chunk position l % CPR.  Loads 0, 1 of the fused weight tile read the
    // gate matrix, loads 2, 3 the up matrix (tile rows 128 .. 255).
    const char *a_ptr = nullptr, *b_ptr0 = nullptr, *b_ptr1 = nullptr;  // uniform
    uint32_t a_voff[LOADS], b_voff[LOADS];
    int kpos = 0;
    int a_iss = 0, b_iss = 0;  // buffers the next loads go to
    auto set_a_sources = [&](const Tile &t) {
        const int ll = opaque_lane(), lrow = ll / CPR, lpos = ll % CPR;
        a_ptr = (const char *)g.A + (int64_t)t.m0 * g.lda * 2;
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int tr = (i * 8 + wave) * ROWS_PER_LOAD + lrow;  // tile row
            const int gchunk = lpos ^ swizzle_key(tr);               // global chunk that lands at position lpos
            const int m = min(tr, t.m_end - 1 - t.m0);
            a_voff[i] = (uint32_t)m * (uint32_t)(g.lda * 2) + (uint32_t)gchunk * 16u;
        }
    };
    auto set_b_sources = [&](const Tile &t, int n0) {
        const int64_t first = ((int64_t)t.slot * g.b_slot_stride + (int64_t)n0 * g.ldb) * 2;
        b_ptr0 = (const char *)g.B0 + first;
        b_ptr1 = FUSED_UP ? (const char *)g.B1 + first : b_ptr0;
        const int ll = opaque_lane(), lrow = ll / CPR, lpos = ll % CPR;
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int tr = (i * 8 + wave) * ROWS_PER_LOAD + lrow;
            const int gchunk = lpos ^ swizzle_key(tr);
            const int n = min(FUSED_UP ? (tr & 127) : tr, g.N - 1 - n0);  // n0 < N
            b_voff[i] = (uint32_t)n * (uint32_t)(g.ldb * 2) + (uint32_t)gchunk * 16u;
        }
        kpos = 0;
    };
    auto issue_a_one = [&](int i) { load16_to_lds(a_ptr, a_voff[i], smem + a_iss * A_BYTES + wave * 1024 + i * 8192); };
    auto issue_b_one = [&](int i) {
        load16_to_lds((FUSED_UP && i >= LOADS / 2) ? b_ptr1 : b_ptr0, b_voff[i],
                      smem + B_BASE + b_iss * B_BYTES + wave * 1024 + i * 8192);
    };
    auto advance_a = [&]() {
        a_ptr += BK * 2;
        a_iss ^= 1;
    };
    // the weight K offset jumps at K segment ends (a step never straddles one)
    auto advance_b = [&]() {
        int64_t step_bytes = BK * 2;
        kpos += BK;
        if (kpos == g.kseg_len) { kpos = 0; step_bytes += (g.kseg_stride - g.kseg_len) * 2; }
        b_ptr0 += step_bytes;
        b_ptr1 += step_bytes;
        b_iss = (b_iss + 1 == NBUF_B) ? 0 : b_iss + 1;
    };
    auto issue_a = [&]() {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) issue_a_one(i);
        advance_a();
    };
    auto issue_b = [&]() {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) issue_b_one(i);
        advance_b();
    };

    // fragments of v_mfma_f32_16x16x32_bf16: 16 rows x 32 K, row = base + (lane & 15) (bases are multiples
    // of 16), chunk 4 * g + (lane >> 4) of the step's K group g (two per step) stored at chunk ^ key(row);
    // per wavefront and group 4 weight fragments (FUSED_UP: two of the gate rows, two of the up rows)
    // and 8 activation fragments.
    const int frow = lane & 15, fkey = swizzle_key(frow);
    const int a_base = (wm * HALF_ROWS + frow) * ROW_BYTES;
    const int b_base = ((FUSED_UP ? wn * 32 : wn * 64) + frow) * ROW_BYTES;
    int pc[2];
#pragma unroll
    for (int gk = 0; gk < 2; ++gk) pc[gk] = ((gk * 4 + (lane >> 4)) ^ fkey) * 16;
    bf16x8_t fa[2][HF], fb[2][4];
    // fragment r of a K group: r < 4 weight rows, else activation rows
    auto fetch_one = [&](int buf, const char *sa, const char *sb, int gk, int r) {
        if (r < 4) {
            const int rows = FUSED_UP ? (r >> 1) * 128 + (r & 1) * 16 : r * 16;
            fb[buf][r] = *(const bf16x8_t *)(sb + b_base + rows * ROW_BYTES + pc[gk]);
        } else {
            fa[buf][r - 4] = *(const bf16x8_t *)(sa + a_base + (r - 4) * 16 * ROW_BYTES + pc[gk]);
        }
    };
    // what a K group needs on entry: its activation fragments and weight fragments 0, 1
    auto fetch_entry = [&](int buf, const char *sa, const char *sb, int gk) {
#pragma unroll
        for (int r = 0; r < 4 + HF; ++r)
            if (r < 2 || r >= 4) fetch_one(buf, sa, sb, gk, r);
    };

    // ---- one K step ---------------------------------------------------------------------------
    // Two K groups of 32 MFMAs each, in two passes: the eight activation fragments with weight fragments
    // 0 and 1, then with 2 and 3.  Registers: the activation fragments live through the group; weight
    // fragments 2 and 3 of a group are read during its first pass, and during the second pass the next
    // group's weight fragments 0, 1 (into the registers pass one has freed) and its activation fragment
    // i right after the current fragment i has had its last MFMA (56 fragment registers plus those in
    // flight, where holding both groups whole would take 96).
    // The weight loads of step g + 2 go out during the first group.  Before the second group the
    // workgroup synchronises once: by then every wavefront has read all of this step's buffers (so the
    // second group's weight fragments 2, 3 are read ahead of the barrier as well), and the activation
    // buffer is handed to the loads of step g + 2, issued during the second group; and each wavefront
    // has waited for its own loads of step g + 1, so after the barrier those have landed.  Loads
    // complete in issue order, so "everything but the newest LOADS loads" covers step g + 1.  The second
    // group's second pass reads the next step's first fragments from the next buffers (CROSS; not
    // across a tile boundary, where the registers are needed for the epilogue).
    // RD_*_POS: the read is issued after the group's MFMA number ..; LD_POS likewise for the four loads.
    int a_con = 0, b_con = 0;  // buffers the current step reads
    constexpr int NM = 4 * HF;                                                 // MFMAs per K group
    constexpr int RD_OWN23_POS[2] = {0, 1};                                    // this group's weight fragments 2, 3
    constexpr int RD_NXT23_POS[2] = {2 * HF + 3, 2 * HF + 5};                  // next group's weights 2, 3 (ahead of the barrier)
    constexpr int LD_POS[4] = {3, 7, 11, 15};
    // next group: weight fragments 0, 1 when pass one is over, activation fragment i after the last MFMA of
    // the current fragment i (number 2 HF + 2 i + 1), the last one after the last MFMA but one
    auto rd_nxt_pos = [](int r) { return r < 2 ? 2 * HF + r : (r - 4 == HF - 1 ? NM - 1 : 2 * HF + 2 + 2 * (r - 4)); };
    auto mfma_group = [&](f32x4_t (&acc)[HF][4], int cur) {
#pragma unroll
        for (int pass = 0; pass < 2; ++pass)
#pragma unroll
            for (int i = 0; i < HF; ++i)
#pragma unroll
                for (int jl = 0; jl < 2; ++jl) {
                    const int j = pass * 2 + jl;
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[cur][j], fa[cur][i], acc[i][j], 0, 0, 0);
                }
    };
    // Reads and loads of one group in program order = issue order wanted (direct loads and fragment reads
    // both touch LDS, so the compiler keeps them in this order).  own23: this group's weight fragments
    // 2, 3 are still to be read; next: read the next group's fragments from (na, nb, ngk) into buffer
    // nbuf, next23: including its weight fragments 2, 3.
    auto group_reads = [&](int cur, const char *ca, const char *cb, int cgk, bool own23, bool next, bool next23, int nbuf,
                           const char *na, const char *nb, int ngk, auto issue_one) {
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            if (own23) {
#pragma unroll
                for (int q = 0; q < 2; ++q)
                    if (RD_OWN23_POS[q] == m) fetch_one(cur, ca, cb, cgk, 2 + q);
            }
            if (next) {
#pragma unroll
                for (int r = 0; r < 4 + HF; ++r)
                    if ((r < 2 || r >= 4) && rd_nxt_pos(r) == m) fetch_one(nbuf, na, nb, ngk, r);
                if (next23) {
#pragma unroll
                    for (int q = 0; q < 2; ++q)
                        if (RD_NXT23_POS[q] == m) fetch_one(nbuf, na, nb, ngk, 2 + q);
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (LD_POS[q] == m) issue_one(q);
        }
    };
    // the same order for the instruction scheduler: after every MFMA the reads and the load placed there
    auto group_sched = [&](bool own23, bool next, bool next23) {
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
            int reads = 0;
            if (own23)
                for (int q = 0; q < 2; ++q) reads += RD_OWN23_POS[q] == m;
            if (next) {
                for (int r = 0; r < 4 + HF; ++r) reads += (r < 2 || r >= 4) && rd_nxt_pos(r) == m;
                if (next23)
                    for (int q = 0; q < 2; ++q) reads += RD_NXT23_POS[q] == m;
            }
            if (reads == 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // LDS reads
            if (reads == 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (LD_POS[q] == m) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);   // 1 VMEM
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    auto step = [&](f32x4_t (&acc)[HF][4], auto cross, bool store_copy = false) {
        constexpr bool CROSS = decltype(cross)::value;
        const char *sa = smem + a_con * A_BYTES, *sb = smem + B_BASE + b_con * B_BYTES;
        a_con ^= 1;
        b_con = (b_con + 1 == NBUF_B) ? 0 : b_con + 1;
        const char *sa_next = smem + a_con * A_BYTES, *sb_next = smem + B_BASE + b_con * B_BYTES;
        group_reads(0, sa, sb, 0, true, true, true, 1, sa, sb, 1, issue_b_one);
        mfma_group(acc, 0);
        group_sched(true, true, true);
        advance_b();
        asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)" ::: "memory");
        asm volatile("s_barrier" ::: "memory");
        // the carried scatter's piece (loaded before this step: covered by the wait above) goes out here, so
        // that its stores have a whole step until the next wait, which has to see them acknowledged
        if (COPY && store_copy) copy_store();
        group_reads(1, sa, sb, 1, false, CROSS, false, 0, sa_next, sb_next, 0, issue_a_one);
        advance_a();
        mfma_group(acc, 1);
        group_sched(false, CROSS, false);
    };
    // the same step for a wavefront with no valid rows in this tile: synchronise and load only
    auto idle_step = [&]() {
        a_con ^= 1;
        b_con = (b_con + 1 == NBUF_B) ? 0 : b_con + 1;
        issue_b();
        asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)" ::: "memory");
        asm volatile("s_barrier" ::: "memory");
        issue_a();
    };
    using T_ = std::integral_constant<bool, true>;
    using F_ = std::integral_constant<bool, false>;

    // ---- epilogue ---------------------------------------------------------------------------------
    // The weight fragment is the MFMA's first operand, so acc[i][j] holds a transposed 16x16 block (rows
    // 16 i .., columns 16 j ..; FUSED_UP: j < 2 gate, j >= 2 the up projection of the same columns):
    // element v of lane l is (n = 4 * (l / 16) + v, m = l % 16), i.e. four consecutive output columns of
    // one row.  Per 32-row sub-tile (two blocks i) the wavefront packs to bf16, transposes through LDS
    // (16-byte chunks XOR-swizzled by row) and writes whole rows with 16-byte stores.  The staging bytes
    // are the four 1 KB pieces of the free weight buffer that this wavefront's own next weight loads
    // fill, so no other wavefront touches them.
    constexpr int BNW = SH::BNW, ROWB = SH::ROWB;
    constexpr int CH = ROWB / 16;               // 16-byte chunks per staged row
    constexpr int KSH = (ROWB == 128) ? 1 : 2;  // rows per 256 bytes of LDS = 1 << KSH
    // byte o of the wavefront's logical 4 KB staging area -> offset inside a weight buffer
    auto stg_off = [&](int o) { return wave * 1024 + (o >> 10) * 8192 + (o & 1023); };
    auto epilogue = [&](f32x4_t (&acc)[HF][4], const Tile &t, int n0, int n_valid) {
        uint16_t *out = (uint16_t *)g.out;
        constexpr int ROWS_PER_IT = 64 / CH;
        const int el = opaque_lane(), er = el & 15, eq = el >> 4;   // not kept across the K loop
        const int rr = el / CH, cc = el % CH;
        const int ncol = n0 + wn * BNW + cc * 8;
        char *stg = smem + B_BASE + b_iss * B_BYTES;  // the buffer read in the tile's last step
#pragma unroll
        for (int i32 = 0; i32 < (HF + 1) / 2; ++i32) {
            if (i32 >= n_valid) break;
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                const int i = i32 * 2 + sub, row = sub * 16 + er;
                if (i >= HF) continue;   // an odd number of blocks: the last sub-tile has 16 rows
                const int wkey = (row >> KSH) & (CH - 1);
#pragma unroll
                for (int jn = 0; jn < (FUSED_UP ? 2 : 4); ++jn) {
                    float h[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        if (FUSED_UP) {
                            const float gt = acc[i][jn][r], up = acc[i][jn + 2][r];
                            h[r] = gt * __frcp_rn(1.0f + __expf(-gt)) * up;
                        } else {
                            h[r] = acc[i][jn][r];
                        }
                    }
                    const uint2 pk = make_uint2(pack_bf16x2(h[0], h[1]), pack_bf16x2(h[2], h[3]));
                    // columns 16 jn + 4 eq .. +3: chunk 2 jn + eq / 2, its low or high 8 bytes
                    *(uint2 *)(stg + stg_off(row * ROWB + (((jn * 2 + (eq >> 1)) ^ wkey) * 16) + (eq & 1) * 8)) = pk;
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // this wavefront's own writes, read back below
#pragma unroll
            for (int it = 0; it < 32 / ROWS_PER_IT; ++it) {
                const int ml = it * ROWS_PER_IT + rr;
                const int hrow = i32 * 32 + ml;                 // row inside the wavefront's half of the tile
                const int row = t.m0 + wm * HALF_ROWS + hrow;
                const int key = (ml >> KSH) & (CH - 1);
                const uint4 v = *(const uint4 *)(stg + stg_off(ml * ROWB + ((cc ^ key) * 16)));
                if (hrow < HALF_ROWS && row < t.m_end && ncol < g.N) *(uint4 *)(out + (int64_t)row * g.ldo + ncol) = v;
            }
            // LDS operations of one wavefront execute in order: the next sub-tile's writes cannot
            // overtake these reads
        }
    };

    // ---- tile loop ----------------------------------------------------------------------------------
    // Per tile of nk steps: steps 0 .. nk-3 load this tile's steps 2 .. nk-1; steps nk-2 and nk-1
    // load steps 0 and 1 of the next tile, or, for the workgroup's last tile, of this tile again (valid
    // addresses, nobody reads the data), so that every step is the same straight code.
    int cur_mt, cur_n0;
    job_tile(job, cur_mt, cur_n0);
    Tile cur = lookup(cur_mt);
    set_a_sources(cur);
    set_b_sources(cur, cur_n0);
    issue_a();
    issue_b();
    issue_a();
    issue_b();  // nk >= 2
    asm volatile("s_waitcnt vmcnt(8)" ::: "memory");  // step 0 landed; the 2 * LOADS loads of step 1 may be in flight
    asm volatile("s_barrier" ::: "memory");
    for (;;) {
        const int next_job = job + nblk;
        const bool has_next = next_job < njobs;  // uniform
        Tile nxt = cur;
        int nxt_n0 = cur_n0;
        if (has_next) {
            int nxt_mt;
            job_tile(next_job, nxt_mt, nxt_n0);
            nxt = lookup(nxt_mt);
        }
        // 32-row sub-tiles of this wavefront that hold at least one valid row (scalar)
        const int n_valid = max(0, min((HF + 1) / 2, (cur.m_end - (cur.m0 + wm * HALF_ROWS) + 31) / 32));
        if (n_valid > 0) {
            f32x4_t acc[HF][4];
#pragma unroll
            for (int i = 0; i < HF; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.0f;
            fetch_entry(0, smem + a_con * A_BYTES, smem + B_BASE + b_con * B_BYTES, 0);
            for (int kt = 0; kt + 2 < nk; ++kt) {
                bool copy_now = false;
                if (COPY && --sc_countdown <= 0) {
                    copy_now = true;
                    sc_countdown = sc_period;
                }
                if (copy_now) copy_issue();
                step(acc, T_{}, copy_now);
            }
            set_a_sources(nxt);
            set_b_sources(nxt, nxt_n0);
            step(acc, T_{});
            step(acc, F_{});
            epilogue(acc, cur, cur_n0, n_valid);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // staging reads done before the buffer is refilled
        } else {
            for (int kt = 0; kt + 2 < nk; ++kt) idle_step();
            set_a_sources(nxt);
            set_b_sources(nxt, nxt_n0);
            idle_step();
            idle_step();
        }
        if (!has_next) break;
        cur = nxt;
        cur_n0 = nxt_n0;
        job = next_job;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no load may still be on its way to LDS when the workgroup ends
    if (COPY) copy_rest();
}

// Rows per m-tile for this launch, as fragments per wavefront (8, 7, 6 or 5).  Tiles are dealt to the
// grid in whole rounds, so 2.6 rounds of full tiles cost 3; lower tiles are more but cheaper, and the
// height whose rounds x cost is smallest wins (ties to the higher tile).  Cost of a tile of HF
// fragments per wavefront relative to the full one: (HF + 2) / 10 (the weight tile's loads and the
// per-tile overheads do not shrink).  Every workgroup computes the same answer from the row segments
// on the device, from one read of their bounds.
template <int SEG_PER_LANE>
__device__ __forceinline__ int tile_height(const SegTable<SEG_PER_LANE> &segs, int n_tiles_n) {
    int best_hf = 8, best_cost = 0x7fffffff;
#pragma unroll
    for (int hf = 8; hf >= 5; --hf) {
        const int tiles = segs.count(32 * hf) * n_tiles_n;
        const int rounds = (tiles + (int)gridDim.x - 1) / (int)gridDim.x;
        const int cost = rounds * (hf + 2);
        if (cost < best_cost) { best_cost = cost; best_hf = hf; }
    }
    return best_hf;
}

// SEG_PER_LANE: 1 for up to 64 row segments, 4 for up to 256.  WHO only names the instantiation
// (EXPERTS: grouped expert FFN, SHARED: always-on shared experts), so that a kernel trace lists the
// two uses separately.
template <bool FUSED_UP, int SEG_PER_LANE, Who WHO>
__global__ __launch_bounds__(THREADS, 1) void gemm_bf16_persist_kernel(const GemmArgs g, int n_tiles_n) {
    SegTable<SEG_PER_LANE> segs;
    segs.load(g, (int)threadIdx.x & 63);
    // Lower tiles only for the experts' down projection: measured, they pay there (mixtral 258 -> 226 us,
    // qwen3moe 62 -> 55 us) and not for the gate+up projection, whose tile time hardly falls with its row
    // count; the shared experts' single segment of T rows fills its rounds with full tiles anyway.
    if constexpr (!FUSED_UP && WHO == EXPERTS) {
        switch (tile_height<SEG_PER_LANE>(segs, n_tiles_n)) {   // uniform over the grid
            case 8: persist_body<FUSED_UP, SEG_PER_LANE, WHO, 8>(g, n_tiles_n, segs); break;
            case 7: persist_body<FUSED_UP, SEG_PER_LANE, WHO, 7>(g, n_tiles_n, segs); break;
            case 6: persist_body<FUSED_UP, SEG_PER_LANE, WHO, 6>(g, n_tiles_n, segs); break;
            default: persist_body<FUSED_UP, SEG_PER_LANE, WHO, 5>(g, n_tiles_n, segs); break;
        }
    } else {
        persist_body<FUSED_UP, SEG_PER_LANE, WHO, 8>(g, n_tiles_n, segs);
    }
}

// Workgroups to launch on a device with `n_cu` compute units: one per compute unit, a multiple of 8.
inline int grid_blocks(int n_cu) {
    const int g = n_cu / N_XCD * N_XCD;
    return g < N_XCD ? N_XCD : g;
}

}  // namespace pers
}  // namespace grace
