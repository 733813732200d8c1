// grace_route: top-k gating, per-expert request counter, locality-first replica pick.
//
// Three launches (two when there are few chunks: every pick block then sums the
// histograms of the chunks before its own instead of reading a scanned copy), all
// integer-exact and free of order-dependent atomics:
//   1. topk_kernel   one wavefront per token: every lane ranks its logits against
//                    all others by (logit desc, expert id asc) through scalar
//                    broadcasts, ranks < k are the choices; softmax weights and a
//                    histogram of the chosen experts per chunk of tokens
//                    (topk_lanes_kernel, four lanes per token with sorted lists of the
//                    best k, for more than 8192 tokens with k <= 8);
//   2. route_scan    exclusive scan of the chunk histograms per expert -> the
//                    number of earlier requests of each expert before each chunk
//                    (the weighted round-robin counter of Section 4.3);
//   3. pick_kernel   one workgroup per 64 tokens walks their assignments in order (every
//                    wavefront 64 of them at a time), ranks equal experts with ballot-based
//                    matching, and maps request number c to the candidate of the tier
//                    Algorithm 4 selects whose cumulative polling-weight interval holds
//                    c mod W.
#include <type_traits>

#include "common.h"
#include "route_device.h"
#include "wave_utils.h"

namespace grace {

constexpr int TOPK_THREADS = 512;  // 8 wavefronts per chunk, TPW tokens each (chunk = 8 * TPW tokens)

constexpr int TOPK_LANES_MIN_T = 8193, TOPK_LANES_MIN_E = 32;  // from here on a few lanes per token (topk_lanes_kernel) where its conditions hold

// One wavefront per token, VPL experts per lane (token_topk); a histogram of the chosen experts per
// chunk of tokens feeds the request counter.
template <int VPL, int TOPK_TOK_PER_WAVE>
__global__ __launch_bounds__(TOPK_THREADS) void topk_kernel(const float *__restrict__ logits, int T, int E, int k,
                                                            int renorm, int32_t *__restrict__ topk_expert,
                                                            float *__restrict__ topk_weight,
                                                            int32_t *__restrict__ chunk_hist,
                                                            int32_t *__restrict__ clear, int n_clear) {
    __shared__ int32_t hist[GRACE_MAX_EXPERTS];
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < E; i += TOPK_THREADS) hist[i] = 0;
    // counters a later kernel of the same call accumulates into
    for (int64_t i = (int64_t)blockIdx.x * TOPK_THREADS + tid; i < n_clear; i += (int64_t)gridDim.x * TOPK_THREADS) clear[i] = 0;
    __syncthreads();
    const int chunk = (int)blockIdx.x;
    const int t_begin = (chunk * (TOPK_THREADS / 64) + wave) * TOPK_TOK_PER_WAVE;
    // all of this wavefront's logits are requested before any is used
    float raw[TOPK_TOK_PER_WAVE][VPL];
#pragma unroll
    for (int i = 0; i < TOPK_TOK_PER_WAVE; ++i)
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
            const int t = t_begin + i, e = lane + 64 * v;
            raw[i][v] = (t < T && e < E) ? logits[(size_t)t * E + e] : -INFINITY;
        }
#pragma unroll
    for (int i = 0; i < TOPK_TOK_PER_WAVE; ++i) {
        const int t = t_begin + i;
        if (t >= T) break;  // uniform per wavefront
        int rank[VPL];
        float weight[VPL];
        token_topk<VPL>(raw[i], lane, E, k, renorm, rank, weight);
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
            const int e = lane + 64 * v;
            if (e < E && rank[v] < k) {
                topk_expert[(size_t)t * k + rank[v]] = e;
                topk_weight[(size_t)t * k + rank[v]] = weight[v];
                atomicAdd(&hist[e], 1);
            }
        }
    }
    __syncthreads();
    for (int i = tid; i < E; i += TOPK_THREADS) chunk_hist[(size_t)chunk * E + i] = hist[i];
}

// The same gate with four lanes per token, for batches large enough that the wavefront-per-token
// kernel above is bound by its vector instructions (about 280 per token there, about 90 here): lane q
// of a token scans experts [q * NV, q * NV + NV) in ascending order and keeps its K best as a sorted
// list (insertion by strict "greater", so equal logits stay in ascending expert order); the lists of
// the four lanes are merged pairwise the same way (the lower lane holds the lower expert ids and keeps
// its entries ahead of equal ones), and lane 0 of the token writes the k <= K choices.  A workgroup
// holds one chunk of tokens (blockDim = chunk tokens * 4).  Needs E % 4 == 0 and 16-byte aligned logits.
constexpr int TOPK_LANES = 4;
template <int K>
struct BestList {
    uint32_t key[K];  // ordered_bits of the logit, descending; 0 = empty
    int id[K];
    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int j = 0; j < K; ++j) { key[j] = 0u; id[j] = 0; }
    }
    // (kx, ix) goes in front of the first entry it beats and behind those it ties with; the entries from
    // there on move down one place.  All K comparisons are against the list as it was (it is sorted, so
    // they are false up to the place of insertion and true from there on) and do not wait for each other.
    __device__ __forceinline__ void insert(uint32_t kx, int ix) {
        bool gt[K];
#pragma unroll
        for (int j = 0; j < K; ++j) gt[j] = kx > key[j];
#pragma unroll
        for (int j = K - 1; j >= 1; --j) {
            const uint32_t in_k = gt[j - 1] ? key[j - 1] : kx;
            const int in_i = gt[j - 1] ? id[j - 1] : ix;
            key[j] = gt[j] ? in_k : key[j];
            id[j] = gt[j] ? in_i : id[j];
        }
        key[0] = gt[0] ? kx : key[0];
        id[0] = gt[0] ? ix : id[0];
    }
};

template <int DPP_CTRL>
__device__ __forceinline__ int dpp_move(int v) {
    return __builtin_amdgcn_update_dpp(v, v, DPP_CTRL, 0xF, 0xF, false);
}

__device__ __forceinline__ float from_ordered_bits(uint32_t kb) {
    return __uint_as_float((kb & 0x80000000u) ? (kb ^ 0x80000000u) : ~kb);
}

template <int NV, int K>
__global__ __launch_bounds__(64 * TOPK_LANES) void topk_lanes_kernel(const float *__restrict__ logits, int T, int E, int k, int renorm,
                                                            int32_t *__restrict__ topk_expert,
                                                            float *__restrict__ topk_weight,
                                                            int32_t *__restrict__ chunk_hist, int32_t *__restrict__ clear,
                                                            int n_clear, int chunk_tokens) {
    constexpr int L = TOPK_LANES;
    static_assert(L == 4, "the merge and the broadcasts below are written for quads of lanes");
    static_assert(NV % 4 == 0, "16-byte loads");
    __shared__ int32_t hist[GRACE_MAX_EXPERTS];
    const int tid = (int)threadIdx.x, nthr = (int)blockDim.x;
    for (int i = tid; i < E; i += nthr) hist[i] = 0;
    for (int64_t i = (int64_t)blockIdx.x * nthr + tid; i < n_clear; i += (int64_t)gridDim.x * nthr) clear[i] = 0;
    __syncthreads();
    const int chunk = (int)blockIdx.x;
    const int q = tid % L;
    const int t = chunk * chunk_tokens + tid / L;
    const bool live = t < T;
    // this lane's logits, all requested before any is used
    float val[NV];
    const int e0 = q * NV;
#pragma unroll
    for (int g = 0; g < NV / 4; ++g) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (live && e0 + 4 * g < E) v = *(const float4 *)(logits + (size_t)t * E + e0 + 4 * g);
        val[4 * g] = v.x; val[4 * g + 1] = v.y; val[4 * g + 2] = v.z; val[4 * g + 3] = v.w;
    }
    BestList<K> best;
    best.clear();
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        float x = val[i];
        if (x == 0.0f) x = 0.0f;  // -0.0 and +0.0 compare equal: make them the same bits
        val[i] = x;
        best.insert((e0 + i < E) ? ordered_bits(x) : 0u, e0 + i);
    }
    // merge: after the step with distance s, lanes with q % (2 s) == 0 hold the best of 2 s lanes
#pragma unroll
    for (int s = 1; s < L; s <<= 1) {
        uint32_t ok[K];
        int oi[K];
#pragma unroll
        for (int j = 0; j < K; ++j) {
            ok[j] = (uint32_t)(s == 1 ? dpp_move<0xB1>((int)best.key[j]) : dpp_move<0x4E>((int)best.key[j]));
            oi[j] = s == 1 ? dpp_move<0xB1>(best.id[j]) : dpp_move<0x4E>(best.id[j]);
        }
#pragma unroll
        for (int j = 0; j < K; ++j) best.insert(ok[j], oi[j]);
    }
    // softmax over all E logits, or over the k chosen ones; the maximum is the first choice
    const float mx = from_ordered_bits(best.key[0]);  // valid in lane q == 0
    float ex[K], sel = 0.0f;
#pragma unroll
    for (int j = 0; j < K; ++j) {
        ex[j] = j < k ? expf(from_ordered_bits(best.key[j]) - mx) : 0.0f;
        sel += ex[j];
    }
    float norm = sel;
    if (!renorm) {  // uniform
        const float mx_all = __builtin_bit_cast(float, dpp_move<0x00>(__builtin_bit_cast(int, mx)));  // the quad's lane 0
        float part[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < NV; ++i) part[i & 3] += (e0 + i < E) ? expf(val[i] - mx_all) : 0.0f;
        float den = (part[0] + part[1]) + (part[2] + part[3]);
        den += __builtin_bit_cast(float, dpp_move<0xB1>(__builtin_bit_cast(int, den)));
        den += __builtin_bit_cast(float, dpp_move<0x4E>(__builtin_bit_cast(int, den)));
        norm = den;
    }
    if (live && q == 0) {
#pragma unroll
        for (int j = 0; j < K; ++j)
            if (j < k) {
                topk_expert[(size_t)t * k + j] = best.id[j];
                topk_weight[(size_t)t * k + j] = ex[j] / norm;
                atomicAdd(&hist[best.id[j]], 1);
            }
    }
    __syncthreads();
    for (int i = tid; i < E; i += nthr) chunk_hist[(size_t)chunk * E + i] = hist[i];
}

__global__ __launch_bounds__(SCAN_THREADS) void route_scan_kernel(const int32_t *__restrict__ hist,
                                                                  int32_t *__restrict__ base, int nchunks, int E,
                                                                  const uint32_t *__restrict__ rr_in,
                                                                  uint32_t *__restrict__ rr_out,
                                                                  int32_t *__restrict__ expert_count,
                                                                  const int32_t *__restrict__ cand_ptr,
                                                                  const uint32_t *__restrict__ cand_cum) {
    __shared__ int32_t totals[GRACE_MAX_EXPERTS];
    __shared__ int32_t part_sums[SCAN_THREADS];
    const int tid = (int)threadIdx.x;
    for (int i = tid; i < E; i += SCAN_THREADS) totals[i] = 0;
    __syncthreads();
    block_scan_chunks(hist, base, nchunks, E, totals, part_sums);
    __syncthreads();
    for (int e = tid; e < E; e += SCAN_THREADS) {
        const int32_t n = totals[e];
        expert_count[e] = n;
        if (rr_out) {
            rr_out[e] = next_rr(rr_in, e, n, cand_ptr, cand_cum);
        }
    }
}

// One workgroup picks the replicas of PICK_TOKENS consecutive tokens = rows_per_block rows of the
// top-k kernel's chunk histograms.
// FOLD = false: chunk_counts is the scanned histogram (requests of each expert before each row).
// FOLD = true: chunk_counts is the raw per-row histogram; the block sums the rows before its own,
// and the last block also writes expert_count and rr_out.
// The assignments are walked in rounds of PICK_THREADS, every wavefront taking 64 consecutive ones:
// it matches equal experts with ballots and leaves the size of every match set in its row of wcnt;
// an exclusive scan over the eight rows, continued from cnt (requests before this round), gives each
// wavefront the number of earlier requests of every expert, and request number c of expert e maps to
// the candidate of the tier Algorithm 4 selects whose cumulative polling-weight interval holds c mod W.
// With inst_hist (zeroed beforehand) every pick is also counted per chunk of PERM_CHUNK assignments
// and instance: the histogram the dispatch permutation starts from (integer atomics: exact in any order).
constexpr int PICK_LDS_CANDS = 1024;  // candidate entries of one view that are staged in LDS (else read from global memory)
constexpr int PICK_THREADS = 512, PICK_WAVES = PICK_THREADS / 64;
constexpr int PICK_TOKENS = 64;       // tokens per workgroup

template <bool FOLD>
__global__ __launch_bounds__(PICK_THREADS) void pick_kernel(const int32_t *__restrict__ topk_expert, int64_t n_assign,
                                                            int E, int k, const int32_t *__restrict__ chunk_counts,
                                                            int nrows, int rows_per_block,
                                                            const uint32_t *__restrict__ rr_in,
                                                            uint32_t *__restrict__ rr_out,
                                                            int32_t *__restrict__ expert_count,
                                                            const int32_t *__restrict__ cand_ptr,
                                                            const int32_t *__restrict__ cand_g,
                                                            const uint32_t *__restrict__ cand_cum,
                                                            int32_t *__restrict__ topk_inst, int nbits,
                                                            int32_t *__restrict__ inst_hist, int I,
                                                            const int32_t *__restrict__ super_tot, int c_first,
                                                            int n_cand) {
    __shared__ int32_t cnt[GRACE_MAX_EXPERTS];                // requests of each expert before the current round
    __shared__ int32_t wcnt[PICK_WAVES][GRACE_MAX_EXPERTS];   // per wavefront: match set sizes, then requests before it
    __shared__ int32_t s_ptr[GRACE_MAX_EXPERTS + 1];  // this view's candidate lists, offsets from its first entry
    __shared__ int32_t s_g[PICK_LDS_CANDS];
    __shared__ uint32_t s_cum[PICK_LDS_CANDS];
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int blk = (int)blockIdx.x;
    const int64_t a0 = (int64_t)blk * PICK_TOKENS * k;
    const int64_t a1 = min(n_assign, a0 + (int64_t)PICK_TOKENS * k);
    const int row0 = blk * rows_per_block;  // first histogram row of this block's tokens
    // the first round's experts and the candidate table are fetched before the counters are
    // prepared, so the picks below do not wait on chains of dependent global loads
    int e_first = (a0 + tid < a1) ? topk_expert[a0 + tid] : -1;
    // c_first = cand_ptr[0], n_cand = cand_ptr[E] - c_first: known to the host, so the staging loads
    // below do not wait for them.  The table entries stay in registers until the counters are prepared:
    // their loads and those of the histogram rows are then in flight together (a kernel's first loads
    // miss every cache level that is flushed between kernels, so each dependent round costs microseconds).
    const bool table_in_lds = n_cand <= PICK_LDS_CANDS;  // uniform
    constexpr int CANDS_PER_THREAD = PICK_LDS_CANDS / PICK_THREADS;
    static_assert(GRACE_MAX_EXPERTS + 1 <= PICK_THREADS && PICK_LDS_CANDS % PICK_THREADS == 0, "one offset, whole entries per thread");
    int32_t st_ptr = 0, st_g[CANDS_PER_THREAD];
    uint32_t st_cum[CANDS_PER_THREAD];
    if (table_in_lds) {
        if (tid <= E) st_ptr = cand_ptr[tid];
#pragma unroll
        for (int q = 0; q < CANDS_PER_THREAD; ++q) {
            const int i = tid + q * PICK_THREADS;
            st_g[q] = 0;
            st_cum[q] = 0u;
            if (i < n_cand) {
                st_g[q] = cand_g[c_first + i];
                st_cum[q] = cand_cum[c_first + i];
            }
        }
    }
    if (FOLD) {
        // requests before this block: the histogram rows 0 .. row0-1, or, with super_tot, the super
        // rows before row0's super-chunk and the rows inside it
        for (int e = tid; e < E; e += PICK_THREADS) cnt[e] = 0;
        __syncthreads();
        if (super_tot) {
            const int s = row0 / FOLD_SUPER;
            block_add_rows<PICK_THREADS>(super_tot, 0, s, E, cnt, tid);
            block_add_rows<PICK_THREADS>(chunk_counts, s * FOLD_SUPER, row0, E, cnt, tid);
        } else {
            block_add_rows<PICK_THREADS>(chunk_counts, 0, row0, E, cnt, tid);
        }
    } else {
        for (int e = tid; e < E; e += PICK_THREADS) cnt[e] = chunk_counts[(size_t)row0 * E + e];
    }
    if (table_in_lds) {
        if (tid <= E) s_ptr[tid] = st_ptr - c_first;
#pragma unroll
        for (int q = 0; q < CANDS_PER_THREAD; ++q) {
            const int i = tid + q * PICK_THREADS;
            if (i < n_cand) {
                s_g[i] = st_g[q];
                s_cum[i] = st_cum[q];
            }
        }
    }
    const int32_t *t_ptr = table_in_lds ? s_ptr : cand_ptr;
    const int32_t *t_g = table_in_lds ? s_g : cand_g;
    const uint32_t *t_cum = table_in_lds ? s_cum : cand_cum;
    const uint64_t lt = lanemask_lt();
    const int ibits = bits_for(I);
    static_assert(PERM_CHUNK % 64 == 0, "a wavefront's assignments must not straddle permutation chunks");
    for (int64_t b0 = a0; b0 < a1; b0 += PICK_THREADS) {
        const int64_t a = b0 + tid;
        const int e_raw = (b0 == a0) ? e_first : (a < a1 ? topk_expert[a] : -1);
        const bool valid = (unsigned)e_raw < (unsigned)E;  // -1 past the end
        const int e = valid ? e_raw : 0;
        for (int i = lane; i < E; i += 64) wcnt[wave][i] = 0;  // this wavefront's row; its LDS operations execute in order
        const uint64_t same = wave_match((uint32_t)e, valid, nbits);
        if (valid && is_last_of(same)) wcnt[wave][e] = (int32_t)__popcll(same);
        __syncthreads();  // also orders the counters prepared above, or the previous round's, before the scan
        for (int i = tid; i < E; i += PICK_THREADS) {
            int32_t run = cnt[i];
#pragma unroll
            for (int w = 0; w < PICK_WAVES; ++w) {
                const int32_t c = wcnt[w][i];
                wcnt[w][i] = run;
                run += c;
            }
            cnt[i] = run;
        }
        __syncthreads();
        int g = 0;
        if (valid) {
            const uint64_t c = (uint64_t)(uint32_t)wcnt[wave][e] + (uint32_t)__popcll(same & lt) + (uint64_t)(rr_in ? rr_in[e] : 0u);
            g = pick_candidate(c, e, t_ptr, t_g, t_cum);
            topk_inst[a] = g;
        }
        if (inst_hist) {
            // a wavefront's 64 assignments lie in one permutation chunk (both are multiples of 64):
            // one atomic per distinct instance, by the highest lane of its match set
            const bool counted = valid && (unsigned)g < (unsigned)I;
            const uint64_t same_g = wave_match((uint32_t)g, counted, ibits);
            if (counted && is_last_of(same_g)) atomicAdd(&inst_hist[(a / PERM_CHUNK) * I + g], (int32_t)__popcll(same_g));
        }
        __syncthreads();  // wcnt is cleared again in the next round
    }
    if (FOLD && blk == (int)gridDim.x - 1) {
        // after its last round the last block's counters hold every request of the call
        for (int e = tid; e < E; e += PICK_THREADS) {
            const int32_t n = cnt[e];
            expert_count[e] = n;
            if (rr_out) rr_out[e] = next_rr(rr_in, e, n, cand_ptr, cand_cum);
        }
    }
}

}  // namespace grace

namespace grace {

// Top-k gate of T >= 1 tokens; chunk_hist receives ceil(T / route_chunk_tokens(T)) x E expert counts.
int launch_topk(const float *logits, int T, int E, int k, int renorm, int32_t *topk_expert, float *topk_weight,
                int32_t *chunk_hist, int32_t *clear, int n_clear, hipStream_t st) {
    const int chunk_tokens = route_chunk_tokens(T);
    const int nchunks = (int)ceil_div(T, chunk_tokens);
    if (T >= TOPK_LANES_MIN_T && E >= TOPK_LANES_MIN_E && k <= 8 && E % 4 == 0 && ((uintptr_t)logits & 15) == 0) {
        const unsigned thr = (unsigned)(chunk_tokens * TOPK_LANES);
        auto launch = [&](auto nv) {  // list length: the next of 2, 4, 6, 8 from k on
            constexpr int NV = decltype(nv)::value;
            auto *kern = k <= 2 ? topk_lanes_kernel<NV, 2> : k <= 4 ? topk_lanes_kernel<NV, 4> : k <= 6 ? topk_lanes_kernel<NV, 6>
                                                                                                       : topk_lanes_kernel<NV, 8>;
            kern<<<nchunks, thr, 0, st>>>(logits, T, E, k, renorm, topk_expert, topk_weight, chunk_hist, clear, n_clear,
                                          chunk_tokens);
        };
        if (E <= 64) launch(std::integral_constant<int, 16>{});
        else if (E <= 128) launch(std::integral_constant<int, 32>{});
        else launch(std::integral_constant<int, 64>{});
        GRACE_LAUNCH_CHECK("topk_lanes_kernel");
        return GRACE_OK;
    }
#define GRACE_TOPK(VPL)                                                                                              \
    if (chunk_tokens == ROUTE_CHUNK_SMALL)                                                                           \
        topk_kernel<VPL, ROUTE_CHUNK_SMALL / (TOPK_THREADS / 64)><<<nchunks, TOPK_THREADS, 0, st>>>(                \
            logits, T, E, k, renorm, topk_expert, topk_weight, chunk_hist, clear, n_clear);                          \
    else if (chunk_tokens == ROUTE_CHUNK_LARGE)                                                                      \
        topk_kernel<VPL, ROUTE_CHUNK_LARGE / (TOPK_THREADS / 64)><<<nchunks, TOPK_THREADS, 0, st>>>(                \
            logits, T, E, k, renorm, topk_expert, topk_weight, chunk_hist, clear, n_clear);                          \
    else                                                                                                             \
        topk_kernel<VPL, ROUTE_CHUNK_HUGE / (TOPK_THREADS / 64)><<<nchunks, TOPK_THREADS, 0, st>>>(                 \
            logits, T, E, k, renorm, topk_expert, topk_weight, chunk_hist, clear, n_clear)
    switch ((E + 63) / 64) {
        case 1: GRACE_TOPK(1); break;
        case 2: GRACE_TOPK(2); break;
        case 3: GRACE_TOPK(3); break;
        default: GRACE_TOPK(4); break;
    }
#undef GRACE_TOPK
    GRACE_LAUNCH_CHECK("topk_kernel");
    return GRACE_OK;
}

int check_route_args(const grace_table *table, int32_t local_rank, grace_policy policy, const float *logits, int32_t T,
                     int32_t E, int32_t k, const uint32_t *rr_in, const uint32_t *rr_out, const int32_t *topk_expert,
                     const float *topk_weight, const int32_t *topk_inst, const int32_t *expert_count, const void *ws) {
    if (!table) return fail(GRACE_EINVAL, "route: table is null");
    if (T < 0) return fail(GRACE_EINVAL, "route: T=%d is negative", T);
    if (E != table->E) return fail(GRACE_ESHAPE, "route: E=%d but the table has %d experts", E, table->E);
    if (k < 1 || k > E || k > GRACE_MAX_TOPK)
        return fail(GRACE_EINVAL, "route: k=%d outside [1, min(E=%d, %d)]", k, E, GRACE_MAX_TOPK);
    if (local_rank < 0 || local_rank >= table->R)
        return fail(GRACE_EINVAL, "route: local_rank=%d outside [0,%d)", local_rank, table->R);
    if (policy != GRACE_POLICY_TAR && policy != GRACE_POLICY_WRR)
        return fail(GRACE_EINVAL, "route: unknown policy %d", (int)policy);
    if ((int64_t)T * k > INT32_MAX) return fail(GRACE_ESHAPE, "route: T*k exceeds 2^31-1");
    if (!expert_count || !ws) return fail(GRACE_EINVAL, "route: expert_count or ws is null");
    if (rr_in && rr_out && (uintptr_t)rr_in < (uintptr_t)(rr_out + E) && (uintptr_t)rr_out < (uintptr_t)(rr_in + E))
        return fail(GRACE_EINVAL, "route: rr_out overlaps rr_in");
    if (T > 0 && (!logits || !topk_expert || !topk_weight || !topk_inst))
        return fail(GRACE_EINVAL, "route: null device pointer");
    return GRACE_OK;
}

}  // namespace grace

namespace grace {

// The launches of grace_route for T >= 0 checked arguments.  With inst_hist (ceil(T*k / PERM_CHUNK) x I
// counters, T >= 1) the picks are also counted per permutation chunk and instance.
int launch_route(const grace_table *table, int32_t local_rank, grace_policy policy, const float *logits, int32_t T,
                 int32_t E, int32_t k, int32_t renorm, const uint32_t *rr_in, uint32_t *rr_out, int32_t *topk_expert,
                 float *topk_weight, int32_t *topk_inst, int32_t *expert_count, void *ws, int32_t *inst_hist,
                 hipStream_t st) {
    const int chunk_tokens = route_chunk_tokens(T);
    const int nchunks = (int)ceil_div(T, chunk_tokens);
    const int I = table->I;
    int32_t *hist = (int32_t *)ws;
    int32_t *base = (int32_t *)((char *)ws + align_up((size_t)nchunks * E * 4, 256));
    const int view = policy == GRACE_POLICY_WRR ? table->R : local_rank;
    const int32_t *cand_ptr = table->d_cand_ptr + (size_t)view * E;
    const int c_first = table->cand_view[view], n_cand = table->cand_view[view + 1] - c_first;
    if (nchunks > 0) {
        const int64_t n_clear = inst_hist ? ceil_div((int64_t)T * k, PERM_CHUNK) * I : 0;
        const int rc_topk = launch_topk(logits, T, E, k, renorm, topk_expert, topk_weight, hist, inst_hist, (int)n_clear, st);
        if (rc_topk != GRACE_OK) return rc_topk;
    }
    int nbits = 0;
    while ((1 << nbits) < E) ++nbits;
    static_assert(PICK_TOKENS % ROUTE_CHUNK_SMALL == 0 && PICK_TOKENS % ROUTE_CHUNK_LARGE == 0 && PICK_TOKENS % ROUTE_CHUNK_HUGE == 0,
                  "a pick block covers whole histogram rows");
    const int rows_per_block = PICK_TOKENS / chunk_tokens;
    const int pick_blocks = (int)ceil_div(T, PICK_TOKENS);
    const int mode = fold_mode(table, nchunks, E);
    if (mode != 0) {
        const int32_t *super_tot = nullptr;
        if (mode == 2) {  // column sums per super-chunk of rows, into the (otherwise unused) scan buffer
            super_sum_kernel<<<(unsigned)ceil_div(nchunks, FOLD_SUPER), SUPER_THREADS, 0, st>>>(hist, nchunks, E, base);
            GRACE_LAUNCH_CHECK("super_sum_kernel");
            super_tot = base;
        }
        pick_kernel<true><<<pick_blocks, PICK_THREADS, 0, st>>>(topk_expert, (int64_t)T * k, E, k, hist, nchunks,
                                                                rows_per_block, rr_in, rr_out, expert_count, cand_ptr,
                                                                table->d_cand_g, table->d_cand_cum, topk_inst, nbits,
                                                                inst_hist, I, super_tot, c_first, n_cand);
        GRACE_LAUNCH_CHECK("pick_kernel");
        return GRACE_OK;
    }
    route_scan_kernel<<<1, SCAN_THREADS, 0, st>>>(hist, base, nchunks, E, rr_in, rr_out, expert_count, cand_ptr,
                                                  table->d_cand_cum);
    GRACE_LAUNCH_CHECK("route_scan_kernel");
    if (nchunks > 0) {
        pick_kernel<false><<<pick_blocks, PICK_THREADS, 0, st>>>(topk_expert, (int64_t)T * k, E, k, base, nchunks,
                                                                 rows_per_block, rr_in, rr_out, expert_count, cand_ptr,
                                                                 table->d_cand_g, table->d_cand_cum, topk_inst, nbits,
                                                                 inst_hist, I, nullptr, c_first, n_cand);
        GRACE_LAUNCH_CHECK("pick_kernel");
    }
    return GRACE_OK;
}

}  // namespace grace

using namespace grace;

extern "C" int grace_route(const grace_table *table, int32_t local_rank, grace_policy policy, const float *logits, int32_t T, int32_t E,
                           int32_t k, int32_t renorm, const uint32_t *rr_in, uint32_t *rr_out, int32_t *topk_expert,
                           float *topk_weight, int32_t *topk_inst, int32_t *expert_count, void *ws, void *stream) {
    const int rc = check_route_args(table, local_rank, policy, logits, T, E, k, rr_in, rr_out, topk_expert, topk_weight,
                                    topk_inst, expert_count, ws);
    if (rc != GRACE_OK) return rc;
    return launch_route(table, local_rank, policy, logits, T, E, k, renorm, rr_in, rr_out, topk_expert, topk_weight,
                        topk_inst, expert_count, ws, nullptr, (hipStream_t)stream);
}
