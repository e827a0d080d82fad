// Token permutation / dispatch packing for one rank: a deterministic, stable
// counting sort of the rank's (token, expert) assignments by local expert,
// then a row gather that either copies BF16 rows or encodes them to MXFP4.
// Stands in for the all-to-all dispatch of the paper's pipeline (Sec.
// "Overhead-Aware Pipeline Orchestration"); the weight encoder overlaps it.
#include "common.h"
#include "hist_reduce.h"
#include "mxfp4_device.h"
#include <type_traits>

namespace realb {

constexpr int kIters = kPermChunk / 64;   // 64 assignments per wave iteration
// Chunks (= waves) per block of the count and rank kernels: kPermGroup (4) for long batches, 16 for short ones.  These
// latency-bound kernels run beside the HBM-bound encoders of the side stream.  Measured, whole layer steps: with more than
// about 500 chunks (32k and 64k tokens) 4-wave blocks are 1 % faster -- a small block finds room on a busy CU sooner --,
// with fewer (16k tokens: 384 chunks, 24 blocks of 16 waves) the large blocks are, by as much in the prefetched form of
// the call.  The workspace is sized for the small groups.
constexpr int kGroupLong = kPermGroup, kGroupShort = 16;
static int perm_group(int n_chunks) { return n_chunks > 512 ? kGroupLong : kGroupShort; }

// Inclusive prefix sum over the 64 lanes with DPP only: four shifts inside each row of 16 lanes, then the
// last lane of row 0 / row 2 is added to the following row, then lane 31 to the upper half.
__device__ __forceinline__ int wave_inclusive_scan(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, false);     // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, false);     // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, false);     // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, false);     // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);     // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);     // row_bcast:31 into rows 2 and 3
    return v;
}
__device__ __forceinline__ int wave_sum(int v) { return __builtin_amdgcn_readlane(wave_inclusive_scan(v), 63); }

// The local expert (or -1) of each of the 4 x 64 assignments a = t*k + j of a wave's chunk.
__device__ __forceinline__ void load_chunk(int (&le)[kIters], const int32_t* __restrict__ topk_ids, int chunk, int n_chunks, int A,
                                           int lo, int lane) {
#pragma unroll
    for (int i = 0; i < kIters; ++i) {
        const int a = chunk * kPermChunk + i * 64 + lane;
        le[i] = (chunk < n_chunks && a < A) ? topk_ids[a] - lo : -1;
    }
}

// Phase 1 (a block = one group of G chunks, one wave per chunk): each wave counts, per local expert, the
// assignments of its chunk of kPermChunk consecutive flat indices (lane e holds expert e's count); the block adds
// them up per expert.  wave_cnt is expert-major [n_local, n_chunks], group_cnt [n_local, n_groups].
// gsum: 64 ints of LDS.
template <int G>
__device__ __forceinline__ void perm_count_body(int* gsum, int group, const int32_t* __restrict__ topk_ids, int A, int lo, int n_local,
                                                int n_chunks, int n_groups, int32_t* __restrict__ wave_cnt,
                                                int32_t* __restrict__ group_cnt) {
    const int lane = threadIdx.x & 63;
    const int chunk = group * G + (threadIdx.x >> 6);
    int le[kIters];
    load_chunk(le, topk_ids, chunk, n_chunks, A, lo, lane);
    if (threadIdx.x < 64) gsum[threadIdx.x] = 0;
    __syncthreads();
    int cnt = 0;
#pragma unroll
    for (int i = 0; i < kIters; ++i)
        for (int e = 0; e < n_local; ++e) {
            const unsigned long long m = __ballot(le[i] == e);
            if (lane == e) cnt += __popcll(m);
        }
    if (chunk < n_chunks && lane < n_local) {
        wave_cnt[(size_t)lane * n_chunks + chunk] = cnt;
        atomicAdd(&gsum[lane], cnt);
    }
    __syncthreads();
    if ((int)threadIdx.x < n_local) group_cnt[(size_t)threadIdx.x * n_groups + group] = gsum[threadIdx.x];
}

template <int G>
__global__ void __launch_bounds__(64 * G) perm_count_kernel(const int32_t* __restrict__ topk_ids, int A, int lo, int n_local,
                                                                  int n_chunks, int n_groups, int32_t* __restrict__ wave_cnt,
                                                                  int32_t* __restrict__ group_cnt) {
    __shared__ int gsum[64];
    perm_count_body<G>(gsum, blockIdx.x, topk_ids, A, lo, n_local, n_chunks, n_groups, wave_cnt, group_cnt);
}

// The layer call's histogram reduce shares a launch with the permutation's count kernel: the first D blocks add up the
// routing kernel's partial histograms, one EP rank each (and hand the per-rank statistics to the host), the other
// blocks count their groups of chunks.  One kernel boundary less on a path made of short, latency-bound kernels.
template <int G>
__global__ void __launch_bounds__(64 * G) reduce_and_count_kernel(const int32_t* __restrict__ hist_part, int n_part, int E, int D,
                                                                        int32_t* __restrict__ expert_cnt, int32_t* __restrict__ expert_vis,
                                                                        int32_t* __restrict__ rank_load, int32_t* __restrict__ rank_vis,
                                                                        unsigned long long* __restrict__ stats_words, int stats_seq,
                                                                        const int32_t* __restrict__ topk_ids,
                                                                        int A, int lo, int n_local, int n_chunks, int n_groups,
                                                                        int32_t* __restrict__ wave_cnt, int32_t* __restrict__ group_cnt) {
    extern __shared__ int32_t dyn[];                  // 2*E/D ints (reduce blocks only)
    __shared__ int gsum[64];
    if ((int)blockIdx.x < D)
        hist_reduce_body(dyn, hist_part, n_part, E, D, blockIdx.x, expert_cnt, expert_vis, rank_load, rank_vis, stats_words, stats_seq);
    else perm_count_body<G>(gsum, blockIdx.x - D, topk_ids, A, lo, n_local, n_chunks, n_groups, wave_cnt, group_cnt);
}

// Phase 2 (same blocks): every block first works out, from the group sums, each expert's total (whose exclusive scan
// over the experts is expert_offsets; block 0 stores it) and the number of its assignments in earlier groups -- wave w
// adds up expert w's column of group_cnt, 64 groups per step -- so no separate scan kernel sits between the two
// phases.  Then each wave walks its chunk again and gives every local assignment its row:
// expert_offsets[e] + (assignments of e in earlier groups) + (in earlier chunks of the group) + (rank inside the chunk).
template <int G>
__global__ void __launch_bounds__(64 * G) perm_rank_kernel(const int32_t* __restrict__ topk_ids, int A, int lo, int n_local,
                                                                 int n_chunks, int n_groups, const int32_t* __restrict__ wave_cnt,
                                                                 const int32_t* __restrict__ group_cnt,
                                                                 int32_t* __restrict__ expert_offsets,
                                                                 int32_t* __restrict__ row_to_assign, int32_t* __restrict__ assign_to_row) {
    __shared__ int before[64], total[64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int group = blockIdx.x;
    const int chunk = group * G + wave;
    int le[kIters];
    load_chunk(le, topk_ids, chunk, n_chunks, A, lo, lane);
    // this lane's expert: its assignments in the earlier chunks of this group
    int within = 0;
    if (lane < n_local) {
        int v[G];
#pragma unroll
        for (int q = 0; q < G; ++q)                          // (q < wave: chunk group*G + q exists whenever this wave's chunk does)
            v[q] = (q < wave && group * G + q < n_chunks) ? wave_cnt[(size_t)lane * n_chunks + group * G + q] : 0;
#pragma unroll
        for (int q = 0; q < G; ++q) within += v[q];
    }
    for (int e = wave; e < n_local; e += G) {
        int b = 0, t = 0;
        for (int q = lane; q < n_groups; q += 64) {
            const int v = group_cnt[(size_t)e * n_groups + q];
            t += v;
            if (q < group) b += v;
        }
        b = wave_sum(b);
        t = wave_sum(t);
        if (lane == 0) { before[e] = b; total[e] = t; }
    }
    __syncthreads();
    const int tot = lane < n_local ? total[lane] : 0;
    const int incl = wave_inclusive_scan(tot);
    if (group == 0 && wave == 0) {
        if (lane < n_local) expert_offsets[lane] = incl - tot;
        if (lane == n_local - 1) expert_offsets[n_local] = incl;
    }
    if (chunk >= n_chunks) return;
    int running = (lane < n_local) ? incl - tot + before[lane] + within : 0;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
#pragma unroll
    for (int i = 0; i < kIters; ++i) {
        const int a = chunk * kPermChunk + i * 64 + lane;
        int row = -1;
        for (int e = 0; e < n_local; ++e) {
            const unsigned long long m = __ballot(le[i] == e);
            const int base = __builtin_amdgcn_readlane(running, e);
            if (le[i] == e) row = base + __popcll(m & lt_mask);
            if (lane == e) running += __popcll(m);
        }
        if (a < A) {
            assign_to_row[a] = row;
            if (row >= 0) row_to_assign[row] = a;
        }
    }
}

// Phase 4: one wave per TOKEN, grid-strided: a token routed to several local experts
// is read (and, on the FP4 path, encoded) once and written to each of its rows.
// H/8 chunks of 16 B per row; FP4: quads of lanes share one 32-element block.
template <bool FP4, int CPL>   // CPL = 16-byte chunks per lane = H / 512 rounded up
__global__ void __launch_bounds__(256) perm_gather_kernel(const u32x4_t* __restrict__ x, const int32_t* __restrict__ assign_to_row,
                                                          int T, int k, int H, u32x4_t* __restrict__ x_perm,
                                                          uint32_t* __restrict__ x_q, uint8_t* __restrict__ x_s, int token_major) {
    // token_major: a token with a local expert is written once, at row index t (the consuming GEMM then
    // fetches rows through row_to_assign), instead of once per row it occupies.
    const int lane = threadIdx.x & 63;
    const int chunks = H >> 3;                             // 16-B chunks per row, multiple of 16
    // A block takes a contiguous range of tokens: the rows of one 32-row group of an expert come from
    // tokens close together, so their scale words (which share 128-byte lines in the tiled scale tensor)
    // are written through the same L2 and leave it as whole lines.
    // Blocks b, b+8, .. share an XCD: each XCD takes one contiguous eighth of the tokens, its blocks
    // contiguous pieces of it.
    // (BF16 rows are whole lines anyway; there the strided assignment of tokens to blocks measured faster.)
    const int per_xcd = (T + 7) >> 3, nb = max((int)gridDim.x >> 3, 1);
    const int x_lo = (int)(blockIdx.x & 7) * per_xcd, x_hi = min(T, x_lo + per_xcd);
    const int per_block = (per_xcd + nb - 1) / nb;
    const int t_lo = FP4 ? x_lo + (int)(blockIdx.x >> 3) * per_block + (int)(threadIdx.x >> 6)
                         : (int)(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6));
    const int t_end = FP4 ? min(x_hi, x_lo + ((int)(blockIdx.x >> 3) + 1) * per_block) : T;
    const int t_step = FP4 ? (int)(blockDim.x >> 6) : (int)(gridDim.x * (blockDim.x >> 6));
    for (int t = t_lo; t < t_end; t += t_step) {
        const int my_row = lane < k ? assign_to_row[(size_t)t * k + lane] : -1;
        if (__ballot(my_row >= 0) == 0ull) continue;       // no local expert for this token
        const u32x4_t* src = x + (size_t)t * chunks;
        u32x4_t v[CPL];
#pragma unroll
        for (int u = 0; u < CPL; ++u) {
            const int c = u * 64 + lane;
            v[u] = c < chunks ? src[c] : u32x4_t{0, 0, 0, 0};
        }
        uint32_t codes[CPL], byte[CPL], word[CPL];
        if (FP4) {
#pragma unroll
            for (int u = 0; u < CPL; ++u) {
                codes[u] = encode_block_quad(v[u], &byte[u]);
                word[u] = byte[u] | ((uint32_t)__shfl_down((int)byte[u], 4) << 8) | ((uint32_t)__shfl_down((int)byte[u], 8) << 16) |
                          ((uint32_t)__shfl_down((int)byte[u], 12) << 24);
            }
        }
        const int n_writes = token_major ? 1 : k;
        for (int j = 0; j < n_writes; ++j) {
            const int r = token_major ? t : __builtin_amdgcn_readlane(my_row, j);
            if (r < 0) continue;
#pragma unroll
            for (int u = 0; u < CPL; ++u) {
                const int c = u * 64 + lane;
                if (c < chunks) {
                    if (FP4) {
                        x_q[(size_t)r * chunks + c] = codes[u];
                        // the four scales of a 128-element K-step are one dword of the tiled tensor: lane 16m
                        // stores the dword packed from lanes 16m, 16m+4, 16m+8, 16m+12 (chunks is a multiple of 16)
                        if ((lane & 15) == 0)
                            *reinterpret_cast<uint32_t*>(x_s + scale_byte_offset(r, c >> 2, chunks >> 4)) = word[u];
                    } else {
                        x_perm[(size_t)r * chunks + c] = v[u];
                    }
                }
            }
        }
    }
}

template <bool FP4>
static void launch_gather(int blocks, hipStream_t s, const void* x, const int32_t* a2r, int T, int k, int H, void* x_perm,
                          uint8_t* x_q, uint8_t* x_s, int token_major = 0) {
    const int cpl = (H / 8 + 63) / 64;
#define REALB_GATHER(CPL)                                                                                              \
    hipLaunchKernelGGL((perm_gather_kernel<FP4, CPL>), dim3(blocks), dim3(256), 0, s, (const u32x4_t*)x, a2r, T, k, H, \
                       (u32x4_t*)x_perm, (uint32_t*)x_q, x_s, token_major)
    if (cpl <= 1) REALB_GATHER(1);
    else if (cpl <= 2) REALB_GATHER(2);
    else if (cpl <= 4) REALB_GATHER(4);
    else if (cpl <= 8) REALB_GATHER(8);
    else REALB_GATHER(16);
#undef REALB_GATHER
}

}  // namespace realb

using namespace realb;

namespace realb {

// The two halves of realb_permute.  The index half (count / rank) does not depend on the
// precision, so the layer can run it while the host is still taking the precision decision.
int permute_indices(Ctx* c, const int32_t* topk_ids, int T, int rank, long long max_rows, int32_t* expert_offsets,
                    int32_t* row_to_assign, int32_t* assign_to_row, hipStream_t s) {
    REALB_REQUIRE(c && expert_offsets, REALB_EINVAL, "NULL argument");
    REALB_REQUIRE(T >= 0 && T <= c->cfg.T_max, REALB_ECAP, "T=%d outside [0, T_max=%d]", T, c->cfg.T_max);
    REALB_REQUIRE(rank >= 0 && rank < c->cfg.D, REALB_EINVAL, "rank=%d outside [0,%d)", rank, c->cfg.D);
    const int k = c->cfg.k, n_local = c->n_local;
    const long long A = (long long)T * k;
    const long long worst = (long long)T * (k < n_local ? k : n_local);
    REALB_REQUIRE(max_rows >= worst, REALB_EINVAL, "max_rows=%lld is below the worst case %lld", max_rows, worst);
    REALB_REQUIRE(T == 0 || (topk_ids && row_to_assign && assign_to_row), REALB_EINVAL, "NULL argument");
    const int n_chunks = ceil_div(A, kPermChunk);
    const int G = perm_group(n_chunks);
    const int n_groups = ceil_div(n_chunks, G);
    const int lo = rank * n_local;
    auto launch = [&](auto g) {
        constexpr int GG = decltype(g)::value;
        if (n_groups > 0)
            hipLaunchKernelGGL(perm_count_kernel<GG>, dim3(n_groups), dim3(64 * GG), 0, s, topk_ids, (int)A, lo, n_local, n_chunks,
                               n_groups, c->wave_cnt, c->group_cnt);
        hipLaunchKernelGGL(perm_rank_kernel<GG>, dim3(n_groups > 0 ? n_groups : 1), dim3(64 * GG), 0, s, topk_ids, (int)A, lo, n_local,
                           n_chunks, n_groups, c->wave_cnt, c->group_cnt, expert_offsets, row_to_assign, assign_to_row);
    };
    if (G == kGroupLong) launch(std::integral_constant<int, kGroupLong>{});
    else launch(std::integral_constant<int, kGroupShort>{});
    REALB_HIP(hipGetLastError());
    return REALB_OK;
}

// Routing and the permutation's index kernels as the layer call issues them: top-k + histograms, then
// [histogram reduce | chunk counts] in one launch -- whose reduce block writes the statistics, tagged with stats_seq,
// to pinned memory -- then the ranking kernel, which runs while the host takes the decision.
int route_and_index(Ctx* c, const float* logits, const uint8_t* is_vision, int T, int rank, long long max_rows, int32_t* topk_ids,
                    float* topk_w, int32_t* expert_cnt, int32_t* expert_vis, int32_t* rank_load, int32_t* rank_vis,
                    int32_t* expert_offsets, int32_t* row_to_assign, int32_t* assign_to_row, int stats_seq, hipStream_t s) {
    REALB_REQUIRE(c && expert_cnt && expert_vis && rank_load && rank_vis && expert_offsets, REALB_EINVAL, "NULL argument");
    REALB_REQUIRE(T >= 0 && T <= c->cfg.T_max, REALB_ECAP, "T=%d outside [0, T_max=%d]", T, c->cfg.T_max);
    REALB_REQUIRE(rank >= 0 && rank < c->cfg.D, REALB_EINVAL, "rank=%d outside [0,%d)", rank, c->cfg.D);
    const int E = c->cfg.E, D = c->cfg.D, k = c->cfg.k, n_local = c->n_local;
    const long long A = (long long)T * k;
    const long long worst = (long long)T * (k < n_local ? k : n_local);
    REALB_REQUIRE(max_rows >= worst, REALB_EINVAL, "max_rows=%lld is below the worst case %lld", max_rows, worst);
    REALB_REQUIRE(T == 0 || (topk_ids && row_to_assign && assign_to_row), REALB_EINVAL, "NULL argument");
    const int n_part = route_topk_only(c, logits, is_vision, T, topk_ids, topk_w, s);
    if (n_part < 0) return n_part;
    const int n_chunks = ceil_div(A, kPermChunk);
    const int G = perm_group(n_chunks);
    const int n_groups = ceil_div(n_chunks, G);
    const int lo = rank * n_local;
    auto launch = [&](auto g) {
        constexpr int GG = decltype(g)::value;
        hipLaunchKernelGGL(reduce_and_count_kernel<GG>, dim3(D + n_groups), dim3(64 * GG), 2 * (size_t)(E / D) * sizeof(int32_t), s,
                           c->hist_part, n_part, E, D, expert_cnt, expert_vis, rank_load, rank_vis, c->stats_words, stats_seq, topk_ids,
                           (int)A, lo, n_local, n_chunks, n_groups, c->wave_cnt, c->group_cnt);
        hipLaunchKernelGGL(perm_rank_kernel<GG>, dim3(n_groups > 0 ? n_groups : 1), dim3(64 * GG), 0, s, topk_ids, (int)A, lo, n_local,
                           n_chunks, n_groups, c->wave_cnt, c->group_cnt, expert_offsets, row_to_assign, assign_to_row);
    };
    if (G == kGroupLong) launch(std::integral_constant<int, kGroupLong>{});
    else launch(std::integral_constant<int, kGroupShort>{});
    REALB_HIP(hipGetLastError());
    return REALB_OK;
}

int permute_gather(Ctx* c, const void* x, const int32_t* assign_to_row, int T, int prec, void* x_perm, uint8_t* x_q,
                   uint8_t* x_s, hipStream_t s, int token_major) {
    REALB_REQUIRE(c != nullptr, REALB_EINVAL, "NULL argument");
    REALB_REQUIRE(prec == REALB_BF16 || prec == REALB_FP4, REALB_EINVAL, "bad precision %d", prec);
    REALB_REQUIRE(T >= 0 && T <= c->cfg.T_max, REALB_ECAP, "T=%d outside [0, T_max=%d]", T, c->cfg.T_max);
    if (T == 0) return REALB_OK;
    REALB_REQUIRE(x && assign_to_row, REALB_EINVAL, "NULL argument");
    REALB_REQUIRE(prec == REALB_BF16 ? x_perm != nullptr : (x_q && x_s), REALB_EINVAL, "NULL row buffer");
    const int k = c->cfg.k, H = c->cfg.H;
    const int blocks = 8 * (T < 32 ? 1 : (T / 32 < 512 ? T / 32 : 512));      // a multiple of 8 (XCDs), 4 waves each
    if (prec == REALB_FP4) launch_gather<true>(blocks, s, x, assign_to_row, T, k, H, nullptr, x_q, x_s, token_major);
    else launch_gather<false>(blocks, s, x, assign_to_row, T, k, H, x_perm, nullptr, nullptr);
    REALB_HIP(hipGetLastError());
    return REALB_OK;
}

}  // namespace realb

extern "C" int realb_permute(realb_ctx* ctx, const void* x, const int32_t* topk_ids, int T, int rank, int prec,
                             long long max_rows, int32_t* expert_offsets, int32_t* row_to_assign, int32_t* assign_to_row,
                             void* x_perm, uint8_t* x_q, uint8_t* x_s, void* stream) {
    REALB_REQUIRE(ctx != nullptr, REALB_EINVAL, "NULL argument");
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    REALB_REQUIRE(prec == REALB_BF16 || prec == REALB_FP4, REALB_EINVAL, "bad precision %d", prec);
    REALB_REQUIRE(T <= 0 || (x && (prec == REALB_BF16 ? x_perm != nullptr : (x_q && x_s))), REALB_EINVAL, "NULL row buffer");
    int rc = permute_indices(c, topk_ids, T, rank, max_rows, expert_offsets, row_to_assign, assign_to_row, as_stream(stream));
    if (rc != REALB_OK) return rc;
    return permute_gather(c, x, assign_to_row, T, prec, x_perm, x_q, x_s, as_stream(stream), 0);
}
