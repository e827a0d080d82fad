// Token permutation / dispatch packing for one rank: a deterministic, stable
// counting sort of the rank's (token, expert) assignments by local expert,
// then a row gather that either copies BF16 rows or encodes them to MXFP4.
// Stands in for the all-to-all dispatch of the paper's pipeline (Sec.
// "Overhead-Aware Pipeline Orchestration"); the weight encoder overlaps it.
#include "common.h"
#include "mxfp4_device.h"

namespace realb {

// Phase 1: each wave counts, per local expert, the assignments of its chunk of
// kPermChunk consecutive flat indices a = t*k + j.  Lane e holds expert e's count.
__global__ void __launch_bounds__(64) perm_count_kernel(const int32_t* __restrict__ topk_ids, int A, int lo, int n_local,
                                                        int32_t* __restrict__ wave_cnt) {
    const int lane = threadIdx.x;
    const int chunk = blockIdx.x;
    const int begin = chunk * kPermChunk;
    const int end = min(begin + kPermChunk, A);
    int cnt = 0;
    for (int a0 = begin; a0 < end; a0 += 64) {
        const int a = a0 + lane;
        const int le = (a < end) ? topk_ids[a] - lo : -1;
        for (int e = 0; e < n_local; ++e) {
            const unsigned long long m = __ballot(le == e);
            if (lane == e) cnt += __popcll(m);
        }
    }
    if (lane < n_local) wave_cnt[chunk * n_local + lane] = cnt;
}

__device__ __forceinline__ int wave_inclusive_scan(int v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int o = __shfl_up(v, d);
        if (lane >= d) v += o;
    }
    return v;
}

// Phase 2 (one block): per expert, exclusive scan of the chunk counts in chunk
// order (in place: counts become the chunk's first rank within the expert), then
// the exclusive scan over experts gives expert_offsets.
__global__ void __launch_bounds__(1024) perm_scan_kernel(int32_t* __restrict__ wave_cnt, int n_chunks, int n_local,
                                                         int32_t* __restrict__ expert_offsets) {
    __shared__ int totals[64];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int n_waves = blockDim.x >> 6;
    for (int e = wave; e < n_local; e += n_waves) {
        int carry = 0;
        for (int c0 = 0; c0 < n_chunks; c0 += 64) {
            const int c = c0 + lane;
            const int v = (c < n_chunks) ? wave_cnt[c * n_local + e] : 0;
            const int incl = wave_inclusive_scan(v, lane);
            if (c < n_chunks) wave_cnt[c * n_local + e] = carry + incl - v;
            carry += __shfl(incl, 63);
        }
        if (lane == 0) totals[e] = carry;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int e = 0; e < n_local; ++e) { expert_offsets[e] = run; run += totals[e]; }
        expert_offsets[n_local] = run;
    }
}

// Phase 3: each wave walks its chunk again and gives every local assignment its
// row: expert_offsets[e] + (rank of the chunk's first) + (rank inside the chunk).
__global__ void __launch_bounds__(64) perm_rank_kernel(const int32_t* __restrict__ topk_ids, int A, int lo, int n_local,
                                                       const int32_t* __restrict__ wave_cnt,
                                                       const int32_t* __restrict__ expert_offsets,
                                                       int32_t* __restrict__ row_to_assign, int32_t* __restrict__ assign_to_row) {
    const int lane = threadIdx.x;
    const int chunk = blockIdx.x;
    const int begin = chunk * kPermChunk;
    const int end = min(begin + kPermChunk, A);
    int running = (lane < n_local) ? expert_offsets[lane] + wave_cnt[chunk * n_local + lane] : 0;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    for (int a0 = begin; a0 < end; a0 += 64) {
        const int a = a0 + lane;
        const int le = (a < end) ? topk_ids[a] - lo : -1;
        int row = -1;
        for (int e = 0; e < n_local; ++e) {
            const unsigned long long m = __ballot(le == e);
            const int base = __shfl(running, e);
            if (le == e) row = base + __popcll(m & lt_mask);
            if (lane == e) running += __popcll(m);
        }
        if (a < end) {
            assign_to_row[a] = row;
            if (row >= 0) row_to_assign[row] = a;
        }
    }
}

// Phase 4: one wave per row, grid-strided; R is read from expert_offsets[n_local].
// H/8 chunks of 16 B per row; FP4: quads of lanes share one 32-element block.
template <bool FP4>
__global__ void __launch_bounds__(256) perm_gather_kernel(const u32x4_t* __restrict__ x, const int32_t* __restrict__ row_to_assign,
                                                          const int32_t* __restrict__ expert_offsets, int n_local, int k,
                                                          int H, u32x4_t* __restrict__ x_perm, uint32_t* __restrict__ x_q,
                                                          uint8_t* __restrict__ x_s) {
    const int R = expert_offsets[n_local];
    const int lane = threadIdx.x & 63;
    const int chunks = H >> 3;                             // 16-B chunks per row, multiple of 16
    const int wave_global = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int n_waves = gridDim.x * (blockDim.x >> 6);
    for (int r = wave_global; r < R; r += n_waves) {
        const int t = row_to_assign[r] / k;
        const u32x4_t* src = x + (size_t)t * chunks;
        for (int c0 = 0; c0 < chunks; c0 += 256) {
            u32x4_t v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + u * 64 + lane;
                v[u] = c < chunks ? src[c] : u32x4_t{0, 0, 0, 0};
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + u * 64 + lane;
                if (FP4) {
                    uint32_t byte;
                    const uint32_t codes = encode_block_quad(v[u], &byte);
                    if (c < chunks) {
                        x_q[(size_t)r * chunks + c] = codes;
                        if ((lane & 3) == 0) x_s[(size_t)r * (chunks >> 2) + (c >> 2)] = (uint8_t)byte;
                    }
                } else if (c < chunks) {
                    x_perm[(size_t)r * chunks + c] = v[u];
                }
            }
        }
    }
}

}  // namespace realb

using namespace realb;

extern "C" int realb_permute(realb_ctx* ctx, const void* x, const int32_t* topk_ids, int T, int rank, int prec,
                             long long max_rows, int32_t* expert_offsets, int32_t* row_to_assign, int32_t* assign_to_row,
                             void* x_perm, uint8_t* x_q, uint8_t* x_s, void* stream) {
    REALB_REQUIRE(ctx && expert_offsets, REALB_EINVAL, "NULL argument");
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    REALB_REQUIRE(T >= 0 && T <= c->cfg.T_max, REALB_ECAP, "T=%d outside [0, T_max=%d]", T, c->cfg.T_max);
    REALB_REQUIRE(rank >= 0 && rank < c->cfg.D, REALB_EINVAL, "rank=%d outside [0,%d)", rank, c->cfg.D);
    REALB_REQUIRE(prec == REALB_BF16 || prec == REALB_FP4, REALB_EINVAL, "bad precision %d", prec);
    const int k = c->cfg.k, n_local = c->n_local, H = c->cfg.H;
    const long long A = (long long)T * k;
    const long long worst = (long long)T * (k < n_local ? k : n_local);
    REALB_REQUIRE(max_rows >= worst, REALB_EINVAL, "max_rows=%lld is below the worst case %lld", max_rows, worst);
    REALB_REQUIRE(T == 0 || (x && topk_ids && row_to_assign && assign_to_row), REALB_EINVAL, "NULL argument");
    REALB_REQUIRE(T == 0 || (prec == REALB_BF16 ? x_perm != nullptr : (x_q && x_s)), REALB_EINVAL, "NULL row buffer");
    hipStream_t s = as_stream(stream);
    const int n_chunks = ceil_div(A, kPermChunk);
    const int lo = rank * n_local;
    if (n_chunks > 0)
        hipLaunchKernelGGL(perm_count_kernel, dim3(n_chunks), dim3(64), 0, s, topk_ids, (int)A, lo, n_local, c->wave_cnt);
    hipLaunchKernelGGL(perm_scan_kernel, dim3(1), dim3(1024), 0, s, c->wave_cnt, n_chunks, n_local, expert_offsets);
    if (n_chunks > 0) {
        hipLaunchKernelGGL(perm_rank_kernel, dim3(n_chunks), dim3(64), 0, s, topk_ids, (int)A, lo, n_local, c->wave_cnt,
                           expert_offsets, row_to_assign, assign_to_row);
        const int blocks = (int)(worst < 4 ? 1 : (worst / 4 < 256 * 16 ? worst / 4 : 256 * 16));
        if (prec == REALB_FP4)
            hipLaunchKernelGGL(perm_gather_kernel<true>, dim3(blocks), dim3(256), 0, s, (const u32x4_t*)x, row_to_assign,
                               expert_offsets, n_local, k, H, (u32x4_t*)nullptr, (uint32_t*)x_q, x_s);
        else
            hipLaunchKernelGGL(perm_gather_kernel<false>, dim3(blocks), dim3(256), 0, s, (const u32x4_t*)x, row_to_assign,
                               expert_offsets, n_local, k, H, (u32x4_t*)x_perm, (uint32_t*)nullptr, (uint8_t*)nullptr);
    }
    REALB_HIP(hipGetLastError());
    return REALB_OK;
}
