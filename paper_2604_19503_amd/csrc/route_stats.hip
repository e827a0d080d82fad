// Stage 1, routing and profiling (paper Sec. "System Overview"; runtime state
// Load_d, N_vd of Sec. "Real-time Modality-aware LB Scheduling"): top-k gating
// with gates renormalised over the selected experts, per-expert and per-rank
// assignment counts, split by modality.
#include "common.h"
#include <math.h>

namespace realb {

// Clears the two histograms (and is the only writer of them before the main kernel).
__global__ void zero_hist_kernel(int32_t* a, int32_t* b, int n) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) { a[i] = 0; b[i] = 0; }
}

// DPP lane exchange inside a row of 16 lanes (no LDS traffic).
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, 0xF, 0xF, false));
}
// After this every lane of a row holds the row's maximum.
__device__ __forceinline__ float row_max(float v) {
    v = fmaxf(v, dpp_f<0xB1>(v));      // quad_perm [1,0,3,2]
    v = fmaxf(v, dpp_f<0x4E>(v));      // quad_perm [2,3,0,1]
    v = fmaxf(v, dpp_f<0x141>(v));     // row_half_mirror
    v = fmaxf(v, dpp_f<0x140>(v));     // row_mirror
    return v;
}
__device__ __forceinline__ float row_sum(float v) {
    v += dpp_f<0xB1>(v);
    v += dpp_f<0x4E>(v);
    v += dpp_f<0x141>(v);
    v += dpp_f<0x140>(v);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
    v = row_max(v);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

// One wave per token.  Lane l holds the EPL consecutive experts l*EPL .. l*EPL+EPL-1,
// so that among equal logits the lowest (lane, slot) is the lowest expert index.
// k rounds of: per-lane best -> wave maximum -> lowest lane holding it wins.
// The block's histograms live in LDS and are flushed with integer atomics.
template <int EPL>
__global__ void __launch_bounds__(256) topk_hist_kernel(const float* __restrict__ logits, const uint8_t* __restrict__ is_vision,
                                                        int T, int E, int k, int32_t* __restrict__ topk_ids,
                                                        float* __restrict__ topk_w, int32_t* __restrict__ expert_cnt,
                                                        int32_t* __restrict__ expert_vis) {
    extern __shared__ int32_t hist[];                 // [2*E]: counts, vision counts
    for (int i = threadIdx.x; i < 2 * E; i += blockDim.x) hist[i] = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int waves_per_block = blockDim.x >> 6;
    const float NEG = -INFINITY;
    for (int t = blockIdx.x * waves_per_block + wave; t < T; t += gridDim.x * waves_per_block) {
        float v[EPL];
        const float* row = logits + (size_t)t * E + lane * EPL;
#pragma unroll
        for (int j = 0; j < EPL; ++j) v[j] = (lane * EPL + j < E) ? row[j] : NEG;
        const int vision = is_vision[t];
        float my_val = 0.f;                           // lane j keeps the j-th selected logit
        int my_id = 0;                                //        and its expert index
        for (int sel = 0; sel < k; ++sel) {
            float best = v[0];
            int slot = 0;
#pragma unroll
            for (int j = 1; j < EPL; ++j)
                if (v[j] > best) { best = v[j]; slot = j; }
            const float wmax = wave_max(best);
            const unsigned long long cand = __ballot(best == wmax);
            const int winner = __ffsll((long long)cand) - 1;
            const int win_slot = __builtin_amdgcn_readlane(slot, winner);
            if (lane == winner) {
#pragma unroll
                for (int j = 0; j < EPL; ++j)
                    if (j == win_slot) v[j] = NEG;
            }
            if (lane == sel) { my_val = wmax; my_id = winner * EPL + win_slot; }
        }
        // gates: softmax over the k selected logits (lane 0 holds the maximum); k <= 16 = one DPP row
        const float top = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_val), 0));
        const float e = lane < k ? expf(my_val - top) : 0.f;
        const float sum = row_sum(e);
        if (lane < k) {
            topk_ids[(size_t)t * k + lane] = my_id;
            topk_w[(size_t)t * k + lane] = e / sum;
            atomicAdd(&hist[my_id], 1);
            if (vision) atomicAdd(&hist[E + my_id], 1);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < E; i += blockDim.x) {
        if (hist[i]) atomicAdd(&expert_cnt[i], hist[i]);
        if (hist[E + i]) atomicAdd(&expert_vis[i], hist[E + i]);
    }
}

// Per-rank sums of the finished histograms (a separate launch: a kernel boundary is the
// cheap way to make the atomics of all XCDs visible; a device-scope fence per block is not).
__global__ void rank_sums_kernel(const int32_t* __restrict__ expert_cnt, const int32_t* __restrict__ expert_vis,
                                 int D, int n_local, int32_t* __restrict__ rank_load, int32_t* __restrict__ rank_vis) {
    const int d = threadIdx.x;
    if (d >= D) return;
    int load = 0, vis = 0;
    for (int e = 0; e < n_local; ++e) {
        load += expert_cnt[d * n_local + e];
        vis += expert_vis[d * n_local + e];
    }
    rank_load[d] = load;
    rank_vis[d] = vis;
}

}  // namespace realb

using namespace realb;

extern "C" int realb_route_stats(realb_ctx* ctx, const float* logits, const uint8_t* is_vision, int T, int32_t* topk_ids,
                                 float* topk_w, int32_t* expert_cnt, int32_t* expert_vis, int32_t* rank_load,
                                 int32_t* rank_vis, void* stream) {
    REALB_REQUIRE(ctx && expert_cnt && expert_vis && rank_load && rank_vis, REALB_EINVAL, "NULL argument");
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    REALB_REQUIRE(T >= 0 && T <= c->cfg.T_max, REALB_ECAP, "T=%d outside [0, T_max=%d]", T, c->cfg.T_max);
    REALB_REQUIRE(T == 0 || (logits && is_vision && topk_ids && topk_w), REALB_EINVAL, "NULL argument");
    hipStream_t s = as_stream(stream);
    const int E = c->cfg.E, k = c->cfg.k, D = c->cfg.D;
    hipLaunchKernelGGL(zero_hist_kernel, dim3(1), dim3(256), 0, s, expert_cnt, expert_vis, E);
    if (T > 0) {
        const int blocks = min(ceil_div(T, 4), 256 * 8);
        const size_t lds = 2 * (size_t)E * sizeof(int32_t);
        const int epl = ceil_div(E, 64);
#define REALB_TOPK(EPL)                                                                                        \
    hipLaunchKernelGGL(topk_hist_kernel<EPL>, dim3(blocks), dim3(256), lds, s, logits, is_vision, T, E, k, \
                       topk_ids, topk_w, expert_cnt, expert_vis)
        if (epl == 1) REALB_TOPK(1);
        else if (epl == 2) REALB_TOPK(2);
        else if (epl <= 4) REALB_TOPK(4);
        else REALB_TOPK(8);
#undef REALB_TOPK
    }
    hipLaunchKernelGGL(rank_sums_kernel, dim3(1), dim3(64), 0, s, expert_cnt, expert_vis, D, c->n_local, rank_load, rank_vis);
    REALB_HIP(hipGetLastError());
    return REALB_OK;
}
