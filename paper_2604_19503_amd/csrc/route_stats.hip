// Stage 1, routing and profiling (paper Sec. "System Overview"; runtime state
// Load_d, N_vd of Sec. "Real-time Modality-aware LB Scheduling"): top-k gating
// with gates renormalised over the selected experts, per-expert and per-rank
// assignment counts, split by modality.
#include "common.h"
#include <math.h>

namespace realb {

__global__ void zero_i32_kernel(int32_t* p, int n) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m));
    return v;
}

// One wave per token.  Lane l holds the EPL consecutive experts l*EPL .. l*EPL+EPL-1,
// so that among equal logits the lowest (lane, slot) is the lowest expert index.
// k rounds of: per-lane best -> wave maximum -> lowest lane holding it wins.
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
            const int win_slot = __shfl(slot, winner);
            if (lane == winner) {
#pragma unroll
                for (int j = 0; j < EPL; ++j)
                    if (j == win_slot) v[j] = NEG;
            }
            if (lane == sel) { my_val = wmax; my_id = winner * EPL + win_slot; }
        }
        // gates: softmax over the k selected logits (lane 0 holds the maximum)
        const float top = __shfl(my_val, 0);
        float e = lane < k ? expf(my_val - top) : 0.f;
        float sum = e;
#pragma unroll
        for (int m = 8; m >= 1; m >>= 1) sum += __shfl_xor(sum, m);   // k <= 16
        if (lane < k) {
            topk_ids[(size_t)t * k + lane] = my_id;
            topk_w[(size_t)t * k + lane] = e / sum;
            atomicAdd(&hist[my_id], 1);
            if (is_vision[t]) atomicAdd(&hist[E + my_id], 1);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < E; i += blockDim.x) {
        if (hist[i]) atomicAdd(&expert_cnt[i], hist[i]);
        if (hist[E + i]) atomicAdd(&expert_vis[i], hist[E + i]);
    }
}

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
    hipLaunchKernelGGL(zero_i32_kernel, dim3(1), dim3(256), 0, s, expert_cnt, E);
    hipLaunchKernelGGL(zero_i32_kernel, dim3(1), dim3(256), 0, s, expert_vis, E);
    if (T > 0) {
        const int blocks = min(ceil_div(T, 4), 256 * 8);
        const size_t lds = 2 * (size_t)E * sizeof(int32_t);
        const int epl = ceil_div(E, 64);
#define REALB_TOPK(EPL)                                                                                     \
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
