// Stage 1, routing and profiling (paper Sec. "System Overview"; runtime state
// Load_d, N_vd of Sec. "Real-time Modality-aware LB Scheduling"): top-k gating
// with gates renormalised over the selected experts, per-expert and per-rank
// assignment counts, split by modality.
#include "common.h"
#include "hist_reduce.h"
#include <math.h>
#include <mutex>

namespace realb {

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
// The block's histograms live in LDS; each block writes its partial histogram to the workspace
// (no global atomics, no pre-zeroing), and a small kernel (one block per EP rank) adds the partials up.
template <int EPL>
__global__ void __launch_bounds__(1024, 2) topk_hist_kernel(const float* __restrict__ logits, const uint8_t* __restrict__ is_vision,
                                                        int T, int E, int k, int32_t* __restrict__ topk_ids,
                                                        float* __restrict__ topk_w, int32_t* __restrict__ hist_part) {
    extern __shared__ int32_t hist[];                 // [2*E]: counts, vision counts
    for (int i = threadIdx.x; i < 2 * E; i += blockDim.x) hist[i] = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int waves_per_block = blockDim.x >> 6;
    const float NEG = -INFINITY;
    // The wave's next token is fetched while the current one is being ranked (one load latency per
    // wave instead of one per token).
    const int stride = gridDim.x * waves_per_block;
    int t = blockIdx.x * waves_per_block + wave;
    float nx[EPL];
    int nx_vision = 0;
    auto fetch = [&](int tok) __attribute__((always_inline)) {
        if (tok < T) {
            const float* row = logits + (size_t)tok * E + lane * EPL;
#pragma unroll
            for (int j = 0; j < EPL; ++j) nx[j] = (lane * EPL + j < E) ? row[j] : NEG;
            nx_vision = is_vision[tok];
        }
    };
    fetch(t);
    for (; t < T; t += stride) {
        float v[EPL];
#pragma unroll
        for (int j = 0; j < EPL; ++j) v[j] = nx[j];
        const int vision = nx_vision;
        fetch(t + stride);
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
    for (int i = threadIdx.x; i < 2 * E; i += blockDim.x) hist_part[(size_t)blockIdx.x * 2 * E + i] = hist[i];
}

__device__ __forceinline__ int row_min_i(int v) {
    v = min(v, __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false));
    v = min(v, __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false));
    v = min(v, __builtin_amdgcn_update_dpp(v, v, 0x141, 0xF, 0xF, false));
    v = min(v, __builtin_amdgcn_update_dpp(v, v, 0x140, 0xF, 0xF, false));
    return v;
}

// Four tokens per wave (E <= 128, a multiple of 16): a row of 16 lanes owns one token, lane j of the
// row holds the EPL = E/16 consecutive experts j*EPL .. j*EPL+EPL-1.  A selection round is the lane's
// best, the row maximum, and the row minimum of the expert index among the lanes that hold that
// maximum (lowest index wins ties) -- DPP only, no scalar round trips, the four rows in lock step.
template <int EPL>
__global__ void __launch_bounds__(1024, 2) topk_hist_rows_kernel(const float* __restrict__ logits, const uint8_t* __restrict__ is_vision,
                                                                 int T, int E, int k, int32_t* __restrict__ topk_ids,
                                                                 float* __restrict__ topk_w, int32_t* __restrict__ hist_part) {
    extern __shared__ int32_t hist[];                 // [2*E]: counts, vision counts
    for (int i = threadIdx.x; i < 2 * E; i += blockDim.x) hist[i] = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int j = lane & 15, r = lane >> 4;
    const int wave = threadIdx.x >> 6;
    const int waves_per_block = blockDim.x >> 6;
    const float NEG = -INFINITY;
    const int stride = gridDim.x * waves_per_block * 4;
    int t = (blockIdx.x * waves_per_block + wave) * 4 + r;
    float nx[EPL];
    int nx_vision = 0;
    auto fetch = [&](int tok) __attribute__((always_inline)) {
        if (tok < T) {
            const float* row = logits + (size_t)tok * E + j * EPL;
#pragma unroll
            for (int q = 0; q < EPL; ++q) nx[q] = row[q];
            nx_vision = is_vision[tok];
        }
    };
    fetch(t);
    for (int t0 = t - r; t0 < T; t0 += stride, t += stride) {      // uniform trip count: rows past T idle but take part in the DPP steps
        float v[EPL];
#pragma unroll
        for (int q = 0; q < EPL; ++q) v[q] = nx[q];
        const int vision = nx_vision;
        const bool live = t < T;
        fetch(t + stride);
        float my_val = NEG;                           // lane j keeps the j-th selected logit of its row's token
        int my_id = 0;
        for (int sel = 0; sel < k; ++sel) {
            float best = v[0];
            int slot = 0;
#pragma unroll
            for (int q = 1; q < EPL; ++q)
                if (v[q] > best) { best = v[q]; slot = q; }
            const float rmax = row_max(best);
            const int widx = row_min_i(best == rmax ? j * EPL + slot : 0x7FFFFFFF);
#pragma unroll
            for (int q = 0; q < EPL; ++q)
                if (widx == j * EPL + q) v[q] = NEG;
            if (j == sel) { my_val = rmax; my_id = widx; }
        }
        // gates: softmax over the k selected logits; the first selected one is the row's largest
        const float top = row_max(j < k ? my_val : NEG);
        const float e = j < k ? expf(my_val - top) : 0.f;
        const float sum = row_sum(e);
        if (live && j < k) {
            topk_ids[(size_t)t * k + j] = my_id;
            topk_w[(size_t)t * k + j] = e / sum;
            atomicAdd(&hist[my_id], 1);
            if (vision) atomicAdd(&hist[E + my_id], 1);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 2 * E; i += blockDim.x) hist_part[(size_t)blockIdx.x * 2 * E + i] = hist[i];
}

__global__ void __launch_bounds__(1024) hist_reduce_kernel(const int32_t* __restrict__ hist_part, int n_part, int E, int D,
                                                           int32_t* __restrict__ expert_cnt, int32_t* __restrict__ expert_vis,
                                                           int32_t* __restrict__ rank_load, int32_t* __restrict__ rank_vis) {
    extern __shared__ int32_t tot[];                  // [2*E]
    hist_reduce_body(tot, hist_part, n_part, E, D, blockIdx.x, expert_cnt, expert_vis, rank_load, rank_vis, nullptr, 0);
}

// Launches the top-k + histogram kernel; returns the number of blocks (= partial histograms written).
// hist_part must hold max_blocks * 2E counters.
static int launch_topk(int num_cus, int max_blocks, int32_t* hist_part, const float* logits, const uint8_t* is_vision, int T,
                       int E, int k, int32_t* topk_ids, float* topk_w, hipStream_t s) {
    int blocks = 0;
    if (T > 0) {
        const size_t lds = 2 * (size_t)E * sizeof(int32_t);
        if (E <= 128 && E % 16 == 0) {                          // four tokens per wave
            blocks = min(min(ceil_div(T, 64), 2 * num_cus), max_blocks);      // 16 waves x 4 tokens in flight per block, two blocks per CU
#define REALB_TOPK_ROWS(EPL)                                                                                      \
    hipLaunchKernelGGL(topk_hist_rows_kernel<EPL>, dim3(blocks), dim3(1024), lds, s, logits, is_vision, T, E, k, \
                       topk_ids, topk_w, hist_part)
            switch (E / 16) {
                case 1: REALB_TOPK_ROWS(1); break;
                case 2: REALB_TOPK_ROWS(2); break;
                case 3: REALB_TOPK_ROWS(3); break;
                case 4: REALB_TOPK_ROWS(4); break;
                case 5: REALB_TOPK_ROWS(5); break;
                case 6: REALB_TOPK_ROWS(6); break;
                case 7: REALB_TOPK_ROWS(7); break;
                default: REALB_TOPK_ROWS(8); break;
            }
#undef REALB_TOPK_ROWS
        } else {
            blocks = min(min(ceil_div(T, 16), 2 * num_cus), max_blocks);      // 16 waves (tokens in flight) per block, two blocks per CU
            const int epl = ceil_div(E, 64);
#define REALB_TOPK(EPL)                                                                                      \
    hipLaunchKernelGGL(topk_hist_kernel<EPL>, dim3(blocks), dim3(1024), lds, s, logits, is_vision, T, E, k, \
                       topk_ids, topk_w, hist_part)
            if (epl == 1) REALB_TOPK(1);
            else if (epl == 2) REALB_TOPK(2);
            else if (epl <= 4) REALB_TOPK(4);
            else REALB_TOPK(8);
#undef REALB_TOPK
        }
    }
    return blocks;
}

// The top-k + histogram kernel and the reduce.
static int launch_route_stats(int num_cus, int max_blocks, int32_t* hist_part, const float* logits,
                              const uint8_t* is_vision, int T, int E, int k, int D, int32_t* topk_ids, float* topk_w,
                              int32_t* expert_cnt, int32_t* expert_vis, int32_t* rank_load, int32_t* rank_vis, hipStream_t s) {
    const int blocks = launch_topk(num_cus, max_blocks, hist_part, logits, is_vision, T, E, k, topk_ids, topk_w, s);
    hipLaunchKernelGGL(hist_reduce_kernel, dim3(D), dim3(1024), 2 * (size_t)(E / D) * sizeof(int32_t), s, hist_part, blocks, E, D,
                       expert_cnt, expert_vis, rank_load, rank_vis);
    REALB_HIP(hipGetLastError());
    return REALB_OK;
}

// Routing for the layer call: only the top-k + histogram kernel; the reduce is fused with the permutation's count kernel
// (route_and_index in permute.hip).  Returns the number of partial histograms, or a negative error code.
int route_topk_only(Ctx* c, const float* logits, const uint8_t* is_vision, int T, int32_t* topk_ids, float* topk_w, hipStream_t s) {
    REALB_REQUIRE(T >= 0 && T <= c->cfg.T_max, REALB_ECAP, "T=%d outside [0, T_max=%d]", T, c->cfg.T_max);
    REALB_REQUIRE(T == 0 || (logits && is_vision && topk_ids && topk_w), REALB_EINVAL, "NULL argument");
    const int blocks = launch_topk(c->num_cus, kRouteBlocksMax, c->hist_part, logits, is_vision, T, c->cfg.E, c->cfg.k, topk_ids, topk_w, s);
    REALB_HIP(hipGetLastError());
    return blocks;
}

// ---- the allocation-free variant's scratch: the per-block partial histograms, in a file-scope device array.
// Every GPU the library runs on holds its own copy at its own address until the process ends; the address is
// looked up once per device (with that device current) and kept, and host code only ever uses that pointer.
constexpr int kStaticBlocksMax = kRouteBlocksMax;
constexpr int kStaticEMax = 512;
constexpr size_t kStaticCounters = (size_t)kStaticBlocksMax * 2 * kStaticEMax;      // 2 MiB of int32
static __device__ __align__(256) int32_t scratch[kStaticCounters];

constexpr int kMaxDevices = 64;
struct StaticSlot { int32_t* ptr; int num_cus; };
static StaticSlot g_static[kMaxDevices];                  // zero-initialised; filled once per device under g_static_mu
static std::mutex g_static_mu;

// The current device's scratch pointer and CU count (looked up on the first call on that device).
int static_scratch_lookup(int32_t** ptr, int* num_cus) {
    int dev = 0;
    REALB_HIP(hipGetDevice(&dev));
    REALB_REQUIRE(dev >= 0 && dev < kMaxDevices, REALB_ECAP, "device index %d exceeds %d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static[dev].ptr) {
        int32_t* p = nullptr;
        int cus = 0;
        REALB_HIP(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
        REALB_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        REALB_REQUIRE(p != nullptr && cus > 0, REALB_EHIP, "no address for the static scratch array on device %d", dev);
        g_static[dev].num_cus = cus;
        g_static[dev].ptr = p;
    }
    if (ptr) *ptr = g_static[dev].ptr;
    if (num_cus) *num_cus = g_static[dev].num_cus;
    return REALB_OK;
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
    return launch_route_stats(c->num_cus, kRouteBlocksMax, c->hist_part, logits, is_vision, T, c->cfg.E, c->cfg.k,
                              c->cfg.D, topk_ids, topk_w, expert_cnt, expert_vis, rank_load, rank_vis, as_stream(stream));
}

extern "C" int realb_route_stats_static(const float* logits, const uint8_t* is_vision, int T, int E, int k, int D,
                                        int32_t* topk_ids, float* topk_w, int32_t* expert_cnt, int32_t* expert_vis,
                                        int32_t* rank_load, int32_t* rank_vis, void* stream) {
    REALB_REQUIRE(expert_cnt && expert_vis && rank_load && rank_vis, REALB_EINVAL, "NULL argument");
    REALB_REQUIRE(E > 0 && k > 0 && D > 0 && E % D == 0, REALB_ESHAPE, "E=%d must be a positive multiple of D=%d", E, D);
    REALB_REQUIRE(E <= kStaticEMax, REALB_ECAP, "E=%d exceeds the static scratch array's maximum of %d experts", E, kStaticEMax);
    REALB_REQUIRE(k <= E && k <= 16, REALB_ESHAPE, "k=%d must be <= min(E,16)", k);
    REALB_REQUIRE(T >= 0 && (long long)T * k < (1ll << 31), REALB_ECAP, "T=%d: T*k must stay below 2^31", T);
    REALB_REQUIRE(T == 0 || (logits && is_vision && topk_ids && topk_w), REALB_EINVAL, "NULL argument");
    int32_t* part = nullptr;
    int num_cus = 0;
    const int rc = static_scratch_lookup(&part, &num_cus);
    if (rc != REALB_OK) return rc;
    // every block overwrites its whole slice of the array and the reduce reads only the slices of this launch,
    // so nothing has to be cleared between calls
    const int max_blocks = (int)(kStaticCounters / (2 * (size_t)E)) < kStaticBlocksMax ? (int)(kStaticCounters / (2 * (size_t)E)) : kStaticBlocksMax;
    return launch_route_stats(num_cus, max_blocks, part, logits, is_vision, T, E, k, D, topk_ids, topk_w, expert_cnt,
                              expert_vis, rank_load, rank_vis, as_stream(stream));
}
