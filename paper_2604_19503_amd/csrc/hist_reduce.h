// Reduction of the routing kernel's per-block partial histograms (one block per EP rank), shared by the stand-alone
// reduce kernel and by the layer call's fused reduce + count launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace realb {

// Adds up the routing kernel's per-block partial histograms (a separate launch: the kernel boundary makes the partials of
// all XCDs visible).  One block per EP rank d: it sums the 2*n_local counters of the rank's experts (counts, then vision
// counts) over the partials and from them the rank's load and vision load -- D short, independent reductions instead
// of one long one, which matters when an HBM-bound kernel runs beside this latency-bound one.
// With stats_words != NULL the two per-rank sums also go to the context's pinned, host-coherent buffer stats_words [2*D]
// (loads, then vision loads), each as one 64-bit word that carries stats_seq in its upper half: the host polls until
// every word shows the sequence number of its call, so realb_layer_forward learns the statistics a few microseconds
// after the blocks have them -- without an event behind the kernel, without waiting for the kernel's other blocks, and
// without a fence (every word validates itself).
// Thread layout: counter c = tid % CW, slice = tid / CW; each slice walks its share of the partials, LDS atomics merge
// the slices.  tot: 2*n_local ints of LDS.
__device__ __forceinline__ void hist_reduce_body(int32_t* tot, const int32_t* __restrict__ hist_part, int n_part, int E, int D, int d,
                                                 int32_t* __restrict__ expert_cnt, int32_t* __restrict__ expert_vis,
                                                 int32_t* __restrict__ rank_load, int32_t* __restrict__ rank_vis,
                                                 unsigned long long* __restrict__ stats_words, int stats_seq) {
    const int n_local = E / D;
    const int C2 = 2 * n_local;                       // <= 128
    const size_t pitch = 2 * (size_t)E;
    for (int i = threadIdx.x; i < C2; i += blockDim.x) tot[i] = 0;
    __syncthreads();
    int cw = 1;
    while (cw < C2) cw <<= 1;                         // counters per slice row, power of two
    const int n_slices = blockDim.x / cw;
    const int c = threadIdx.x % cw, slice = threadIdx.x / cw;
    if (c < C2 && slice < n_slices) {
        const int col = c < n_local ? d * n_local + c : E + d * n_local + (c - n_local);
        int sum = 0;
        int b = slice;
        for (; b + 31 * n_slices < n_part; b += 32 * n_slices) {       // 32 independent loads in flight per thread
            int v[32];
#pragma unroll
            for (int i = 0; i < 32; ++i) v[i] = hist_part[(size_t)(b + i * n_slices) * pitch + col];
#pragma unroll
            for (int i = 0; i < 32; ++i) sum += v[i];
        }
        for (; b < n_part; b += n_slices) sum += hist_part[(size_t)b * pitch + col];
        if (sum) atomicAdd(&tot[c], sum);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < n_local; i += blockDim.x) {
        expert_cnt[d * n_local + i] = tot[i];
        expert_vis[d * n_local + i] = tot[n_local + i];
    }
    if (threadIdx.x == 0) {
        int load = 0, vis = 0;
        for (int e = 0; e < n_local; ++e) { load += tot[e]; vis += tot[n_local + e]; }
        rank_load[d] = load;
        rank_vis[d] = vis;
        if (stats_words) {                            // pinned host copy for the policy: no copy launches, no event
            const unsigned long long tag = (unsigned long long)(uint32_t)stats_seq << 32;
            __hip_atomic_store(stats_words + d, tag | (uint32_t)load, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            __hip_atomic_store(stats_words + D + d, tag | (uint32_t)vis, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
}

}  // namespace realb
