// Internal declarations shared by the library's translation units (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>
#include "../../include/realb.h"

namespace realb {

constexpr int kWave = 64;
constexpr int kPermChunk = 256;    // assignments ranked by one wave in permute
// Smallest group of chunks that one block of the permutation's count and rank kernels handles (the workspace holds one
// per-expert sum per group).
constexpr int kPermGroup = 4;
constexpr int kRouteBlocksMax = 512;   // most blocks the routing kernel is launched with (two per CU on 256 CUs)

struct Ctx {
    realb_config cfg;
    int n_local;
    int device;
    int num_cus;
    double M;
    // device workspace
    int32_t* wave_cnt;     // [n_local, n_chunks]  per-chunk local-expert counts of the permutation (one allocation with group_cnt)
    int32_t* group_cnt;    // [n_local, n_groups]  the same summed over groups of kPermGroup chunks
    int n_chunks_max;
    int32_t* hist_part;    // [kRouteBlocksMax, 2*E]  per-block partial histograms of route_stats
    // pinned host staging for the policy's inputs
    int32_t* stats_host;   // [2*D]: rank loads, rank vision loads (copy target of realb_select_precision)
    unsigned long long* stats_words;   // [2*D], host-coherent: the same, written by the layer call's reduce block, each word
                                       // tagged with the call's sequence number (see hist_reduce_body)
    int stats_seq;         // sequence number of the last layer call's statistics (never 0)
    hipStream_t side;      // side stream for the weight encoder
    hipEvent_t ev_fork, ev_join;
    hipEvent_t ev_prefetch;   // end of the last cross-layer prefetch on the side stream
    bool prefetch_pending;    // ev_prefetch has been recorded and not yet been waited for by a caller's stream
    int gemm_reserve;         // compute units the grouped GEMMs' persistent grids leave free (set around a prefetching call)
    // optional per-stage timing of the layer calls (realb_stage_timing): events recorded on the caller's stream
    bool stage_timing;
    bool stage_valid;      // a whole layer call has recorded all boundaries since timing was switched on
    hipEvent_t stage_ev[REALB_N_STAGES + 1];
};

void set_error(const char* fmt, ...);
// Waits until the reduce block launched on `s` has written the statistics tagged `seq` to stats_words, then evaluates the policy.
int select_precision_pinned(Ctx* c, int T, int force, int32_t* prec_host, double* ib_global_host, double* M_after_host,
                            int seq, hipStream_t s);
int permute_indices(Ctx* c, const int32_t* topk_ids, int T, int rank, long long max_rows, int32_t* expert_offsets,
                    int32_t* row_to_assign, int32_t* assign_to_row, hipStream_t s);
int launch_gate_up_bf16_gather(Ctx* c, const int32_t* expert_offsets, int n_local, long long max_rows, const void* x, int T,
                               const int32_t* row_to_assign, const void* w13, void* h_mid, hipStream_t s);
bool gate_up_gather_supported(const Ctx* c, int T, bool fp4);
int launch_gate_up_fp4_gather(Ctx* c, const int32_t* expert_offsets, int n_local, long long max_rows, const uint8_t* x_q,
                              const uint8_t* x_s, int T, const int32_t* row_to_assign, const uint8_t* w13_q,
                              const uint8_t* w13_s, uint8_t* h_q, uint8_t* h_s, hipStream_t s);
int route_topk_only(Ctx* c, const float* logits, const uint8_t* is_vision, int T, int32_t* topk_ids, float* topk_w, hipStream_t s);
int route_and_index(Ctx* c, const float* logits, const uint8_t* is_vision, int T, int rank, long long max_rows, int32_t* topk_ids,
                    float* topk_w, int32_t* expert_cnt, int32_t* expert_vis, int32_t* rank_load, int32_t* rank_vis,
                    int32_t* expert_offsets, int32_t* row_to_assign, int32_t* assign_to_row, int stats_seq, hipStream_t s);
int permute_gather(Ctx* c, const void* x, const int32_t* assign_to_row, int T, int prec, void* x_perm, uint8_t* x_q,
                   uint8_t* x_s, hipStream_t s, int token_major);
// BF16 -> MXFP4 encoder on one matrix [rows0, K0], or two when rows1 > 0, in a single launch.
int launch_quantize_flat(const void* src0, long long rows0, int K0, uint8_t* q0, uint8_t* s0,
                         const void* src1, long long rows1, int K1, uint8_t* q1, uint8_t* s1, hipStream_t stream);
int hip_fail(hipError_t e, const char* what);
// Address (on the current device) of the file-scope scratch array of realb_route_stats_static and the device's CU
// count; looked up once per device and cached.  Either output may be NULL.
int static_scratch_lookup(int32_t** ptr, int* num_cus);

#define REALB_HIP(call)                                                        \
    do {                                                                       \
        hipError_t e__ = (call);                                               \
        if (e__ != hipSuccess) return ::realb::hip_fail(e__, #call);           \
    } while (0)

#define REALB_REQUIRE(cond, code, ...)                                         \
    do {                                                                       \
        if (!(cond)) { ::realb::set_error(__VA_ARGS__); return (code); }       \
    } while (0)

// Stage boundary i of a layer call (no-op unless stage timing is on).
inline void stage_mark(Ctx* c, hipStream_t s, int i) {
    if (c->stage_timing) (void)hipEventRecord(c->stage_ev[i], s);
}

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }
inline int ceil_div(long long a, long long b) { return (int)((a + b - 1) / b); }

}  // namespace realb
