/*
 * realb.h -- C ABI of the ReaLB rank-layer library for AMD MI355X (gfx950).
 *
 * One expert-parallel (EP) rank's MoE layer whose GEMM precision (BF16 or FP4)
 * is chosen at run time from the router's statistics, following
 *   "ReaLB: Real-Time Load Balancing for Multimodal MoE Inference"
 *   (Sec. "Methodology": System Overview stages 1-4, Real-time Modality-aware LB
 *   Scheduling, Overhead-Aware Pipeline Orchestration; Appendix "Implementation
 *   Details": Quantization Details).
 *
 * Conventions for every entry point
 *   - Pointers are DEVICE pointers unless the parameter name ends in _host.
 *   - All tensors are dense, row-major, allocated and owned by the caller; the
 *     library never frees or reallocates caller memory and never writes to the
 *     weight tensors.  The only memory the library allocates is the context's
 *     workspace, in realb_create, freed in realb_destroy.
 *   - BF16 tensors are passed as void* to 16-bit patterns.
 *   - FP4 tensors are OCP MXFP4: 4-bit E2M1 codes (bit 3 sign; magnitudes
 *     0,.5,1,1.5,2,3,4,6), two per byte with the even element in the low nibble,
 *     plus one E8M0 scale byte (2^(byte-127)) per block of 32 consecutive elements
 *     along the contraction dimension.  Scale tensors are K-STEP TILED, the order in
 *     which the block-scaled MFMA consumes them: for a matrix [rows, K] (K a multiple
 *     of 128, KD = K/128) the byte of (row, block kb) is at
 *         (((row/32)*KD + kb/4)*32 + row%32)*4 + kb%4,
 *     i.e. the 4 scales of one row at one 128-element K-step form a dword and 32
 *     consecutive rows are contiguous; the tensor covers ceil(rows/32)*32 rows, so a
 *     scale buffer "u8 [rows, K/32]" below holds ceil(rows/32)*32*K/32 bytes.  Weight
 *     tensors [n_local, N, K] count as n_local*N rows.  The paper's NVFP4 (blocks of 16, E4M3
 *     scale, global scale) is mapped onto this format because gfx950's
 *     block-scaled matrix instructions take E8M0 scales.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls
 *     are asynchronous on that stream unless stated otherwise.
 *   - Return value: REALB_OK or a negative error code; realb_last_error() gives
 *     the message of the calling thread's last failure.  Nothing aborts or throws.
 *     Non-finite inputs are outside the contract.
 *   - Shapes: H and I multiples of 128 (one K-step of the GEMMs is 128 bytes of a BF16 row or 256 FP4
 *     values, and scale tensors are tiled by 128-element K-steps), H <= 8192; E a multiple of D; 1 <= k <= min(E, 16);
 *     E <= 512; n_local = E/D <= 64.  Expert e lives on rank e / n_local.
 */
#ifndef REALB_H
#define REALB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct realb_ctx realb_ctx;

enum { REALB_OK = 0, REALB_EINVAL = -1, REALB_ESHAPE = -2, REALB_ECAP = -3, REALB_EHIP = -4 };
enum { REALB_BF16 = 0, REALB_FP4 = 1 };
enum { REALB_FORCE_NONE = -1 };

/* Layer shape and policy constants (paper Sec. "Setup": C = 1, M initially 0.9,
 * tau = 1.5, Gamma = 2048; AIMD factors of the AIMD equation: 0.5 and +0.1). */
typedef struct {
    int T_max;          /* largest token count of any call */
    int E, k, D;        /* routed experts, experts per token, EP ranks */
    int H, I;           /* hidden size, SwiGLU intermediate size */
    double C;           /* hotspot threshold on IB_d */
    double tau;         /* congestion threshold on IB_global */
    double M_init;      /* initial vision-ratio threshold M */
    double aimd_mul;    /* multiplicative decrease factor */
    double aimd_add;    /* additive increase step (result capped at 1) */
    long long Gamma;    /* LB gate: policy active only if T > Gamma */
    int aimd_enabled;   /* 0: M stays fixed (the fixed-threshold variants) */
    int update_first;   /* 1: update M from this layer's IB_global, then decide */
} realb_config;

/* Fills *cfg with the paper's constants for the given shape. */
void realb_default_config(realb_config* cfg, int T_max, int E, int k, int D, int H, int I);

/* Creates a context: validates the shape, allocates the device workspace (sized
 * from T_max, k, E, D) and pinned host staging, sets M = M_init.  Uses the
 * current HIP device.  REALB_ESHAPE for unsupported shapes. */
int realb_create(const realb_config* cfg, realb_ctx** out);
int realb_destroy(realb_ctx* ctx);
const char* realb_last_error(void);

/* Device memory, in bytes, that realb_create allocates for this configuration (the permutation's per-chunk
 * counters and the routing kernel's per-block partial histograms); besides it a context holds 24*D bytes of
 * pinned host memory, one stream and its events.  Host-only, no GPU needed; 0 for an unsupported shape
 * (realb_last_error says why). */
size_t realb_workspace_bytes(const realb_config* cfg);

/* Where the E8M0 scale of (row, 32-element block kb) of a matrix [rows, K] lives in a K-step-tiled scale
 * tensor (the formula of the conventions above, as the library itself evaluates it); (size_t)-1 for
 * arguments out of range.  realb_scale_index_map writes the offsets of every (row, kb), row-major
 * [rows, K/32], to host memory: canonical[row][kb] = tiled[idx[row][kb]].  Host-only. */
size_t realb_scale_offset(long long row, int kb, int K);
int realb_scale_index_map(long long rows, int K, int64_t* idx_host);

/* The AIMD threshold M carried across layers (host scalar). */
double realb_get_M(const realb_ctx* ctx);
int realb_set_M(realb_ctx* ctx, double M);

/* Stage 1, routing and profiling (Sec. "System Overview"; runtime state of Sec.
 * "Real-time Modality-aware LB Scheduling").
 *   logits     f32 [T,E]      router logits
 *   is_vision  u8  [T]        1 = vision token
 *   topk_ids   i32 [T,k]  out experts in order of descending logit (ties: lower index)
 *   topk_w     f32 [T,k]  out softmax over the k selected logits
 *   expert_cnt i32 [E]    out assignments per expert
 *   expert_vis i32 [E]    out of those, assignments of vision tokens
 *   rank_load  i32 [D]    out Load_d = assignments on rank d
 *   rank_vis   i32 [D]    out N_vd   = vision assignments on rank d
 * T may be 0 (all counts 0).  REALB_ECAP if T > T_max. */
int realb_route_stats(realb_ctx* ctx, const float* logits, const uint8_t* is_vision, int T,
                      int32_t* topk_ids, float* topk_w, int32_t* expert_cnt, int32_t* expert_vis,
                      int32_t* rank_load, int32_t* rank_vis, void* stream);

/* realb_route_stats for callers that cannot allocate device memory and hold no context: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * kernels as realb_route_stats, with the shape passed directly; the per-block partial histograms, which
 * realb_route_stats keeps in the context's workspace, live in a 2 MiB array inside the library's device
 * image (one copy per GPU, held until the process ends).  Calls no hipMalloc / hipFree and no allocating
 * library routine; the array's address is looked up on the first call on a device (or by realb_create).
 * Limits: E <= 512 (REALB_ECAP beyond), 1 <= k <= min(E, 16), E a multiple of D, T*k < 2^31.
 * All calls on one GPU share the array: calls that overlap on one GPU (different streams or threads)
 * race and are not supported; calls ordered on one stream, or otherwise serialised, are fine.  Nothing
 * needs clearing between calls. */
int realb_route_stats_static(const float* logits, const uint8_t* is_vision, int T, int E, int k, int D,
                             int32_t* topk_ids, float* topk_w, int32_t* expert_cnt, int32_t* expert_vis,
                             int32_t* rank_load, int32_t* rank_vis, void* stream);

/* Stage 2, modality-aware LB scheduling: LB gate (T > Gamma), AIMD update of M,
 * hotspot set {d : IB_d > C}, FP4 iff hotspot and R_vd > M (Sec. "Real-time
 * Modality-aware LB Scheduling", "LB Gate").  force = REALB_BF16 / REALB_FP4
 * overrides the policy for every rank and leaves M untouched.
 * Copies rank_load / rank_vis (device, [D]) to the host and SYNCHRONISES the
 * stream; evaluates the policy on the host; updates the context's M.
 *   prec_host [D] out, ib_global_host / M_after_host: optional (may be NULL). */
int realb_select_precision(realb_ctx* ctx, const int32_t* rank_load, const int32_t* rank_vis, int T,
                           int force, int32_t* prec_host, double* ib_global_host, double* M_after_host,
                           void* stream);

/* The same policy as a pure host function (no GPU, no context): all pointers are
 * host pointers; *M_inout is read and updated. */
int realb_select_precision_host(const realb_config* cfg, const int32_t* rank_load_host,
                                const int32_t* rank_vis_host, int T, int force, double* M_inout,
                                int32_t* prec_host, double* ib_global_host);

/* Stage 3, on-the-fly precision transformation of this rank's expert weights
 * (Sec. "Overhead-Aware Pipeline Orchestration", Overlapping Pipeline): BF16 ->
 * MXFP4, blocks of 32 along the contraction dimension.  Weights are only read.
 *   w13  bf16 [n_local, 2I, H]  rows [0,I) gate, [I,2I) up     -> w13_q u8 [n_local,2I,H/2], w13_s u8 [n_local,2I,H/32]
 *   w2   bf16 [n_local, H, I]                                   -> w2_q  u8 [n_local,H,I/2],  w2_s  u8 [n_local,H,I/32]
 * Meant to be issued on a side stream so that it overlaps realb_permute. */
int realb_quantize_experts_fp4(realb_ctx* ctx, const void* w13, const void* w2, int n_local,
                               uint8_t* w13_q, uint8_t* w13_s, uint8_t* w2_q, uint8_t* w2_s, void* stream);

/* The same encoder on any BF16 matrix [rows, K] (K multiple of 128): q u8 [rows,K/2],
 * s u8 [rows,K/32] (K-step tiled).  No context needed. */
int realb_quantize_rows_fp4(const void* x, long long rows, int K, uint8_t* q, uint8_t* s, void* stream);

/* NVFP4-faithful variant of the encoder, for measuring what the mapping onto MXFP4 costs (paper
 * Appendix "Implementation Details", Quantization Details: E2M1 elements, groups of 16, an FP8
 * E4M3 scale per group from the group's absolute maximum / 6.0 and a global scale, rounded into
 * FP8 and clamped, values mapped to the nearest FP4 value).  No GEMM of this library reads it.
 *   x bf16 [rows, K] (K multiple of 16), global_scale > 0 (host scalar; the usual choice is the
 *   tensor's max |x| / (6 * 448), see realb_amax_bf16)
 *   q u8 [rows, K/2] codes as above;  s u8 [rows, K/16] E4M3 bytes (bias 7, max 448), plain row-major.
 * Rounding decisions in IEEE binary32: s_local = amax/6, r = s_local/global_scale, byte = nearest-even
 * E4M3(r) clamped to 448, s_eff = E4M3(byte)*global_scale, code = nearest-even E2M1(|x|/s_eff), saturating;
 * a group whose scale rounds to 0 gets byte 0 and zero magnitudes; sign bits are kept. */
int realb_quantize_rows_nvfp4(const void* x, long long rows, int K, float global_scale, uint8_t* q, uint8_t* s,
                              void* stream);

/* max |x| over n BF16 elements (n multiple of 8) as a float, written to *amax (device). */
int realb_amax_bf16(const void* x, long long n, float* amax, void* stream);

/* Token permutation / dispatch packing for rank `rank` (the local stand-in for
 * the all-to-all dispatch of Sec. "Overhead-Aware Pipeline Orchestration").
 * Rows are this rank's assignments sorted by (local expert, a = t*k + j).
 *   x              bf16 [T,H]
 *   topk_ids       i32  [T,k]
 *   expert_offsets i32  [n_local+1] out  exclusive prefix of local expert counts
 *   row_to_assign  i32  [>= R]      out  a of each row (R = expert_offsets[n_local])
 *   assign_to_row  i32  [T*k]       out  row of each assignment, -1 if not local
 *   prec == REALB_BF16: x_perm bf16 [>= R, H] out  (x_q, x_s ignored, may be NULL)
 *   prec == REALB_FP4 : x_q u8 [>= R, H/2], x_s u8 [>= R, H/32] out (x_perm ignored)
 * Row buffers must hold max_rows rows; REALB_EINVAL if max_rows < min(T*k, T*n_local)
 * (the worst case), since R is only known on the device. */
int realb_permute(realb_ctx* ctx, const void* x, const int32_t* topk_ids, int T, int rank, int prec,
                  long long max_rows, int32_t* expert_offsets, int32_t* row_to_assign, int32_t* assign_to_row,
                  void* x_perm, uint8_t* x_q, uint8_t* x_s, void* stream);

/* Stage 4, balanced MoE execution: SwiGLU expert FFN as two grouped GEMMs over
 * the expert segments given by expert_offsets (read on the device).
 *   gate/up: G,U = X . W13^T (FP32 accumulate), h = silu(G)*U, h rounded to BF16;
 *            FP4 path: that BF16 h is encoded to MXFP4 along I (W4A4).
 *   down:    Y = h . W2^T (FP32 accumulate), rounded to BF16.
 *   prec == REALB_BF16: x = x_perm bf16 [max_rows,H], w13/w2 = BF16 weights, x_s/w13_s/w2_s ignored,
 *                       h_mid bf16 [max_rows,I] (workspace/out), h_s ignored
 *   prec == REALB_FP4 : x = x_q, w13 = w13_q, w2 = w2_q with their scale tensors,
 *                       h_mid u8 [max_rows,I/2], h_s u8 [max_rows,I/32] (workspace/out)
 *   y_rows bf16 [max_rows,H] out; only rows < R are written. */
int realb_grouped_moe_ffn(realb_ctx* ctx, int prec, const int32_t* expert_offsets, int n_local,
                          long long max_rows, const void* x, const uint8_t* x_s,
                          const void* w13, const uint8_t* w13_s, const void* w2, const uint8_t* w2_s,
                          void* h_mid, uint8_t* h_s, void* y_rows, void* stream);

/* The two GEMMs of realb_grouped_moe_ffn as separate calls (same arguments and
 * layouts): gate/up writes h_mid (and h_s), down reads them and writes y_rows.
 * realb_grouped_moe_ffn is exactly gate_up followed by down on the same stream. */
int realb_grouped_moe_ffn_gate_up(realb_ctx* ctx, int prec, const int32_t* expert_offsets, int n_local,
                                  long long max_rows, const void* x, const uint8_t* x_s,
                                  const void* w13, const uint8_t* w13_s, void* h_mid, uint8_t* h_s, void* stream);
int realb_grouped_moe_ffn_down(realb_ctx* ctx, int prec, const int32_t* expert_offsets, int n_local,
                               long long max_rows, const void* h_mid, const uint8_t* h_s,
                               const void* w2, const uint8_t* w2_s, void* y_rows, void* stream);

/* Tuning hook for the grouped GEMMs' kernel: 0 = automatic (default: 16 where the output
 * width is a multiple of its tile -- I % 128 == 0 for gate/up, H % 256 == 0 for down -- else 2),
 * 16 = persistent 256x256 tiles fed by direct-to-LDS loads, 2 = register-staged 256x128
 * tiles with two blocks per CU, 8 = register-staged 256x256 tiles with one block per CU.
 * Process-wide; outputs are bit-identical for every choice (the accumulation order along K
 * does not change).  REALB_EINVAL for any other value. */
int realb_set_gemm_tile(int wn);

/* Unpermute + weighted combine (local part of the result combination):
 * out[t] = sum over j with assign_to_row[t*k+j] >= 0 of topk_w[t,j] * y_rows[row],
 * FP32 accumulate in order of j, rounded once to BF16; tokens with no local
 * expert give 0.   out bf16 [T,H]. */
int realb_combine(realb_ctx* ctx, const void* y_rows, const int32_t* assign_to_row, const float* topk_w,
                  int T, void* out, void* stream);

/* All tensors of one layer call, for realb_layer_forward. */
typedef struct {
    /* inputs */
    const float* logits; const uint8_t* is_vision; const void* x; int T;
    const void* w13; const void* w2;            /* this rank's BF16 expert weights */
    int rank; int force;
    int overlap;                                /* weight encoding: 0 = on `stream`, 1 = on the context's side stream,
                                                   2 = skipped (w13_q .. w2_s already hold this layer's encoded weights),
                                                   3 = speculative (realb_layer_forward only): W13's is issued on the side
                                                       stream BEFORE routing, so that it fills the wait for the host's
                                                       decision, W2's on `stream` once the decision is FP4; W13's is
                                                       unused if the decision is BF16 (in modes 3 and 4 the activations
                                                       of all T tokens are encoded there ahead of the decision as well),
                                                   4 = prefetched: w13_q .. w2_s are being filled by the previous call's
                                                       cross-layer prefetch (see next_w13 below); the GEMMs wait for it */
    long long max_rows;
    /* cross-layer prefetch (optional, all NULL / 0 to disable): the NEXT layer's BF16 weights and the buffers that
       receive their FP4 encoding.  The encoder for them is issued on the context's side stream right behind this
       layer's gate/up GEMM launch and runs beside this layer's two GEMMs, which leave `reserve_cus` compute units
       free for it (their persistent grids shrink by that many blocks).  The next call then passes those buffers as
       w13_q .. w2_s with overlap = 4.  The buffers must differ from this call's w13_q .. w2_s. */
    const void* next_w13; const void* next_w2;
    uint8_t* next_w13_q; uint8_t* next_w13_s; uint8_t* next_w2_q; uint8_t* next_w2_s;
    int reserve_cus;
    /* outputs / workspaces (caller-allocated) */
    int32_t* topk_ids; float* topk_w; int32_t* expert_cnt; int32_t* expert_vis;
    int32_t* rank_load; int32_t* rank_vis;
    int32_t* expert_offsets; int32_t* row_to_assign; int32_t* assign_to_row;
    void* x_perm; uint8_t* x_q; uint8_t* x_s;
    uint8_t* w13_q; uint8_t* w13_s; uint8_t* w2_q; uint8_t* w2_s;
    void* h_mid; uint8_t* h_s; void* y_rows; void* out;
    /* results (host) */
    int32_t prec_host[64]; double ib_global; double M_after;
} realb_layer_io;

/* (realb_layer_forward / realb_rank_forward fuse the permutation's gather into the gate/up GEMM where
 * that GEMM can fetch its rows through row_to_assign: on the BF16 path x_perm is then left unwritten, and
 * on the FP4 path x_q / x_s hold one encoded row per TOKEN that has a local expert -- row index = token
 * index, scales tiled by token index -- instead of one per permuted row.  realb_permute itself always
 * produces the permuted rows described above.) */

/* Runs the whole path for one rank on `stream`: route_stats -> select_precision
 * (host decision: the calling thread spins until the routing statistics, which a kernel on `stream` writes to
 * host-coherent pinned memory, have arrived -- so the call returns only after everything that preceded it on `stream`
 * and its own routing kernels have run; an error of the stream ends the wait) -> [FP4 only: quantize_experts_fp4, on the
 * context's side stream when io->overlap, concurrent with] permute ->
 * grouped_moe_ffn -> combine.  The side stream is joined before the GEMMs.
 * With next_w13 set, the next layer's weights are encoded on the side stream beside this layer's GEMMs
 * (cross-layer form of the overlapping pipeline of Sec. "Overhead-Aware Pipeline Orchestration": the
 * GEMMs are compute-bound and leave the memory system idle, as the dispatch does in the paper); that
 * encoding is joined by the NEXT call (overlap = 4), or by realb_prefetch_join. */
int realb_layer_forward(realb_ctx* ctx, realb_layer_io* io, void* stream);

/* Runs permute .. combine for one rank with a precision already decided and
 * routing already computed (used to time simulated ranks one after the other). */
int realb_rank_forward(realb_ctx* ctx, realb_layer_io* io, int prec, void* stream);

/* Measurement aid: per-stage GPU time of the layer calls.  While enabled, realb_layer_forward and
 * realb_rank_forward record timing events on the caller's stream at their stage boundaries (a few
 * microseconds of overhead per call, so leave it off when timing whole steps); realb_stage_ms waits for
 * the last call and returns, in milliseconds, how long each stage of THAT call took on the GPU:
 *   [0] route_stats  [1] permutation indices (realb_layer_forward interleaves the two groups of kernels and reports
 *   their sum under [0])  [2] host decision + weight encoding on the caller's stream
 *   [3] gather / activation encoding, incl. any wait for the side stream's encoders  [4] gate/up GEMM  [5] down GEMM  [6] combine
 * (realb_rank_forward: [0] holds only the few microseconds between two markers).  ms_host receives
 * REALB_N_STAGES floats.  REALB_EINVAL if timing is off or no call has been made since it was switched on. */
enum { REALB_N_STAGES = 7 };
int realb_stage_timing(realb_ctx* ctx, int enable);
int realb_stage_ms(realb_ctx* ctx, float* ms_host);

/* Makes `stream` wait for the cross-layer prefetch issued by the last realb_layer_forward / realb_rank_forward
 * call of this context (e.g. before the caller frees or reuses the next_* buffers without running the next layer). */
int realb_prefetch_join(realb_ctx* ctx, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* REALB_H */
