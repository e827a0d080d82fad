// The rank layer end to end: the paper's four-stage pipeline (Sec. "System
// Overview") with the weight transformation overlapped with dispatch packing
// (Sec. "Overhead-Aware Pipeline Orchestration"): the encoder runs on the
// context's side stream while the permutation runs on the caller's stream, and
// is joined before the GEMMs.
#include "common.h"

using namespace realb;

// quant_in_flight: the weight encoding was already issued on the side stream (speculative mode)
// and ev_join marks its end.  indices_done: the permutation's index kernels are already on the stream.
static int rank_forward_steps(realb_ctx* ctx, realb_layer_io* io, int prec, void* stream, bool quant_in_flight,
                              bool indices_done, bool* forked) {
    REALB_REQUIRE(ctx && io, REALB_EINVAL, "NULL argument");
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    REALB_REQUIRE(prec == REALB_BF16 || prec == REALB_FP4, REALB_EINVAL, "bad precision %d", prec);
    hipStream_t s = as_stream(stream);
    int rc;
    const bool fp4 = prec == REALB_FP4;
    const bool side = io->overlap == 1 || quant_in_flight;
    // everything that can be refused is checked before any work goes to the side stream
    REALB_REQUIRE(io->T >= 0 && io->T <= c->cfg.T_max, REALB_ECAP, "T=%d outside [0, T_max=%d]", io->T, c->cfg.T_max);
    REALB_REQUIRE(io->rank >= 0 && io->rank < c->cfg.D, REALB_EINVAL, "rank=%d outside [0,%d)", io->rank, c->cfg.D);
    REALB_REQUIRE(io->max_rows >= (long long)io->T * (c->cfg.k < c->n_local ? c->cfg.k : c->n_local), REALB_EINVAL,
                  "max_rows=%lld is below the worst case", io->max_rows);
    REALB_REQUIRE(io->expert_offsets && io->h_mid && io->y_rows && io->w2 && io->w13, REALB_EINVAL, "NULL argument");
    REALB_REQUIRE(io->T == 0 || (io->x && io->topk_ids && io->topk_w && io->row_to_assign && io->assign_to_row && io->out), REALB_EINVAL,
                  "NULL argument");
    if (fp4) REALB_REQUIRE(io->w13_q && io->w13_s && io->w2_q && io->w2_s && io->x_q && io->x_s && io->h_s, REALB_EINVAL, "NULL FP4 buffer");
    if (fp4 && io->overlap != 2 && !quant_in_flight) {
        if (side) {
            REALB_HIP(hipEventRecord(c->ev_fork, s));
            REALB_HIP(hipStreamWaitEvent(c->side, c->ev_fork, 0));
            *forked = true;                                  // from here on an error return must still join the side stream
            rc = realb_quantize_experts_fp4(ctx, io->w13, io->w2, c->n_local, io->w13_q, io->w13_s, io->w2_q, io->w2_s, c->side);
            REALB_HIP(hipEventRecord(c->ev_join, c->side));
            if (rc != REALB_OK) return rc;
        } else {
            rc = realb_quantize_experts_fp4(ctx, io->w13, io->w2, c->n_local, io->w13_q, io->w13_s, io->w2_q, io->w2_s, stream);
            if (rc != REALB_OK) return rc;
        }
    }
    if (!indices_done) {
        rc = permute_indices(c, io->topk_ids, io->T, io->rank, io->max_rows, io->expert_offsets, io->row_to_assign,
                             io->assign_to_row, s);
        if (rc != REALB_OK) return rc;
    }
    // Where the gate/up GEMM can fetch its rows through row_to_assign, the permuted copy of the activations is
    // not materialised: BF16 rows come straight from x; FP4 rows from codes and scales written once per TOKEN.
    const bool gather = io->row_to_assign && io->x && gate_up_gather_supported(c, io->T, fp4);
    if (fp4 || !gather) {
        rc = permute_gather(c, io->x, io->assign_to_row, io->T, prec, io->x_perm, io->x_q, io->x_s, s, gather ? 1 : 0);
        if (rc != REALB_OK) return rc;
    }
    if (fp4 && side) REALB_HIP(hipStreamWaitEvent(s, c->ev_join, 0));
    if (gather) {
        REALB_REQUIRE(io->h_mid && io->w2 && io->y_rows, REALB_EINVAL, "NULL argument");
        if (fp4) {
            REALB_REQUIRE(io->x_q && io->x_s && io->h_s, REALB_EINVAL, "NULL argument");
            rc = launch_gate_up_fp4_gather(c, io->expert_offsets, c->n_local, io->max_rows, io->x_q, io->x_s, io->T,
                                           io->row_to_assign, io->w13_q, io->w13_s, (uint8_t*)io->h_mid, io->h_s, s);
        } else {
            REALB_REQUIRE(io->w13 != nullptr, REALB_EINVAL, "NULL argument");
            rc = launch_gate_up_bf16_gather(c, io->expert_offsets, c->n_local, io->max_rows, io->x, io->T, io->row_to_assign,
                                            io->w13, io->h_mid, s);
        }
        if (rc != REALB_OK) return rc;
        rc = realb_grouped_moe_ffn_down(ctx, prec, io->expert_offsets, c->n_local, io->max_rows, io->h_mid, fp4 ? io->h_s : nullptr,
                                        fp4 ? (const void*)io->w2_q : io->w2, fp4 ? io->w2_s : nullptr, io->y_rows, stream);
    } else if (fp4) {
        rc = realb_grouped_moe_ffn(ctx, prec, io->expert_offsets, c->n_local, io->max_rows, io->x_q, io->x_s, io->w13_q,
                                   io->w13_s, io->w2_q, io->w2_s, io->h_mid, io->h_s, io->y_rows, stream);
    } else {
        rc = realb_grouped_moe_ffn(ctx, prec, io->expert_offsets, c->n_local, io->max_rows, io->x_perm, nullptr, io->w13,
                                   nullptr, io->w2, nullptr, io->h_mid, nullptr, io->y_rows, stream);
    }
    if (rc != REALB_OK) return rc;
    rc = realb_combine(ctx, io->y_rows, io->assign_to_row, io->topk_w, io->T, io->out, stream);
    if (rc != REALB_OK) return rc;
    // a speculative encoding that was not used still has to end before the caller's stream moves on
    if (quant_in_flight && !fp4) REALB_HIP(hipStreamWaitEvent(s, c->ev_join, 0));
    return REALB_OK;
}

// Runs the steps; if one of them fails while the weight encoder is in flight on the side stream, the caller's
// stream is still made to wait for it, so that the caller may free or reuse the FP4 weight buffers after its
// stream has drained, whatever this call returned.
static int rank_forward_impl(realb_ctx* ctx, realb_layer_io* io, int prec, void* stream, bool quant_in_flight,
                             bool indices_done) {
    bool forked = quant_in_flight;
    const int rc = rank_forward_steps(ctx, io, prec, stream, quant_in_flight, indices_done, &forked);
    if (rc != REALB_OK && forked && ctx)
        (void)hipStreamWaitEvent(as_stream(stream), reinterpret_cast<Ctx*>(ctx)->ev_join, 0);
    return rc;
}

extern "C" int realb_rank_forward(realb_ctx* ctx, realb_layer_io* io, int prec, void* stream) {
    return rank_forward_impl(ctx, io, prec, stream, false, false);
}

extern "C" int realb_layer_forward(realb_ctx* ctx, realb_layer_io* io, void* stream) {
    REALB_REQUIRE(ctx && io, REALB_EINVAL, "NULL argument");
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    REALB_REQUIRE(io->rank >= 0 && io->rank < c->cfg.D, REALB_EINVAL, "rank=%d outside [0,%d)", io->rank, c->cfg.D);
    int rc;
    // Everything that can be refused is checked before anything is enqueued.
    REALB_REQUIRE(io->force == REALB_FORCE_NONE || io->force == REALB_BF16 || io->force == REALB_FP4, REALB_EINVAL,
                  "bad force value %d", io->force);
    REALB_REQUIRE(io->T >= 0 && io->T <= c->cfg.T_max, REALB_ECAP, "T=%d outside [0, T_max=%d]", io->T, c->cfg.T_max);
    REALB_REQUIRE(io->max_rows >= (long long)io->T * (c->cfg.k < c->n_local ? c->cfg.k : c->n_local), REALB_EINVAL,
                  "max_rows=%lld is below the worst case", io->max_rows);
    REALB_REQUIRE(io->expert_cnt && io->expert_vis && io->rank_load && io->rank_vis && io->expert_offsets, REALB_EINVAL, "NULL argument");
    REALB_REQUIRE(io->T == 0 || (io->logits && io->is_vision && io->topk_ids && io->topk_w && io->row_to_assign && io->assign_to_row),
                  REALB_EINVAL, "NULL argument");
    // Speculative mode: the weight encoding depends on the weights only, so it can start on the
    // side stream before routing and fill the window in which the GPU waits for the host's
    // precision decision.  If the decision is BF16 its output is simply not used.
    const bool speculative = io->overlap == 3 && io->force != REALB_BF16;
    if (speculative) {
        REALB_REQUIRE(io->w13 && io->w2 && io->w13_q && io->w13_s && io->w2_q && io->w2_s, REALB_EINVAL, "NULL FP4 weight buffer");
        hipStream_t s = as_stream(stream);
        REALB_HIP(hipEventRecord(c->ev_fork, s));
        REALB_HIP(hipStreamWaitEvent(c->side, c->ev_fork, 0));
        rc = realb_quantize_experts_fp4(ctx, io->w13, io->w2, c->n_local, io->w13_q, io->w13_s, io->w2_q, io->w2_s, c->side);
        REALB_HIP(hipEventRecord(c->ev_join, c->side));
        if (rc != REALB_OK) { (void)hipStreamWaitEvent(s, c->ev_join, 0); return rc; }
    }
    // an error between here and rank_forward_impl (which joins by itself) still joins the side stream
    auto fail = [&](int code) { if (speculative) (void)hipStreamWaitEvent(as_stream(stream), c->ev_join, 0); return code; };
    rc = realb_route_stats(ctx, io->logits, io->is_vision, io->T, io->topk_ids, io->topk_w, io->expert_cnt, io->expert_vis,
                           io->rank_load, io->rank_vis, stream);
    if (rc != REALB_OK) return fail(rc);
    // The statistics reach pinned host memory with the histogram reduce.  The permutation's index
    // kernels do not depend on the precision, so they go out first and run while the host waits for
    // the event, takes the decision and launches the rest: the GPU does not idle across the decision.
    const hipError_t he = hipEventRecord(c->ev_stats, as_stream(stream));
    if (he != hipSuccess) return fail(hip_fail(he, "hipEventRecord"));
    rc = permute_indices(c, io->topk_ids, io->T, io->rank, io->max_rows, io->expert_offsets, io->row_to_assign,
                         io->assign_to_row, as_stream(stream));
    if (rc != REALB_OK) return fail(rc);
    rc = select_precision_pinned(c, io->T, io->force, io->prec_host, &io->ib_global, &io->M_after, c->ev_stats);
    if (rc != REALB_OK) return fail(rc);
    return rank_forward_impl(ctx, io, io->prec_host[io->rank], stream, speculative, true);
}
