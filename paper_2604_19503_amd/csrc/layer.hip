// The rank layer end to end: the paper's four-stage pipeline (Sec. "System
// Overview") with the weight transformation overlapped with other work
// (Sec. "Overhead-Aware Pipeline Orchestration"): the encoders run on the
// context's side stream -- after the decision beside the permutation, ahead of
// the decision beside the routing and index kernels, or, for the NEXT layer's
// weights, beside this layer's GEMMs -- and are joined before the kernels that
// read their output.
#include "common.h"

using namespace realb;

// Checks of a layer call's arguments that do not depend on the precision; made before anything is enqueued.
static int validate_io(const Ctx* c, const realb_layer_io* io) {
    REALB_REQUIRE(io->T >= 0 && io->T <= c->cfg.T_max, REALB_ECAP, "T=%d outside [0, T_max=%d]", io->T, c->cfg.T_max);
    REALB_REQUIRE(io->rank >= 0 && io->rank < c->cfg.D, REALB_EINVAL, "rank=%d outside [0,%d)", io->rank, c->cfg.D);
    REALB_REQUIRE(io->max_rows >= (long long)io->T * (c->cfg.k < c->n_local ? c->cfg.k : c->n_local), REALB_EINVAL,
                  "max_rows=%lld is below the worst case", io->max_rows);
    REALB_REQUIRE(io->overlap >= 0 && io->overlap <= 4, REALB_EINVAL, "bad overlap value %d", io->overlap);
    REALB_REQUIRE(io->expert_offsets && io->h_mid && io->y_rows && io->w2 && io->w13, REALB_EINVAL, "NULL argument");
    REALB_REQUIRE(io->T == 0 || (io->x && io->topk_ids && io->topk_w && io->row_to_assign && io->assign_to_row && io->out), REALB_EINVAL,
                  "NULL argument");
    if (io->next_w13 != nullptr || io->next_w2 != nullptr) {      // cross-layer prefetch requested
        REALB_REQUIRE(io->next_w13 && io->next_w2 && io->next_w13_q && io->next_w13_s && io->next_w2_q && io->next_w2_s, REALB_EINVAL,
                      "cross-layer prefetch needs next_w13, next_w2 and all four next_* buffers");
        REALB_REQUIRE(io->next_w13_q != io->w13_q && io->next_w13_s != io->w13_s && io->next_w2_q != io->w2_q && io->next_w2_s != io->w2_s,
                      REALB_EINVAL, "the prefetch buffers must differ from this layer's FP4 weight buffers");
        REALB_REQUIRE(io->reserve_cus >= 0 && io->reserve_cus < c->num_cus, REALB_EINVAL, "reserve_cus=%d outside [0, %d)", io->reserve_cus, c->num_cus);
    }
    return REALB_OK;
}

// quant_in_flight: the weight encoding was already issued on the side stream (speculative mode);
// act_in_flight: so was the FP4 encoding of every token's activations (one row per token, the form the
// gathering gate/up GEMM reads); ev_join marks the end of both.  indices_done: the permutation's index
// kernels are already on the stream.
static int rank_forward_steps(realb_ctx* ctx, realb_layer_io* io, int prec, void* stream, bool quant_in_flight, bool act_in_flight,
                              bool indices_done, bool* forked, bool* prefetched) {
    REALB_REQUIRE(ctx && io, REALB_EINVAL, "NULL argument");
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    REALB_REQUIRE(prec == REALB_BF16 || prec == REALB_FP4, REALB_EINVAL, "bad precision %d", prec);
    hipStream_t s = as_stream(stream);
    int rc;
    const bool fp4 = prec == REALB_FP4;
    const bool side = io->overlap == 1 || quant_in_flight;
    // everything that can be refused is checked before any work goes to the side stream
    rc = validate_io(c, io);
    if (rc != REALB_OK) return rc;
    if (fp4) REALB_REQUIRE(io->w13_q && io->w13_s && io->w2_q && io->w2_s && io->x_q && io->x_s && io->h_s, REALB_EINVAL, "NULL FP4 buffer");
    const bool prefetch = io->next_w13 != nullptr;       // cross-layer prefetch of the NEXT layer's weights, beside this layer's GEMMs
    // weights encoded by the previous call's prefetch: everything this call enqueues from here on comes after it.
    // With the activations in flight on the side stream no wait of its own is needed (each cross-stream wait costs the
    // caller's stream microseconds): their encoding was issued behind that prefetch on the same stream, and this call
    // waits for it (ev_join) whatever the precision (the next prefetch goes to that same stream, behind both).
    if (c->prefetch_pending && (io->overlap == 4 || prefetch)) {
        if (!act_in_flight) REALB_HIP(hipStreamWaitEvent(s, c->ev_prefetch, 0));
        c->prefetch_pending = false;
    }
    const bool encoded = io->overlap == 2 || io->overlap == 4;
    auto issue_prefetch = [&]() -> int {                  // called right behind the launch of the first GEMM
        if (!prefetch) return REALB_OK;
        REALB_HIP(hipStreamWaitEvent(c->side, c->ev_fork, 0));
        *prefetched = true;
        const int prc = realb_quantize_experts_fp4(ctx, io->next_w13, io->next_w2, c->n_local, io->next_w13_q, io->next_w13_s,
                                                   io->next_w2_q, io->next_w2_s, c->side);
        REALB_HIP(hipEventRecord(c->ev_prefetch, c->side));
        c->prefetch_pending = true;
        return prc;
    };
    const bool encode_now = fp4 && !encoded && !quant_in_flight;
    if (encode_now && side) {
        REALB_HIP(hipEventRecord(c->ev_fork, s));
        REALB_HIP(hipStreamWaitEvent(c->side, c->ev_fork, 0));
        *forked = true;                                  // from here on an error return must still join the side stream
        rc = realb_quantize_experts_fp4(ctx, io->w13, io->w2, c->n_local, io->w13_q, io->w13_s, io->w2_q, io->w2_s, c->side);
        REALB_HIP(hipEventRecord(c->ev_join, c->side));
        if (rc != REALB_OK) return rc;
    }
    if (!indices_done) {
        stage_mark(c, s, 0);
        stage_mark(c, s, 1);
        rc = permute_indices(c, io->topk_ids, io->T, io->rank, io->max_rows, io->expert_offsets, io->row_to_assign,
                             io->assign_to_row, s);
        if (rc != REALB_OK) return rc;
        stage_mark(c, s, 2);
    }
    if (encode_now && !side) {
        rc = realb_quantize_experts_fp4(ctx, io->w13, io->w2, c->n_local, io->w13_q, io->w13_s, io->w2_q, io->w2_s, stream);
        if (rc != REALB_OK) return rc;
    }
    stage_mark(c, s, 3);
    // Where the gate/up GEMM can fetch its rows through row_to_assign, the permuted copy of the activations is
    // not materialised: BF16 rows come straight from x; FP4 rows from codes and scales written once per TOKEN.
    const bool gather = io->row_to_assign && io->x && gate_up_gather_supported(c, io->T, fp4);
    if ((fp4 && !(act_in_flight && gather)) || !gather) {
        rc = permute_gather(c, io->x, io->assign_to_row, io->T, prec, io->x_perm, io->x_q, io->x_s, s, gather ? 1 : 0);
        if (rc != REALB_OK) return rc;
    }
    // speculative mode: what went to the side stream ahead of the decision is what the gate/up GEMM needs (activations, W13);
    // W2 is encoded here, on the caller's stream, while that is still in flight -- the caller's stream would idle until the join
    // anyway, a BF16 decision never pays for it, and the down GEMM then needs no second cross-stream wait (each costs microseconds).
    if (fp4 && quant_in_flight) {
        rc = launch_quantize_flat(io->w2, (long long)c->n_local * c->cfg.H, c->cfg.I, io->w2_q, io->w2_s, nullptr, 0, 0, nullptr, nullptr, s);
        if (rc != REALB_OK) return rc;
    }
    if (fp4 && ((side && !encoded) || act_in_flight)) REALB_HIP(hipStreamWaitEvent(s, c->ev_join, 0));
    if (prefetch) {
        REALB_HIP(hipEventRecord(c->ev_fork, s));         // the prefetch may start once the stream is here, beside the GEMMs
        c->gemm_reserve = io->reserve_cus;
    }
    struct ReserveReset { Ctx* c; ~ReserveReset() { c->gemm_reserve = 0; } } reserve_reset{c};
    stage_mark(c, s, 4);                              // (behind the joins: waiting for the side stream counts as stage [3])
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
        stage_mark(c, s, 5);
        rc = issue_prefetch();
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
    if (!gather) {
        stage_mark(c, s, 5);                             // (the two GEMMs went out in one call: their time is reported under [4])
        rc = issue_prefetch();
        if (rc != REALB_OK) return rc;
    }
    stage_mark(c, s, 6);
    rc = realb_combine(ctx, io->y_rows, io->assign_to_row, io->topk_w, io->T, io->out, stream);
    if (rc != REALB_OK) return rc;
    stage_mark(c, s, 7);
    c->stage_valid = c->stage_timing;
    // a speculative encoding that was not used still has to end before the caller's stream moves on
    if ((quant_in_flight || act_in_flight) && !fp4) REALB_HIP(hipStreamWaitEvent(s, c->ev_join, 0));
    return REALB_OK;
}

// Runs the steps; if one of them fails while the weight encoder is in flight on the side stream, the caller's
// stream is still made to wait for it, so that the caller may free or reuse the FP4 weight buffers after its
// stream has drained, whatever this call returned.
static int rank_forward_impl(realb_ctx* ctx, realb_layer_io* io, int prec, void* stream, bool quant_in_flight, bool act_in_flight,
                             bool indices_done) {
    bool forked = quant_in_flight || act_in_flight, prefetched = false;
    const int rc = rank_forward_steps(ctx, io, prec, stream, quant_in_flight, act_in_flight, indices_done, &forked, &prefetched);
    if (rc != REALB_OK && ctx) {
        Ctx* c = reinterpret_cast<Ctx*>(ctx);
        if (forked) (void)hipStreamWaitEvent(as_stream(stream), c->ev_join, 0);
        if (prefetched) { (void)hipStreamWaitEvent(as_stream(stream), c->ev_prefetch, 0); c->prefetch_pending = false; }
    }
    return rc;
}

extern "C" int realb_rank_forward(realb_ctx* ctx, realb_layer_io* io, int prec, void* stream) {
    return rank_forward_impl(ctx, io, prec, stream, false, false, false);
}

extern "C" int realb_layer_forward(realb_ctx* ctx, realb_layer_io* io, void* stream) {
    REALB_REQUIRE(ctx && io, REALB_EINVAL, "NULL argument");
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    // Everything that can be refused is checked before anything is enqueued.
    int rc = validate_io(c, io);
    if (rc != REALB_OK) return rc;
    REALB_REQUIRE(io->force == REALB_FORCE_NONE || io->force == REALB_BF16 || io->force == REALB_FP4, REALB_EINVAL,
                  "bad force value %d", io->force);
    REALB_REQUIRE(io->expert_cnt && io->expert_vis && io->rank_load && io->rank_vis, REALB_EINVAL, "NULL argument");
    REALB_REQUIRE(io->T == 0 || (io->logits && io->is_vision), REALB_EINVAL, "NULL argument");
    if (io->force == REALB_FP4)
        REALB_REQUIRE(io->w13_q && io->w13_s && io->w2_q && io->w2_s && io->x_q && io->x_s && io->h_s, REALB_EINVAL, "NULL FP4 buffer");
    // Speculative mode: the weight encoding depends on the weights only, so it can start on the
    // side stream before routing and fill the window in which the GPU waits for the host's
    // precision decision.  If the decision is BF16 its output is simply not used.
    // In the two modes in which the caller already bets on FP4 (speculative, prefetched) the activations are encoded
    // ahead of the decision as well: every token once, on the side stream, beside the latency-bound routing and index
    // kernels -- the form the gathering gate/up GEMM reads (row index = token index), so the gather kernel disappears.
    const bool spec_w = io->overlap == 3 && io->force != REALB_BF16;
    const bool spec_x = (io->overlap == 3 || io->overlap == 4) && io->force != REALB_BF16 && io->T > 0 && io->x && io->x_q && io->x_s &&
                        gate_up_gather_supported(c, io->T, true);
    const bool speculative = spec_w || spec_x;
    if (speculative) {
        if (spec_w) REALB_REQUIRE(io->w13 && io->w2 && io->w13_q && io->w13_s && io->w2_q && io->w2_s, REALB_EINVAL, "NULL FP4 weight buffer");
        hipStream_t s = as_stream(stream);
        REALB_HIP(hipEventRecord(c->ev_fork, s));
        REALB_HIP(hipStreamWaitEvent(c->side, c->ev_fork, 0));
        rc = REALB_OK;
        // side stream: what the gate/up GEMM needs -- the activations and W13 (W2 follows on the caller's stream, after the decision)
        if (spec_x) rc = launch_quantize_flat(io->x, io->T, c->cfg.H, io->x_q, io->x_s, nullptr, 0, 0, nullptr, nullptr, c->side);
        if (rc == REALB_OK && spec_w)
            rc = launch_quantize_flat(io->w13, (long long)c->n_local * 2 * c->cfg.I, c->cfg.H, io->w13_q, io->w13_s, nullptr, 0, 0, nullptr,
                                      nullptr, c->side);
        REALB_HIP(hipEventRecord(c->ev_join, c->side));
        if (rc != REALB_OK) { (void)hipStreamWaitEvent(s, c->ev_join, 0); return rc; }
    }
    // an error between here and rank_forward_impl (which joins by itself) still joins the side stream
    auto fail = [&](int code) { if (speculative) (void)hipStreamWaitEvent(as_stream(stream), c->ev_join, 0); return code; };
    stage_mark(c, as_stream(stream), 0);
    // The statistics reach pinned host memory with the histogram reduce, which then publishes this call's sequence
    // number there.  The permutation's index kernels do not depend on the precision, so they are interleaved with the
    // routing kernels (the reduce shares a launch with the permutation's count kernel) and the ranking kernel runs
    // while the host polls for the number, takes the decision and launches the rest.
    if (++c->stats_seq <= 0) c->stats_seq = 1;
    rc = route_and_index(c, io->logits, io->is_vision, io->T, io->rank, io->max_rows, io->topk_ids, io->topk_w, io->expert_cnt,
                         io->expert_vis, io->rank_load, io->rank_vis, io->expert_offsets, io->row_to_assign, io->assign_to_row,
                         c->stats_seq, as_stream(stream));
    if (rc != REALB_OK) return fail(rc);
    stage_mark(c, as_stream(stream), 1);
    stage_mark(c, as_stream(stream), 2);
    rc = select_precision_pinned(c, io->T, io->force, io->prec_host, &io->ib_global, &io->M_after, c->stats_seq, as_stream(stream));
    if (rc != REALB_OK) return fail(rc);
    return rank_forward_impl(ctx, io, io->prec_host[io->rank], stream, spec_w, spec_x, true);
}

extern "C" int realb_prefetch_join(realb_ctx* ctx, void* stream) {
    REALB_REQUIRE(ctx != nullptr, REALB_EINVAL, "ctx is NULL");
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (c->prefetch_pending) {
        REALB_HIP(hipStreamWaitEvent(as_stream(stream), c->ev_prefetch, 0));
        c->prefetch_pending = false;
    }
    return REALB_OK;
}
