// Context, error reporting and the host-side precision policy.
#include "common.h"
#include "mxfp4_device.h"
#include <string.h>
#include <new>

namespace realb {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int hip_fail(hipError_t e, const char* what) {
    set_error("HIP error %d (%s) in %s", (int)e, hipGetErrorString(e), what);
    return REALB_EHIP;
}

static int check_shape(const realb_config* c) {
    REALB_REQUIRE(c != nullptr, REALB_EINVAL, "config is NULL");
    REALB_REQUIRE(c->T_max >= 0 && c->E > 0 && c->k > 0 && c->D > 0 && c->H > 0 && c->I > 0, REALB_ESHAPE,
                  "non-positive dimension");
    REALB_REQUIRE(c->E % c->D == 0, REALB_ESHAPE, "E=%d is not a multiple of D=%d", c->E, c->D);
    REALB_REQUIRE(c->k <= c->E && c->k <= 16, REALB_ESHAPE, "k=%d must be <= min(E,16)", c->k);
    REALB_REQUIRE(c->E <= 512, REALB_ESHAPE, "E=%d exceeds 512", c->E);
    REALB_REQUIRE(c->E / c->D <= 64, REALB_ESHAPE, "n_local=%d exceeds 64", c->E / c->D);
    REALB_REQUIRE(c->D <= 64, REALB_ESHAPE, "D=%d exceeds 64", c->D);
    REALB_REQUIRE(c->H % 128 == 0 && c->I % 128 == 0, REALB_ESHAPE, "H=%d and I=%d must be multiples of 128", c->H, c->I);
    REALB_REQUIRE(c->H <= 8192, REALB_ESHAPE, "H=%d exceeds 8192", c->H);
    REALB_REQUIRE((long long)c->T_max * c->k < (1ll << 31), REALB_ESHAPE, "T_max*k overflows int32");
    return REALB_OK;
}

// The two device buffers of a context's workspace.
static int n_chunks_max(const realb_config* c) { return ceil_div((long long)c->T_max * c->k, kPermChunk) + 1; }
static size_t wave_cnt_bytes(const realb_config* c) {      // chunk counts, then their sums over groups of chunks
    return ((size_t)n_chunks_max(c) + ceil_div(n_chunks_max(c), kPermGroup)) * (c->E / c->D) * sizeof(int32_t);
}
static size_t hist_part_bytes(const realb_config* c) { return (size_t)kRouteBlocksMax * 2 * c->E * sizeof(int32_t); }

// Precision policy (paper Sec. "Real-time Modality-aware LB Scheduling" and "LB
// Gate").  Ratios are never formed: IB_d > C is load_d*D > C*(T*k), IB_global >
// tau is max_load*D > tau*(T*k), R_vd > M is vis_d > M*load_d, each side in double.
static void policy(const realb_config& c, const int32_t* load, const int32_t* vis, int T, int force,
                   double* M_inout, int32_t* prec, double* ib_global) {
    const int D = c.D;
    const double total = (double)((long long)T * c.k);
    long long max_load = 0;
    for (int d = 0; d < D; ++d) max_load = load[d] > max_load ? load[d] : max_load;
    const double max_ld = (double)(max_load * D);
    if (ib_global) *ib_global = total > 0 ? max_ld / total : 0.0;
    if (force != REALB_FORCE_NONE) {
        for (int d = 0; d < D; ++d) prec[d] = force;
        return;
    }
    if (!((long long)T > c.Gamma)) {                      // LB gate closed: standard execution
        for (int d = 0; d < D; ++d) prec[d] = REALB_BF16;
        return;
    }
    double M = *M_inout, M_new = M;
    if (c.aimd_enabled) {
        const bool congested = max_ld > c.tau * total;
        if (congested) M_new = c.aimd_mul * M;
        else { M_new = M + c.aimd_add; if (M_new > 1.0) M_new = 1.0; }
    }
    const double M_dec = c.update_first ? M_new : M;
    for (int d = 0; d < D; ++d) {
        const bool hot = (double)((long long)load[d] * D) > c.C * total;
        const bool vision_heavy = (double)vis[d] > M_dec * (double)load[d];
        prec[d] = (hot && vision_heavy && load[d] > 0) ? REALB_FP4 : REALB_BF16;
    }
    *M_inout = M_new;
}

// Policy on the pinned host copy of the statistics.  The reduce block of the kernel launched on `s` writes them as
// 64-bit words whose upper halves carry `seq`; the host polls until every word shows it.  Every few thousand polls it
// also asks the stream: a stream that has drained (or failed) without the words arriving ends the wait with an
// error instead of a hang.
int select_precision_pinned(Ctx* c, int T, int force, int32_t* prec_host, double* ib_global_host, double* M_after_host,
                            int seq, hipStream_t s) {
    const int n = 2 * c->cfg.D;
    auto arrived = [&]() {
        for (int i = 0; i < n; ++i) {
            const unsigned long long w = __atomic_load_n(c->stats_words + i, __ATOMIC_ACQUIRE);
            if ((uint32_t)(w >> 32) != (uint32_t)seq) return false;
            c->stats_host[i] = (int32_t)(uint32_t)w;
        }
        return true;
    };
    for (unsigned spin = 1; !arrived(); ++spin) {
        if ((spin & 0xFFF) == 0) {
            const hipError_t q = hipStreamQuery(s);
            if (q == hipSuccess) {                        // everything enqueued has run: the words must be there now
                REALB_REQUIRE(arrived(), REALB_EHIP, "routing statistics never reached the host");
                break;
            }
            if (q != hipErrorNotReady) REALB_HIP(q);
        }
        __builtin_ia32_pause();
    }
    policy(c->cfg, c->stats_host, c->stats_host + c->cfg.D, T, force, &c->M, prec_host, ib_global_host);
    if (M_after_host) *M_after_host = c->M;
    return REALB_OK;
}

}  // namespace realb

using namespace realb;

extern "C" {

void realb_default_config(realb_config* cfg, int T_max, int E, int k, int D, int H, int I) {
    if (!cfg) return;
    memset(cfg, 0, sizeof(*cfg));
    cfg->T_max = T_max; cfg->E = E; cfg->k = k; cfg->D = D; cfg->H = H; cfg->I = I;
    cfg->C = 1.0; cfg->tau = 1.5; cfg->M_init = 0.9; cfg->aimd_mul = 0.5; cfg->aimd_add = 0.1;
    cfg->Gamma = 2048; cfg->aimd_enabled = 1; cfg->update_first = 1;
}

const char* realb_last_error(void) { return g_err; }

int realb_create(const realb_config* cfg, realb_ctx** out) {
    REALB_REQUIRE(out != nullptr, REALB_EINVAL, "out is NULL");
    *out = nullptr;
    int rc = check_shape(cfg);
    if (rc != REALB_OK) return rc;
    Ctx* c = new (std::nothrow) Ctx();
    REALB_REQUIRE(c != nullptr, REALB_EINVAL, "out of host memory");
    c->cfg = *cfg;
    c->n_local = cfg->E / cfg->D;
    c->M = cfg->M_init;
    c->wave_cnt = nullptr; c->group_cnt = nullptr; c->hist_part = nullptr; c->stats_host = nullptr; c->stats_words = nullptr; c->side = nullptr; c->ev_fork = nullptr; c->ev_join = nullptr; c->stats_seq = 0; c->ev_prefetch = nullptr; c->prefetch_pending = false; c->gemm_reserve = 0; c->stage_timing = false; c->stage_valid = false;
    for (auto& ev : c->stage_ev) ev = nullptr;
    hipError_t e = hipGetDevice(&c->device);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&c->num_cus, hipDeviceAttributeMultiprocessorCount, c->device);
    c->n_chunks_max = n_chunks_max(cfg);
    if (e == hipSuccess) e = hipMalloc((void**)&c->wave_cnt, wave_cnt_bytes(cfg));
    if (e == hipSuccess) c->group_cnt = c->wave_cnt + (size_t)c->n_chunks_max * c->n_local;
    if (e == hipSuccess) e = hipMalloc((void**)&c->hist_part, hist_part_bytes(cfg));
    if (e == hipSuccess) e = hipHostMalloc((void**)&c->stats_host, 2 * cfg->D * sizeof(int32_t), hipHostMallocDefault);
    if (e == hipSuccess) e = hipHostMalloc((void**)&c->stats_words, 2 * cfg->D * sizeof(unsigned long long), hipHostMallocCoherent);
    if (e == hipSuccess) memset(c->stats_words, 0, 2 * cfg->D * sizeof(unsigned long long));
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_prefetch, hipEventDisableTiming);
    if (e != hipSuccess) {
        realb_destroy(reinterpret_cast<realb_ctx*>(c));
        return hip_fail(e, "realb_create");
    }
    // set-up for the allocation-free routing call on this device (address of its static scratch array)
    rc = static_scratch_lookup(nullptr, nullptr);
    if (rc != REALB_OK) {
        realb_destroy(reinterpret_cast<realb_ctx*>(c));
        return rc;
    }
    *out = reinterpret_cast<realb_ctx*>(c);
    return REALB_OK;
}

int realb_destroy(realb_ctx* ctx) {
    if (!ctx) return REALB_OK;
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (c->wave_cnt) (void)hipFree(c->wave_cnt);
    if (c->hist_part) (void)hipFree(c->hist_part);
    if (c->stats_host) (void)hipHostFree(c->stats_host);
    if (c->stats_words) (void)hipHostFree(c->stats_words);
    if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
    if (c->ev_join) (void)hipEventDestroy(c->ev_join);
    if (c->ev_prefetch) (void)hipEventDestroy(c->ev_prefetch);
    for (auto& ev : c->stage_ev)
        if (ev) (void)hipEventDestroy(ev);
    if (c->side) (void)hipStreamDestroy(c->side);
    delete c;
    return REALB_OK;
}

size_t realb_workspace_bytes(const realb_config* cfg) {
    if (check_shape(cfg) != REALB_OK) return 0;
    return wave_cnt_bytes(cfg) + hist_part_bytes(cfg);
}

size_t realb_scale_offset(long long row, int kb, int K) {
    if (row < 0 || kb < 0 || K <= 0 || K % 128 != 0 || kb >= K / 32) return (size_t)-1;
    return scale_byte_offset(row, kb, K >> 7);
}

int realb_scale_index_map(long long rows, int K, int64_t* idx_host) {
    REALB_REQUIRE(rows >= 0 && K > 0 && K % 128 == 0, REALB_ESHAPE, "rows=%lld K=%d: K must be a positive multiple of 128", rows, K);
    REALB_REQUIRE(rows == 0 || idx_host != nullptr, REALB_EINVAL, "NULL argument");
    const int nb = K / 32, KD = K >> 7;
    for (long long r = 0; r < rows; ++r)
        for (int kb = 0; kb < nb; ++kb) idx_host[r * nb + kb] = (int64_t)scale_byte_offset(r, kb, KD);
    return REALB_OK;
}

int realb_stage_timing(realb_ctx* ctx, int enable) {
    REALB_REQUIRE(ctx != nullptr, REALB_EINVAL, "ctx is NULL");
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    if (enable)
        for (auto& ev : c->stage_ev)
            if (!ev) REALB_HIP(hipEventCreate(&ev));
    c->stage_timing = false;                       // no valid measurement until the next layer call
    c->stage_valid = false;
    c->stage_timing = enable != 0;
    return REALB_OK;
}

int realb_stage_ms(realb_ctx* ctx, float* ms_host) {
    REALB_REQUIRE(ctx && ms_host, REALB_EINVAL, "NULL argument");
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    REALB_REQUIRE(c->stage_timing && c->stage_valid, REALB_EINVAL, "stage timing is off, or no layer call since it was switched on");
    REALB_HIP(hipEventSynchronize(c->stage_ev[REALB_N_STAGES]));
    for (int i = 0; i < REALB_N_STAGES; ++i) REALB_HIP(hipEventElapsedTime(&ms_host[i], c->stage_ev[i], c->stage_ev[i + 1]));
    return REALB_OK;
}

double realb_get_M(const realb_ctx* ctx) { return ctx ? reinterpret_cast<const Ctx*>(ctx)->M : 0.0; }

int realb_set_M(realb_ctx* ctx, double M) {
    REALB_REQUIRE(ctx != nullptr, REALB_EINVAL, "ctx is NULL");
    reinterpret_cast<Ctx*>(ctx)->M = M;
    return REALB_OK;
}

int realb_select_precision_host(const realb_config* cfg, const int32_t* rank_load_host, const int32_t* rank_vis_host,
                                int T, int force, double* M_inout, int32_t* prec_host, double* ib_global_host) {
    REALB_REQUIRE(cfg && rank_load_host && rank_vis_host && M_inout && prec_host, REALB_EINVAL, "NULL argument");
    REALB_REQUIRE(cfg->D > 0 && cfg->k > 0 && T >= 0, REALB_ESHAPE, "bad D, k or T");
    REALB_REQUIRE(force == REALB_FORCE_NONE || force == REALB_BF16 || force == REALB_FP4, REALB_EINVAL, "bad force value %d", force);
    policy(*cfg, rank_load_host, rank_vis_host, T, force, M_inout, prec_host, ib_global_host);
    return REALB_OK;
}

int realb_select_precision(realb_ctx* ctx, const int32_t* rank_load, const int32_t* rank_vis, int T, int force,
                           int32_t* prec_host, double* ib_global_host, double* M_after_host, void* stream) {
    REALB_REQUIRE(ctx && rank_load && rank_vis && prec_host, REALB_EINVAL, "NULL argument");
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    REALB_REQUIRE(T >= 0 && T <= c->cfg.T_max, REALB_ECAP, "T=%d outside [0, T_max=%d]", T, c->cfg.T_max);
    REALB_REQUIRE(force == REALB_FORCE_NONE || force == REALB_BF16 || force == REALB_FP4, REALB_EINVAL, "bad force value %d", force);
    const int D = c->cfg.D;
    hipStream_t s = as_stream(stream);
    REALB_HIP(hipMemcpyAsync(c->stats_host, rank_load, D * sizeof(int32_t), hipMemcpyDeviceToHost, s));
    REALB_HIP(hipMemcpyAsync(c->stats_host + D, rank_vis, D * sizeof(int32_t), hipMemcpyDeviceToHost, s));
    REALB_HIP(hipStreamSynchronize(s));
    policy(c->cfg, c->stats_host, c->stats_host + D, T, force, &c->M, prec_host, ib_global_host);
    if (M_after_host) *M_after_host = c->M;
    return REALB_OK;
}

}  // extern "C"
