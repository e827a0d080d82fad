// On-the-fly BF16 -> MXFP4 weight transformation (paper Sec. "Overhead-Aware
// Pipeline Orchestration", Overlapping Pipeline): a pure HBM stream, 2 B read
// and 17/32 B written per element.  Scale bytes go to their K-step-tiled positions.
#include "common.h"
#include "mxfp4_device.h"

namespace realb {

// A tensor is a flat sequence of 32-element blocks (rows are multiples of 128 long and
// contiguous).  A quad of lanes encodes one block: each lane loads 16 B (8 values), the quad
// shares the maximum, each lane stores 4 B of codes and the quad's first lane stores the scale
// byte at its K-step-tiled position.  UNROLL independent loads per lane keep enough bytes in flight.
// One launch covers up to two tensors (the rank's W13 and W2): the first `blocks0` blocks take
// tensor 0, the rest tensor 1, so that the second tensor's stream starts while the first one's last
// blocks drain instead of behind a kernel boundary.
struct QuantTensor {
    const u32x4_t* src;      // BF16 values, 16-byte chunks
    uint32_t* q;             // codes, one dword per chunk
    uint8_t* s;              // scales, K-step tiled
    long long n_chunks;
    int cpr;                 // chunks per row = K / 8
    float inv_cpr;
};
struct QuantJob { QuantTensor t[2]; unsigned blocks0; };

#ifndef REALB_QUANT_UNROLL
#define REALB_QUANT_UNROLL 4
#endif

template <int UNROLL>
__global__ void __launch_bounds__(256) quantize_flat_kernel(const QuantJob job) {
    const bool second = blockIdx.x >= job.blocks0;                                // uniform per block
    const QuantTensor& t = job.t[second ? 1 : 0];
    const u32x4_t* __restrict__ src = t.src;
    uint32_t* __restrict__ q = t.q;
    uint8_t* __restrict__ s = t.s;
    const long long n_chunks = t.n_chunks;
    const int cpr = t.cpr;
    const long long block_base = ((long long)(blockIdx.x - (second ? job.blocks0 : 0u)) * UNROLL) * 256;
    const int KD = cpr >> 4;                                  // K-steps per row (128 elements = 16 chunks)
    const unsigned row_b = (unsigned)block_base / (unsigned)cpr;             // one division per thread; n_chunks < 2^31
    const int in_row0 = (int)((unsigned)block_base - row_b * (unsigned)cpr);
    u32x4_t v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const long long c = block_base + (long long)u * 256 + threadIdx.x;
        v[u] = c < n_chunks ? __builtin_nontemporal_load(src + c) : u32x4_t{0, 0, 0, 0};
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const long long cb = block_base + (long long)u * 256;     // uniform: first chunk of this pass
        const long long c = cb + threadIdx.x;
        uint32_t byte;
        const uint32_t codes = encode_block_quad(v[u], &byte);    // whole quads are in or out of range together
        if (c < n_chunks) {
            __builtin_nontemporal_store(codes, q + c);
            if ((threadIdx.x & 3) == 0) {
                const int in_row = in_row0 + u * 256 + threadIdx.x;                  // < cpr + 256 * UNROLL
                const int dr = (int)(((float)in_row + 0.5f) * t.inv_cpr);            // exact: in_row < 2^16
                s[scale_byte_offset(row_b + dr, (in_row - dr * cpr) >> 2, KD)] = (uint8_t)byte;
            }
        }
    }
}

static int fill_tensor(QuantTensor* t, const void* src, long long rows, int K, uint8_t* q, uint8_t* s, unsigned* blocks) {
    constexpr long long per_block = 256ll * REALB_QUANT_UNROLL;
    const long long n_chunks = rows * (K / 8);
    REALB_REQUIRE(n_chunks < (1ll << 31), REALB_ECAP, "tensor too large for one launch");
    *t = QuantTensor{(const u32x4_t*)src, (uint32_t*)q, s, n_chunks, K / 8, 1.0f / (float)(K / 8)};
    *blocks = (unsigned)((n_chunks + per_block - 1) / per_block);
    return REALB_OK;
}

// Encodes one tensor [rows0, K0], or two when rows1 > 0, in a single launch.
int launch_quantize_flat(const void* src0, long long rows0, int K0, uint8_t* q0, uint8_t* s0,
                         const void* src1, long long rows1, int K1, uint8_t* q1, uint8_t* s1, hipStream_t stream) {
    QuantJob job{};
    unsigned b0 = 0, b1 = 0;
    int rc = fill_tensor(&job.t[0], src0, rows0, K0, q0, s0, &b0);
    if (rc != REALB_OK) return rc;
    if (rows1 > 0) {
        rc = fill_tensor(&job.t[1], src1, rows1, K1, q1, s1, &b1);
        if (rc != REALB_OK) return rc;
    }
    job.blocks0 = b0;
    if (b0 + b1 == 0) return REALB_OK;
    REALB_REQUIRE((unsigned long long)b0 + b1 < (1ull << 31), REALB_ECAP, "too many blocks");
    hipLaunchKernelGGL(quantize_flat_kernel<REALB_QUANT_UNROLL>, dim3(b0 + b1), dim3(256), 0, stream, job);
    REALB_HIP(hipGetLastError());
    return REALB_OK;
}

}  // namespace realb

using namespace realb;

extern "C" {

int realb_quantize_rows_fp4(const void* x, long long rows, int K, uint8_t* q, uint8_t* s, void* stream) {
    REALB_REQUIRE(rows >= 0 && K > 0 && K % 128 == 0 && K <= 65536, REALB_ESHAPE, "rows=%lld K=%d: K must be a positive multiple of 128", rows, K);
    if (rows == 0) return REALB_OK;
    REALB_REQUIRE(x && q && s, REALB_EINVAL, "NULL argument");
    return launch_quantize_flat(x, rows, K, q, s, nullptr, 0, 0, nullptr, nullptr, as_stream(stream));
}

int realb_quantize_experts_fp4(realb_ctx* ctx, const void* w13, const void* w2, int n_local, uint8_t* w13_q,
                               uint8_t* w13_s, uint8_t* w2_q, uint8_t* w2_s, void* stream) {
    REALB_REQUIRE(ctx && w13 && w2 && w13_q && w13_s && w2_q && w2_s, REALB_EINVAL, "NULL argument");
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    REALB_REQUIRE(n_local >= 0 && n_local <= c->n_local, REALB_ECAP, "n_local=%d exceeds the context's %d", n_local, c->n_local);
    return launch_quantize_flat(w13, (long long)n_local * 2 * c->cfg.I, c->cfg.H, w13_q, w13_s,
                                w2, (long long)n_local * c->cfg.H, c->cfg.I, w2_q, w2_s, as_stream(stream));
}

}  // extern "C"
