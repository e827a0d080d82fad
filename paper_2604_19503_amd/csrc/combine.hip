// Unpermute + weighted combine: the rank-local part of the paper's result
// combination (Sec. "MoE Load Balancing Systems", Communication).  HBM-bound:
// reads each expert-output row once, writes each token row once.
#include "common.h"

namespace realb {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4c_t;

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// float -> bf16 pattern, nearest-even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// One block per token (grid-strided); each thread owns 8 consecutive columns per
// pass.  The k rows of a token are accumulated in FP32 in order of j.
template <int KMAX>
__global__ void __launch_bounds__(256) combine_kernel(const u32x4c_t* __restrict__ y_rows, const int32_t* __restrict__ assign_to_row,
                                                      const float* __restrict__ topk_w, int T, int k, int H,
                                                      u32x4c_t* __restrict__ out) {
    const int chunks = H >> 3;
    for (int t = blockIdx.x; t < T; t += gridDim.x) {
        int rows[KMAX];
        float w[KMAX];
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {
            rows[j] = j < k ? assign_to_row[(size_t)t * k + j] : -1;
            w[j] = j < k ? topk_w[(size_t)t * k + j] : 0.f;
        }
        for (int c = threadIdx.x; c < chunks; c += blockDim.x) {
            float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int j = 0; j < KMAX; ++j) {
                if (rows[j] >= 0) {
                    const u32x4c_t v = y_rows[(size_t)rows[j] * chunks + c];
                    acc[0] = fmaf(w[j], bf16_lo(v.x), acc[0]); acc[1] = fmaf(w[j], bf16_hi(v.x), acc[1]);
                    acc[2] = fmaf(w[j], bf16_lo(v.y), acc[2]); acc[3] = fmaf(w[j], bf16_hi(v.y), acc[3]);
                    acc[4] = fmaf(w[j], bf16_lo(v.z), acc[4]); acc[5] = fmaf(w[j], bf16_hi(v.z), acc[5]);
                    acc[6] = fmaf(w[j], bf16_lo(v.w), acc[6]); acc[7] = fmaf(w[j], bf16_hi(v.w), acc[7]);
                }
            }
            u32x4c_t o = {pack_bf16(acc[0], acc[1]), pack_bf16(acc[2], acc[3]), pack_bf16(acc[4], acc[5]),
                          pack_bf16(acc[6], acc[7])};
            out[(size_t)t * chunks + c] = o;
        }
    }
}

}  // namespace realb

using namespace realb;

extern "C" int realb_combine(realb_ctx* ctx, const void* y_rows, const int32_t* assign_to_row, const float* topk_w, int T,
                             void* out, void* stream) {
    REALB_REQUIRE(ctx != nullptr, REALB_EINVAL, "ctx is NULL");
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    REALB_REQUIRE(T >= 0 && T <= c->cfg.T_max, REALB_ECAP, "T=%d outside [0, T_max=%d]", T, c->cfg.T_max);
    if (T == 0) return REALB_OK;
    REALB_REQUIRE(y_rows && assign_to_row && topk_w && out, REALB_EINVAL, "NULL argument");
    const int k = c->cfg.k, H = c->cfg.H;
    const int blocks = T < 256 * 64 ? T : 256 * 64;
    hipStream_t s = as_stream(stream);
    if (k <= 8)
        hipLaunchKernelGGL(combine_kernel<8>, dim3(blocks), dim3(256), 0, s, (const u32x4c_t*)y_rows, assign_to_row, topk_w, T, k, H, (u32x4c_t*)out);
    else
        hipLaunchKernelGGL(combine_kernel<16>, dim3(blocks), dim3(256), 0, s, (const u32x4c_t*)y_rows, assign_to_row, topk_w, T, k, H, (u32x4c_t*)out);
    REALB_HIP(hipGetLastError());
    return REALB_OK;
}
