// NVFP4-faithful variant of the encoder (paper Appendix "Implementation Details", Quantization
// Details): E2M1 elements in groups of 16 with an FP8 E4M3 scale per group, derived from the
// group's absolute maximum divided by 6.0 and a per-tensor global scale, rounded into FP8 and
// clamped; each value divided by the scale and mapped to the nearest E2M1 value.  It exists to
// measure what the mapping onto MXFP4 (power-of-two scales per 32, which the block-scaled
// matrix instructions of gfx950 take) costs; no GEMM here consumes its output.
//
// Every rounding decision is taken in IEEE binary32, in a fixed order:
//   s_local = amax / 6;  r = s_local / g;  byte = E4M3 nearest-even(r), clamped to 448;
//   s_eff = E4M3(byte) * g;  q = |x| / s_eff;  code = E2M1 nearest-even(q), saturating.
#include "common.h"
#include "mxfp4_device.h"

namespace realb {

// E4M3 byte (bias 7, subnormals, largest value 448) nearest to r >= 0, ties to the even mantissa.
__device__ __forceinline__ uint32_t e4m3_from_f32(float r) {
    if (r < 0.015625f) return (uint32_t)__float2int_rn(r * 512.0f);      // subnormal range: multiples of 2^-9; 8 = the first normal
    uint32_t u = __float_as_uint(r);
    u += 0x7FFFFu + ((u >> 20) & 1u);                                    // nearest even on the 20 dropped mantissa bits
    return min((u >> 20) - (120u << 3), 0x7Eu);
}

__device__ __forceinline__ float e4m3_to_f32(uint32_t b) {
    const uint32_t e = b >> 3, m = b & 7u;
    return e == 0 ? (float)m * 0.001953125f : __uint_as_float(((e + 120u) << 23) | (m << 20));
}

// Magnitude code of the E2M1 value nearest to q >= 0, half-way points to the even code, saturating.
__device__ __forceinline__ uint32_t e2m1_from_f32(float q) {
    return (uint32_t)(q > 0.25f) + (uint32_t)(q >= 0.75f) + (uint32_t)(q > 1.25f) + (uint32_t)(q >= 1.75f) +
           (uint32_t)(q > 2.5f) + (uint32_t)(q >= 3.5f) + (uint32_t)(q > 5.0f);
}

// A pair of lanes encodes one group of 16: each lane loads 16 B (8 values), the pair shares the maximum.
__global__ void __launch_bounds__(256) nvfp4_quantize_kernel(const u32x4_t* __restrict__ src, uint32_t* __restrict__ q,
                                                             uint8_t* __restrict__ s, long long n_chunks, float g) {
    const long long c = (long long)blockIdx.x * 256 + threadIdx.x;
    const u32x4_t v = c < n_chunks ? __builtin_nontemporal_load(src + c) : u32x4_t{0, 0, 0, 0};
    uint32_t amax = amax_bits8(v);
    amax = max(amax, (uint32_t)__builtin_amdgcn_mov_dpp((int)amax, 0xB1, 0xF, 0xF, true));     // lanes 1,0,3,2
    const float s_local = __fdiv_rn(__uint_as_float(amax << 16), 6.0f);
    const uint32_t byte = e4m3_from_f32(__fdiv_rn(s_local, g));
    const float s_eff = __fmul_rn(e4m3_to_f32(byte), g);
    const uint32_t d[4] = {v.x, v.y, v.z, v.w};
    uint32_t codes = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t bits = (d[i] >> (16 * h)) & 0xFFFFu;
            const float a = __uint_as_float((bits & 0x7FFFu) << 16);
            const uint32_t mag = s_eff == 0.0f ? 0u : e2m1_from_f32(__fdiv_rn(a, s_eff));
            codes |= (((bits >> 15) << 3) | mag) << (4 * (2 * i + h));
        }
    }
    if (c < n_chunks) {
        __builtin_nontemporal_store(codes, q + c);
        if ((threadIdx.x & 1) == 0) s[c >> 1] = (uint8_t)byte;
    }
}

__global__ void amax_zero_kernel(uint32_t* out) { *out = 0; }

// max |x| of a BF16 tensor as the bit pattern of the equal float (patterns of non-negative floats
// order like unsigned integers, so an integer atomic maximum combines the blocks).
__global__ void __launch_bounds__(256) amax_kernel(const u32x4_t* __restrict__ src, long long n_chunks, uint32_t* out) {
    uint32_t m = 0;
    for (long long c = (long long)blockIdx.x * 256 + threadIdx.x; c < n_chunks; c += (long long)gridDim.x * 256)
        m = max(m, amax_bits8(src[c]));
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, d));
    if ((threadIdx.x & 63) == 0 && m) atomicMax(out, m << 16);
}

}  // namespace realb

using namespace realb;

extern "C" int realb_amax_bf16(const void* x, long long n, float* amax, void* stream) {
    REALB_REQUIRE(amax && (x || n == 0), REALB_EINVAL, "NULL argument");
    REALB_REQUIRE(n >= 0 && n % 8 == 0, REALB_ESHAPE, "element count %lld must be a non-negative multiple of 8", n);
    hipStream_t s = as_stream(stream);
    hipLaunchKernelGGL(amax_zero_kernel, dim3(1), dim3(1), 0, s, reinterpret_cast<uint32_t*>(amax));
    if (n) {
        const long long n_chunks = n / 8;
        const long long want = (n_chunks + 255) / 256;
        const long long blocks = want < 2048 ? want : 2048;
        hipLaunchKernelGGL(amax_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (const u32x4_t*)x, n_chunks,
                           reinterpret_cast<uint32_t*>(amax));
    }
    REALB_HIP(hipGetLastError());
    return REALB_OK;
}

extern "C" int realb_quantize_rows_nvfp4(const void* x, long long rows, int K, float global_scale, uint8_t* q, uint8_t* s,
                                         void* stream) {
    REALB_REQUIRE(rows >= 0 && K > 0 && K % 16 == 0, REALB_ESHAPE, "rows=%lld K=%d: K must be a positive multiple of 16", rows, K);
    REALB_REQUIRE(global_scale > 0.0f && global_scale < INFINITY, REALB_EINVAL, "global scale must be positive and finite");
    if (rows == 0) return REALB_OK;
    REALB_REQUIRE(x && q && s, REALB_EINVAL, "NULL argument");
    const long long n_chunks = rows * (K / 8);
    const long long blocks = (n_chunks + 255) / 256;
    REALB_REQUIRE(blocks < (1ll << 31), REALB_ECAP, "tensor too large for one launch");
    hipLaunchKernelGGL(nvfp4_quantize_kernel, dim3((unsigned)blocks), dim3(256), 0, as_stream(stream), (const u32x4_t*)x,
                       (uint32_t*)q, s, n_chunks, global_scale);
    REALB_HIP(hipGetLastError());
    return REALB_OK;
}
