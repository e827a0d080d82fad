// Device-side MXFP4 encoding of BF16 data (paper Appendix "Implementation
// Details", Quantization Details, mapped to OCP MXFP4: E2M1 codes, one E8M0
// scale per 32 elements, scale exponent = floor(log2 amax) - 2).
//
// The E2M1 rounding itself is done by the gfx950 converter
// v_cvt_scalef32_pk_fp4_bf16, which divides by the power of two held in the
// exponent field of its scale operand, rounds to nearest with ties to the even
// code, saturates at +-6 and keeps the input's sign bit; it was checked against
// an exact-rational enumeration for every finite BF16 pattern.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace realb {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) unsigned short u16x2_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;

// Where a scale byte lives.  Scale tensors are "K-step tiled" so that the block-scaled MFMA can
// fetch them straight from memory: for a matrix [rows, K] with KD = K/128 K-steps, the 4 scale
// bytes of (row, K-step) form one dword, and the dwords of 32 consecutive rows at one K-step are
// contiguous (128 bytes):   byte(row, kb) at (((row/32)*KD + kb/4)*32 + row%32)*4 + kb%4.
// The tensor covers ceil(rows/32)*32 rows.
__host__ __device__ __forceinline__ size_t scale_byte_offset(long long row, int kb, int KD) {
    return ((((size_t)(row >> 5) * KD + (kb >> 2)) * 32 + (row & 31)) << 2) + (kb & 3);
}

// max |.| of the two BF16 halves of each of 4 dwords, as a 15-bit integer pattern.
__device__ __forceinline__ uint32_t amax_bits8(const u32x4_t& v) {
    u16x2_t a = __builtin_bit_cast(u16x2_t, v.x & 0x7FFF7FFFu);
    u16x2_t b = __builtin_bit_cast(u16x2_t, v.y & 0x7FFF7FFFu);
    u16x2_t c = __builtin_bit_cast(u16x2_t, v.z & 0x7FFF7FFFu);
    u16x2_t d = __builtin_bit_cast(u16x2_t, v.w & 0x7FFF7FFFu);
    u16x2_t m = __builtin_elementwise_max(__builtin_elementwise_max(a, b), __builtin_elementwise_max(c, d));
    return max((uint32_t)m.x, (uint32_t)m.y);
}

// E8M0 byte of a block whose largest magnitude has the BF16 pattern `amax`:
// 127 for an all-zero block, else max(exponent field - 2, 0)  (the clamp covers
// exponent fields 0 and 1, i.e. subnormal and near-subnormal maxima).
__device__ __forceinline__ uint32_t e8m0_from_amax(uint32_t amax) {
    int ef = (int)(amax >> 7);
    uint32_t byte = (uint32_t)max(ef - 2, 0);
    return amax == 0 ? 127u : byte;
}

// The converter's scale operand: only its exponent field is used, byte 0 acts as 2^-127.
__device__ __forceinline__ float scale_operand(uint32_t e8m0) { return __uint_as_float(e8m0 << 23); }

// 8 BF16 values (4 dwords) -> 8 codes packed in one dword, first element in the lowest nibble.
__device__ __forceinline__ uint32_t encode8(const u32x4_t& v, float scale) {
    // element reads go through scalars: bit-casting a vector-element lvalue directly reads element 0
    const uint32_t d0 = v.x, d1 = v.y, d2 = v.z, d3 = v.w;
    uint32_t r = 0;
    r = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(r, __builtin_bit_cast(bf16x2_t, d0), scale, 0);
    r = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(r, __builtin_bit_cast(bf16x2_t, d1), scale, 1);
    r = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(r, __builtin_bit_cast(bf16x2_t, d2), scale, 2);
    r = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(r, __builtin_bit_cast(bf16x2_t, d3), scale, 3);
    return r;
}

// max over the 4 lanes of an aligned quad (lanes 4q..4q+3), via DPP quad permutes.
__device__ __forceinline__ uint32_t quad_max(uint32_t v) {
    uint32_t o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);   // lanes 1,0,3,2
    v = max(v, o);
    o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);            // lanes 2,3,0,1
    return max(v, o);
}

// One MX block handled by 4 neighbouring lanes, each holding 8 consecutive values.
// Returns this lane's 8 codes; *e8m0 is the block's scale byte (same in the 4 lanes).
__device__ __forceinline__ uint32_t encode_block_quad(const u32x4_t& v, uint32_t* e8m0) {
    uint32_t byte = e8m0_from_amax(quad_max(amax_bits8(v)));
    *e8m0 = byte;
    return encode8(v, scale_operand(byte));
}

// One MX block held entirely by one lane (32 values in 4 x uint4).
__device__ __forceinline__ u32x4_t encode_block_lane(const u32x4_t (&v)[4], uint32_t* e8m0) {
    uint32_t amax = max(max(amax_bits8(v[0]), amax_bits8(v[1])), max(amax_bits8(v[2]), amax_bits8(v[3])));
    uint32_t byte = e8m0_from_amax(amax);
    *e8m0 = byte;
    float sc = scale_operand(byte);
    u32x4_t r = {encode8(v[0], sc), encode8(v[1], sc), encode8(v[2], sc), encode8(v[3], sc)};
    return r;
}

}  // namespace realb
