// Stage 4, balanced MoE execution (paper Sec. "System Overview"): the SwiGLU
// expert FFN of one rank as two grouped GEMMs, in the precision the scheduler
// picked -- BF16 operands on v_mfma_f32_32x32x16_bf16, or MXFP4 operands (W4A4)
// on the block-scaled v_mfma_scale_f32_32x32x64_f8f6f4.
//
// Both precisions share one kernel body because their tiles are byte-identical:
// a K-step is 64 bytes of every operand row (32 BF16 or 128 FP4 values), made of
// two MFMA K-slices of 32 bytes, and a lane's fragment is 16 contiguous bytes of
// one row (8 BF16 values, or the 32 FP4 values of exactly one MX block, whose
// E8M0 scale is therefore one byte per lane).
//
// Block tile: 256 activation rows x 128 weight rows, 4 waves as 2x2, each wave
// 128 x 64 = 4 x 2 MFMA tiles of 32x32 (128 accumulator registers).
//   gate/up : the 128 weight rows are 64 gate rows n0.. and the 64 matching up
//             rows I+n0.., arranged so a wave holds gate and up of the same 32
//             columns -> SwiGLU is element-wise in registers; h is rounded to
//             BF16, staged in LDS, then stored as BF16 or re-encoded to MXFP4.
//   down    : 128 output columns, staged in LDS, stored as BF16 rows.
// Tiles never straddle experts; row tails are clamped on load and masked on
// store.  expert_offsets is read on the device, so no host round trip.
#include "common.h"
#include "mxfp4_device.h"

namespace realb {

typedef __attribute__((ext_vector_type(8))) int v8i_t;
typedef __attribute__((ext_vector_type(16))) float v16f_t;
typedef __attribute__((ext_vector_type(8))) __bf16 v8bf_t;

constexpr int BM = 256;              // activation rows per block
constexpr int BNW = 128;             // weight rows per block
constexpr int KSTEP_BYTES = 64;      // bytes of each operand row per K-step
// LDS stage layout: a 64-byte row segment is split into its four 16-byte parts p = 2*slice + half
// (the unit one lane feeds to one MFMA), and each part has its own sub-array indexed by row:
// [p][row][16 B].  A wave's fragment read (32 consecutive rows, fixed p) is then 512 contiguous
// bytes, and the 32-byte pad between sub-arrays spreads the four parts a lane quad writes over
// different banks.
constexpr int SUB_A = BM * 16 + 32;
constexpr int SUB_B = BNW * 16 + 32;
constexpr int REGION_A = 4 * SUB_A;
constexpr int STAGE_BYTES = 4 * SUB_A + 4 * SUB_B;       // 24832
constexpr int HST = 128 + 16;        // LDS row stride of the staged h tile (64 bf16 + pad)
constexpr int YST = 256 + 16;        // LDS row stride of the staged y tile (128 bf16 + pad)

struct GemmParams {
    const uint8_t* A;        // activations: bf16 [rows,K] or fp4 codes [rows,K/2]
    const uint8_t* As;       // fp4: scales [rows,K/32]
    const uint8_t* W;        // weights: [n_local, w_rows, K] in the same encoding
    const uint8_t* Ws;
    uint8_t* out;            // gate/up: h (bf16 [rows,I] or codes [rows,I/2]); down: y bf16 [rows,H]
    uint8_t* outs;           // gate/up fp4: h scales [rows,I/32]
    const int32_t* offs;     // expert_offsets [n_local+1]
    int n_local;
    int K;                   // contraction length in elements
    int w_rows;              // weight rows per expert (2I or H)
    int n_out;               // output columns (I or H)
    int n_tiles_n;           // column tiles (I/64 or H/128)
};

__host__ __device__ __forceinline__ size_t lds_scale_stride_dwords(int K) { return (size_t)((K >> 7) | 1); }

template <bool FP4, int OPSEL>
__device__ __forceinline__ void mma(v16f_t& acc, const u32x4_t& a, const u32x4_t& b, int sa, int sb) {
    if constexpr (FP4) {
        v8i_t a8 = {(int)a.x, (int)a.y, (int)a.z, (int)a.w, 0, 0, 0, 0};
        v8i_t b8 = {(int)b.x, (int)b.y, (int)b.z, (int)b.w, 0, 0, 0, 0};
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, acc, 4, 4, OPSEL, sa, OPSEL, sb);
    } else {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf_t, a), __builtin_bit_cast(v8bf_t, b), acc, 0, 0, 0);
    }
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    __bf16 b = (__bf16)f;
    return __builtin_bit_cast(uint16_t, b);
}

template <bool FP4, bool GATEUP>
__global__ void __launch_bounds__(256, 2) ffn_gemm_kernel(const GemmParams p) {
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, half = lane >> 5;

    // ---- which tile: blocks b, b+8, b+16, .. share an XCD (and its L2), so each XCD takes a
    //      contiguous range of tiles = consecutive row tiles over all column tiles.
    int total_m = 0;
    for (int e = 0; e < p.n_local; ++e) total_m += (p.offs[e + 1] - p.offs[e] + BM - 1) / BM;
    const int total = total_m * p.n_tiles_n;
    const int per_xcd = (total + 7) >> 3;
    const int slot = blockIdx.x >> 3;
    const int tile = (blockIdx.x & 7) * per_xcd + slot;
    if (slot >= per_xcd || tile >= total) return;
    int mi = tile / p.n_tiles_n;
    const int nt = tile - mi * p.n_tiles_n;
    int e = 0, seg_lo = 0, seg_hi = 0;
    for (; e < p.n_local; ++e) {
        seg_lo = p.offs[e];
        seg_hi = p.offs[e + 1];
        const int te = (seg_hi - seg_lo + BM - 1) / BM;
        if (mi < te) break;
        mi -= te;
    }
    const int row0 = seg_lo + mi * BM;
    const int n0 = nt * (GATEUP ? 64 : 128);
    const int I_up = p.w_rows >> 1;                       // gate/up: offset of the up rows
    const size_t rowbytes = FP4 ? (size_t)(p.K >> 1) : (size_t)p.K * 2;
    const int nks = (int)(rowbytes / KSTEP_BYTES);

    // ---- global -> LDS copy assignment: 16-byte chunks, 4 per 64-byte row segment
    const int part = tid & 3;
    const uint8_t* a_src[4];
    int a_dst[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = (tid >> 2) + 64 * j;
        const int gr = min(row0 + r, seg_hi - 1);
        a_src[j] = p.A + (size_t)gr * rowbytes + part * 16;
        a_dst[j] = part * SUB_A + r * 16;
    }
    const uint8_t* b_src[2];
    int b_dst[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int br = (tid >> 2) + 64 * j;
        const int wrow = GATEUP ? (j == 0 ? n0 + br : I_up + n0 + (br - 64)) : n0 + br;
        b_src[j] = p.W + ((size_t)e * p.w_rows + wrow) * rowbytes + part * 16;
        b_dst[j] = REGION_A + part * SUB_B + br * 16;
    }

    // ---- FP4: all scale bytes of the tile's rows, one dword per row per K-step
    uint32_t* sc = reinterpret_cast<uint32_t*>(smem + 2 * STAGE_BYTES);
    const int spd = (int)lds_scale_stride_dwords(p.K);
    if constexpr (FP4) {
        const int kd = p.K >> 7;
        const size_t srow = (size_t)(p.K >> 5);
        for (int idx = tid; idx < (BM + BNW) * kd; idx += 256) {
            const int row = idx / kd, d = idx - row * kd;
            const uint8_t* src;
            if (row < BM) {
                src = p.As + (size_t)min(row0 + row, seg_hi - 1) * srow;
            } else {
                const int br = row - BM;
                const int wrow = GATEUP ? (br < 64 ? n0 + br : I_up + n0 + (br - 64)) : n0 + br;
                src = p.Ws + ((size_t)e * p.w_rows + wrow) * srow;
            }
            sc[row * spd + d] = *reinterpret_cast<const uint32_t*>(src + 4 * d);
        }
    }

    v16f_t acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // ---- software pipeline: LDS holds K-step ks (double buffered), registers hold K-step ks+1,
    //      whose global loads were issued a whole iteration earlier; the scheduling barriers keep
    //      the LDS refill and the next loads BEHIND the iteration's MFMAs.
    u32x4_t ga[4], gb[2];
#pragma unroll
    for (int j = 0; j < 4; ++j) ga[j] = *reinterpret_cast<const u32x4_t*>(a_src[j]);
#pragma unroll
    for (int j = 0; j < 2; ++j) gb[j] = *reinterpret_cast<const u32x4_t*>(b_src[j]);
#pragma unroll
    for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4_t*>(smem + a_dst[j]) = ga[j];
#pragma unroll
    for (int j = 0; j < 2; ++j) *reinterpret_cast<u32x4_t*>(smem + b_dst[j]) = gb[j];
    if (nks > 1) {
#pragma unroll
        for (int j = 0; j < 4; ++j) ga[j] = *reinterpret_cast<const u32x4_t*>(a_src[j] + KSTEP_BYTES);
#pragma unroll
        for (int j = 0; j < 2; ++j) gb[j] = *reinterpret_cast<const u32x4_t*>(b_src[j] + KSTEP_BYTES);
    }
    __syncthreads();

    // fragment addresses inside a stage
    const int a_frag = half * SUB_A + (wm * 128 + li) * 16;                    // + mt*512 + slice*2*SUB_A
    const int b_row0 = GATEUP ? wn * 32 : wn * 64;                             // tile 0 rows
    const int b_row1 = GATEUP ? 64 + wn * 32 : wn * 64 + 32;                   // tile 1 rows
    const int b_frag0 = REGION_A + half * SUB_B + (b_row0 + li) * 16;          // + slice*2*SUB_B
    const int b_frag1 = REGION_A + half * SUB_B + (b_row1 + li) * 16;
    const int sa_idx = (wm * 128 + li) * spd;                                  // + mt*32*spd + ks
    const int sb_idx0 = (BM + b_row0 + li) * spd;
    const int sb_idx1 = (BM + b_row1 + li) * spd;
    const int sshift = half * 8;

    for (int ks = 0; ks < nks; ++ks) {
        const uint8_t* st = smem + (ks & 1) * STAGE_BYTES;
        int sa[4] = {0, 0, 0, 0}, sb[2] = {0, 0};
        if constexpr (FP4) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) sa[mt] = (int)(sc[sa_idx + mt * 32 * spd + ks] >> sshift);
            sb[0] = (int)(sc[sb_idx0 + ks] >> sshift);
            sb[1] = (int)(sc[sb_idx1 + ks] >> sshift);
        }
        u32x4_t fa0[4], fb0[2], fa1[4], fb1[2];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) fa0[mt] = *reinterpret_cast<const u32x4_t*>(st + a_frag + mt * 512);
        fb0[0] = *reinterpret_cast<const u32x4_t*>(st + b_frag0);
        fb0[1] = *reinterpret_cast<const u32x4_t*>(st + b_frag1);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) fa1[mt] = *reinterpret_cast<const u32x4_t*>(st + 2 * SUB_A + a_frag + mt * 512);
        fb1[0] = *reinterpret_cast<const u32x4_t*>(st + 2 * SUB_B + b_frag0);
        fb1[1] = *reinterpret_cast<const u32x4_t*>(st + 2 * SUB_B + b_frag1);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {                     // K-slice 0: scale bytes 0/1 of the K-step's dword
            mma<FP4, 0>(acc[mt][0], fa0[mt], fb0[0], sa[mt], sb[0]);
            mma<FP4, 0>(acc[mt][1], fa0[mt], fb0[1], sa[mt], sb[1]);
        }
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {                     // K-slice 1: scale bytes 2/3
            mma<FP4, 2>(acc[mt][0], fa1[mt], fb1[0], sa[mt], sb[0]);
            mma<FP4, 2>(acc[mt][1], fa1[mt], fb1[1], sa[mt], sb[1]);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (ks + 1 < nks) {
            uint8_t* nx = smem + ((ks + 1) & 1) * STAGE_BYTES;
#pragma unroll
            for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4_t*>(nx + a_dst[j]) = ga[j];
#pragma unroll
            for (int j = 0; j < 2; ++j) *reinterpret_cast<u32x4_t*>(nx + b_dst[j]) = gb[j];
        }
        __builtin_amdgcn_sched_barrier(0);
        if (ks + 2 < nks) {
#pragma unroll
            for (int j = 0; j < 4; ++j) ga[j] = *reinterpret_cast<const u32x4_t*>(a_src[j] + (size_t)(ks + 2) * KSTEP_BYTES);
#pragma unroll
            for (int j = 0; j < 2; ++j) gb[j] = *reinterpret_cast<const u32x4_t*>(b_src[j] + (size_t)(ks + 2) * KSTEP_BYTES);
        }
        __syncthreads();
    }

    // ---- epilogue.  acc[mt][nt][r] is row mt*32 + (r/4)*8 + half*4 + r%4 of the wave's 128,
    //      column li of the wave's nt-th 32-column tile.  The operand stages are free now.
    const int rows_valid = seg_hi - row0;                 // rows of this tile that exist (may exceed BM)
    if constexpr (GATEUP) {
        uint8_t* hst = smem;                               // [256][HST] bf16 h tile
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float g = acc[mt][0][r], u = acc[mt][1][r];
                const float h = g * u / (1.0f + __expf(-g));
                const int row = wm * 128 + mt * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
                *reinterpret_cast<uint16_t*>(hst + row * HST + (wn * 32 + li) * 2) = f32_to_bf16_rne(h);
            }
        __syncthreads();
        if constexpr (FP4) {
            const size_t qrow = (size_t)(p.n_out >> 1), srow = (size_t)(p.n_out >> 5);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int u = tid + 256 * j;
                const int row = u >> 1, blk = u & 1;
                u32x4_t v[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) v[q] = *reinterpret_cast<const u32x4_t*>(hst + row * HST + blk * 64 + q * 16);
                uint32_t byte;
                const u32x4_t codes = encode_block_lane(v, &byte);
                if (row < rows_valid) {
                    *reinterpret_cast<u32x4_t*>(p.out + (size_t)(row0 + row) * qrow + (n0 >> 1) + blk * 16) = codes;
                    p.outs[(size_t)(row0 + row) * srow + (n0 >> 5) + blk] = (uint8_t)byte;
                }
            }
        } else {
            const size_t orow = (size_t)p.n_out * 2;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int c = tid + 256 * j;
                const int row = c >> 3, pc = c & 7;
                if (row < rows_valid)
                    *reinterpret_cast<u32x4_t*>(p.out + (size_t)(row0 + row) * orow + (size_t)n0 * 2 + pc * 16) =
                        *reinterpret_cast<const u32x4_t*>(hst + row * HST + pc * 16);
            }
        }
    } else {
        uint8_t* yst = smem;                               // [128][YST] bf16, one 128-row half at a time
        const size_t orow = (size_t)p.n_out * 2;
#pragma unroll
        for (int hm = 0; hm < 2; ++hm) {
            if (wm == hm) {
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                    for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int row = mt * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
                            *reinterpret_cast<uint16_t*>(yst + row * YST + (wn * 64 + t2 * 32 + li) * 2) = f32_to_bf16_rne(acc[mt][t2][r]);
                        }
            }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int c = tid + 256 * j;
                const int row = c >> 4, pc = c & 15;
                if (hm * 128 + row < rows_valid)
                    *reinterpret_cast<u32x4_t*>(p.out + (size_t)(row0 + hm * 128 + row) * orow + (size_t)n0 * 2 + pc * 16) =
                        *reinterpret_cast<const u32x4_t*>(yst + row * YST + pc * 16);
            }
            __syncthreads();
        }
    }
}

template <bool FP4, bool GATEUP>
static int launch_gemm(const GemmParams& p, long long max_rows, hipStream_t s) {
    const size_t scale_bytes = FP4 ? (size_t)(BM + BNW) * lds_scale_stride_dwords(p.K) * 4 : 0;
    const size_t lds = 2 * (size_t)STAGE_BYTES + scale_bytes;        // the epilogue staging (<= 36.9 KB) aliases the stages
    static bool attr_done = false;                                   // per instantiation
    if (!attr_done) {
        REALB_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&ffn_gemm_kernel<FP4, GATEUP>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 / 2));
        attr_done = true;
    }
    const long long m_tiles_max = (max_rows + BM - 1) / BM + p.n_local;
    const long long total_max = m_tiles_max * p.n_tiles_n;
    const long long grid = 8 * ((total_max + 7) / 8);
    REALB_REQUIRE(grid < (1ll << 31), REALB_ECAP, "too many tiles");
    REALB_REQUIRE(lds <= 80 * 1024, REALB_ESHAPE, "K=%d needs %zu bytes of LDS", p.K, lds);
    hipLaunchKernelGGL((ffn_gemm_kernel<FP4, GATEUP>), dim3((unsigned)grid), dim3(256), lds, s, p);
    REALB_HIP(hipGetLastError());
    return REALB_OK;
}

}  // namespace realb

using namespace realb;

static int ffn_stages(realb_ctx* ctx, int prec, int stages, const int32_t* expert_offsets, int n_local, long long max_rows,
                      const void* x, const uint8_t* x_s, const void* w13, const uint8_t* w13_s, const void* w2,
                      const uint8_t* w2_s, void* h_mid, uint8_t* h_s, void* y_rows, void* stream) {
    REALB_REQUIRE(ctx && expert_offsets, REALB_EINVAL, "NULL argument");
    Ctx* c = reinterpret_cast<Ctx*>(ctx);
    REALB_REQUIRE(prec == REALB_BF16 || prec == REALB_FP4, REALB_EINVAL, "bad precision %d", prec);
    REALB_REQUIRE(n_local >= 0 && n_local <= c->n_local, REALB_ECAP, "n_local=%d exceeds the context's %d", n_local, c->n_local);
    REALB_REQUIRE(max_rows >= 0, REALB_EINVAL, "max_rows < 0");
    if (max_rows == 0 || n_local == 0) return REALB_OK;
    const bool s1 = stages & 1, s2 = stages & 2;
    REALB_REQUIRE(h_mid && (!s1 || (x && w13)) && (!s2 || (w2 && y_rows)), REALB_EINVAL, "NULL argument");
    REALB_REQUIRE(prec == REALB_BF16 || (h_s && (!s1 || (x_s && w13_s)) && (!s2 || w2_s)), REALB_EINVAL,
                  "NULL scale tensor on the FP4 path");
    const int H = c->cfg.H, I = c->cfg.I;
    hipStream_t s = as_stream(stream);
    GemmParams g1{(const uint8_t*)x, x_s, (const uint8_t*)w13, w13_s, (uint8_t*)h_mid, h_s, expert_offsets, n_local, H, 2 * I, I, I / 64};
    GemmParams g2{(const uint8_t*)h_mid, h_s, (const uint8_t*)w2, w2_s, (uint8_t*)y_rows, nullptr, expert_offsets, n_local, I, H, H, H / 128};
    int rc = REALB_OK;
    if (prec == REALB_FP4) {
        if (s1) rc = launch_gemm<true, true>(g1, max_rows, s);
        if (rc == REALB_OK && s2) rc = launch_gemm<true, false>(g2, max_rows, s);
    } else {
        if (s1) rc = launch_gemm<false, true>(g1, max_rows, s);
        if (rc == REALB_OK && s2) rc = launch_gemm<false, false>(g2, max_rows, s);
    }
    return rc;
}

extern "C" int realb_grouped_moe_ffn(realb_ctx* ctx, int prec, const int32_t* expert_offsets, int n_local, long long max_rows,
                                     const void* x, const uint8_t* x_s, const void* w13, const uint8_t* w13_s,
                                     const void* w2, const uint8_t* w2_s, void* h_mid, uint8_t* h_s, void* y_rows,
                                     void* stream) {
    return ffn_stages(ctx, prec, 3, expert_offsets, n_local, max_rows, x, x_s, w13, w13_s, w2, w2_s, h_mid, h_s, y_rows, stream);
}

extern "C" int realb_grouped_moe_ffn_gate_up(realb_ctx* ctx, int prec, const int32_t* expert_offsets, int n_local,
                                             long long max_rows, const void* x, const uint8_t* x_s, const void* w13,
                                             const uint8_t* w13_s, void* h_mid, uint8_t* h_s, void* stream) {
    return ffn_stages(ctx, prec, 1, expert_offsets, n_local, max_rows, x, x_s, w13, w13_s, nullptr, nullptr, h_mid, h_s, nullptr, stream);
}

extern "C" int realb_grouped_moe_ffn_down(realb_ctx* ctx, int prec, const int32_t* expert_offsets, int n_local,
                                          long long max_rows, const void* h_mid, const uint8_t* h_s, const void* w2,
                                          const uint8_t* w2_s, void* y_rows, void* stream) {
    return ffn_stages(ctx, prec, 2, expert_offsets, n_local, max_rows, nullptr, nullptr, nullptr, nullptr, w2, w2_s,
                      const_cast<void*>(h_mid), const_cast<uint8_t*>(h_s), y_rows, stream);
}
