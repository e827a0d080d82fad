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
// The MFMA runs "transposed": the weight rows are its A operand and the
// activation rows its B operand, so a lane ends up with one activation row and
// 16 weight rows.  The weight rows of a 32-row tile are stored in LDS in a
// permuted order chosen so that those 16 are CONSECUTIVE output columns
// (columns 16*half .. 16*half+15 of the tile, half = lane/32).  The epilogues
// therefore need no LDS and no barrier:
//   gate/up : a wave holds the gate and the up tile of the same 32 columns, so
//             SwiGLU is element-wise in registers; h is rounded to BF16 and a
//             lane stores 32 contiguous bytes, or -- FP4 path -- shares the
//             block maximum with lane^32 (the other 16 columns of the MX block),
//             encodes its 16 values and stores 8 contiguous code bytes.
//   down    : a lane stores 32 contiguous bytes of its output row per tile.
// Tiles never straddle experts; row tails are clamped on load and masked on
// store.  expert_offsets is read on the device, so no host round trip.
#include "common.h"
#include "mxfp4_device.h"
#include <atomic>

namespace realb {

// Devices (bit = device index) on which a kernel instantiation has had its dynamic-LDS limit raised.
static bool first_use_on_device(std::atomic<unsigned long long>& seen, int device) {
    const unsigned long long bit = 1ull << (device & 63);
    return (seen.load(std::memory_order_acquire) & bit) == 0;
}
static void mark_used_on_device(std::atomic<unsigned long long>& seen, int device) {
    seen.fetch_or(1ull << (device & 63), std::memory_order_release);
}

typedef __attribute__((ext_vector_type(8))) int v8i_t;
typedef __attribute__((ext_vector_type(16))) float v16f_t;
typedef __attribute__((ext_vector_type(8))) __bf16 v8bf_t;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2_t;

constexpr int BM = 256;              // activation rows per block
constexpr int KSTEP_BYTES = 64;      // bytes of each operand row per K-step

// Tile geometry: the block has 2 x WGN waves (rows x columns); a wave owns 128 activation rows
// x WN*32 weight rows, i.e. 4 x WN MFMA tiles of 32x32.
//
// LDS stage layout: a 64-byte row segment is split into its four 16-byte parts p = 2*slice + half
// (the unit one lane feeds to one MFMA), and each part has its own sub-array indexed by row:
// [p][row][16 B].  A wave's fragment read (32 consecutive rows, fixed p) is then 512 contiguous
// bytes, and the 32-byte pad between sub-arrays spreads the four parts a lane quad writes over
// different banks.
template <int WN, int WGN>
struct Geo {
    static constexpr int NT = 128 * WGN;                // threads per block
    static constexpr int BNW = 32 * WN * WGN;           // weight rows per block
    static constexpr int GC = BNW / 2;                  // gate/up: h columns per block
    static constexpr int SUB_A = BM * 16 + 32;
    static constexpr int SUB_B = BNW * 16 + 32;
    static constexpr int REGION_A = 4 * SUB_A;
    static constexpr int STAGE = 4 * SUB_A + 4 * SUB_B;
    static constexpr int JA = BM * 4 / NT;              // 16-byte global loads per thread per K-step, activations
    static constexpr int JB = BNW * 4 / NT;             //                                           , weights
};

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
    int n_tiles_n;           // column tiles (I/GC or H/BNW)
    const int32_t* row_src;  // gathering gate/up GEMM only: row_to_assign; row r's activations are A[row_src[r] / k]
    uint32_t src_magic;      //   a / k == (a * src_magic) >> src_shift for 0 <= a < 2^31  (k = experts per token)
    int src_shift;
};

// Exact division of 0 <= a < 2^31 by a small constant k through one multiplication: with s = ceil(log2 k) and
// m = floor(2^(31+s) / k) + 1 < 2^32, the excess m*k - 2^(31+s) is at most k <= 2^s, so a*m / 2^(31+s) exceeds
// a/k by less than 1/k and the floors agree.
static void division_magic(int k, uint32_t* magic, int* shift) {
    int s = 0;
    while ((1 << s) < k) ++s;
    *magic = (uint32_t)((1ull << (31 + s)) / (unsigned)k + 1);
    *shift = 31 + s;
}
__device__ __forceinline__ int div_by_magic(int a, uint32_t magic, int shift) {
    return (int)(((unsigned long long)(uint32_t)a * magic) >> shift);
}

// acc += W_tile (A operand, 32 weight rows) x X_tile^T (B operand, 32 activation rows)
template <bool FP4, int OPSEL>
__device__ __forceinline__ void mma(v16f_t& acc, const u32x4_t& w, const u32x4_t& x, int sw, int sx) {
    if constexpr (FP4) {
        v8i_t a8 = {(int)w.x, (int)w.y, (int)w.z, (int)w.w, 0, 0, 0, 0};
        v8i_t b8 = {(int)x.x, (int)x.y, (int)x.z, (int)x.w, 0, 0, 0, 0};
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, acc, 4, 4, OPSEL, sw, OPSEL, sx);
    } else {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf_t, w), __builtin_bit_cast(v8bf_t, x), acc, 0, 0, 0);
    }
}

// two floats -> two BF16 (nearest even) in one dword, first in the low half
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf2;
    bf2 v = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, v);
}

// Weight row (within the expert) of row `br` of the block's weight tile.
template <bool GATEUP, int GC>
__device__ __forceinline__ int w_tile_row(int br, int n0, int I_up) {
    if constexpr (GATEUP) return br < GC ? n0 + br : I_up + n0 + (br - GC);
    else return n0 + br;
}

// LDS slot of weight-tile row br: inside each group of 32 rows, row 16h + 4g + q sits in slot
// 8g + 4h + q.  MFMA output row i = 8g + 4h + q lands in lane half h, register 4g + q, so the
// lane's 16 registers are weight rows 16h .. 16h+15 of the tile, in order.
__device__ __forceinline__ int w_slot(int br) { return (br & ~31) | (((br >> 2) & 3) << 3) | (((br >> 4) & 1) << 2) | (br & 3); }
// inverse: the weight-tile row that lane li (slot li) feeds to the MFMA
__device__ __forceinline__ int w_row_of_lane(int li) { return (((li >> 2) & 1) << 4) | ((li >> 3) << 2) | (li & 3); }

struct TileInfo {
    int e;        // local expert
    int row0;     // first activation row of the tile
    int seg_hi;   // end of the expert's row segment
    int n0;       // first output column of the tile
};

// Tile index -> (expert, row tile, column tile); column tiles are the fast index.
__device__ __forceinline__ TileInfo decode_tile(const GemmParams& p, int tile, int cols_per_tile) {
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
    return TileInfo{e, seg_lo + mi * BM, seg_hi, nt * cols_per_tile};
}

// BF16 outputs larger than what the memory-side cache would keep for the kernel that reads them next are
// streamed past it with non-temporal stores (uniform per launch).
__device__ __forceinline__ bool stream_output(const GemmParams& p) {
    const long long rows = __builtin_amdgcn_readfirstlane(p.offs[p.n_local]);
    return rows * p.n_out * 2 > (160ll << 20);
}

// Stores a 32-row x 32-column BF16 tile held as "lane (li, half) owns 16 consecutive columns of row li"
// (c0 = its first 8 columns, c1 = the next 8).  Writing it as held would touch 32 rows with two
// separate 16-byte pieces per instruction; a CU sustains only ~16 B/clk of such stores.  Neighbouring
// lanes therefore swap halves (DPP quad permute), so that one instruction writes the even rows and the
// next the odd rows, four lanes covering 64 contiguous bytes of a row: 16 rows per instruction, ~3x the
// store rate measured.  `base` points at column 0 of tile row 0; rows >= rows_left are not written.
// NT: non-temporal stores.  They drain faster, but the output then bypasses the memory-side cache, from
// which the next kernel would otherwise read it back: worth it only for outputs too large to stay there.
// Prepares the two store registers of store_tile_rows: ra = this lane's 16-byte piece of the even row of its
// pair, rb = of the odd row.
__device__ __forceinline__ void swap_halves(int lane, const u32x4_t& c0, const u32x4_t& c1, u32x4_t& ra, u32x4_t& rb) {
    const bool odd = lane & 1;
    const uint32_t a0[4] = {c0.x, c0.y, c0.z, c0.w}, a1[4] = {c1.x, c1.y, c1.z, c1.w};
    uint32_t xa[4], xb[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t n0 = (uint32_t)__builtin_amdgcn_mov_dpp((int)a0[d], 0xB1, 0xF, 0xF, true);   // the pair neighbour's c0
        const uint32_t n1 = (uint32_t)__builtin_amdgcn_mov_dpp((int)a1[d], 0xB1, 0xF, 0xF, true);   //                      c1
        xa[d] = odd ? n1 : a0[d];          // even row of the pair: even lane gives its c0, odd lane the even lane's c1
        xb[d] = odd ? a1[d] : n0;          // odd row of the pair:  even lane gives the odd lane's c0, odd lane its c1
    }
    ra = u32x4_t{xa[0], xa[1], xa[2], xa[3]};
    rb = u32x4_t{xb[0], xb[1], xb[2], xb[3]};
}
template <bool NT>
__device__ __forceinline__ void store16(uint8_t* dst, const u32x4_t& v, bool on) {
    if constexpr (NT) {
        if (on) __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t*>(dst));
    } else {
        if (on) *reinterpret_cast<u32x4_t*>(dst) = v;
    }
}
template <bool NT>
__device__ __forceinline__ void store_tile_rows(uint8_t* base, size_t row_pitch, int lane, int rows_left,
                                                const u32x4_t& c0, const u32x4_t& c1) {
    const int li = lane & 31, half = lane >> 5;
    u32x4_t ra, rb;
    swap_halves(lane, c0, c1, ra, rb);
    const int row_a = li & ~1;
    uint8_t* dst = base + (size_t)row_a * row_pitch + (half * 2 + (lane & 1)) * 16;
    store16<NT>(dst, ra, row_a < rows_left);
    store16<NT>(dst + row_pitch, rb, row_a + 1 < rows_left);
}
// Two neighbouring 32-column tiles of the same 32 rows (128 contiguous bytes per row).  The two 64-byte halves of
// a row's line are written by consecutive instructions, so that they reach the memory side together (streamed
// stores of half lines that arrive far apart cost extra write traffic).
template <bool NT>
__device__ __forceinline__ void store_tile_pair(uint8_t* base, size_t row_pitch, int lane, int rows_left, const u32x4_t& p0,
                                                const u32x4_t& p1, const u32x4_t& q0, const u32x4_t& q1) {
    const int li = lane & 31, half = lane >> 5;
    u32x4_t pa, pb, qa, qb;
    swap_halves(lane, p0, p1, pa, pb);
    swap_halves(lane, q0, q1, qa, qb);
    const int row_a = li & ~1;
    uint8_t* dst = base + (size_t)row_a * row_pitch + (half * 2 + (lane & 1)) * 16;
    store16<NT>(dst, pa, row_a < rows_left);
    store16<NT>(dst + 64, qa, row_a < rows_left);
    store16<NT>(dst + row_pitch, pb, row_a + 1 < rows_left);
    store16<NT>(dst + row_pitch + 64, qb, row_a + 1 < rows_left);
}

// Epilogue of one 32-row tile of a wave (row tile `mt` of its four), straight from registers.  a[t][r] belongs to
// activation row wm*128 + mt*32 + li of the block tile and to column 16*half + r of the wave's t-th 32-column tile.
// rows_valid = rows of the block tile that exist (may exceed the tile height).
template <bool FP4, bool GATEUP, int WN, bool NT>
__device__ __forceinline__ void epilogue_mt(const GemmParams& p, v16f_t (&a)[WN], int mt, int row0, int rows_valid, int n0,
                                            int wm, int wn, int li, int half) {
    const int lane = half * 32 + li;
    const int tile_row0 = wm * 128 + mt * 32;
    if constexpr (GATEUP) {
        constexpr int HT = WN / 2;                     // h column tiles per wave
        const int m = tile_row0 + li;
        const bool valid = m < rows_valid;
        const size_t grow = (size_t)(row0 + m);
#pragma unroll
        for (int t = 0; t < HT; ++t) {
            const int ctile = n0 + wn * HT * 32 + t * 32;  // first h column of the 32-column tile
            uint32_t hb[8];                                // 16 BF16 values: columns ctile + 16*half + 0..15
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const float g0 = a[t][2 * q], u0 = a[t + HT][2 * q];
                const float g1 = a[t][2 * q + 1], u1 = a[t + HT][2 * q + 1];
                hb[q] = pack_bf16x2(g0 * u0 * __builtin_amdgcn_rcpf(1.0f + __expf(-g0)),
                                    g1 * u1 * __builtin_amdgcn_rcpf(1.0f + __expf(-g1)));
            }
            if constexpr (FP4) {
                const u32x4_t v0 = {hb[0], hb[1], hb[2], hb[3]}, v1 = {hb[4], hb[5], hb[6], hb[7]};
                uint32_t amax = max(amax_bits8(v0), amax_bits8(v1));
                // the block's other 16 columns sit in lane^32: swapping the upper half of one copy with the lower half of
                // another leaves {lo, lo} and {hi, hi}, whose maximum is the pair's -- one VALU instruction, no LDS round trip
                const auto halves = __builtin_amdgcn_permlane32_swap(amax, amax, false, false);
                amax = max(halves[0], halves[1]);
                const uint32_t byte = e8m0_from_amax(amax);
                const float scl = scale_operand(byte);
                const u32x2_t codes = {encode8(v0, scl), encode8(v1, scl)};
                if (valid) {
                    *reinterpret_cast<u32x2_t*>(p.out + grow * (size_t)(p.n_out >> 1) + (ctile >> 1) + half * 8) = codes;
                    if (half == 0) p.outs[scale_byte_offset((long long)grow, ctile >> 5, p.n_out >> 7)] = (uint8_t)byte;
                }
            } else {
                store_tile_rows<NT>(p.out + ((size_t)(row0 + tile_row0) * p.n_out + ctile) * 2, (size_t)p.n_out * 2, lane,
                                    rows_valid - tile_row0, u32x4_t{hb[0], hb[1], hb[2], hb[3]}, u32x4_t{hb[4], hb[5], hb[6], hb[7]});
            }
        }
    } else {
        auto lo8 = [&](int t) __attribute__((always_inline)) {
            return u32x4_t{pack_bf16x2(a[t][0], a[t][1]), pack_bf16x2(a[t][2], a[t][3]),
                           pack_bf16x2(a[t][4], a[t][5]), pack_bf16x2(a[t][6], a[t][7])};
        };
        auto hi8 = [&](int t) __attribute__((always_inline)) {
            return u32x4_t{pack_bf16x2(a[t][8], a[t][9]), pack_bf16x2(a[t][10], a[t][11]),
                           pack_bf16x2(a[t][12], a[t][13]), pack_bf16x2(a[t][14], a[t][15])};
        };
        static_assert(WN % 2 == 0, "column tiles are stored in pairs");
#pragma unroll
        for (int t = 0; t < WN; t += 2) {
            const int col0 = n0 + wn * WN * 32 + t * 32;
            store_tile_pair<NT>(p.out + ((size_t)(row0 + tile_row0) * p.n_out + col0) * 2, (size_t)p.n_out * 2, lane,
                                rows_valid - tile_row0, lo8(t), hi8(t), lo8(t + 1), hi8(t + 1));
        }
    }
}

// Epilogue of a wave's whole 128-row tile.
template <bool FP4, bool GATEUP, int WN, bool NT>
__device__ __forceinline__ void epilogue(const GemmParams& p, v16f_t (&acc)[4][WN], int row0, int rows_valid, int n0,
                                         int wm, int wn, int li, int half) {
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) epilogue_mt<FP4, GATEUP, WN, NT>(p, acc[mt], mt, row0, rows_valid, n0, wm, wn, li, half);
}

// Persistent blocks of an XCD that take tiles: the fewest that finish the XCD's per_xcd tiles in as many rounds as all the
// launched ones would; the others exit at once.  A partly filled last round takes as long as a full one, so the idle
// blocks gain nothing -- and compute units left entirely free make the working ones faster (config 2, 1595 and 1160
// tiles: 29 instead of 32 blocks per XCD, both GEMMs 3.8 % faster; fewer active CUs share the power budget and the
// memory system), besides leaving room for whatever runs beside the GEMM.  FP4 only: the BF16 GEMMs move four times the
// bytes, their partly filled last round IS shorter (fewer blocks share the bandwidth), and they measured 1.2 % slower so.
__device__ __forceinline__ int working_slots(int per_xcd, int launched) {
    if (per_xcd <= 0) return 0;
    const int rounds = (per_xcd + launched - 1) / launched;
    return (per_xcd + rounds - 1) / rounds;
}

// Blocks b, b+8, b+16, .. share an XCD (and its L2), so each XCD takes a contiguous range of tiles
// (consecutive row tiles over all column tiles).  BF16: persistent blocks, one per residency slot,
// walk their XCD's range with a stride, and while a tile's epilogue runs the first K-step of the
// block's next tile is already in flight.  FP4: one tile per block (grid = worst-case tile count).
template <bool FP4, bool GATEUP, int WN, int WGN, int MINB>
__global__ void __launch_bounds__(128 * WGN, MINB) ffn_gemm_kernel(const GemmParams p) {
    using G = Geo<WN, WGN>;
    constexpr int NT = G::NT;
    constexpr int COLS = GATEUP ? G::GC : G::BNW;
    constexpr bool PERSIST = !FP4;    // the FP4 body has no registers to spare for a tile carried across the epilogue
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int li = lane & 31, half = lane >> 5;

    int total_m = 0;
    for (int e = 0; e < p.n_local; ++e) total_m += (p.offs[e + 1] - p.offs[e] + BM - 1) / BM;
    const int total = total_m * p.n_tiles_n;
    const int per_xcd = (total + 7) >> 3;
    const int nslots = FP4 ? working_slots(per_xcd, (int)(gridDim.x >> 3)) : (int)(gridDim.x >> 3);
    if ((int)(blockIdx.x >> 3) >= nslots) return;
    const int tile_hi = min(total, ((int)(blockIdx.x & 7) + 1) * per_xcd);
    int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (tile >= tile_hi) return;
    const bool nt_out = stream_output(p);

    const int I_up = p.w_rows >> 1;                       // gate/up: offset of the up rows
    const size_t rowbytes = FP4 ? (size_t)(p.K >> 1) : (size_t)p.K * 2;
    const int nks = (int)(rowbytes / KSTEP_BYTES);
    const int kd = p.K >> 7;                              // FP4: K-steps = scale dwords per row
    const uint32_t* As32 = reinterpret_cast<const uint32_t*>(p.As);
    const uint32_t* Ws32 = reinterpret_cast<const uint32_t*>(p.Ws);

    // ---- tile-independent: LDS destinations of this thread's 16-byte chunks (4 per 64-byte row
    //      segment) and the fragment / scale addresses of this lane
    const int part = tid & 3;
    int a_dst[G::JA], b_dst[G::JB];
#pragma unroll
    for (int j = 0; j < G::JA; ++j) a_dst[j] = part * G::SUB_A + ((tid >> 2) + (NT / 4) * j) * 16;
#pragma unroll
    for (int j = 0; j < G::JB; ++j) b_dst[j] = G::REGION_A + part * G::SUB_B + w_slot((tid >> 2) + (NT / 4) * j) * 16;
    int b_rows[WN];                                       // first weight-tile row of each of this wave's column tiles
#pragma unroll
    for (int t = 0; t < WN; ++t) {
        if constexpr (GATEUP) b_rows[t] = (t < WN / 2 ? 0 : G::GC) + wn * (WN / 2) * 32 + (t % (WN / 2)) * 32;
        else b_rows[t] = wn * WN * 32 + t * 32;
    }
    const int a_frag = half * G::SUB_A + (wm * 128 + li) * 16;                 // + mt*512 + slice*2*SUB_A
    int b_frag[WN];
#pragma unroll
    for (int t = 0; t < WN; ++t) b_frag[t] = G::REGION_A + half * G::SUB_B + (b_rows[t] + li) * 16;   // + slice*2*SUB_B
    const int sshift = half * 8;

    // ---- per-tile prefetch state: source pointers and the first K-step
    const uint8_t* a_src[G::JA];
    const uint8_t* b_src[G::JB];
    u32x4_t ga[G::JA], gb[G::JB];
    // FP4: dword index (K-step 0) of this lane's scale words in the K-step-tiled scale tensors; a
    // wave's 32 rows at one K-step are one contiguous 128-byte line (two when the rows straddle
    // a group of 32), so the scales go from memory to the MFMA operand registers directly.
    int sa_off[4], sb_off[WN];
    uint32_t sa_nx[4], sb_nx[WN];                         // scale words of the next K-step
    TileInfo ti = decode_tile(p, tile, COLS);

    auto prefetch_tile = [&](const TileInfo& t) {
#pragma unroll
        for (int j = 0; j < G::JA; ++j) {
            const int gr = min(t.row0 + (tid >> 2) + (NT / 4) * j, t.seg_hi - 1);
            a_src[j] = p.A + (size_t)gr * rowbytes + part * 16;
        }
#pragma unroll
        for (int j = 0; j < G::JB; ++j) {
            const int br = (tid >> 2) + (NT / 4) * j;
            b_src[j] = p.W + ((size_t)t.e * p.w_rows + w_tile_row<GATEUP, G::GC>(br, t.n0, I_up)) * rowbytes + part * 16;
        }
#pragma unroll
        for (int j = 0; j < G::JA; ++j) ga[j] = *reinterpret_cast<const u32x4_t*>(a_src[j]);
#pragma unroll
        for (int j = 0; j < G::JB; ++j) gb[j] = *reinterpret_cast<const u32x4_t*>(b_src[j]);
        if constexpr (FP4) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
                const int row = min(t.row0 + wm * 128 + mt * 32 + li, t.seg_hi - 1);
                sa_off[mt] = ((row >> 5) * kd) * 32 + (row & 31);
                sa_nx[mt] = As32[sa_off[mt]];
            }
#pragma unroll
            for (int c = 0; c < WN; ++c) {
                const int wrow = t.e * p.w_rows + w_tile_row<GATEUP, G::GC>(b_rows[c] + w_row_of_lane(li), t.n0, I_up);
                sb_off[c] = ((wrow >> 5) * kd) * 32 + (wrow & 31);
                sb_nx[c] = Ws32[sb_off[c]];
            }
        }
    };
    prefetch_tile(ti);

    while (true) {
        // ---- scales and the prefetched first K-step go to LDS, K-step 1 starts
#pragma unroll
        for (int j = 0; j < G::JA; ++j) *reinterpret_cast<u32x4_t*>(smem + a_dst[j]) = ga[j];
#pragma unroll
        for (int j = 0; j < G::JB; ++j) *reinterpret_cast<u32x4_t*>(smem + b_dst[j]) = gb[j];
        if (nks > 1) {
#pragma unroll
            for (int j = 0; j < G::JA; ++j) ga[j] = *reinterpret_cast<const u32x4_t*>(a_src[j] + KSTEP_BYTES);
#pragma unroll
            for (int j = 0; j < G::JB; ++j) gb[j] = *reinterpret_cast<const u32x4_t*>(b_src[j] + KSTEP_BYTES);
        }
        __syncthreads();

        v16f_t acc[4][WN];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < WN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

        // ---- main loop: LDS holds K-step ks (double buffered), registers hold K-step ks+1,
        //      whose global loads were issued a whole iteration earlier.
        for (int ks = 0; ks < nks; ++ks) {
            const uint8_t* st = smem + (ks & 1) * G::STAGE;
            int sa[4] = {0, 0, 0, 0}, sb[WN];
#pragma unroll
            for (int t = 0; t < WN; ++t) sb[t] = 0;
            if constexpr (FP4) {
#pragma unroll
                for (int mt = 0; mt < 4; ++mt) sa[mt] = (int)(sa_nx[mt] >> sshift);
#pragma unroll
                for (int t = 0; t < WN; ++t) sb[t] = (int)(sb_nx[t] >> sshift);
                if (ks + 1 < nks) {
#pragma unroll
                    for (int mt = 0; mt < 4; ++mt) sa_nx[mt] = As32[sa_off[mt] + (ks + 1) * 32];
#pragma unroll
                    for (int t = 0; t < WN; ++t) sb_nx[t] = Ws32[sb_off[t] + (ks + 1) * 32];
                }
            }
            u32x4_t fa0[4], fb0[WN], fa1[4], fb1[WN];
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) fa0[mt] = *reinterpret_cast<const u32x4_t*>(st + a_frag + mt * 512);
#pragma unroll
            for (int t = 0; t < WN; ++t) fb0[t] = *reinterpret_cast<const u32x4_t*>(st + b_frag[t]);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) fa1[mt] = *reinterpret_cast<const u32x4_t*>(st + 2 * G::SUB_A + a_frag + mt * 512);
#pragma unroll
            for (int t = 0; t < WN; ++t) fb1[t] = *reinterpret_cast<const u32x4_t*>(st + 2 * G::SUB_B + b_frag[t]);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)                   // K-slice 0: scale bytes 0/1 of the K-step's dword
#pragma unroll
                for (int t = 0; t < WN; ++t) mma<FP4, 0>(acc[mt][t], fb0[t], fa0[mt], sb[t], sa[mt]);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)                   // K-slice 1: scale bytes 2/3
#pragma unroll
                for (int t = 0; t < WN; ++t) mma<FP4, 2>(acc[mt][t], fb1[t], fa1[mt], sb[t], sa[mt]);
            __builtin_amdgcn_sched_barrier(0);
            if (ks + 1 < nks) {
                uint8_t* nx = smem + ((ks + 1) & 1) * G::STAGE;
#pragma unroll
                for (int j = 0; j < G::JA; ++j) *reinterpret_cast<u32x4_t*>(nx + a_dst[j]) = ga[j];
#pragma unroll
                for (int j = 0; j < G::JB; ++j) *reinterpret_cast<u32x4_t*>(nx + b_dst[j]) = gb[j];
            }
            __builtin_amdgcn_sched_barrier(0);
            if (ks + 2 < nks) {
#pragma unroll
                for (int j = 0; j < G::JA; ++j) ga[j] = *reinterpret_cast<const u32x4_t*>(a_src[j] + (size_t)(ks + 2) * KSTEP_BYTES);
#pragma unroll
                for (int j = 0; j < G::JB; ++j) gb[j] = *reinterpret_cast<const u32x4_t*>(b_src[j] + (size_t)(ks + 2) * KSTEP_BYTES);
            }
            __syncthreads();
        }

        // ---- the block's next tile: get its first K-step moving before the epilogue
        const TileInfo cur = ti;
        const bool more = PERSIST && tile + nslots < tile_hi;
        if (more) {
            tile += nslots;
            ti = decode_tile(p, tile, COLS);
            prefetch_tile(ti);
        }

        // ---- epilogue, straight from registers
        if (nt_out) epilogue<FP4, GATEUP, WN, true>(p, acc, cur.row0, cur.seg_hi - cur.row0, cur.n0, wm, wn, li, half);
        else epilogue<FP4, GATEUP, WN, false>(p, acc, cur.row0, cur.seg_hi - cur.row0, cur.n0, wm, wn, li, half);
        if (!more) break;
    }
}

// ---------------------------------------------------------------------------------------------
// 256 x 256 tile kernel with direct-to-LDS loads (the default where the output width allows).
//
// What bounds the grouped GEMM on this chip is the path from L2 into the CU, not the MFMA rate:
// a CU takes in about one 1-KB vector-memory instruction per 18-26 cycles, and the vector L1
// fetches whole 128-byte lines.  So this kernel
//   - fetches 128 bytes of every operand row per K-step (a full line: 256 FP4 or 64 BF16 values,
//     four MFMA K-slices), which halves the L2->L1 traffic of 64-byte steps;
//   - uses a 256 x 256 block tile (8 waves of 128 x 64), the largest whose two 64-KB stages fit the
//     160 KB of LDS, to minimise bytes fetched per MFMA;
//   - loads with global_load_lds_dwordx4 (memory -> LDS without passing through registers): a wave
//     instruction carries 8 rows x 128 B and lands as 1 KB of contiguous LDS.  Inside a 128-byte LDS
//     row the eight 16-byte parts are XOR-swizzled by (row>>1)&7 (done on the global address of
//     each lane, since the LDS side of the transfer is fixed), which makes the 32-row x 16-byte
//     fragment reads bank-conflict free;
//   - spreads the transfer instructions between MFMAs (a wave blocks while the memory pipeline accepts
//     an instruction, and eight waves issuing at once stall all MFMA issue) and keeps the producer a
//     whole K-step ahead, so that no transfer is waited for;
//   - is persistent: a block walks its XCD's tile range and its producer runs across tile boundaries
//     (the expert table sits in LDS, so switching tiles touches no global memory); only the
//     register-only epilogue sits between two tiles' MFMA streams;
//   - FP4: stages the E8M0 scales through LDS as well (global_load_lds_dword, 32 rows x 2 dwords
//     per instruction), because one vector-memory instruction per lane-dword costs as much issue
//     time as a 1-KB one.
// The accumulation order along K is that of the other kernel, so results are bit-identical.
namespace t256 {
constexpr int KB = 128;                    // bytes of each operand row per K-step
constexpr int REGION_W = 256 * KB;         // weight rows follow the 256 activation rows
constexpr int STAGE = 512 * KB;            // 64 KB
constexpr int SC_BASE = 2 * STAGE;         // FP4: scale staging, per stage [512 rows][2 dwords]
constexpr int SC_STAGE = 512 * 8;
constexpr int SC_W = 256 * 8;
constexpr int TAB_BASE = SC_BASE + 2 * SC_STAGE;   // expert table, 3 x 64 ints
constexpr int TOK_BASE = TAB_BASE + 3 * 64 * 4;    // gathering kernel: row_to_assign entries of a tile, two buffers x 8 waves x 64 ints
constexpr int TOK_BUF = 8 * 64 * 4;
constexpr int LDS_BYTES = TOK_BASE + 2 * TOK_BUF;
}  // namespace t256

__device__ __forceinline__ void lds_dma16(const uint8_t* g, uint8_t* l) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                     (__attribute__((address_space(3))) void*)l, 16, 0, 0);
}
__device__ __forceinline__ void lds_dma4(const uint32_t* g, uint8_t* l) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                     (__attribute__((address_space(3))) void*)l, 4, 0, 0);
}

// GATHER (gate/up only): the activation rows are fetched straight from a token-indexed matrix (x itself,
// or the tokens' FP4 codes and scales) through row_to_assign, so no permuted copy has to be written.
template <bool FP4, bool GATEUP, bool GATHER = false>
__global__ void __launch_bounds__(512, 1) ffn_gemm256_kernel(const GemmParams p) {
    using namespace t256;
    constexpr int COLS = GATEUP ? 128 : 256;   // output columns per block
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int li = lane & 31, half = lane >> 5;

    // Expert table in LDS: entry e holds expert e's row segment and the inclusive prefix of row-tile
    // counts (entries up to 63 repeat the total), so that decoding a tile index is one LDS read per
    // lane, a ballot and three broadcast reads -- no global memory access between tiles.
    int* tab = reinterpret_cast<int*>(smem + TAB_BASE);    // [0,64) prefix, [64,128) segment start, [128,192) segment end
    int total_m;
    {
        int off_lo = 0, off_hi = 0;
        if (lane < p.n_local) { off_lo = p.offs[lane]; off_hi = p.offs[lane + 1]; }
        int cum = (off_hi - off_lo + BM - 1) / BM;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int o = __shfl_up(cum, d);
            if (lane >= d) cum += o;
        }
        total_m = __builtin_amdgcn_readlane(cum, 63);
        if (wave == 0) { tab[lane] = cum; tab[64 + lane] = off_lo; tab[128 + lane] = off_hi; }
        __syncthreads();
    }
    const int total = total_m * p.n_tiles_n;
    auto decode = [&](int t) __attribute__((always_inline)) {
        const int mi = t / p.n_tiles_n, nt = t - mi * p.n_tiles_n;
        const int e = __builtin_amdgcn_readfirstlane(__popcll(__ballot(tab[lane] <= mi)));   // experts that end at or before row tile mi
        const int lo = __builtin_amdgcn_readfirstlane(tab[64 + e]), hi = __builtin_amdgcn_readfirstlane(tab[128 + e]);
        const int first = e == 0 ? 0 : __builtin_amdgcn_readfirstlane(tab[e - 1]);
        return TileInfo{e, lo + (mi - first) * BM, hi, nt * COLS};
    };
    const int per_xcd = (total + 7) >> 3;
    const int nslots = FP4 ? working_slots(per_xcd, (int)(gridDim.x >> 3)) : (int)(gridDim.x >> 3);
    if ((int)(blockIdx.x >> 3) >= nslots) return;
    const int tile_hi = min(total, ((int)(blockIdx.x & 7) + 1) * per_xcd);
    int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (tile >= tile_hi) return;

    const bool nt_out = stream_output(p);
    const int I_up = p.w_rows >> 1;
    const uint32_t rowbytes = FP4 ? (uint32_t)(p.K >> 1) : (uint32_t)p.K * 2;
    const int nks = (int)((rowbytes + KB - 1) / KB);
    // last K-step holds 64 bytes per row: FP4 rows only (K is a multiple of 128 values, so a BF16 row is whole K-steps)
    const bool tail_half = FP4 && (rowbytes % KB) != 0;
    const int kd = p.K >> 7;                              // FP4: scale dwords per row

    // ---- consumer side: fragment offsets inside a stage
    const int sw = (li >> 1) & 7;
    const int f_off0 = li * KB + ((half ^ sw) << 4);       // slice s reads part 2s+half: offset f_off0 ^ (s << 5)
    const int a_base = wm * 128 * KB;
    int b_pos[2];                                         // first LDS weight position of the wave's two column tiles
    if constexpr (GATEUP) { b_pos[0] = wn * 32; b_pos[1] = 128 + wn * 32; }
    else { b_pos[0] = wn * 64; b_pos[1] = wn * 64 + 32; }

    // ---- producer side: this wave moves activation rows and weight positions 32*wave .. 32*wave+31
    //      (four instructions of 8 rows each) and the scale dwords of the same rows.  Addresses are a
    //      per-tile scalar base plus a 32-bit per-lane offset.
    const int prow = lane >> 3;                           // row inside an 8-row instruction
    // 16-byte part a lane fetches in instruction j: (lane&7) ^ key, key = (R>>1)&7 = (4*(j&1) + (lane>>4)) & 7
    // for LDS row R = 32*wave + 8*j + prow of the instruction.
    auto part16 = [&](int q) __attribute__((always_inline)) { return (uint32_t)(((lane & 7) ^ ((q * 4 + (lane >> 4)) & 7)) << 4); };
    // Weights: LDS position R holds weight-tile row (R & ~31) | w_row_of_lane(R & 31), which for
    // R & 31 = 8*j + prow is 16*((prow>>2)&1) + 4*j + (prow&3): instruction j is 4*j rows below
    // instruction 0, a scalar offset.  Per lane only the two part offsets differ (by parity of j).
    uint32_t b_voff[2];
    {
        const int br0 = wave * 32 + (((prow >> 2) & 1) << 4) + (prow & 3);
#pragma unroll
        for (int q = 0; q < 2; ++q) b_voff[q] = (uint32_t)w_tile_row<GATEUP, 128>(br0, 0, I_up) * rowbytes + part16(q);
    }
    int a_last = 0;                                       // scalar: last existing row of the tile being fetched
    uint32_t a_goff[GATHER ? 4 : 1];                      // GATHER: byte offset of this lane's source row, per instruction
    const int srow = wave * 32 + (lane >> 1), swhich = lane & 1;
    int sa_idx = 0, sb_idx = 0;                           // FP4: dword index of this lane's scale word, K-step 0
    const uint8_t* a_tile = nullptr;                      // scalar: first activation row / weight row of the tile being fetched
    const uint8_t* b_tile = nullptr;

    TileInfo ti = decode(tile);
    // GATHER: the row_to_assign entries of a tile's rows are brought into LDS one tile ahead (a wave fetches the
    // entries of its own 32 rows with one direct-to-LDS transfer and later reads back only what it fetched), so
    // that switching tiles never waits for global memory: a register load at the switch would stall the producer
    // for a full memory latency, behind every transfer in flight.
    int tokbuf = 0;
    auto fetch_tokens = [&](const TileInfo& t, int buf) __attribute__((always_inline)) {
        if constexpr (GATHER) {
            const int row0 = __builtin_amdgcn_readfirstlane(t.row0), rows = __builtin_amdgcn_readfirstlane(t.seg_hi - t.row0);
            const int r = row0 + min(wave * 32 + (lane & 31), rows - 1);          // rows past the segment: its last row again
            lds_dma4(reinterpret_cast<const uint32_t*>(p.row_src) + r, smem + TOK_BASE + buf * TOK_BUF + wave * 256);
        }
    };
    auto setup_src = [&](const TileInfo& t) __attribute__((always_inline)) {
        const int row0 = __builtin_amdgcn_readfirstlane(t.row0), rows = __builtin_amdgcn_readfirstlane(t.seg_hi - t.row0);
        const int e = __builtin_amdgcn_readfirstlane(t.e), n0 = __builtin_amdgcn_readfirstlane(t.n0);
        a_tile = GATHER ? p.A : p.A + (size_t)row0 * rowbytes;
        b_tile = p.W + ((size_t)e * p.w_rows + n0) * rowbytes;
        a_last = rows - 1;
        const int* toks = reinterpret_cast<const int*>(smem + TOK_BASE + tokbuf * TOK_BUF) + wave * 64;   // this tile's entries (GATHER)
        if constexpr (GATHER) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                a_goff[j] = (uint32_t)div_by_magic(toks[j * 8 + prow], p.src_magic, p.src_shift) * rowbytes + part16(j & 1);
        }
        if constexpr (FP4) {
            int gr = row0 + min(srow, rows - 1);
            if constexpr (GATHER) gr = div_by_magic(toks[lane >> 1], p.src_magic, p.src_shift);   // the token that holds this row's codes and scales
            sa_idx = ((gr >> 5) * kd) * 32 + (gr & 31);
            const int br = (srow & ~31) | w_row_of_lane(srow & 31);
            const int wr = e * p.w_rows + w_tile_row<GATEUP, 128>(br, n0, I_up);
            sb_idx = ((wr >> 5) * kd) * 32 + (wr & 31);
        }
    };
    // One producer instruction of K-step k into stage `dstg`: op 0/1 = scales (FP4), 2..5 = activations, 6..9 = weights.
    auto issue = [&](int op, int k, int dstg) __attribute__((always_inline)) {
        if (op < 2) {
            if constexpr (FP4) {
                const int ko = min(2 * k + swhich, kd - 1) * 32;
                uint8_t* l = smem + SC_BASE + dstg * SC_STAGE + wave * 256;
                if (op == 0) lds_dma4(reinterpret_cast<const uint32_t*>(p.As) + (uint32_t)(sa_idx + ko), l);
                else lds_dma4(reinterpret_cast<const uint32_t*>(p.Ws) + (uint32_t)(sb_idx + ko), l + SC_W);
            }
        } else {
            const int j = (op - 2) & 3;
            const bool halfstep = tail_half && k == nks - 1;
            // half step: lanes of parts 4..7 fetch parts 0..3 again (the row has only 64 bytes left)
            const uint32_t koff = (uint32_t)(k * KB) - (halfstep ? (uint32_t)(((lane << 4) ^ ((j & 1) << 6)) & 64) : 0u);
            uint8_t* l = smem + dstg * STAGE + (wave * 4 + j) * 1024;
            if (op < 6) {
                uint32_t v;
                if constexpr (GATHER) v = a_goff[j];
                else v = (uint32_t)min(wave * 32 + j * 8 + prow, a_last) * rowbytes + part16(j & 1);   // rows past the segment: its last row again
                lds_dma16(a_tile + (v + koff), l);
            } else {
                lds_dma16(b_tile + (size_t)(j * 4) * rowbytes + (b_voff[j & 1] + koff), l + REGION_W);
            }
        }
    };

    // ---- producer position: the K-step it fetches next (pk of tile ptile).  Past the block's last tile
    //      it keeps refetching that tile's steps, which nobody reads.
    int ptile = tile, pk = 0;
    auto advance = [&]() __attribute__((always_inline)) {
        if (++pk == nks) {
            pk = 0;
            if (ptile + nslots < tile_hi) {
                ptile += nslots;
                if constexpr (GATHER) tokbuf ^= 1;                     // fetched while the previous tile was being produced
                setup_src(decode(ptile));
                if constexpr (GATHER) {
                    if (ptile + nslots < tile_hi) fetch_tokens(decode(ptile + nslots), tokbuf ^ 1);
                }
            }
        }
    };
    if constexpr (GATHER) {
        fetch_tokens(ti, 0);
        if (tile + nslots < tile_hi) fetch_tokens(decode(tile + nslots), 1);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    setup_src(ti);
#pragma unroll
    for (int op = 0; op < 10; ++op) issue(op, 0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    advance();
#pragma unroll
    for (int op = 2; op < 6; ++op) issue(op, pk, 1);      // first half of the second step (see below)

    // One flat loop over the (tile, K-step) pairs of this block, with a single copy of the K-step code:
    // the steps of a tile follow each other without a seam, and the producer runs ahead across tile
    // boundaries.  Inside a step the block barrier sits after the third K-slice: by then every wave
    // holds its fourth slice in registers, so the stage is free, and behind the barrier
    //   - the first fragments and the scales of the NEXT step are read while the fourth slice
    //     multiplies (no LDS latency is exposed at the start of a step), and
    //   - the producer starts on the step AFTER the next one: its activation rows go out between the
    //     MFMAs of the fourth slice, its weight rows and scales between those of the next step's first
    //     slice, so every transfer has a whole step to land before the barrier that publishes it.
    int stg = 0, ks = 0;
    v16f_t acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    int cur_row0 = ti.row0, cur_rows = ti.seg_hi - ti.row0, cur_n0 = ti.n0;

    u32x4_t fa[2][4], fb[2][2];                           // fragment double buffer (slice parity)
    int sa[4][2], sb[2][2];                               // FP4: scale words of the step, [.][0] slices 0-1, [.][1] slices 2-3
    auto read_frags = [&](int s, int slot, const uint8_t* st) __attribute__((always_inline)) {
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) fa[slot][mt] = *reinterpret_cast<const u32x4_t*>(st + a_base + mt * 32 * KB + (f_off0 ^ (s << 5)));
#pragma unroll
        for (int t = 0; t < 2; ++t) fb[slot][t] = *reinterpret_cast<const u32x4_t*>(st + REGION_W + b_pos[t] * KB + (f_off0 ^ (s << 5)));
    };
    // the same reads in four parts (part 0: row tile 0 and both column tiles, part 1: row tile 1, ...)
    auto read_frags_part = [&](int part, int s, int slot, const uint8_t* st) __attribute__((always_inline)) {
        fa[slot][part] = *reinterpret_cast<const u32x4_t*>(st + a_base + part * 32 * KB + (f_off0 ^ (s << 5)));
        if (part == 0) {
#pragma unroll
            for (int t = 0; t < 2; ++t) fb[slot][t] = *reinterpret_cast<const u32x4_t*>(st + REGION_W + b_pos[t] * KB + (f_off0 ^ (s << 5)));
        }
    };
    u32x2_t ra[4], rb[2];                                 // FP4: raw scale words as read from LDS
    auto read_scales = [&](int stage) __attribute__((always_inline)) {
        if constexpr (FP4) {
            const uint8_t* sc = smem + SC_BASE + stage * SC_STAGE;
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) ra[mt] = *reinterpret_cast<const u32x2_t*>(sc + (wm * 128 + mt * 32 + li) * 8);
#pragma unroll
            for (int t = 0; t < 2; ++t) rb[t] = *reinterpret_cast<const u32x2_t*>(sc + SC_W + (b_pos[t] + li) * 8);
        }
    };
    auto read_scales_part = [&](int part, int stage) __attribute__((always_inline)) {   // the same in four parts, like the fragments
        if constexpr (FP4) {
            const uint8_t* sc = smem + SC_BASE + stage * SC_STAGE;
            ra[part] = *reinterpret_cast<const u32x2_t*>(sc + (wm * 128 + part * 32 + li) * 8);
            if (part == 0) {
#pragma unroll
                for (int t = 0; t < 2; ++t) rb[t] = *reinterpret_cast<const u32x2_t*>(sc + SC_W + (b_pos[t] + li) * 8);
            }
        }
    };
    auto take_scales = [&]() __attribute__((always_inline)) {     // this lane's byte pair of each word (op_sel picks the byte)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
            sa[mt][0] = FP4 ? (int)(ra[mt].x >> (half * 8)) : 0;
            sa[mt][1] = FP4 ? (int)(ra[mt].y >> (half * 8)) : 0;
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            sb[t][0] = FP4 ? (int)(rb[t].x >> (half * 8)) : 0;
            sb[t][1] = FP4 ? (int)(rb[t].y >> (half * 8)) : 0;
        }
    };
    read_scales(0);
    read_frags(0, 0, smem);
    take_scales();

    while (true) {
        const bool last = ks == nks - 1;
        const bool full = !(last && tail_half);           // all four K-slices present
        const uint8_t* st = smem + stg * STAGE;

        // MFMAs of slice s out of fragment slot s&1.  PRODUCE 1: after each row tile's MFMAs one weight
        // transfer (and the two scale transfers) of producer step pk into the other stage; PRODUCE 2:
        // one activation transfer of the producer's new step into the stage just released.
        // Slice s multiplies out of fragment slot s&1.  The fragments of the following slice (next = s+1,
        // or next = 4: the first slice of the next step, with its scales, out of the stage that has just
        // been published) are requested into the other slot, a quarter of them after each row tile's MFMAs
        // (one burst of six reads behind the first row tile measured 0.5-1 % slower: the LDS also takes
        // the transfers' writes); the wait in front of this slice's first MFMA does not cover the new requests.
        auto slice = [&](int s, int produce, bool multiply, int next) __attribute__((always_inline)) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
                if (multiply) {
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        if (s & 1) mma<FP4, 2>(acc[mt][t], fb[s & 1][t], fa[s & 1][mt], sb[t][s >> 1], sa[mt][s >> 1]);
                        else mma<FP4, 0>(acc[mt][t], fb[s & 1][t], fa[s & 1][mt], sb[t][s >> 1], sa[mt][s >> 1]);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                if (next >= 0) {
                    if (next < 4) read_frags_part(mt, next, next & 1, st);
                    else { read_scales_part(mt, stg); read_frags_part(mt, 0, 0, smem + stg * STAGE); }
                }
                if (produce == 1) {
                    if (FP4 && mt < 2) issue(mt, pk, stg ^ 1);
                    issue(6 + mt, pk, stg ^ 1);
                } else if (produce == 2) {
                    issue(2 + mt, pk, stg ^ 1);           // (stg already flipped: the stage this step has just left)
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        slice(0, 1, true, 1);
        slice(1, 0, true, 2);                             // (half step: slice 2 holds stale bytes that are never multiplied)
        if (full) slice(2, 0, true, 3);
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        stg ^= 1;
        advance();
        __builtin_amdgcn_sched_barrier(0);
        slice(3, 2, full, 4);                             // (half step: the producer's transfers and the requests only)
        __builtin_amdgcn_sched_barrier(0);
        take_scales();

        ++ks;
        if (last) {
            if (nt_out) epilogue<FP4, GATEUP, 2, true>(p, acc, cur_row0, cur_rows, cur_n0, wm, wn, li, half);
            else epilogue<FP4, GATEUP, 2, false>(p, acc, cur_row0, cur_rows, cur_n0, wm, wn, li, half);
            tile += nslots;
            if (tile >= tile_hi) break;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
            ti = decode(tile);
            cur_row0 = ti.row0; cur_rows = ti.seg_hi - ti.row0; cur_n0 = ti.n0;
            ks = 0;
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // no transfer may still be writing this block's LDS when it ends
}

template <bool FP4, bool GATEUP, bool GATHER = false>
static int launch_gemm256(GemmParams p, long long max_rows, const Ctx* c, hipStream_t s) {
    const int num_cus = c->num_cus;
    p.n_tiles_n = p.n_out / (GATEUP ? 128 : 256);
    const size_t lds = t256::LDS_BYTES;
    static std::atomic<unsigned long long> attr_seen{0};            // per instantiation, one bit per device
    if (first_use_on_device(attr_seen, c->device)) {                // (setting it twice from two threads is harmless)
        REALB_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&ffn_gemm256_kernel<FP4, GATEUP, GATHER>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        mark_used_on_device(attr_seen, c->device);
    }
    const long long m_tiles_max = (max_rows + BM - 1) / BM + p.n_local;
    const long long total_max = m_tiles_max * p.n_tiles_n;
    // one persistent block per CU, a multiple of 8 (XCDs); a prefetching layer call leaves some CUs to the weight encoder
    const long long avail = (long long)num_cus - c->gemm_reserve;
    const long long slots = avail >= 16 ? 8ll * (c->gemm_reserve > 0 ? avail / 8 : (avail + 7) / 8) : 8;
    const long long grid = total_max < slots ? 8 * ((total_max + 7) / 8) : slots;
    hipLaunchKernelGGL((ffn_gemm256_kernel<FP4, GATEUP, GATHER>), dim3((unsigned)grid), dim3(512), lds, s, p);
    REALB_HIP(hipGetLastError());
    return REALB_OK;
}

// Block tile choices (selector g_tile): 16 = the direct-to-LDS 256x256 kernel above (automatic choice
// where the output width is a multiple of its tile); the register-staged kernel with 64-byte K-steps
// as 2 = 256x128, 4 waves, two blocks per CU, or 8 = 256x256, 8 waves of 128x64, one block per CU.
template <bool FP4, bool GATEUP, int WN, int WGN, int MINB>
static int launch_gemm_geo(GemmParams p, long long max_rows, const Ctx* c, hipStream_t s) {
    using G = Geo<WN, WGN>;
    const int num_cus = c->num_cus;
    p.n_tiles_n = GATEUP ? p.n_out / G::GC : p.n_out / G::BNW;
    const size_t lds = 2 * (size_t)G::STAGE;
    const size_t lds_cap = MINB == 2 ? 80 * 1024 : 160 * 1024;
    static std::atomic<unsigned long long> attr_seen{0};            // per instantiation, one bit per device
    if (first_use_on_device(attr_seen, c->device)) {
        REALB_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&ffn_gemm_kernel<FP4, GATEUP, WN, WGN, MINB>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_cap));
        mark_used_on_device(attr_seen, c->device);
    }
    const long long m_tiles_max = (max_rows + BM - 1) / BM + p.n_local;
    const long long total_max = m_tiles_max * p.n_tiles_n;
    const long long slots = 8ll * (((long long)num_cus * MINB + 7) / 8);   // one block per residency slot, multiple of 8 (XCDs)
    const long long all_tiles = 8 * ((total_max + 7) / 8);
    const long long grid = (FP4 || total_max < slots) ? all_tiles : slots;                // FP4: one tile per block
    REALB_REQUIRE(grid < (1ll << 31), REALB_ECAP, "too many tiles");
    REALB_REQUIRE(lds <= lds_cap, REALB_ESHAPE, "K=%d needs %zu bytes of LDS", p.K, lds);
    hipLaunchKernelGGL((ffn_gemm_kernel<FP4, GATEUP, WN, WGN, MINB>), dim3((unsigned)grid), dim3(G::NT), lds, s, p);
    REALB_HIP(hipGetLastError());
    return REALB_OK;
}

static std::atomic<int> g_tile{0};    // 0 = automatic; 2, 8 or 16 forces a kernel (set through realb_set_gemm_tile)

template <bool FP4, bool GATEUP>
static int launch_gemm(const GemmParams& p, long long max_rows, const Ctx* c, hipStream_t s) {
    const int unit256 = GATEUP ? 128 : 256;             // output columns per block of the 256-wide tile
    const bool can256 = p.n_out % unit256 == 0;
    const int forced = g_tile.load(std::memory_order_relaxed);
    const int sel = !can256 ? 2 : (forced == 0 ? 16 : forced);
    if (sel == 16) return launch_gemm256<FP4, GATEUP>(p, max_rows, c, s);
    if (sel == 8) return launch_gemm_geo<FP4, GATEUP, 2, 4, 1>(p, max_rows, c, s);
    return launch_gemm_geo<FP4, GATEUP, 2, 2, 2>(p, max_rows, c, s);
}

// Whether the gathering gate/up GEMM below applies (kernel selection, 32-bit row offsets).
bool gate_up_gather_supported(const Ctx* c, int T, bool fp4) {
    const long long bytes = (long long)T * c->cfg.H * (fp4 ? 1 : 4) / 2;
    const int forced = g_tile.load(std::memory_order_relaxed);
    return (forced == 0 || forced == 16) && c->cfg.I % 128 == 0 && T > 0 && bytes < (1ll << 32);
}

// BF16 gate/up GEMM that gathers its activation rows from the token matrix x [T,H] through row_to_assign
// (the permutation's gather fused into the GEMM's loads).  Returns REALB_ESHAPE if this shape or the
// selected kernel cannot do it; the caller then materialises the permuted rows and uses the plain GEMM.
int launch_gate_up_bf16_gather(Ctx* c, const int32_t* expert_offsets, int n_local, long long max_rows, const void* x, int T,
                               const int32_t* row_to_assign, const void* w13, void* h_mid, hipStream_t s) {
    const int H = c->cfg.H, I = c->cfg.I;
    if (!gate_up_gather_supported(c, T, false)) return REALB_ESHAPE;
    GemmParams g{(const uint8_t*)x, nullptr, (const uint8_t*)w13, nullptr, (uint8_t*)h_mid, nullptr, expert_offsets, n_local,
                 H, 2 * I, I, 0, row_to_assign, 0, 0};
    division_magic(c->cfg.k, &g.src_magic, &g.src_shift);
    return launch_gemm256<false, true, true>(g, max_rows, c, s);
}

// The same for the FP4 path: x_q / x_s hold one encoded row per TOKEN (row index = token index).
int launch_gate_up_fp4_gather(Ctx* c, const int32_t* expert_offsets, int n_local, long long max_rows, const uint8_t* x_q,
                              const uint8_t* x_s, int T, const int32_t* row_to_assign, const uint8_t* w13_q,
                              const uint8_t* w13_s, uint8_t* h_q, uint8_t* h_s, hipStream_t s) {
    const int H = c->cfg.H, I = c->cfg.I;
    if (!gate_up_gather_supported(c, T, true)) return REALB_ESHAPE;
    GemmParams g{x_q, x_s, w13_q, w13_s, h_q, h_s, expert_offsets, n_local, H, 2 * I, I, 0, row_to_assign, 0, 0};
    division_magic(c->cfg.k, &g.src_magic, &g.src_shift);
    return launch_gemm256<true, true, true>(g, max_rows, c, s);
}

}  // namespace realb

using namespace realb;

extern "C" int realb_set_gemm_tile(int wn) {
    REALB_REQUIRE(wn == 0 || wn == 2 || wn == 8 || wn == 16, REALB_EINVAL, "tile selector must be 0, 2, 8 or 16");
    g_tile.store(wn, std::memory_order_relaxed);
    return REALB_OK;
}

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
    GemmParams g1{(const uint8_t*)x, x_s, (const uint8_t*)w13, w13_s, (uint8_t*)h_mid, h_s, expert_offsets, n_local, H, 2 * I, I, 0, nullptr, 0, 0};
    GemmParams g2{(const uint8_t*)h_mid, h_s, (const uint8_t*)w2, w2_s, (uint8_t*)y_rows, nullptr, expert_offsets, n_local, I, H, H, 0, nullptr, 0, 0};
    int rc = REALB_OK;
    if (prec == REALB_FP4) {
        if (s1) rc = launch_gemm<true, true>(g1, max_rows, c, s);
        if (rc == REALB_OK && s2) rc = launch_gemm<true, false>(g2, max_rows, c, s);
    } else {
        if (s1) rc = launch_gemm<false, true>(g1, max_rows, c, s);
        if (rc == REALB_OK && s2) rc = launch_gemm<false, false>(g2, max_rows, c, s);
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
