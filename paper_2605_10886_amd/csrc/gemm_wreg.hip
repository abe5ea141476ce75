// Skinny FP8 GEMM with the row norm fused: W stays in registers, X streams through LDS.
//
// The layers this serves (K * N <= 256 KB: 256 x 1024, 512 x 512, 1024 x 256, 256 x 256 ...) are bound by the
// HBM traffic of X and O, not by the matrix pipe: per 32 rows of X a CU reads 32 K bytes, writes 64 N bytes and
// spends well under a microsecond on MFMAs.  A tiled kernel re-streams W through LDS for every tile and runs
// load -> compute -> normalize -> store one after the other; here
//   * each of the 8 waves keeps its N / 8 columns of W (all of K) in registers for the whole launch (at most
//     128 registers per lane: the 256 KB of W fill half the register file of a CU), so W costs no LDS or L2
//     traffic after the first block;
//   * X arrives in blocks of 32 rows through a ring of 3-4 LDS buffers, requested 2-3 blocks ahead by waves
//     0..3 ONLY; the bf16 output leaves through an LDS staging buffer and is stored by waves 4..7 ONLY.  The
//     counter that tracks a wave's outstanding memory operations counts loads and stores together, so a wave
//     that did both would have to wait for its stores (an HBM round trip) before it could tell that the next
//     block has landed; with the roles split, the loaders' counter sees only loads (which return in order) and
//     the storers never wait at all.
//   * the row statistics of a block are exchanged between the 8 waves through LDS (the tile spans the row).
// One workgroup per CU walks a contiguous range of row blocks (a grouped launch keeps a workgroup inside one
// problem as long as possible; W is reloaded when the problem changes).
//
// MFMA operand roles and the W row permutation are those of gemm_panel32.hip: W rows -> MFMA rows, X rows ->
// MFMA columns, so a lane ends with 16 consecutive output columns of one output row (= lane % 32).
#include "gemm_common.h"

#include <type_traits>

namespace loka {

typedef float v16f __attribute__((ext_vector_type(16)));

template <int WNC, int KS, int RT>
struct WregCfg {
    static constexpr int NIW = WNC / 32;                  // 32-column MFMA tiles per wave
    static constexpr int KB = KS * 64;                    // bytes per row of X / W
    static constexpr int NT = 8 * WNC;                    // columns the workgroup covers
    static constexpr int RB = 32 * RT;                    // rows per block
    static constexpr int XBYTES = RB * KB;
    static constexpr int OBYTES = RB * NT * 2;
    static constexpr int NBUF_ = (131072 - OBYTES) / XBYTES;
    static constexpr int NBUF = NBUF_ > 4 ? 4 : NBUF_ < 2 ? 2 : NBUF_;
    static constexpr int LPW = XBYTES / 1024 / 4;         // X loads of 1 KB per loader wave per block
    static constexpr int SXL = (RB + 63) / 64;            // loads of 64 row scales per loader wave per block
    static constexpr int LDW = LPW + SXL;
    static constexpr int SWIN = KB / 16 < 16 ? KB / 16 : 16;   // swizzle window, 16-byte chunks
    static constexpr int OFF_X = 0;
    static constexpr int OFF_SX = OFF_X + NBUF * XBYTES;  // [NBUF][4 loaders][SXL][64] fp32
    static constexpr int OFF_OB = OFF_SX + NBUF * 4 * SXL * 256;   // [RB][NT] bf16, chunk c of row r at c ^ (r % 16)
    static constexpr int OFF_SW = OFF_OB + OBYTES;        // [NT] fp32 column scales (0 beyond N)
    static constexpr int OFF_GM = OFF_SW + NT * 4;        // [NT] fp32 gamma (1 when absent)
    static constexpr int OFF_BT = OFF_GM + NT * 4;        // [NT] fp32 beta (0 when absent)
    static constexpr int OFF_RED = OFF_BT + NT * 4;       // [RB][9] (count, mean, M2, -); 9: rows on distinct banks
    static constexpr int LDS_RUN = OFF_RED + RB * 9 * 16;
    static constexpr int STAGE = NT * KB < 131072 ? NT * KB : 131072;   // W staging at the start of a problem (overlays the rest)
    static constexpr int LDS = LDS_RUN > STAGE ? LDS_RUN : STAGE;
    static_assert(LDS <= 160 * 1024, "LDS budget");
    static_assert(LPW >= 1, "a block is at least 4 KB");
};

// Quantize prologue (GemmParams::qpro): the workgroup first quantizes ITS OWN rows of the bf16 activation - row
// blocks [b0, b1), the only ones it will read - exactly as the quantize entry point would (row amax, scale = amax /
// 448, code = e4m3(x * (448 / amax)); same helper functions, same bits) and writes codes and row scales to global
// memory where the caller wants them.  The layer costs one launch instead of two.  The bf16 rows of the first QB
// blocks are requested at kernel entry and travel while the weights are loaded; they are converted once the weights
// are in registers, and the codes of the blocks the ring would have requested first go straight into their ring slots
// (the main loop starts without a round trip for X).  Later blocks stream back from global memory (this XCD's L2)
// like any FP8 input: no other workgroup reads these rows, so the only ordering needed is inside the workgroup -
// every wave waits for its stores to be acknowledged (s_waitcnt vmcnt(0)) before the barrier in front of the first
// such read.
// Wave w owns rows [w RB / 8, +RB / 8) of a block; a row is spread over CH_ROW consecutive lanes (or over IPR loads
// of a whole wave).
template <class C, int KB, int RB>
struct QuantPrologue {
    static constexpr int CH_ROW = KB / 8;                                  // 16-byte chunks of bf16 per row
    static constexpr int RPI = CH_ROW >= 64 ? 1 : 64 / CH_ROW;             // rows per wave instruction
    static constexpr int IPR = CH_ROW >= 64 ? CH_ROW / 64 : 1;             // instructions per row
    static constexpr int RW = RB / 8;                                      // rows per wave and block
    static constexpr int NLD = RW * IPR / RPI;                             // loads per lane and block
    static constexpr int NRG = NLD / IPR;                                  // rows per lane and block
    static constexpr int QB = 16 / NLD >= 1 ? 16 / NLD : 1;                // blocks per chunk: 64 registers of raw bf16
    static_assert(RW * IPR % RPI == 0 && NLD >= 1 && NRG <= 16 && CH_ROW >= 16, "quantize prologue: block shape");
    static_assert(QB >= C::NBUF - 1, "the blocks the ring starts with lie in the first chunk");

    // requests the bf16 rows of blocks [bb, bb + QB) (below b1)
    static __device__ __forceinline__ void fetch(const GemmParams& p, int bb, int b1, int blocks_per_problem, int wave,
                                                 u32x4 (&raw)[QB][NLD]) {
        int lv = static_cast<int>(threadIdx.x) & 63;
        asm volatile("; lane id" : "+v"(lv));
#pragma unroll
        for (int u = 0; u < QB; ++u) {
            // always QB * NLD loads, so that a caller can wait for "all but these": a block past the end is requested
            // beyond the descriptor's bound and reads as zeros
            const bool dead = bb + u >= b1;                                // (uniform)
            const int b = dead ? bb : bb + u;
            const int g = b / blocks_per_problem, m0 = (b - g * blocks_per_problem) * RB;
            const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<uint16_t*>(p.xb + static_cast<int64_t>(g) * p.strideX), 0, static_cast<unsigned>(p.M) * (2u * KB), 0x00020000);
#pragma unroll
            for (int j = 0; j < NLD; ++j) {
                const int row = wave * RW + (j / IPR) * RPI + (IPR == 1 ? lv / CH_ROW : 0);
                const int chunk = IPR == 1 ? lv % CH_ROW : (j % IPR) * 64 + lv;
                // (the whole offset is the per-lane one, which the descriptor's bound applies to: rows past M read as zeros)
                const unsigned off = static_cast<unsigned>(m0 + row) * (2u * KB) + static_cast<unsigned>(chunk * 16);
                raw[u][j] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(xr, dead ? 0xFFFFFF00u : off, 0, 0));
            }
        }
    }

    // converts them (the loads have landed) and stores codes and scales to global memory; blocks below lds_end also
    // into their ring slots, in the layout the loads-to-LDS produce.  The chunk's QB * NRG <= 16 rows per lane group
    // share ONE division pair per lane (lane i of a row's lane group computes the scale and factor of the chunk's i-th
    // row).  The pass is bound by its vector instructions (two waves per SIMD, every element costs a handful), so the
    // instruction count is what is kept down.
    static __device__ __forceinline__ void convert(const GemmParams& p, int bb, int b1, int blocks_per_problem, int wave,
                                                   const u32x4 (&raw)[QB][NLD], uint8_t* smem, int lds_end) {
        static_assert(QB * NRG <= 16, "one row per lane of a 16-lane group");
        int lv = static_cast<int>(threadIdx.x) & 63;
        asm volatile("; lane id" : "+v"(lv));
        // row amax: integer max of the 15-bit magnitudes (exact), lanes of the row by xor shuffles
        // (a lane's 8 or 16 magnitudes as packed 16-bit maxima; the 16 lanes of a row of the data-parallel primitives by
        // four of those, with no LDS round trip; rows of lanes by xor shuffles)
        typedef unsigned short us2 __attribute__((ext_vector_type(2)));
        unsigned am[QB][NRG];
#pragma unroll
        for (int u = 0; u < QB; ++u) {
            if (bb + u >= b1) {                                             // (uniform) nothing was fetched
#pragma unroll
                for (int rg = 0; rg < NRG; ++rg) am[u][rg] = 0u;
                continue;
            }
#pragma unroll
            for (int rg = 0; rg < NRG; ++rg) {
                us2 a2 = {0, 0};
#pragma unroll
                for (int i = 0; i < IPR; ++i) {
                    const u32x4 w = raw[u][rg * IPR + i];
#pragma unroll
                    for (int e = 0; e < 4; ++e) a2 = __builtin_elementwise_max(a2, __builtin_bit_cast(us2, w[e] & 0x7FFF7FFFu));
                }
                unsigned a = a2[0] > a2[1] ? a2[0] : a2[1];
                unsigned o;
                o = static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(a), 0xB1, 0xF, 0xF, false));   // lane ^ 1
                a = a > o ? a : o;
                o = static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(a), 0x4E, 0xF, 0xF, false));   // lane ^ 2
                a = a > o ? a : o;
                o = static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(a), 0x141, 0xF, 0xF, false));  // the other quad of 8
                a = a > o ? a : o;
                o = static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(a), 0x140, 0xF, 0xF, false));  // the other half of 16
                a = a > o ? a : o;
#pragma unroll
                for (int msk = 16; msk < (CH_ROW < 64 ? CH_ROW : 64); msk <<= 1) {
                    o = static_cast<unsigned>(__shfl_xor(static_cast<int>(a), msk, 64));
                    a = a > o ? a : o;
                }
                am[u][rg] = a;
            }
        }
        unsigned mine = am[0][0];
#pragma unroll
        for (int u = 0; u < QB; ++u)
#pragma unroll
            for (int rg = 0; rg < NRG; ++rg) mine = (lv & 15) == u * NRG + rg ? am[u][rg] : mine;
        float scale_l, inv_l;
        group_scale(__uint_as_float(mine << 16), scale_l, inv_l);
        const int grp_base = IPR == 1 ? (lv / CH_ROW) * CH_ROW : 0;         // first lane of this lane's row group
#pragma unroll
        for (int u = 0; u < QB; ++u) {
            if (bb + u >= b1) continue;                                     // (uniform)
            constexpr bool dead = false;
            const int b = bb + u;
            const int g = b / blocks_per_problem, m0 = (b - g * blocks_per_problem) * RB;
            uint8_t* const xq = const_cast<uint8_t*>(p.X) + static_cast<int64_t>(g) * p.strideX;
            float* const sxo = const_cast<float*>(p.sx) + static_cast<int64_t>(g) * p.strideSx;
            const bool to_lds = b < lds_end;                                // (uniform)
            uint8_t* const dst = smem + C::OFF_X + (b % C::NBUF) * C::XBYTES;
            float* const sxl = reinterpret_cast<float*>(smem + C::OFF_SX + (b % C::NBUF) * 4 * C::SXL * 256);
#pragma unroll
            for (int rg = 0; rg < NRG; ++rg) {
                const float scale = __shfl(scale_l, grp_base + u * NRG + rg, 64), inv = __shfl(inv_l, grp_base + u * NRG + rg, 64);
                const int row = wave * RW + rg * RPI + (IPR == 1 ? lv / CH_ROW : 0);
                const bool live = !dead && m0 + row < p.M;
#pragma unroll
                for (int i = 0; i < IPR; ++i) {
                    const u32x4 w = raw[u][rg * IPR + i];
                    const int chunk = IPR == 1 ? lv % CH_ROW : i * 64 + lv;  // 8 elements -> 8 codes = half a 16-byte chunk
                    u32x2 o;
                    o.x = e4m3x4(bf16_lo(w.x) * inv, bf16_hi(w.x) * inv, bf16_lo(w.y) * inv, bf16_hi(w.y) * inv);
                    o.y = e4m3x4(bf16_lo(w.z) * inv, bf16_hi(w.z) * inv, bf16_lo(w.w) * inv, bf16_hi(w.w) * inv);
                    if (live) *reinterpret_cast<u32x2*>(xq + static_cast<int64_t>(m0 + row) * KB + chunk * 8) = o;
                    if (live && chunk == 0) sxo[m0 + row] = scale;
                    if (to_lds) {
                        *reinterpret_cast<u32x2*>(dst + row * KB + ((((chunk >> 1) ^ (row & (C::SWIN - 1))) << 4) | ((chunk & 1) << 3))) = o;
                        if (chunk == 0) sxl[row] = scale;
                    }
                }
            }
        }
    }
};

template <int WNC, int KS, int RT, bool FP8OUT, bool BF16IN>
__global__ __launch_bounds__(512) void gemm_wreg_kernel(const GemmParams p, const int blocks_per_problem) {
    using C = WregCfg<WNC, KS, RT>;
    constexpr int NIW = C::NIW, KB = C::KB, NT = C::NT, RB = C::RB, NBUF = C::NBUF, LPW = C::LPW, LDW = C::LDW, SXL = C::SXL;
    constexpr int KEYMASK = C::SWIN - 1;
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool loader = wave < 4, storer = wave >= 4;
    const bool ln = p.norm == LOKA_NORM_LAYERNORM;
    const bool tensor_x = p.x_mode == LOKA_SCALE_TENSOR, tensor_w = p.w_mode == LOKA_SCALE_TENSOR;
    const float inv_n = 1.0f / static_cast<float>(p.N);
    const bool blocknorm = p.norm == LOKA_NORM_BLOCKNORM, hswish = p.act == LOKA_ACT_HARDSWISH;
    constexpr int WPG = 256 / WNC;          // waves per BlockNorm group of 256 columns
    const bool affine = (p.gamma != nullptr && (ln || p.norm == LOKA_NORM_RMSNORM)) || (p.beta != nullptr && ln);

    // contiguous range of row blocks of this workgroup
    const int64_t total = static_cast<int64_t>(p.batch) * blocks_per_problem;
    const int b0 = static_cast<int>(total * blockIdx.x / gridDim.x), b1 = static_cast<int>(total * (blockIdx.x + 1) / gridDim.x);
    if (b0 >= b1) return;

    // ---- loader side: block `b` -> ring slot b % NBUF.  Lane i of load `ld` fills bytes [16 i, +16) of the
    // ld-th KB of the block: row (1024 ld + 16 i) / KB, chunk position pos; it fetches chunk pos ^ key(row).
    auto issue_block = [&](int b) __attribute__((always_inline)) {
        const int g = b / blocks_per_problem, m0 = (b - g * blocks_per_problem) * RB;
        const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint8_t*>(p.X + static_cast<int64_t>(g) * p.strideX), 0, p.M * KB, 0x00020000);
        uint8_t* const dst = smem + C::OFF_X + (b % NBUF) * C::XBYTES;
        int lv = lane;
        asm volatile("; lane id" : "+v"(lv));                           // (offsets recomputed here, not kept in registers)
#pragma unroll
        for (int q = 0; q < LPW; ++q) {
            const int ld = wave + 4 * q;
            const int byte = ld * 1024 + lv * 16;
            const int row = byte / KB, pos = (byte % KB) >> 4;
            const int voff = row * KB + ((pos ^ (row & KEYMASK)) << 4);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, (__attribute__((address_space(3))) void*)(dst + ld * 1024), 16, voff,
                                                     m0 * KB, 0, 0);
        }
        // row scales of the block, 64 per load (4 bytes per lane); rows past M read as 0
        const __amdgpu_buffer_rsrc_t sr = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float*>(p.sx + static_cast<int64_t>(g) * p.strideSx), 0, tensor_x ? 4 : p.M * 4, 0x00020000);
#pragma unroll
        for (int q = 0; q < SXL; ++q)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                sr, (__attribute__((address_space(3))) void*)(smem + C::OFF_SX + (((b % NBUF) * 4 + wave) * SXL + q) * 256), 4,
                tensor_x ? 0 : (m0 + 64 * q + lv) * 4, 0, 0, 0);
    };

    // ---- fused rowwise quantization (BF16IN): X arrives as bf16 and is quantized here exactly as the quantize
    // entry point would (row amax, scale = amax / 448, code = e4m3(x * (448 / amax))), so the FP8 copy of X never
    // travels through HBM.  All 8 waves fetch: wave w owns rows [w RB / 8, +RB / 8) of a block, NLD loads of 16
    // bytes (8 elements) per lane, a row spread over CH_ROW consecutive lanes (or over IPR loads of a whole wave).
    // fetch(b) requests block b into registers; convert(b) (one iteration later) reduces the row amax across the
    // row's lanes, computes the two divisions ONCE per lane for a different row each (an IEEE division costs
    // hundreds of cycles) and hands the results round by lane shuffles, converts and writes codes and scales
    // into block b's ring slot in the layout the loads-to-LDS produce on the other path.
    constexpr int CH_ROW = KB / 8;                                  // 16-byte chunks of bf16 per row
    constexpr int RPI = CH_ROW >= 64 ? 1 : 64 / CH_ROW;             // rows per wave instruction
    constexpr int IPR = CH_ROW >= 64 ? CH_ROW / 64 : 1;             // instructions per row
    constexpr int RW = RB / 8;                                      // rows per wave and block
    constexpr int NLD = BF16IN ? RW * IPR / RPI : IPR;              // loads per lane and block
    constexpr int NRG = NLD / IPR;                                  // rows per lane and block
    static_assert(!BF16IN || (RW * IPR % RPI == 0 && NLD >= 1 && NRG <= 16), "fused quantization: block shape");
    u32x4 raw[NLD];
    auto fetch = [&](int b) __attribute__((always_inline)) {
        const int g = b / blocks_per_problem, m0 = (b - g * blocks_per_problem) * RB;
        const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t*>(p.xb + static_cast<int64_t>(g) * p.strideX), 0, static_cast<unsigned>(p.M) * (2u * KB), 0x00020000);
        int lv = lane;
        asm volatile("; lane id" : "+v"(lv));
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            const int row = wave * RW + (j / IPR) * RPI + (IPR == 1 ? lv / CH_ROW : 0);
            const int chunk = IPR == 1 ? lv % CH_ROW : (j % IPR) * 64 + lv;
            // (the whole offset is the per-lane one, which the descriptor's bound applies to: rows past M read as zeros)
            raw[j] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(
                                                   xr, static_cast<unsigned>(m0 + row) * (2u * KB) + static_cast<unsigned>(chunk * 16), 0, 0));
        }
    };
    auto convert = [&](int b) __attribute__((always_inline)) {
        const int g = b / blocks_per_problem, m0 = (b - g * blocks_per_problem) * RB;
        uint8_t* const dst = smem + C::OFF_X + (b % NBUF) * C::XBYTES;
        float* const sxl = reinterpret_cast<float*>(smem + C::OFF_SX + (b % NBUF) * 4 * SXL * 256);
        int lv = lane;
        asm volatile("; lane id" : "+v"(lv));
        // row amax: integer max of the 15-bit magnitudes (exact), lanes of the row by xor shuffles
        unsigned am[NRG];
#pragma unroll
        for (int rg = 0; rg < NRG; ++rg) {
            unsigned a = 0u;
#pragma unroll
            for (int i = 0; i < IPR; ++i) {
                const u32x4 w = raw[rg * IPR + i];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const unsigned lo = w[e] & 0x7FFFu, hi = (w[e] >> 16) & 0x7FFFu;
                    a = a > lo ? a : lo;
                    a = a > hi ? a : hi;
                }
            }
#pragma unroll
            for (int msk = 1; msk < (CH_ROW < 64 ? CH_ROW : 64); msk <<= 1) {
                const unsigned o = static_cast<unsigned>(__shfl_xor(static_cast<int>(a), msk, 64));
                a = a > o ? a : o;
            }
            am[rg] = a;
        }
        // lane (lv % 16) = rg of each row's lane group computes that row's scale and factor
        unsigned mine = am[0];
#pragma unroll
        for (int rg = 1; rg < NRG; ++rg) mine = (lv & 15) == rg ? am[rg] : mine;
        float scale_l, inv_l;
        group_scale(__uint_as_float(mine << 16), scale_l, inv_l);
        const int grp_base = IPR == 1 ? (lv / CH_ROW) * CH_ROW : 0;         // first lane of this lane's row group
#pragma unroll
        for (int rg = 0; rg < NRG; ++rg) {
            const float scale = __shfl(scale_l, grp_base + rg, 64), inv = __shfl(inv_l, grp_base + rg, 64);
            const int row = wave * RW + rg * RPI + (IPR == 1 ? lv / CH_ROW : 0);
#pragma unroll
            for (int i = 0; i < IPR; ++i) {
                const u32x4 w = raw[rg * IPR + i];
                const int chunk = IPR == 1 ? lv % CH_ROW : i * 64 + lv;      // 8 elements = half a 16-byte chunk of codes
                u32x2 o;
                o.x = e4m3x4(bf16_lo(w.x) * inv, bf16_hi(w.x) * inv, bf16_lo(w.y) * inv, bf16_hi(w.y) * inv);
                o.y = e4m3x4(bf16_lo(w.z) * inv, bf16_hi(w.z) * inv, bf16_lo(w.w) * inv, bf16_hi(w.w) * inv);
                *reinterpret_cast<u32x2*>(dst + row * KB + ((((chunk >> 1) ^ (row & KEYMASK)) << 4) | ((chunk & 1) << 3))) = o;
                if (chunk == 0) {
                    sxl[row] = scale;
                    if (p.sx_out && m0 + row < p.M) p.sx_out[static_cast<int64_t>(g) * p.M + m0 + row] = scale;
                }
            }
        }
    };

    // ---- W fragments of this wave's columns, all of K: wreg[ni][j] feeds MFMA rows with W rows (= output
    // columns) wave * WNC + 32 ni + wperm(lane), K bytes [64 j + 32 hk, +32).  W passes through LDS in rounds of
    // up to 128 KB, fetched in whole 1 KB runs (every workgroup reads the same W: fragment-shaped 16-byte
    // reads straight from global memory put 8x the requests on the same few L2 lines and take twice as long).
    // The staging area overlays the X ring and the output buffer: callers re-request X afterwards.
    v8i wreg[NIW][KS];
    using QP = QuantPrologue<C, KB, RB>;
    u32x4 rawq[QP::QB][QP::NLD];
    auto load_problem = [&](int g, bool first) __attribute__((always_inline)) {
        constexpr int RROWS = 131072 / KB;                              // W rows per round
        constexpr int ROUNDS = (NT + RROWS - 1) / RROWS;
        int lv = lane;
        asm volatile("; lane id" : "+v"(lv));                           // (offsets recomputed here, not kept in registers)
        const int l32 = lv & 31, hk = lv >> 5;
        const int wperm = 16 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3);
        const __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint8_t*>(p.W + static_cast<int64_t>(g) * p.strideW), 0, p.N * KB, 0x00020000);
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            constexpr int ROWS_ALL = NT < RROWS ? NT : RROWS;
            const int rows = (r + 1) * RROWS <= NT ? ROWS_ALL : NT - r * RROWS;   // compile-time after unrolling
            __syncthreads();                                            // the staging area is free
            for (int ld = wave; ld < rows * KB / 1024; ld += 8) {
                const int byte = ld * 1024 + lv * 16;
                const int row = byte / KB, pos = (byte % KB) >> 4;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, (__attribute__((address_space(3))) void*)(smem + ld * 1024), 16,
                                                         row * KB + ((pos ^ (row & KEYMASK)) << 4), r * RROWS * KB, 0, 0);
            }
            // quantize prologue: the bf16 rows of the workgroup's first blocks are requested BEHIND the first round of W
            // (loads return in order: W, which comes from L2, is not held up by rows that come from HBM) and travel
            // while W's fragments are read and the next round is fetched
            if (!BF16IN && r == 0 && first && p.qpro) {
                QP::fetch(p, b0, b1, blocks_per_problem, wave, rawq);
                wait_vmcnt<QP::QB * QP::NLD>();
            } else {
                wait_vmcnt<0>();
            }
            __syncthreads();
#pragma unroll
            for (int ni = 0; ni < NIW; ++ni) {
                const int tb = wave * WNC + ni * 32;                    // first W row of the tile
                if (tb >= r * RROWS && tb < r * RROWS + rows) {
                    const int row = tb - r * RROWS + wperm;
                    const uint8_t* src = smem + row * KB;
                    const int key = row & KEYMASK;
#pragma unroll
                    for (int j = 0; j < KS; ++j) {
                        const v4i lo = *reinterpret_cast<const v4i*>(src + (((4 * j + 2 * hk) ^ key) << 4));
                        const v4i hi = *reinterpret_cast<const v4i*>(src + (((4 * j + 2 * hk + 1) ^ key) << 4));
                        wreg[ni][j] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    }
                }
            }
        }
        __syncthreads();                                                // fragments are read: the area may be reused
        const float* swg = p.sw + static_cast<int64_t>(g) * p.strideSw;
        float* swl = reinterpret_cast<float*>(smem + C::OFF_SW);
        float* gml = reinterpret_cast<float*>(smem + C::OFF_GM);
        float* btl = reinterpret_cast<float*>(smem + C::OFF_BT);
        for (int n = threadIdx.x; n < NT; n += 512) {
            const bool in = n < p.N;
            swl[n] = in ? (tensor_w ? swg[0] : swg[n]) : 0.f;
            gml[n] = (in && p.gamma && (ln || p.norm == LOKA_NORM_RMSNORM)) ? bf16_bits_to_f32(p.gamma[n]) : 1.f;
            btl[n] = (in && p.beta && ln) ? bf16_bits_to_f32(p.beta[n]) : 0.f;
        }
    };
    // W and the tables of problem g, then the first requests for X from block `bf` on
    const bool qpro = !BF16IN && p.qpro != 0;
    bool ack_pending = false;      // quantize prologue: stores of codes that will be read back are not yet known to have arrived
    auto start_problem = [&](int g, int bf, bool first) __attribute__((always_inline)) {
        load_problem(g, first);
        if (BF16IN) {
            fetch(bf);
            wait_vmcnt<0>();
            convert(bf);
            if (bf + 1 < b1) fetch(bf + 1);
        } else if (qpro && first) {
            // (load_problem has waited for every load of this wave and ended with a barrier: the rows are here, the
            // ring is free)  The blocks the ring would request now get their codes directly; the rest of the
            // workgroup's blocks are converted chunk by chunk; then every store must be acknowledged before the
            // first block is read back
            wait_vmcnt<0>();
            QP::convert(p, b0, b1, blocks_per_problem, wave, rawq, smem, bf + NBUF - 1);
            for (int bb = b0 + QP::QB; bb < b1; bb += QP::QB) {
                QP::fetch(p, bb, b1, blocks_per_problem, wave, rawq);
                wait_vmcnt<0>();
                QP::convert(p, bb, b1, blocks_per_problem, wave, rawq, smem, 0);
            }
            // blocks beyond the ring's first ones - and every block of a later problem, whose start requests its
            // blocks anew - are read back from global memory: not before every wave's stores have been acknowledged,
            // which the first iteration of the main loop checks after its MFMAs
            ack_pending = b1 - bf > NBUF - 1 || (b1 - 1) / blocks_per_problem != bf / blocks_per_problem;
        } else if (loader) {
#pragma unroll
            for (int i = 0; i < NBUF - 1; ++i)
                if (bf + i < b1) issue_block(bf + i);
        }
        __syncthreads();                                                // scales / gamma / beta are in LDS
    };

    int cur_g = b0 / blocks_per_problem;
    start_problem(cur_g, b0, true);

    // Deferred stores (bf16 output from FP8 input): a finished block is not written out at its end by the four
    // storer waves, where the other four would wait at the next barrier while the store path takes its 64 bytes
    // per clock, but by all eight waves, one instruction at a time between the MFMAs of the NEXT block: the
    // staging buffer is not written again before that block's statistics are merged (without a norm: before a
    // barrier of its own), and a wave held up by the store path leaves the matrix pipe to the other wave of its
    // SIMD.
    // With FP8 output the deferred step also converts: a lane reads 16 staged bf16 values, scales them with the
    // row's quantization factor (left in LDS by the block's epilogue) and stores 16 codes.
    constexpr bool DEFER = !BF16IN;
    constexpr int CPR = FP8OUT ? NT / 16 : NT / 8;                      // 16-byte output chunks per row
    constexpr int SW_ = DEFER ? 8 : 4;                                  // waves that store (deferred: all of them)
    constexpr int INSTR_ = RB * CPR / 64 / SW_;
    constexpr int INSTR = INSTR_ > 0 ? INSTR_ : 1;                      // store instructions per storing wave and block
    bool pending = false;
    int pend_g = 0, pend_m0 = 0;
    __amdgpu_buffer_rsrc_t pend_rsrc = __builtin_amdgcn_make_buffer_rsrc(p.out, 0, 0, 0x00020000);   // (bf16 output) the pending block's rows
    // store instruction s of the pending block: 64 consecutive chunks (1 KB), whole rows
    auto store_step = [&](int s, int sg, int sm0) __attribute__((always_inline)) {
        int lid = lane;
        asm volatile("; store lane id" : "+v"(lid));
        const int id = ((DEFER ? wave : wave - 4) + SW_ * s) * 64 + lid;
        const int r = id / CPR, c = id % CPR;
        if (FP8OUT) {
            if (r < RB) {
                const uint8_t* ob = smem + C::OFF_OB + r * (NT * 2);
                const u32x4 v0 = *reinterpret_cast<const u32x4*>(ob + (((2 * c) ^ (r & 15)) << 4));
                const u32x4 v1 = *reinterpret_cast<const u32x4*>(ob + (((2 * c + 1) ^ (r & 15)) << 4));
                const float iq = (reinterpret_cast<const float2*>(smem + C::OFF_RED) + 1)[(r * 9 + 8) * 2].y;
                u32x4 ck;
                ck.x = e4m3x4(bf16_lo(v0.x) * iq, bf16_hi(v0.x) * iq, bf16_lo(v0.y) * iq, bf16_hi(v0.y) * iq);
                ck.y = e4m3x4(bf16_lo(v0.z) * iq, bf16_hi(v0.z) * iq, bf16_lo(v0.w) * iq, bf16_hi(v0.w) * iq);
                ck.z = e4m3x4(bf16_lo(v1.x) * iq, bf16_hi(v1.x) * iq, bf16_lo(v1.y) * iq, bf16_hi(v1.y) * iq);
                ck.w = e4m3x4(bf16_lo(v1.z) * iq, bf16_hi(v1.z) * iq, bf16_lo(v1.w) * iq, bf16_hi(v1.w) * iq);
                uint8_t* const oq = p.outq + static_cast<int64_t>(sg) * p.strideO;
                if (sm0 + r < p.M && c * 16 < p.N)
                    __builtin_nontemporal_store(ck, reinterpret_cast<u32x4*>(oq + static_cast<int64_t>(sm0 + r) * p.N + c * 16));
            }
            return;
        }
        // bf16 output: a buffer store relative to the block's first row.  The descriptor ends with the last row that
        // exists (rows past M are dropped by its bound, no compare and no branch), the per-lane offset is 32 bits wide
        // (a block is at most RB * N * 2 bytes), columns past N get an offset beyond the bound.
        const unsigned ur = static_cast<unsigned>(id) / CPR, uc = static_cast<unsigned>(id) % CPR;
        const u32x4 pk = *reinterpret_cast<const u32x4*>(smem + C::OFF_OB + ur * (NT * 2) + ((uc ^ (ur & 15)) << 4));
        const unsigned voff = uc * 8 < static_cast<unsigned>(p.N) ? ur * (2u * static_cast<unsigned>(p.N)) + uc * 16 : 0xFFFFFFF0u;
        __builtin_amdgcn_raw_buffer_store_b128(pk, pend_rsrc, static_cast<int>(voff), 0, 2 /* streaming (nt) */);
    };
    // descriptor of block (sg, sm0) of the bf16 output: its rows that exist
    auto out_rsrc = [&](int sg, int sm0) __attribute__((always_inline)) {
        const int rows_here = p.M - sm0 < RB ? p.M - sm0 : RB;
        return __builtin_amdgcn_make_buffer_rsrc(
            p.out + static_cast<int64_t>(sg) * p.strideO + static_cast<int64_t>(sm0) * p.N, 0, rows_here * p.N * 2, 0x00020000);
    };
    auto flush_pending = [&]() __attribute__((always_inline)) {
        if ((DEFER || storer) && pending) {
#pragma unroll
            for (int s = 0; s < INSTR; ++s) {
                if (s % 2 == 0) __builtin_amdgcn_sched_barrier(0);      // two in flight: W leaves few registers free
                store_step(s, pend_g, pend_m0);
            }
        }
        pending = false;
    };

    // (loaders) block bb has landed: newer requests (up to NBUF - 2 blocks) may still be in flight.  The counter
    // also holds this wave's deferred stores, all newer than the loads: "at most n operations outstanding" with
    // n counting the newer LOADS then still implies that block bb is complete (loads complete in order).
    auto wait_landed = [&](int bb) __attribute__((always_inline)) {
        const int newer = b1 - 1 - bb < NBUF - 2 ? b1 - 1 - bb : NBUF - 2;
        if (p.y) wait_vmcnt<0>();                                       // Y stores share the counter
        else if (newer >= 2) wait_vmcnt<(NBUF >= 4 ? 2 : 0) * LDW>();
        else if (newer == 1) wait_vmcnt<(NBUF >= 3 ? 1 : 0) * LDW>();
        else wait_vmcnt<0>();
    };

    for (int b = b0; b < b1; ++b) {
        const int g = b / blocks_per_problem, m0 = (b - g * blocks_per_problem) * RB;
        const int tile = b;
        (void)tile;
        bool fresh = b == b0;
        if (g != cur_g) {
            fresh = true;
            if (DEFER) {
                flush_pending();                                        // the staging of W overwrites the buffer
                __syncthreads();
            }
            // (the staging of W overwrites the X blocks requested so far: they are requested again)
            if (loader || BF16IN) wait_vmcnt<0>();
            start_problem(g, b, false);
            cur_g = g;
        }
        if (BF16IN) {
            // block b + 1 was requested an iteration ago: quantize it into its ring slot (the slot of block b - 1,
            // whose reads ended before that iteration's statistics barrier)
            if (b + 1 < b1) {
                wait_vmcnt<0>();
                convert(b + 1);
            }
            lds_barrier();
        } else if (fresh || !DEFER) {
            // (with deferred stores the previous block's last barrier has already covered this)
            if (loader) wait_landed(b);
            lds_barrier();
        }
        if (BF16IN) {
            if (b + 2 < b1) fetch(b + 2);                                // in flight for a whole iteration
        } else if (loader && b + NBUF - 1 < b1 && !ack_pending) {
            issue_block(b + NBUF - 1);                                  // into the slot block b - 1 left
        }

        // Per-lane offsets are recomputed from an opaque copy of the lane id in every block: derived from a
        // loop-invariant value the compiler would keep dozens of addresses in registers, which W needs.
        int lanev = lane;
        asm volatile("; per-block lane id" : "+v"(lanev));
        const int l32 = lanev & 31, hk = lanev >> 5;
        const int xkey = l32 & KEYMASK;
        const int x_rd = l32 * KB + (((2 * hk) ^ xkey) << 4);          // + 32 KB rt, ^ (64 j + 16 h) per fragment half
        int colbase[NIW];
        float cnt_lane = 0.f;
#pragma unroll
        for (int ni = 0; ni < NIW; ++ni) {
            colbase[ni] = wave * WNC + ni * 32 + hk * 16;
            if (colbase[ni] < p.N) cnt_lane += 16.f;                    // N % 16 == 0
        }
        uint8_t* const obuf = smem + C::OFF_OB;
        float4* const red = reinterpret_cast<float4*>(smem + C::OFF_RED);

        // ---- MFMAs: for each K step of 64, RT row tiles x NIW column tiles
        const uint8_t* xs = smem + C::OFF_X + (b % NBUF) * C::XBYTES;
        v16f acc[RT][NIW];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int ni = 0; ni < NIW; ++ni)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[rt][ni][i] = 0.f;
        // X fragments one or two (row tile, K step) pairs ahead of the MFMAs that use them
        constexpr int XD = (NIW * KS + RT * NIW * 2) >= 20 ? 2 : 3;     // ring of fragments (registers are short when W fills 128)
        constexpr int NS = KS * RT;
        v8i xf[XD];
        auto read_xf = [&](int q) __attribute__((always_inline)) {      // q = j * RT + rt
            const int j = q / RT, rt = q % RT;
            const v4i lo = *reinterpret_cast<const v4i*>(xs + rt * 32 * KB + (x_rd ^ (64 * j)));
            const v4i hi = *reinterpret_cast<const v4i*>(xs + rt * 32 * KB + (x_rd ^ (64 * j + 16)));
            xf[q % XD] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        };
#pragma unroll
        for (int q = 0; q < XD - 1 && q < NS; ++q) read_xf(q);
        auto mma_loop = [&](auto store_tag) __attribute__((always_inline)) {
            constexpr bool STORES = decltype(store_tag)::value;
            constexpr int TM = NS * NIW;                                // MFMAs of the block
#pragma unroll
            for (int q = 0; q < NS; ++q) {
                __builtin_amdgcn_sched_barrier(0);
                if (q + XD - 1 < NS) read_xf(q + XD - 1);
#pragma unroll
                for (int ni = 0; ni < NIW; ++ni) {
                    acc[q % RT][ni] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wreg[ni][q / RT], xf[q % XD],
                                                                                     acc[q % RT][ni], 0, 0, 0, 0, 0, 0);
                    if (STORES) {
                        // the pending block's stores, spread evenly over the MFMAs, in source order
                        const int t = q * NIW + ni;
#pragma unroll
                        for (int s = t * INSTR / TM; s < (t + 1) * INSTR / TM; ++s) {
                            __builtin_amdgcn_sched_barrier(0);
                            store_step(s, pend_g, pend_m0);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        };
        if (DEFER && pending) mma_loop(std::true_type{}); else mma_loop(std::false_type{});
        if (DEFER) pending = false;                                     // the previous block is on its way
        __builtin_amdgcn_sched_barrier(0);
        if (!BF16IN && ack_pending) wait_vmcnt<0>();                    // (quantize prologue) this wave's codes have arrived ...

        // ---- scales, row statistics (lane -> pair of lanes with the same row -> the 8 waves through LDS)
        const float* sxl = reinterpret_cast<const float*>(smem + C::OFF_SX + (b % NBUF) * 4 * SXL * 256);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const float sxm = sxl[rt * 32 + l32];
#pragma unroll
            for (int ni = 0; ni < NIW; ++ni) {
                __builtin_amdgcn_sched_barrier(0);      // one tile's table reads at a time: W leaves few registers free
                const v4f* sw4 = reinterpret_cast<const v4f*>(smem + C::OFF_SW + colbase[ni] * 4);
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const v4f s = sw4[a];
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[rt][ni][4 * a + e] *= s[e] * sxm;
                }
            }
            const int m = m0 + rt * 32 + l32;
            if (p.y && m < p.M) {
                float* yrow = p.y + static_cast<int64_t>(g) * p.strideO + static_cast<int64_t>(m) * p.N;
#pragma unroll
                for (int ni = 0; ni < NIW; ++ni)
                    if (colbase[ni] < p.N) {
#pragma unroll
                        for (int a = 0; a < 4; ++a)
                            *reinterpret_cast<v4f*>(yrow + colbase[ni] + 4 * a) =
                                v4f{acc[rt][ni][4 * a], acc[rt][ni][4 * a + 1], acc[rt][ni][4 * a + 2], acc[rt][ni][4 * a + 3]};
                    }
            }
            if (p.norm != LOKA_NORM_NONE) {
                float n_ = cnt_lane, mean = 0.f, m2 = 0.f;
                if (ln) {
                    float s = 0.f;
#pragma unroll
                    for (int ni = 0; ni < NIW; ++ni)
                        if (colbase[ni] < p.N) {
#pragma unroll
                            for (int i = 0; i < 16; ++i) s += acc[rt][ni][i];
                        }
                    mean = n_ > 0.f ? s * __builtin_amdgcn_rcpf(n_) : 0.f;
#pragma unroll
                    for (int ni = 0; ni < NIW; ++ni)
                        if (colbase[ni] < p.N) {
#pragma unroll
                            for (int i = 0; i < 16; ++i) { const float d = acc[rt][ni][i] - mean; m2 = __builtin_fmaf(d, d, m2); }
                        }
                    // lanes l and l ^ 32 hold the same row: symmetric merge, identical bits on both
                    const float nb = wave_shfl_xor(n_, 32), mb = wave_shfl_xor(mean, 32), m2b = wave_shfl_xor(m2, 32);
                    const float nn = n_ + nb;
                    if (nn > 0.f) {
                        const float d = mb - mean;
                        const float rn = __builtin_amdgcn_rcpf(nn);
                        const float newmean = (n_ * mean + nb * mb) * rn;
                        m2 = m2 + m2b + d * d * (n_ * nb * rn);
                        mean = newmean;
                    }
                    n_ = nn;
                } else {
#pragma unroll
                    for (int ni = 0; ni < NIW; ++ni)
                        if (colbase[ni] < p.N) {
#pragma unroll
                            for (int i = 0; i < 16; ++i) m2 = __builtin_fmaf(acc[rt][ni][i], acc[rt][ni][i], m2);
                        }
                    m2 += wave_shfl_xor(m2, 32);
                }
                if (hk == 0) red[(rt * 32 + l32) * 9 + wave] = make_float4(n_, mean, m2, 0.f);
            }
        }
        float mean_r[RT], rstd_r[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) { mean_r[rt] = 0.f; rstd_r[rt] = 1.f; }
        if (p.norm != LOKA_NORM_NONE) {
            lds_barrier();
            // The two lanes that hold a row (l and l ^ 32) take four waves' entries each and add their halves (a + b ==
            // b + a: identical bits on both, in every wave).  LayerNorm: the parts' counts add up to N exactly, so the
            // row mean is sum(n_w mean_w) / N and the centred sum of squares is sum(m2_w + n_w (mean_w - mean)^2) - the
            // combination of per-part (count, mean, M2) written without the chain of pairwise merges and their
            // reciprocals (an empty part has count 0 and mean 0 and adds nothing).
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                float tm2 = 0.f, tmean = 0.f;
                float4 r[4];
#pragma unroll
                for (int w = 0; w < 4; ++w) r[w] = red[(rt * 32 + l32) * 9 + 4 * hk + w];
                if (ln) {
                    float s1 = 0.f;
#pragma unroll
                    for (int w = 0; w < 4; ++w) s1 = __builtin_fmaf(r[w].x, r[w].y, s1);
                    s1 += wave_shfl_xor(s1, 32);
                    tmean = s1 * inv_n;
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        const float d = r[w].y - tmean;
                        tm2 += __builtin_fmaf(r[w].x * d, d, r[w].z);
                    }
                } else {
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        // BlockNorm: only the waves that share this wave's group of 256 columns
                        if (!blocknorm || (4 * hk + w) / WPG == wave / WPG) tm2 += r[w].z;
                    }
                }
                tm2 += wave_shfl_xor(tm2, 32);
                mean_r[rt] = tmean;
                rstd_r[rt] = __builtin_amdgcn_rsqf(tm2 * (blocknorm ? 1.0f / 256.0f : inv_n) + p.eps);
            }
        } else if (DEFER) {
            lds_barrier();      // every wave has read its part of the previous block out of the staging buffer
        }
        if (!BF16IN && ack_pending) {
            // ... and, a barrier later, every wave's: the first block that is read back may be requested
            if (loader && b + NBUF - 1 < b1) issue_block(b + NBUF - 1);
            ack_pending = false;
        }

        // normalized (+ affine, + activation) values of 8 consecutive columns of row tile rt, as packed bf16
        // (without gamma and beta the affine step is x * 1 + 0: skipped, and its table reads with it)
        auto norm8 = [&](auto affine_tag, int rt, int ni, int half, const v4f gq0, const v4f gq1, const v4f bq0,
                         const v4f bq1, const float rstd) __attribute__((always_inline)) {
            constexpr bool AFFINE = decltype(affine_tag)::value;
            const float nmr = -mean_r[rt] * rstd;
            float o[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                o[e] = __builtin_fmaf(acc[rt][ni][8 * half + e], rstd, nmr);
                o[4 + e] = __builtin_fmaf(acc[rt][ni][8 * half + 4 + e], rstd, nmr);
                if (AFFINE) {
                    o[e] = __builtin_fmaf(o[e], gq0[e], bq0[e]);
                    o[4 + e] = __builtin_fmaf(o[4 + e], gq1[e], bq1[e]);
                }
            }
            if (hswish) {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    o[e] = o[e] * __builtin_fminf(__builtin_fmaxf(o[e] + 3.0f, 0.0f), 6.0f) * (1.0f / 6.0f);
            }
            u32x4 pk;
            pk.x = pack_bf16x2(o[0], o[1]); pk.y = pack_bf16x2(o[2], o[3]);
            pk.z = pack_bf16x2(o[4], o[5]); pk.w = pack_bf16x2(o[6], o[7]);
            return pk;
        };
        // ---- bf16 into the staging buffer (row 32 rt + l32; 16-byte chunk c at position c ^ (row % 16)); with FP8
        // output also the lane's maximum of the bf16 magnitudes per row tile (integer max: exact)
        unsigned amax_b[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) amax_b[rt] = 0u;
        auto stage = [&](auto affine_tag) __attribute__((always_inline)) {
            constexpr bool AFFINE = decltype(affine_tag)::value;
#pragma unroll
            for (int ni = 0; ni < NIW; ++ni) {
                const v4f* g4 = reinterpret_cast<const v4f*>(smem + C::OFF_GM + colbase[ni] * 4);
                const v4f* b4 = reinterpret_cast<const v4f*>(smem + C::OFF_BT + colbase[ni] * 4);
                const bool in = colbase[ni] < p.N;
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    __builtin_amdgcn_sched_barrier(0);
                    v4f gq0 = {}, gq1 = {}, bq0 = {}, bq1 = {};
                    if (AFFINE) { gq0 = g4[2 * half]; gq1 = g4[2 * half + 1]; bq0 = b4[2 * half]; bq1 = b4[2 * half + 1]; }
                    const int c = (colbase[ni] >> 3) + half;
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) {
                        const u32x4 pk = norm8(affine_tag, rt, ni, half, gq0, gq1, bq0, bq1, rstd_r[rt]);
                        *reinterpret_cast<u32x4*>(obuf + (rt * 32 + l32) * (NT * 2) + ((c ^ (l32 & 15)) << 4)) = pk;
                        if (FP8OUT) {
                            // (two 16-bit magnitudes per word, packed integer maximum; the halves are folded after the loop)
                            typedef unsigned short us2 __attribute__((ext_vector_type(2)));
                            us2 a = __builtin_bit_cast(us2, amax_b[rt]);
#pragma unroll
                            for (int e = 0; e < 4; ++e) a = __builtin_elementwise_max(a, __builtin_bit_cast(us2, pk[e] & 0x7FFF7FFFu));
                            if (in) amax_b[rt] = __builtin_bit_cast(unsigned, a);
                        }
                    }
                }
            }
        };
        if (affine) stage(std::true_type{}); else stage(std::false_type{});
        if (FP8OUT) {
            // ---- FP8 output for the next layer: the staged bf16 values quantized per row exactly as the quantize
            // entry point would quantize the stored bf16 tensor (amax over the row of |bf16 value|, scale =
            // amax / 448, code = e4m3(value * (448 / amax))).  The row amax crosses the 8 waves in the unused fourth
            // word of the statistics entries; RB threads then compute the row's scale pair once and leave
            // it in the row's spare entry, where the conversion (store_step, deferred like the bf16 stores) finds
            // it.  (The normalized values are computed once: recomputing them after the amax was known cost a second
            // pass over the accumulators, 85 against 58 us at 65536 x 256 x 1024.)
            unsigned* const redq = reinterpret_cast<unsigned*>(smem + C::OFF_RED) + 3;
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                amax_b[rt] = (amax_b[rt] & 0xFFFFu) > (amax_b[rt] >> 16) ? (amax_b[rt] & 0xFFFFu) : (amax_b[rt] >> 16);
                const unsigned o2 = static_cast<unsigned>(__shfl_xor(static_cast<int>(amax_b[rt]), 32, 64));
                amax_b[rt] = amax_b[rt] > o2 ? amax_b[rt] : o2;
                if (hk == 0) redq[((rt * 32 + l32) * 9 + wave) * 4] = amax_b[rt];
            }
            lds_barrier();
            float2* const sq = reinterpret_cast<float2*>(smem + C::OFF_RED) + 1;       // words 2, 3 of entry [row][8]
            // (by a storer wave: a loader's memory counter must not hold a store this young when it next checks
            // that its X block has landed)
            if (threadIdx.x >= 256 && threadIdx.x < 256 + RB) {
                int tl = static_cast<int>(threadIdx.x) - 256;
                asm volatile("; row id" : "+v"(tl));
                unsigned a = 0u;
#pragma unroll
                for (int w = 0; w < 8; ++w) { const unsigned v = redq[(tl * 9 + w) * 4]; a = a > v ? a : v; }
                float scale, inv;
                group_scale(__uint_as_float(a << 16), scale, inv);
                sq[(tl * 9 + 8) * 2] = make_float2(scale, inv);
                if (m0 + tl < p.M) p.outs[static_cast<int64_t>(g) * p.M + m0 + tl] = scale;
            }
        }
        // (deferred stores: this barrier is also the next block's "X has landed" barrier)
        if (DEFER && loader && b + 1 < b1 && (b + 1) / blocks_per_problem == g) wait_landed(b + 1);
        lds_barrier();
        // ---- the block is written out: now, or between the MFMAs of the next block
        pending = true; pend_g = g; pend_m0 = m0;
        if (!FP8OUT) pend_rsrc = out_rsrc(g, m0);
        if (!DEFER || b + 1 == b1) flush_pending();
    }
}

// ---------------------------------------------------------------------------------------------- host side
namespace {

struct WregInst {
    int wnc, ks, rb;
    const void* fn;      // bf16 output
    const void* fn_q;    // e4m3 output
    const void* fn_b;    // bf16 input, quantized in the kernel
    size_t lds;
    void (*launch)(const GemmParams&, int, dim3, hipStream_t);
};

// Fused quantization is built where the registers allow it: the configurations whose W fragments already fill 128
// registers per lane (K * N = 256 KB) have no room for a block of raw bf16 beside them (the compiler spills hundreds
// of registers per lane).
template <int WNC, int KS, int RT>
constexpr bool kWregFused = WNC * KS < 512;

template <int WNC, int KS, int RT>
void launch_wreg(const GemmParams& p, int bpp, dim3 grid, hipStream_t s) {
    if (p.xb && !p.qpro) {
        if constexpr (kWregFused<WNC, KS, RT>)
            gemm_wreg_kernel<WNC, KS, RT, false, true><<<grid, 512, WregCfg<WNC, KS, RT>::LDS, s>>>(p, bpp);
    } else if (p.outq) gemm_wreg_kernel<WNC, KS, RT, true, false><<<grid, 512, WregCfg<WNC, KS, RT>::LDS, s>>>(p, bpp);
    else gemm_wreg_kernel<WNC, KS, RT, false, false><<<grid, 512, WregCfg<WNC, KS, RT>::LDS, s>>>(p, bpp);
}

template <int WNC, int KS, int RT>
const void* wreg_fused_fn() {
    if constexpr (kWregFused<WNC, KS, RT>) return reinterpret_cast<const void*>(&gemm_wreg_kernel<WNC, KS, RT, false, true>);
    else return nullptr;
}

#define LOKA_WREG(WNC, KS, RT)                                                                                   \
    {WNC, KS, 32 * RT, reinterpret_cast<const void*>(&gemm_wreg_kernel<WNC, KS, RT, false, false>),               \
     reinterpret_cast<const void*>(&gemm_wreg_kernel<WNC, KS, RT, true, false>),                                  \
     wreg_fused_fn<WNC, KS, RT>(), WregCfg<WNC, KS, RT>::LDS,                                                     \
     &launch_wreg<WNC, KS, RT>}

// columns per wave, K / 64, row tiles per block (as many as registers and LDS allow: fewer, longer iterations)
const WregInst kWreg[] = {
    LOKA_WREG(32, 2, 4),  LOKA_WREG(32, 4, 4), LOKA_WREG(32, 8, 2), LOKA_WREG(32, 16, 1),
    LOKA_WREG(64, 2, 2),  LOKA_WREG(64, 4, 2), LOKA_WREG(64, 8, 1),
    LOKA_WREG(128, 2, 1), LOKA_WREG(128, 4, 1),
};

const WregInst* wreg_pick(int64_t N, int64_t K) {
    if (K % 64) return nullptr;
    const int ks = static_cast<int>(K / 64);
    const int wnc = N <= 256 ? 32 : N <= 512 ? 64 : N <= 1024 ? 128 : 0;
    for (const WregInst& w : kWreg)
        if (w.wnc == wnc && w.ks == ks) return &w;
    return nullptr;
}

}  // namespace

bool wreg_supports_fused(int64_t M, int64_t N, int64_t K) {
    const WregInst* w = wreg_pick(N, K);
    return w != nullptr && w->fn_b != nullptr && M * K < (int64_t(1) << 31);
}

bool wreg_supports(int64_t M, int64_t N, int64_t K) {
    return wreg_pick(N, K) != nullptr && M * K < (int64_t(1) << 31) && M * 4 < (int64_t(1) << 31);
}

// Workgroups to launch and the kernel's entry (for the dynamic-LDS attribute); 0 when unsupported.
int wreg_plan(int64_t M, int64_t N, int64_t K, int64_t batch, int cus, bool fp8_out, bool bf16_in, const void** fn,
              size_t* lds) {
    const WregInst* w = wreg_pick(N, K);
    if (!w) return 0;
    *fn = bf16_in ? w->fn_b : fp8_out ? w->fn_q : w->fn;
    *lds = w->lds;
    const int64_t blocks = batch * ((M + w->rb - 1) / w->rb);
    return static_cast<int>(blocks < cus ? blocks : cus);
}

void wreg_launch(const GemmParams& p, dim3 grid, hipStream_t s) {
    const WregInst* w = wreg_pick(p.N, p.KB);
    w->launch(p, (p.M + w->rb - 1) / w->rb, grid, s);
}

}  // namespace loka
