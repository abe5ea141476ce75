// Large-tile FP8 GEMM with the row norm fused across workgroups: 256 x 256 tiles, 8 waves,
// v_mfma_f32_32x32x64_f8f6f4, persistent panel-synchronous schedule (see gemm.hip for the schedule's
// description; this file is its throughput-oriented instantiation).
//
// Why a second kernel: measured on MI355X, back-to-back 16x16x128 MFMAs issued by ONE wave reach ~70-80 %
// of the FP8 rate (each instruction reads 16 operand registers for 32 cycles of work), while 32x32x64
// reaches 98 % (same operand registers, 64 cycles of work).  In the ping-pong main loop only one wave
// per SIMD computes at a time, so the 32x32x64 form is the one that keeps the matrix pipe full.
//
// Work split: waves 0..3 own rows 0..127 of the tile, waves 4..7 rows 128..255; wave w % 4 owns columns
// [64 (w % 4), +64).  Per K step of 128 bytes a wave runs 4 (row tiles of 32) x 2
// (column tiles of 32) x 2 (K halves of 64) = 16 MFMAs from 12 operand fragments of 8 registers.
//
// Operand roles are swapped as in gemm.hip (W rows -> MFMA rows, X rows -> MFMA columns).  MFMA row
// rho = 8a + 4h + b (a = 0..3, h = lane / 32, b = 0..3) is fed W row 16h + 4a + b of the 32-row tile, so a
// lane ends with 16 CONSECUTIVE output columns (accumulator element i <-> column 16h + i) of one output
// row m = lane % 32, and the two lanes that share a row cover 32 consecutive columns.
//
// LDS: rows of 128 bytes, chunk c of row r at position c ^ key(r); X rows are read 16 consecutive rows at a
// time (key = (r >> 1) & 7); the W read pattern above touches rows {16h + 4a + b} with a in a pair
// {0,1} or {2,3} per 16 lanes: key = bits (1, 2, 4) of r.  Both give 16 lanes x 16 bytes on 64 distinct banks.
#include "gemm_common.h"

namespace loka {

typedef float v16f __attribute__((ext_vector_type(16)));

// BW: 0 = one scale per row / column / tensor (applied in the epilogue); 1 = block scales, accumulators rescaled
// per K block; 2 = power-of-two block scales handed to the matrix cores (scaled MFMA), nothing to rescale.
// FP8OUT: instead of bf16 O the tile leaves as e4m3 codes with one scale per output row, exactly what a rowwise
// quantization of the bf16 output would give.  Without an affine step the normalized value (y - mean) * rstd grows
// with y, and so does its bf16 rounding: the row's largest magnitude is reached at the row's largest or smallest
// y, so the row minimum and maximum travel with the row statistics in the ONE exchange between the workgroups of a
// panel and every workgroup derives the row scale from them.  With gamma / beta the extremum can sit anywhere: the
// tile is normalized first and the row amax of the result crosses the workgroups in a second exchange.
// F8: 0 = bf16 output, 1 = FP8 output without gamma / beta (one exchange), 2 = FP8 output with gamma / beta, BlockNorm
// or an activation (the row amax of the result crosses the workgroups in a second exchange; an instantiation of its
// own because it keeps the packed normalized tile in registers).
// Quantize prologue (QPRO instantiation; GemmParams::qpro): when a tile spans the whole output row (N <= 256), the 256
// rows of X a tile reads are read by no other workgroup, so the workgroup can quantize them itself - rowwise, exactly
// as the quantize entry point would (row amax, scale = amax / 448, code = e4m3(x * (448 / amax)); same helper
// functions, same bits) - write codes and row scales where the caller wants them, and then stream them back like any
// FP8 input (they come from this XCD's L2).  One launch instead of two; the only ordering needed is inside the
// workgroup: every wave waits for its stores to be acknowledged before the barrier in front of the first read.
// Wave w takes rows [32 w, +32) of each of the workgroup's tiles, RG rows at a time (16 loads of 16 bytes per lane in
// flight, the next group requested before the current one is converted); a row is LPR loads of a whole wave
// (K = 512 LPR elements).
template <int LPR>
__device__ __forceinline__ void panel32_quantize_own_rows(const GemmParams& p, int tile_first, int tile_stride, int total_tiles,
                                                          int wave) {
    constexpr int RG = 16 / LPR;                 // rows per group
    constexpr int NG = 32 / RG;                  // groups per tile and wave
    typedef unsigned short us2 __attribute__((ext_vector_type(2)));
    int lv = static_cast<int>(threadIdx.x) & 63;
    asm volatile("; lane id" : "+v"(lv));
    const int K = p.KB;                          // elements per row (= bytes per row of codes)
    u32x4 raw[2][RG][LPR];
    // group q of the workgroup's tile sequence: tile tile_first + (q / NG) * tile_stride, rows 32 wave + (q % NG) * RG + [0, RG)
    const int ntiles = tile_first < total_tiles ? (total_tiles - 1 - tile_first) / tile_stride + 1 : 0;
    const int ngroups = ntiles * NG;
    auto locate = [&](int q, int& g, int& m0) __attribute__((always_inline)) {
        const int tile = tile_first + (q / NG) * tile_stride;
        g = tile / p.tiles_m;                    // (tiles_n == 1)
        m0 = (tile - g * p.tiles_m) * 256 + 32 * wave + (q % NG) * RG;
    };
    auto fetch = [&](int q, u32x4 (&dst)[RG][LPR]) __attribute__((always_inline)) {
        int g, m0;
        locate(q, g, m0);
        const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t*>(p.xb + static_cast<int64_t>(g) * p.strideX), 0, static_cast<unsigned>(p.M) * (2u * K), 0x00020000);
#pragma unroll
        for (int rr = 0; rr < RG; ++rr)
#pragma unroll
            for (int i = 0; i < LPR; ++i)
                // (rows past M lie beyond the descriptor's bound and read as zeros)
                dst[rr][i] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(
                                                           xr, static_cast<unsigned>(m0 + rr) * (2u * K) + static_cast<unsigned>((i * 64 + lv) * 16), 0, 0));
    };
    auto convert = [&](int q, const u32x4 (&src)[RG][LPR]) __attribute__((always_inline)) {
        int g, m0;
        locate(q, g, m0);
        uint8_t* const xq = const_cast<uint8_t*>(p.X) + static_cast<int64_t>(g) * p.strideX;
        float* const sxo = const_cast<float*>(p.sx) + static_cast<int64_t>(g) * p.strideSx;
        // row amax: packed 16-bit maxima of the magnitudes (exact), the 16 lanes of a DPP row by four data-parallel
        // moves, the four rows of lanes by two xor shuffles
        unsigned mine = 0u;
#pragma unroll
        for (int rr = 0; rr < RG; ++rr) {
            us2 a2 = {0, 0};
#pragma unroll
            for (int i = 0; i < LPR; ++i)
#pragma unroll
                for (int e = 0; e < 4; ++e) a2 = __builtin_elementwise_max(a2, __builtin_bit_cast(us2, src[rr][i][e] & 0x7FFF7FFFu));
            unsigned a = a2[0] > a2[1] ? a2[0] : a2[1], o;
            o = static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(a), 0xB1, 0xF, 0xF, false)); a = a > o ? a : o;
            o = static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(a), 0x4E, 0xF, 0xF, false)); a = a > o ? a : o;
            o = static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(a), 0x141, 0xF, 0xF, false)); a = a > o ? a : o;
            o = static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(a), 0x140, 0xF, 0xF, false)); a = a > o ? a : o;
            o = static_cast<unsigned>(__shfl_xor(static_cast<int>(a), 16, 64)); a = a > o ? a : o;
            o = static_cast<unsigned>(__shfl_xor(static_cast<int>(a), 32, 64)); a = a > o ? a : o;
            mine = lv == rr ? a : mine;          // lane rr keeps row rr's amax: one division pair per lane, not per row and lane
        }
        float scale_l, inv_l;
        group_scale(__uint_as_float(mine << 16), scale_l, inv_l);
        if (lv < RG && m0 + lv < p.M) sxo[m0 + lv] = scale_l;
#pragma unroll
        for (int rr = 0; rr < RG; ++rr) {
            const float inv = __shfl(inv_l, rr, 64);
            const bool live = m0 + rr < p.M;
#pragma unroll
            for (int i = 0; i < LPR; ++i) {
                const u32x4 w = src[rr][i];
                u32x2 o;
                o.x = e4m3x4(bf16_lo(w.x) * inv, bf16_hi(w.x) * inv, bf16_lo(w.y) * inv, bf16_hi(w.y) * inv);
                o.y = e4m3x4(bf16_lo(w.z) * inv, bf16_hi(w.z) * inv, bf16_lo(w.w) * inv, bf16_hi(w.w) * inv);
                if (live) *reinterpret_cast<u32x2*>(xq + static_cast<int64_t>(m0 + rr) * K + (i * 64 + lv) * 8) = o;
            }
        }
    };
    if (ngroups > 0) fetch(0, raw[0]);
    for (int q = 0; q < ngroups; q += 2) {
        // (two groups per iteration so that the buffers keep compile-time names)
        if (q + 1 < ngroups) { fetch(q + 1, raw[1]); wait_vmcnt<RG * LPR>(); } else wait_vmcnt<0>();
        convert(q, raw[0]);
        if (q + 1 < ngroups) {
            // ("at most RG * LPR operations outstanding" covers group q + 1 although the stores of group q are in
            // flight too: loads return in order, so whatever part of the completed operations are stores, the completed
            // loads are the oldest ones, and there are at least as many of them as group q + 1 has)
            if (q + 2 < ngroups) { fetch(q + 2, raw[0]); wait_vmcnt<RG * LPR>(); } else wait_vmcnt<0>();
            convert(q + 1, raw[1]);
        }
    }
    wait_vmcnt<0>();                             // codes and scales are in L2 before this wave passes the barrier
}

template <int EPI, int BW, int F8, bool QPRO = false>
__global__ __launch_bounds__(512) void gemm_panel32_kernel(const GemmParams p) {
    constexpr bool FP8OUT = F8 != 0;
    constexpr bool BLOCKWISE = BW != 0;
    constexpr int BM = 256, BN = 256, NW = 8, WM = 128, WN = 64, MI = 4, NI = 2;
    constexpr int ES = 256 * 128;           // one ring entry: 256 rows x 128 bytes of X or of W
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wave_m = wave >> 2, wave_n = wave & 3;
    const bool grp_b = wave >= 4;           // the second wave of each SIMD
    const int l32 = lane & 31, hk = lane >> 5;

    const int total_tiles = p.tiles_m * p.tiles_n * p.batch;
    int tile_first = blockIdx.x, tile_stride = total_tiles;
    if (EPI == EPI_PANEL_SYNC) {
        const int G = gridDim.x;
        tile_first = (G % 8 == 0) ? (blockIdx.x % 8) * (G / 8) + blockIdx.x / 8 : blockIdx.x;
        tile_stride = G;
        // the workspace remembers which launch used it last (a wait that runs out records the same value beside it)
        if (p.header && blockIdx.x == 0 && threadIdx.x == 0)
            __hip_atomic_store(p.header, p.nonce, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // loop-invariant lane offsets
    const int ld_row = lane >> 3, ld_pos = lane & 7;
    const int x_lane_off = ld_row * p.KB + (((ld_pos ^ (ld_row >> 1)) << 4) ^ ((wave & 1) << 6));
    const int w_lane_off = ld_row * p.KB + (((ld_pos ^ ((ld_row >> 1) & 3)) << 4) ^ (((wave >> 1) & 1) << 6));
    // fragment read offsets inside a stage: K half s uses chunks 4s + 2hk, 4s + 2hk + 1
    const int xrow = wave_m * WM + l32;                                    // + 32 mi
    const int xkey = (xrow >> 1) & 7;
    const int x_off0 = xrow * 128 + (((2 * hk) ^ xkey) << 4), x_off1 = xrow * 128 + (((2 * hk + 1) ^ xkey) << 4);
    const int wperm = 16 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3);  // W row of the 32-row tile this lane feeds
    const int wrow = wave_n * WN + wperm;                                  // + 32 ni
    const int wkey = ((wrow >> 1) & 1) | (((wrow >> 2) & 1) << 1) | (((wrow >> 4) & 1) << 2);
    const int w_off0 = wrow * 128 + (((2 * hk) ^ wkey) << 4), w_off1 = wrow * 128 + (((2 * hk + 1) ^ wkey) << 4);
    const int ksteps = p.KB / 128;

    // buffer descriptors of the tile whose operands are being streamed (bounds = the rows that exist: rows
    // past the end of X or W read as zeros)
    __amdgpu_buffer_rsrc_t x_rsrc, w_rsrc;
    auto set_rsrc = [&](int tile_id) __attribute__((always_inline)) {
        int t = tile_id;
        const int tn_ = t % p.tiles_n; t /= p.tiles_n;
        const int tm_ = t % p.tiles_m;
        const int g_ = t / p.tiles_m;
        const int m0_ = tm_ * BM, n0_ = tn_ * BN;
        const int x_rows = p.M - m0_ < BM ? p.M - m0_ : BM, w_rows = p.N - n0_ < BN ? p.N - n0_ : BN;
        x_rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint8_t*>(p.X + static_cast<int64_t>(g_) * p.strideX + static_cast<int64_t>(m0_) * p.KB), 0,
            x_rows * p.KB, 0x00020000);
        w_rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint8_t*>(p.W + static_cast<int64_t>(g_) * p.strideW + static_cast<int64_t>(n0_) * p.KB), 0,
            w_rows * p.KB, 0x00020000);
    };
    bool prefetched = false;        // ring entries X(0) W(0) X(1) W(1) of `tile` were requested during the previous epilogue
    if (QPRO) {
        if (p.KB == 512) panel32_quantize_own_rows<1>(p, tile_first, tile_stride, total_tiles, wave);
        else if (p.KB == 1024) panel32_quantize_own_rows<2>(p, tile_first, tile_stride, total_tiles, wave);
        else panel32_quantize_own_rows<4>(p, tile_first, tile_stride, total_tiles, wave);
        __syncthreads();
    }

  for (int tile = tile_first; tile < total_tiles; tile += tile_stride) {
    int t = tile;
    const int tn = t % p.tiles_n; t /= p.tiles_n;
    const int tm = t % p.tiles_m;
    const int g = t / p.tiles_m;
    const int m0 = tm * BM, n0 = tn * BN;
    const float* sxg = p.sx + static_cast<int64_t>(g) * p.strideSx;
    const float* swg = p.sw + static_cast<int64_t>(g) * p.strideSw;
    if (!prefetched) set_rsrc(tile);
    // this wave's share of one ring entry (the X or the W rows of K step kb / 128) is four loads of 1 KB:
    // row groups wave, wave + 8, wave + 16, wave + 24; load j of an entry
    auto issue_x1 = [&](int slot, int kb, int j) __attribute__((always_inline)) {
        const int grp = wave + j * NW;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            x_rsrc, (__attribute__((address_space(3))) void*)(smem + slot * ES + grp * 1024), 16, x_lane_off,
            grp * 8 * p.KB + kb, 0, 0);
    };
    auto issue_w1 = [&](int slot, int kb, int j) __attribute__((always_inline)) {
        const int grp = wave + j * NW;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            w_rsrc, (__attribute__((address_space(3))) void*)(smem + slot * ES + grp * 1024), 16, w_lane_off,
            grp * 8 * p.KB + kb, 0, 0);
    };
    auto issue_x = [&](int slot, int kb) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 4; ++j) issue_x1(slot, kb, j);
    };
    auto issue_w = [&](int slot, int kb) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 4; ++j) issue_w1(slot, kb, j);
    };

    v16f acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;

    // Blockwise scales (1 x 128 for X, 128 x 128 for W): the accumulators are kept in units of the CURRENT K
    // block's scale s(kb) = sx[m, kb] * sw[kb, n / 128] (one value per lane and row tile: a wave's 64 columns lie
    // inside one 128-column block).  Entering block kb they are multiplied by s(kb - 1) / s(kb), the MFMAs of
    // the block then accumulate raw code products on top, and the epilogue multiplies by the last s: the sum
    // over kb of s(kb) * P(kb) without a second set of accumulators for the per-block partial products P.  The
    // 16 multiplies per tile and K step sit in front of the tile's first MFMA of the step (the vector ALU is idle
    // there).  One extra fp32 rounding of the running sum per K step (and a 1-ulp reciprocal in the ratio):
    // K / 128 * 2^-23 relative to sum |terms|, two orders below the matrix pipe's own truncation.
    // The scales of block k + 1 are fetched at the start of step k.
    // Power-of-two block scales (BW == 2): every scale is 2^(e - 127) with e its fp32 exponent field, which is the
    // 8-bit scale format of the scaled MFMA: the instruction multiplies the products of a 32-element K run by
    // 2^(ea - 127) * 2^(eb - 127), ea / eb taken from the lane that holds the run.  A lane's X fragment is one
    // row's run (scale of that row and K block), a W fragment's 32 rows lie in one 128-column block (one scale
    // for the wave).  The accumulators then hold the scaled sum itself and the epilogue multiplies by nothing.
    // X's block scales lie [row][K block]: a lane reading one value per K step touches a cache line of its own each
    // time (as many L2 requests per step as the operands themselves need).  When a row's scales are 16-byte aligned
    // (K a multiple of 512) a lane fetches four K blocks at once, every fourth step.
    float s_cur[MI], r_sc[MI], sx_nx[MI], sw_nx = 0.f;
    v4f sx_q[MI];
    const bool quad = BLOCKWISE && (ksteps & 3) == 0;
    auto pick = [](const v4f& v, int j) __attribute__((always_inline)) {
        return j == 0 ? v[0] : j == 1 ? v[1] : j == 2 ? v[2] : v[3];
    };
    int sc_x[MI], sc_w = 127;
    const int bw_nb = ((n0 + wave_n * WN < p.N ? n0 + wave_n * WN : p.N - 1) >> 7), bw_nblk = p.N >> 7;
    auto bw_row = [&](int mi) __attribute__((always_inline)) {
        const int m = m0 + wave_m * WM + mi * 32 + l32;
        return static_cast<int64_t>(m < p.M ? m : p.M - 1) * ksteps;
    };
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        s_cur[mi] = 1.f; r_sc[mi] = 1.f; sx_nx[mi] = 1.f; sc_x[mi] = 127;
        sx_q[mi] = v4f{1.f, 1.f, 1.f, 1.f};
    }
    if (BLOCKWISE) {
        const float sw0 = swg[bw_nb];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            float sx0;
            if (quad) { sx_q[mi] = *reinterpret_cast<const v4f*>(sxg + bw_row(mi)); sx0 = sx_q[mi][0]; }
            else sx0 = sxg[bw_row(mi)];
            if (BW == 1) s_cur[mi] = sx0 * sw0;
            else sc_x[mi] = static_cast<int>(__float_as_uint(sx0) >> 23);
        }
        if (BW == 2) sc_w = static_cast<int>(__float_as_uint(sw0) >> 23);
    }
    // ratio for the step that begins (its scales were fetched one step earlier), then the fetch for the next one
    auto bw_step = [&](int k) __attribute__((always_inline)) {
        if (!BLOCKWISE) return;
        if (k >= 1 && quad) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) sx_nx[mi] = pick(sx_q[mi], k & 3);
        }
        if (k >= 1 && BW == 1) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const float s_new = sx_nx[mi] * sw_nx;
                r_sc[mi] = s_cur[mi] * __builtin_amdgcn_rcpf(s_new);
                s_cur[mi] = s_new;
            }
        }
        if (k >= 1 && BW == 2) {
            sc_w = static_cast<int>(__float_as_uint(sw_nx) >> 23);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) sc_x[mi] = static_cast<int>(__float_as_uint(sx_nx[mi]) >> 23);
        }
        if (k + 1 < ksteps) {
            sw_nx = swg[static_cast<int64_t>(k + 1) * bw_nblk + bw_nb];
            if (!quad) {
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) sx_nx[mi] = sxg[bw_row(mi) + k + 1];
            } else if (((k + 1) & 3) == 0) {
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) sx_q[mi] = *reinterpret_cast<const v4f*>(sxg + bw_row(mi) + k + 1);
            }
        }
    };

    // Fragments of one K half (64 bytes): 2 W (two sets, double buffered) and 4 X (one set, refilled in place
    // as soon as the two MFMAs that use a fragment have been issued) of 8 registers each.
    v8i bx[MI], aw[2][NI];
    auto read_w = [&](int slot, int s, int set) __attribute__((always_inline)) {
        const uint8_t* ws = smem + slot * ES;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const v4i lo = *reinterpret_cast<const v4i*>(ws + (w_off0 ^ (s << 6)) + ni * 32 * 128);
            const v4i hi = *reinterpret_cast<const v4i*>(ws + (w_off1 ^ (s << 6)) + ni * 32 * 128);
            aw[set][ni] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
    };
    auto read_x = [&](int slot, int s, int mi) __attribute__((always_inline)) {
        const uint8_t* xs = smem + slot * ES + mi * 32 * 128;
        const v4i lo = *reinterpret_cast<const v4i*>(xs + (x_off0 ^ (s << 6)));
        const v4i hi = *reinterpret_cast<const v4i*>(xs + (x_off1 ^ (s << 6)));
        bx[mi] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    };
    auto mfma_one = [&](int mi, int ni, int set) __attribute__((always_inline)) {
        if (BW == 2)
            acc[mi][ni] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(aw[set][ni], bx[mi], acc[mi][ni], 0, 0, 0, sc_w, 0,
                                                                         sc_x[mi]);
        else
            acc[mi][ni] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(aw[set][ni], bx[mi], acc[mi][ni], 0, 0, 0, 0, 0, 0);
    };
    auto mfma_row = [&](int mi, int set) __attribute__((always_inline)) {
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) mfma_one(mi, ni, set);
    };
    // MFMAs of the K half whose W fragments are in SET, with the LDS reads of K half S_READ of the entries in
    // slots SLOT_X / SLOT_W, and this wave's four loads of one new ring entry (LD: 0 none, 1 an X entry, 2 a W
    // entry; into ld_slot, K offset ld_kb), spread between them in source order.  The matrix pipe then always
    // has an instruction queued: a burst of LDS reads or of loads keeps a wave in the issue stage for hundreds
    // of cycles (the load path accepts 64 bytes per clock per CU).  The two waves of a SIMD (w, w + 4) issue
    // their loads in different gaps, so one of them is always free to feed the pipe.
#define LOKA_HALF_STEP(SLOT_X, SLOT_W, S_READ, SET, LD, RESC)                              \
    do {                                                                             \
        __builtin_amdgcn_sched_barrier(0);                                           \
        read_w(SLOT_W, S_READ, (SET) ^ 1);                                           \
        _Pragma("unroll") for (int mi = 0; mi < MI; ++mi) {                          \
            __builtin_amdgcn_sched_barrier(0);                                       \
            if (BW == 1 && (RESC)) {                                                 \
                _Pragma("unroll") for (int ni = 0; ni < NI; ++ni)                    \
                    _Pragma("unroll") for (int i = 0; i < 16; ++i) acc[mi][ni][i] *= r_sc[mi]; \
            }                                                                        \
            mfma_one(mi, 0, SET);                                                    \
            __builtin_amdgcn_sched_barrier(0);                                       \
            if ((LD) == 1 && ld_x && !grp_b) issue_x1(ld_x_slot, ld_x_kb, mi);       \
            if ((LD) == 2 && ld_w && !grp_b) issue_w1(ld_w_slot, ld_w_kb, mi);       \
            __builtin_amdgcn_sched_barrier(0);                                       \
            mfma_one(mi, 1, SET);                                                    \
            __builtin_amdgcn_sched_barrier(0);                                       \
            read_x(SLOT_X, S_READ, mi);                                              \
            if ((LD) == 1 && ld_x && grp_b) issue_x1(ld_x_slot, ld_x_kb, mi);        \
            if ((LD) == 2 && ld_w && grp_b) issue_w1(ld_w_slot, ld_w_kb, mi);        \
        }                                                                            \
        __builtin_amdgcn_sched_barrier(0);                                           \
    } while (0)

    // ---- main loop.  LDS holds a ring of five 32 KB entries X(0) W(0) X(1) W(1) X(2) ...; entry e lives in
    // slot e % 5.  One barrier per K step, in its middle, when every wave has read X(k) and W(k) completely and
    // every wave's share of X(k + 1), W(k + 1) has landed.  The slot of X(k) then takes W(k + 2) (loads issued
    // in the second half of step k), the slot of W(k) takes X(k + 3) (first half of step k + 1): an X entry is
    // requested 1.5 steps before its first read, a W entry one step (half the bytes of a stage: the round
    // trip through L2 under load is ~1 us for 64 KB, ~0.6 us for 32 KB; a step is ~1.2 us).
    // All of a wave's loads return in issue order, so "vmcnt(4)" = everything but the newest entry's share.
    auto mod5 = [](int v) { return v >= 5 ? v - 5 : v; };
    // entry e of a tile lives in slot (e + 1) % 5: slot 0, which the epilogue uses as scratch, is the last to fill
    if (!prefetched) {
        issue_x(1, 0);
        issue_w(2, 0);
        if (ksteps > 1) { issue_x(3, 128); issue_w(4, 128); }
    }
    if (ksteps > 2) issue_x(0, 256);
    if (ksteps > 2) {
        // loads return in issue order, so "at most 4 (12) outstanding" covers X(0), W(0) whatever else (the
        // previous tile's stores) is still in flight
        if (prefetched) __builtin_amdgcn_s_waitcnt(0x0F74); else __builtin_amdgcn_s_waitcnt(0x0F7C);
    } else if (ksteps > 1 && !prefetched) {
        __builtin_amdgcn_s_waitcnt(0x0F78);
    } else {
        __builtin_amdgcn_s_waitcnt(0x0F70);
    }
    lds_barrier();
    read_w(2, 0, 0);
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) read_x(1, 0, mi);
    int e5 = 1;                                                 // slot of X(k)
    // (the last K step is peeled: MFMAs under a condition inside the loop make the compiler copy accumulators)
    for (int k = 0; k + 1 < ksteps; ++k) {
        const int sw_cur = mod5(e5 + 1), sx_nxt = mod5(e5 + 2), sw_nxt = mod5(e5 + 3);
        const bool ld_x = k >= 1 && k + 2 < ksteps, ld_w = k + 2 < ksteps;
        const int ld_x_slot = mod5(e5 + 4), ld_x_kb = (k + 2) * 128;    // X(k + 2) -> the slot W(k - 1) left
        const int ld_w_slot = e5, ld_w_kb = (k + 2) * 128;              // W(k + 2) -> the slot X(k) leaves
        bw_step(k);
        LOKA_HALF_STEP(e5, sw_cur, 1, 0, 1, 1);
        // all but this step's newest loads: X(k + 2) (4) and, blockwise, the scales of block k + 1 (MI + 1)
        if (ld_w) { if (BLOCKWISE) __builtin_amdgcn_s_waitcnt(0x0F79); else __builtin_amdgcn_s_waitcnt(0x0F74); }
        else __builtin_amdgcn_s_waitcnt(0x0F70);
        lds_barrier();                                          // (also waits for this wave's LDS reads)
        LOKA_HALF_STEP(sx_nxt, sw_nxt, 0, 1, 2, 0);
        e5 = sx_nxt;
    }
    {
        const bool ld_x = false, ld_w = false;
        const int ld_x_slot = 0, ld_x_kb = 0, ld_w_slot = 0, ld_w_kb = 0;
        bw_step(ksteps - 1);
        LOKA_HALF_STEP(e5, mod5(e5 + 1), 1, 0, 0, 1);
        (void)ld_x; (void)ld_w; (void)ld_x_slot; (void)ld_x_kb; (void)ld_w_slot; (void)ld_w_kb;
    }
    {   // Epilogue scope.  Lane- and thread-derived offsets restart from opaque copies of the ids: derived from
        // loop-invariant values the compiler would compute them once before the tile loop and keep dozens of
        // registers live through the main loop.
    int lane_o = static_cast<int>(threadIdx.x) & 63, tid_o = static_cast<int>(threadIdx.x);
    asm volatile("; epilogue ids" : "+v"(lane_o), "+v"(tid_o));
    const int lane = lane_o, l32 = lane & 31, hk = lane >> 5;
    const unsigned tid = static_cast<unsigned>(tid_o);
    (void)lane;
    int n_o = p.N;                                          // (1 / N likewise: recomputed per tile, not kept in a register)
    asm volatile("; row length" : "+s"(n_o));
    const float inv_n = 1.0f / static_cast<float>(n_o);
    // scales of this lane's rows and columns: requested before the last eight MFMAs so that the round trip
    // through L2 is covered (the fragment registers of the other K half are free by now)
    // lane: rows m(mi) = m0 + 128 wave_m + 32 mi + l32; columns ncol(ni) + [0, 16), ncol = n0 + 64 wave_n + 32 ni + 16 hk
    const bool tensor_x = p.x_mode == LOKA_SCALE_TENSOR, tensor_w = p.w_mode == LOKA_SCALE_TENSOR;
    int ncol[NI];
    float cnt_lane = 0.f;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        ncol[ni] = n0 + wave_n * WN + ni * 32 + hk * 16;
        if (ncol[ni] < p.N) cnt_lane += 16.f;               // N % 16 == 0: a run of 16 is all in or all out
    }
    v4f s4[NI][4];
    float sxm[MI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            if (BLOCKWISE) s4[ni][a] = v4f{1.f, 1.f, 1.f, 1.f};
            else if (tensor_w) { const float s = swg[0]; s4[ni][a] = v4f{s, s, s, s}; }
            else s4[ni][a] = ncol[ni] < p.N ? *reinterpret_cast<const v4f*>(swg + ncol[ni] + 4 * a) : v4f{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        int m = m0 + wave_m * WM + mi * 32 + l32;
        m = m < p.M ? m : p.M - 1;
        sxm[mi] = BW == 1 ? s_cur[mi] : BW == 2 ? 1.f : tensor_x ? sxg[0] : sxg[m];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) mfma_row(mi, 1);
#undef LOKA_HALF_STEP
    __syncthreads();                                        // LDS is free for the epilogue
    // the next tile's first four ring entries stream in while this tile's statistics are exchanged
    prefetched = tile + tile_stride < total_tiles;
    if (prefetched) {
        set_rsrc(tile + tile_stride);
        issue_x(1, 0);
        issue_w(2, 0);
        if (ksteps > 1) { issue_x(3, 128); issue_w(4, 128); }
    }

    // ------------------------------------------------------------------ epilogue
    float* red = reinterpret_cast<float*>(smem);                                   // [BM][4][3]
    float2* fin = reinterpret_cast<float2*>(smem) + BM * 4 * 3 / 2 + 8;            // [BM] (mean, rstd)
    float* finq = reinterpret_cast<float*>(fin + BM);                              // [BM] 448 / amax of the output row (FP8OUT)
    float* red2 = reinterpret_cast<float*>(smem + 16384);                          // [BM][4][2] (min, max) (FP8OUT); the
                                                                                   // transpose buffers take its place later
    const int64_t obase = static_cast<int64_t>(g) * p.strideO;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][ni][i] *= s4[ni][i >> 2][i & 3] * sxm[mi];
    if (p.y) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int m = m0 + wave_m * WM + mi * 32 + l32;
            if (m < p.M) {
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    if (ncol[ni] < p.N) {
                        float* dst = p.y + obase + static_cast<int64_t>(m) * p.N + ncol[ni];
#pragma unroll
                        for (int a = 0; a < 4; ++a)
                            *reinterpret_cast<v4f*>(dst + 4 * a) =
                                v4f{acc[mi][ni][4 * a], acc[mi][ni][4 * a + 1], acc[mi][ni][4 * a + 2], acc[mi][ni][4 * a + 3]};
                    }
            }
        }
    }

    float mean_r[MI], rstd_r[MI];
    const bool ln = p.norm == LOKA_NORM_LAYERNORM;
    // FP8 output with gamma / beta: the row amax is only known after the affine step, and crosses the workgroups in
    // a second exchange (below); the row extremes of the pre-norm values are then of no use
    constexpr bool affine_q = F8 == 2;
    float iq_r[MI];
    if (p.norm == LOKA_NORM_NONE) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) { mean_r[mi] = 0.f; rstd_r[mi] = 1.f; iq_r[mi] = 1.f; }
    } else {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            float n_ = cnt_lane, mean = 0.f, m2 = 0.f;
            if (ln) {
                float s = 0.f;
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    if (ncol[ni] < p.N) {
#pragma unroll
                        for (int i = 0; i < 16; ++i) s += acc[mi][ni][i];
                    }
                mean = n_ > 0.f ? s * __builtin_amdgcn_rcpf(n_) : 0.f;
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    if (ncol[ni] < p.N) {
#pragma unroll
                        for (int i = 0; i < 16; ++i) { const float d = acc[mi][ni][i] - mean; m2 = __builtin_fmaf(d, d, m2); }
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
                for (int ni = 0; ni < NI; ++ni)
                    if (ncol[ni] < p.N) {
#pragma unroll
                        for (int i = 0; i < 16; ++i) m2 = __builtin_fmaf(acc[mi][ni][i], acc[mi][ni][i], m2);
                    }
                m2 += wave_shfl_xor(m2, 32);
            }
            if (hk == 0) {
                float* r3 = red + ((wave_m * WM + mi * 32 + l32) * 4 + wave_n) * 3;
                r3[0] = n_; r3[1] = mean; r3[2] = m2;
            }
            if (FP8OUT && !affine_q) {
                float lo = __builtin_inff(), hi = -__builtin_inff();
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    if (ncol[ni] < p.N) {
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            lo = __builtin_fminf(lo, acc[mi][ni][i]);
                            hi = __builtin_fmaxf(hi, acc[mi][ni][i]);
                        }
                    }
                lo = __builtin_fminf(lo, wave_shfl_xor(lo, 32));
                hi = __builtin_fmaxf(hi, wave_shfl_xor(hi, 32));
                if (hk == 0) {
                    float* r2 = red2 + ((wave_m * WM + mi * 32 + l32) * 4 + wave_n) * 2;
                    r2[0] = lo; r2[1] = hi;
                }
            }
        }
        __syncthreads();
        // tile statistics per row: thread r < 256 merges the four column waves in order
        float t_mean = 0.f, t_m2 = 0.f, t_lo = __builtin_inff(), t_hi = -__builtin_inff();
        if (tid < BM) {
            float n_ = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float* r3 = red + (tid * 4 + w) * 3;
                if (ln) merge_stats(n_, t_mean, t_m2, r3[0], r3[1], r3[2]);
                else t_m2 += r3[2];
                if (FP8OUT && !affine_q) {
                    t_lo = __builtin_fminf(t_lo, red2[(tid * 4 + w) * 2]);
                    t_hi = __builtin_fmaxf(t_hi, red2[(tid * 4 + w) * 2 + 1]);
                }
            }
        }
        // FP8OUT: the row scale from the row's extreme pre-norm values, through the very operations the
        // normalization applies to every element (one fused multiply-add, bf16 rounding)
        auto row_scale = [&](int r, float mean, float rstd, float lo, float hi) __attribute__((always_inline)) {
            const float nmr = -mean * rstd;
            const unsigned pk = pack_bf16x2(__builtin_fmaf(lo, rstd, nmr), __builtin_fmaf(hi, rstd, nmr));
            const unsigned a = pk & 0x7FFFu, b = (pk >> 16) & 0x7FFFu;
            float scale, inv;
            group_scale(__uint_as_float((a > b ? a : b) << 16), scale, inv);
            if (!(rstd == rstd)) scale = rstd;                    // poisoned row: the scale says so
            finq[r] = inv;
            if (tn == 0 && m0 + r < p.M) p.outs[static_cast<int64_t>(g) * p.M + m0 + r] = scale;
        };
        const bool blocknorm = p.norm == LOKA_NORM_BLOCKNORM;   // groups of 256 columns = this tile: nothing to exchange
        bool arrived = true;                                    // false: a wait for the panel's other tiles ran out
        int* const lds_word = reinterpret_cast<int*>(smem + 16000);   // (free between finq and red2)
        if (EPI == EPI_PANEL_SYNC && !blocknorm && p.tiles_n > 1) {
            // publish (mean, M2) of this tile per row, signal, wait for the panel's other tiles, merge all tiles
            const int panel = g * p.tiles_m + tm;
            // Exchange area of a panel: [tiles_n][256 rows] records of 8 bytes, so that a tile's 256 threads write
            // one contiguous 2 KB run and the merging threads of consecutive rows read consecutive records (a
            // row-major [row][tile] layout makes every lane of a load touch a cache line of its own, and the 256
            // workgroups' merges then queue at the L2 channels).  (min, max) per row and tile: a second array of the
            // same shape behind the statistics of all panels.
            unsigned long long* pbase = reinterpret_cast<unsigned long long*>(p.part) + static_cast<int64_t>(panel) * p.tiles_n * BM;
            const int64_t mm_off = static_cast<int64_t>(p.batch) * p.tiles_m * p.tiles_n * BM;
            if (tid < BM) {
                unsigned long long* dst = pbase + tn * BM + tid;
                __hip_atomic_store(dst, static_cast<unsigned long long>(__float_as_uint(t_mean)) |
                                            (static_cast<unsigned long long>(__float_as_uint(t_m2)) << 32),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (FP8OUT && !affine_q)
                    __hip_atomic_store(dst + mm_off, static_cast<unsigned long long>(__float_as_uint(t_lo)) |
                                                         (static_cast<unsigned long long>(__float_as_uint(t_hi)) << 32),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            arrived = panel_publish_and_wait(p, p.flags + static_cast<int64_t>(panel) * p.tiles_n, tn, p.tiles_n, lds_word);
            // two threads per row, each folds a contiguous half of the row's tiles in order (device-coherent
            // 8-byte loads), symmetric merge of the halves: identical bits in every workgroup of the panel
            {
                const int r = static_cast<int>(tid) >> 1, sub = static_cast<int>(tid) & 1;
                const unsigned long long* src = pbase + r;
                const int TH = (p.tiles_n + 1) >> 1;
                float n_ = 0.f, mean = 0.f, m2 = 0.f, lo = __builtin_inff(), hi = -__builtin_inff();
                for (int t0 = sub * TH; t0 < (sub + 1) * TH && t0 < p.tiles_n; t0 += 8) {
                    unsigned long long raw[8], raw2[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        int tt = t0 + u;
                        tt = tt < p.tiles_n ? tt : p.tiles_n - 1;
                        raw[u] = __hip_atomic_load(src + tt * BM, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        if (FP8OUT && !affine_q) raw2[u] = __hip_atomic_load(src + mm_off + tt * BM, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int tt = t0 + u;
                        if (tt < (sub + 1) * TH && tt < p.tiles_n) {
                            const float a = __uint_as_float(static_cast<unsigned>(raw[u]));
                            const float b2 = __uint_as_float(static_cast<unsigned>(raw[u] >> 32));
                            const int wcols = (tt + 1) * BN <= p.N ? BN : p.N - tt * BN;
                            if (ln) merge_stats(n_, mean, m2, static_cast<float>(wcols), a, b2);
                            else m2 += b2;
                            if (FP8OUT && !affine_q) {
                                lo = __builtin_fminf(lo, __uint_as_float(static_cast<unsigned>(raw2[u])));
                                hi = __builtin_fmaxf(hi, __uint_as_float(static_cast<unsigned>(raw2[u] >> 32)));
                            }
                        }
                    }
                }
                const float nb = wave_shfl_xor(n_, 1), mb = wave_shfl_xor(mean, 1), m2b = wave_shfl_xor(m2, 1);
                if (ln) {
                    const float nn = n_ + nb;
                    if (nn > 0.f) {
                        const float d = mb - mean;
                        const float rn = __builtin_amdgcn_rcpf(nn);
                        const float newmean = (n_ * mean + nb * mb) * rn;
                        m2 = m2 + m2b + d * d * (n_ * nb * rn);
                        mean = newmean;
                    }
                } else {
                    m2 = m2 + m2b;
                }
                if (FP8OUT && !affine_q) {
                    lo = __builtin_fminf(lo, wave_shfl_xor(lo, 1));
                    hi = __builtin_fmaxf(hi, wave_shfl_xor(hi, 1));
                }
                if (sub == 0) {
                    // (a wait that ran out: the statistics are not to be trusted; the tile's rows leave as NaN, their
                    // FP8 row scale as NaN)
                    const float2 f = arrived ? make_float2(ln ? mean : 0.f, __builtin_amdgcn_rsqf(m2 * inv_n + p.eps))
                                             : make_float2(__builtin_nanf(""), __builtin_nanf(""));
                    fin[r] = f;
                    if (FP8OUT && !affine_q) row_scale(r, f.x, f.y, lo, hi);
                }
            }
        } else {
            // the tile spans the whole row (N <= 256): finalize here
            if (tid < BM) {
                const float2 f = make_float2(ln ? t_mean : 0.f, __builtin_amdgcn_rsqf(t_m2 * (blocknorm ? 1.0f / BN : inv_n) + p.eps));
                fin[tid] = f;
                if (FP8OUT && !affine_q) row_scale(static_cast<int>(tid), f.x, f.y, t_lo, t_hi);
            }
        }
        __syncthreads();
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const float2 f = fin[wave_m * WM + mi * 32 + l32];
            mean_r[mi] = f.x;
            rstd_r[mi] = f.y;
            if (FP8OUT && !affine_q) iq_r[mi] = finq[wave_m * WM + mi * 32 + l32];
        }
    }
    float nmr_r[MI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) nmr_r[mi] = -mean_r[mi] * rstd_r[mi];

    // ---- normalize, affine, bf16 store.  A lane holds 16 consecutive columns of ONE row per 32 x 32 sub-tile;
    // stored from there, an instruction would touch 32 rows with 32 bytes each.  Each wave instead passes the
    // sub-tile through 2 KB of its own LDS (64-byte rows, 16-byte chunk c of row r at position c ^ (r / 4 % 4):
    // conflict-free both ways) and stores it with 4 lanes per row: 16 full 64-byte runs per instruction.
    // LDS executes one wave's instructions in order, so the same buffer serves every sub-tile without a barrier.
    const bool has_g = p.gamma != nullptr && (ln || p.norm == LOKA_NORM_RMSNORM), has_b = p.beta != nullptr && ln;
    const bool hswish = p.act == LOKA_ACT_HARDSWISH;
    // gamma and beta of this lane's 16 columns of sub-tile ni (1 and 0 where absent or past N)
    auto load_affine = [&](int ni, float (&gm)[16], float (&bt)[16]) __attribute__((always_inline)) {
#pragma unroll
        for (int e = 0; e < 16; ++e) { gm[e] = 1.f; bt[e] = 0.f; }
        if (ncol[ni] >= p.N) return;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            if (has_g) {
                const u32x4 w = *reinterpret_cast<const u32x4*>(p.gamma + ncol[ni] + 8 * half);
                float* q = gm + 8 * half;
                q[0] = bf16_lo(w.x); q[1] = bf16_hi(w.x); q[2] = bf16_lo(w.y); q[3] = bf16_hi(w.y);
                q[4] = bf16_lo(w.z); q[5] = bf16_hi(w.z); q[6] = bf16_lo(w.w); q[7] = bf16_hi(w.w);
            }
            if (has_b) {
                const u32x4 w = *reinterpret_cast<const u32x4*>(p.beta + ncol[ni] + 8 * half);
                float* q = bt + 8 * half;
                q[0] = bf16_lo(w.x); q[1] = bf16_hi(w.x); q[2] = bf16_lo(w.y); q[3] = bf16_hi(w.y);
                q[4] = bf16_lo(w.z); q[5] = bf16_hi(w.z); q[6] = bf16_lo(w.w); q[7] = bf16_hi(w.w);
            }
        }
    };
    uint8_t* const tbuf = smem + 16384 + wave * 2048;
    const int t_wr = l32 * 64, t_key = (l32 >> 2) & 3;
    const int t_row = lane >> 2, t_c = lane & 3;                       // store side: row (+ 16 j), chunk
    if (FP8OUT) {
        (void)hswish;
        // With gamma / beta: the normalized bf16 values replace the accumulators (64 packed registers), their row
        // amax crosses the waves through LDS and the workgroups through a second exchange (records in the area the
        // row extremes use otherwise, a second arrival counter per panel), and the cast follows.
        unsigned opk[MI][NI][4][2];
        if (affine_q) {
            unsigned am[MI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) am[mi] = 0u;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                float gm[16], bt[16];
                load_affine(ni, gm, bt);
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float o[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            o[e] = __builtin_fmaf(acc[mi][ni][4 * q + e], rstd_r[mi], nmr_r[mi]);
                            if (has_g || has_b) o[e] = __builtin_fmaf(o[e], gm[4 * q + e], bt[4 * q + e]);
                            if (hswish) o[e] = o[e] * __builtin_fminf(__builtin_fmaxf(o[e] + 3.0f, 0.0f), 6.0f) * (1.0f / 6.0f);
                        }
                        const unsigned p0 = pack_bf16x2(o[0], o[1]), p1 = pack_bf16x2(o[2], o[3]);
                        opk[mi][ni][q][0] = p0; opk[mi][ni][q][1] = p1;
                        if (ncol[ni] < p.N) {
                            const unsigned a0 = p0 & 0x7FFFu, a1 = (p0 >> 16) & 0x7FFFu, a2 = p1 & 0x7FFFu, a3 = (p1 >> 16) & 0x7FFFu;
                            const unsigned a01 = a0 > a1 ? a0 : a1, a23 = a2 > a3 ? a2 : a3;
                            const unsigned a = a01 > a23 ? a01 : a23;
                            am[mi] = am[mi] > a ? am[mi] : a;
                        }
                    }
            }
            unsigned* amw = reinterpret_cast<unsigned*>(smem + 16384);        // [BM][4]: row amax per column wave
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const unsigned other = static_cast<unsigned>(__shfl_xor(static_cast<int>(am[mi]), 32, 64));
                am[mi] = am[mi] > other ? am[mi] : other;
                if (hk == 0) amw[(wave_m * WM + mi * 32 + l32) * 4 + wave_n] = am[mi];
            }
            __syncthreads();
            unsigned t_am = 0u;
            if (tid < BM) {
#pragma unroll
                for (int w = 0; w < 4; ++w) { const unsigned a = amw[tid * 4 + w]; t_am = t_am > a ? t_am : a; }
            }
            bool amax_ok = true;
            auto row_scale_am = [&](int r, unsigned a) __attribute__((always_inline)) {
                float scale, inv;
                group_scale(__uint_as_float(a << 16), scale, inv);
                if (!amax_ok) scale = __builtin_nanf("");           // the wait for the other tiles' amax ran out
                finq[r] = inv;
                if (tn == 0 && m0 + r < p.M) p.outs[static_cast<int64_t>(g) * p.M + m0 + r] = scale;
            };
            if (p.tiles_n > 1) {
                const int panel = g * p.tiles_m + tm;
                const int64_t mm_off = static_cast<int64_t>(p.batch) * p.tiles_m * p.tiles_n * BM;
                unsigned long long* pam = reinterpret_cast<unsigned long long*>(p.part) + mm_off +
                                          static_cast<int64_t>(panel) * p.tiles_n * BM;
                if (tid < BM) {
                    __hip_atomic_store(pam + tn * BM + tid, static_cast<unsigned long long>(t_am), __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                }
                // (the second set of arrival words of the panel)
                const bool arrived2 = panel_publish_and_wait(
                    p, p.flags + (static_cast<int64_t>(p.batch) * p.tiles_m + panel) * p.tiles_n, tn, p.tiles_n,
                    reinterpret_cast<int*>(smem + 16000));
                amax_ok = arrived2;
                {
                    const int r = static_cast<int>(tid) >> 1, sub = static_cast<int>(tid) & 1;
                    const int TH = (p.tiles_n + 1) >> 1;
                    unsigned a = 0u;
                    for (int t0 = sub * TH; t0 < (sub + 1) * TH && t0 < p.tiles_n; t0 += 8) {
                        unsigned long long raw[8];
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            int tt = t0 + u;
                            tt = tt < p.tiles_n ? tt : p.tiles_n - 1;
                            raw[u] = __hip_atomic_load(pam + tt * BM + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        }
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            const unsigned v = static_cast<unsigned>(raw[u]);      // (a clamped index repeats a tile: harmless for a maximum)
                            a = a > v ? a : v;
                        }
                    }
                    const unsigned other = static_cast<unsigned>(__shfl_xor(static_cast<int>(a), 1, 64));
                    a = a > other ? a : other;
                    if (sub == 0) row_scale_am(r, a);
                }
            } else if (tid < BM) {
                row_scale_am(static_cast<int>(tid), t_am);
            }
            __syncthreads();
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) iq_r[mi] = finq[wave_m * WM + mi * 32 + l32];
            __syncthreads();                  // amw (aliasing the transpose buffers) and finq are read
        }
        // 16 codes per lane and sub-tile; the wave's 64 columns of 32 rows pass through the transpose buffer at once
        // (64-byte rows of codes) and leave as full 64-byte runs, 4 lanes per row
        const int col = n0 + wave_n * WN + t_c * 16;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                unsigned ck[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    unsigned p0, p1;
                    if (affine_q) {
                        p0 = opk[mi][ni][q][0]; p1 = opk[mi][ni][q][1];
                    } else {
                        float o[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = __builtin_fmaf(acc[mi][ni][4 * q + e], rstd_r[mi], nmr_r[mi]);
                        p0 = pack_bf16x2(o[0], o[1]); p1 = pack_bf16x2(o[2], o[3]);
                    }
                    ck[q] = e4m3x4(bf16_lo(p0) * iq_r[mi], bf16_hi(p0) * iq_r[mi], bf16_lo(p1) * iq_r[mi], bf16_hi(p1) * iq_r[mi]);
                }
                *reinterpret_cast<u32x4*>(tbuf + t_wr + (((2 * ni + hk) ^ t_key) << 4)) = u32x4{ck[0], ck[1], ck[2], ck[3]};
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int r = 16 * j + t_row;
                const u32x4 ck = *reinterpret_cast<const u32x4*>(tbuf + r * 64 + ((t_c ^ ((r >> 2) & 3)) << 4));
                const int m = m0 + wave_m * WM + mi * 32 + r;
                if (m < p.M && col < p.N)
                    __builtin_nontemporal_store(ck, reinterpret_cast<u32x4*>(p.outq + obase + static_cast<int64_t>(m) * p.N + col));
            }
        }
    } else {
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        float gm[16], bt[16];
        load_affine(ni, gm, bt);
        const int col = n0 + wave_n * WN + ni * 32 + t_c * 8;         // store side: this lane's 8 columns
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                float o[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    // (y - mean) * rstd as one fused multiply-add, the affine part as another
                    o[e] = __builtin_fmaf(acc[mi][ni][8 * half + e], rstd_r[mi], nmr_r[mi]);
                    if (has_g || has_b) o[e] = __builtin_fmaf(o[e], gm[8 * half + e], bt[8 * half + e]);
                    if (hswish) o[e] = o[e] * __builtin_fminf(__builtin_fmaxf(o[e] + 3.0f, 0.0f), 6.0f) * (1.0f / 6.0f);
                }
                u32x4 pk;
                pk.x = pack_bf16x2(o[0], o[1]); pk.y = pack_bf16x2(o[2], o[3]);
                pk.z = pack_bf16x2(o[4], o[5]); pk.w = pack_bf16x2(o[6], o[7]);
                *reinterpret_cast<u32x4*>(tbuf + t_wr + (((2 * hk + half) ^ t_key) << 4)) = pk;
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int r = 16 * j + t_row;
                const u32x4 pk = *reinterpret_cast<const u32x4*>(tbuf + r * 64 + ((t_c ^ ((r >> 2) & 3)) << 4));
                const int m = m0 + wave_m * WM + mi * 32 + r;
                if (m < p.M && col < p.N)
                    __builtin_nontemporal_store(pk, reinterpret_cast<u32x4*>(p.out + obase + static_cast<int64_t>(m) * p.N + col));
            }
        }
    }
    }
    }
    lds_barrier();              // the epilogue's scratch (slot 0) is read: the next tile may load into it.  The
                                // stores stay in flight.
  }
}

constexpr size_t kPanel32Lds = 5 * 256 * 128;   // the ring; the epilogue's scratch aliases it

// The normalized value is not a growing function of the pre-norm value along the row: gamma / beta take part (the
// kernel ignores gamma outside LayerNorm / RMSNorm and beta outside LayerNorm), or the row is normalized group by
// group (BlockNorm), or an activation follows.  The FP8-output launch then takes the form with the second exchange.
bool panel32_affine(const GemmParams& p) {
    const bool ln = p.norm == LOKA_NORM_LAYERNORM;
    return (p.gamma != nullptr && (ln || p.norm == LOKA_NORM_RMSNORM)) || (p.beta != nullptr && ln) ||
           p.norm == LOKA_NORM_BLOCKNORM || p.act != LOKA_ACT_NONE;
}
// bw: 0 plain scales, 1 block scales, 2 power-of-two block scales (see the kernel); fp8out with bw == 0 only
const void* panel32_fn(int bw, bool fp8out, bool affine, bool qpro) {
    if (qpro) return (bw != 0 || fp8out) ? nullptr : reinterpret_cast<const void*>(&gemm_panel32_kernel<EPI_PANEL_SYNC, 0, 0, true>);
    if (fp8out) return bw != 0 ? nullptr
                       : affine ? reinterpret_cast<const void*>(&gemm_panel32_kernel<EPI_PANEL_SYNC, 0, 2>)
                                : reinterpret_cast<const void*>(&gemm_panel32_kernel<EPI_PANEL_SYNC, 0, 1>);
    return bw == 2   ? reinterpret_cast<const void*>(&gemm_panel32_kernel<EPI_PANEL_SYNC, 2, 0>)
           : bw == 1 ? reinterpret_cast<const void*>(&gemm_panel32_kernel<EPI_PANEL_SYNC, 1, 0>)
                     : reinterpret_cast<const void*>(&gemm_panel32_kernel<EPI_PANEL_SYNC, 0, 0>);
}
size_t panel32_lds() { return kPanel32Lds; }
void panel32_launch(const GemmParams& p, int bw, dim3 grid, hipStream_t s) {
    if (p.qpro) gemm_panel32_kernel<EPI_PANEL_SYNC, 0, 0, true><<<grid, 512, kPanel32Lds, s>>>(p);
    else if (p.outq && panel32_affine(p)) gemm_panel32_kernel<EPI_PANEL_SYNC, 0, 2><<<grid, 512, kPanel32Lds, s>>>(p);
    else if (p.outq) gemm_panel32_kernel<EPI_PANEL_SYNC, 0, 1><<<grid, 512, kPanel32Lds, s>>>(p);
    else if (bw == 2) gemm_panel32_kernel<EPI_PANEL_SYNC, 2, 0><<<grid, 512, kPanel32Lds, s>>>(p);
    else if (bw == 1) gemm_panel32_kernel<EPI_PANEL_SYNC, 1, 0><<<grid, 512, kPanel32Lds, s>>>(p);
    else gemm_panel32_kernel<EPI_PANEL_SYNC, 0, 0><<<grid, 512, kPanel32Lds, s>>>(p);
}

}  // namespace loka
