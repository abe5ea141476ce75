// FP8 (e4m3) GEMM with the dequantization scales and the row LayerNorm / RMSNorm
// fused into the epilogue, plus the BF16 reference GEMM that shares its skeleton.
//
// Data flow of one workgroup (tile BM rows of X by BN columns of W):
//   global --global_load_lds (16 B per lane, straight into LDS)--> double-buffered
//   K-slices of 128 bytes per row --ds_read_b128--> MFMA operand registers
//   --v_mfma_f32_16x16x128_f8f6f4 (FP8) / v_mfma_f32_16x16x32_bf16--> fp32 accumulators
//   --epilogue in registers + a few LDS words--> bf16 O (and optionally fp32 Y).
//
// Operand roles are swapped on purpose: rows of W feed the MFMA's row operand and rows
// of X its column operand, so D[n][m] lands with lane l holding column m = l % 16 and
// four consecutive n.  The W rows handed to each MFMA are permuted so that each pair of
// MFMA tiles gives a lane 8 CONSECUTIVE output columns of one row m, and the four lanes
// that share the row 32 consecutive columns: scales, statistics and 16-byte stores need
// no transpose, and the row statistics need only two cross-lane steps (lanes l, l^16,
// l^32, l^48 share a row).
//
// LDS rows are 128 bytes = 8 chunks of 16 bytes; chunk c of row r is stored at chunk
// position c ^ key(r).  The LDS has 64 banks of 4 bytes and serves a ds_read_b128 sixteen
// lanes at a time, so the 16 rows those lanes address must differ in (row parity, chunk
// position): key(r) takes 8 values over the 8 same-parity rows of each operand's read pattern.
#include "gemm_common.h"

#include <atomic>
#include <chrono>
#include <mutex>
#include <vector>

namespace loka {

// Eight e4m3 codes (two 32-bit words) widened to bf16 in registers: every e4m3 value is a bf16 value, so the
// conversion is exact, and the BF16 matrix instruction multiplies bf16 operands exactly (a 16-bit significand product
// fits the fp32 accumulator's input).  The EXACT instantiations contract FP8 operands this way: FP8's memory traffic,
// no alignment loss inside the matrix pipe (the FP8 instructions align the 8 products of a group to the largest and
// drop what falls 14 bits below), twice the matrix-pipe time.
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
__device__ __forceinline__ v8bf e4m3x8_to_bf16(int w0, int w1) {
    const v2bf a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w0, 1.0f, false);
    const v2bf b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w0, 1.0f, true);
    const v2bf c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w1, 1.0f, false);
    const v2bf d = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w1, 1.0f, true);
    return v8bf{a[0], a[1], b[0], b[1], c[0], c[1], d[0], d[1]};
}

// Stages of 128 bytes per row kept in LDS, and the bytes a launch asks for: two stages (one in flight) everywhere but in
// the eight-wave form of the split-K schedule, whose short chains of K steps need several loads in flight to hide the
// memory latency (its ring also carries 1 KB of block scales per stage).
constexpr int gemm_stages(int epi, int waves) { return (epi == EPI_SPLITK && waves == 8) ? 4 : 2; }
constexpr size_t gemm_lds_bytes(int bm, int bn_sub, int epi, int waves) {
    return static_cast<size_t>(gemm_stages(epi, waves)) * (bm * 128 + bn_sub * 128 + (gemm_stages(epi, waves) > 2 ? 1024 : 0));
}

template <int BM, int BN_SUB, int NSPLIT, int WAVES_M, int WAVES_N, bool IS_BF16, bool BLOCKWISE, int EPI, bool EXACT = false>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void gemm_kernel(const GemmParams p) {
    static_assert(!EXACT || (!IS_BF16 && !BLOCKWISE), "the exact-product form is built for the non-blockwise FP8 recipes");
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WM = BM / WAVES_M;           // rows of X per wave
    constexpr int WN = BN_SUB / WAVES_N;       // columns per wave and N-part
    constexpr int MI = WM / 16;
    constexpr int NI = WN / 16;
    constexpr int BN = BN_SUB * NSPLIT;
    constexpr int XS = BM * 128;               // bytes of one X stage
    constexpr int WS = BN_SUB * 128;           // bytes of one W stage
    constexpr int NST = gemm_stages(EPI, NW);  // stages in LDS (split K with eight waves: a ring of 4, three in flight)
    constexpr bool RING = NST > 2;
    static_assert(WM % 16 == 0 && WN % 16 == 0 && (NI == 2 || NI == 4 || NI == 8), "tile shape");
    static_assert(BM % 8 == 0 && BN_SUB % 8 == 0, "loader works on 8-row groups");
    static_assert(!(BLOCKWISE && (WN > 128 || 128 % WN)), "a wave's columns must stay inside one 128-column block");

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    uint8_t* const xbuf = smem;                // NST stages
    uint8_t* const wbuf = smem + NST * XS;     // NST stages

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
    const int l16 = lane & 15, q = lane >> 4;

    // Tiles are enumerated (problem, m tile, n tile), n fastest.  The one-tile-per-workgroup schedules
    // take tile blockIdx.x.  The panel-synchronous schedule is persistent: gridDim.x (a multiple of
    // tiles_n, all co-resident) workgroups walk the tile list in rounds of gridDim.x tiles, so the
    // tiles_n workgroups that share a row panel always run in the same round.  Workgroups are handed
    // to the 8 XCDs round-robin; logical slot (id % 8) * (grid / 8) + id / 8 keeps a panel's
    // workgroups (and the W tiles they stream) on one XCD's L2 when grid is a multiple of 8 * tiles_n.
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
  for (int tile = tile_first; tile < total_tiles; tile += tile_stride) {
    int t = tile;
    const int tn = t % p.tiles_n; t /= p.tiles_n;
    const int tm = t % p.tiles_m; t /= p.tiles_m;
    // EPI_SPLITK: the launch has ksplit workgroups per output tile (blockIdx.y), each contracts its own range of K steps
    const int g = t;
    const int ks = EPI == EPI_SPLITK ? static_cast<int>(blockIdx.y) : 0;
    const int k_lo = ks * p.k_per_split;                       // first K step of this workgroup
    const int kb0 = k_lo * 128;
    const int m0 = tm * BM, n0 = tn * BN;

    const uint8_t* Xg = p.X + static_cast<int64_t>(g) * p.strideX;
    const uint8_t* Wg = p.W + static_cast<int64_t>(g) * p.strideW;

    // ---- loader: one wave-load moves 8 rows x 128 B; lane -> (row lane/8, chunk position lane%8)
    const int ld_row = lane >> 3, ld_pos = lane & 7;
    // X rows are read 16 consecutive rows at a time: key(r) = (r >> 1) & 7
    auto x_key = [](int r) { return (r >> 1) & 7; };
    // W rows are read as rows u*32 + g*8 + v*4 + i (g = 0..3, i = 0..3) of a wave's WN rows:
    // key(r) = ((r >> 1) & 1) | (((r >> 3) & 3) << 1)
    auto w_key = [](int r) { return ((r >> 1) & 1) | (((r >> 3) & 3) << 1); };

    // A stage is XG + WGR groups of 8 rows; wave w loads X groups w, w + NW, ... (entries j < XJ) and
    // W groups w, w + NW, ... (entries j >= XJ); an entry can be issued on its own, so the loads can be
    // spread between the MFMAs of the running stage.
    // Addressing: buffer loads straight into LDS.  One buffer descriptor per operand covers exactly the
    // tile's valid rows (scalar registers), one loop-invariant 32-bit per-lane offset per operand
    // (row-in-group * KB + swizzled chunk * 16; the group-dependent part of the swizzle key depends only
    // on the wave, because NW and XG are multiples of 4), and a uniform scalar offset per entry (group
    // row offset + K offset).  Rows past the end of a ragged M or N tail fall outside the descriptor and
    // load zeros; their results are never stored.
    constexpr int XG = BM / 8, WGR = BN_SUB / 8;
    static_assert(XG % NW == 0 && WGR % NW == 0 && NW % 4 == 0 && XG % 4 == 0, "loader split");
    constexpr int XJ = XG / NW, JN = XJ + WGR / NW;
    const int x_chunk = ((ld_pos ^ (ld_row >> 1)) << 4) ^ ((wave & 1) << 6);       // byte offset inside the 128-byte K step
    const int w_chunk = ((ld_pos ^ ((ld_row >> 1) & 1)) << 4) ^ ((wave & 3) << 5);
    const int x_lane_off = ld_row * p.KB + x_chunk;
    const int w_lane_off = ld_row * p.KB + w_chunk;
    // K need not be a multiple of the 128-byte step (a multiple of 16 bytes is enough): in the last step of such a K the
    // lanes whose 16-byte chunk lies past the end of the row get an offset beyond every descriptor's bound and load
    // zeros (in BOTH operands: a stray NaN code times zero would still be NaN), so the step contracts zeros there.
    const int ktail = p.KB & 127;
    const int x_lane_tail = x_chunk < ktail ? x_lane_off : 0x7FFFFFFF;
    const int w_lane_tail = w_chunk < ktail ? w_lane_off : 0x7FFFFFFF;
    const int x_rows = p.M - m0 < BM ? p.M - m0 : BM, w_rows = p.N - n0 < BN ? p.N - n0 : BN;
    const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(Xg + static_cast<int64_t>(m0) * p.KB), 0, x_rows * p.KB, 0x00020000);
    const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(Wg + static_cast<int64_t>(n0) * p.KB), 0, w_rows * p.KB, 0x00020000);
    auto issue_j = [&](int j, int stage_x, int stage_w, int kb, int h, bool with_x) __attribute__((always_inline)) {
        kb += kb0;
        const bool tail = kb + 128 > p.KB;                    // uniform: the ragged last step
        if (j < XJ) {
            if (with_x) {
                const int grp = wave + j * NW;                // uniform
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    x_rsrc, (__attribute__((address_space(3))) void*)(xbuf + stage_x * XS + grp * 1024), 16,
                    tail ? x_lane_tail : x_lane_off, grp * 8 * p.KB + kb, 0, 0);
            }
        } else {
            const int grp = wave + (j - XJ) * NW;             // uniform
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                w_rsrc, (__attribute__((address_space(3))) void*)(wbuf + stage_w * WS + grp * 1024), 16,
                tail ? w_lane_tail : w_lane_off, (h * BN_SUB + grp * 8) * p.KB + kb, 0, 0);
        }
    };

    // ---- fragment addresses (bytes inside a stage)
    // FP8: a lane supplies K bytes [32q, 32q+32) = chunks 2q, 2q+1 (any K order works as long
    // as both operands use the same one).  BF16: two MFMAs per 128-byte row, lane chunk q and 4+q.
    const int c0 = IS_BF16 ? q : 2 * q, c1 = IS_BF16 ? 4 + q : 2 * q + 1;
    const int xrow = wave_m * WM + l16;                         // + mi * 16
    const int xkey = x_key(xrow);
    const int x_off0 = xrow * 128 + ((c0 ^ xkey) << 4), x_off1 = xrow * 128 + ((c1 ^ xkey) << 4);
    const int wrow = wave_n * WN + (l16 >> 2) * 8 + (l16 & 3);    // + coff_of(ti)
    const int wkey = w_key(wrow);
    const int w_off0 = wrow * 128 + ((c0 ^ wkey) << 4), w_off1 = wrow * 128 + ((c1 ^ wkey) << 4);

    v4f acc[NSPLIT][MI][NI];
#pragma unroll
    for (int h = 0; h < NSPLIT; ++h)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ti = 0; ti < NI; ++ti) acc[h][mi][ti] = v4f{0.f, 0.f, 0.f, 0.f};

    const int ksteps_all = (p.KB + 127) / 128;
    const int ksteps = EPI == EPI_SPLITK ? (ksteps_all - k_lo < p.k_per_split ? ksteps_all - k_lo : p.k_per_split) : ksteps_all;
    const int iters = ksteps * NSPLIT;

    // blockwise scales: sx[m, kb] per row of this lane, sw[kb, nb] per N-part
    const float* sxg = p.sx + static_cast<int64_t>(g) * p.strideSx;
    const float* swg = p.sw + static_cast<int64_t>(g) * p.strideSw;

    if constexpr (!RING) {
#pragma unroll
        for (int j = 0; j < JN; ++j) issue_j(j, 0, 0, 0, 0, true);   // stage 0, every wave's share
    }

    // loads of the next stage are issued in the first ISSUE_STEPS tile steps of the running stage
    constexpr int ISSUE_STEPS = NI >= 4 ? NI / 2 : NI;
    constexpr int J_PER_STEP = (JN + ISSUE_STEPS - 1) / ISSUE_STEPS;

    // Ping-pong schedule for the 8-wave 256-row tiles: waves 0..3 (group A, upper 128 rows) and 4..7
    // (group B, lower 128 rows) sit one of each on every SIMD.  Each K step has two phases separated by
    // workgroup barriers: while A reads its 12 operand fragments of stage k from LDS, B runs the 32 MFMAs
    // of stage k-1 from registers; then A computes stage k while B reads stage k.  The MFMA pipe of every
    // SIMD always has a computing wave, and the LDS reads of one group hide behind the other's MFMAs.
    constexpr bool PINGPONG = (NW == 8 && WAVES_M == 2 && NSPLIT == 1 && !IS_BF16 && !BLOCKWISE && !EXACT && EPI != EPI_SPLITK);
    if constexpr (RING) {
        // Split K: a workgroup's share is a chain of short K steps (8 MFMAs per wave) whose operands come from HBM.
        // With one stage in flight every step waits a whole memory round trip (measured: 1.7 - 2.5 us per step, whatever
        // the number of ranges).  Here a ring of NST stages keeps NST - 1 of them in flight: the loads of stage k + NST - 1
        // go out between the MFMAs of stage k, into the slot stage k - 1 left, and the wait at the top of a step leaves
        // the newer stages' loads outstanding (loads complete in order, every wave issues the same number per stage).
        // (Measured at 65536 x 256 x 1024 as a weight gradient: 0.9 us per step, of which 0.55 us remain with neither
        // loads nor LDS reads in the loop - the MFMAs into fresh accumulators and the 32 multiply-adds that promote
        // them, wave by wave; reading the next step's fragments into a second register set between the MFMAs changes
        // nothing.  The four-wave instantiation keeps the two-stage loop below, two workgroups per CU covering each
        // other's round trips: per CU and step it is the faster one once a range has more than about a hundred steps.)
        // Block scales travel with their stage: a per-step load from global memory in the loop would be younger than
        // the stages in flight, and waiting for it would wait for them.  Waves 0 and 1 fetch the step's scale of 64 rows
        // of X each (one 4-byte load per lane, straight into LDS), wave 2 the scale of the W block, the other waves a load
        // that is out of range (zeros, into a spare quarter of the slot): the same count on every wave.
        static_assert(NSPLIT == 1 && !IS_BF16 && !EXACT && NST == 4, "split K: plain FP8 tiles on a ring of four stages");
        static_assert(!BLOCKWISE || (NW >= 4 && BM == 128 && BN == 128), "scale loads are laid out for a 128 x 128 tile and at least four waves");
        constexpr int D = NST - 1;
        constexpr int JT = JN + (BLOCKWISE ? 1 : 0);                    // loads per wave and stage
        uint8_t* const sbuf = smem + NST * (XS + WS);                   // [NST][256 floats]: sx of the tile's rows, then sw
        // (descriptor and step from wave-uniform values, handed over through scalar registers: derived from branches on
        // the wave id the compiler would wrap every scale load in a loop over the lanes' descriptors)
        int s_rows = p.M - m0 - 64 * wave;
        s_rows = s_rows < 0 ? 0 : (s_rows > 64 ? 64 : s_rows);
        const float* s_base = wave < 2 ? sxg + static_cast<int64_t>(m0 + 64 * wave) * ksteps_all : swg + (n0 >> 7);
        int s_rec = wave < 2 ? s_rows * ksteps_all * 4 : (wave == 2 ? (ksteps_all * (p.N >> 7) - (n0 >> 7)) * 4 : 0);
        int s_step = wave < 2 ? 4 : (p.N >> 7) * 4;                     // bytes from one K step's scale to the next
        const uint64_t s_addr = reinterpret_cast<uint64_t>(s_base);
        const uint64_t s_addr_u = static_cast<uint64_t>(static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(s_addr)))) |
                                  (static_cast<uint64_t>(static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(s_addr >> 32)))) << 32);
        s_rec = __builtin_amdgcn_readfirstlane(BLOCKWISE ? s_rec : 0);
        s_step = __builtin_amdgcn_readfirstlane(s_step);
        const __amdgpu_buffer_rsrc_t s_rsrc =
            __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<float*>(s_addr_u), 0, s_rec, 0x00020000);
        // waves 0, 1: the lane's row (checked against the descriptor's bound); wave 2: lane 0 takes the block's scale
        const int s_voff = wave < 2 ? lane * ksteps_all * 4 : (lane == 0 ? 0 : 0x7FFFFFF0);
        auto issue_stage = [&](int j0, int j1, int slot, int k) __attribute__((always_inline)) {
            if (BLOCKWISE && j0 == 0)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(s_rsrc, (__attribute__((address_space(3))) void*)(sbuf + slot * 1024 + (wave < 3 ? wave : 3) * 256),
                                                         4, s_voff, (k_lo + k) * s_step, 0, 0);
#pragma unroll
            for (int j = j0; j < j1 && j < JN; ++j) issue_j(j, slot, slot, k * 128, 0, true);
        };
#pragma unroll
        for (int s = 0; s < D; ++s)
            if (s < ksteps) issue_stage(0, JN, s, s);
        for (int k = 0; k < ksteps; ++k) {
            const int newer = ksteps - 1 - k < D - 1 ? ksteps - 1 - k : D - 1;   // stages requested after stage k
            if (newer >= 2) wait_vmcnt<2 * JT>();
            else if (newer == 1) wait_vmcnt<JT>();
            else wait_vmcnt<0>();
            lds_barrier();                                      // everyone's share of stage k is here; everyone left step k - 1
            const bool more = k + D < ksteps;
            const int slot = k % NST, nslot = (k + D) % NST;
            const uint8_t* xs = xbuf + slot * XS;
            const uint8_t* ws = wbuf + slot * WS;
            v8i bx[MI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const v4i lo = *reinterpret_cast<const v4i*>(xs + x_off0 + mi * 16 * 128);
                const v4i hi = *reinterpret_cast<const v4i*>(xs + x_off1 + mi * 16 * 128);
                bx[mi] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            }
            float sxk[MI], swk = 0.f;
            if (BLOCKWISE) {
                const float* sl = reinterpret_cast<const float*>(sbuf + slot * 1024);
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) sxk[mi] = sl[wave_m * WM + mi * 16 + l16];
                swk = sl[128];
            }
            v4i lo = *reinterpret_cast<const v4i*>(ws + w_off0);
            v4i hi = *reinterpret_cast<const v4i*>(ws + w_off1);      // coff_of(0) == 0
#pragma unroll
            for (int ti = 0; ti < NI; ++ti) {
                if (more && ti < ISSUE_STEPS) issue_stage(ti * J_PER_STEP, (ti + 1) * J_PER_STEP, nslot, k + D);
                v4i lo_n = lo, hi_n = hi;
                if (ti + 1 < NI) {
                    lo_n = *reinterpret_cast<const v4i*>(ws + w_off0 + coff_of(ti + 1) * 128);
                    hi_n = *reinterpret_cast<const v4i*>(ws + w_off1 + coff_of(ti + 1) * 128);
                }
                const v8i aw = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) {
                    if (BLOCKWISE) {
                        // promote this 128-wide K block into the fp32 accumulator with its scales
                        const v4f c = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aw, bx[mi], v4f{0.f, 0.f, 0.f, 0.f},
                                                                                        0, 0, 0, 0, 0, 0);
                        const float s = sxk[mi] * swk;
                        acc[0][mi][ti] += c * s;
                    } else {
                        acc[0][mi][ti] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aw, bx[mi], acc[0][mi][ti],
                                                                                         0, 0, 0, 0, 0, 0);
                    }
                }
                lo = lo_n;
                hi = hi_n;
            }
        }
    } else if constexpr (PINGPONG) {
        const bool grp_b = wave >= 4;                           // wave-uniform
        v8i bx[MI], aw[NI];
        auto read_frags = [&](int k) __attribute__((always_inline)) {
            const uint8_t* xs = xbuf + (k & 1) * XS;
            const uint8_t* ws = wbuf + (k & 1) * WS;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const v4i lo = *reinterpret_cast<const v4i*>(xs + x_off0 + mi * 16 * 128);
                const v4i hi = *reinterpret_cast<const v4i*>(xs + x_off1 + mi * 16 * 128);
                bx[mi] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            }
#pragma unroll
            for (int ti = 0; ti < NI; ++ti) {
                const v4i lo = *reinterpret_cast<const v4i*>(ws + w_off0 + coff_of(ti) * 128);
                const v4i hi = *reinterpret_cast<const v4i*>(ws + w_off1 + coff_of(ti) * 128);
                aw[ti] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            }
        };
        auto compute = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int ti = 0; ti < NI; ++ti)
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
                    acc[0][mi][ti] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aw[ti], bx[mi], acc[0][mi][ti],
                                                                                     0, 0, 0, 0, 0, 0);
        };
        // Group B runs the same loop one phase behind A (one extra barrier up front, one fewer at the end),
        // so the loop body has no group-dependent control flow around the accumulators.  A issues its share
        // of stage k+1 after the top barrier of step k and waits for it before the next top barrier; B issues
        // its share of stage k+2 after its mid barrier and waits before its next mid barrier: each share has a
        // full K step to land, and every stage is complete one barrier before its first reader.
        if (grp_b) {
            if (ksteps > 1) {
#pragma unroll
                for (int j = 0; j < JN; ++j) issue_j(j, 1, 1, 128, 0, true);
            }
            __builtin_amdgcn_s_waitcnt(0x0F70);
            lds_barrier();
        }
        for (int k = 0; k < ksteps; ++k) {
            if (!grp_b) __builtin_amdgcn_s_waitcnt(0x0F70);
            lds_barrier();
            if (!grp_b && k + 1 < ksteps) {
#pragma unroll
                for (int j = 0; j < JN; ++j) issue_j(j, (k + 1) & 1, (k + 1) & 1, (k + 1) * 128, 0, true);
            }
            read_frags(k);
            if (grp_b) __builtin_amdgcn_s_waitcnt(0x0F70);
            lds_barrier();
            if (grp_b && k + 2 < ksteps) {
#pragma unroll
                for (int j = 0; j < JN; ++j) issue_j(j, k & 1, k & 1, (k + 2) * 128, 0, true);
            }
            compute();
        }
        if (!grp_b) lds_barrier();
    } else {
    for (int it = 0; it < iters; ++it) {
        const int k = it / NSPLIT, h = it % NSPLIT;
        __builtin_amdgcn_s_waitcnt(0x0F70);                     // vmcnt(0): this wave's loads for stage `it` have landed
        __syncthreads();                                        // everyone's have; everyone left iteration it-1
        const bool more = it + 1 < iters;
        const int k1 = (it + 1) / NSPLIT, h1 = (it + 1) % NSPLIT;
        const uint8_t* xs = xbuf + (k & 1) * XS;
        const uint8_t* ws = wbuf + (it & 1) * WS;

        v8i bx[MI];
        v8bf xe[EXACT ? MI : 1][4];          // EXACT: the lane's 32 K positions as four bf16 operands of 8
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const v4i lo = *reinterpret_cast<const v4i*>(xs + x_off0 + mi * 16 * 128);
            const v4i hi = *reinterpret_cast<const v4i*>(xs + x_off1 + mi * 16 * 128);
            bx[mi] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            if (EXACT) {
                xe[mi][0] = e4m3x8_to_bf16(lo[0], lo[1]); xe[mi][1] = e4m3x8_to_bf16(lo[2], lo[3]);
                xe[mi][2] = e4m3x8_to_bf16(hi[0], hi[1]); xe[mi][3] = e4m3x8_to_bf16(hi[2], hi[3]);
            }
        }
        float sxk[MI];
        if (BLOCKWISE) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                int m = m0 + wave_m * WM + mi * 16 + l16;
                m = m < p.M ? m : p.M - 1;
                sxk[mi] = sxg[static_cast<int64_t>(m) * ksteps_all + k_lo + k];
            }
        }
#pragma unroll
        for (int hh = 0; hh < NSPLIT; ++hh) {
            if (hh != h) continue;
            float swk = 0.f;
            if (BLOCKWISE) {
                int nrun = n0 + hh * BN_SUB + wave_n * WN + q * 8;
                nrun = nrun < p.N ? nrun : p.N - 1;
                swk = swg[static_cast<int64_t>(k_lo + k) * (p.N >> 7) + (nrun >> 7)];
            }
            // W fragments are fetched one tile ahead of the MFMAs that consume them
            v4i lo = *reinterpret_cast<const v4i*>(ws + w_off0);
            v4i hi = *reinterpret_cast<const v4i*>(ws + w_off1);      // coff_of(0) == 0
#pragma unroll
            for (int ti = 0; ti < NI; ++ti) {
                if (more && ti < ISSUE_STEPS) {
#pragma unroll
                    for (int j = ti * J_PER_STEP; j < (ti + 1) * J_PER_STEP && j < JN; ++j)
                        issue_j(j, k1 & 1, (it + 1) & 1, k1 * 128, h1, h1 == 0);
                }
                v4i lo_n = lo, hi_n = hi;
                if (ti + 1 < NI) {
                    lo_n = *reinterpret_cast<const v4i*>(ws + w_off0 + coff_of(ti + 1) * 128);
                    hi_n = *reinterpret_cast<const v4i*>(ws + w_off1 + coff_of(ti + 1) * 128);
                }
                v8bf we[4];                  // EXACT: this W fragment as four bf16 operands (same K positions as xe)
                if (EXACT) {
                    we[0] = e4m3x8_to_bf16(lo[0], lo[1]); we[1] = e4m3x8_to_bf16(lo[2], lo[3]);
                    we[2] = e4m3x8_to_bf16(hi[0], hi[1]); we[3] = e4m3x8_to_bf16(hi[2], hi[3]);
                }
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) {
                    if (EXACT) {
                        v4f c = acc[hh][mi][ti];
#pragma unroll
                        for (int j = 0; j < 4; ++j) c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(we[j], xe[mi][j], c, 0, 0, 0);
                        acc[hh][mi][ti] = c;
                    } else if (IS_BF16) {
                        v4f c = acc[hh][mi][ti];
                        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, lo),
                                                                    __builtin_bit_cast(v8bf, v4i{bx[mi][0], bx[mi][1], bx[mi][2], bx[mi][3]}),
                                                                    c, 0, 0, 0);
                        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, hi),
                                                                    __builtin_bit_cast(v8bf, v4i{bx[mi][4], bx[mi][5], bx[mi][6], bx[mi][7]}),
                                                                    c, 0, 0, 0);
                        acc[hh][mi][ti] = c;
                    } else {
                        const v8i aw = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                        if (BLOCKWISE) {
                            // promote this 128-wide K block into the fp32 accumulator with its scales
                            v4f c = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aw, bx[mi], v4f{0.f, 0.f, 0.f, 0.f},
                                                                                     0, 0, 0, 0, 0, 0);
                            const float s = sxk[mi] * swk;
                            acc[hh][mi][ti] += c * s;
                        } else {
                            acc[hh][mi][ti] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aw, bx[mi], acc[hh][mi][ti],
                                                                                               0, 0, 0, 0, 0, 0);
                        }
                    }
                }
                lo = lo_n;
                hi = hi_n;
            }
        }
    }
    }

    // ------------------------------------------------------------------ epilogue
    // lane owns row m (per mi) and, per N-part h and tile ti, columns ncol(h) + coff_of(ti) + [0, 4)
    __syncthreads();                       // all waves are done reading the stages: LDS is free
    float* red = reinterpret_cast<float*>(smem);   // [BM][WAVES_N][3]
    const int64_t obase = static_cast<int64_t>(g) * p.strideO;
    const bool tensor_x = p.x_mode == LOKA_SCALE_TENSOR, tensor_w = p.w_mode == LOKA_SCALE_TENSOR;

    int ncol[NSPLIT];
    float cnt_lane = 0.f;                  // valid columns this lane holds per row
#pragma unroll
    for (int h = 0; h < NSPLIT; ++h) {
        ncol[h] = n0 + h * BN_SUB + wave_n * WN + q * 8;
#pragma unroll
        for (int ti = 0; ti < NI; ++ti)
            if (ncol[h] + coff_of(ti) < p.N) cnt_lane += 4.f;
    }

    // apply scales in place
    if (!BLOCKWISE && !IS_BF16) {
#pragma unroll
        for (int h = 0; h < NSPLIT; ++h)
#pragma unroll
            for (int ti = 0; ti < NI; ++ti) {
                const int n = ncol[h] + coff_of(ti);
                v4f s4;
                if (tensor_w) {
                    const float s = swg[0];
                    s4 = v4f{s, s, s, s};
                } else {
                    s4 = (n < p.N) ? *reinterpret_cast<const v4f*>(swg + n) : v4f{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) {
                    int m = m0 + wave_m * WM + mi * 16 + l16;
                    m = m < p.M ? m : p.M - 1;
                    const float sxm = tensor_x ? sxg[0] : sxg[m];
                    acc[h][mi][ti] *= s4 * sxm;
                }
            }
    }

    if (p.y) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int m = m0 + wave_m * WM + mi * 16 + l16;
            if (m < p.M) {
#pragma unroll
                for (int h = 0; h < NSPLIT; ++h)
#pragma unroll
                    for (int ti = 0; ti < NI; ++ti) {
                        const int n = ncol[h] + coff_of(ti);
                        if (n < p.N)
                            *reinterpret_cast<v4f*>(p.y + obase + static_cast<int64_t>(m) * p.N + n) = acc[h][mi][ti];
                    }
            }
        }
    }
    if (IS_BF16) continue;                 // reference GEMM: fp32 Y only
    if (EPI == EPI_SPLITK) {
        // this K range's share of Y (scales applied: they are factors of every term) goes to the partial buffer; a second
        // kernel adds the ranges in a fixed order and normalizes the row
        float* const part = p.part + (static_cast<int64_t>(ks) * p.batch + g) * p.M * p.N;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int m = m0 + wave_m * WM + mi * 16 + l16;
            if (m < p.M) {
#pragma unroll
                for (int h = 0; h < NSPLIT; ++h)
#pragma unroll
                    for (int ti = 0; ti < NI; ++ti) {
                        const int n = ncol[h] + coff_of(ti);
                        if (n < p.N) *reinterpret_cast<v4f*>(part + static_cast<int64_t>(m) * p.N + n) = acc[h][mi][ti];
                    }
            }
        }
        continue;
    }

    // ---- row statistics (reciprocals and the inverse square root are the 1-ulp hardware ones: their
    // error is four orders of magnitude below a bf16 ulp, and the IEEE sequences are ~300 cycles each)
    const float inv_n = 1.0f / static_cast<float>(p.N);
    float mean_r[MI], rstd_r[MI];
    if (p.norm == LOKA_NORM_NONE) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) { mean_r[mi] = 0.f; rstd_r[mi] = 1.f; }
    } else {
        const bool ln = p.norm == LOKA_NORM_LAYERNORM;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            float n_ = cnt_lane, mean = 0.f, m2 = 0.f;
            if (ln) {
                float s = 0.f;
#pragma unroll
                for (int h = 0; h < NSPLIT; ++h)
#pragma unroll
                    for (int ti = 0; ti < NI; ++ti)
                        if (ncol[h] + coff_of(ti) < p.N)
                            s += (acc[h][mi][ti][0] + acc[h][mi][ti][1]) + (acc[h][mi][ti][2] + acc[h][mi][ti][3]);
                mean = n_ > 0.f ? s * __builtin_amdgcn_rcpf(n_) : 0.f;
#pragma unroll
                for (int h = 0; h < NSPLIT; ++h)
#pragma unroll
                    for (int ti = 0; ti < NI; ++ti)
                        if (ncol[h] + coff_of(ti) < p.N) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float d = acc[h][mi][ti][e] - mean;
                                m2 += d * d;
                            }
                        }
                // lanes l, l^16, l^32, l^48 hold the same row
#pragma unroll
                for (int msk = 16; msk < 64; msk <<= 1) {
                    const float nb = wave_shfl_xor(n_, msk), mb = wave_shfl_xor(mean, msk), m2b = wave_shfl_xor(m2, msk);
                    // symmetric form so both partners compute identical bits
                    const float nn = n_ + nb;
                    if (nn > 0.f) {
                        const float d = mb - mean;
                        const float rn = __builtin_amdgcn_rcpf(nn);
                        const float newmean = (n_ * mean + nb * mb) * rn;
                        m2 = m2 + m2b + d * d * (n_ * nb * rn);
                        mean = newmean;
                    }
                    n_ = nn;
                }
            } else {
#pragma unroll
                for (int h = 0; h < NSPLIT; ++h)
#pragma unroll
                    for (int ti = 0; ti < NI; ++ti)
                        if (ncol[h] + coff_of(ti) < p.N) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) m2 += acc[h][mi][ti][e] * acc[h][mi][ti][e];
                        }
                m2 += wave_shfl_xor(m2, 16);
                m2 += wave_shfl_xor(m2, 32);
            }
            if (WAVES_N > 1) {
                const int row = wave_m * WM + mi * 16 + l16;
                if (q == 0) {
                    float* r3 = red + (row * WAVES_N + wave_n) * 3;
                    r3[0] = n_; r3[1] = mean; r3[2] = m2;
                }
            }
            mean_r[mi] = mean; rstd_r[mi] = m2;        // rstd_r holds M2 / sumsq until finalized
            if (WAVES_N == 1 && EPI == EPI_ROW_IN_TILE) {
                rstd_r[mi] = __builtin_amdgcn_rsqf(m2 * inv_n + p.eps);
            }
        }
        if (WAVES_N > 1) {
            __syncthreads();
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const int row = wave_m * WM + mi * 16 + l16;
                float n_ = 0.f, mean = 0.f, m2 = 0.f;
#pragma unroll
                for (int w = 0; w < WAVES_N; ++w) {             // fixed order: every wave gets identical bits
                    const float* r3 = red + (row * WAVES_N + w) * 3;
                    if (ln) merge_stats(n_, mean, m2, r3[0], r3[1], r3[2]);
                    else m2 += r3[2];
                }
                mean_r[mi] = mean; rstd_r[mi] = m2;
                if (EPI == EPI_ROW_IN_TILE) {
                    rstd_r[mi] = __builtin_amdgcn_rsqf(m2 * inv_n + p.eps);
                }
            }
        }
    }

    if (EPI == EPI_PARTIAL_STATS) {
        // the row spans several workgroups: publish this tile's (mean, M2) [or (sumsq, 0)] and leave the
        // normalization to the second pass; Y has been stored above
        if (p.norm != LOKA_NORM_NONE && wave_n == 0 && q == 0) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const int m = m0 + wave_m * WM + mi * 16 + l16;
                if (m < p.M) {
                    float* dst = p.part + (static_cast<int64_t>(g) * p.M + m) * (2 * p.tiles_n) + 2 * tn;
                    dst[0] = mean_r[mi];
                    dst[1] = rstd_r[mi];
                }
            }
        }
        if (p.norm != LOKA_NORM_NONE) continue;
    }

    if (EPI == EPI_PANEL_SYNC && p.norm != LOKA_NORM_NONE) {
        // The row spans tiles_n workgroups that run in the same round.  Each publishes its tile's
        // (mean, M2) [or (0, sumsq)] per row, signals its arrival, waits until all tiles_n have arrived, and
        // merges every tile's statistics in one fixed order, so all of them normalize with identical row
        // statistics.  Only these few words per row leave the CU.
        const int panel = g * p.tiles_m + tm;
        float* prow = p.part + (static_cast<int64_t>(g) * p.M) * (2 * p.tiles_n);
        if (wave_n == 0 && q == 0) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const int m = m0 + wave_m * WM + mi * 16 + l16;
                if (m < p.M) {
                    float* dst = prow + static_cast<int64_t>(m) * (2 * p.tiles_n) + 2 * tn;
                    // device-coherent (write-through) stores: no L2-wide write-back is needed to publish them
                    __hip_atomic_store(dst, mean_r[mi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(dst + 1, rstd_r[mi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
        int* lds_word = reinterpret_cast<int*>(smem) + BM * WAVES_N * 3 + 4;                  // between `red` and `fin`
        const bool arrived = panel_publish_and_wait(p, p.flags + static_cast<int64_t>(panel) * p.tiles_n, tn, p.tiles_n, lds_word);
        const bool ln = p.norm == LOKA_NORM_LAYERNORM;
        // Merge: the workgroup's BM rows are spread over its threads (TPR threads per row, each folding a
        // contiguous share of the row's tiles_n entries in order, read with device-coherent 8-byte loads
        // that bypass stale cache lines); shares are combined with the symmetric merge, the row's final
        // (mean, rstd) goes through LDS to the lanes that own the row.  Every workgroup of the panel runs
        // the same procedure on the same words, so all of them normalize with identical statistics.
        {
            constexpr int T = NW * 64, TPR = T / BM >= 1 ? T / BM : 1;
            static_assert(T % BM == 0 || T < BM, "threads per row");
            float2* fin = reinterpret_cast<float2*>(smem) + BM * WAVES_N * 3 / 2 + 8;   // after `red`
            for (int r0 = 0; r0 < BM; r0 += T / TPR) {
                const int r = r0 + static_cast<int>(threadIdx.x) / TPR, sub = static_cast<int>(threadIdx.x) % TPR;
                int m = m0 + r;
                m = m < p.M ? m : p.M - 1;
                const float* src = prow + static_cast<int64_t>(m) * (2 * p.tiles_n);
                const int TH = (p.tiles_n + TPR - 1) / TPR;
                float n_ = 0.f, mean = 0.f, m2 = 0.f;
                for (int t0 = sub * TH; t0 < (sub + 1) * TH && t0 < p.tiles_n; t0 += 8) {
                    unsigned long long raw[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        int tt = t0 + u;
                        tt = tt < p.tiles_n ? tt : p.tiles_n - 1;
                        raw[u] = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(src + 2 * tt),
                                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
                        }
                    }
                }
#pragma unroll
                for (int msk = 1; msk < TPR; msk <<= 1) {
                    const float nb = wave_shfl_xor(n_, msk), mb = wave_shfl_xor(mean, msk), m2b = wave_shfl_xor(m2, msk);
                    if (ln) {
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
                        m2 = m2 + m2b;
                    }
                }
                // (a wait that ran out: the row statistics are not to be trusted, the tile's rows leave as NaN)
                if (sub == 0 && r < BM)
                    fin[r] = arrived ? make_float2(ln ? mean : 0.f, __builtin_amdgcn_rsqf(m2 * inv_n + p.eps))
                                     : make_float2(__builtin_nanf(""), __builtin_nanf(""));
            }
            __syncthreads();
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const float2 f = fin[wave_m * WM + mi * 16 + l16];
                mean_r[mi] = f.x;
                rstd_r[mi] = f.y;
            }
        }
    }

    // ---- normalize, affine, bf16 store
    const bool has_g = p.gamma != nullptr, has_b = p.beta != nullptr && p.norm == LOKA_NORM_LAYERNORM;
#pragma unroll
    for (int h = 0; h < NSPLIT; ++h) {
#pragma unroll
        for (int tp = 0; tp < NI; tp += 2) {                    // two tiles = 8 columns = one 16-byte store
            const int n = ncol[h] + coff_of(tp);
            if (n >= p.N) continue;
            float gm[8], bt[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) { gm[e] = 1.f; bt[e] = 0.f; }
            if (has_g && p.norm != LOKA_NORM_NONE) {
                const u32x4 w = *reinterpret_cast<const u32x4*>(p.gamma + n);
                gm[0] = bf16_lo(w.x); gm[1] = bf16_hi(w.x); gm[2] = bf16_lo(w.y); gm[3] = bf16_hi(w.y);
                gm[4] = bf16_lo(w.z); gm[5] = bf16_hi(w.z); gm[6] = bf16_lo(w.w); gm[7] = bf16_hi(w.w);
            }
            if (has_b) {
                const u32x4 w = *reinterpret_cast<const u32x4*>(p.beta + n);
                bt[0] = bf16_lo(w.x); bt[1] = bf16_hi(w.x); bt[2] = bf16_lo(w.y); bt[3] = bf16_hi(w.y);
                bt[4] = bf16_lo(w.z); bt[5] = bf16_hi(w.z); bt[6] = bf16_lo(w.w); bt[7] = bf16_hi(w.w);
            }
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const int m = m0 + wave_m * WM + mi * 16 + l16;
                if (m >= p.M) continue;
                float o[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float yv = acc[h][mi][tp + (e >> 2)][e & 3];
                    o[e] = (yv - mean_r[mi]) * rstd_r[mi];
                    if (has_g && p.norm != LOKA_NORM_NONE) o[e] *= gm[e];
                    if (has_b) o[e] += bt[e];
                }
                u32x4 pk;
                pk.x = pack_bf16x2(o[0], o[1]); pk.y = pack_bf16x2(o[2], o[3]);
                pk.z = pack_bf16x2(o[4], o[5]); pk.w = pack_bf16x2(o[6], o[7]);
                u32x4* dst = reinterpret_cast<u32x4*>(p.out + obase + static_cast<int64_t>(m) * p.N + n);
                if (EPI == EPI_PANEL_SYNC) __builtin_nontemporal_store(pk, dst);   // streamed: keeps X / W in the L2
                else *dst = pk;
            }
        }
    }
  }  // tile loop
}

// Second pass of the two-pass schedule: combine the per-tile statistics of each row in a
// fixed order and normalize fp32 Y into bf16 O.  One wave per row.
__global__ __launch_bounds__(256) void norm_rows_kernel(const float* __restrict__ y, const float* __restrict__ part,
                                                        int64_t rows, int N, int tiles_n, int tile_w, int norm,
                                                        float eps, const uint16_t* __restrict__ gamma,
                                                        const uint16_t* __restrict__ beta, uint16_t* __restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int64_t r = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (r >= rows) return;
    float n_ = 0.f, mean = 0.f, m2 = 0.f;
    for (int t = 0; t < tiles_n; ++t) {
        const float a = part[r * 2 * tiles_n + 2 * t], b = part[r * 2 * tiles_n + 2 * t + 1];
        const int w = (t + 1) * tile_w <= N ? tile_w : N - t * tile_w;
        if (norm == LOKA_NORM_LAYERNORM) merge_stats(n_, mean, m2, static_cast<float>(w), a, b);
        else m2 += b;
    }
    if (norm != LOKA_NORM_LAYERNORM) mean = 0.f;
    const float rstd = 1.0f / sqrtf(m2 / static_cast<float>(N) + eps);
    const bool has_b = beta != nullptr && norm == LOKA_NORM_LAYERNORM;
    for (int c = lane * 8; c < N; c += 512) {
        const v4f a = *reinterpret_cast<const v4f*>(y + r * N + c);
        const v4f b = *reinterpret_cast<const v4f*>(y + r * N + c + 4);
        float o[8] = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
        float gm[8], bt[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { gm[e] = 1.f; bt[e] = 0.f; }
        if (gamma) {
            const u32x4 w = *reinterpret_cast<const u32x4*>(gamma + c);
            gm[0] = bf16_lo(w.x); gm[1] = bf16_hi(w.x); gm[2] = bf16_lo(w.y); gm[3] = bf16_hi(w.y);
            gm[4] = bf16_lo(w.z); gm[5] = bf16_hi(w.z); gm[6] = bf16_lo(w.w); gm[7] = bf16_hi(w.w);
        }
        if (has_b) {
            const u32x4 w = *reinterpret_cast<const u32x4*>(beta + c);
            bt[0] = bf16_lo(w.x); bt[1] = bf16_hi(w.x); bt[2] = bf16_lo(w.y); bt[3] = bf16_hi(w.y);
            bt[4] = bf16_lo(w.z); bt[5] = bf16_hi(w.z); bt[6] = bf16_lo(w.w); bt[7] = bf16_hi(w.w);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            o[e] = (o[e] - mean) * rstd;
            if (gamma) o[e] *= gm[e];
            if (has_b) o[e] += bt[e];
        }
        u32x4 pk;
        pk.x = pack_bf16x2(o[0], o[1]); pk.y = pack_bf16x2(o[2], o[3]);
        pk.z = pack_bf16x2(o[4], o[5]); pk.w = pack_bf16x2(o[6], o[7]);
        *reinterpret_cast<u32x4*>(out + r * N + c) = pk;
    }
}

// Second kernel of the split-K schedule: WPR waves per output row (1, or 4 = a whole workgroup when the output has
// few rows, as a weight gradient does) add the row's ksplit partial sums in a fixed order (repeatable bits; eight
// partials are requested before the first is added, so the loads overlap while the additions keep their order), take
// the row statistics of the sum in registers (two sweeps over the thread's values: no E[y^2] - mean^2 cancellation),
// normalize and write bf16 O (and fp32 Y when asked).  N <= 8192: a thread holds N / (64 WPR) values.
// part: [ksplit][rows][N] fp32 with rows = batch * M; row r of problem g lies at g * strideO + m * N in O / Y.
constexpr int kSplitkMaxN = 8192;
template <int WPR>
__global__ __launch_bounds__(256) void splitk_norm_rows_kernel(const float* __restrict__ part, int ksplit, int64_t rows,
                                                               int M, int N, int64_t strideO, int norm, float eps,
                                                               const uint16_t* __restrict__ gamma,
                                                               const uint16_t* __restrict__ beta, uint16_t* __restrict__ out,
                                                               float* __restrict__ y) {
    constexpr int TPR = 64 * WPR;                    // threads per row
    __shared__ float red[4];
    const int tr = threadIdx.x & (TPR - 1);
    const int64_t r = static_cast<int64_t>(blockIdx.x) * (256 / TPR) + threadIdx.x / TPR;
    if (WPR == 1 && r >= rows) return;               // (WPR == 4: one row per workgroup, the grid is exactly the rows)
    constexpr int MAXC = kSplitkMaxN / (4 * TPR);    // float4 chunks per thread
    v4f v[MAXC];
    const int chunks = N >> 2;
    const int64_t slab = rows * static_cast<int64_t>(N);
    const float* src = part + r * N;
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
        const int c = tr + TPR * j;
        v[j] = v4f{0.f, 0.f, 0.f, 0.f};
        if (c < chunks) {
            const float* sc = src + 4 * c;
            int k = 0;
            for (; k + 8 <= ksplit; k += 8) {
                v4f t[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) t[u] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(sc + (k + u) * slab));
#pragma unroll
                for (int u = 0; u < 8; ++u) v[j] += t[u];
            }
            for (; k < ksplit; ++k) v[j] += __builtin_nontemporal_load(reinterpret_cast<const v4f*>(sc + k * slab));
            s += (v[j][0] + v[j][1]) + (v[j][2] + v[j][3]);
        }
    }
    const int64_t g = r / M, m = r - g * M;
    const int64_t obase = g * strideO + m * N;
    if (y) {
#pragma unroll
        for (int j = 0; j < MAXC; ++j) {
            const int c = tr + TPR * j;
            if (c < chunks) *reinterpret_cast<v4f*>(y + obase + 4 * c) = v[j];
        }
    }
    // sum over the row's threads: the wave by shuffles, the (up to four) waves through LDS in wave order
    auto row_sum = [&](float x) __attribute__((always_inline)) {
        for (int msk = 1; msk < 64; msk <<= 1) x += wave_shfl_xor(x, msk);
        if (WPR > 1) {
            __syncthreads();                         // (the previous use of red has been read)
            if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
            __syncthreads();
            x = (red[0] + red[1]) + (red[2] + red[3]);
        }
        return x;
    };
    float mean = 0.f, rstd = 1.f;
    if (norm == LOKA_NORM_LAYERNORM || norm == LOKA_NORM_RMSNORM) {
        if (norm == LOKA_NORM_LAYERNORM) mean = row_sum(s) / static_cast<float>(N);
        float m2 = 0.f;
#pragma unroll
        for (int j = 0; j < MAXC; ++j) {
            const int c = tr + TPR * j;
            if (c < chunks) {
#pragma unroll
                for (int e = 0; e < 4; ++e) { const float d = v[j][e] - mean; m2 += d * d; }
            }
        }
        rstd = 1.0f / sqrtf(row_sum(m2) / static_cast<float>(N) + eps);
    }
    const bool has_g = gamma != nullptr && norm != LOKA_NORM_NONE, has_b = beta != nullptr && norm == LOKA_NORM_LAYERNORM;
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
        const int c = tr + TPR * j;
        if (c >= chunks) continue;
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (v[j][e] - mean) * rstd;
        if (has_g) {
            const u32x2 w = *reinterpret_cast<const u32x2*>(gamma + 4 * c);
            o[0] *= bf16_lo(w.x); o[1] *= bf16_hi(w.x); o[2] *= bf16_lo(w.y); o[3] *= bf16_hi(w.y);
        }
        if (has_b) {
            const u32x2 w = *reinterpret_cast<const u32x2*>(beta + 4 * c);
            o[0] += bf16_lo(w.x); o[1] += bf16_hi(w.x); o[2] += bf16_lo(w.y); o[3] += bf16_hi(w.y);
        }
        u32x2 pk;
        pk.x = pack_bf16x2(o[0], o[1]); pk.y = pack_bf16x2(o[2], o[3]);
        *reinterpret_cast<u32x2*>(out + obase + 4 * c) = pk;
    }
}

// [K, N] bf16 -> [N, K] bf16 (the reference GEMM reads K-contiguous operands like the FP8 one)
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const uint16_t* __restrict__ w, int K, int N,
                                                             uint16_t* __restrict__ wt) {
    __shared__ uint16_t tile[64][66];
    const int k0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int kk = i >> 6, nn = i & 63;
        if (k0 + kk < K && n0 + nn < N) tile[kk][nn] = w[static_cast<int64_t>(k0 + kk) * N + n0 + nn];
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int nn = i >> 6, kk = i & 63;
        if (k0 + kk < K && n0 + nn < N) wt[static_cast<int64_t>(n0 + nn) * K + k0 + kk] = tile[kk][nn];
    }
}

// ------------------------------------------------------------------------------ host side
struct VariantInfo {
    const char* name;
    int bm, bn;            // workgroup tile (bn = full width the tile covers)
    int threads;
    int epi;               // EPI_*
    size_t lds;
    void (*launch)(const GemmParams&, bool blockwise, dim3 grid, hipStream_t s);
    const void* fn_plain;
    const void* fn_block;
};

template <int BM, int BN_SUB, int NSPLIT, int WAVES_M, int WAVES_N, int EPI>
static void launch_fp8(const GemmParams& p, bool blockwise, dim3 grid, hipStream_t s) {
    constexpr size_t lds = gemm_lds_bytes(BM, BN_SUB, EPI, WAVES_M * WAVES_N);
    constexpr int threads = WAVES_M * WAVES_N * 64;
    if (blockwise) gemm_kernel<BM, BN_SUB, NSPLIT, WAVES_M, WAVES_N, false, true, EPI><<<grid, threads, lds, s>>>(p);
    else gemm_kernel<BM, BN_SUB, NSPLIT, WAVES_M, WAVES_N, false, false, EPI><<<grid, threads, lds, s>>>(p);
}

// gemm_wreg.hip
bool wreg_supports(int64_t M, int64_t N, int64_t K);
bool wreg_supports_fused(int64_t M, int64_t N, int64_t K);
int wreg_plan(int64_t M, int64_t N, int64_t K, int64_t batch, int cus, bool fp8_out, bool bf16_in, const void** fn, size_t* lds);
void wreg_launch(const GemmParams& p, dim3 grid, hipStream_t s);
static void launch_wreg_any(const GemmParams& p, bool, dim3 grid, hipStream_t s) { wreg_launch(p, grid, s); }
static const char kWregName[] = "wreg32";

// gemm_strip.hip
bool strip_supports(int64_t M, int64_t N, int64_t K);
bool strip_supports_fused(int64_t M, int64_t N, int64_t K);
int strip_plan(int64_t M, int64_t N, int64_t K, int64_t batch, int cus, bool bf16_in, bool fp8_out, const void** fn, size_t* lds);
void strip_launch(const GemmParams& p, dim3 grid, hipStream_t s);
static void launch_strip_any(const GemmParams& p, bool, dim3 grid, hipStream_t s) { strip_launch(p, grid, s); }
static const char kStripName[] = "strip32";
static const char kPanel32Name[] = "panel32_256x256";

// gemm_panel32.hip
const void* panel32_fn(int bw, bool fp8out, bool affine, bool qpro = false);
bool panel32_affine(const GemmParams& p);
size_t panel32_lds();
void panel32_launch(const GemmParams& p, int bw, dim3 grid, hipStream_t s);
// block scales: power-of-two ones go to the matrix cores, others rescale the accumulators
static int panel32_bw(const GemmParams& p, bool blockwise) { return !blockwise ? 0 : scale_mode_is_pow2(p.x_mode) ? 2 : 1; }
static void launch_panel32(const GemmParams& p, bool blockwise, dim3 grid, hipStream_t s) {
    panel32_launch(p, panel32_bw(p, blockwise), grid, s);
}

template <int BM, int BN_SUB, int NSPLIT, int WAVES_M, int WAVES_N, int EPI>
static void launch_exact(const GemmParams& p, bool, dim3 grid, hipStream_t s) {
    constexpr size_t lds = 2 * (BM * 128 + BN_SUB * 128);
    gemm_kernel<BM, BN_SUB, NSPLIT, WAVES_M, WAVES_N, false, false, EPI, true><<<grid, WAVES_M * WAVES_N * 64, lds, s>>>(p);
}
#define LOKA_VARIANT_EXACT(NAME, BM, BN_SUB, NSPLIT, WAVES_M, WAVES_N, EPI)                                  \
    {NAME, BM, BN_SUB * NSPLIT, WAVES_M * WAVES_N * 64, EPI, 2 * (BM * 128 + BN_SUB * 128),                  \
     &launch_exact<BM, BN_SUB, NSPLIT, WAVES_M, WAVES_N, EPI>,                                               \
     reinterpret_cast<const void*>(&gemm_kernel<BM, BN_SUB, NSPLIT, WAVES_M, WAVES_N, false, false, EPI, true>), nullptr}

#define LOKA_VARIANT(NAME, BM, BN_SUB, NSPLIT, WAVES_M, WAVES_N, EPI)                                        \
    {NAME, BM, BN_SUB * NSPLIT, WAVES_M * WAVES_N * 64, EPI, gemm_lds_bytes(BM, BN_SUB, EPI, WAVES_M * WAVES_N), \
     &launch_fp8<BM, BN_SUB, NSPLIT, WAVES_M, WAVES_N, EPI>,                                                 \
     reinterpret_cast<const void*>(&gemm_kernel<BM, BN_SUB, NSPLIT, WAVES_M, WAVES_N, false, false, EPI>),   \
     reinterpret_cast<const void*>(&gemm_kernel<BM, BN_SUB, NSPLIT, WAVES_M, WAVES_N, false, true, EPI>)}

static const VariantInfo kVariants[] = {
    // rows normalized inside the tile (the tile spans the whole row)
    LOKA_VARIANT("row32x128", 32, 128, 1, 1, 4, EPI_ROW_IN_TILE),
    LOKA_VARIANT("row64x128", 64, 128, 1, 2, 2, EPI_ROW_IN_TILE),
    LOKA_VARIANT("row64x256", 64, 256, 1, 1, 4, EPI_ROW_IN_TILE),
    LOKA_VARIANT("row128x256", 128, 256, 1, 2, 4, EPI_ROW_IN_TILE),
    LOKA_VARIANT("row64x512", 64, 512, 1, 1, 8, EPI_ROW_IN_TILE),
    LOKA_VARIANT("row64x1024", 64, 512, 2, 1, 8, EPI_ROW_IN_TILE),
    // exact products: e4m3 operands widened to bf16 in registers and contracted on the BF16 matrix instruction (the
    // accuracy-first candidates of the non-blockwise recipes: fp32 Y agrees with exact arithmetic up to fp32 summation)
    LOKA_VARIANT_EXACT("exact64x256", 64, 256, 1, 1, 4, EPI_ROW_IN_TILE),
    LOKA_VARIANT_EXACT("exact64x512", 64, 512, 1, 1, 8, EPI_ROW_IN_TILE),
    LOKA_VARIANT_EXACT("exact64x1024", 64, 512, 2, 1, 8, EPI_ROW_IN_TILE),
    // skinny layers (K * N <= 256 KB, non-blockwise scales): W resident in registers, X streamed in 32-row
    // blocks; one of several instantiations behind one name, workgroup count and LDS decided at launch
    {kWregName, 32, 1024, 512, EPI_ROW_IN_TILE, 0, &launch_wreg_any, nullptr, nullptr},
    // small layers (K * N <= 128 KB, N <= 256, non-blockwise scales): W resident in LDS, one 32-row strip per wave,
    // no synchronization between the waves of a workgroup; workgroup count and LDS decided at launch
    {kStripName, 32, 256, 512, EPI_ROW_IN_TILE, 0, &launch_strip_any, nullptr, nullptr},
    // rows spanning several workgroups: Y + per-tile statistics, then a normalization pass
    LOKA_VARIANT("twopass128x128", 128, 128, 1, 2, 2, EPI_PARTIAL_STATS),
    LOKA_VARIANT("twopass256x256", 256, 256, 1, 2, 2, EPI_PARTIAL_STATS),
    LOKA_VARIANT("twopass256x256w8", 256, 256, 1, 2, 4, EPI_PARTIAL_STATS),
    // split K: layers with few output tiles and a long K (weight gradients, the widest layers at small batch); ksplit
    // workgroups per tile contract a K range each into fp32 partial sums, a second kernel adds them and normalizes.
    // Two forms: eight waves on a ring of four LDS stages, one workgroup per CU (short ranges: a weight gradient), and
    // four waves on two stages, two workgroups per CU (long ranges)
    LOKA_VARIANT("splitk128x128", 128, 128, 1, 2, 4, EPI_SPLITK),
    LOKA_VARIANT("splitk128x128s2", 128, 128, 1, 2, 2, EPI_SPLITK),
    // persistent, panel-synchronous: the tiles_n workgroups of a row panel exchange row statistics
    // through a few words of global memory and normalize their own tile in registers
    LOKA_VARIANT("panel256x256w8", 256, 256, 1, 2, 4, EPI_PANEL_SYNC),
    // the same schedule on 32x32x64 MFMAs: the throughput variant
    {kPanel32Name, 256, 256, 512, EPI_PANEL_SYNC, panel32_lds(), &launch_panel32, panel32_fn(0, false, false), panel32_fn(1, false, false)},
};
constexpr int kMaxRowTiles = 256;     // shape limit of the panel-synchronous schedule (a row's tiles must be co-resident:
                                      // the launch checks them against the CU count of the device it runs on)
constexpr unsigned kSpinLimit = 1u << 18;   // polls of ~1 us each (a device-scope load and a short sleep): far beyond any main loop
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

int variant_count() { return kNumVariants; }
const char* variant_name(int v) { return (v >= 0 && v < kNumVariants) ? kVariants[v].name : nullptr; }
int variant_epilogue(int v) { return kVariants[v].epi; }
bool variant_supports(const loka_gemm_desc* d, int v);
// kernels that can take bf16 X and quantize it per row themselves (loka_fp8_linear_norm)
bool variant_supports_fused(const loka_gemm_desc* d, int v) {
    if (v < 0 || v >= kNumVariants || !variant_supports(d, v) || d->x_mode != LOKA_SCALE_ROW) return false;
    if (kVariants[v].name == kWregName) return wreg_supports_fused(d->M, d->N, d->K);
    if (kVariants[v].name == kStripName) return strip_supports_fused(d->M, d->N, d->K);
    return false;
}
// the streaming kernel with its quantize prologue (loka_fp8_linear_norm_xq): every shape the kernel covers, row scales
// for X, one problem or separate activations per problem
bool variant_supports_xq(const loka_gemm_desc* d, int v) {
    if (v < 0 || v >= kNumVariants || !variant_supports(d, v) || d->x_mode != LOKA_SCALE_ROW) return false;
    if (d->batch != 1 && d->strideX == 0) return false;
    if (kVariants[v].name == kWregName) return true;
    // the large-tile kernel when a tile spans the output row (its rows of X then belong to one workgroup) and a row of
    // X is 1, 2 or 4 loads of a whole wave
    if (kVariants[v].name == kPanel32Name)
        return d->N <= 256 && (d->K == 512 || d->K == 1024 || d->K == 2048) && d->M * d->K < (int64_t(1) << 31);
    return false;
}
int default_variant(const loka_gemm_desc* d);
// the library's choice for the shape when it has the prologue, else the first kernel that has it
int variant_xq_default(const loka_gemm_desc* d) {
    const int v0 = default_variant(d);
    if (variant_supports_xq(d, v0)) return v0;
    for (int v = 0; v < kNumVariants; ++v)
        if (variant_supports_xq(d, v)) return v;
    return -1;
}
// the kernel the fused entry point uses when the caller names none: the strip kernel where it applies (waves that
// never synchronize, one strip each), else the streaming kernel
int variant_fused_default(const loka_gemm_desc* d) {
    int wreg = -1;
    for (int v = 0; v < kNumVariants; ++v) {
        if (!variant_supports_fused(d, v)) continue;
        if (kVariants[v].name == kStripName) return v;
        wreg = v;
    }
    return wreg;
}
int variant_streaming_id() {
    for (int v = 0; v < kNumVariants; ++v)
        if (kVariants[v].name == kWregName) return v;
    return -1;
}
bool variant_is_streaming(int v) { return kVariants[v].name == kWregName; }
bool variant_is_strip(int v) { return kVariants[v].name == kStripName; }
bool variant_is_panel32(int v) { return kVariants[v].name == kPanel32Name; }
bool variant_is_exact(int v) { return kVariants[v].launch != nullptr && kVariants[v].name[0] == 'e' && kVariants[v].name[1] == 'x'; }
int variant_bn(int v) { return kVariants[v].bn; }
int variant_bm(int v) { return kVariants[v].bm; }

// Split K: the number of K ranges and their length in 128-byte steps.  The ring form: as many ranges as give an
// MI355X's 256 CUs one workgroup each and no more (its stages fill a CU's LDS: a 257th workgroup would be a second
// round).  The two-stage form: about two workgroups per CU.  At least 4 steps per range, at most 64 ranges.  (Fixed
// figures, not the device's CU count: the workspace size follows from them and must not depend on the device.)
static void splitk_plan(const loka_gemm_desc* d, const VariantInfo& vi, int* ksplit, int* per) {
    const int64_t tiles = ((d->M + vi.bm - 1) / vi.bm) * ((d->N + vi.bn - 1) / vi.bn) * d->batch;
    const int64_t steps = (d->K + 127) / 128;
    int64_t want = vi.threads == 512 ? 256 / tiles : (512 + tiles - 1) / tiles;
    if (want > 64) want = 64;
    if (want > steps / 4) want = steps / 4;
    if (want < 1) want = 1;
    const int64_t len = (steps + want - 1) / want;
    *per = static_cast<int>(len);
    *ksplit = static_cast<int>((steps + len - 1) / len);
}

bool variant_supports(const loka_gemm_desc* d, int v);
// the split-K form for the shape: the ring form unless its ranges would be long (measured: 65536 x 256 x 1024 as a weight
// gradient, 32 steps per range, 43.5 us against 48.5 us for the two-stage form; 2048 x 123200 x 1024, 482 steps per range,
// 437 us against 400 us), the other form where only one of them splits K at all
int variant_splitk_choice(const loka_gemm_desc* d) {
    int ring = -1, two = -1;
    for (int v = 0; v < kNumVariants; ++v) {
        if (kVariants[v].epi != EPI_SPLITK || !variant_supports(d, v)) continue;
        if (kVariants[v].threads == 512) ring = v; else two = v;
    }
    if (ring < 0 || two < 0) return ring >= 0 ? ring : two;
    int ksplit = 1, per = 1;
    splitk_plan(d, kVariants[ring], &ksplit, &per);
    return per <= 128 ? ring : two;
}

bool variant_supports(const loka_gemm_desc* d, int v) {
    if (v < 0 || v >= kNumVariants) return false;
    const VariantInfo& vi = kVariants[v];
    if (vi.name == kWregName) return !scale_mode_is_block(d->x_mode) && wreg_supports(d->M, d->N, d->K);
    if (vi.name == kStripName)
        return !scale_mode_is_block(d->x_mode) && d->norm != LOKA_NORM_BLOCKNORM && strip_supports(d->M, d->N, d->K);
    // a K that is not a multiple of 128 (the non-blockwise recipes allow any multiple of 16): the general tiled kernel
    // masks the tail of the last K step; the 32x32 panel kernel does not
    if (vi.name == kPanel32Name && d->K % 128) return false;
    // BlockNorm (groups of 256 columns) is built into the kernels whose tile is 256 columns wide
    if (d->norm == LOKA_NORM_BLOCKNORM && vi.launch != &launch_panel32) return false;
    if ((scale_mode_is_block(d->x_mode) ? vi.fn_block : vi.fn_plain) == nullptr) return false;
    if (vi.epi == EPI_SPLITK) {
        // (offered where K actually gets split: with a single range it is the two-pass schedule with more traffic)
        int ksplit = 1, per = 1;
        splitk_plan(d, vi, &ksplit, &per);
        if (d->N > kSplitkMaxN || d->norm == LOKA_NORM_BLOCKNORM || ksplit < 2) return false;
    }
    if (vi.epi == EPI_ROW_IN_TILE && d->N > vi.bn) return false;
    if (vi.epi == EPI_PANEL_SYNC && (d->N + vi.bn - 1) / vi.bn > kMaxRowTiles) return false;
    if (static_cast<int64_t>(vi.bm > vi.bn ? vi.bm : vi.bn) * d->K >= (int64_t(1) << 31)) return false;   // tile-relative offsets are 32-bit
    const int64_t tiles = ((d->M + vi.bm - 1) / vi.bm) * ((d->N + vi.bn - 1) / vi.bn) * d->batch;
    return tiles < (int64_t(1) << 31);
}

// the variant's workspace starts with the flag a workgroup raises when its bounded wait for the panel runs out
// The panel-synchronous launch exchanges row statistics between workgroups (and has a bounded wait with an error
// flag) unless there is nothing to exchange: no row norm, groups inside a tile, or - in the 32x32 kernel, which
// then finalizes in the tile - a single tile per row.
// With FP8 output the 32x32 kernel also exchanges under BlockNorm: the groups stay inside a tile, the row amax of
// the result does not.
static bool panel_exchanges(const loka_gemm_desc* d, const VariantInfo& vi, bool fp8out = false) {
    if (vi.epi != EPI_PANEL_SYNC || d->norm == LOKA_NORM_NONE) return false;
    if (d->norm == LOKA_NORM_BLOCKNORM && !(fp8out && vi.name == kPanel32Name)) return false;
    return !(vi.name == kPanel32Name && d->N <= vi.bn);
}

bool variant_has_wait_flag(const loka_gemm_desc* d, int v, bool fp8out) { return panel_exchanges(d, kVariants[v], fp8out); }

// one 8-byte arrival word per (row panel, tile of the panel); the 32x32 kernel has a second set for the second
// exchange of its FP8-output form
static size_t panel_flag_bytes(const loka_gemm_desc* d, const VariantInfo& vi) {
    const int64_t panels = d->batch * ((d->M + vi.bm - 1) / vi.bm), tiles_n = (d->N + vi.bn - 1) / vi.bn;
    return (static_cast<size_t>(panels) * tiles_n * 8 * (vi.name == kPanel32Name ? 2 : 1) + 255) & ~size_t(255);
}

size_t variant_workspace(const loka_gemm_desc* d, int v, bool fp8out) {
    const VariantInfo& vi = kVariants[v];
    if (vi.epi == EPI_SPLITK) {
        int ksplit = 1, per = 1;
        splitk_plan(d, vi, &ksplit, &per);
        return static_cast<size_t>(ksplit) * d->batch * d->M * d->N * sizeof(float);
    }
    if (vi.epi == EPI_ROW_IN_TILE || d->norm == LOKA_NORM_NONE) return 0;
    if (d->norm == LOKA_NORM_BLOCKNORM && !panel_exchanges(d, vi, fp8out)) return 0;
    const int64_t tiles_n = (d->N + vi.bn - 1) / vi.bn;
    size_t stats = static_cast<size_t>(d->batch) * d->M * tiles_n * 2 * sizeof(float);
    // the 32x32 panel kernel keeps a record for every row of every 256-row panel, and its FP8-output form exchanges
    // the row minimum and maximum as well
    if (vi.name == kPanel32Name) stats = static_cast<size_t>(d->batch) * ((d->M + vi.bm - 1) / vi.bm) * vi.bm * tiles_n * 2 * sizeof(float) * 2;
    stats = (stats + 255) & ~size_t(255);
    if (vi.epi == EPI_PANEL_SYNC) {
        if (!panel_exchanges(d, vi, fp8out)) return 0;
        // [header, 256 B: launch nonce, nonce of the last launch with a wait that ran out][arrival words][per-tile row statistics]
        return 256 + panel_flag_bytes(d, vi) + stats;
    }
    // fp32 Y staging for the normalization pass (used when the caller does not ask for Y)
    return stats + static_cast<size_t>(d->batch) * d->M * d->N * sizeof(float);
}

__global__ void zero_u32_kernel(uint32_t* p, int64_t n) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// ---- what a launch needs to know about the device and its kernels, asked once per process and device.
// The hot calls then do nothing but fill the parameter block and launch.
namespace {
constexpr int kMaxDevices = 64;
struct FnState { const void* fn; size_t lds; int threads; int per_cu; };   // attribute set; workgroups per CU (-1: not asked yet)
struct DeviceState {
    int cus = 0;                       // 0: not asked yet
    std::vector<FnState> fns;
};
std::mutex g_dev_mu;
DeviceState g_dev[kMaxDevices];
std::atomic<long long> g_spin_override{-1};   // loka_test_set_spin_limit
std::atomic<unsigned long long> g_nonce_seq{0};
}  // namespace

// Current device and its CU count.
static loka_status device_cus(int* dev, int* cus) {
    LOKA_HIP_TRY(hipGetDevice(dev));
    if (*dev < 0 || *dev >= kMaxDevices) return LOKA_ERR_HIP;
    std::lock_guard<std::mutex> lk(g_dev_mu);
    DeviceState& st = g_dev[*dev];
    if (st.cus == 0) LOKA_HIP_TRY(hipDeviceGetAttribute(&st.cus, hipDeviceAttributeMultiprocessorCount, *dev));
    *cus = st.cus;
    return LOKA_OK;
}
int device_cu_count() {
    int dev = 0, cus = 0;
    return device_cus(&dev, &cus) == LOKA_OK ? cus : 0;
}

// Makes `fn` launchable with `lds` bytes of dynamic LDS on device `dev` (once) and returns how many of its
// workgroups fit a CU (asked once).
static loka_status prepare_fn(int dev, const void* fn, int threads, size_t lds, int* per_cu) {
    std::lock_guard<std::mutex> lk(g_dev_mu);
    for (FnState& f : g_dev[dev].fns)
        if (f.fn == fn && f.lds == lds && f.threads == threads) {
            if (per_cu && f.per_cu < 0) LOKA_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&f.per_cu, fn, threads, lds));
            if (per_cu) *per_cu = f.per_cu;
            return LOKA_OK;
        }
    FnState f{fn, lds, threads, -1};
    LOKA_HIP_TRY(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)));
    if (per_cu) LOKA_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&f.per_cu, fn, threads, lds));
    g_dev[dev].fns.push_back(f);
    if (per_cu) *per_cu = f.per_cu;
    return LOKA_OK;
}

// A 64-bit value no earlier launch of this process has used and stale memory will not hold: odd, never 0.
static unsigned long long fresh_nonce() {
    static const unsigned long long seed = [] {
        unsigned long long z = static_cast<unsigned long long>(std::chrono::steady_clock::now().time_since_epoch().count());
        z ^= reinterpret_cast<uintptr_t>(&g_nonce_seq) * 0x9E3779B97F4A7C15ull;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }();
    return (seed + 4ull * g_nonce_seq.fetch_add(1, std::memory_order_relaxed)) | 1ull;
}

void test_set_spin_limit(long long polls) { g_spin_override.store(polls, std::memory_order_relaxed); }

static loka_status gemm_norm_launch_impl(const loka_gemm_desc* d, int v, const uint8_t* xq, const float* sx, const uint8_t* wq,
                                        const float* sw, const void* gamma, const void* beta, void* out, float* y,
                                        uint8_t* outq, float* outs, const void* x_bf16, float* sx_out, void* workspace,
                                        hipStream_t s, bool quantize_prologue = false);

loka_status fp8_gemm_norm_launch(const loka_gemm_desc* d, int v, const uint8_t* xq, const float* sx, const uint8_t* wq,
                                 const float* sw, const void* gamma, const void* beta, void* out, float* y,
                                 uint8_t* outq, float* outs, void* workspace, hipStream_t s) {
    return gemm_norm_launch_impl(d, v, xq, sx, wq, sw, gamma, beta, out, y, outq, outs, nullptr, nullptr, workspace, s);
}

// bf16 X quantized row by row inside the streaming kernel (v must be that variant)
loka_status fp8_linear_norm_launch(const loka_gemm_desc* d, int v, const void* x_bf16, const uint8_t* wq, const float* sw,
                                   const void* gamma, const void* beta, void* out, float* y, float* sx_out, hipStream_t s) {
    if (!variant_supports_fused(d, v)) return LOKA_ERR_UNSUPPORTED;
    return gemm_norm_launch_impl(d, v, nullptr, nullptr, wq, sw, gamma, beta, out, y, nullptr, nullptr, x_bf16, sx_out, nullptr, s);
}

// bf16 X quantized row by row by the workgroup that consumes the rows, codes and scales handed back (v must be the
// streaming kernel's variant; every shape it covers)
loka_status fp8_linear_norm_xq_launch(const loka_gemm_desc* d, int v, const void* x_bf16, uint8_t* xq_out, float* sx_out,
                                      const uint8_t* wq, const float* sw, const void* gamma, const void* beta, void* out,
                                      float* y, hipStream_t s) {
    if (!variant_supports_xq(d, v)) return LOKA_ERR_UNSUPPORTED;
    return gemm_norm_launch_impl(d, v, xq_out, sx_out, wq, sw, gamma, beta, out, y, nullptr, nullptr, x_bf16, nullptr, nullptr, s,
                                 true);
}

static loka_status gemm_norm_launch_impl(const loka_gemm_desc* d, int v, const uint8_t* xq, const float* sx, const uint8_t* wq,
                                        const float* sw, const void* gamma, const void* beta, void* out, float* y,
                                        uint8_t* outq, float* outs, const void* x_bf16, float* sx_out, void* workspace,
                                        hipStream_t s, bool quantize_prologue) {
    const VariantInfo& vi = kVariants[v];
    const bool blockwise = scale_mode_is_block(d->x_mode);
    GemmParams p{};
    p.X = xq; p.W = wq;
    p.M = static_cast<int>(d->M); p.N = static_cast<int>(d->N); p.KB = static_cast<int>(d->K);
    p.batch = static_cast<int>(d->batch);
    p.strideX = d->strideX; p.strideW = d->strideW; p.strideO = d->strideO;
    p.sx = sx; p.sw = sw;
    p.strideSx = d->strideX ? loka_scale_count(static_cast<loka_scale_mode>(d->x_mode), d->M, d->K) : 0;
    p.strideSw = d->strideW ? loka_scale_count(static_cast<loka_scale_mode>(d->w_mode), d->K, d->N) : 0;
    p.x_mode = d->x_mode; p.w_mode = d->w_mode;
    p.gamma = static_cast<const uint16_t*>(gamma); p.beta = static_cast<const uint16_t*>(beta);
    p.out = static_cast<uint16_t*>(out); p.y = y;
    p.outq = outq; p.outs = outs;
    p.xb = static_cast<const uint16_t*>(x_bf16); p.sx_out = sx_out;
    p.qpro = quantize_prologue ? 1 : 0;
    // FP8 output: the row stays inside one workgroup (streaming kernel) or one wave (strip kernel), or - panel kernel -
    // the row amax crosses the workgroups: as the row's extreme pre-norm values along with the row statistics when
    // there is no gamma / beta (the normalized value then grows with the pre-norm value), else in a second exchange.
    // The second exchange also serves BlockNorm (+ Hard-Swish), whose statistics never leave the tile.  A row norm is
    // required; non-blockwise scales.
    if (outq && vi.name == kPanel32Name) {
        if (blockwise || d->norm == LOKA_NORM_NONE) return LOKA_ERR_UNSUPPORTED;
    } else if (outq && vi.name != kWregName && vi.name != kStripName) {
        return LOKA_ERR_UNSUPPORTED;
    }
    p.norm = d->norm; p.eps = d->eps; p.block_n = d->block_n; p.act = d->act;
    p.tiles_m = static_cast<int>((d->M + vi.bm - 1) / vi.bm);
    p.tiles_n = static_cast<int>((d->N + vi.bn - 1) / vi.bn);
    const bool two_pass = vi.epi == EPI_PARTIAL_STATS && d->norm != LOKA_NORM_NONE && d->norm != LOKA_NORM_BLOCKNORM;
    if (two_pass) {
        size_t stats = static_cast<size_t>(d->batch) * d->M * p.tiles_n * 2 * sizeof(float);
        stats = (stats + 255) & ~size_t(255);
        p.part = static_cast<float*>(workspace);
        if (!y) p.y = reinterpret_cast<float*>(static_cast<uint8_t*>(workspace) + stats);
    }
    int dev = 0, cus = 0;
    if (device_cus(&dev, &cus) != LOKA_OK) return LOKA_ERR_HIP;
    if (vi.name == kWregName || vi.name == kStripName) {
        const void* fn = nullptr;
        size_t lds = 0;
        const int wgs = vi.name == kWregName
                            ? wreg_plan(d->M, d->N, d->K, d->batch, cus, p.outq != nullptr, p.xb != nullptr && !p.qpro, &fn, &lds)
                            : strip_plan(d->M, d->N, d->K, d->batch, cus, p.xb != nullptr, p.outq != nullptr, &fn, &lds);
        if (wgs <= 0) return LOKA_ERR_UNSUPPORTED;
        if (prepare_fn(dev, fn, vi.threads, lds, nullptr) != LOKA_OK) return LOKA_ERR_HIP;
        vi.launch(p, false, dim3(static_cast<unsigned>(wgs)), s);
        return hipGetLastError() == hipSuccess ? LOKA_OK : LOKA_ERR_HIP;
    }
    const void* kfn = blockwise ? vi.fn_block : vi.fn_plain;
    if (vi.name == kPanel32Name) kfn = panel32_fn(panel32_bw(p, blockwise), outq != nullptr, panel32_affine(p), p.qpro != 0);
    if (!kfn) return LOKA_ERR_UNSUPPORTED;
    int per_cu = 0;
    if (prepare_fn(dev, kfn, vi.threads, vi.lds, &per_cu) != LOKA_OK) return LOKA_ERR_HIP;
    dim3 grid(static_cast<unsigned>(static_cast<int64_t>(p.tiles_m) * p.tiles_n * p.batch));
    if (vi.epi == EPI_PANEL_SYNC) {
        // persistent grid: a multiple of tiles_n workgroups, all resident at once (one per CU)
        const int64_t slots = static_cast<int64_t>(cus) * (per_cu > 0 ? 1 : 0);
        int64_t g = (slots / p.tiles_n) * p.tiles_n;
        if (g <= 0) return LOKA_ERR_UNSUPPORTED;
        if (g > grid.x) g = (static_cast<int64_t>(grid.x) / p.tiles_n) * p.tiles_n;   // fewer tiles than slots
        grid = dim3(static_cast<unsigned>(g));
        if (panel_exchanges(d, vi, outq != nullptr)) {
            const size_t flag_bytes = panel_flag_bytes(d, vi);
            uint8_t* ws = static_cast<uint8_t*>(workspace);
            p.header = reinterpret_cast<unsigned long long*>(ws);
            p.flags = reinterpret_cast<unsigned long long*>(ws + 256);
            p.part = reinterpret_cast<float*>(ws + 256 + flag_bytes);
            p.spin_limit = kSpinLimit;
            p.nonce = fresh_nonce();
            p.expect = p.nonce;
            // Test hook for the error path (loka_test_set_spin_limit): a limit of 0 polls also makes the workgroups
            // look for a value nobody writes, so that every wait runs out after its first poll whatever the timing
            // (the kernel still ends; the rows of that launch leave as NaN).
            const long long ov = g_spin_override.load(std::memory_order_relaxed);
            if (ov >= 0) {
                p.spin_limit = static_cast<unsigned>(ov);
                if (ov == 0) p.expect = p.nonce + 2;
            }
            // Arrival words are compared with the launch's nonce, which is new for every launch: nothing to clear.
            // A launch that is being recorded into a graph will be replayed with the SAME nonce, so there the header
            // and the arrival words are cleared by a kernel in front of it (part of the recording).
            hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
            if (hipStreamIsCapturing(s, &cap) != hipSuccess) return LOKA_ERR_HIP;
            if (cap != hipStreamCaptureStatusNone) {
                const int64_t words = (256 + static_cast<int64_t>(flag_bytes)) / 4;
                zero_u32_kernel<<<dim3(static_cast<unsigned>((words + 255) / 256)), 256, 0, s>>>(
                    reinterpret_cast<uint32_t*>(ws), words);
            }
        }
    }
    if (vi.epi == EPI_SPLITK) {
        splitk_plan(d, vi, &p.ksplit, &p.k_per_split);
        p.part = static_cast<float*>(workspace);
        p.y = nullptr;                                  // (the second kernel writes Y)
        grid.y = static_cast<unsigned>(p.ksplit);
        vi.launch(p, blockwise, grid, s);
        const int64_t rows = static_cast<int64_t>(d->batch) * d->M;
        // few rows (a weight gradient's K x N output): a workgroup per row, else a wave per row
        if (rows < 8192)
            splitk_norm_rows_kernel<4><<<dim3(static_cast<unsigned>(rows)), 256, 0, s>>>(
                p.part, p.ksplit, rows, p.M, p.N, p.strideO, d->norm, d->eps, p.gamma, p.beta, p.out, y);
        else
            splitk_norm_rows_kernel<1><<<dim3(static_cast<unsigned>((rows + 3) / 4)), 256, 0, s>>>(
                p.part, p.ksplit, rows, p.M, p.N, p.strideO, d->norm, d->eps, p.gamma, p.beta, p.out, y);
        return hipGetLastError() == hipSuccess ? LOKA_OK : LOKA_ERR_HIP;
    }
    vi.launch(p, blockwise, grid, s);
    if (two_pass) {
        // with a strided batch the rows of all problems are contiguous only when strideO == M*N
        for (int g = 0; g < p.batch; ++g) {
            const float* yg = p.y + static_cast<int64_t>(g) * p.strideO;
            const float* pg = p.part + static_cast<int64_t>(g) * d->M * p.tiles_n * 2;
            uint16_t* og = p.out + static_cast<int64_t>(g) * p.strideO;
            norm_rows_kernel<<<dim3(static_cast<unsigned>((d->M + 3) / 4)), 256, 0, s>>>(
                yg, pg, d->M, p.N, p.tiles_n, vi.bn, d->norm, d->eps, p.gamma, p.beta, og);
        }
    }
    return hipGetLastError() == hipSuccess ? LOKA_OK : LOKA_ERR_HIP;
}

// BF16 reference GEMM: 128 x 128 tiles, fp32 Y only.
size_t bf16_gemm_workspace_bytes(const loka_gemm_desc* d) {
    const int64_t nw = d->strideW ? d->batch : 1;
    return static_cast<size_t>(nw) * d->K * d->N * 2;
}

// weights_ready: the workspace already holds the transposed weights of an earlier call with the same w (the
// dispatcher times the reference with its weights prepared once, like the FP8 candidates' quantized weights)
loka_status bf16_gemm_launch(const loka_gemm_desc* d, const void* x, const void* w, float* yref, void* workspace,
                             hipStream_t s, bool weights_ready) {
    uint16_t* wt = static_cast<uint16_t*>(workspace);
    const int64_t nw = d->strideW ? d->batch : 1;
    for (int64_t g = 0; g < nw && !weights_ready; ++g) {
        dim3 grid(static_cast<unsigned>((d->N + 63) / 64), static_cast<unsigned>((d->K + 63) / 64));
        transpose_bf16_kernel<<<grid, 256, 0, s>>>(static_cast<const uint16_t*>(w) + g * d->strideW,
                                                   static_cast<int>(d->K), static_cast<int>(d->N), wt + g * d->K * d->N);
    }
    constexpr int BM = 128, BN = 128;
    GemmParams p{};
    p.X = static_cast<const uint8_t*>(x); p.W = reinterpret_cast<const uint8_t*>(wt);
    p.M = static_cast<int>(d->M); p.N = static_cast<int>(d->N); p.KB = static_cast<int>(d->K * 2);
    p.batch = static_cast<int>(d->batch);
    p.strideX = d->strideX * 2; p.strideW = d->strideW ? d->K * d->N * 2 : 0; p.strideO = d->strideO;
    p.y = yref;
    p.norm = LOKA_NORM_NONE;
    p.tiles_m = static_cast<int>((d->M + BM - 1) / BM);
    p.tiles_n = static_cast<int>((d->N + BN - 1) / BN);
    auto fn = &gemm_kernel<BM, BN, 1, 2, 2, true, false, EPI_PARTIAL_STATS>;
    constexpr size_t lds = 2 * (BM * 128 + BN * 128);
    int dev = 0, cus = 0;
    if (device_cus(&dev, &cus) != LOKA_OK || prepare_fn(dev, reinterpret_cast<const void*>(fn), 256, lds, nullptr) != LOKA_OK)
        return LOKA_ERR_HIP;
    const dim3 grid(static_cast<unsigned>(static_cast<int64_t>(p.tiles_m) * p.tiles_n * p.batch));
    fn<<<grid, 256, lds, s>>>(p);
    return hipGetLastError() == hipSuccess ? LOKA_OK : LOKA_ERR_HIP;
}

}  // namespace loka
