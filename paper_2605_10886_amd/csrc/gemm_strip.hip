// Small-layer FP8 GEMM with the row norm fused, one row strip per WAVE: W in LDS, X straight into registers.
//
// For the many small GEMMs of a recommendation model (Section 2.1; K * N <= 128 KB, N <= 256: 256 x 256, 512 x 256,
// 1024 x 128, ...)
// a whole output row fits the accumulators of ONE wave: a wave takes 32 rows of X, multiplies them with all of
// W (resident in LDS for the whole problem, read fragment by fragment), and scales, normalizes and stores its
// 32 x N outputs from registers.  The row statistics need two lanes (l, l ^ 32) and no other wave, so after the
// weights are in place the 8 waves of a workgroup never synchronize: each runs load -> MFMA -> normalize -> store
// at its own pace, and the phases of different waves overlap on the CU.  (The streaming kernel for skinny
// layers splits the row over its 8 waves and runs those phases one after the other behind workgroup barriers;
// measured at 64 x (4096 x 256 x 256) it needs 7.4 us per 128 rows against 3.1 us of HBM time.)
//
// X does not pass through LDS: the MFMA operand of a lane is 32 consecutive K bytes of one row, which two
// 16-byte loads fetch directly (two lanes cover a 64-byte run of the row); the next strip's operands are
// requested before the current strip is multiplied.  Roles and the W row permutation are those of the other
// 32 x 32 x 64 kernels: W rows -> MFMA rows, X rows -> MFMA columns, so a lane ends with 16 consecutive output
// columns per column block of one output row (= lane % 32).
#include "gemm_common.h"

#include <type_traits>

namespace loka {

typedef float v16f __attribute__((ext_vector_type(16)));


template <int NB, int KS, int NPH>
struct StripCfg {
    static constexpr int NT = NB * 32;                    // columns the accumulators cover
    static constexpr int KB = KS * 64;                    // K bytes per phase = bytes per row of the W slab in LDS
    static constexpr int KBT = NPH * KB;                  // bytes per row of X / W in memory
    static constexpr int SWIN = KB / 16 < 16 ? KB / 16 : 16;
    static constexpr int OFF_W = 0;                       // [NT][KB], 16-byte chunk c of row r at c ^ (r % SWIN)
    static constexpr int OFF_SW = NT * KB;                // [NT] fp32 column scales (0 beyond N)
    static constexpr int OFF_GM = OFF_SW + NT * 4;        // [NT] fp32 gamma (1 when absent)
    static constexpr int OFF_BT = OFF_GM + NT * 4;        // [NT] fp32 beta (0 when absent)
    static constexpr int OFF_T = OFF_BT + NT * 4;         // [8 waves][2 KB] output staging (see the epilogue)
    static constexpr int LDS = OFF_T + 8 * 2048;
    static_assert(LDS <= 160 * 1024, "W, the tables and the staging buffers must fit the LDS");
};

// NWV waves per workgroup; BF16IN: X arrives as bf16 and is quantized per row (amax, scale, e4m3 cast: the
// arithmetic of the quantize kernel, bit for bit) on its way into the MFMA operand registers, so the FP8 copy of X
// never exists in memory (Section 3.2: quantization fused with the layer).  A strip's 32 x K bf16 values are a
// second set of 16 KS registers per lane that must stay live through the previous strip's epilogue: those
// instances run with 4 waves of up to 512 registers instead of 8 of 256.
template <int NB, int KS, int NPH, int NWV, bool BF16IN, bool FP8OUT>
__global__ __launch_bounds__(NWV * 64) void gemm_strip_kernel(const GemmParams p, const int strips_per_problem) {
    using C = StripCfg<NB, KS, NPH>;
    static_assert(!BF16IN || NPH == 1, "fused quantization needs the whole row of X in one pass");
    constexpr int NT = C::NT, KB = C::KB, KBT = C::KBT, KEYMASK = C::SWIN - 1;
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, hk = lane >> 5;
    const bool ln = p.norm == LOKA_NORM_LAYERNORM;
    const bool tensor_x = p.x_mode == LOKA_SCALE_TENSOR, tensor_w = p.w_mode == LOKA_SCALE_TENSOR;
    const float inv_n = 1.0f / static_cast<float>(p.N);
    const bool affine = p.norm != LOKA_NORM_NONE && (p.gamma != nullptr || (p.beta != nullptr && ln));

    float cnt_lane = 0.f;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
        if (nb * 32 + hk * 16 < p.N) cnt_lane += 16.f;     // N % 16 == 0: a run of 16 columns is all in or all out

    // contiguous range of strips of this workgroup (strip = 32 rows of one problem)
    const int64_t total = static_cast<int64_t>(p.batch) * strips_per_problem;
    int t = static_cast<int>(total * blockIdx.x / gridDim.x);
    const int t1 = static_cast<int>(total * (blockIdx.x + 1) / gridDim.x);

    while (t < t1) {
        const int g = t / strips_per_problem;
        const int seg_end = (g + 1) * strips_per_problem < t1 ? (g + 1) * strips_per_problem : t1;

        // ---- tables of problem g; its weights (the K slab of phase ph) on request
        __syncthreads();                                    // every wave has finished with the previous problem
        const __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint8_t*>(p.W + static_cast<int64_t>(g) * p.strideW), 0, static_cast<unsigned>(p.N) * KBT, 0x00020000);
        auto load_w = [&](int ph) __attribute__((always_inline)) {
            for (int ld = wave; ld < NT * KB / 1024; ld += NWV) {
                const int byte = ld * 1024 + lane * 16;
                const int row = byte / KB, pos = (byte % KB) >> 4;
                // rows past N lie behind the descriptor's bound (the offset is the per-lane one) and read as zeros
                __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, (__attribute__((address_space(3))) void*)(smem + C::OFF_W + ld * 1024),
                                                         16, row * KBT + ph * KB + ((pos ^ (row & KEYMASK)) << 4), 0, 0, 0);
            }
        };
        {
            const float* swg = p.sw + static_cast<int64_t>(g) * p.strideSw;
            float* swl = reinterpret_cast<float*>(smem + C::OFF_SW);
            float* gml = reinterpret_cast<float*>(smem + C::OFF_GM);
            float* btl = reinterpret_cast<float*>(smem + C::OFF_BT);
            for (int n = threadIdx.x; n < NT; n += NWV * 64) {
                const bool in = n < p.N;
                swl[n] = in ? (tensor_w ? swg[0] : swg[n]) : 0.f;
                gml[n] = (in && p.gamma && p.norm != LOKA_NORM_NONE) ? bf16_bits_to_f32(p.gamma[n]) : 1.f;
                btl[n] = (in && p.beta && ln) ? bf16_bits_to_f32(p.beta[n]) : 0.f;
            }
        }
        if (NPH == 1) {
            load_w(0);
            wait_vmcnt<0>();
            __syncthreads();
        }

        const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint8_t*>(p.X + static_cast<int64_t>(g) * p.strideX), 0, static_cast<unsigned>(p.M) * KBT, 0x00020000);
        const float* sxg = p.sx + static_cast<int64_t>(g) * p.strideSx;
        const int s_base = g * strips_per_problem;

        // operands of strip s, phase ph: row m0 + l32, K bytes [KB ph + 64 j + 32 hk, +32) per K step (rows past M
        // read as zeros)
        auto load_x = [&](int s, int ph, v8i (&x)[KS], float& sxm) __attribute__((always_inline)) {
            const int m = (s - s_base) * 32 + l32;
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                const unsigned off = static_cast<unsigned>(m) * KBT + static_cast<unsigned>(ph * KB + (4 * j + 2 * hk) * 16);
                const v4i lo = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(xr, off, 0, 0));
                const v4i hi = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(xr, off + 16u, 0, 0));
                x[j] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            }
            sxm = tensor_x ? sxg[0] : (m < p.M ? sxg[m] : 0.f);
        };

        // Fused quantization: the lane's 32 bf16 values per K step (row m0 + l32, K elements [64 j + 32 hk, +32): 64
        // bytes, four loads), then row amax (integer max of the magnitudes, this lane and lane ^ 32 hold the row),
        // scale pair, cast.  Rows past M read as zeros.
        const __amdgpu_buffer_rsrc_t xbr = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t*>(BF16IN ? p.xb + static_cast<int64_t>(g) * p.strideX : nullptr), 0,
            static_cast<unsigned>(p.M) * KBT * 2u, 0x00020000);
        auto load_raw = [&](int s, u32x4 (&raw)[KS][4]) __attribute__((always_inline)) {
            const int m = (s - s_base) * 32 + l32;
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                const unsigned off = static_cast<unsigned>(m) * (KBT * 2u) + static_cast<unsigned>((64 * j + 32 * hk) * 2);
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    raw[j][q] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(xbr, off + 16u * q, 0, 0));
            }
        };
        // loads i0 <= i < i1 of the KS * 4 that make up a raw strip (i = 4 j + q)
        auto load_raw_part = [&](int s, u32x4 (&raw)[KS][4], int i0, int i1) __attribute__((always_inline)) {
            int lane_o = lane;
            asm volatile("; per-strip lane id" : "+v"(lane_o));
            const int m = (s - s_base) * 32 + (lane_o & 31);
#pragma unroll
            for (int i = 0; i < KS * 4; ++i)
                if (i >= i0 && i < i1) {
                    const unsigned off = static_cast<unsigned>(m) * (KBT * 2u) +
                                         static_cast<unsigned>((64 * (i / 4) + 32 * (lane_o >> 5)) * 2 + 16 * (i % 4));
                    raw[i / 4][i % 4] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(xbr, off, 0, 0));
                }
        };
        auto convert = [&](int s, const u32x4 (&raw)[KS][4], v8i (&x)[KS], float& sxm) __attribute__((always_inline)) {
            unsigned am = 0u;                                   // max over the lane's values of the 15 magnitude bits
#pragma unroll
            for (int j = 0; j < KS; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const unsigned w = raw[j][q][e];
                        const unsigned lo = w & 0x7FFFu, hi = (w >> 16) & 0x7FFFu;
                        am = am > lo ? am : lo;
                        am = am > hi ? am : hi;
                    }
            const unsigned other = static_cast<unsigned>(__shfl_xor(static_cast<int>(am), 32, 64));
            am = am > other ? am : other;
            float scale, inv;
            group_scale(__uint_as_float(am << 16), scale, inv);
            sxm = scale;
            const int m = (s - s_base) * 32 + l32;
            if (p.sx_out && hk == 0 && m < p.M) p.sx_out[static_cast<int64_t>(g) * p.M + m] = scale;
#pragma unroll
            for (int j = 0; j < KS; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const u32x4 w = raw[j][q];
                    x[j][2 * q] = static_cast<int>(e4m3x4(bf16_lo(w.x) * inv, bf16_hi(w.x) * inv, bf16_lo(w.y) * inv, bf16_hi(w.y) * inv));
                    x[j][2 * q + 1] = static_cast<int>(e4m3x4(bf16_lo(w.z) * inv, bf16_hi(w.z) * inv, bf16_lo(w.w) * inv, bf16_hi(w.w) * inv));
                }
        };

        // MFMAs of one phase of a strip.  Lane-derived LDS addresses restart from an opaque copy of the lane id in
        // every call: W and the tables do not change between strips, and derived from loop invariants their reads
        // would be hoisted out of the strip loop into hundreds of registers.
        auto mma = [&](const v8i (&x)[KS], v16f (&acc)[NB]) __attribute__((always_inline)) {
            int lane_o = lane;
            asm volatile("; per-strip lane id" : "+v"(lane_o));
            const int l32 = lane_o & 31, hk = lane_o >> 5;
            // W fragment addresses: MFMA row rho of a 32-row block is fed W row wperm(rho) (see the file comment);
            // 32 nb rows further down for column block nb (which does not change the swizzle key: SWIN <= 16)
            const int wperm = 16 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3);
            const int wkey = wperm & KEYMASK;
            // W fragments are read PF MFMAs ahead of their use (an LDS round trip is several MFMAs long)
            const uint8_t* wbase = smem + C::OFF_W + wperm * KB;
            constexpr int NF = NB * KS, PF = 4;
            v8i wf[PF];
            auto read_w = [&](int f) __attribute__((always_inline)) {           // f = j * NB + nb
                const int j = f / NB, nb = f % NB;
                const v4i lo = *reinterpret_cast<const v4i*>(wbase + nb * 32 * KB + (((4 * j + 2 * hk) ^ wkey) << 4));
                const v4i hi = *reinterpret_cast<const v4i*>(wbase + nb * 32 * KB + (((4 * j + 2 * hk + 1) ^ wkey) << 4));
                wf[f % PF] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            };
#pragma unroll
            for (int f = 0; f < PF - 1 && f < NF; ++f) read_w(f);
#pragma unroll
            for (int f = 0; f < NF; ++f) {
                __builtin_amdgcn_sched_barrier(0);
                if (f + PF - 1 < NF) read_w(f + PF - 1);
                acc[f % NB] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wf[f % PF], x[f / NB], acc[f % NB], 0, 0, 0, 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        };

        // scales, row statistics, normalization and store of one strip, from registers
        // (after_block(nb) runs when column block nb has been stored and its 16 accumulators are dead)
        auto epilogue = [&](int s, const float sxm, v16f (&acc)[NB], auto after_block) __attribute__((always_inline)) {
            int lane_o = lane;
            asm volatile("; per-strip lane id" : "+v"(lane_o));
            const int l32 = lane_o & 31, hk = lane_o >> 5;
            const int m = (s - s_base) * 32 + l32;

            // ---- scales: Y = acc * sx[m] * sw[n]
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const v4f* sw4 = reinterpret_cast<const v4f*>(smem + C::OFF_SW + (nb * 32 + hk * 16) * 4);
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const v4f sc = sw4[a];
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[nb][4 * a + e] *= sc[e] * sxm;
                }
            }
            if (p.y && m < p.M) {
                float* yrow = p.y + static_cast<int64_t>(g) * p.strideO + static_cast<int64_t>(m) * p.N;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    if (nb * 32 + hk * 16 < p.N) {
#pragma unroll
                        for (int a = 0; a < 4; ++a)
                            *reinterpret_cast<v4f*>(yrow + nb * 32 + hk * 16 + 4 * a) =
                                v4f{acc[nb][4 * a], acc[nb][4 * a + 1], acc[nb][4 * a + 2], acc[nb][4 * a + 3]};
                    }
            }

            // ---- row statistics: this lane's columns, then the lane that holds the row's other columns
            float mean = 0.f, rstd = 1.f;
            if (p.norm != LOKA_NORM_NONE) {
                float m2 = 0.f;
                if (ln) {
                    float n_ = cnt_lane, sum = 0.f;
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        if (nb * 32 + hk * 16 < p.N) {
#pragma unroll
                            for (int i = 0; i < 16; ++i) sum += acc[nb][i];
                        }
                    mean = n_ > 0.f ? sum * __builtin_amdgcn_rcpf(n_) : 0.f;
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        if (nb * 32 + hk * 16 < p.N) {
#pragma unroll
                            for (int i = 0; i < 16; ++i) { const float d = acc[nb][i] - mean; m2 = __builtin_fmaf(d, d, m2); }
                        }
                    // symmetric Chan merge: identical bits on both lanes
                    const float nb_ = wave_shfl_xor(n_, 32), mb = wave_shfl_xor(mean, 32), m2b = wave_shfl_xor(m2, 32);
                    const float nn = n_ + nb_;
                    if (nn > 0.f) {
                        const float d = mb - mean;
                        const float rn = __builtin_amdgcn_rcpf(nn);
                        const float newmean = (n_ * mean + nb_ * mb) * rn;
                        m2 = m2 + m2b + d * d * (n_ * nb_ * rn);
                        mean = newmean;
                    }
                } else {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        if (nb * 32 + hk * 16 < p.N) {
#pragma unroll
                            for (int i = 0; i < 16; ++i) m2 = __builtin_fmaf(acc[nb][i], acc[nb][i], m2);
                        }
                    m2 += wave_shfl_xor(m2, 32);
                }
                rstd = __builtin_amdgcn_rsqf(m2 * inv_n + p.eps);
            }
            const float nmr = -mean * rstd;

            // ---- normalize, affine, bf16.  A lane holds 16 consecutive columns (32 bytes) of ONE row per column
            // block; stored from there an instruction writes 16-byte pieces 32 bytes apart in 32 rows.  Each wave
            // instead passes the 32 x 64-byte block through 2 KB of its own LDS (16-byte chunk c of row r at
            // position c ^ (r / 4 % 4): conflict-free both ways) and stores it with 4 lanes per row: 16 full 64-byte
            // runs per instruction.  LDS executes one wave's instructions in order: no barrier, one buffer.
            uint8_t* const tbuf = smem + C::OFF_T + wave * 2048;
            const int t_wr = l32 * 64, t_key = (l32 >> 2) & 3;
            const int t_row = lane_o >> 2, t_c = lane_o & 3;                   // store side: row (+ 16 j), chunk
            uint16_t* const obase = p.out + static_cast<int64_t>(g) * p.strideO + static_cast<int64_t>((s - s_base) * 32) * p.N;
            // (without gamma and beta the affine step is x * 1 + 0: skipped, same bits, no table reads)
            auto normalize_store = [&](auto affine_tag) __attribute__((always_inline)) {
                constexpr bool AFFINE = decltype(affine_tag)::value;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int col = nb * 32 + hk * 16;
                    const v4f* g4 = reinterpret_cast<const v4f*>(smem + C::OFF_GM + col * 4);
                    const v4f* b4 = reinterpret_cast<const v4f*>(smem + C::OFF_BT + col * 4);
#pragma unroll
                    for (int half = 0; half < 2; ++half) {
                        float o[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) o[e] = __builtin_fmaf(acc[nb][8 * half + e], rstd, nmr);
                        if (AFFINE) {
                            const v4f gq0 = g4[2 * half], gq1 = g4[2 * half + 1], bq0 = b4[2 * half], bq1 = b4[2 * half + 1];
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                o[e] = __builtin_fmaf(o[e], gq0[e], bq0[e]);
                                o[4 + e] = __builtin_fmaf(o[4 + e], gq1[e], bq1[e]);
                            }
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
                        const int ccol = nb * 32 + t_c * 8;
                        if ((s - s_base) * 32 + r < p.M && ccol < p.N)
                            *reinterpret_cast<u32x4*>(obase + static_cast<int64_t>(r) * p.N + ccol) = pk;
                    }
                    after_block(nb);
                }
            };
            // FP8 output for the next layer (Section 3.2: quantization fused before the output is written): the
            // bf16 values above, quantized per row exactly as the quantize entry point would quantize the stored bf16
            // tensor.  The whole row lives in this lane and lane ^ 32, so the row amax needs one exchange; the values
            // are then computed a second time (keeping 128 packed values would not fit beside the accumulators),
            // cast, and leave through the same staging buffer, two column blocks (64 codes per row) at a time.
            auto normalize_store_fp8 = [&](auto affine_tag) __attribute__((always_inline)) {
                constexpr bool AFFINE = decltype(affine_tag)::value;
                auto packed8 = [&](int nb, int half) __attribute__((always_inline)) {
                    const int col = nb * 32 + hk * 16;
                    float o[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] = __builtin_fmaf(acc[nb][8 * half + e], rstd, nmr);
                    if (AFFINE) {
                        const v4f* g4 = reinterpret_cast<const v4f*>(smem + C::OFF_GM + col * 4);
                        const v4f* b4 = reinterpret_cast<const v4f*>(smem + C::OFF_BT + col * 4);
                        const v4f gq0 = g4[2 * half], gq1 = g4[2 * half + 1], bq0 = b4[2 * half], bq1 = b4[2 * half + 1];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            o[e] = __builtin_fmaf(o[e], gq0[e], bq0[e]);
                            o[4 + e] = __builtin_fmaf(o[4 + e], gq1[e], bq1[e]);
                        }
                    }
                    u32x4 pk;
                    pk.x = pack_bf16x2(o[0], o[1]); pk.y = pack_bf16x2(o[2], o[3]);
                    pk.z = pack_bf16x2(o[4], o[5]); pk.w = pack_bf16x2(o[6], o[7]);
                    return pk;
                };
                unsigned am = 0u;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    if (nb * 32 + hk * 16 < p.N) {
#pragma unroll
                        for (int half = 0; half < 2; ++half) {
                            const u32x4 pk = packed8(nb, half);
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const unsigned lo = pk[e] & 0x7FFFu, hi = (pk[e] >> 16) & 0x7FFFu;
                                am = am > lo ? am : lo;
                                am = am > hi ? am : hi;
                            }
                        }
                    }
                const unsigned other = static_cast<unsigned>(__shfl_xor(static_cast<int>(am), 32, 64));
                am = am > other ? am : other;
                float scale, inv;
                group_scale(__uint_as_float(am << 16), scale, inv);
                if (hk == 0 && m < p.M) p.outs[static_cast<int64_t>(g) * p.M + m] = scale;
                uint8_t* const qbase = p.outq + static_cast<int64_t>(g) * p.strideO + static_cast<int64_t>((s - s_base) * 32) * p.N;
#pragma unroll
                for (int nbp = 0; nbp < NB / 2; ++nbp) {
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        const int nb = 2 * nbp + q;
                        const u32x4 p0 = packed8(nb, 0), p1 = packed8(nb, 1);
                        u32x4 ck;
                        ck.x = e4m3x4(bf16_lo(p0.x) * inv, bf16_hi(p0.x) * inv, bf16_lo(p0.y) * inv, bf16_hi(p0.y) * inv);
                        ck.y = e4m3x4(bf16_lo(p0.z) * inv, bf16_hi(p0.z) * inv, bf16_lo(p0.w) * inv, bf16_hi(p0.w) * inv);
                        ck.z = e4m3x4(bf16_lo(p1.x) * inv, bf16_hi(p1.x) * inv, bf16_lo(p1.y) * inv, bf16_hi(p1.y) * inv);
                        ck.w = e4m3x4(bf16_lo(p1.z) * inv, bf16_hi(p1.z) * inv, bf16_lo(p1.w) * inv, bf16_hi(p1.w) * inv);
                        *reinterpret_cast<u32x4*>(tbuf + t_wr + (((2 * q + hk) ^ t_key) << 4)) = ck;
                    }
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const int r = 16 * j + t_row;
                        const u32x4 ck = *reinterpret_cast<const u32x4*>(tbuf + r * 64 + ((t_c ^ ((r >> 2) & 3)) << 4));
                        const int ccol = nbp * 64 + t_c * 16;
                        if ((s - s_base) * 32 + r < p.M && ccol < p.N)
                            *reinterpret_cast<u32x4*>(qbase + static_cast<int64_t>(r) * p.N + ccol) = ck;
                    }
                    after_block(2 * nbp);
                    after_block(2 * nbp + 1);
                }
            };
            // (an instantiation of its own: in one kernel with the bf16 form the larger shapes spill more)
            if (FP8OUT) {
                if (affine) normalize_store_fp8(std::true_type{}); else normalize_store_fp8(std::false_type{});
            } else {
                if (affine) normalize_store(std::true_type{}); else normalize_store(std::false_type{});
            }
        };

        // ---- this wave's strips of the segment
        v8i x[KS];
        float sxm = 0.f;
        if (NPH == 1 && BF16IN) {
            // as below, with the raw strip in a register set of its own: requested right after the previous strip's
            // values have been cast, in flight through that strip's MFMAs and epilogue
            // With 8 waves and the larger shapes the raw strip and the accumulators do not fit 256 registers side by
            // side: the next strip is then requested piece by piece from inside the epilogue, each piece into the
            // registers of a column block that has just been stored (LATE); the wave waits for it afterwards, and the
            // other seven cover.
            constexpr bool LATE = NWV == 8 && !(NB == 4 && KS <= 4);
            u32x4 raw[KS][4];
            int s = t + wave;
            if (s < seg_end) load_raw(s, raw);
            while (s < seg_end) {
                convert(s, raw, x, sxm);
                const bool more = s + NWV < seg_end;
                if (!LATE && more) load_raw(s + NWV, raw);
                __builtin_amdgcn_sched_barrier(0);
                v16f acc[NB];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[nb][i] = 0.f;
                mma(x, acc);
                epilogue(s, sxm, acc, [&](int nb) __attribute__((always_inline)) {
                    if (LATE && more) load_raw_part(s + NWV, raw, nb * (KS * 4) / NB, (nb + 1) * (KS * 4) / NB);
                });
                s += NWV;
            }
        } else if (NPH == 1) {
            // W is complete in LDS: the waves run on their own.  The next strip's operands are requested into the
            // same registers right after the last MFMA (x is dead then) and arrive during the epilogue.
            int s = t + wave;
            if (s < seg_end) load_x(s, 0, x, sxm);
            while (s < seg_end) {
                v16f acc[NB];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[nb][i] = 0.f;
                mma(x, acc);
                const float sx_cur = sxm;
                if (s + NWV < seg_end) load_x(s + NWV, 0, x, sxm);
                __builtin_amdgcn_sched_barrier(0);
                epilogue(s, sx_cur, acc, [](int) {});
                s += NWV;
            }
        } else {
            // W is longer than the LDS: rounds of 8 strips (one per wave), and per round NPH phases in which all
            // waves multiply the same K slab of W; the epilogues still run unsynchronized
            const int rounds = (seg_end - t + NWV - 1) / NWV;
            for (int r = 0; r < rounds; ++r) {
                const int s = t + NWV * r + wave;
                const bool active = s < seg_end;
                v16f acc[NB];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[nb][i] = 0.f;
                for (int ph = 0; ph < NPH; ++ph) {
                    __syncthreads();                            // every wave has read the previous slab (and the tables are written)
                    load_w(ph);
                    if (active) load_x(s, ph, x, sxm);
                    wait_vmcnt<0>();
                    __syncthreads();
                    if (active) mma(x, acc);
                }
                if (active) epilogue(s, sxm, acc, [](int) {});
            }
        }
        t = seg_end;
    }
}

// ---------------------------------------------------------------------------------------------- host side
namespace {

struct StripInst {
    int nb, ks, nph;
    const void* fn;
    const void* fn_fused;      // bf16 X, quantization fused (single-phase instances only)
    const void* fn_q;          // e4m3 output
    size_t lds;
    void (*launch)(const GemmParams&, int, dim3, hipStream_t);
};

// waves of a fused-quantization instance: 8 where accumulators, the raw strip and the operands fit 256 registers
// (N <= 128 with K <= 256; N = 256 with K = 128 and the piecewise request), else 4 with up to 512 each (measured:
// the 8-wave forms that spill are slower than the 4-wave ones, 94 against 71-81 us at 64 x (4096 x 256 x 256))
constexpr int fused_waves(int nb, int ks) { return ((nb == 4 && ks <= 4) || (nb == 8 && ks == 2)) ? 8 : 4; }

template <int NB, int KS, int NPH>
void launch_strip(const GemmParams& p, int spp, dim3 grid, hipStream_t s) {
    if (p.xb) {
        if constexpr (NPH == 1 && KS <= 8)                      // (K = 1024: the raw strip alone would be 256 registers)
            gemm_strip_kernel<NB, KS, NPH, fused_waves(NB, KS), true, false><<<grid, fused_waves(NB, KS) * 64, StripCfg<NB, KS, NPH>::LDS, s>>>(p, spp);
    } else if (p.outq) {
        gemm_strip_kernel<NB, KS, NPH, 8, false, true><<<grid, 512, StripCfg<NB, KS, NPH>::LDS, s>>>(p, spp);
    } else {
        gemm_strip_kernel<NB, KS, NPH, 8, false, false><<<grid, 512, StripCfg<NB, KS, NPH>::LDS, s>>>(p, spp);
    }
}

template <int NB, int KS, int NPH>
const void* strip_fused_fn() {
    if constexpr (NPH == 1 && KS <= 8) return reinterpret_cast<const void*>(&gemm_strip_kernel<NB, KS, NPH, fused_waves(NB, KS), true, false>);
    else return nullptr;
}

#define LOKA_STRIP(NB, KS, NPH)                                                                                     \
    {NB, KS, NPH, reinterpret_cast<const void*>(&gemm_strip_kernel<NB, KS, NPH, 8, false, false>), strip_fused_fn<NB, KS, NPH>(), \
     reinterpret_cast<const void*>(&gemm_strip_kernel<NB, KS, NPH, 8, false, true>), StripCfg<NB, KS, NPH>::LDS,          \
     &launch_strip<NB, KS, NPH>}

// column blocks, K steps per phase, phases (K = 64 KS NPH; one phase when W fits the LDS)
const StripInst kStrip[] = {LOKA_STRIP(4, 2, 1), LOKA_STRIP(4, 4, 1), LOKA_STRIP(4, 8, 1), LOKA_STRIP(4, 16, 1),
                            LOKA_STRIP(8, 2, 1), LOKA_STRIP(8, 4, 1), LOKA_STRIP(8, 8, 1), LOKA_STRIP(8, 8, 2)};

const StripInst* strip_pick(int64_t N, int64_t K) {
    if (K % 64 || N > 256) return nullptr;
    const int ks = static_cast<int>(K / 64), nb = N <= 128 ? 4 : 8;
    for (const StripInst& w : kStrip)
        if (w.nb == nb && w.ks * w.nph == ks) return &w;
    return nullptr;
}

}  // namespace

bool strip_supports(int64_t M, int64_t N, int64_t K) {
    return strip_pick(N, K) != nullptr && M * K < (int64_t(1) << 31) && M < (int64_t(1) << 26);
}

// Workgroups to launch and the kernel's entry (for the dynamic-LDS attribute); 0 when unsupported.
bool strip_supports_fused(int64_t M, int64_t N, int64_t K) {
    const StripInst* w = strip_pick(N, K);
    return w != nullptr && w->fn_fused != nullptr && strip_supports(M, N, K) && M * K < (int64_t(1) << 30);
}

int strip_plan(int64_t M, int64_t N, int64_t K, int64_t batch, int cus, bool bf16_in, bool fp8_out, const void** fn,
               size_t* lds) {
    const StripInst* w = strip_pick(N, K);
    if (!w || (bf16_in && (!w->fn_fused || fp8_out))) return 0;
    *fn = bf16_in ? w->fn_fused : fp8_out ? w->fn_q : w->fn;
    *lds = w->lds;
    const int64_t strips = batch * ((M + 31) / 32);
    const int waves = bf16_in ? fused_waves(w->nb, w->ks) : 8;
    const int64_t wgs = (strips + waves - 1) / waves;       // at least one strip per wave
    return static_cast<int>(wgs < cus ? wgs : cus);
}

void strip_launch(const GemmParams& p, dim3 grid, hipStream_t s) {
    const StripInst* w = strip_pick(p.N, p.KB);
    w->launch(p, (p.M + 31) / 32, grid, s);
}

}  // namespace loka
