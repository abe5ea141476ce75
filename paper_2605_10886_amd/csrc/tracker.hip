// Online distribution tracker of the probe (Section 3.1, "Online Distribution Learning": the batched
// Welford tracker for activations, after Chan et al.).  One batch X [B, K] (bf16) is merged into the running
// summary (n, mu [K], Sigma [K, K] = unnormalized scatter, fp32):
//   mu_b = column means,  S_b = (X - 1 mu_b^T)^T (X - 1 mu_b^T),  n' = n + B,  delta = mu_b - mu,
//   mu' = mu + (B / n') delta,   Sigma' = Sigma + S_b + (n B / n') delta delta^T.
//
// How it runs here.  S_b is computed as X^T X - B mu_b mu_b^T: the raw second moment is a dense
// contraction over the batch rows and goes to the BF16 matrix cores (products of two bf16 values are exact
// in fp32; accumulation is fp32), the column sums are accumulated in fp64 on the vector ALUs, and the
// subtraction, the delta delta^T term and the merge with the stored state are done in fp64 and rounded once.
//
//   tracker_scatter_kernel   one workgroup per (tile pair ti <= tj of 256 x 256 outputs, one of S row ranges of
//                            the batch): raw partial scatter -> workspace (fp32); workgroups on diagonal
//                            tiles also write fp64 column sums of their 256 columns
//   tracker_mean_kernel      folds the column sums of the S ranges in a fixed order: mu_b, delta (fp64,
//                            workspace), mu' in place
//   tracker_merge_kernel     folds the partial scatters in a fixed order, forms S_b and the rank-1 term and
//                            updates Sigma (both triangles; the mirror image goes through an LDS transpose)
//
// The contraction runs over the rows of a row-major matrix, i.e. over the strided dimension of both MFMA
// operands: an MFMA lane needs 8 consecutive batch rows of ONE column.  Each 8 x 8 block of X is transposed
// once, in registers, on its way from global memory to LDS (byte permutes), so that an operand fragment is a
// single 16-byte LDS read.  The MFMA's k order is irrelevant here because both operands come from the same
// rows in the same order.
#include "gemm_common.h"

namespace loka {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int TRK_T = 256;                      // output tile (columns i x columns j) per workgroup
constexpr int TRK_MS = 64;                      // batch rows per pipeline stage (four MFMA k steps of 16)
constexpr int TRK_TILEB = TRK_MS * TRK_T * 2;   // one operand tile of a stage (32 KB)
constexpr int TRK_STAGEB = 2 * TRK_TILEB;       // i tile, then j tile
constexpr size_t TRK_LDS = 2 * TRK_STAGEB + 2 * TRK_T * sizeof(double);
constexpr int TRK_PLAN_SLOTS = 256;             // cost model only: workgroups assumed in flight per round (the CU count of an
                                                // MI355X).  It steers the number of row splits (and with it the workspace
                                                // size, which must not depend on the device); results do not depend on it

// Work decomposition: workgroup = (tile pair ti <= tj, one of S equal row ranges of the batch).  All
// workgroups in flight walk their rows at the same pace, so the workgroups of an XCD that share a column
// tile find it in that XCD's L2.  S trades the rounding of pairs * S to whole rounds of 256 workgroups
// against the fp32 partial tile every workgroup leaves in the workspace (256 KB written and read back).
struct TrackerPlan {
    int T, pairs, splits;
    int64_t rows_per_split;
    size_t off_colsum, off_mub, off_delta, bytes;
};

TrackerPlan tracker_plan(int64_t B, int64_t K) {
    TrackerPlan pl{};
    pl.T = static_cast<int>((K + TRK_T - 1) / TRK_T);
    pl.pairs = pl.T * (pl.T + 1) / 2;
    const int64_t steps = (B + TRK_MS - 1) / TRK_MS;
    int64_t max_s = steps / 2 > 0 ? steps / 2 : 1;                    // at least 2 stages per workgroup
    if (max_s > 256) max_s = 256;
    // estimated time in units of one stage (about 1.2 us): rounds * (stages per workgroup + start-up) for the
    // scatter, and 0.1 per partial tile (256 KB written, then read back by the merge, at HBM speed)
    int64_t best_s = 1;
    double best = 1e300;
    for (int64_t sp = 1; sp <= max_s; ++sp) {
        const int64_t rounds = (static_cast<int64_t>(pl.pairs) * sp + TRK_PLAN_SLOTS - 1) / TRK_PLAN_SLOTS;
        const double cost = static_cast<double>(rounds) * ((steps + sp - 1) / sp + 3) + 0.1 * pl.pairs * static_cast<double>(sp);
        if (cost < best) { best = cost; best_s = sp; }
    }
    int64_t rows = (B + best_s - 1) / best_s;
    rows = (rows + TRK_MS - 1) / TRK_MS * TRK_MS;
    pl.rows_per_split = rows;
    pl.splits = static_cast<int>((B + rows - 1) / rows);
    const size_t slots = static_cast<size_t>(pl.splits) * pl.pairs;
    const size_t kp = static_cast<size_t>(pl.T) * TRK_T;
    pl.off_colsum = slots * TRK_T * TRK_T * sizeof(float);
    pl.off_mub = pl.off_colsum + slots * TRK_T * sizeof(double);
    pl.off_delta = pl.off_mub + kp * sizeof(double);
    pl.bytes = pl.off_delta + kp * sizeof(double);
    return pl;
}

struct TrackerParams {
    const uint16_t* x;
    int64_t B, ld, rows_per_split;
    int K, T, pairs, splits;
    float* partial;      // [splits][pairs][256][256]
    double* colsum;      // [splits][pairs][256] (written for diagonal pairs only)
};

__device__ __forceinline__ void pair_to_tiles(int pair, int T, int& ti, int& tj) {
    int i = 0, rem = pair;
    while (rem >= T - i) { rem -= T - i; ++i; }
    ti = i; tj = i + rem;
}
__host__ __device__ __forceinline__ int diag_pair(int t, int T) { return t * T - t * (t - 1) / 2; }

// 8 waves: wave (wi, wj) of a 2 x 4 arrangement owns 4 x 2 MFMA blocks of 32 x 32 (v_mfma_f32_32x32x16_bf16).
//
// Staging.  A stage is 64 batch rows x 256 columns per operand.  Thread (c = chunk of 8 columns, g = group
// of 8 rows) fetches its 8 x 8 block (8 loads of 16 bytes, 512-byte runs per row across 32 lanes), transposes
// it in registers (32 byte permutes) and writes one 16-byte word per column: the 8 contraction values an
// MFMA lane needs, so an operand fragment is ONE ds_read_b128.  LDS layout of a tile: [row group g][position
// pos][16 bytes] with column 8 c + e at position 32 e + c: the 32 lanes that write column e of their chunks
// write 512 consecutive bytes, and MFMA block t (positions 32 t .. 32 t + 31) is the set of columns 8 m + t,
// m = 0..31 = the block's MFMA row (or column) index.  Which tile column lands on which MFMA row is free as
// long as the epilogue knows: wave (wi, wj) owns blocks 4 wi .. 4 wi + 3 on the i side, 2 wj, 2 wj + 1 on the j side.
// Waves 0..3 stage the i tile, waves 4..7 the j tile (nothing on a diagonal pair, where both operands are
// the i tile).  The loads of stage s + 1 are in flight while stage s is multiplied (registers), two LDS
// buffers, one barrier per stage.
__global__ __launch_bounds__(512) void tracker_scatter_kernel(const TrackerParams p) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    double* red = reinterpret_cast<double*>(smem + 2 * TRK_STAGEB);           // [2][256]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wi = wave >> 2, wj = wave & 3;
    const int ldB = static_cast<int>(p.ld) * 2;

    // consecutive logical ids sit on one XCD (the dispatcher deals workgroups round-robin over the 8 XCDs)
    const int G = gridDim.x;
    const int id = (G % 8 == 0) ? (blockIdx.x % 8) * (G / 8) + blockIdx.x / 8 : blockIdx.x;
    const int split = id / p.pairs, pair = id - split * p.pairs;
    const int64_t row_begin = static_cast<int64_t>(split) * p.rows_per_split;
    const int64_t row_end = row_begin + p.rows_per_split < p.B ? row_begin + p.rows_per_split : p.B;
    const int nst = static_cast<int>((row_end - row_begin + TRK_MS - 1) / TRK_MS);
    int ti, tj;
    pair_to_tiles(pair, p.T, ti, tj);
    const bool diag = ti == tj;

    // staging role of this thread
    const bool stager = wave < 4 || !diag;
    const int my_tile = wave < 4 ? ti : tj;
    const int sc = tid & 31, sg = (tid & 255) >> 5;                         // column chunk, row group
    // everything that decides whether a load is in range sits in the per-lane offset: rows past the end of
    // the batch fall behind the descriptor's byte count, columns past K get an offset beyond any descriptor
    const unsigned st_voff = (my_tile * TRK_T + sc * 8 < p.K) ? static_cast<unsigned>(sg * 8 * ldB + sc * 16) : 0x80000000u;
    const int st_lds = (wave < 4 ? 0 : TRK_TILEB) + sg * 4096 + sc * 16;    // + 512 e per column of the chunk
    u32x4 in[8];
    auto fetch = [&](int st) __attribute__((always_inline)) {
        if (!stager) return;
        const int64_t r0 = row_begin + static_cast<int64_t>(st) * TRK_MS;
        int64_t rows_valid = row_end - r0;
        rows_valid = rows_valid > TRK_MS ? TRK_MS : rows_valid;
        const int rec = static_cast<int>(rows_valid) * ldB - my_tile * TRK_T * 2;
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t*>(p.x + r0 * p.ld + my_tile * TRK_T), 0, rec, 0x00020000);
#pragma unroll
        for (int r = 0; r < 8; ++r)
            in[r] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, st_voff + static_cast<unsigned>(r * ldB), 0, 0));
    };
    auto stage = [&](int buf) __attribute__((always_inline)) {
        if (!stager) return;
        uint8_t* dst = smem + buf * TRK_STAGEB + st_lds;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            u32x4 o;
            const unsigned sel = (e & 1) ? 0x07060302u : 0x05040100u;
            o.x = __builtin_amdgcn_perm(in[1][e >> 1], in[0][e >> 1], sel);
            o.y = __builtin_amdgcn_perm(in[3][e >> 1], in[2][e >> 1], sel);
            o.z = __builtin_amdgcn_perm(in[5][e >> 1], in[4][e >> 1], sel);
            o.w = __builtin_amdgcn_perm(in[7][e >> 1], in[6][e >> 1], sel);
            *reinterpret_cast<u32x4*>(dst + e * 512) = o;
        }
    };

    // fragment reads: lane (m = lane % 32, h = lane / 32) takes position 32 t + m of row group 2 kk + h
    const int fr_off = (lane >> 5) * 4096 + (lane & 31) * 16;
    const int a_off = fr_off + wi * 4 * 512, b_off = fr_off + wj * 2 * 512;
    auto read_frags = [&](const uint8_t* At, const uint8_t* Bt, int kk, v8bf (&fa)[4], v8bf (&fb)[2]) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < 4; ++t) fa[t] = __builtin_bit_cast(v8bf, *reinterpret_cast<const u32x4*>(At + a_off + t * 512 + kk * 8192));
#pragma unroll
        for (int e = 0; e < 2; ++e) fb[e] = __builtin_bit_cast(v8bf, *reinterpret_cast<const u32x4*>(Bt + b_off + e * 512 + kk * 8192));
    };
    v16f acc[4][2];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][e][r] = 0.f;
    auto mma = [&](const v8bf (&fa)[4], const v8bf (&fb)[2]) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int e = 0; e < 2; ++e)
                acc[t][e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[t], fb[e], acc[t][e], 0, 0, 0);
    };
    // issue order of one k step: an MFMA, then one LDS read of the next step's fragments, six times over
    auto interleave = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 6; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
    };
    // column sums (diagonal pairs): thread = (position tid % 256, row groups 4 (tid / 256) .. + 3), fp64
    double cs = 0.0;
    const int cs_off = (tid >> 8) * 4 * 4096 + (tid & 255) * 16;

    fetch(0);
    stage(0);
    __syncthreads();
    for (int s = 0; s < nst; ++s) {
        const uint8_t* At = smem + (s & 1) * TRK_STAGEB;
        const uint8_t* Bt = diag ? At : At + TRK_TILEB;
        // the two waves of a SIMD (w, w + 4) request their blocks of the next stage at different times: a wave
        // sits in the load issue until the memory pipeline has taken its requests, and should not do so together
        // with the wave that shares its matrix pipe.  (Measured: both groups at the start of the stage 750 us
        // at B = 32768, K = 4096; staggered 690 us; the eight loads spread over the stage, two per k step, with
        // a second register set so that they have a whole stage to land: 955 us.)
        if (s + 1 < nst && wave < 4) fetch(s + 1);
        v8bf fa0[4], fb0[2], fa1[4], fb1[2];
        read_frags(At, Bt, 0, fa0, fb0);
        read_frags(At, Bt, 1, fa1, fb1);
        mma(fa0, fb0);
        interleave();
        if (s + 1 < nst && wave >= 4) fetch(s + 1);
        read_frags(At, Bt, 2, fa0, fb0);
        mma(fa1, fb1);
        interleave();
        read_frags(At, Bt, 3, fa1, fb1);
        mma(fa0, fb0);
        interleave();
        mma(fa1, fb1);
        if (diag) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const u32x4 v = *reinterpret_cast<const u32x4*>(At + cs_off + g * 4096);
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    cs += static_cast<double>(bf16_lo(v[w]));
                    cs += static_cast<double>(bf16_hi(v[w]));
                }
            }
        }
        if (s + 1 < nst) stage((s + 1) & 1);
        __syncthreads();
    }

    // raw partial scatter: element r of a lane is MFMA row R = 8 (r / 4) + 4 h + r % 4, MFMA column C = lane % 32 of its
    // block; block (ta, tb) row R is tile row 8 R + 4 wi + ta, column C is tile column 8 C + 2 wj + tb: a lane holds
    // pairs of columns 32 bytes apart.  Stored straight from registers every instruction would scatter 8-byte pieces
    // over 64 cache lines (measured: 70 us of the 780 us at B = 32768, K = 4096); the tile goes through the stage
    // buffers instead, 128 rows at a time (R < 16, then R >= 16 = elements r < 8, then r >= 8), and leaves as whole
    // 1 KB rows.  LDS row: the four waves' columns side by side, position 64 wj + ((2 C + tb) ^ (wj >= 2 ? 32 : 0)), so
    // that the writes of 32 lanes are 256 consecutive bytes and the two 8-byte reads of the 32 lanes that share a
    // row half fall on different banks.
    // (offsets recomputed from an opaque copy of the lane id: derived from a loop invariant, the compiler
    // would keep the addresses alive across the main loop, in registers the accumulators need)
    int lane_o = lane, tid_o = tid;
    asm volatile("" : "+v"(lane_o), "+v"(tid_o));
    float* const stg = reinterpret_cast<float*>(smem);
    const int st_w = (8 * 4 * (lane_o >> 5) + 4 * wi) * 256 + wj * 64 + ((2 * (lane_o & 31)) ^ ((wj >> 1) * 32));
    const int q4 = tid_o & 63, cq = q4 >> 1, uq = q4 & 1;
    const int st_r = (tid_o >> 6) * 256 + (2 * uq) * 64 + ((2 * cq) ^ (uq * 32));
    float* const out = p.partial + static_cast<int64_t>(id) * (TRK_T * TRK_T) + (tid_o >> 6) * TRK_T + 4 * q4;
#pragma unroll
    for (int ps = 0; ps < 2; ++ps) {
        if (ps) __syncthreads();                                        // the first half has been read out of LDS
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int r8 = 0; r8 < 8; ++r8) {
                const int r = 8 * ps + r8;
                // local row 8 R' + 4 wi + t with R' = 8 (r8 / 4) + 4 h + r8 % 4
                *reinterpret_cast<f32x2_t*>(stg + st_w + (64 * (r8 >> 2) + 8 * (r8 & 3) + t) * 256) = f32x2_t{acc[t][0][r], acc[t][1][r]};
            }
        __syncthreads();
#pragma unroll 4
        for (int it = 0; it < 16; ++it) {
            const f32x2_t lo = *reinterpret_cast<const f32x2_t*>(stg + st_r + it * 8 * 256);
            const f32x2_t hi = *reinterpret_cast<const f32x2_t*>(stg + st_r + it * 8 * 256 + 64);
            *reinterpret_cast<v4f*>(out + (128 * ps + it * 8) * TRK_T) = v4f{lo[0], lo[1], hi[0], hi[1]};
        }
    }
    if (diag) {
        // position pos holds column 8 (pos % 32) + pos / 32
        const int pos = tid & 255, col = 8 * (pos & 31) + (pos >> 5);
        red[(tid >> 8) * TRK_T + col] = cs;
        __syncthreads();
        if (tid < TRK_T) p.colsum[static_cast<int64_t>(id) * TRK_T + tid] = red[tid] + red[TRK_T + tid];
    }
}

__global__ __launch_bounds__(256) void tracker_mean_kernel(const double* __restrict__ colsum, int T, int pairs, int splits,
                                                           int K, int64_t B, int64_t n_old, float* __restrict__ mu,
                                                           double* __restrict__ mub, double* __restrict__ delta) {
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= T * TRK_T) return;
    if (k >= K) { mub[k] = 0.0; delta[k] = 0.0; return; }
    const int t = k / TRK_T;
    const double* src = colsum + static_cast<int64_t>(diag_pair(t, T)) * TRK_T + (k - t * TRK_T);
    const int64_t stride = static_cast<int64_t>(pairs) * TRK_T;
    double s = 0.0;
#pragma unroll 8
    for (int sp = 0; sp < splits; ++sp) s += src[sp * stride];
    const double mb = s / static_cast<double>(B);
    const double m0 = static_cast<double>(mu[k]);
    const double d = mb - m0;
    const double n_new = static_cast<double>(n_old) + static_cast<double>(B);
    mub[k] = mb;
    delta[k] = d;
    mu[k] = static_cast<float>(m0 + static_cast<double>(B) / n_new * d);
}

// grid (pairs, 64): workgroup y handles the 32 x 32 block (y / 8, y % 8) of its pair's tile, one run of four
// columns per thread, and, for an off-diagonal pair, the mirrored block of the lower triangle (through a
// transposing LDS tile, so both triangles are written in full 128-byte runs).
__global__ __launch_bounds__(256) void tracker_merge_kernel(const float* __restrict__ partial, int T, int pairs, int splits,
                                                            int K, int64_t B, double coef, const double* __restrict__ mub,
                                                            const double* __restrict__ delta, float* __restrict__ sigma) {
    __shared__ double tr[32][33];
    const int tid = threadIdx.x, tq = tid & 7, ty = tid >> 3;            // 8 runs of four columns x 32 rows
    const int pair = blockIdx.x, bi = blockIdx.y >> 3, bj = blockIdx.y & 7;
    int ti, tj;
    pair_to_tiles(pair, T, ti, tj);
    const bool diag = ti == tj;
    const double Bd = static_cast<double>(B);
    const int64_t tile_elems = TRK_T * TRK_T, stride = static_cast<int64_t>(pairs) * tile_elems;
    const int il = bi * 32 + ty, jl = bj * 32 + 4 * tq;
    const int i = ti * TRK_T + il, j = tj * TRK_T + jl;                  // K % 8 == 0: a run is inside or outside
    double c[4] = {0.0, 0.0, 0.0, 0.0};
    if (i < K && j < K) {
        const float* src = partial + static_cast<int64_t>(pair) * tile_elems + il * TRK_T + jl;
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
#pragma unroll 8
        for (int sp = 0; sp < splits; ++sp) {
            const v4f v = *reinterpret_cast<const v4f*>(src + sp * stride);
            s0 += static_cast<double>(v[0]); s1 += static_cast<double>(v[1]);
            s2 += static_cast<double>(v[2]); s3 += static_cast<double>(v[3]);
        }
        const double sv[4] = {s0, s1, s2, s3};
        float* dst = sigma + static_cast<int64_t>(i) * K + j;
        const v4f old = *reinterpret_cast<const v4f*>(dst);
        v4f nw;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            // products of the two columns first: (i, j) and (j, i) then give identical bits
            const double sb = sv[e] - Bd * (mub[i] * mub[j + e]);
            c[e] = sb + coef * (delta[i] * delta[j + e]);
            nw[e] = static_cast<float>(static_cast<double>(old[e]) + c[e]);
        }
        *reinterpret_cast<v4f*>(dst) = nw;
    }
    if (!diag) {
#pragma unroll
        for (int e = 0; e < 4; ++e) tr[ty][4 * tq + e] = c[e];
        __syncthreads();
        // mirrored block: row jl2 of the lower triangle takes column jl2 of the block just computed
        const int jl2 = bj * 32 + ty, il2 = bi * 32 + 4 * tq;
        const int i2 = ti * TRK_T + il2, j2 = tj * TRK_T + jl2;
        if (i2 < K && j2 < K) {
            float* dst = sigma + static_cast<int64_t>(j2) * K + i2;
            const v4f old = *reinterpret_cast<const v4f*>(dst);
            v4f nw;
#pragma unroll
            for (int e = 0; e < 4; ++e) nw[e] = static_cast<float>(static_cast<double>(old[e]) + tr[4 * tq + e][ty]);
            *reinterpret_cast<v4f*>(dst) = nw;
        }
    }
}

size_t tracker_workspace_bytes(int64_t B, int64_t K) { return tracker_plan(B, K).bytes; }

loka_status tracker_update_launch(const void* x, int64_t B, int64_t K, int64_t ld, int64_t n_old, float* mu, float* sigma,
                                  void* workspace, hipStream_t s) {
    const TrackerPlan pl = tracker_plan(B, K);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    double* colsum = reinterpret_cast<double*>(ws + pl.off_colsum);
    double* mub = reinterpret_cast<double*>(ws + pl.off_mub);
    double* delta = reinterpret_cast<double*>(ws + pl.off_delta);
    TrackerParams p{};
    p.x = static_cast<const uint16_t*>(x); p.B = B; p.ld = ld; p.K = static_cast<int>(K);
    p.T = pl.T; p.pairs = pl.pairs; p.splits = pl.splits; p.rows_per_split = pl.rows_per_split;
    p.partial = reinterpret_cast<float*>(ws); p.colsum = colsum;
    // set on every call (a host-side table write): no process-wide state, and correct on whichever device is current
    LOKA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&tracker_scatter_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(TRK_LDS)));
    tracker_scatter_kernel<<<dim3(pl.pairs * pl.splits), 512, TRK_LDS, s>>>(p);
    const int KP = pl.T * TRK_T;
    tracker_mean_kernel<<<dim3((KP + 255) / 256), 256, 0, s>>>(colsum, pl.T, pl.pairs, pl.splits, static_cast<int>(K), B, n_old,
                                                               mu, mub, delta);
    const double n_new = static_cast<double>(n_old) + static_cast<double>(B);
    const double coef = static_cast<double>(n_old) * static_cast<double>(B) / n_new;
    tracker_merge_kernel<<<dim3(pl.pairs, 64), 256, 0, s>>>(p.partial, pl.T, pl.pairs, pl.splits, static_cast<int>(K), B, coef,
                                                            mub, delta, sigma);
    return hipGetLastError() == hipSuccess ? LOKA_OK : LOKA_ERR_HIP;
}

}  // namespace loka
