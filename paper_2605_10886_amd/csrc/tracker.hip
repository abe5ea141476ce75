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
// operands.  The staged rows stay row-major in LDS and the operand fragments (8 contraction values of one
// column per lane) come out of the transposing LDS read of gfx950 (ds_read_b64_tr_b16): within 16 lanes,
// source lane 4 e + q supplies the address of 4 consecutive columns (4 q .. 4 q + 3) of contraction row e,
// and lane i receives column i of rows e = 0..3.  Two such reads fill one operand of
// v_mfma_f32_32x32x16_bf16.  The MFMA's k order is irrelevant here because both operands come from the same
// rows in the same order.
#include "gemm_common.h"

namespace loka {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int TRK_T = 256;                      // output tile (columns i x columns j) per workgroup
constexpr int TRK_MS = 32;                      // batch rows per pipeline stage (two MFMA k steps of 16)
constexpr int TRK_NS = 4;                       // LDS ring: stages in flight
constexpr int TRK_ROWB = TRK_T * 2;             // bytes of one staged row
constexpr int TRK_TILEB = TRK_MS * TRK_ROWB;    // one operand tile of a stage (16 KB)
constexpr int TRK_STAGEB = 2 * TRK_TILEB;       // i tile, then j tile
constexpr size_t TRK_LDS = TRK_NS * TRK_STAGEB + 4 * TRK_T * sizeof(double);
constexpr int TRK_CUS = 256;                    // workgroups resident at once (one per CU)

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
    int64_t max_s = steps / 4 > 0 ? steps / 4 : 1;                    // at least 4 steps per workgroup
    if (max_s > 256) max_s = 256;
    // estimated time in units of one step (about 0.5 us): rounds * (steps per workgroup + start-up) for the
    // scatter, and 0.2 per partial tile (256 KB written, then read back by the merge, at HBM speed)
    int64_t best_s = 1;
    double best = 1e300;
    for (int64_t sp = 1; sp <= max_s; ++sp) {
        const int64_t rounds = (static_cast<int64_t>(pl.pairs) * sp + TRK_CUS - 1) / TRK_CUS;
        const double cost = static_cast<double>(rounds) * ((steps + sp - 1) / sp + 6) + 0.2 * pl.pairs * static_cast<double>(sp);
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

// 8 waves: wave (wi, wj) of a 2 x 4 arrangement owns tile rows [128 wi, +128) x tile columns [64 wj, +64)
// = 4 x 2 MFMA blocks of 32 x 32 (v_mfma_f32_32x32x16_bf16).
//
// LDS stage: rows of 512 bytes (256 columns); the 64-byte unit u of row r sits at unit u ^ (r & 3) of its
// 256-byte quarter, so the four consecutive rows a transposing read touches (64 bytes of each per half-wave)
// cover all 64 banks once.  A wave's load instruction brings two rows (64 lanes x 16 bytes written back to
// back); the swizzle is applied on the global side (which 16-byte chunk a lane fetches).
typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));

__device__ __forceinline__ v8bf tr_fragment(const uint8_t* lo, const uint8_t* hi) {
    const v4s a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)(lo));
    const v4s b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)(hi));
    const v8s f{a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
    return __builtin_bit_cast(v8bf, f);
}

__global__ __launch_bounds__(512) void tracker_scatter_kernel(const TrackerParams p) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    double* red = reinterpret_cast<double*>(smem + TRK_NS * TRK_STAGEB);      // [4][256]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wi = wave >> 2, wj = wave & 3;
    const int ldB = static_cast<int>(p.ld) * 2;

    // fragment read offsets inside a tile: lane (group g = lane / 16, j = lane % 16) addresses columns
    // 16 (g & 1) + 4 (j % 4) .. + 3 of row 8 (g >> 1) + j / 4 (+ 4 for the second read, + 16 for the second k step)
    const int fr_row = 8 * (lane >> 5) + ((lane & 15) >> 2);
    const int fr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);                 // within a 32-column block
    const int fr_key = (fr_row & 3) << 6;                                       // rows + 4, + 16 share it
    const int a_off = fr_row * TRK_ROWB + ((wi * 256 + fr_col * 2) ^ fr_key);   // + 64 t per 32-column block
    const int b_off = fr_row * TRK_ROWB + ((wj * 128 + fr_col * 2) ^ fr_key);
    // column-sum read: word tid % 128 (two columns) of rows 8 (tid / 128) + r
    const int cw = tid & 127, crg = tid >> 7;
    const int c_off = (8 * crg) * TRK_ROWB + cw * 4;
    // consecutive logical ids sit on one XCD (the dispatcher deals workgroups round-robin over the 8 XCDs)
    const int G = gridDim.x;
    const int id = (G % 8 == 0) ? (blockIdx.x % 8) * (G / 8) + blockIdx.x / 8 : blockIdx.x;
    {
        const int split = id / p.pairs, pair = id - split * p.pairs;
        const int64_t row_begin = static_cast<int64_t>(split) * p.rows_per_split;
        const int64_t row_end = row_begin + p.rows_per_split < p.B ? row_begin + p.rows_per_split : p.B;
        const int nsteps = static_cast<int>((row_end - row_begin + TRK_MS - 1) / TRK_MS);
        const int slot = id;
        int ti, tj;
        pair_to_tiles(pair, p.T, ti, tj);
        const bool diag = ti == tj;

        // loader geometry.  Load j of a wave covers row pair g = (wave + 8 j) % 16 of the i tile (j < 2) or
        // of the j tile; its rows are 2 g + lane / 32 with g & 1 = wave & 1 for every j.  Everything that
        // decides whether a lane is in range sits in the per-lane offset: rows past the end of the batch fall
        // behind the descriptor's byte count, columns past K get an offset beyond any descriptor.
        const int lr = lane >> 5, chunk = (lane & 31) ^ (((2 * (wave & 1) + lr) & 3) << 2);
        const int col_a = ti * TRK_T + chunk * 8, col_b = tj * TRK_T + chunk * 8;
        const unsigned voff_a = col_a < p.K ? static_cast<unsigned>(lr * ldB + chunk * 16) : 0x80000000u;
        const unsigned voff_b = col_b < p.K ? static_cast<unsigned>(lr * ldB + chunk * 16) : 0x80000000u;
        auto issue = [&](int step) __attribute__((always_inline)) {
            const int64_t r0 = row_begin + static_cast<int64_t>(step) * TRK_MS;
            int64_t rows_valid = row_end - r0;
            rows_valid = rows_valid < 0 ? 0 : rows_valid > TRK_MS ? TRK_MS : rows_valid;
            const int rec_a = rows_valid ? static_cast<int>(rows_valid) * ldB - ti * TRK_T * 2 : 0;
            const int rec_b = rows_valid && !diag ? static_cast<int>(rows_valid) * ldB - tj * TRK_T * 2 : 0;
            const uint16_t* rowp = p.x + (rows_valid ? r0 : 0) * p.ld;
            const __amdgpu_buffer_rsrc_t rs_a = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<uint16_t*>(rowp + ti * TRK_T), 0, rec_a, 0x00020000);
            const __amdgpu_buffer_rsrc_t rs_b = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<uint16_t*>(rowp + tj * TRK_T), 0, rec_b, 0x00020000);
            uint8_t* st = smem + (step & (TRK_NS - 1)) * TRK_STAGEB;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int g = (wave + 8 * j) & 15;                     // uniform
                const unsigned rowoff = static_cast<unsigned>(2 * g * ldB);
                if (j < 2)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_a, (__attribute__((address_space(3))) void*)(st + g * 1024),
                                                             16, voff_a + rowoff, 0, 0, 0);
                else
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        rs_b, (__attribute__((address_space(3))) void*)(st + TRK_TILEB + g * 1024), 16, voff_b + rowoff, 0, 0, 0);
            }
        };

        v16f acc[4][2];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[t][e][r] = 0.f;
        double cs0 = 0.0, cs1 = 0.0;

        // Software pipeline: the fragments of k step q + 1 are read from LDS while the MFMAs of k step q run
        // (a wave that reads all fragments and then issues all MFMAs leaves the matrix pipe idle during the
        // reads: the other wave of the SIMD is in the same phase).  One barrier per stage, in the middle of it.
        auto read_frags = [&](const uint8_t* At, const uint8_t* Bt, int kk, v8bf (&fa)[4], v8bf (&fb)[2])
                              __attribute__((always_inline)) {
#pragma unroll
            for (int t = 0; t < 4; ++t)
                fa[t] = tr_fragment(At + (a_off ^ (t << 6)) + kk * 16 * TRK_ROWB, At + (a_off ^ (t << 6)) + (kk * 16 + 4) * TRK_ROWB);
#pragma unroll
            for (int e = 0; e < 2; ++e)
                fb[e] = tr_fragment(Bt + (b_off ^ (e << 6)) + kk * 16 * TRK_ROWB, Bt + (b_off ^ (e << 6)) + (kk * 16 + 4) * TRK_ROWB);
        };
        auto mma = [&](const v8bf (&fa)[4], const v8bf (&fb)[2]) __attribute__((always_inline)) {
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int e = 0; e < 2; ++e)
                    acc[t][e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[t], fb[e], acc[t][e], 0, 0, 0);
        };
        // issue order of one k step: an MFMA, then two LDS reads of the next step's fragments, six times over
        auto interleave = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < 6; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        };

#pragma unroll
        for (int s = 0; s < TRK_NS - 1; ++s) issue(s);
        wait_vmcnt<(TRK_NS - 2) * 4>();              // this wave's share of stage 0 has landed (loads return in order)
        lds_barrier();
        issue(TRK_NS - 1);
        v8bf fa0[4], fb0[2], fa1[4], fb1[2];
        read_frags(smem, diag ? smem : smem + TRK_TILEB, 0, fa0, fb0);
        for (int s = 0; s < nsteps; ++s) {
            const uint8_t* At = smem + (s & (TRK_NS - 1)) * TRK_STAGEB;
            const uint8_t* Bt = diag ? At : At + TRK_TILEB;
            read_frags(At, Bt, 1, fa1, fb1);
            mma(fa0, fb0);
            interleave();
            if (diag) {
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    const uint32_t w = *reinterpret_cast<const uint32_t*>(At + ((c_off + r * TRK_ROWB) ^ ((r & 3) << 6)));
                    cs0 += static_cast<double>(bf16_lo(w));
                    cs1 += static_cast<double>(bf16_hi(w));
                }
            }
            wait_vmcnt<(TRK_NS - 2) * 4>();          // stage s + 1 has landed
            lds_barrier();                            // for everyone; and everyone has read all of stage s
            issue(s + TRK_NS);                        // into the buffer of stage s (past the end: empty descriptors)
            const uint8_t* An = smem + ((s + 1) & (TRK_NS - 1)) * TRK_STAGEB;
            read_frags(An, diag ? An : An + TRK_TILEB, 0, fa0, fb0);   // past the last stage: read, never used
            mma(fa1, fb1);
            interleave();
        }
        wait_vmcnt<0>();                              // the empty tail loads too, before the wave may end

        // raw partial scatter: element r of a lane is row 8 (r / 4) + 4 h + r % 4 of a 32 x 32 block, column p5;
        // block (t, e) holds tile rows 128 wi + 32 t + row and tile columns 64 wj + 32 e + p5
        // (offsets recomputed from an opaque copy of the lane id: derived from a loop invariant, the compiler
        // would keep the store addresses alive across the main loop, in registers the accumulators need)
        int lane_o = lane;
        asm volatile("" : "+v"(lane_o));
        float* out = p.partial + static_cast<int64_t>(slot) * (TRK_T * TRK_T) + (wi * 128 + 4 * (lane_o >> 5)) * TRK_T +
                     wj * 64 + (lane_o & 31);
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int r = 0; r < 16; ++r) out[(32 * t + 8 * (r >> 2) + (r & 3)) * TRK_T + 32 * e] = acc[t][e][r];
        if (diag) {
            red[crg * TRK_T + 2 * cw] = cs0;
            red[crg * TRK_T + 2 * cw + 1] = cs1;
            __syncthreads();
            if (tid < TRK_T) {
                const double sum = ((red[tid] + red[TRK_T + tid]) + red[2 * TRK_T + tid]) + red[3 * TRK_T + tid];
                p.colsum[static_cast<int64_t>(slot) * TRK_T + tid] = sum;
            }
        }
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
    static bool lds_set = false;                 // per process; the attribute belongs to the function
    if (!lds_set) {
        LOKA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&tracker_scatter_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(TRK_LDS)));
        lds_set = true;
    }
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
