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
//   tracker_scatter_kernel   grid (tile pairs ti <= tj of 128 x 128 outputs, splits over the batch rows):
//                            raw partial scatter of its rows for its tile -> workspace (fp32);
//                            diagonal tiles also write fp64 column sums of their 128 columns
//   tracker_mean_kernel      folds the column sums over the splits in a fixed order: mu_b, delta (fp64,
//                            workspace), mu' in place
//   tracker_merge_kernel     folds the partial scatters in a fixed order, forms S_b and the rank-1 term and
//                            updates Sigma (both triangles; the mirror image goes through an LDS transpose)
//
// The contraction runs over the rows of a row-major matrix, i.e. over the strided dimension of both MFMA
// operands.  The operand fragments (8 contraction values of one column per lane) are built in registers:
// a lane reads the 32-bit word holding columns (2p, 2p+1) from 8 consecutive rows and two byte-permutes
// per register pair split them into one fragment for column 2p and one for column 2p+1.  The MFMA's k
// order is irrelevant here because both operands come from the same rows in the same order.
#include "common.h"

namespace loka {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int TRK_T = 128;                      // output tile (columns i x columns j) per workgroup
constexpr int TRK_MS = 32;                      // batch rows per step (two MFMA k steps of 16)
constexpr int TRK_ROWB = TRK_T * 2 + 16;        // LDS bytes per staged row; the pad puts rows r and r + 8 32 banks apart
constexpr int TRK_TILEB = TRK_MS * TRK_ROWB;

struct TrackerPlan {
    int T, pairs, splits;
    int64_t rows_per_split;
    size_t off_colsum, off_mub, off_delta, bytes;
};

TrackerPlan tracker_plan(int64_t B, int64_t K) {
    TrackerPlan pl{};
    pl.T = static_cast<int>((K + TRK_T - 1) / TRK_T);
    pl.pairs = pl.T * (pl.T + 1) / 2;
    int64_t want = (1024 + pl.pairs - 1) / pl.pairs;          // about four workgroups per CU in flight
    const int64_t max_splits = (B + 255) / 256;               // at least 256 rows per split
    if (want > max_splits) want = max_splits;
    if (want > 256) want = 256;
    if (want < 1) want = 1;
    int64_t rows = (B + want - 1) / want;
    rows = (rows + TRK_MS - 1) / TRK_MS * TRK_MS;
    pl.rows_per_split = rows;
    pl.splits = static_cast<int>((B + rows - 1) / rows);
    const size_t partial = static_cast<size_t>(pl.splits) * pl.pairs * TRK_T * TRK_T * sizeof(float);
    const size_t kp = static_cast<size_t>(pl.T) * TRK_T;
    pl.off_colsum = partial;
    pl.off_mub = pl.off_colsum + static_cast<size_t>(pl.splits) * kp * sizeof(double);
    pl.off_delta = pl.off_mub + kp * sizeof(double);
    pl.bytes = pl.off_delta + kp * sizeof(double);
    return pl;
}

__device__ __forceinline__ void pair_to_tiles(int pair, int T, int& ti, int& tj) {
    int i = 0, rem = pair;
    while (rem >= T - i) { rem -= T - i; ++i; }
    ti = i; tj = i + rem;
}

__global__ __launch_bounds__(256) void tracker_scatter_kernel(const uint16_t* __restrict__ x, int64_t B, int K, int64_t ld,
                                                              int T, int pairs, int64_t rows_per_split,
                                                              float* __restrict__ partial, double* __restrict__ colsum) {
    __shared__ __attribute__((aligned(16))) uint8_t smem[2][2][TRK_TILEB];
    __shared__ double red[4][TRK_T];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int p = lane & 31, h = lane >> 5;
    const int wi = wave >> 1, wj = wave & 1;
    const int pair = blockIdx.x, split = blockIdx.y;
    int ti, tj;
    pair_to_tiles(pair, T, ti, tj);
    const bool diag = ti == tj;
    const int64_t row0 = static_cast<int64_t>(split) * rows_per_split;
    const int64_t row_end = row0 + rows_per_split < B ? row0 + rows_per_split : B;
    const int nsteps = static_cast<int>((row_end - row0 + TRK_MS - 1) / TRK_MS);

    // loader: 32 rows x 16 chunks of 16 bytes per operand tile, two chunks per thread
    const int ld_r = tid >> 4, ld_c = tid & 15;            // rows ld_r and ld_r + 16
    const int col_a = ti * TRK_T + ld_c * 8, col_b = tj * TRK_T + ld_c * 8;
    const bool ok_a = col_a < K, ok_b = col_b < K && !diag;
    u32x4 ra[2], rb[2];
    auto fetch = [&](int s) {
        for (int u = 0; u < 2; ++u) {
            const int64_t row = row0 + static_cast<int64_t>(s) * TRK_MS + ld_r + 16 * u;
            const bool rok = row < row_end;
            ra[u] = u32x4{0u, 0u, 0u, 0u};
            rb[u] = u32x4{0u, 0u, 0u, 0u};
            if (rok && ok_a) ra[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(x + row * ld + col_a));
            if (rok && ok_b) rb[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(x + row * ld + col_b));
        }
    };
    auto stage = [&](int buf) {
        for (int u = 0; u < 2; ++u) {
            const int off = (ld_r + 16 * u) * TRK_ROWB + ld_c * 16;
            *reinterpret_cast<u32x4*>(&smem[buf][0][off]) = ra[u];
            if (!diag) *reinterpret_cast<u32x4*>(&smem[buf][1][off]) = rb[u];
        }
    };

    v16f acc[2][2];
    for (int a = 0; a < 2; ++a)
        for (int b = 0; b < 2; ++b)
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
    double cs0 = 0.0, cs1 = 0.0;

    fetch(0);
    stage(0);
    __syncthreads();
    for (int s = 0; s < nsteps; ++s) {
        const int buf = s & 1;
        if (s + 1 < nsteps) fetch(s + 1);
        const uint8_t* At = &smem[buf][0][wi * 128 + p * 4];
        const uint8_t* Bt = &smem[buf][diag ? 0 : 1][wj * 128 + p * 4];
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            uint32_t a[8], b[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const int row = kk * 16 + h * 8 + r;
                a[r] = *reinterpret_cast<const uint32_t*>(At + row * TRK_ROWB);
                b[r] = *reinterpret_cast<const uint32_t*>(Bt + row * TRK_ROWB);
            }
            v4i ae, ao, be, bo;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                // low halves (column 2p) / high halves (column 2p + 1) of two consecutive rows
                ae[q] = static_cast<int>(__builtin_amdgcn_perm(a[2 * q + 1], a[2 * q], 0x05040100u));
                ao[q] = static_cast<int>(__builtin_amdgcn_perm(a[2 * q + 1], a[2 * q], 0x07060302u));
                be[q] = static_cast<int>(__builtin_amdgcn_perm(b[2 * q + 1], b[2 * q], 0x05040100u));
                bo[q] = static_cast<int>(__builtin_amdgcn_perm(b[2 * q + 1], b[2 * q], 0x07060302u));
            }
            const v8bf fae = __builtin_bit_cast(v8bf, ae), fao = __builtin_bit_cast(v8bf, ao);
            const v8bf fbe = __builtin_bit_cast(v8bf, be), fbo = __builtin_bit_cast(v8bf, bo);
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fae, fbe, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fae, fbo, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fao, fbe, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fao, fbo, acc[1][1], 0, 0, 0);
        }
        if (diag) {
            // column sums of the staged rows in fp64: word `lane` (two columns), rows 8 wave .. 8 wave + 7
            const uint8_t* Ct = &smem[buf][0][lane * 4];
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const uint32_t w = *reinterpret_cast<const uint32_t*>(Ct + (wave * 8 + r) * TRK_ROWB);
                cs0 += static_cast<double>(bf16_lo(w));
                cs1 += static_cast<double>(bf16_hi(w));
            }
        }
        if (s + 1 < nsteps) stage(buf ^ 1);
        __syncthreads();
    }

    // raw partial scatter of this split: element r of a lane is row 8 (r / 4) + 4 h + r % 4 of the 32 x 32
    // block, column p; block (ea, eb) holds tile rows 2 * row + ea and tile columns 2 * p + eb
    float* out = partial + (static_cast<int64_t>(split) * pairs + pair) * (TRK_T * TRK_T);
#pragma unroll
    for (int ea = 0; ea < 2; ++ea) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int il = wi * 64 + 2 * (8 * (r >> 2) + 4 * h + (r & 3)) + ea;
            const int jl = wj * 64 + 2 * p;
            f32x2_t v{acc[ea][0][r], acc[ea][1][r]};
            *reinterpret_cast<f32x2_t*>(out + il * TRK_T + jl) = v;
        }
    }
    if (diag) {
        red[wave][2 * lane] = cs0;
        red[wave][2 * lane + 1] = cs1;
        __syncthreads();
        if (tid < TRK_T) {
            const double s = ((red[0][tid] + red[1][tid]) + red[2][tid]) + red[3][tid];
            colsum[(static_cast<int64_t>(split) * T + ti) * TRK_T + tid] = s;
        }
    }
}

__global__ __launch_bounds__(256) void tracker_mean_kernel(const double* __restrict__ colsum, int splits, int KP, int K,
                                                           int64_t B, int64_t n_old, float* __restrict__ mu,
                                                           double* __restrict__ mub, double* __restrict__ delta) {
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= KP) return;
    double s = 0.0;
    for (int sp = 0; sp < splits; ++sp) s += colsum[static_cast<int64_t>(sp) * KP + k];
    if (k >= K) { mub[k] = 0.0; delta[k] = 0.0; return; }
    const double mb = s / static_cast<double>(B);
    const double m0 = static_cast<double>(mu[k]);
    const double d = mb - m0;
    const double n_new = static_cast<double>(n_old) + static_cast<double>(B);
    mub[k] = mb;
    delta[k] = d;
    mu[k] = static_cast<float>(m0 + static_cast<double>(B) / n_new * d);
}

__global__ __launch_bounds__(256) void tracker_merge_kernel(const float* __restrict__ partial, int splits, int pairs, int T,
                                                            int K, int64_t B, double coef, const double* __restrict__ mub,
                                                            const double* __restrict__ delta, float* __restrict__ sigma) {
    __shared__ double tr[32][33];
    const int tid = threadIdx.x, tx = tid & 31, ty = tid >> 5;
    const int pair = blockIdx.x;
    int ti, tj;
    pair_to_tiles(pair, T, ti, tj);
    const bool diag = ti == tj;
    const double Bd = static_cast<double>(B);
    const int64_t tile_elems = TRK_T * TRK_T, split_stride = static_cast<int64_t>(pairs) * tile_elems;
    const float* base = partial + static_cast<int64_t>(pair) * tile_elems;
    for (int bi = 0; bi < 4; ++bi) {
        for (int bj = 0; bj < 4; ++bj) {
            for (int rr = 0; rr < 4; ++rr) {
                const int il = bi * 32 + ty * 4 + rr, jl = bj * 32 + tx;
                const int i = ti * TRK_T + il, j = tj * TRK_T + jl;
                double c = 0.0;
                if (i < K && j < K) {
                    double s = 0.0;
                    for (int sp = 0; sp < splits; ++sp) s += static_cast<double>(base[sp * split_stride + il * TRK_T + jl]);
                    // products of the two columns first: (i, j) and (j, i) then give identical bits
                    const double sb = s - Bd * (mub[i] * mub[j]);
                    c = sb + coef * (delta[i] * delta[j]);
                    float* dst = sigma + static_cast<int64_t>(i) * K + j;
                    *dst = static_cast<float>(static_cast<double>(*dst) + c);
                }
                if (!diag) tr[ty * 4 + rr][tx] = c;
            }
            if (!diag) {
                __syncthreads();
                for (int rr = 0; rr < 4; ++rr) {
                    const int jl = bj * 32 + ty * 4 + rr, il = bi * 32 + tx;
                    const int i = ti * TRK_T + il, j = tj * TRK_T + jl;
                    if (i < K && j < K) {
                        float* dst = sigma + static_cast<int64_t>(j) * K + i;
                        *dst = static_cast<float>(static_cast<double>(*dst) + tr[tx][ty * 4 + rr]);
                    }
                }
                __syncthreads();
            }
        }
    }
}

size_t tracker_workspace_bytes(int64_t B, int64_t K) { return tracker_plan(B, K).bytes; }

loka_status tracker_update_launch(const void* x, int64_t B, int64_t K, int64_t ld, int64_t n_old, float* mu, float* sigma,
                                  void* workspace, hipStream_t s) {
    const TrackerPlan pl = tracker_plan(B, K);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    float* partial = reinterpret_cast<float*>(ws);
    double* colsum = reinterpret_cast<double*>(ws + pl.off_colsum);
    double* mub = reinterpret_cast<double*>(ws + pl.off_mub);
    double* delta = reinterpret_cast<double*>(ws + pl.off_delta);
    const int KP = pl.T * TRK_T;
    tracker_scatter_kernel<<<dim3(pl.pairs, pl.splits), 256, 0, s>>>(static_cast<const uint16_t*>(x), B, static_cast<int>(K), ld,
                                                                     pl.T, pl.pairs, pl.rows_per_split, partial, colsum);
    tracker_mean_kernel<<<dim3((KP + 255) / 256), 256, 0, s>>>(colsum, pl.splits, KP, static_cast<int>(K), B, n_old, mu, mub,
                                                               delta);
    const double n_new = static_cast<double>(n_old) + static_cast<double>(B);
    const double coef = static_cast<double>(n_old) * static_cast<double>(B) / n_new;
    tracker_merge_kernel<<<dim3(pl.pairs), 256, 0, s>>>(partial, pl.splits, pl.pairs, pl.T, static_cast<int>(K), B, coef, mub,
                                                        delta, sigma);
    return hipGetLastError() == hipSuccess ? LOKA_OK : LOKA_ERR_HIP;
}

}  // namespace loka
