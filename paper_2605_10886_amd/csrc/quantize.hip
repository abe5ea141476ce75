// amax -> scale -> OCP e4m3 cast of bf16 matrices (bandwidth-bound streaming kernels).
//
// ROW and BLOCK_1x128 scaling are single-pass: the lanes that share a scale group
// keep their elements in registers between the amax reduction and the cast, so the
// matrix is read once (2 B/elem) and the codes written once (1 B/elem).
// TENSOR, COL and BLOCK_128x128 scaling need every row of a group before the first
// cast: an amax pass (atomic max on the bit pattern of non-negative floats), a tiny
// finalize kernel (scale = amax/448, inv = 448/amax, one division each), and a cast
// pass that can also write the transposed layout used for weights.
#include "common.h"

namespace loka {

// ---------------------------------------------------------------------------------
// Single pass: TPR lanes share one row (TPR = 16, 32 or 64); each lane holds CPL
// chunks of 8 consecutive bf16 (one 16-byte load each); a wave works on RU row sets at
// once so that enough loads are in flight.  GW = lanes per scale group: TPR for ROW
// scaling (one group per row), 16 for 1x128 blocks (16 lanes x 8 elements).
template <int TPR, int CPL, int RU, bool BLOCK128>
__global__ __launch_bounds__(256) void quant_rows_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                         int64_t ld, uint8_t* __restrict__ q,
                                                         float* __restrict__ scales, const int pow2) {
    constexpr int ROWS_PER_WAVE = (64 / TPR) * RU;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int lr = lane % TPR;               // lane within its row
    const int sub = lane / TPR;              // which of the wave's concurrent rows
    const int64_t chunks = cols >> 3;        // 8-element chunks per row
    const int64_t row0 = (static_cast<int64_t>(blockIdx.x) * 4 + wave) * ROWS_PER_WAVE;

    u32x4 v[RU][CPL];
#pragma unroll
    for (int u = 0; u < RU; ++u) {
        const int64_t r = row0 + u * (64 / TPR) + sub;
#pragma unroll
        for (int j = 0; j < CPL; ++j) {
            const int64_t c = lr + static_cast<int64_t>(j) * TPR;
            if (r < rows && c < chunks)
                v[u][j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(x + r * ld + c * 8));
            else
                v[u][j] = u32x4{0u, 0u, 0u, 0u};
        }
    }
#pragma unroll
    for (int u = 0; u < RU; ++u) {
        const int64_t r = row0 + u * (64 / TPR) + sub;
        float am[CPL];
#pragma unroll
        for (int j = 0; j < CPL; ++j) {
            const u32x4 w = v[u][j];
            float a = fmaxf(fabsf(bf16_lo(w.x)), fabsf(bf16_hi(w.x)));
            a = fmaxf(a, fmaxf(fabsf(bf16_lo(w.y)), fabsf(bf16_hi(w.y))));
            a = fmaxf(a, fmaxf(fabsf(bf16_lo(w.z)), fabsf(bf16_hi(w.z))));
            a = fmaxf(a, fmaxf(fabsf(bf16_lo(w.w)), fabsf(bf16_hi(w.w))));
            am[j] = a;
        }
        if (!BLOCK128) {
#pragma unroll
            for (int j = 1; j < CPL; ++j) am[0] = fmaxf(am[0], am[j]);
#pragma unroll
            for (int m = 1; m < TPR; m <<= 1) am[0] = fmaxf(am[0], wave_shfl_xor(am[0], m));
        } else {
#pragma unroll
            for (int j = 0; j < CPL; ++j)
#pragma unroll
                for (int m = 1; m < 16; m <<= 1) am[j] = fmaxf(am[j], wave_shfl_xor(am[j], m));
        }
#pragma unroll
        for (int j = 0; j < CPL; ++j) {
            const int64_t c = lr + static_cast<int64_t>(j) * TPR;
            float scale, inv;
            group_scale_any(BLOCK128 && pow2, BLOCK128 ? am[j] : am[0], scale, inv);
            if (r < rows && c < chunks) {
                const u32x4 w = v[u][j];
                u32x2 o;
                o.x = e4m3x4(bf16_lo(w.x) * inv, bf16_hi(w.x) * inv, bf16_lo(w.y) * inv, bf16_hi(w.y) * inv);
                o.y = e4m3x4(bf16_lo(w.z) * inv, bf16_hi(w.z) * inv, bf16_lo(w.w) * inv, bf16_hi(w.w) * inv);
                // plain store: the GEMM that follows reads the codes from the last-level cache (measured at
                // 32768 x 4096: the GEMM runs 3 % faster than after a streaming store, this kernel no slower)
                *reinterpret_cast<u32x2*>(q + r * cols + c * 8) = o;
                if (BLOCK128) {
                    if ((c & 15) == 0) scales[r * (cols >> 7) + (c >> 4)] = scale;
                } else if (j == 0 && lr == 0) {
                    scales[r] = scale;
                }
            }
        }
    }
}

// Rows longer than the register-resident kernel covers: one workgroup per row, two
// sweeps over the row (the second one hits the cache).
template <bool BLOCK128>
__global__ __launch_bounds__(256) void quant_long_rows_kernel(const uint16_t* __restrict__ x, int64_t rows,
                                                              int64_t cols, int64_t ld, uint8_t* __restrict__ q,
                                                              float* __restrict__ scales, const int pow2) {
    __shared__ float red[4];
    const int64_t r = blockIdx.x;
    const int64_t chunks = cols >> 3;
    const uint16_t* xr = x + r * ld;
    float inv_row = 0.f;
    if (!BLOCK128) {
        float a = 0.f;
        for (int64_t c = threadIdx.x; c < chunks; c += 256) {
            const u32x4 w = *reinterpret_cast<const u32x4*>(xr + c * 8);
            a = fmaxf(a, fmaxf(fabsf(bf16_lo(w.x)), fabsf(bf16_hi(w.x))));
            a = fmaxf(a, fmaxf(fabsf(bf16_lo(w.y)), fabsf(bf16_hi(w.y))));
            a = fmaxf(a, fmaxf(fabsf(bf16_lo(w.z)), fabsf(bf16_hi(w.z))));
            a = fmaxf(a, fmaxf(fabsf(bf16_lo(w.w)), fabsf(bf16_hi(w.w))));
        }
        for (int m = 1; m < 64; m <<= 1) a = fmaxf(a, wave_shfl_xor(a, m));
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = a;
        __syncthreads();
        a = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        float scale;
        group_scale(a, scale, inv_row);
        if (threadIdx.x == 0) scales[r] = scale;
    }
    // chunks is a multiple of 16 for 1x128 blocks, so the 16 lanes of a group stay together
    for (int64_t c0 = 0; c0 < chunks; c0 += 256) {
        const int64_t c = c0 + threadIdx.x;
        const bool ok = c < chunks;
        u32x4 w = u32x4{0u, 0u, 0u, 0u};
        if (ok) w = *reinterpret_cast<const u32x4*>(xr + c * 8);
        float inv = inv_row;
        if (BLOCK128) {
            float a = fmaxf(fabsf(bf16_lo(w.x)), fabsf(bf16_hi(w.x)));
            a = fmaxf(a, fmaxf(fabsf(bf16_lo(w.y)), fabsf(bf16_hi(w.y))));
            a = fmaxf(a, fmaxf(fabsf(bf16_lo(w.z)), fabsf(bf16_hi(w.z))));
            a = fmaxf(a, fmaxf(fabsf(bf16_lo(w.w)), fabsf(bf16_hi(w.w))));
            for (int m = 1; m < 16; m <<= 1) a = fmaxf(a, wave_shfl_xor(a, m));
            float scale;
            group_scale_any(pow2, a, scale, inv);
            if (ok && (c & 15) == 0) scales[r * (cols >> 7) + (c >> 4)] = scale;
        }
        if (ok) {
            u32x2 o;
            o.x = e4m3x4(bf16_lo(w.x) * inv, bf16_hi(w.x) * inv, bf16_lo(w.y) * inv, bf16_hi(w.y) * inv);
            o.y = e4m3x4(bf16_lo(w.z) * inv, bf16_hi(w.z) * inv, bf16_lo(w.w) * inv, bf16_hi(w.w) * inv);
            *reinterpret_cast<u32x2*>(q + r * cols + c * 8) = o;
        }
    }
}

// ---------------------------------------------------------------------------------
// Multi-pass path.  Workspace layout: uint32 amax_bits[ng] followed by float inv[ng].
__global__ void fill_u32_kernel(uint32_t* p, int64_t n, uint32_t v) {
    int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

__device__ __forceinline__ float chunk_amax(const u32x4 w) {
    float a = fmaxf(fabsf(bf16_lo(w.x)), fabsf(bf16_hi(w.x)));
    a = fmaxf(a, fmaxf(fabsf(bf16_lo(w.y)), fabsf(bf16_hi(w.y))));
    a = fmaxf(a, fmaxf(fabsf(bf16_lo(w.z)), fabsf(bf16_hi(w.z))));
    return fmaxf(a, fmaxf(fabsf(bf16_lo(w.w)), fabsf(bf16_hi(w.w))));
}

// TENSOR: grid-stride over all chunks, one atomic per workgroup.
__global__ __launch_bounds__(256) void amax_tensor_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                          int64_t ld, uint32_t* __restrict__ amax_bits) {
    __shared__ float red[4];
    const int64_t chunks = cols >> 3;
    const int64_t total = rows * chunks;
    float a = 0.f;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < total;
         i += static_cast<int64_t>(gridDim.x) * 256) {
        const int64_t r = i / chunks, c = i - r * chunks;
        a = fmaxf(a, chunk_amax(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(x + r * ld + c * 8))));
    }
    for (int m = 1; m < 64; m <<= 1) a = fmaxf(a, wave_shfl_xor(a, m));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = a;
    __syncthreads();
    if (threadIdx.x == 0) {
        a = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        atomicMax(amax_bits, __float_as_uint(a));
    }
}

// COL: a workgroup owns 2048 columns x ROWS_PER_BLOCK rows; each thread keeps the
// maxima of its 8 columns and publishes them with 8 atomics.
constexpr int kColRowsPerBlock = 64;
__global__ __launch_bounds__(256) void amax_col_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                       int64_t ld, uint32_t* __restrict__ amax_bits) {
    const int64_t c = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;      // chunk column
    if (c >= (cols >> 3)) return;
    const int64_t r0 = static_cast<int64_t>(blockIdx.y) * kColRowsPerBlock;
    const int64_t r1 = r0 + kColRowsPerBlock < rows ? r0 + kColRowsPerBlock : rows;
    float a[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int64_t r = r0; r < r1; ++r) {
        const u32x4 w = *reinterpret_cast<const u32x4*>(x + r * ld + c * 8);
        a[0] = fmaxf(a[0], fabsf(bf16_lo(w.x))); a[1] = fmaxf(a[1], fabsf(bf16_hi(w.x)));
        a[2] = fmaxf(a[2], fabsf(bf16_lo(w.y))); a[3] = fmaxf(a[3], fabsf(bf16_hi(w.y)));
        a[4] = fmaxf(a[4], fabsf(bf16_lo(w.z))); a[5] = fmaxf(a[5], fabsf(bf16_hi(w.z)));
        a[6] = fmaxf(a[6], fabsf(bf16_lo(w.w))); a[7] = fmaxf(a[7], fabsf(bf16_hi(w.w)));
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) atomicMax(amax_bits + c * 8 + j, __float_as_uint(a[j]));
}

__global__ void finalize_scales_kernel(const uint32_t* __restrict__ amax_bits, float* __restrict__ inv,
                                       float* __restrict__ scales, int64_t ng, const int pow2) {
    int64_t g = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (g < ng) {
        float s, i;
        group_scale_any(pow2, __uint_as_float(amax_bits[g]), s, i);
        scales[g] = s;
        inv[g] = i;
    }
}

// Cast pass.  MODE selects how a chunk finds its factor(s); TRANSPOSE writes q[c, r].
template <int MODE>
__device__ __forceinline__ void load_inv8(const float* __restrict__ inv, int64_t r, int64_t c8, int64_t cols,
                                          float (&f)[8]) {
    if (MODE == LOKA_SCALE_TENSOR) {
        const float v = inv[0];
#pragma unroll
        for (int j = 0; j < 8; ++j) f[j] = v;
    } else {
        const float4 a = *reinterpret_cast<const float4*>(inv + c8);
        const float4 b = *reinterpret_cast<const float4*>(inv + c8 + 4);
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
    }
}

template <int MODE>
__global__ __launch_bounds__(256) void cast_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                   int64_t ld, const float* __restrict__ inv,
                                                   uint8_t* __restrict__ q) {
    const int64_t chunks = cols >> 3;
    const int64_t total = rows * chunks;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < total;
         i += static_cast<int64_t>(gridDim.x) * 256) {
        const int64_t r = i / chunks, c = i - r * chunks;
        const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(x + r * ld + c * 8));
        float f[8];
        load_inv8<MODE>(inv, r, c * 8, cols, f);
        u32x2 o;
        o.x = e4m3x4(bf16_lo(w.x) * f[0], bf16_hi(w.x) * f[1], bf16_lo(w.y) * f[2], bf16_hi(w.y) * f[3]);
        o.y = e4m3x4(bf16_lo(w.z) * f[4], bf16_hi(w.z) * f[5], bf16_lo(w.w) * f[6], bf16_hi(w.w) * f[7]);
        *reinterpret_cast<u32x2*>(q + r * cols + c * 8) = o;   // plain store: the consumer reads the codes next
    }
}

// 64 x 64 tile through LDS; rows % 16 == 0 and cols % 16 == 0, so 16-row / 8-column
// pieces are either fully inside or fully outside the matrix.
template <int MODE>
__global__ __launch_bounds__(256) void cast_transpose_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                             int64_t ld, const float* __restrict__ inv,
                                                             uint8_t* __restrict__ q) {
    __shared__ uint8_t tile[64][64 + 16];        // [c][r], padded rows keep 16-byte alignment
    const int64_t r0 = static_cast<int64_t>(blockIdx.y) * 64, c0 = static_cast<int64_t>(blockIdx.x) * 64;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int idx = threadIdx.x + s * 256;   // 512 chunks: 64 rows x 8 chunks
        const int rr = idx >> 3, cc = (idx & 7) * 8;
        const int64_t r = r0 + rr, c = c0 + cc;
        if (r < rows && c < cols) {
            const u32x4 w = *reinterpret_cast<const u32x4*>(x + r * ld + c);
            float f[8];
            load_inv8<MODE>(inv, r, c, cols, f);
            const uint32_t lo = e4m3x4(bf16_lo(w.x) * f[0], bf16_hi(w.x) * f[1], bf16_lo(w.y) * f[2], bf16_hi(w.y) * f[3]);
            const uint32_t hi = e4m3x4(bf16_lo(w.z) * f[4], bf16_hi(w.z) * f[5], bf16_lo(w.w) * f[6], bf16_hi(w.w) * f[7]);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                tile[cc + j][rr] = static_cast<uint8_t>(lo >> (8 * j));
                tile[cc + 4 + j][rr] = static_cast<uint8_t>(hi >> (8 * j));
            }
        }
    }
    __syncthreads();
    const int cc = threadIdx.x >> 2, rr = (threadIdx.x & 3) * 16;
    const int64_t c = c0 + cc, r = r0 + rr;
    if (c < cols && r < rows)
        *reinterpret_cast<u32x4*>(q + c * rows + r) = *reinterpret_cast<const u32x4*>(&tile[cc][rr]);
}

// Single-pass quantization of the modes whose scale groups fit one workgroup: a workgroup takes a 128 x 128 tile
// (8 sweeps of 16 rows x 16 chunks of 8 elements: 32 registers per thread), finds the amax of its groups on chip,
// scales, casts and stores - every element is read once and written once (3 bytes per element).
//   COLGROUPS == false: the whole tile is one group (BLOCK_128x128 and its power-of-two form); scales [rows/128][cols/128]
//   COLGROUPS == true:  every column of the tile is a group (BLOCK_128x1); scales [cols][rows/128]
//   TRANSPOSE: codes leave as [cols, rows] through an LDS tile (64-byte runs per output row)
// rows % 128 == 0; cols % 16 == 0 (COLGROUPS) or % 128 == 0: chunks past the last column are skipped.
template <bool COLGROUPS, bool TRANSPOSE>
__global__ __launch_bounds__(256) void quant_tile128_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                            int64_t ld, uint8_t* __restrict__ q, float* __restrict__ scales,
                                                            const int pow2) {
    __shared__ float red[4 * 128];                      // per wave: column maxima (COLGROUPS) or one value
    __shared__ float inv_s[128];
    __shared__ __attribute__((aligned(16))) uint8_t tile[TRANSPOSE ? 128 * (128 + 16) : 16];   // [c][r], rows padded to 144 bytes
    const int t = static_cast<int>(threadIdx.x), lane = t & 63, wave = t >> 6;
    const int cc = t & 15, rr = t >> 4;                 // chunk column; the thread's 8 consecutive rows are rr * 8 + [0, 8)
    const int64_t r0 = static_cast<int64_t>(blockIdx.y) * 128, c0 = static_cast<int64_t>(blockIdx.x) * 128;
    const bool live = c0 + cc * 8 < cols;
    u32x4 w[8];
#pragma unroll
    for (int sw = 0; sw < 8; ++sw) {
        w[sw] = u32x4{0u, 0u, 0u, 0u};
        if (live) w[sw] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(x + (r0 + rr * 8 + sw) * ld + c0 + cc * 8));
    }
    float inv8[8];
    if (COLGROUPS) {
        float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int sw = 0; sw < 8; ++sw) {
            a[0] = fmaxf(a[0], fabsf(bf16_lo(w[sw].x))); a[1] = fmaxf(a[1], fabsf(bf16_hi(w[sw].x)));
            a[2] = fmaxf(a[2], fabsf(bf16_lo(w[sw].y))); a[3] = fmaxf(a[3], fabsf(bf16_hi(w[sw].y)));
            a[4] = fmaxf(a[4], fabsf(bf16_lo(w[sw].z))); a[5] = fmaxf(a[5], fabsf(bf16_hi(w[sw].z)));
            a[6] = fmaxf(a[6], fabsf(bf16_lo(w[sw].w))); a[7] = fmaxf(a[7], fabsf(bf16_hi(w[sw].w)));
        }
        // lanes l, l ^ 16, l ^ 32, l ^ 48 of a wave hold the same columns (rows rr differ); then the 4 waves through LDS
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            a[j] = fmaxf(a[j], wave_shfl_xor(a[j], 16));
            a[j] = fmaxf(a[j], wave_shfl_xor(a[j], 32));
        }
        if (lane < 16) {
#pragma unroll
            for (int j = 0; j < 8; ++j) red[wave * 128 + cc * 8 + j] = a[j];
        }
        __syncthreads();
        if (t < 128) {
            const float am = fmaxf(fmaxf(red[t], red[128 + t]), fmaxf(red[256 + t], red[384 + t]));
            float sc, iv;
            group_scale_any(pow2 != 0, am, sc, iv);
            inv_s[t] = iv;
            if (c0 + t < cols) scales[(c0 + t) * (rows >> 7) + blockIdx.y] = sc;
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; ++j) inv8[j] = inv_s[cc * 8 + j];
    } else {
        float a = 0.f;
#pragma unroll
        for (int sw = 0; sw < 8; ++sw) a = fmaxf(a, chunk_amax(w[sw]));
        for (int m = 1; m < 64; m <<= 1) a = fmaxf(a, wave_shfl_xor(a, m));
        if (lane == 0) red[wave] = a;
        __syncthreads();
        float sc, iv;
        group_scale_any(pow2 != 0, fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])), sc, iv);
        if (t == 0) scales[blockIdx.y * (cols >> 7) + blockIdx.x] = sc;
#pragma unroll
        for (int j = 0; j < 8; ++j) inv8[j] = iv;
    }
    uint32_t lo[8], hi[8];                              // codes of row rr * 8 + sw, columns cc * 8 + [0, 4) and + [4, 8)
#pragma unroll
    for (int sw = 0; sw < 8; ++sw) {
        lo[sw] = e4m3x4(bf16_lo(w[sw].x) * inv8[0], bf16_hi(w[sw].x) * inv8[1], bf16_lo(w[sw].y) * inv8[2], bf16_hi(w[sw].y) * inv8[3]);
        hi[sw] = e4m3x4(bf16_lo(w[sw].z) * inv8[4], bf16_hi(w[sw].z) * inv8[5], bf16_lo(w[sw].w) * inv8[6], bf16_hi(w[sw].w) * inv8[7]);
        if (!TRANSPOSE && live) *reinterpret_cast<u32x2*>(q + (r0 + rr * 8 + sw) * cols + c0 + cc * 8) = u32x2{lo[sw], hi[sw]};
    }
    if (TRANSPOSE) {
        // the thread's 8 x 8 block of codes is transposed in registers (byte permutes on 4 x 4 sub-blocks), so that each
        // of its 8 columns becomes one 8-byte run of consecutive rows; the runs go through LDS and leave as 64-byte runs
        auto t4 = [](uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3, uint32_t (&c)[4]) __attribute__((always_inline)) {
            const uint32_t p0 = __builtin_amdgcn_perm(a1, a0, 0x05010400u), p1 = __builtin_amdgcn_perm(a1, a0, 0x07030602u);
            const uint32_t p2 = __builtin_amdgcn_perm(a3, a2, 0x05010400u), p3 = __builtin_amdgcn_perm(a3, a2, 0x07030602u);
            c[0] = __builtin_amdgcn_perm(p2, p0, 0x05040100u); c[1] = __builtin_amdgcn_perm(p2, p0, 0x07060302u);
            c[2] = __builtin_amdgcn_perm(p3, p1, 0x05040100u); c[3] = __builtin_amdgcn_perm(p3, p1, 0x07060302u);
        };
        uint32_t a[4], b[4], c[4], d[4];
        t4(lo[0], lo[1], lo[2], lo[3], a);                  // columns 0..3, rows 0..3
        t4(lo[4], lo[5], lo[6], lo[7], b);                  // columns 0..3, rows 4..7
        t4(hi[0], hi[1], hi[2], hi[3], c);                  // columns 4..7, rows 0..3
        t4(hi[4], hi[5], hi[6], hi[7], d);                  // columns 4..7, rows 4..7
        // (LDS row = output row: 16 runs of 8 codes, run rr at position rr ^ cc with cc = the row's chunk column: the 64
        // lanes of a write then spread over all banks two deep, where unswizzled they met on 16 of the 64)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            *reinterpret_cast<u32x2*>(tile + (cc * 8 + j) * 144 + ((rr ^ cc) << 3)) = u32x2{a[j], b[j]};
            *reinterpret_cast<u32x2*>(tile + (cc * 8 + 4 + j) * 144 + ((rr ^ cc) << 3)) = u32x2{c[j], d[j]};
        }
        __syncthreads();
        // output row c0 + c: 128 codes.  Eight consecutive lanes write one row's 128 bytes, a store instruction of a
        // wave eight whole rows (full cache lines per request: with a thread per half row, four stores apart, every
        // instruction scattered 16-byte pieces over 32 lines)
        const int chunk = t & 7;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = j * 32 + (t >> 3), key = col >> 3;           // the row's runs 2 chunk, 2 chunk + 1 sit at ^ key
            u32x4 v = *reinterpret_cast<const u32x4*>(tile + col * 144 + ((chunk ^ (key >> 1)) << 4));
            if (key & 1) v = u32x4{v.z, v.w, v.x, v.y};
            if (c0 + col < cols) *reinterpret_cast<u32x4*>(q + (c0 + col) * rows + r0 + chunk * 16) = v;
        }
    }
}

__global__ void e4m3_from_f32_kernel(const float* __restrict__ t, uint8_t* __restrict__ codes, int64_t n) {
    int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) codes[i] = static_cast<uint8_t>(e4m3x4(t[i], 0.f, 0.f, 0.f) & 0xFFu);
}

// ---------------------------------------------------------------------------------
template <bool B128>
static void launch_rows(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, uint8_t* q, float* scales,
                        int pow2, hipStream_t s) {
    const int64_t chunks = cols / 8;
    auto grid = [&](int rows_per_wave) {
        return dim3(static_cast<unsigned>((rows + 4 * rows_per_wave - 1) / (4 * rows_per_wave)));
    };
#define LOKA_QR(TPR, CPL, RU) \
    quant_rows_kernel<TPR, CPL, RU, B128><<<grid((64 / TPR) * RU), 256, 0, s>>>(x, rows, cols, ld, q, scales, pow2)
    // Rows per wave: enough loads in flight per lane when the launch has many waves per SIMD anyway, fewer rows
    // per wave (more waves) when the whole tensor would otherwise be a handful of waves per SIMD.
    const bool few = rows * chunks < (int64_t(1) << 21);      // under 32 MB of bf16 (measured: 16384 x 512 8.8 -> 6.7 us)
    if (chunks <= 16) LOKA_QR(16, 1, 2);
    else if (chunks <= 32) { if (few) LOKA_QR(32, 1, 1); else LOKA_QR(32, 1, 4); }
    else if (chunks <= 64) { if (few) LOKA_QR(64, 1, 2); else LOKA_QR(64, 1, 8); }
    else if (chunks <= 128) { if (few) LOKA_QR(64, 2, 1); else LOKA_QR(64, 2, 4); }
    else if (chunks <= 256) LOKA_QR(64, 4, 2);
    else if (chunks <= 512) LOKA_QR(64, 8, 1);
    else if (chunks <= 1024) LOKA_QR(64, 16, 1);
    else quant_long_rows_kernel<B128><<<dim3(static_cast<unsigned>(rows)), 256, 0, s>>>(x, rows, cols, ld, q, scales, pow2);
#undef LOKA_QR
}

template <int MODE>
static void launch_cast(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, const float* inv, uint8_t* q,
                        int transpose_out, hipStream_t s) {
    if (transpose_out) {
        dim3 g(static_cast<unsigned>((cols + 63) / 64), static_cast<unsigned>((rows + 63) / 64));
        cast_transpose_kernel<MODE><<<g, 256, 0, s>>>(x, rows, cols, ld, inv, q);
    } else {
        const int64_t total = rows * (cols / 8);
        int64_t blocks = (total + 255) / 256;
        if (blocks > 256 * 64) blocks = 256 * 64;
        cast_kernel<MODE><<<dim3(static_cast<unsigned>(blocks)), 256, 0, s>>>(x, rows, cols, ld, inv, q);
    }
}

loka_status quantize_launch(const void* x_bf16, int64_t rows, int64_t cols, int64_t ld, loka_scale_mode mode,
                            int transpose_out, uint8_t* q, float* scales, void* workspace, hipStream_t s) {
    const uint16_t* x = static_cast<const uint16_t*>(x_bf16);
    // the power-of-two block modes: the plain block modes' passes with another scale rule
    const int pow2 = mode == LOKA_SCALE_BLOCK_1x128_POW2 || mode == LOKA_SCALE_BLOCK_128x128_POW2;
    if (mode == LOKA_SCALE_BLOCK_1x128_POW2) mode = LOKA_SCALE_BLOCK_1x128;
    if (mode == LOKA_SCALE_BLOCK_128x128_POW2) mode = LOKA_SCALE_BLOCK_128x128;
    if (!transpose_out && (mode == LOKA_SCALE_ROW || mode == LOKA_SCALE_BLOCK_1x128)) {
        if (mode == LOKA_SCALE_ROW) launch_rows<false>(x, rows, cols, ld, q, scales, 0, s);
        else launch_rows<true>(x, rows, cols, ld, q, scales, pow2, s);
        return hipGetLastError() == hipSuccess ? LOKA_OK : LOKA_ERR_HIP;
    }
    if (mode == LOKA_SCALE_BLOCK_128x128 || mode == LOKA_SCALE_BLOCK_128x1) {
        // groups that fit a workgroup: one pass
        const dim3 g(static_cast<unsigned>((cols + 127) / 128), static_cast<unsigned>(rows / 128));
        if (mode == LOKA_SCALE_BLOCK_128x1) quant_tile128_kernel<true, true><<<g, 256, 0, s>>>(x, rows, cols, ld, q, scales, 0);
        else if (transpose_out) quant_tile128_kernel<false, true><<<g, 256, 0, s>>>(x, rows, cols, ld, q, scales, pow2);
        else quant_tile128_kernel<false, false><<<g, 256, 0, s>>>(x, rows, cols, ld, q, scales, pow2);
        return hipGetLastError() == hipSuccess ? LOKA_OK : LOKA_ERR_HIP;
    }
    const int64_t ng = loka_scale_count(mode, rows, cols);
    uint32_t* amax_bits = static_cast<uint32_t*>(workspace);
    float* inv = reinterpret_cast<float*>(amax_bits + ng);
    if (mode == LOKA_SCALE_TENSOR) {
        fill_u32_kernel<<<1, 64, 0, s>>>(amax_bits, 1, 0u);
        const int64_t total = rows * (cols / 8);
        int64_t blocks = (total + 255) / 256;
        if (blocks > 256 * 16) blocks = 256 * 16;
        amax_tensor_kernel<<<dim3(static_cast<unsigned>(blocks)), 256, 0, s>>>(x, rows, cols, ld, amax_bits);
    } else if (mode == LOKA_SCALE_COL) {
        fill_u32_kernel<<<dim3(static_cast<unsigned>((ng + 255) / 256)), 256, 0, s>>>(amax_bits, ng, 0u);
        dim3 g(static_cast<unsigned>((cols / 8 + 255) / 256),
               static_cast<unsigned>((rows + kColRowsPerBlock - 1) / kColRowsPerBlock));
        amax_col_kernel<<<g, 256, 0, s>>>(x, rows, cols, ld, amax_bits);
    }
    finalize_scales_kernel<<<dim3(static_cast<unsigned>((ng + 255) / 256)), 256, 0, s>>>(amax_bits, inv, scales, ng, pow2);
    if (mode == LOKA_SCALE_TENSOR) launch_cast<LOKA_SCALE_TENSOR>(x, rows, cols, ld, inv, q, transpose_out, s);
    else launch_cast<LOKA_SCALE_COL>(x, rows, cols, ld, inv, q, transpose_out, s);
    return hipGetLastError() == hipSuccess ? LOKA_OK : LOKA_ERR_HIP;
}

loka_status e4m3_from_f32_launch(const float* t, uint8_t* codes, int64_t n, hipStream_t s) {
    e4m3_from_f32_kernel<<<dim3(static_cast<unsigned>((n + 255) / 256)), 256, 0, s>>>(t, codes, n);
    return hipGetLastError() == hipSuccess ? LOKA_OK : LOKA_ERR_HIP;
}

}  // namespace loka
