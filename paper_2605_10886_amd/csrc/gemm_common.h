// Definitions shared by the GEMM translation units (gemm.hip, gemm_panel32.hip).
#pragma once

#include "common.h"

namespace loka {

enum { EPI_ROW_IN_TILE = 0, EPI_PARTIAL_STATS = 1, EPI_PANEL_SYNC = 2 };

struct GemmParams {
    const uint8_t* X;      // [batch][M][KB] bytes (KB = K for FP8, 2K for BF16)
    const uint8_t* W;      // [batch][N][KB]
    int M, N, KB;
    int batch;
    int64_t strideX, strideW;   // bytes between problems
    int64_t strideO;            // elements between problems (O, Y)
    const float* sx;
    const float* sw;
    int64_t strideSx, strideSw; // scales between problems
    int x_mode, w_mode;
    const uint16_t* gamma;
    const uint16_t* beta;
    uint16_t* out;
    uint8_t* outq;         // FP8 output instead of `out`: e4m3 codes [batch][M][N] ...
    float* outs;           // ... and their row scales [batch][M]
    const uint16_t* xb;    // fused quantization (streaming kernel): bf16 X [batch][M][K] instead of X / sx ...
    float* sx_out;         // ... and, optionally, where the row scales it computes are written [batch][M]
    float* y;
    int norm;              // loka_norm
    int block_n, act;      // LOKA_NORM_BLOCKNORM group width; loka_act
    float eps;
    int tiles_m, tiles_n;
    float* part;           // EPI_PARTIAL_STATS / EPI_PANEL_SYNC: [batch][M][tiles_n * 2] (mean, M2) or (0, sumsq)
                           // (gemm_panel32.hip: [batch][tiles_m][tiles_n][256] such pairs, then as many (min, max) pairs)
    unsigned* counters;    // EPI_PANEL_SYNC: arrivals per (problem, m tile), zeroed before the launch
    unsigned* error_flag;  // EPI_PANEL_SYNC: set when a bounded wait ran out
    unsigned spin_limit;
    unsigned arrivals;     // EPI_PANEL_SYNC: counter value a workgroup waits for (tiles_n; one more in the error-path test)
};

#ifdef LOKA_DEBUG_TIMES
// per translation unit: each GEMM source exports its own reader
static __device__ unsigned long long loka_dbg_times[8 * 4096];
#define LOKA_STAMP(slot) do { if (threadIdx.x == 0 && tile < 4096) loka_dbg_times[tile * 8 + (slot)] = wall_clock64(); } while (0)
#else
#define LOKA_STAMP(slot) do { } while (0)
#endif

// Output column of MFMA tile ti, element i, for a lane of group q (= lane / 16), relative to the wave's
// first column: (ti / 2) * 32 + q * 8 + (ti % 2) * 4 + i.  A lane owns 8 consecutive columns per tile pair,
// and the four lane groups of a row together cover 32 consecutive columns: one 16-byte bf16 store per
// lane writes full 64-byte runs per row.
__host__ __device__ constexpr int coff_of(int ti) { return (ti >> 1) * 32 + (ti & 1) * 4; }

// Workgroup barrier that orders LDS traffic only: LDS reads/writes issued before it are complete, but
// global loads (including the loads that stream the next stage into LDS) stay in flight across it.
// Completion of those is awaited explicitly (s_waitcnt vmcnt) where a stage is about to be read.
// Written as an instruction sequence: a fence builtin on the LDS address space makes the compiler wait for
// vmcnt(0) as well whenever loads-to-LDS are outstanding, which would expose their full latency each phase.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// Waits until at most N_ of this wave's vector-memory operations are outstanding (6-bit count, split
// over two fields of the instruction's immediate); the LDS and scalar counters are left alone.
template <int N_>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N_ & 15) | ((N_ >> 4) << 14));
}

// Chan's pairwise merge of (count, mean, M2).
__device__ __forceinline__ void merge_stats(float& n, float& mean, float& m2, float nb, float mb, float m2b) {
    const float nn = n + nb;
    if (nb > 0.f) {
        const float d = mb - mean;
        const float f = nb * __builtin_amdgcn_rcpf(nn);   // nn > 0 here; 1-ulp reciprocal (an IEEE divide costs ~300 cycles)
        mean = mean + d * f;
        m2 = m2 + m2b + d * d * n * f;
        n = nn;
    }
}

}  // namespace loka
