// Definitions shared by the GEMM translation units (gemm.hip, gemm_panel32.hip).
#pragma once

#include "common.h"

namespace loka {

enum { EPI_ROW_IN_TILE = 0, EPI_PARTIAL_STATS = 1, EPI_PANEL_SYNC = 2, EPI_SPLITK = 3 };

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
    int qpro;              // quantize prologue (streaming kernel): xb is quantized row by row into X / sx (written, then read back)
    float* y;
    int norm;              // loka_norm
    int block_n, act;      // LOKA_NORM_BLOCKNORM group width; loka_act
    float eps;
    int tiles_m, tiles_n;
    int ksplit, k_per_split;   // EPI_SPLITK: number of K ranges, and 128-byte K steps per range; part = [ksplit][batch][M][N] fp32
    float* part;           // EPI_PARTIAL_STATS / EPI_PANEL_SYNC: [batch][M][tiles_n * 2] (mean, M2) or (0, sumsq)
                           // (gemm_panel32.hip: [batch][tiles_m][tiles_n][256] such pairs, then as many (min, max) pairs)
    // EPI_PANEL_SYNC, the exchange between the workgroups of a row panel (see panel_publish_and_wait):
    unsigned long long* flags;   // [exchanges][batch * tiles_m][tiles_n] arrival words; a tile has arrived when its word == nonce
    unsigned long long* header;  // [0] nonce of the last launch on this workspace, [1] nonce of the last launch with a wait that ran out
    unsigned long long nonce;    // launch-unique, never 0
    unsigned long long expect;   // value the waits look for: nonce (nonce + 2, which nobody writes, in the error-path test)
    unsigned spin_limit;
};

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

// The exchange between the tiles_n workgroups that share a row panel (Section 3.2, Case 2: a row wider than a
// workgroup's tile).  Called by every thread of the workgroup after its per-row records have been STORED with
// device-coherent (agent-scope atomic, write-through) stores:
//   1. every wave waits until its own stores have been acknowledged (s_waitcnt vmcnt(0): a store is acknowledged once
//      it is visible at the scope it was issued with, here the device), then the workgroup barrier: all records of
//      this tile are visible device-wide;
//   2. wave 0 stores the tile's arrival word (= the launch's nonce; device-coherent) - program order after 1 - and polls
//      the panel's tiles_n arrival words (lanes = tiles; device-coherent loads that bypass this XCD's caches) until all
//      equal `expect`, sleeping between polls, for at most spin_limit polls;
//   3. barrier; the caller's threads then read the other tiles' records with device-coherent loads, issued after the
//      poll that saw every arrival word (loads are not issued early on this hardware, and they bypass the non-coherent
//      caches), so they return what was stored before step 2 of the publishing workgroup.
// No L2-wide write-back or invalidate is involved: the records and words are the only data that cross workgroups.
// Arrival words are compared with a nonce instead of counted, so nothing has to be zeroed between launches: a stale
// or uninitialised word never equals a fresh 64-bit nonce.
// Returns false when the wait ran out (never when all tiles_n workgroups are resident, which the launch arranges):
// the launch's nonce is then recorded in header[1] and the caller poisons the rows of its tile.
// `lds_word` is one LDS word the workgroup does not otherwise use during the call.
__device__ __forceinline__ bool panel_publish_and_wait(const GemmParams& p, unsigned long long* words, int tn, int tiles_n,
                                                       int* lds_word) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // (with the clobber the record stores stay in front of it)
    __syncthreads();
    if (threadIdx.x < 64) {
        int lane = static_cast<int>(threadIdx.x);
        asm volatile("; lane id" : "+v"(lane));           // (an opaque copy: addresses derived from it are not hoisted out of the tile loop)
        // (the two 64-bit values restart from the scalar registers here: taken from the parameter block directly, the
        // compiler moves them into vector registers once, before the tile loop, and spills them through the main loop)
        unsigned n_lo = static_cast<unsigned>(p.nonce), n_hi = static_cast<unsigned>(p.nonce >> 32);
        unsigned e_lo = static_cast<unsigned>(p.expect), e_hi = static_cast<unsigned>(p.expect >> 32);
        asm volatile("; arrival values" : "+s"(n_lo), "+s"(n_hi), "+s"(e_lo), "+s"(e_hi));
        const unsigned long long nonce = (static_cast<unsigned long long>(n_hi) << 32) | n_lo;
        const unsigned long long expect = (static_cast<unsigned long long>(e_hi) << 32) | e_lo;
        if (lane == 0) __hip_atomic_store(words + tn, nonce, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        unsigned spins = 0;
        bool failed = false;
        for (;;) {
            bool here = true;
            for (int t = lane; t < tiles_n; t += 64)
                here = here && __hip_atomic_load(words + t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == expect;
            if (__builtin_amdgcn_ballot_w64(!here) == 0) break;
            if (++spins > p.spin_limit) { failed = true; break; }
            __builtin_amdgcn_s_sleep(2);      // (measured at 32768 x 4096 x 4096: 16 costs 2 % of the kernel, 0 gains nothing more)
        }
        if (lane == 0) {
            if (failed) __hip_atomic_store(p.header + 1, nonce, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *lds_word = failed ? 1 : 0;
        }
    }
    __syncthreads();
    return *lds_word == 0;
}

}  // namespace loka
