// Measured ceilings of the machine the library runs on: what the FP8 / BF16 matrix pipes deliver from registers
// alone, and what a plain copy moves through HBM.  A measurement aid (loka_machine_ceiling): the benchmark reports a
// kernel's rate against these beside its rate against the datasheet peaks, because the sustained shader clock under
// matrix load sits below the clock the datasheet figures assume.
#include "common.h"

namespace loka {

typedef float v16f __attribute__((ext_vector_type(16)));

// One wave issues back-to-back MFMAs on 8 independent accumulator sets; operands never change (the result is
// meaningless, only the issue rate matters).  The accumulators are written out so the loop cannot be removed.
// VARIED: every one of the 8 instructions of a round takes different operand registers filled with pseudo-random
// codes of both signs and all exponents (as quantized data has), so that consecutive instructions toggle the
// multipliers' inputs; otherwise all instructions take the same two registers of small positive codes (the least
// switching activity the pipe can see: the highest clock it will hold).
template <bool BF16, bool VARIED>
__global__ __launch_bounds__(512) void mfma_rate_kernel(float* sink, int iters) {
    v16f acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    const int t = static_cast<int>(threadIdx.x);
    constexpr int NS = VARIED ? 8 : 1;
    v8i a[NS], b[NS];
    if (VARIED) {
        unsigned z = 0x9E3779B9u * static_cast<unsigned>(t + 1) + blockIdx.x;
#pragma unroll
        for (int j = 0; j < NS; ++j)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                z = z * 1664525u + 1013904223u;
                unsigned wa = z ^ (z >> 15);
                z = z * 1664525u + 1013904223u;
                unsigned wb = z ^ (z >> 13);
                // no NaN codes (0x7F / 0xFF): clear bit 0 of bytes whose low seven bits are all ones
                wa &= ~(((wa & (wa >> 1) & (wa >> 2) & (wa >> 3) & (wa >> 4) & (wa >> 5) & (wa >> 6)) & 0x01010101u));
                wb &= ~(((wb & (wb >> 1) & (wb >> 2) & (wb >> 3) & (wb >> 4) & (wb >> 5) & (wb >> 6)) & 0x01010101u));
                // (BF16: keep the exponents moderate so the sums stay finite)
                a[j][i] = BF16 ? static_cast<int>((wa & 0x8FFF8FFFu) | 0x30003000u) : static_cast<int>(wa);
                b[j][i] = BF16 ? static_cast<int>((wb & 0x8FFF8FFFu) | 0x30003000u) : static_cast<int>(wb);
            }
    } else {
        a[0] = v8i{t, t + 1, t + 2, t + 3, t + 4, t + 5, t + 6, t + 7};
        b[0] = v8i{t * 3, t * 3 + 1, t * 3 + 2, t * 3 + 3, t * 3 + 4, t * 3 + 5, t * 3 + 6, t * 3 + 7};
        a[0] &= v8i{0x3F3F3F3F, 0x3F3F3F3F, 0x3F3F3F3F, 0x3F3F3F3F, 0x3F3F3F3F, 0x3F3F3F3F, 0x3F3F3F3F, 0x3F3F3F3F};   // small finite codes
        b[0] &= v8i{0x3F3F3F3F, 0x3F3F3F3F, 0x3F3F3F3F, 0x3F3F3F3F, 0x3F3F3F3F, 0x3F3F3F3F, 0x3F3F3F3F, 0x3F3F3F3F};
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const v8i aj = a[VARIED ? j : 0], bj = b[VARIED ? j : 0];
            if (BF16) {
                const v4i a4 = v4i{aj[0], aj[1], aj[2], aj[3]}, b4 = v4i{bj[0], bj[1], bj[2], bj[3]};
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a4), __builtin_bit_cast(v8bf, b4), acc[j], 0, 0, 0);
            } else {
                acc[j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(aj, bj, acc[j], 0, 0, 0, 0, 0, 0);
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[j][i];
    if (s == 123.456f) sink[blockIdx.x * blockDim.x + threadIdx.x] = s;     // (never true: keeps the loop)
}

// Plain streaming copy: every thread keeps 8 loads of 16 bytes in flight (a workgroup moves 32 KB per round).
__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t n16) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * 2048;
    for (int64_t base = static_cast<int64_t>(blockIdx.x) * 2048 + threadIdx.x; base < n16; base += stride) {
        u32x4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (base + 256 * j < n16) v[j] = __builtin_nontemporal_load(src + base + 256 * j);
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (base + 256 * j < n16) __builtin_nontemporal_store(v[j], dst + base + 256 * j);
    }
}

// The same measurement with the 16x16x128 form of the FP8 instruction (half the outputs, twice the K per instruction:
// the same flops per cycle, twice the operand registers read per flop).
template <bool VARIED>
__global__ __launch_bounds__(512) void mfma_rate16_kernel(float* sink, int iters) {
    v4f acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = v4f{0.f, 0.f, 0.f, 0.f};
    const int t = static_cast<int>(threadIdx.x);
    v8i a[8], b[8];
    unsigned z = 0x9E3779B9u * static_cast<unsigned>(t + 1) + blockIdx.x;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            z = z * 1664525u + 1013904223u;
            unsigned wa = z ^ (z >> 15);
            z = z * 1664525u + 1013904223u;
            unsigned wb = z ^ (z >> 13);
            wa &= ~(((wa & (wa >> 1) & (wa >> 2) & (wa >> 3) & (wa >> 4) & (wa >> 5) & (wa >> 6)) & 0x01010101u));   // no NaN codes
            wb &= ~(((wb & (wb >> 1) & (wb >> 2) & (wb >> 3) & (wb >> 4) & (wb >> 5) & (wb >> 6)) & 0x01010101u));
            a[j][i] = VARIED ? static_cast<int>(wa) : 0x38383838;
            b[j][i] = VARIED ? static_cast<int>(wb) : 0x38383838;
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[j], b[j], acc[j], 0, 0, 0, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) s += (acc[j][0] + acc[j][1]) + (acc[j][2] + acc[j][3]);
    if (s == 123.456f) sink[blockIdx.x * blockDim.x + threadIdx.x] = s;     // (never true: keeps the loop)
}

// The large-layer kernel's operand stream without its arithmetic, on that kernel's schedule for a 32768 x 4096 x 4096
// layer: one workgroup of 8 waves per CU walks tiles first, first + G, ... (the same XCD-aware numbering: the 16
// workgroups of a 256-row panel run side by side on one XCD and share the panel, all panels share the weight matrix)
// and pulls, per K step of 128 bytes, the tile's 256 rows of X and 256 rows of W (64 KB) into a ring of five 32 KB LDS
// entries with loads that write LDS directly (four 1 KB loads per wave and entry, eight rows of 128 bytes each: the
// kernel's own request shape), at most one older step outstanding at the step's barrier.  Nothing reads the LDS: what
// is measured is how fast L2 and what lies behind it deliver this schedule's operands to the CUs.
__global__ __launch_bounds__(512) void lds_stream_kernel(const uint8_t* __restrict__ x, const uint8_t* __restrict__ w, int kb_row,
                                                         int tiles_n, int total_tiles, float* sink) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem_stream[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int ksteps = kb_row / 128;
    const int G = gridDim.x;
    const int tile_first = (G % 8 == 0) ? (blockIdx.x % 8) * (G / 8) + blockIdx.x / 8 : blockIdx.x;
    const int lane_off = (lane >> 3) * kb_row + (((lane & 7) ^ (lane >> 4)) << 4);
    int e = 0;
    for (int tile = tile_first; tile < total_tiles; tile += G) {
        const int tn = tile % tiles_n, tm = tile / tiles_n;
        const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint8_t*>(x + static_cast<int64_t>(tm) * 256 * kb_row), 0, 256 * kb_row, 0x00020000);
        const __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint8_t*>(w + static_cast<int64_t>(tn) * 256 * kb_row), 0, 256 * kb_row, 0x00020000);
        for (int k = 0; k < ksteps; ++k) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int grp = wave + 8 * j;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    xr, (__attribute__((address_space(3))) void*)(smem_stream + (e % 5) * 32768 + grp * 1024), 16, lane_off,
                    grp * 8 * kb_row + k * 128, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int grp = wave + 8 * j;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    wr, (__attribute__((address_space(3))) void*)(smem_stream + ((e + 1) % 5) * 32768 + grp * 1024), 16, lane_off,
                    grp * 8 * kb_row + k * 128, 0, 0);
            }
            e += 2;
            __builtin_amdgcn_s_waitcnt(0x0F70 | 8);        // all but the newest step's loads of this wave have landed
            __builtin_amdgcn_s_barrier();
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    const float v = reinterpret_cast<const float*>(smem_stream)[threadIdx.x];
    if (v == 123.456f && sink) sink[blockIdx.x] = v;        // (keeps the loads; sink is null in the measurement)
}

int device_cu_count();

// kind 0 / 1: FP8 / BF16 matrix rate in TFLOP/s over ~`millis` ms of back-to-back launches (the clock settles during
// the first tens of milliseconds under load; the rate of the LAST launch is returned);  kind 2: copy rate in GB/s
// (bytes read + written) of `scratch_bytes` / 2 bytes from the first half of `scratch` to the second;  kind 3: rate in
// GB/s at which the large-layer kernel's operand stream reaches the LDS of all CUs (no arithmetic);  kind 4 / 5: as
// 0 / 1 with operands that differ from instruction to instruction (pseudo-random codes);  kind 6 / 7: the FP8 rate
// with the 16x16x128 form of the instruction, on constant and on changing operands.
loka_status machine_ceiling(int kind, double millis, void* scratch, size_t scratch_bytes, double* value, hipStream_t s) {
    const int cus = device_cu_count();
    if (cus <= 0) return LOKA_ERR_HIP;
    hipEvent_t e0, e1;
    LOKA_HIP_TRY(hipEventCreate(&e0));
    LOKA_HIP_TRY(hipEventCreate(&e1));
    struct Guard { hipEvent_t a, b; ~Guard() { (void)hipEventDestroy(a); (void)hipEventDestroy(b); } } guard{e0, e1};
    float ms = 0.f;
    double total = 0.0, last = 0.0;
    if (kind == 6 || kind == 7) {
        const int iters = 8192;
        const double flops = static_cast<double>(cus) * 8 * iters * 8 * 2.0 * 16 * 16 * 128;
        while (total < millis) {
            LOKA_HIP_TRY(hipEventRecord(e0, s));
            if (kind == 6) mfma_rate16_kernel<false><<<dim3(cus), 512, 0, s>>>(static_cast<float*>(scratch), iters);
            else mfma_rate16_kernel<true><<<dim3(cus), 512, 0, s>>>(static_cast<float*>(scratch), iters);
            LOKA_HIP_TRY(hipEventRecord(e1, s));
            LOKA_HIP_TRY(hipEventSynchronize(e1));
            LOKA_HIP_TRY(hipEventElapsedTime(&ms, e0, e1));
            total += ms;
            last = flops / (ms * 1e-3) / 1e12;
        }
    } else if (kind == 0 || kind == 1 || kind == 4 || kind == 5) {
        const int iters = 4096;
        // per launch: CUs x 8 waves x iters x 8 MFMAs of 2 * 32 * 32 * K flops
        const double flops = static_cast<double>(cus) * 8 * iters * 8 * 2.0 * 32 * 32 * ((kind == 0 || kind == 4) ? 64 : 16);
        while (total < millis) {
            LOKA_HIP_TRY(hipEventRecord(e0, s));
            if (kind == 0) mfma_rate_kernel<false, false><<<dim3(cus), 512, 0, s>>>(static_cast<float*>(scratch), iters);
            else if (kind == 1) mfma_rate_kernel<true, false><<<dim3(cus), 512, 0, s>>>(static_cast<float*>(scratch), iters);
            else if (kind == 4) mfma_rate_kernel<false, true><<<dim3(cus), 512, 0, s>>>(static_cast<float*>(scratch), iters);
            else mfma_rate_kernel<true, true><<<dim3(cus), 512, 0, s>>>(static_cast<float*>(scratch), iters);
            LOKA_HIP_TRY(hipEventRecord(e1, s));
            LOKA_HIP_TRY(hipEventSynchronize(e1));
            LOKA_HIP_TRY(hipEventElapsedTime(&ms, e0, e1));
            total += ms;
            last = flops / (ms * 1e-3) / 1e12;
        }
    } else if (kind == 3) {
        // X 32768 x 4096 bytes (128 panels of 256 rows), W 4096 x 4096 (16 tiles), 32 K steps per tile, 2048 tiles
        const int kb_row = 4096, tiles_m = 128, tiles_n = 16;
        const size_t need = static_cast<size_t>(tiles_m + tiles_n) * 256 * kb_row;
        if (scratch_bytes < need) return LOKA_ERR_WORKSPACE;
        LOKA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&lds_stream_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 5 * 32768));
        const uint8_t* x = static_cast<const uint8_t*>(scratch);
        const uint8_t* w = x + static_cast<size_t>(tiles_m) * 256 * kb_row;
        const int grid = (cus / tiles_n) * tiles_n;           // whole panels side by side, as the kernel launches
        if (grid <= 0) return LOKA_ERR_UNSUPPORTED;
        const double bytes = static_cast<double>(tiles_m) * tiles_n * (kb_row / 128) * 65536.0;
        while (total < millis) {
            LOKA_HIP_TRY(hipEventRecord(e0, s));
            lds_stream_kernel<<<dim3(grid), 512, 5 * 32768, s>>>(x, w, kb_row, tiles_n, tiles_m * tiles_n, nullptr);
            LOKA_HIP_TRY(hipEventRecord(e1, s));
            LOKA_HIP_TRY(hipEventSynchronize(e1));
            LOKA_HIP_TRY(hipEventElapsedTime(&ms, e0, e1));
            total += ms;
            last = bytes / (ms * 1e-3) / 1e9;
        }
    } else {
        const int64_t n16 = static_cast<int64_t>(scratch_bytes / 2 / 16);
        const u32x4* src = static_cast<const u32x4*>(scratch);
        u32x4* dst = static_cast<u32x4*>(scratch) + n16;
        while (total < millis) {
            LOKA_HIP_TRY(hipEventRecord(e0, s));
            copy_kernel<<<dim3(cus * 16), 256, 0, s>>>(src, dst, n16);
            LOKA_HIP_TRY(hipEventRecord(e1, s));
            LOKA_HIP_TRY(hipEventSynchronize(e1));
            LOKA_HIP_TRY(hipEventElapsedTime(&ms, e0, e1));
            total += ms;
            last = 2.0 * n16 * 16 / (ms * 1e-3) / 1e9;
        }
    }
    *value = last;
    return LOKA_OK;
}

}  // namespace loka
