// Probe error statistics of Y against Yref: a streaming reduction (8 B read per
// element pair, bandwidth bound).  Row maxima are exact; the sums are accumulated in
// fp64 per lane, reduced per workgroup, and combined by one workgroup in a fixed
// order, so repeated runs give identical bits.
#include "common.h"

namespace loka {

constexpr int kProbeBlocks = 2048;   // persistent grid: partial sums per workgroup

struct ProbePartial {
    double sse, ssr, rel;
    float mx;
    float pad;
};

__device__ __forceinline__ double wave_sum_f64(double v) {
    for (int m = 1; m < 64; m <<= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// TPR lanes per row (16, 32 or 64), float4 chunks, UNR chunk loads in flight per array.
template <int TPR, int UNR>
__global__ __launch_bounds__(256) void probe_kernel(const float* __restrict__ y, const float* __restrict__ yref,
                                                    int64_t M, int64_t N, int64_t ld, float* __restrict__ rowmax,
                                                    ProbePartial* __restrict__ partials) {
    __shared__ ProbePartial red[4];
    constexpr int RPW = 64 / TPR;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lr = lane % TPR, sub = lane / TPR;
    const int64_t chunks = N >> 2;
    const int64_t wave_id = static_cast<int64_t>(blockIdx.x) * 4 + wave;
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * 4;
    double sse = 0.0, ssr = 0.0, rel = 0.0;
    float gmax = 0.f;
    for (int64_t rb = wave_id * RPW; rb < M; rb += n_waves * RPW) {
        const int64_t r = rb + sub;
        float rm = 0.f;
        if (r < M) {
            const float* yr = y + r * ld;
            const float* fr = yref + r * ld;
            for (int64_t c0 = lr; c0 < chunks; c0 += static_cast<int64_t>(TPR) * UNR) {
                v4f a[UNR], b[UNR];
#pragma unroll
                for (int u = 0; u < UNR; ++u) {
                    const int64_t c = c0 + static_cast<int64_t>(u) * TPR;
                    if (c < chunks) {
                        a[u] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(yr + c * 4));
                        b[u] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(fr + c * 4));
                    } else {
                        a[u] = v4f{0.f, 0.f, 0.f, 0.f};
                        b[u] = v4f{0.f, 0.f, 0.f, 0.f};
                    }
                }
#pragma unroll
                for (int u = 0; u < UNR; ++u) {
                    const bool ok = (c0 + static_cast<int64_t>(u) * TPR) < chunks;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float d = a[u][e] - b[u][e];
                        const float ad = fabsf(d);
                        rm = fmaxf(rm, ad);
                        const double dd = static_cast<double>(d), rr = static_cast<double>(b[u][e]);
                        sse = fma(dd, dd, sse);
                        ssr = fma(rr, rr, ssr);
                        // |d| / max(|ref|, 1e-30): fp32 reciprocal (1 ulp), accumulated in fp64
                        const float den = fmaxf(fabsf(b[u][e]), 1e-30f);
                        if (ok) rel += static_cast<double>(ad * __builtin_amdgcn_rcpf(den));
                    }
                }
            }
        }
        for (int m = 1; m < TPR; m <<= 1) rm = fmaxf(rm, wave_shfl_xor(rm, m));
        if (r < M && lr == 0 && rowmax) rowmax[r] = rm;
        gmax = fmaxf(gmax, rm);
    }
    sse = wave_sum_f64(sse);
    ssr = wave_sum_f64(ssr);
    rel = wave_sum_f64(rel);
    for (int m = 1; m < 64; m <<= 1) gmax = fmaxf(gmax, wave_shfl_xor(gmax, m));
    if (lane == 0) {
        red[wave].sse = sse; red[wave].ssr = ssr; red[wave].rel = rel; red[wave].mx = gmax;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        ProbePartial p = red[0];
        for (int w = 1; w < 4; ++w) {
            p.sse += red[w].sse; p.ssr += red[w].ssr; p.rel += red[w].rel; p.mx = fmaxf(p.mx, red[w].mx);
        }
        p.pad = 0.f;
        partials[blockIdx.x] = p;
    }
}

// One workgroup; thread t sums partials t, t+256, ... in order, then a fixed tree.
__global__ __launch_bounds__(256) void probe_finalize_kernel(const ProbePartial* __restrict__ partials, int n,
                                                             int64_t M, int64_t N,
                                                             loka_probe_stats* __restrict__ stats) {
    __shared__ double s0[256], s1[256], s2[256];
    __shared__ float s3[256];
    double sse = 0.0, ssr = 0.0, rel = 0.0;
    float mx = 0.f;
    for (int i = threadIdx.x; i < n; i += 256) {
        sse += partials[i].sse; ssr += partials[i].ssr; rel += partials[i].rel; mx = fmaxf(mx, partials[i].mx);
    }
    s0[threadIdx.x] = sse; s1[threadIdx.x] = ssr; s2[threadIdx.x] = rel; s3[threadIdx.x] = mx;
    __syncthreads();
    for (unsigned w = 128; w > 0; w >>= 1) {
        if (threadIdx.x < w) {
            s0[threadIdx.x] += s0[threadIdx.x + w];
            s1[threadIdx.x] += s1[threadIdx.x + w];
            s2[threadIdx.x] += s2[threadIdx.x + w];
            s3[threadIdx.x] = fmaxf(s3[threadIdx.x], s3[threadIdx.x + w]);
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const double e = s0[0], r = s1[0];
        stats->sum_sq_err = e;
        stats->sum_sq_ref = r;
        stats->rel_fro = r > 0.0 ? sqrt(e) / sqrt(r) : (e > 0.0 ? __builtin_inf() : 0.0);
        stats->max_abs = static_cast<double>(s3[0]);
        stats->mere = s2[0] / (static_cast<double>(M) * static_cast<double>(N));
    }
}

size_t probe_workspace_bytes() { return sizeof(ProbePartial) * kProbeBlocks; }

loka_status probe_launch(const float* y, const float* yref, int64_t M, int64_t N, int64_t ld,
                         loka_probe_stats* stats, float* rowmax, void* workspace, hipStream_t s) {
    ProbePartial* partials = static_cast<ProbePartial*>(workspace);
    const int64_t chunks = N / 4;
    int blocks;
    auto nblocks = [&](int rpw) {
        int64_t waves = (M + rpw - 1) / rpw;
        int64_t b = (waves + 3) / 4;
        return static_cast<int>(b < kProbeBlocks ? b : kProbeBlocks);
    };
    if (chunks <= 16) {
        blocks = nblocks(4);
        probe_kernel<16, 1><<<blocks, 256, 0, s>>>(y, yref, M, N, ld, rowmax, partials);
    } else if (chunks <= 32) {
        blocks = nblocks(2);
        probe_kernel<32, 1><<<blocks, 256, 0, s>>>(y, yref, M, N, ld, rowmax, partials);
    } else if (chunks <= 128) {
        blocks = nblocks(1);
        probe_kernel<64, 2><<<blocks, 256, 0, s>>>(y, yref, M, N, ld, rowmax, partials);
    } else {
        blocks = nblocks(1);
        probe_kernel<64, 4><<<blocks, 256, 0, s>>>(y, yref, M, N, ld, rowmax, partials);
    }
    probe_finalize_kernel<<<1, 256, 0, s>>>(partials, blocks, M, N, stats);
    return hipGetLastError() == hipSuccess ? LOKA_OK : LOKA_ERR_HIP;
}

}  // namespace loka
