// C ABI of the library: argument validation (host only, before any HIP call) and
// forwarding to the kernel launchers.  See include/loka.h for the contract.
#include "common.h"

#include <cstdlib>
#include <cstring>
#include <mutex>

namespace loka {
// quantize.hip
loka_status quantize_launch(const void*, int64_t, int64_t, int64_t, loka_scale_mode, int, uint8_t*, float*, void*,
                            hipStream_t);
loka_status e4m3_from_f32_launch(const float*, uint8_t*, int64_t, hipStream_t);
// gemm.hip
int variant_count();
const char* variant_name(int);
bool variant_supports(const loka_gemm_desc*, int);
size_t variant_workspace(const loka_gemm_desc*, int, bool fp8out = false);
loka_status fp8_gemm_norm_launch(const loka_gemm_desc*, int, const uint8_t*, const float*, const uint8_t*, const float*,
                                 const void*, const void*, void*, float*, uint8_t*, float*, void*, hipStream_t);
int variant_streaming_id();
bool variant_is_streaming(int);
bool variant_is_strip(int);
bool variant_is_panel32(int);
bool variant_supports_fused(const loka_gemm_desc*, int);
bool variant_supports_xq(const loka_gemm_desc*, int);
int variant_xq_default(const loka_gemm_desc*);
loka_status fp8_linear_norm_xq_launch(const loka_gemm_desc*, int, const void*, uint8_t*, float*, const uint8_t*, const float*,
                                      const void*, const void*, void*, float*, hipStream_t);
int variant_fused_default(const loka_gemm_desc*);
loka_status fp8_linear_norm_launch(const loka_gemm_desc*, int, const void*, const uint8_t*, const float*, const void*,
                                   const void*, void*, float*, float*, hipStream_t);
bool variant_has_wait_flag(const loka_gemm_desc*, int, bool fp8out = false);
void test_set_spin_limit(long long);
// ceiling.hip
loka_status machine_ceiling(int, double, void*, size_t, double*, hipStream_t);
size_t bf16_gemm_workspace_bytes(const loka_gemm_desc*);
loka_status bf16_gemm_launch(const loka_gemm_desc*, const void*, const void*, float*, void*, hipStream_t, bool weights_ready = false);
// probe.hip
size_t probe_workspace_bytes();
loka_status probe_launch(const float*, const float*, int64_t, int64_t, int64_t, loka_probe_stats*, float*, void*,
                         hipStream_t);
// dispatch.hip
int default_variant(const loka_gemm_desc*);
// tracker.hip
size_t tracker_workspace_bytes(int64_t, int64_t);
loka_status tracker_update_launch(const void*, int64_t, int64_t, int64_t, int64_t, float*, float*, void*, hipStream_t);

static bool mode_ok(int m) { return m >= LOKA_SCALE_TENSOR && m <= LOKA_SCALE_BLOCK_128x128_POW2; }       // modes a GEMM operand can have
static bool quant_mode_ok(int m) { return m >= LOKA_SCALE_TENSOR && m <= LOKA_SCALE_BLOCK_128x1; }
static bool is_block_x(int m) { return m == LOKA_SCALE_BLOCK_1x128 || m == LOKA_SCALE_BLOCK_1x128_POW2; }
static bool is_block_w(int m) { return m == LOKA_SCALE_BLOCK_128x128 || m == LOKA_SCALE_BLOCK_128x128_POW2; }

// Shape / enum validation shared by the GEMM entry points; does not look at pointers.
loka_status validate_desc(const loka_gemm_desc* d, bool fp8) {
    if (!d) return LOKA_ERR_NULL;
    if (d->M <= 0 || d->N <= 0 || d->K <= 0 || d->batch <= 0) return LOKA_ERR_SHAPE;
    if (d->M > INT32_MAX || d->N > INT32_MAX || d->K > INT32_MAX / 2 || d->batch > INT32_MAX) return LOKA_ERR_SHAPE;
    if (d->N % 16) return LOKA_ERR_SHAPE;
    if (fp8 ? (d->K % 16) : (d->K % 8)) return LOKA_ERR_SHAPE;
    if (d->strideX < 0 || d->strideW < 0 || d->strideO < 0) return LOKA_ERR_SHAPE;
    if (d->batch > 1 && d->strideO < d->M * d->N) return LOKA_ERR_SHAPE;
    if ((d->strideX % 16) || (d->strideW % 16) || (d->strideO % 8)) return LOKA_ERR_ALIGN;
    if (!fp8) return LOKA_OK;
    if (!mode_ok(d->x_mode) || !mode_ok(d->w_mode)) return LOKA_ERR_UNSUPPORTED;
    if (d->norm < LOKA_NORM_NONE || d->norm > LOKA_NORM_BLOCKNORM) return LOKA_ERR_UNSUPPORTED;
    if (d->act < LOKA_ACT_NONE || d->act > LOKA_ACT_HARDSWISH) return LOKA_ERR_UNSUPPORTED;
    if (d->act != LOKA_ACT_NONE && d->norm != LOKA_NORM_BLOCKNORM) return LOKA_ERR_UNSUPPORTED;
    if (d->norm == LOKA_NORM_BLOCKNORM) {
        if (d->block_n <= 0 || d->N % d->block_n) return LOKA_ERR_SHAPE;
        if (d->block_n != 256) return LOKA_ERR_UNSUPPORTED;
    }
    const bool xb = is_block_x(d->x_mode), wb = is_block_w(d->w_mode);
    if (xb != wb) return LOKA_ERR_UNSUPPORTED;
    // (power-of-two scales on both operands or on neither: the scaled matrix instruction takes both)
    if ((d->x_mode == LOKA_SCALE_BLOCK_1x128_POW2) != (d->w_mode == LOKA_SCALE_BLOCK_128x128_POW2)) return LOKA_ERR_UNSUPPORTED;
    if (xb && (d->N % 128 || d->K % 128)) return LOKA_ERR_SHAPE;
    if (!xb) {
        if (!(d->x_mode == LOKA_SCALE_TENSOR || d->x_mode == LOKA_SCALE_ROW)) return LOKA_ERR_UNSUPPORTED;
        if (!(d->w_mode == LOKA_SCALE_TENSOR || d->w_mode == LOKA_SCALE_COL)) return LOKA_ERR_UNSUPPORTED;
    }
    if (!(d->eps >= 0.f)) return LOKA_ERR_UNSUPPORTED;
    return LOKA_OK;
}

int resolve_variant(const loka_gemm_desc* d) {
    if (d->variant >= 0) return variant_supports(d, d->variant) ? d->variant : -1;
    return default_variant(d);
}

}  // namespace loka

using namespace loka;

extern "C" {

const char* loka_status_string(loka_status s) {
    switch (s) {
        case LOKA_OK: return "ok";
        case LOKA_ERR_NULL: return "null pointer";
        case LOKA_ERR_SHAPE: return "bad shape";
        case LOKA_ERR_ALIGN: return "misaligned pointer or stride";
        case LOKA_ERR_UNSUPPORTED: return "unsupported combination";
        case LOKA_ERR_WORKSPACE: return "workspace missing or too small";
        case LOKA_ERR_HIP: return "HIP runtime error";
        case LOKA_ERR_NO_CANDIDATE: return "no FP8 candidate within the error budget";
        case LOKA_ERR_TIMEOUT: return "a bounded wait inside the launch ran out";
    }
    return "unknown status";
}

int64_t loka_scale_count(loka_scale_mode mode, int64_t rows, int64_t cols) {
    if (rows <= 0 || cols <= 0) return -1;
    switch (mode) {
        case LOKA_SCALE_TENSOR: return 1;
        case LOKA_SCALE_ROW: return rows;
        case LOKA_SCALE_COL: return cols;
        case LOKA_SCALE_BLOCK_1x128:
        case LOKA_SCALE_BLOCK_1x128_POW2: return (cols % 128) ? -1 : rows * (cols / 128);
        case LOKA_SCALE_BLOCK_128x128:
        case LOKA_SCALE_BLOCK_128x128_POW2: return (cols % 128 || rows % 128) ? -1 : (rows / 128) * (cols / 128);
        case LOKA_SCALE_BLOCK_128x1: return (rows % 128) ? -1 : (rows / 128) * cols;
    }
    return -1;
}

size_t loka_quantize_workspace(loka_scale_mode mode, int64_t rows, int64_t cols, int transpose_out) {
    if (!transpose_out && (mode == LOKA_SCALE_ROW || is_block_x(mode))) return 0;
    if (is_block_w(mode) || mode == LOKA_SCALE_BLOCK_128x1) return 0;      // groups that fit a workgroup: one pass
    const int64_t ng = loka_scale_count(mode, rows, cols);
    if (ng < 0) return 0;
    return static_cast<size_t>(ng) * 8;       // amax bits + quantization factors
}

loka_status loka_quantize(const void* x_bf16, int64_t rows, int64_t cols, int64_t ld, loka_scale_mode mode,
                          int transpose_out, uint8_t* q, float* scales, void* workspace, size_t ws_bytes,
                          void* hip_stream) {
    if (!x_bf16 || !q || !scales) return LOKA_ERR_NULL;
    if (!quant_mode_ok(mode)) return LOKA_ERR_UNSUPPORTED;
    if (rows <= 0 || cols <= 0 || ld < cols) return LOKA_ERR_SHAPE;
    if (cols % 16 || (transpose_out && rows % 16)) return LOKA_ERR_SHAPE;
    if (loka_scale_count(mode, rows, cols) < 0) return LOKA_ERR_SHAPE;
    if (ld % 8) return LOKA_ERR_ALIGN;
    if (!aligned16(x_bf16) || !aligned16(q) || (reinterpret_cast<uintptr_t>(scales) & 3u)) return LOKA_ERR_ALIGN;
    if (transpose_out && (mode == LOKA_SCALE_ROW || is_block_x(mode))) return LOKA_ERR_UNSUPPORTED;
    if (!transpose_out && mode == LOKA_SCALE_BLOCK_128x1) return LOKA_ERR_UNSUPPORTED;
    const size_t need = loka_quantize_workspace(mode, rows, cols, transpose_out);
    if (need && (!workspace || ws_bytes < need)) return LOKA_ERR_WORKSPACE;
    if (need && !aligned16(workspace)) return LOKA_ERR_ALIGN;
    return quantize_launch(x_bf16, rows, cols, ld, mode, transpose_out, q, scales, workspace,
                           static_cast<hipStream_t>(hip_stream));
}

loka_status loka_e4m3_from_f32(const float* t, uint8_t* codes, int64_t n, void* hip_stream) {
    if (!t || !codes) return LOKA_ERR_NULL;
    if (n <= 0) return LOKA_ERR_SHAPE;
    return e4m3_from_f32_launch(t, codes, n, static_cast<hipStream_t>(hip_stream));
}

int loka_variant_count(void) { return variant_count(); }
const char* loka_variant_name(int variant) { return variant_name(variant); }

int loka_variant_supports(const loka_gemm_desc* desc, int variant) {
    if (validate_desc(desc, true) != LOKA_OK) return 0;
    return variant_supports(desc, variant) ? 1 : 0;
}

// ---- loka_fp8_gemm_norm_static: the scratch of loka_fp8_gemm_norm in library-owned device memory.
// `static_scratch` is a host-side stand-in for a device array: its device address is asked from the runtime once per
// device (with that device current) and only that address is ever handed to kernels or copies.
constexpr size_t kStaticScratchBytes = LOKA_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char static_scratch[kStaticScratchBytes];
namespace {
constexpr int kScratchMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kScratchMaxDevices] = {};
}  // namespace

// Device address of the current device's copy of the array (set-up on the first call per device).
static loka_status static_scratch_address(void** ptr) {
    int dev = 0;
    LOKA_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kScratchMaxDevices) return LOKA_ERR_HIP;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        LOKA_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(static_scratch)));
        if (!p) return LOKA_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return LOKA_OK;
}

loka_status loka_fp8_gemm_norm_static(const loka_gemm_desc* desc, const uint8_t* xq, const float* sx, const uint8_t* wq,
                                      const float* sw, const void* gamma_bf16, const void* beta_bf16, void* out_bf16,
                                      float* y_fp32, void* hip_stream) {
    if (!desc || !xq || !sx || !wq || !sw || !out_bf16) return LOKA_ERR_NULL;
    const loka_status st = validate_desc(desc, true);
    if (st != LOKA_OK) return st;
    if (!aligned16(xq) || !aligned16(wq) || !aligned16(sx) || !aligned16(sw) || !aligned16(out_bf16) ||
        !aligned16(y_fp32) || !aligned16(gamma_bf16) || !aligned16(beta_bf16))
        return LOKA_ERR_ALIGN;
    const int v = resolve_variant(desc);
    if (v < 0) return LOKA_ERR_UNSUPPORTED;
    const size_t need = variant_workspace(desc, v);
    if (need > kStaticScratchBytes) return LOKA_ERR_WORKSPACE;      // beyond the array: use loka_fp8_gemm_norm with a workspace
    void* ws = nullptr;
    if (need) {
        const loka_status sa = static_scratch_address(&ws);
        if (sa != LOKA_OK) return sa;
    }
    return fp8_gemm_norm_launch(desc, v, xq, sx, wq, sw, gamma_bf16, beta_bf16, out_bf16, y_fp32, nullptr, nullptr, ws,
                                static_cast<hipStream_t>(hip_stream));
}

size_t loka_fp8_gemm_norm_workspace(const loka_gemm_desc* desc) {
    if (validate_desc(desc, true) != LOKA_OK) return 0;
    const int v = resolve_variant(desc);
    return v < 0 ? 0 : variant_workspace(desc, v);
}

loka_status loka_fp8_gemm_norm(const loka_gemm_desc* desc, const uint8_t* xq, const float* sx, const uint8_t* wq,
                               const float* sw, const void* gamma_bf16, const void* beta_bf16, void* out_bf16,
                               float* y_fp32, void* workspace, size_t ws_bytes, void* hip_stream) {
    if (!desc || !xq || !sx || !wq || !sw || !out_bf16) return LOKA_ERR_NULL;
    const loka_status st = validate_desc(desc, true);
    if (st != LOKA_OK) return st;
    if (!aligned16(xq) || !aligned16(wq) || !aligned16(sx) || !aligned16(sw) || !aligned16(out_bf16) ||
        !aligned16(y_fp32) || !aligned16(gamma_bf16) || !aligned16(beta_bf16))
        return LOKA_ERR_ALIGN;
    const int v = resolve_variant(desc);
    if (v < 0) return LOKA_ERR_UNSUPPORTED;
    const size_t need = variant_workspace(desc, v);
    if (need && (!workspace || ws_bytes < need)) return LOKA_ERR_WORKSPACE;
    if (need && !aligned16(workspace)) return LOKA_ERR_ALIGN;
    return fp8_gemm_norm_launch(desc, v, xq, sx, wq, sw, gamma_bf16, beta_bf16, out_bf16, y_fp32, nullptr, nullptr,
                                workspace, static_cast<hipStream_t>(hip_stream));
}

loka_status loka_fp8_linear_norm(const loka_gemm_desc* desc, const void* x_bf16, const uint8_t* wq, const float* sw,
                                 const void* gamma_bf16, const void* beta_bf16, void* out_bf16, float* y_fp32,
                                 float* sx_out, void* hip_stream) {
    if (!desc || !x_bf16 || !wq || !sw || !out_bf16) return LOKA_ERR_NULL;
    const loka_status st = validate_desc(desc, true);
    if (st != LOKA_OK) return st;
    if (desc->x_mode != LOKA_SCALE_ROW) return LOKA_ERR_UNSUPPORTED;
    if (!aligned16(x_bf16) || !aligned16(wq) || !aligned16(sw) || !aligned16(out_bf16) || !aligned16(y_fp32) ||
        !aligned16(gamma_bf16) || !aligned16(beta_bf16) || !aligned16(sx_out))
        return LOKA_ERR_ALIGN;
    // kernels that keep whole rows of X in one workgroup (strip32, wreg32): the row amax needs no second pass
    const int v = desc->variant >= 0 ? desc->variant : variant_fused_default(desc);
    if (v < 0 || !variant_supports_fused(desc, v)) return LOKA_ERR_UNSUPPORTED;
    return fp8_linear_norm_launch(desc, v, x_bf16, wq, sw, gamma_bf16, beta_bf16, out_bf16, y_fp32, sx_out,
                                  static_cast<hipStream_t>(hip_stream));
}

loka_status loka_fp8_linear_norm_xq(const loka_gemm_desc* desc, const void* x_bf16, uint8_t* xq_out, float* sx_out,
                                    const uint8_t* wq, const float* sw, const void* gamma_bf16, const void* beta_bf16,
                                    void* out_bf16, float* y_fp32, void* hip_stream) {
    if (!desc || !x_bf16 || !xq_out || !sx_out || !wq || !sw || !out_bf16) return LOKA_ERR_NULL;
    const loka_status st = validate_desc(desc, true);
    if (st != LOKA_OK) return st;
    if (desc->x_mode != LOKA_SCALE_ROW) return LOKA_ERR_UNSUPPORTED;
    if (!aligned16(x_bf16) || !aligned16(xq_out) || !aligned16(sx_out) || !aligned16(wq) || !aligned16(sw) ||
        !aligned16(out_bf16) || !aligned16(y_fp32) || !aligned16(gamma_bf16) || !aligned16(beta_bf16))
        return LOKA_ERR_ALIGN;
    const int v = desc->variant >= 0 ? desc->variant : variant_xq_default(desc);
    if (v < 0 || !variant_supports_xq(desc, v)) return LOKA_ERR_UNSUPPORTED;
    return fp8_linear_norm_xq_launch(desc, v, x_bf16, xq_out, sx_out, wq, sw, gamma_bf16, beta_bf16, out_bf16, y_fp32,
                                     static_cast<hipStream_t>(hip_stream));
}

// The kernels with an FP8-output epilogue: the two that keep a whole output row inside one workgroup (streaming) or
// one wave (strip), and the large-layer panel kernel (which sends the row extremes along with the row statistics).
// The one the caller names, else the library's choice for the shape when it is one of the three, else the
// streaming one where it can run the shape, else the panel kernel.  -1 when the named variant has no such epilogue
// or cannot run the shape.
static int fp8out_variant(const loka_gemm_desc* desc) {
    auto usable = [&](int v) {
        return v >= 0 && (variant_is_streaming(v) || variant_is_strip(v) || variant_is_panel32(v)) && variant_supports(desc, v);
    };
    if (desc->variant >= 0) return usable(desc->variant) ? desc->variant : -1;
    const int v = default_variant(desc);
    if (usable(v)) return v;
    if (usable(variant_streaming_id())) return variant_streaming_id();
    for (int u = 0; u < variant_count(); ++u)             // the panel kernel takes every shape the two others do not
        if (variant_is_panel32(u) && usable(u)) return u;
    return -1;
}

loka_status loka_fp8_gemm_norm_check(const loka_gemm_desc* desc, const void* workspace, size_t ws_bytes, void* hip_stream) {
    if (!desc) return LOKA_ERR_NULL;
    const loka_status st = validate_desc(desc, true);
    if (st != LOKA_OK) return st;
    // the variant loka_fp8_gemm_norm runs for desc, or (desc->variant < 0 only: the two choices can differ) the one
    // loka_fp8_gemm_norm_fp8out runs; every workspace with a bounded wait begins with the flag
    int v = resolve_variant(desc);
    bool q = false;
    if (v < 0 || !variant_has_wait_flag(desc, v)) {
        const int vq = fp8out_variant(desc);
        if (vq >= 0 && variant_has_wait_flag(desc, vq, true)) { v = vq; q = true; }
    }
    if (v < 0) return LOKA_ERR_UNSUPPORTED;
    if (!variant_has_wait_flag(desc, v, q)) return LOKA_OK;
    if (!workspace || ws_bytes < variant_workspace(desc, v, q)) return LOKA_ERR_WORKSPACE;
    // header of the workspace: [0] the nonce of the last launch that used it, [1] the nonce of the last launch in
    // which a wait ran out (0 in both: never used)
    unsigned long long hdr[2] = {0, 0};
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    LOKA_HIP_TRY(hipMemcpyAsync(hdr, workspace, sizeof(hdr), hipMemcpyDeviceToHost, s));
    LOKA_HIP_TRY(hipStreamSynchronize(s));
    return (hdr[0] != 0 && hdr[0] == hdr[1]) ? LOKA_ERR_TIMEOUT : LOKA_OK;
}

void loka_test_set_spin_limit(int64_t polls) { test_set_spin_limit(polls); }

loka_status loka_machine_ceiling(int kind, double millis, void* scratch, size_t scratch_bytes, double* value_host,
                                 void* hip_stream) {
    if (!scratch || !value_host) return LOKA_ERR_NULL;
    if (kind < 0 || kind > 7 || !(millis > 0.0)) return LOKA_ERR_UNSUPPORTED;
    if (!aligned16(scratch)) return LOKA_ERR_ALIGN;
    if (scratch_bytes < (size_t(1) << 22) || (kind == 2 && scratch_bytes < (size_t(1) << 26))) return LOKA_ERR_WORKSPACE;
    return machine_ceiling(kind, millis, scratch, scratch_bytes, value_host, static_cast<hipStream_t>(hip_stream));
}

size_t loka_fp8_gemm_norm_fp8out_workspace(const loka_gemm_desc* desc) {
    if (validate_desc(desc, true) != LOKA_OK) return 0;
    const int v = fp8out_variant(desc);
    return v < 0 ? 0 : variant_workspace(desc, v, true);
}

loka_status loka_fp8_gemm_norm_fp8out(const loka_gemm_desc* desc, const uint8_t* xq, const float* sx, const uint8_t* wq,
                                      const float* sw, const void* gamma_bf16, const void* beta_bf16, uint8_t* oq,
                                      float* so, float* y_fp32, void* workspace, size_t ws_bytes, void* hip_stream) {
    if (!desc || !xq || !sx || !wq || !sw || !oq || !so) return LOKA_ERR_NULL;
    const loka_status st = validate_desc(desc, true);
    if (st != LOKA_OK) return st;
    if (!aligned16(xq) || !aligned16(wq) || !aligned16(sx) || !aligned16(sw) || !aligned16(oq) || !aligned16(so) ||
        !aligned16(y_fp32) || !aligned16(gamma_bf16) || !aligned16(beta_bf16))
        return LOKA_ERR_ALIGN;
    const int v = fp8out_variant(desc);
    if (v < 0) return LOKA_ERR_UNSUPPORTED;
    const size_t need = variant_workspace(desc, v, true);
    if (need && (!workspace || ws_bytes < need)) return LOKA_ERR_WORKSPACE;
    if (need && !aligned16(workspace)) return LOKA_ERR_ALIGN;
    return fp8_gemm_norm_launch(desc, v, xq, sx, wq, sw, gamma_bf16, beta_bf16, nullptr, y_fp32, oq, so, workspace,
                                static_cast<hipStream_t>(hip_stream));
}

size_t loka_bf16_gemm_workspace(const loka_gemm_desc* desc) {
    if (validate_desc(desc, false) != LOKA_OK) return 0;
    return bf16_gemm_workspace_bytes(desc);
}

loka_status loka_bf16_gemm(const loka_gemm_desc* desc, const void* x_bf16, const void* w_bf16, float* yref_fp32,
                           void* workspace, size_t ws_bytes, void* hip_stream) {
    if (!desc || !x_bf16 || !w_bf16 || !yref_fp32) return LOKA_ERR_NULL;
    const loka_status st = validate_desc(desc, false);
    if (st != LOKA_OK) return st;
    if (!aligned16(x_bf16) || !aligned16(w_bf16) || !aligned16(yref_fp32)) return LOKA_ERR_ALIGN;
    const size_t need = bf16_gemm_workspace_bytes(desc);
    if (!workspace || ws_bytes < need) return LOKA_ERR_WORKSPACE;
    if (!aligned16(workspace)) return LOKA_ERR_ALIGN;
    return bf16_gemm_launch(desc, x_bf16, w_bf16, yref_fp32, workspace, static_cast<hipStream_t>(hip_stream));
}

size_t loka_probe_error_workspace(int64_t M, int64_t N) {
    (void)M; (void)N;
    return probe_workspace_bytes();
}

loka_status loka_probe_error(const float* y, const float* yref, int64_t M, int64_t N, int64_t ld,
                             loka_probe_stats* stats_device, float* rowmax_device, void* workspace, size_t ws_bytes,
                             void* hip_stream) {
    if (!y || !yref || !stats_device) return LOKA_ERR_NULL;
    if (M <= 0 || N <= 0 || ld < N) return LOKA_ERR_SHAPE;
    if (N % 4 || ld % 4) return LOKA_ERR_SHAPE;
    if (!aligned16(y) || !aligned16(yref) || (reinterpret_cast<uintptr_t>(stats_device) & 7u)) return LOKA_ERR_ALIGN;
    if (!workspace || ws_bytes < probe_workspace_bytes()) return LOKA_ERR_WORKSPACE;
    if (!aligned16(workspace)) return LOKA_ERR_ALIGN;
    return probe_launch(y, yref, M, N, ld, stats_device, rowmax_device, workspace,
                        static_cast<hipStream_t>(hip_stream));
}

// Shape rules of the tracker, shared by the workspace query and the call.
static loka_status validate_tracker(int64_t B, int64_t K, int64_t ld, int64_t n_old) {
    if (B <= 0 || K <= 0 || ld < K || n_old < 0) return LOKA_ERR_SHAPE;
    if (K % 8 || ld % 8) return LOKA_ERR_SHAPE;
    if (K > 32768 || B > (INT64_C(1) << 40) || n_old > (INT64_C(1) << 52)) return LOKA_ERR_SHAPE;
    return LOKA_OK;
}

size_t loka_tracker_update_workspace(int64_t B, int64_t K) {
    if (validate_tracker(B, K, K, 0) != LOKA_OK) return 0;
    return tracker_workspace_bytes(B, K);
}

loka_status loka_tracker_update(const void* x_bf16, int64_t B, int64_t K, int64_t ld, int64_t n_old, float* mu,
                                float* sigma, void* workspace, size_t ws_bytes, void* hip_stream) {
    if (!x_bf16 || !mu || !sigma) return LOKA_ERR_NULL;
    const loka_status st = validate_tracker(B, K, ld, n_old);
    if (st != LOKA_OK) return st;
    if (!aligned16(x_bf16) || !aligned16(mu) || !aligned16(sigma)) return LOKA_ERR_ALIGN;
    if (!workspace || ws_bytes < tracker_workspace_bytes(B, K)) return LOKA_ERR_WORKSPACE;
    if (!aligned16(workspace)) return LOKA_ERR_ALIGN;
    return tracker_update_launch(x_bf16, B, K, ld, n_old, mu, sigma, workspace, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
