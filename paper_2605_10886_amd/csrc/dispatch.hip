// Per-shape dispatch: profile the library's own candidates (scale recipe x kernel
// variant) on sample operands, keep those within the error budget and above the
// speedup floor, take the fastest, remember the answer per shape.
#include "common.h"

#include <cstdio>
#include <cstdlib>
#include <map>
#include <mutex>
#include <tuple>
#include <vector>

namespace loka {

int variant_count();
const char* variant_name(int);
bool variant_supports(const loka_gemm_desc*, int);
int variant_epilogue(int);
bool variant_is_streaming(int);
bool variant_is_strip(int);
bool variant_is_exact(int);
int variant_bn(int);
int variant_splitk_choice(const loka_gemm_desc*);
int variant_bm(int);
loka_status validate_desc(const loka_gemm_desc* d, bool fp8);
loka_status bf16_gemm_launch(const loka_gemm_desc*, const void*, const void*, float*, void*, hipStream_t, bool weights_ready);

namespace {

// what a profiled choice depends on besides the shape: the epilogue (norm, group width, activation), whether the
// problems of a grouped launch share one weight, and the device it was measured on
using Epilogue = std::tuple<int, int, int, int, int>;                                    // norm block_n act shared_w device
using ShapeKey = std::tuple<int64_t, int64_t, int64_t, int64_t, Epilogue, double, double>;   // M N K batch epilogue budget floor
using RecipeKey = std::tuple<int64_t, int64_t, int64_t, int64_t, Epilogue, int, int>;        // M N K batch epilogue x_mode w_mode

Epilogue epilogue_of(const loka_gemm_desc* d) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) dev = -1;          // (no device: host-only queries still get an answer)
    return Epilogue(d->norm, d->norm == LOKA_NORM_BLOCKNORM ? d->block_n : 0, d->act, d->batch > 1 && d->strideW == 0 ? 1 : 0, dev);
}

struct CachedChoice {
    loka_choice choice;
    loka_status status;
};

std::mutex g_mu;
std::map<ShapeKey, CachedChoice> g_choices;
std::map<RecipeKey, int> g_best_variant;

bool log_on() {       // LOKA_LOG, read once per process
    static const bool on = [] { const char* e = std::getenv("LOKA_LOG"); return e && e[0] && e[0] != '0'; }();
    return on;
}

struct DevBuf {
    void* p = nullptr;
    ~DevBuf() { if (p) (void)hipFree(p); }
    hipError_t alloc(size_t n) { return hipMalloc(&p, n ? n : 16); }
    template <class T> T* as() { return static_cast<T*>(p); }
};

}  // namespace

// Static choice when nothing was profiled: the narrowest tile that still spans the row
// (so the norm stays in the tile), taller tiles once M is large enough to fill the chip;
// rows wider than every such tile go to the two-pass schedule.
int default_variant(const loka_gemm_desc* d) {
    {
        const RecipeKey rk(d->M, d->N, d->K, d->batch, epilogue_of(d), d->x_mode, d->w_mode);
        std::lock_guard<std::mutex> lk(g_mu);
        auto it = g_best_variant.find(rk);
        if (it != g_best_variant.end() && variant_supports(d, it->second)) return it->second;
    }
    if (d->norm == LOKA_NORM_BLOCKNORM) {
        // groups never leave a workgroup: the streaming kernel for skinny layers with many rows (unless K is
        // long and there is a 256 x 256 tile per CU), the large-tile kernel otherwise
        const int64_t t256 = ((d->M + 255) / 256) * ((d->N + 255) / 256) * d->batch;
        const bool stream = d->M * d->batch >= 8192 && !(t256 >= 256 && d->K >= 1024);
        for (int pass = 0; pass < 2; ++pass)
            for (int v = variant_count() - 1; v >= 0; --v)
                if (variant_supports(d, v) && (pass == 1 || variant_is_streaming(v) == stream)) return v;
        return -1;
    }
    // few output tiles and a long K (weight gradients; the widest layers at small batch): split K over several
    // workgroups per tile (measured at 2048 x 123200 x 1024 with LayerNorm: see the variant's table entry)
    {
        const int64_t t128 = ((d->M + 127) / 128) * ((d->N + 127) / 128) * d->batch;
        if (t128 <= 128 && d->K >= 2048) {
            const int v = variant_splitk_choice(d);
            if (v >= 0) return v;
        }
    }
    // Measured on the skinny shapes (65536 x 1024 x 256, 65536 x 256 x 1024, 16384 x 512 x 512, 64 x 4096 x 256 x 256):
    // with at least one 256 x 256 tile per CU the large-tile kernel wins when K is long and the row fits one
    // tile (no cross-workgroup exchange then), and for blockwise scales, which the streaming kernel lacks.
    const int64_t tiles256 = ((d->M + 255) / 256) * ((d->N + 255) / 256) * d->batch;
    const bool blockwise = scale_mode_is_block(d->x_mode);
    if (tiles256 >= 256 && d->N <= 1024 && (blockwise || (d->N <= 256 && d->K >= 1024))) {
        for (int v = variant_count() - 1; v >= 0; --v)
            if (variant_supports(d, v) && variant_epilogue(v) == 2) return v;
    }
    // small layers (K * N <= 128 KB, N <= 256) with enough rows: W in LDS, one row strip per wave (measured against
    // the streaming kernel: 64 x (4096 x 256 x 256) 42.5 against 63 us, 65536 x 256 x 128 10.9 against 19.4 us,
    // 65536 x 128 x 256 15.7 against 19.7 us, 65536 x 512 x 128 13.1 against 21.6 us)
    // (only where W fits the LDS in one piece: the variant that streams K slabs of W is left to the profiler)
    if (d->M * d->batch >= 8192 && (d->N <= 128 ? 128 : 256) * d->K <= 131072) {
        for (int v = 0; v < variant_count(); ++v)
            if (variant_is_strip(v) && variant_supports(d, v)) return v;
    }
    // skinny layers with enough rows to give every CU several row blocks: W in registers, X streamed
    if (d->M * d->batch >= 8192) {
        for (int v = 0; v < variant_count(); ++v)
            if (variant_is_streaming(v) && variant_supports(d, v)) return v;
    }
    int best = -1;
    int64_t best_bn = 0, best_bm = 0;
    for (int v = 0; v < variant_count(); ++v) {
        // (the exact-product forms of these tiles are never the static choice: they trade speed for accuracy)
        if (variant_epilogue(v) != 0 || variant_is_streaming(v) || variant_is_strip(v) || variant_is_exact(v) || !variant_supports(d, v)) continue;
        const int64_t bn = variant_bn(v), bm = variant_bm(v);
        const int64_t tiles = ((d->M + bm - 1) / bm) * d->batch;
        bool better;
        if (best < 0) better = true;
        else if (bn != best_bn) better = bn < best_bn;
        else better = bm > best_bm && tiles >= 1024;     // taller tile only with >= 4 tiles per CU left
        if (better) { best = v; best_bn = bn; best_bm = bm; }
    }
    if (best >= 0) return best;
    // rows wider than a tile: the persistent panel-synchronous schedule once there is enough work to fill
    // the chip for several rounds, the small two-pass tile otherwise
    // (later table entries of a kind are the faster ones where they apply: 32x32x64 MFMAs for non-blockwise scales)
    const bool big = d->M * d->N * d->batch >= (int64_t(1) << 24);
    if (big) {
        for (int v = variant_count() - 1; v >= 0; --v)
            if (variant_supports(d, v) && variant_epilogue(v) == 2) return v;
    }
    for (int v = 0; v < variant_count(); ++v)
        if (variant_supports(d, v) && variant_epilogue(v) == 1) return v;
    for (int v = 0; v < variant_count(); ++v)
        if (variant_supports(d, v)) return v;
    return -1;
}

}  // namespace loka

using namespace loka;

extern "C" {

int loka_dispatch_select(int n, const double* usec, const double* err, double budget, double min_speedup,
                         double usec_bf16) {
    int best = -1;
    for (int i = 0; i < n; ++i) {
        if (!(err[i] <= budget)) continue;
        if (min_speedup > 0.0 && !(usec_bf16 / usec[i] >= min_speedup)) continue;
        if (best < 0 || usec[i] < usec[best]) best = i;
    }
    return best;
}

void loka_dispatch_clear(void) {
    std::lock_guard<std::mutex> lk(g_mu);
    g_choices.clear();
    g_best_variant.clear();
}

int loka_default_variant(const loka_gemm_desc* desc) {
    if (validate_desc(desc, true) != LOKA_OK) return -1;
    return default_variant(desc);
}

loka_status loka_dispatch(const loka_gemm_desc* shape, const void* x_bf16, const void* w_bf16, double err_budget,
                          double min_speedup, loka_choice* choice, loka_candidate* table, int table_cap, int* n_table,
                          void* hip_stream) {
    if (!shape || !x_bf16 || !w_bf16 || !choice) return LOKA_ERR_NULL;
    if (n_table) *n_table = 0;
    loka_gemm_desc d = *shape;
    d.x_mode = LOKA_SCALE_ROW; d.w_mode = LOKA_SCALE_COL; d.variant = -1;
    if (d.batch > 0) { d.strideX = d.M * d.K; d.strideO = d.M * d.N; d.strideW = shape->strideW ? d.N * d.K : 0; }
    loka_status st = validate_desc(&d, true);
    if (st != LOKA_OK) return st;
    if (!(err_budget >= 0.0)) return LOKA_ERR_UNSUPPORTED;
    if (!aligned16(x_bf16) || !aligned16(w_bf16)) return LOKA_ERR_ALIGN;

    const ShapeKey key(d.M, d.N, d.K, d.batch, epilogue_of(&d), err_budget, min_speedup);
    {
        std::lock_guard<std::mutex> lk(g_mu);
        auto it = g_choices.find(key);
        if (it != g_choices.end()) {
            *choice = it->second.choice;
            choice->from_cache = 1;
            return it->second.status;
        }
    }

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int64_t M = d.M, N = d.N, K = d.K, B = d.batch;
    const int64_t nW = d.strideW ? B : 1;
    const uint16_t* xb = static_cast<const uint16_t*>(x_bf16);
    const uint16_t* wb = static_cast<const uint16_t*>(w_bf16);

    // scratch
    DevBuf xq, wq, sx, sw, out, y, yref, ws_q, ws_g, ws_b, ws_p, stats_d, rowmax;
    const size_t sx_max = static_cast<size_t>(B) * M * (K / 128 + 1), sw_max = static_cast<size_t>(nW) * (N + (K / 128) * (N / 128 + 1));
    size_t ws_gemm = 0;
    for (int v = 0; v < variant_count(); ++v) {
        loka_gemm_desc t = d; t.variant = v;
        if (variant_supports(&t, v)) { size_t w = loka_fp8_gemm_norm_workspace(&t); if (w > ws_gemm) ws_gemm = w; }
    }
    size_t ws_quant = 0;
    for (int m = 0; m <= LOKA_SCALE_BLOCK_128x128_POW2; ++m) {
        size_t a = loka_quantize_workspace(static_cast<loka_scale_mode>(m), M, K, 0);
        size_t b = loka_quantize_workspace(static_cast<loka_scale_mode>(m), K, N, 1);
        if (a > ws_quant) ws_quant = a;
        if (b > ws_quant) ws_quant = b;
    }
    const size_t ws_bf16 = loka_bf16_gemm_workspace(&d), ws_probe = loka_probe_error_workspace(B * M, N);
    LOKA_HIP_TRY(xq.alloc(static_cast<size_t>(B) * M * K));
    LOKA_HIP_TRY(wq.alloc(static_cast<size_t>(nW) * N * K));
    LOKA_HIP_TRY(sx.alloc(sx_max * 4));
    LOKA_HIP_TRY(sw.alloc(sw_max * 4));
    LOKA_HIP_TRY(out.alloc(static_cast<size_t>(B) * M * N * 2));
    LOKA_HIP_TRY(y.alloc(static_cast<size_t>(B) * M * N * 4));
    LOKA_HIP_TRY(yref.alloc(static_cast<size_t>(B) * M * N * 4));
    LOKA_HIP_TRY(ws_q.alloc(ws_quant));
    LOKA_HIP_TRY(ws_g.alloc(ws_gemm));
    LOKA_HIP_TRY(ws_b.alloc(ws_bf16));
    LOKA_HIP_TRY(ws_p.alloc(ws_probe));
    LOKA_HIP_TRY(stats_d.alloc(sizeof(loka_probe_stats)));
    LOKA_HIP_TRY(rowmax.alloc(static_cast<size_t>(B) * M * 4));

    hipEvent_t e0, e1;
    LOKA_HIP_TRY(hipEventCreate(&e0));
    LOKA_HIP_TRY(hipEventCreate(&e1));
    struct EvGuard { hipEvent_t a, b; ~EvGuard() { (void)hipEventDestroy(a); (void)hipEventDestroy(b); } } evg{e0, e1};
    constexpr int kWarm = 2, kTimed = 5;

    auto time_region = [&](auto&& body, float* usec) -> loka_status {
        for (int i = 0; i < kWarm; ++i) { loka_status r = body(); if (r != LOKA_OK) return r; }
        LOKA_HIP_TRY(hipEventRecord(e0, s));
        for (int i = 0; i < kTimed; ++i) { loka_status r = body(); if (r != LOKA_OK) return r; }
        LOKA_HIP_TRY(hipEventRecord(e1, s));
        LOKA_HIP_TRY(hipEventSynchronize(e1));
        float ms = 0.f;
        LOKA_HIP_TRY(hipEventElapsedTime(&ms, e0, e1));
        *usec = ms * 1000.f / kTimed;
        return LOKA_OK;
    };

    // BF16 reference: Yref and the baseline time
    // (its weights are transposed once, outside the timed region: the same offline weight preparation the FP8
    // candidates get, whose weights are quantized before their timing starts)
    float usec_bf16 = 0.f;
    st = loka_bf16_gemm(&d, xb, wb, yref.as<float>(), ws_b.p, ws_bf16, s);
    if (st != LOKA_OK) return st;
    st = time_region([&] { return bf16_gemm_launch(&d, xb, wb, yref.as<float>(), ws_b.p, s, true); }, &usec_bf16);
    if (st != LOKA_OK) return st;

    struct Recipe { int xm, wm; };
    std::vector<Recipe> recipes = {{LOKA_SCALE_TENSOR, LOKA_SCALE_TENSOR}, {LOKA_SCALE_ROW, LOKA_SCALE_COL}};
    if (N % 128 == 0 && K % 128 == 0) {
        recipes.push_back({LOKA_SCALE_BLOCK_1x128, LOKA_SCALE_BLOCK_128x128});
        recipes.push_back({LOKA_SCALE_BLOCK_1x128_POW2, LOKA_SCALE_BLOCK_128x128_POW2});
    }

    std::vector<loka_candidate> cands;
    for (const Recipe& rc : recipes) {
        loka_gemm_desc t = d;
        t.x_mode = rc.xm; t.w_mode = rc.wm;
        const loka_scale_mode xm = static_cast<loka_scale_mode>(rc.xm), wm = static_cast<loka_scale_mode>(rc.wm);
        const int64_t sx_per = loka_scale_count(xm, M, K), sw_per = loka_scale_count(wm, K, N);
        // weights are quantized once, outside the timed region (they are static between optimizer steps)
        for (int64_t g = 0; g < nW; ++g) {
            st = loka_quantize(wb + g * K * N, K, N, N, wm, 1, wq.as<uint8_t>() + g * N * K, sw.as<float>() + g * sw_per,
                               ws_q.p, ws_quant, s);
            if (st != LOKA_OK) return st;
        }
        auto quant_x = [&]() -> loka_status {
            if (xm == LOKA_SCALE_TENSOR) {
                for (int64_t g = 0; g < B; ++g) {
                    loka_status r = loka_quantize(xb + g * M * K, M, K, K, xm, 0, xq.as<uint8_t>() + g * M * K,
                                                  sx.as<float>() + g * sx_per, ws_q.p, ws_quant, s);
                    if (r != LOKA_OK) return r;
                }
                return LOKA_OK;
            }
            // row-local scales: all problems' rows in one launch
            return loka_quantize(xb, B * M, K, K, xm, 0, xq.as<uint8_t>(), sx.as<float>(), ws_q.p, ws_quant, s);
        };
        int best_v = -1;
        float best_usec = 0.f;
        for (int v = 0; v < variant_count(); ++v) {
            t.variant = v;
            if (!variant_supports(&t, v)) continue;
            loka_candidate c{};
            c.x_mode = rc.xm; c.w_mode = rc.wm; c.variant = v;
            auto gemm = [&](float* yout) {
                return loka_fp8_gemm_norm(&t, xq.as<uint8_t>(), sx.as<float>(), wq.as<uint8_t>(), sw.as<float>(), nullptr,
                                          nullptr, out.p, yout, ws_g.p, ws_gemm, s);
            };
            st = quant_x();
            if (st != LOKA_OK) return st;
            st = time_region([&] { return gemm(nullptr); }, &c.usec_gemm);
            if (st != LOKA_OK) return st;
            st = time_region([&] { loka_status r = quant_x(); return r != LOKA_OK ? r : gemm(nullptr); }, &c.usec);
            if (st != LOKA_OK) return st;
            // probe this candidate's pre-norm Y against the reference
            st = gemm(y.as<float>());
            if (st != LOKA_OK) return st;
            st = loka_probe_error(y.as<float>(), yref.as<float>(), B * M, N, N, stats_d.as<loka_probe_stats>(),
                                  rowmax.as<float>(), ws_p.p, ws_probe, s);
            if (st != LOKA_OK) return st;
            LOKA_HIP_TRY(hipMemcpyAsync(&c.stats, stats_d.p, sizeof(loka_probe_stats), hipMemcpyDeviceToHost, s));
            LOKA_HIP_TRY(hipStreamSynchronize(s));
            // a candidate whose cross-workgroup wait ran out (the device was not its alone) produced no result:
            // neither its time nor its error means anything
            st = loka_fp8_gemm_norm_check(&t, ws_g.p, ws_gemm, s);
            if (st == LOKA_ERR_TIMEOUT) {
                if (log_on()) std::fprintf(stderr, "[loka] %s: a bounded wait ran out, candidate dropped\n", variant_name(v));
                continue;
            }
            if (st != LOKA_OK) return st;
            cands.push_back(c);
            if (best_v < 0 || c.usec_gemm < best_usec) { best_v = v; best_usec = c.usec_gemm; }
        }
        if (best_v >= 0) {
            std::lock_guard<std::mutex> lk(g_mu);
            g_best_variant[RecipeKey(M, N, K, B, epilogue_of(&d), rc.xm, rc.wm)] = best_v;
        }
    }

    std::vector<double> usec(cands.size()), err(cands.size());
    for (size_t i = 0; i < cands.size(); ++i) { usec[i] = cands[i].usec; err[i] = cands[i].stats.rel_fro; }
    const int pick = loka_dispatch_select(static_cast<int>(cands.size()), usec.data(), err.data(), err_budget,
                                          min_speedup, usec_bf16);
    for (size_t i = 0; i < cands.size(); ++i)
        cands[i].feasible = (err[i] <= err_budget) && !(min_speedup > 0.0 && !(usec_bf16 / usec[i] >= min_speedup));

    CachedChoice cc{};
    cc.choice.usec_bf16 = usec_bf16;
    cc.choice.from_cache = 0;
    if (pick >= 0) {
        cc.choice.x_mode = cands[pick].x_mode; cc.choice.w_mode = cands[pick].w_mode; cc.choice.variant = cands[pick].variant;
        cc.choice.usec = cands[pick].usec; cc.choice.stats = cands[pick].stats;
        cc.status = LOKA_OK;
    } else {
        cc.choice.x_mode = cc.choice.w_mode = cc.choice.variant = -1;
        cc.choice.usec = usec_bf16;
        cc.status = LOKA_ERR_NO_CANDIDATE;
    }
    if (log_on()) {
        for (const auto& c : cands)
            std::fprintf(stderr, "[loka] M=%lld N=%lld K=%lld B=%lld x=%d w=%d %-16s %8.1f us (gemm %8.1f) rel_fro %.4g mere %.4g %s\n",
                         (long long)M, (long long)N, (long long)K, (long long)B, c.x_mode, c.w_mode, variant_name(c.variant),
                         c.usec, c.usec_gemm, c.stats.rel_fro, c.stats.mere, c.feasible ? "feasible" : "-");
        std::fprintf(stderr, "[loka] bf16 reference %.1f us (%.0f %% of the 2.5 PFLOP/s BF16 peak; weights prepared outside the timing); budget %.3g floor %.3g -> %s\n",
                     usec_bf16, 100.0 * 2.0 * M * N * K * B / (usec_bf16 * 1e-6) / 2.5e15, err_budget, min_speedup,
                     pick >= 0 ? variant_name(cands[pick].variant) : "no FP8 candidate (stay in BF16)");
    }
    {
        std::lock_guard<std::mutex> lk(g_mu);
        g_choices[key] = cc;
    }
    *choice = cc.choice;
    if (table && table_cap > 0) {
        const int n = static_cast<int>(cands.size()) < table_cap ? static_cast<int>(cands.size()) : table_cap;
        for (int i = 0; i < n; ++i) table[i] = cands[i];
        if (n_table) *n_table = n;
    } else if (n_table) {
        *n_table = static_cast<int>(cands.size());
    }
    return cc.status;
}

}  // extern "C"
