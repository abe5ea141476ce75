/* loka.h -- C ABI of the MI355X (gfx950) FP8 hot path of LoKA-style low-precision
 * linear layers: quantize -> FP8 GEMM -> scale epilogue fused with the row
 * LayerNorm/RMSNorm -> probe error statistics -> per-shape dispatch.
 *
 * Conventions that hold for every entry point unless its comment says otherwise:
 *  - every data pointer is a DEVICE pointer owned by the caller (hipMalloc or any
 *    allocator built on it); the library keeps no reference after the call's
 *    kernels have run;
 *  - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream);
 *    the call enqueues its kernels on it and returns without synchronizing;
 *  - the hot calls never allocate: scratch comes from the caller through
 *    `workspace`, sized by the matching *_workspace() query (0 bytes => NULL is fine);
 *  - errors are return codes, never aborts or exceptions; arguments are validated
 *    before the first HIP call, so validation can be exercised on a host without a GPU;
 *  - matrices are row-major; bf16 is the upper half of an IEEE binary32; FP8 is
 *    OCP e4m3 (1-4-3, bias 7, no Inf, max 448) stored one code per byte.
 */
#ifndef LOKA_H
#define LOKA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LOKA_OK = 0,
    LOKA_ERR_NULL = 1,         /* a required pointer is NULL */
    LOKA_ERR_SHAPE = 2,        /* non-positive size, K not a multiple of 16, a block mode that does not divide the shape, ld < cols */
    LOKA_ERR_ALIGN = 3,        /* a pointer or stride is not 16-byte aligned */
    LOKA_ERR_UNSUPPORTED = 4,  /* enum out of range, or a scale/norm/N/variant combination no kernel covers */
    LOKA_ERR_WORKSPACE = 5,    /* workspace NULL or smaller than the *_workspace() query */
    LOKA_ERR_HIP = 6,          /* a HIP runtime call failed (launch error, no device) */
    LOKA_ERR_NO_CANDIDATE = 7, /* dispatch: no FP8 variant meets the error budget / speedup floor */
    LOKA_ERR_TIMEOUT = 8       /* loka_fp8_gemm_norm_check: a bounded wait inside the last launch ran out; its output is invalid */
} loka_status;

/* Scale granularity of a [rows, cols] matrix (Section 3.3, "Library and Recipe
 * Selection": tensorwise, rowwise and blockwise quantization strategies). */
typedef enum {
    LOKA_SCALE_TENSOR = 0,        /* one scale                                  -> 1 */
    LOKA_SCALE_ROW = 1,           /* one per row                                -> rows */
    LOKA_SCALE_COL = 2,           /* one per column (weights: per output channel)-> cols */
    LOKA_SCALE_BLOCK_1x128 = 3,   /* one per (row, 128 consecutive columns)     -> rows * cols/128 */
    LOKA_SCALE_BLOCK_128x128 = 4, /* one per 128 x 128 block                    -> rows/128 * cols/128 */
    /* The two block modes with POWER-OF-TWO scales (an extension of this library to the block recipe of
     * Section 3.3, "Library and Recipe Selection"; group layout and counts as modes 3 and 4):
     *   scales[g] = the smallest power of two s with amax_g / s <= 448   (amax_g = max(max|x|, 1e-12)),
     *   q = e4m3_rne(x / s)   (an exact scaling: the only rounding is the e4m3 cast).
     * Every scale is exactly representable by an 8-bit exponent, so the GEMM can hand the per-block scales to the
     * matrix cores (scaled MFMA) instead of rescaling accumulators: see loka_fp8_gemm_norm. */
    LOKA_SCALE_BLOCK_1x128_POW2 = 5,
    LOKA_SCALE_BLOCK_128x128_POW2 = 6,
    /* loka_quantize only, with transpose_out: one scale per (128 consecutive ROWS, column) -> rows/128 * cols, ordered
     * [column][row block].  The transposed codes [cols, rows] with these scales ARE a BLOCK_1x128 operand (its groups run
     * along the rows of the input): what the weight-gradient GEMM of the backward pass needs, whose contraction runs
     * over the batch rows (Section 3.3, "Trainer Integration": dW = X^T dY with X quantized this way and dY quantized
     * BLOCK_128x128 with transpose_out; see loka_fp8_gemm_norm).  rows % 128 == 0. */
    LOKA_SCALE_BLOCK_128x1 = 7
} loka_scale_mode;

/* Row normalization fused into the GEMM epilogue (Section 3.2, "Block-wise
 * Normalization", Case 1: the whole output row is normalized while the tile is
 * still on chip and equals the standard layer). */
typedef enum {
    LOKA_NORM_NONE = 0,
    LOKA_NORM_LAYERNORM = 1,
    LOKA_NORM_RMSNORM = 2,
    /* BlockNorm (Section 3.2, "Block-wise Normalization", the final formulation): the row is cut into
     * consecutive groups of block_n columns, each RMS-normalized on its own, no learned parameters:
     * RMSNorm(Y.view(-1, BlockN)).view(B, N).  Statistics never leave the workgroup that owns the group. */
    LOKA_NORM_BLOCKNORM = 3
} loka_norm;

/* Activation fused after the normalization (Section 3.2, "Hard Swish"):
 * h-swish(x) = x * ReLU6(x + 3) / 6.  Only with LOKA_NORM_BLOCKNORM. */
typedef enum { LOKA_ACT_NONE = 0, LOKA_ACT_HARDSWISH = 1 } loka_act;

const char* loka_status_string(loka_status s);

/* Number of fp32 scales `mode` produces for a [rows, cols] matrix; -1 when the
 * mode is out of range or (block modes) does not divide the shape. Host only. */
int64_t loka_scale_count(loka_scale_mode mode, int64_t rows, int64_t cols);

/* ---------------------------------------------------------------- quantize
 * amax -> scale -> OCP e4m3 cast of a bf16 matrix (the quantization step whose
 * overhead Section 2.3, "Throughput Analysis", puts above 30 % of GEMM latency).
 * Per scale group g:  amax_g = max(max|x|, 1e-12);  scales[g] = amax_g / 448
 * (the DEQUANTIZATION factor, one fp32 division);  q = e4m3_rne(clamp(x * (448 /
 * amax_g), -448, 448)) with one fp32 division for 448/amax_g and one fp32 multiply
 * per element.  Codes and scales are bit-exact with that recipe.
 *
 *   x_bf16   [rows, ld] bf16, ld >= cols, ld % 8 == 0, 16-byte aligned
 *   q        [rows, cols] uint8, or [cols, rows] when transpose_out != 0 (used for
 *            weights W[K, N] -> Wq[N, K] so the GEMM reads K-contiguous operands)
 *   scales   [loka_scale_count(mode, rows, cols)] fp32, group order: row-major over
 *            (row group, column group)
 *   cols must be a multiple of 16 (rows too when transpose_out != 0).
 * Workspace: loka_quantize_workspace() bytes (non-zero only for TENSOR and COL, whose groups span workgroups: amax
 * pass, scales, cast pass; every other mode is ONE pass, 3 bytes of traffic per element); contents are scratch.
 * transpose_out is not supported for ROW and the BLOCK_1x128 modes and is required for BLOCK_128x1
 * (LOKA_ERR_UNSUPPORTED).  The power-of-two modes replace the two divisions by the rule stated at the enum. */
size_t loka_quantize_workspace(loka_scale_mode mode, int64_t rows, int64_t cols, int transpose_out);
loka_status loka_quantize(const void* x_bf16, int64_t rows, int64_t cols, int64_t ld, loka_scale_mode mode,
                          int transpose_out, uint8_t* q, float* scales, void* workspace, size_t ws_bytes,
                          void* hip_stream);

/* Test aid: OCP e4m3 cast (round-to-nearest-even, saturating) of n device floats with
 * the same device routine loka_quantize uses.  t and codes are device pointers. */
loka_status loka_e4m3_from_f32(const float* t, uint8_t* codes, int64_t n, void* hip_stream);

/* Measurement aid: what this machine delivers for the two resources the kernels are bound by, so that a rate can be
 * reported against a MEASURED ceiling beside the datasheet peak (the sustained shader clock under matrix load is
 * below the clock the datasheet assumes).
 *   kind 0: FP8 matrix rate, TFLOP/s (register-resident 32x32x64 matrix instructions back to back on every CU)
 *   kind 1: BF16 matrix rate, TFLOP/s (32x32x16)
 *   kind 2: HBM copy rate, GB/s (bytes read + written), first half of `scratch` copied to the second
 *   kind 3: operand delivery rate, GB/s: the large-layer kernel's operand stream for a 32768 x 4096 x 4096 layer on
 *           that kernel's schedule (per CU and K step 32 KB of a row panel shared by the 16 workgroups of the panel and
 *           32 KB of the weight matrix, loads that write LDS directly, the kernel's request shape and depth) with no
 *           arithmetic; scratch at least 144 MiB (LOKA_ERR_WORKSPACE otherwise)
 *   kind 4, 5: as 0, 1, but every instruction of a round takes different operand registers filled with pseudo-random
 *           codes (consecutive instructions toggle the multipliers' inputs as quantized data does; kinds 0 and 1
 *           repeat one pair of registers of small codes, the least switching activity and the highest clock)
 *   kind 6, 7: the FP8 rate with the 16x16x128 form of the matrix instruction, on constant (6) and on changing (7)
 *           operands (kinds 0 and 4 use the 32x32x64 form, which the large-layer kernel issues)
 * Runs back-to-back launches for about `millis` milliseconds (clocks settle under load during the first tens of
 * milliseconds) and returns the LAST launch's rate in *value_host (host memory).  scratch: device memory, 16-byte
 * aligned, at least 4 MiB (kind 2: at least 64 MiB; use >= 1 GiB to stay clear of the last-level cache).
 * SYNCHRONIZES; not a hot call. */
loka_status loka_machine_ceiling(int kind, double millis, void* scratch, size_t scratch_bytes, double* value_host,
                                 void* hip_stream);

/* ---------------------------------------------------------------- FP8 GEMM + fused norm
 * O = norm( (Xq . Wq^T) scaled )  for `batch` independent problems of one shape
 * (Section 2.1: LRMs are dominated by many small GEMMs each followed by a
 * normalization; Section 3.2: the normalization is applied in the GEMM epilogue
 * while the output tile is on chip).
 *   acc[m,n] = sum_k dq(xq[m,k]) * dq(wq[n,k])           FP8 MFMA, fp32 accumulate
 *   Y[m,n]   = acc * sx * sw                              TENSOR/ROW x TENSOR/COL scales
 *            = sum_kb acc_kb * sx[m,kb] * sw[kb, n/128]   BLOCK_1x128 x BLOCK_128x128: each
 *                                                         128-wide K block is promoted to an
 *                                                         fp32 accumulator with its scales
 *                                                         (the _POW2 modes: same sum; x_mode and
 *                                                         w_mode must both be _POW2 or neither)
 *   O[m,n]   = bf16_rne( LayerNorm / RMSNorm / identity over the N entries of row m )
 *     LayerNorm: (Y-mu)/sqrt(var+eps)*gamma+beta, biased variance;  RMSNorm: Y/sqrt(mean(Y^2)+eps)*gamma.
 *     BlockNorm: Y/sqrt(mean over the element's group of block_n columns (Y^2)+eps), then the activation;
 *     gamma and beta are ignored.
 * There is no bias input (Section 3.2, "No Bias").
 * Supported scale pairs: x in {TENSOR, ROW} with w in {TENSOR, COL}; or x = BLOCK_1x128
 * with w = BLOCK_128x128 (needs N % 128 == 0 and K % 128 == 0).  K % 16 == 0, N % 16 == 0 (a K that is not a
 * multiple of 128 is taken by the general tiled kernels, which mask the tail of the last K step).
 */
typedef struct {
    int64_t M, N, K;
    int64_t batch;            /* >= 1 independent problems in one launch (grouped small GEMMs) */
    int64_t strideX;          /* elements between consecutive problems' Xq ([M,K] each); 0 = shared */
    int64_t strideW;          /* ... Wq ([N,K] each); 0 = one weight shared by all problems */
    int64_t strideO;          /* ... O and Y ([M,N] each) */
    int32_t x_mode, w_mode;   /* loka_scale_mode of sx / sw; problem g's scales start at g * loka_scale_count(...)
                                 (at 0 when the operand's stride is 0) */
    int32_t norm;             /* loka_norm */
    float eps;
    int32_t variant;          /* kernel variant id (see loka_variant_name), or -1 = library's choice for the shape.
                               * The choice behind -1 is looked up at every call and a loka_dispatch (or
                               * loka_dispatch_clear) in between can change it: a caller that sizes a workspace, launches
                               * and checks in separate calls while another thread may dispatch should resolve it once
                               * (variant = loka_default_variant(desc)) and pass the same id to all three. */
    int32_t block_n;          /* LOKA_NORM_BLOCKNORM: group width; 256 is built (N % 256 == 0).  Ignored otherwise */
    int32_t act;              /* loka_act; LOKA_ACT_HARDSWISH needs LOKA_NORM_BLOCKNORM */
} loka_gemm_desc;

int loka_variant_count(void);
const char* loka_variant_name(int variant);      /* NULL when out of range */
/* 1 when `variant` can run `desc` (shape limits of the tile and its epilogue schedule). Host only. */
int loka_variant_supports(const loka_gemm_desc* desc, int variant);

/*   xq  [batch][M, K] codes         sx  scales of X         wq [batch][N, K] codes      sw scales of W
 *   gamma, beta: bf16 [N] or NULL (= 1 / 0), shared by all problems; beta is ignored by RMSNorm
 *   out_bf16 [batch][M, N] bf16 (required)
 *   y_fp32   [batch][M, N] fp32 pre-norm Y for the probe, or NULL to skip that store
 * Workspace: loka_fp8_gemm_norm_workspace(desc) bytes (non-zero only for variants whose row
 * statistics cross workgroups).  Returns LOKA_ERR_UNSUPPORTED when desc->variant cannot run
 * the shape.  */
size_t loka_fp8_gemm_norm_workspace(const loka_gemm_desc* desc);
loka_status loka_fp8_gemm_norm(const loka_gemm_desc* desc, const uint8_t* xq, const float* sx, const uint8_t* wq,
                               const float* sw, const void* gamma_bf16, const void* beta_bf16, void* out_bf16,
                               float* y_fp32, void* workspace, size_t ws_bytes, void* hip_stream);

/* Variants whose row statistics cross workgroups inside one launch (rows wider than a tile) make every
 * workgroup wait for the other tiles of its row panel.  The wait is bounded: if it runs out (it never does when
 * the launch's workgroups are all resident, which the launch arranges on an otherwise idle device), the workgroup
 * marks the launch in the workspace, writes the rows of its tile as NaN (FP8 output: a NaN row scale) so that
 * nothing downstream can take them for results, and goes on: the kernel always ends.  This call reports
 * the mark of the LAST loka_fp8_gemm_norm or loka_fp8_gemm_norm_fp8out call that used `workspace` with `desc`:
 * LOKA_OK, or LOKA_ERR_TIMEOUT.
 * It SYNCHRONIZES hip_stream (4 bytes are copied to the host); variants without such a wait return LOKA_OK
 * without touching the GPU.  Not needed on the hot path; meant for health checks and tests. */
loka_status loka_fp8_gemm_norm_check(const loka_gemm_desc* desc, const void* workspace, size_t ws_bytes, void* hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, serving loops that must not call the
 * allocator, harnesses that forbid it): loka_fp8_gemm_norm with its workspace taken from a device array the LIBRARY
 * owns (16 MiB per GPU the library runs on, held until the process ends) instead of from the caller.  Same arguments
 * otherwise, same kernels, same bits in out_bf16 / y_fp32.  The call allocates nothing and calls no allocating
 * routine; the first call on a device asks the runtime for the array's address on that device (set-up).
 *   - LOKA_ERR_WORKSPACE when the variant chosen for `desc` needs more scratch than
 *     LOKA_STATIC_SCRATCH_BYTES (loka_fp8_gemm_norm_workspace(desc) tells how much): use
 *     loka_fp8_gemm_norm with a caller-owned workspace for those.
 *   - Every call on a GPU uses that GPU's one array: calls that may overlap on one GPU (different streams, different
 *     threads) race on it and must be serialized by the caller.  Nothing in the array has to be cleared between
 *     calls (the kernels recognize stale contents), and no call relies on what an earlier one left there.
 *   - A bounded wait that runs out (see loka_fp8_gemm_norm_check; there is no workspace to hand to it here) shows
 *     in the output itself: the affected rows are NaN. */
#define LOKA_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
loka_status loka_fp8_gemm_norm_static(const loka_gemm_desc* desc, const uint8_t* xq, const float* sx, const uint8_t* wq,
                                      const float* sw, const void* gamma_bf16, const void* beta_bf16, void* out_bf16,
                                      float* y_fp32, void* hip_stream);

/* Test aid for the error path of those bounded waits: from now on every such wait polls at most `polls` times
 * (process-wide; a negative value restores the library's limit).  With polls == 0 the waits also look for a value
 * no workgroup writes, so every one of them runs out after its first poll whatever the timing: the kernels still
 * end, the rows of the affected tiles are written as NaN (bf16 output) or get a NaN row scale (FP8 output), and
 * loka_fp8_gemm_norm_check reports LOKA_ERR_TIMEOUT.  Host only; takes effect at the next launch. */
void loka_test_set_spin_limit(int64_t polls);

/* FP8 output for the next layer (Section 3.2, "Block-wise Normalization", Case 1: once a row is normalized
 * inside the kernel, the activation and the quantization for the next layer can join the same epilogue, before
 * anything is written to HBM).  Same computation as loka_fp8_gemm_norm, but instead of bf16 O the call
 * writes what loka_quantize(O_bf16, LOKA_SCALE_ROW) would produce from it, bit for bit:
 *   oq [batch][M, N] e4m3 codes,  so [batch][M] fp32 row scales (amax of the row's bf16 values / 448).
 * The next layer's loka_fp8_gemm_norm takes (oq, so) as its (xq, sx) with x_mode = LOKA_SCALE_ROW.
 * Built into three kernels, non-blockwise input scales:
 *   "wreg32"  (streaming skinny-layer kernel: N <= 1024, K in {128, 256, 512, 1024}, K * N <= 256 KB) and
 *   "strip32" (small-layer strip kernel: N <= 256, K * N <= 256 KB): the whole output row is in one workgroup /
 *             wave; every norm, gamma / beta and activation loka_fp8_gemm_norm takes;
 *   "panel32_256x256" (large layers, rows wider than a tile): LayerNorm, RMSNorm or BlockNorm (+ Hard-Swish).
 *             LayerNorm / RMSNorm without gamma / beta: the normalized value grows with the pre-norm value, so the
 *             row minimum and maximum, sent along with the row statistics in the one exchange between the row's
 *             workgroups, decide the row scale; with gamma / beta, under BlockNorm or with an activation the row
 *             amax of the result crosses the workgroups in a second exchange.  LOKA_NORM_NONE: unsupported.
 * desc->variant names one, or -1: the library's choice for the shape when it is one of the three, else the
 * streaming kernel where it covers the shape, else the panel kernel.  LOKA_ERR_UNSUPPORTED otherwise.
 * Workspace: loka_fp8_gemm_norm_fp8out_workspace(desc) bytes (non-zero only for the panel kernel with rows wider
 * than 256 columns - also under BlockNorm, where loka_fp8_gemm_norm needs none -; NULL / 0 otherwise), device memory, 16-byte aligned, not shared with a call still running;
 * loka_fp8_gemm_norm_check reports the panel kernel's bounded wait on it as for loka_fp8_gemm_norm.
 * y_fp32 as above (NULL to skip).  oq, so: device pointers, 16-byte aligned, caller-owned. */
size_t loka_fp8_gemm_norm_fp8out_workspace(const loka_gemm_desc* desc);
loka_status loka_fp8_gemm_norm_fp8out(const loka_gemm_desc* desc, const uint8_t* xq, const float* sx, const uint8_t* wq,
                                      const float* sw, const void* gamma_bf16, const void* beta_bf16, uint8_t* oq,
                                      float* so, float* y_fp32, void* workspace, size_t ws_bytes, void* hip_stream);

/* Quantization fused into the layer (Section 2.3, "Throughput Analysis": quantization overhead can exceed 30 % of
 * the GEMM's latency, and memory traffic for the low-precision copy can cancel the gain; Section 3.2: activation
 * and (de)quantization can be fused).  One call = loka_quantize(x, LOKA_SCALE_ROW) followed by loka_fp8_gemm_norm,
 * with identical bits in every output (the same kernel variant in both), but the e4m3 copy of X never exists in
 * HBM: a kernel that keeps whole rows of X in one workgroup reads bf16 rows, takes the row amax, scales, converts
 * and multiplies.
 *   x_bf16 [batch][M, K] bf16 (strideX in elements), desc->x_mode must be LOKA_SCALE_ROW; wq, sw, gamma, beta,
 *   out_bf16, y_fp32 as in loka_fp8_gemm_norm;  sx_out: fp32 [batch][M] row scales (amax / 448) or NULL.
 * Two kernels take it: the small-layer strip kernel (variant "strip32": N <= 256, K in {128, 256, 512}, W resident
 * in LDS) and the streaming skinny-layer kernel ("wreg32": N <= 1024, K in {128, 256, 512, 1024}, K * N < 256 KB).
 * desc->variant names one, or -1: the strip kernel where it applies, else the streaming kernel.
 * LOKA_ERR_UNSUPPORTED for every other shape or variant (use the two calls).  No workspace. */
loka_status loka_fp8_linear_norm(const loka_gemm_desc* desc, const void* x_bf16, const uint8_t* wq, const float* sw,
                                 const void* gamma_bf16, const void* beta_bf16, void* out_bf16, float* y_fp32,
                                 float* sx_out, void* hip_stream);

/* The same layer in one launch for EVERY shape the streaming kernel covers (variant "wreg32": N <= 1024, K in
 * {128, 256, 512, 1024}, K * N <= 256 KB - the skinny layers of Section 2.1, where Section 2.3 finds the quantization
 * pass above 30 % of the GEMM's latency) and, on the large-tile kernel (variant "panel32_256x256"), for layers whose
 * output row fits one tile (N <= 256) with K in {512, 1024, 2048}; with the quantized activation handed back: each
 * workgroup first quantizes the rows it is about to consume (row amax, scale = amax / 448, e4m3 codes: the bits
 * loka_quantize(x, LOKA_SCALE_ROW) writes), stores them to xq_out / sx_out, and streams them back from its L2; the rest
 * is the kernel of loka_fp8_gemm_norm, so out_bf16 and y_fp32 carry the bits of the two calls on the same variant.  A
 * trainer keeps xq_out / sx_out where it would have kept the output of the separate quantize call.
 *   x_bf16 [batch][M, K] bf16 (strideX in elements; with batch > 1 strideX must not be 0);
 *   xq_out [batch][M, K] e4m3 codes and sx_out [batch][M] fp32 row scales: device memory, 16-byte aligned, written by
 *   the call, not to be read or written by anything else until the call's kernel has finished;
 *   wq, sw, gamma, beta, out_bf16, y_fp32 as in loka_fp8_gemm_norm.  desc->x_mode must be LOKA_SCALE_ROW;
 *   desc->variant names one of the two kernels, or is -1: the library's choice for the shape where that kernel has
 *   the prologue, else the other.  LOKA_ERR_UNSUPPORTED for shapes neither covers.
 * No workspace, no allocation. */
loka_status loka_fp8_linear_norm_xq(const loka_gemm_desc* desc, const void* x_bf16, uint8_t* xq_out, float* sx_out,
                                    const uint8_t* wq, const float* sw, const void* gamma_bf16, const void* beta_bf16,
                                    void* out_bf16, float* y_fp32, void* hip_stream);

/* ---------------------------------------------------------------- probe reference
 * Yref = X . W from the UNQUANTIZED bf16 operands with fp32 accumulation: the
 * high-precision reference the probe measures FP8 against (Section 2.3, "Error
 * Analysis"; the paper's reference is TF32, this build's is BF16 operands with fp32
 * accumulate).  x [batch][M, K] bf16, w [batch][K, N] bf16 (strideW 0 = shared),
 * yref [batch][M, N] fp32.  Only M, N, K, batch and the strides of `desc` are read.
 * K % 8 == 0, N % 16 == 0.  Workspace: loka_bf16_gemm_workspace() bytes (a transposed copy of W). */
size_t loka_bf16_gemm_workspace(const loka_gemm_desc* desc);
loka_status loka_bf16_gemm(const loka_gemm_desc* desc, const void* x_bf16, const void* w_bf16, float* yref_fp32,
                           void* workspace, size_t ws_bytes, void* hip_stream);

/* ---------------------------------------------------------------- probe error statistics
 * Error of Y against Yref (Section 2.3, "Error Analysis"), both fp32 [M, ld]:
 *   d = Y - Yref (one fp32 subtraction)
 *   rowmax[m]  = max_n |d|            (bit-exact)           max_abs = max_m rowmax[m]
 *   rel_fro    = sqrt(sum d^2) / sqrt(sum Yref^2)            (fp64 sums)
 *   mere       = (1/(M N)) * sum |d| / max(|Yref|, 1e-30)    the paper's MERE read as a mean
 * The sums are combined in a fixed order, so results are repeatable run to run.
 * stats_device: one loka_probe_stats in DEVICE memory; rowmax_device: fp32 [M] or NULL.
 * ld % 4 == 0, N % 4 == 0.  */
typedef struct {
    double rel_fro;
    double max_abs;
    double mere;
    double sum_sq_err;
    double sum_sq_ref;
} loka_probe_stats;

size_t loka_probe_error_workspace(int64_t M, int64_t N);
loka_status loka_probe_error(const float* y, const float* yref, int64_t M, int64_t N, int64_t ld,
                             loka_probe_stats* stats_device, float* rowmax_device, void* workspace, size_t ws_bytes,
                             void* hip_stream);

/* ---------------------------------------------------------------- probe online tracker
 * Merges one batch of activations into the running distribution summary of a layer's input (Section 3.1,
 * "Online Distribution Learning": mean tracked by streaming, covariance by a batched Welford tracker that
 * needs O(K^2) memory).  State: n (kept by the caller), mu [K] fp32, sigma [K, K] fp32 = the UNNORMALIZED
 * scatter sum_m (x_m - mu)(x_m - mu)^T of all rows seen so far (unbiased covariance = sigma / (n - 1)).
 *   mu_b  = column means of X            S_b = (X - 1 mu_b^T)^T (X - 1 mu_b^T)
 *   n'    = n_old + B                    delta = mu_b - mu
 *   mu'   = mu + (B / n') delta          sigma' = sigma + S_b + (n_old B / n') delta delta^T
 * S_b is evaluated as X^T X - B mu_b mu_b^T with X^T X on the BF16 matrix cores (exact products, fp32
 * accumulation over the batch rows), column sums in fp64, the subtraction and the merge in fp64, one rounding
 * to fp32.  Both triangles of sigma are written; results are repeatable run to run (fixed reduction order).
 *   x_bf16 [B, ld] bf16 (ld >= K, K % 8 == 0, ld % 8 == 0, K <= 32768), 16-byte aligned
 *   mu, sigma: device, updated in place; start a stream of batches from n_old = 0, mu = 0, sigma = 0
 * The new row count n_old + B is the caller's to keep.
 * Workspace: loka_tracker_update_workspace(B, K) bytes (partial scatters of the batch splits); scratch. */
size_t loka_tracker_update_workspace(int64_t B, int64_t K);
loka_status loka_tracker_update(const void* x_bf16, int64_t B, int64_t K, int64_t ld, int64_t n_old, float* mu,
                                float* sigma, void* workspace, size_t ws_bytes, void* hip_stream);

/* ---------------------------------------------------------------- dispatch
 * Per-shape selection (Section 3.3, "Library and Recipe Selection"): among the
 * library's own candidates (scale recipe x kernel variant) keep those whose probe
 * error is within the budget and whose speedup over the BF16 GEMM reaches
 * min_speedup, and take the fastest.  The paper's typical thresholds are an error
 * bound of 0.2 on MERE and a speedup floor of 1.05; here the budget applies to
 * rel_fro (MERE is reported in the candidate table).  */
typedef struct {
    int32_t x_mode, w_mode;   /* scale recipe */
    int32_t variant;          /* kernel variant */
    int32_t feasible;         /* met the budget and the speedup floor */
    float usec;               /* quantize(X) + GEMM+norm, average of the timed launches */
    float usec_gemm;          /* GEMM+norm alone */
    loka_probe_stats stats;   /* probe of this candidate's Y against the BF16 reference */
} loka_candidate;

typedef struct {
    int32_t x_mode, w_mode, variant;
    int32_t from_cache;       /* 1 when the per-shape cache answered */
    float usec;               /* of the chosen candidate */
    float usec_bf16;          /* BF16 reference GEMM on the same shape */
    loka_probe_stats stats;
} loka_choice;

/* Pure host rule, exposed so it can be tested with injected tables: index of the
 * fastest candidate with err[i] <= budget and (min_speedup <= 0 or usec_bf16/usec[i] >=
 * min_speedup); ties to the lowest index; -1 when none qualifies. */
int loka_dispatch_select(int n, const double* usec, const double* err, double budget, double min_speedup,
                         double usec_bf16);

/* Profiles every candidate that supports `shape` on the given bf16 operands
 * (x [batch][M,K], w [batch][K,N], device), fills `choice`, and remembers it per
 * (M, N, K, batch, norm, budget, min_speedup).  Later calls with the same key return the
 * cached choice without touching the GPU.  This call ALLOCATES device scratch and
 * SYNCHRONIZES the stream; it is a profiling step, not a hot call.
 * `table`/`table_cap`/`n_table` (optional) receive one row per profiled candidate.
 * shape->x_mode, w_mode and variant are ignored.
 * Returns LOKA_ERR_NO_CANDIDATE (and x_mode = w_mode = variant = -1 in `choice`, meaning: keep
 * this layer in BF16 -- the outcome the paper's Limitations describe for layers that do not
 * tolerate low precision) when the feasible set is empty.  */
loka_status loka_dispatch(const loka_gemm_desc* shape, const void* x_bf16, const void* w_bf16, double err_budget,
                          double min_speedup, loka_choice* choice, loka_candidate* table, int table_cap, int* n_table,
                          void* hip_stream);
/* Forget every cached choice (host only). */
void loka_dispatch_clear(void);
/* Variant the library would run for desc with variant = -1 (cached dispatch choice for the
 * shape and recipe if there is one, else a static heuristic); -1 when nothing supports it. */
int loka_default_variant(const loka_gemm_desc* desc);

#ifdef __cplusplus
}
#endif
#endif /* LOKA_H */
