/*
 * tweo.h - C ABI of the MI355X (gfx950) library for the per-tensor FP8 linear
 * layer with the fused TWEO activation-outlier penalty, and for the W8A8
 * per-tensor static INT8 linear layer (TWEO, arXiv 2511.23225).
 *
 * Conventions that hold for every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller; the library
 *     never allocates, frees or synchronises.  Pointers are 16-byte aligned.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream).  Scalars that depend on device data (amax, scales,
 *     penalty) stay on the device.
 *   - Tensors are dense row-major, last index contiguous.  bf16 tensors are
 *     passed as void* (2 bytes per element), E4M3 tensors as uint8_t codes
 *     (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no infinities,
 *     largest finite value 448, code 0x7F/0xFF = NaN).
 *   - Arguments are validated before anything is launched.  Errors come back
 *     as a status code; nothing aborts or throws across the ABI.  After an
 *     error the outputs are unspecified.
 *   - Identical inputs give byte-identical outputs (no floating-point atomics,
 *     fixed reduction orders).
 */
#ifndef TWEO_H
#define TWEO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TWEO_OK = 0,
    TWEO_ERR_INVALID_ARG = 1, /* NULL where not allowed, non-positive size, misaligned pointer */
    TWEO_ERR_UNSUPPORTED = 2, /* shape or option outside what the kernels handle            */
    TWEO_ERR_WORKSPACE = 3,   /* workspace NULL or smaller than tweo_workspace_bytes()      */
    TWEO_ERR_HIP = 4          /* a launch failed (hipGetLastError() != hipSuccess)          */
} tweo_status;

/* Hyper-parameters of the TWEO loss (Sec. 3.3).  The paper uses tau = 3, p = 4
 * in all experiments (Sec. 4.1) and eps = 1e-6.  p must be a positive even or
 * odd integer <= 8; p = 4 is the fast path. */
typedef struct {
    float tau;
    float eps;
    int p;
} tweo_penalty_cfg;

/* Operations tweo_workspace_bytes() knows about. */
enum {
    TWEO_OP_FP8_LINEAR_FWD = 0,
    TWEO_OP_FP8_LINEAR_BWD = 1,
    TWEO_OP_W8A8_LINEAR = 2,
    TWEO_OP_FP8_LINEAR_FWD_BF16 = 3,
    TWEO_OP_FP8_LINEAR_BWD_BF16 = 4,
    TWEO_OP_LAYERNORM_QUANTIZE = 5 /* M = rows; N, K unused (pass 1) */
};

/* Bytes of device workspace the given operation can use for these sizes (a
 * multiple of 256; never 0).  The workspace needs no initialisation and may be
 * reused by the next call on the same stream.  For the two *_BF16 operations
 * it starts with 4 KB that are always required (the amax launch leaves one
 * maximum per workgroup there and the cast launch reduces them, so nothing has
 * to be cleared and no atomic is used).  Then the parts of the plain
 * operations: the TWEO
 * penalty partial sums of a forward call (a few KB, required whenever a penalty
 * is asked for: less is TWEO_ERR_WORKSPACE), then - only after
 * tweo_set_stream_k(1) - scratch that lets a GEMM whose tile count does not fill
 * the CUs evenly split the K loop of its last tiles over all CUs (two fp32 tiles
 * per CU, 128 MB on a 256-CU device; only counted when a contraction of the
 * operation is at least 2048 long).  A caller that passes a workspace without
 * the second part gets the same results up to the fp32 summation order, from
 * the plain schedule.  The second part also serves, without any switch, a GEMM
 * without penalty whose output has far fewer 256x256 tiles than the device has
 * CUs under a contraction of 16384 or more (weight gradients of narrow layers
 * over many tokens): several workgroups share a tile, each multiplies a run of
 * K and stores fp32 sums here (runs x rows x cols x 4 bytes), a second launch
 * adds the runs in index order - run-to-run identical results. */
size_t tweo_workspace_bytes(int op, int64_t M, int64_t N, int64_t K);

const char *tweo_status_string(tweo_status s);

/*
 * Per-tensor amax (Sec. 4.3: one scaling factor for the entire tensor;
 * Sec. 4.4 Eq. 4: max(|X|)).
 *   x_bf16   [n] bf16, n >= 1
 *   amax_out one fp32 on the device; overwritten with max_i |x_i| (exact).  An
 *            Inf in x gives Inf, a NaN gives NaN (the maximum is taken on the
 *            15-bit magnitude patterns).
 */
tweo_status tweo_amax(const void *x_bf16, int64_t n, float *amax_out, void *stream);

/*
 * Per-tensor E4M3 quantize-cast (Sec. 4.3; E4M3 range +-448, Sec. 1).
 *   scale = 448 / *amax (fp32 division; amax of 0, Inf or NaN gives scale 1; a
 *   quotient that overflows gives FLT_MAX), scale_inv = 1 / scale.
 *   q[r,c] = e4m3( fp32(x[r,c]) * scale ), round to nearest even, saturating at
 *   +-448, NaN -> NaN code.
 *   x_bf16 [rows, cols]; cols % 8 == 0.
 *   amax   one fp32 on the device (e.g. from tweo_amax).
 *   q      [rows, cols] codes.           qT  [cols, rows] codes or NULL.
 *   scale_out, scale_inv_out: one fp32 each on the device, or NULL.
 */
tweo_status tweo_quantize_e4m3(const void *x_bf16, int64_t rows, int64_t cols, const float *amax,
                               uint8_t *q, uint8_t *qT, float *scale_out, float *scale_inv_out,
                               void *stream);

/*
 * The same cast into E5M2, the gradient format of the HYBRID recipe the paper
 * trained with (Sec. 4.3: E4M3 for activations and weights, E5M2 for
 * gradients): scale = 57344 / *amax with the same guards, q = e5m2(fp32(x) *
 * scale), round to nearest even, saturating at +-57344 (a cast never produces
 * an infinity), NaN -> a NaN code.  Arguments and errors as tweo_quantize_e4m3.
 */
tweo_status tweo_quantize_e5m2(const void *x_bf16, int64_t rows, int64_t cols, const float *amax,
                               uint8_t *q, uint8_t *qT, float *scale_out, float *scale_inv_out,
                               void *stream);

/*
 * Delayed scaling, the form of per-tensor scaling the paper trained with
 * (Sec. 4.3: one scale per tensor, amax history of length 16): the cast of step
 * t uses scale_t = 448 / max(amax_{t-16} .. amax_{t-1}), fixed before the tensor
 * is seen, and returns the tensor's own amax to the history, so the tensor is
 * read once (2 B read + 1 (+1) B written per element, against two reads with
 * tweo_amax + tweo_quantize_e4m3).  The paper names the history length, not the
 * reduction over it: the maximum is used.  An empty history (the first call on a
 * state: pass bootstrap != 0) takes the scale from the tensor's own amax, i.e. a
 * current-scaling step.  Values beyond the delayed scale's range saturate to
 * +-448.  Guards on the scale as in tweo_quantize_e4m3.
 *
 * The state is TWEO_DELAYED_STATE_WORDS 32-bit words of device memory owned by
 * the caller, one per scaled tensor; it is the only state of the recipe (copy it
 * out to checkpoint it).  Word layout: [0..15] amax ring, [16] accumulator (0
 * between calls), [17] next scale, [18] its inverse, [19] ring position,
 * [20] entries filled, [21] the scale the last cast used, [22] its inverse -
 * TWEO_DELAYED_USED_SCALE_INV is the word a GEMM dequantises with.
 *   tweo_delayed_state_init: clears a state (scales = 1).
 *   tweo_quantize_e4m3_delayed: x_bf16 [rows, cols] -> q [rows, cols], optional
 *   qT [cols, rows]; updates the state.  Arguments and errors as
 *   tweo_quantize_e4m3; state 16-byte aligned.
 */
#define TWEO_DELAYED_STATE_WORDS 32
#define TWEO_DELAYED_NEXT_SCALE 17
#define TWEO_DELAYED_USED_SCALE 21
#define TWEO_DELAYED_USED_SCALE_INV 22
size_t tweo_delayed_state_bytes(void);
tweo_status tweo_delayed_state_init(void *state, void *stream);
tweo_status tweo_quantize_e4m3_delayed(const void *x_bf16, int64_t rows, int64_t cols, void *state,
                                       int bootstrap, uint8_t *q, uint8_t *qT, void *stream);
/* The same for a tensor that is cast to E5M2 (the gradients of the HYBRID recipe,
 * Sec. 4.3): scale = 57344 / max(history), saturation at +-57344, a state of its own. */
tweo_status tweo_quantize_e5m2_delayed(const void *x_bf16, int64_t rows, int64_t cols, void *state,
                                       int bootstrap, uint8_t *q, uint8_t *qT, void *stream);

/*
 * LayerNorm feeding the per-tensor FP8 cast (Sec. 4.3: the LayerNorm components
 * run under FP8 together with the linear layers, so the normalised activation is
 * what the next linear's cast consumes).  The paper gives no formula; the
 * textbook row-wise normalisation is taken:
 *   h[r,c]  = x[r,c]                      or, with a residual, bf16( x[r,c] + residual[r,c] )
 *   mu_r    = mean_c h[r,c],  var_r = mean_c (h[r,c] - mu_r)^2        (biased)
 *   y[r,c]  = bf16( (h[r,c] - mu_r) / sqrt(var_r + eps) * gamma[c] + beta[c] )
 *   q[r,c]  = e4m3( fp32(y[r,c]) * scale ),  qT[c,r] = q[r,c]
 * The statistics and the normalisation are computed in fp64 and y is rounded once
 * to bf16: it is the activation as a model stores it, and amax, scale and codes
 * are those tweo_amax + tweo_quantize_e4m3 give on that bf16 tensor.  The
 * statistics themselves are never quantised.
 *   tweo_layernorm_quantize_e4m3: current scaling, scale = 448 / max|y|.
 *   tweo_layernorm_quantize_e4m3_delayed: delayed scaling on `state` as
 *   tweo_quantize_e4m3_delayed (the tensor's amax enters the history).
 *   x_bf16 [rows, cols]; rows % 16 == 0, cols % 16 == 0.
 *   residual_bf16 [rows, cols] or NULL; with a residual h_out_bf16 [rows, cols]
 *   is required and receives h (the updated residual stream); it may be x_bf16
 *   or residual_bf16 themselves (in place).  Without one it is ignored.
 *   gamma_bf16 [cols]; beta_bf16 [cols] or NULL (= 0); eps >= 0.
 *   y_out_bf16 [rows, cols] or NULL (the normalised activation, if wanted).
 *   q [rows, cols]; qT [cols, rows] or NULL; amax_out, scale_out, scale_inv_out:
 *   one device fp32 each or NULL.
 *   workspace: tweo_workspace_bytes(TWEO_OP_LAYERNORM_QUANTIZE, rows, 1, 1) bytes,
 *   16-byte aligned (the row statistics, 16 bytes per row, and 2.3 KB of maxima),
 *   else TWEO_ERR_WORKSPACE.  After the call it holds (mean, 1/sqrt(var+eps)) as
 *   two doubles per row from byte 2304 on, which is what a backward pass needs.
 * HBM traffic: the rows are read once from memory (2 B/element, + 2 + 2 with a
 * residual); the later passes re-read them from the caches when the tensor fits
 * there; 1 B/element written per copy of the codes.
 * Errors: TWEO_ERR_INVALID_ARG (null, misaligned, negative or NaN eps, residual
 * without h_out), TWEO_ERR_UNSUPPORTED (shape), TWEO_ERR_WORKSPACE.
 */
tweo_status tweo_layernorm_quantize_e4m3(const void *x_bf16, const void *residual_bf16,
                                         const void *gamma_bf16, const void *beta_bf16, int64_t rows,
                                         int64_t cols, float eps, void *h_out_bf16, void *y_out_bf16,
                                         float *amax_out, uint8_t *q, uint8_t *qT, float *scale_out,
                                         float *scale_inv_out, void *workspace, size_t workspace_bytes,
                                         void *stream);
tweo_status tweo_layernorm_quantize_e4m3_delayed(const void *x_bf16, const void *residual_bf16,
                                                 const void *gamma_bf16, const void *beta_bf16,
                                                 int64_t rows, int64_t cols, float eps, void *state,
                                                 int bootstrap, void *h_out_bf16, void *y_out_bf16,
                                                 uint8_t *q, uint8_t *qT, void *workspace,
                                                 size_t workspace_bytes, void *stream);

/*
 * FP8 linear forward with the TWEO penalty fused into the epilogue
 * (Sec. 4.3 for the per-tensor FP8 linear; Sec. 3.3 for the penalty).
 *   acc[m,n] = sum_k dec(xq[m,k]) * dec(wq[n,k])            (fp32 accumulate)
 *   y[m,n]   = bf16( acc[m,n] * (*sx_inv) * (*sw_inv) + residual[m,n] )
 *   *penalty_sum = sum_{m,n} ( |y[m,n]| / (tau + eps) )^p   over the stored y
 * The caller forms the mean (divide by M*N), the 1/L layer average and the
 * lambda(t) weight of the total loss.  Passing the residual stream as
 * `residual` on the block's last linear makes y the block output
 * x + MLP(LN(x)) that the paper penalises.
 *   xq [M,K], wq [N,K] codes, K % 16 == 0.   sx_inv, sw_inv: device fp32.
 *   residual_bf16 [M,N] or NULL.             y_bf16 [M,N], N % 8 == 0.
 *   pen NULL (or penalty_sum NULL) = no penalty.  penalty_sum: device fp64.
 */
tweo_status tweo_fp8_linear_fwd(const uint8_t *xq, const float *sx_inv, const uint8_t *wq,
                                const float *sw_inv, const void *residual_bf16, int64_t M,
                                int64_t N, int64_t K, void *y_bf16, const tweo_penalty_cfg *pen,
                                double *penalty_sum, void *workspace, size_t workspace_bytes,
                                void *stream);

/*
 * tweo_fp8_linear_fwd for callers that cannot allocate device memory and have no
 * workspace to pass (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): the same forward GEMM with the same fused penalty, the
 * partial sums kept in a device array inside the library (tweo_static_scratch_bytes()
 * = 1 MiB per GPU, held until the process ends) instead of a workspace.  Calls no
 * hipMalloc / hipFree and no allocating routine; the array's device address is
 * looked up once per device on the first call there.
 *   Arguments, layouts, results and errors as tweo_fp8_linear_fwd, without the
 *   workspace.  The results are the same bits.
 *   Limit: with a penalty, ceil(M/64) * ceil(N/64) * 4 bytes must fit the array
 *   (M * N up to about 10^9 elements), else TWEO_ERR_UNSUPPORTED.
 *   Every call on a GPU uses that GPU's one array: calls that overlap in time on
 *   one GPU (different streams, different threads) race on it.  Nothing in it has
 *   to start at zero and nothing of an earlier call's contents is read.
 */
size_t tweo_static_scratch_bytes(void);
tweo_status tweo_fp8_linear_fwd_static(const uint8_t *xq, const float *sx_inv, const uint8_t *wq,
                                       const float *sw_inv, const void *residual_bf16, int64_t M,
                                       int64_t N, int64_t K, void *y_bf16, const tweo_penalty_cfg *pen,
                                       double *penalty_sum, void *stream);

/*
 * FP8 linear backward (autograd of the layer above under the same recipe).
 *   dx[m,k] = bf16( (sum_n dec(dyq[m,n]) dec(wq[n,k])) * (*sdy_inv) * (*sw_inv) )
 *   dw[n,k] = bf16( (sum_m dec(dyq[m,n]) dec(xq[m,k])) * (*sdy_inv) * (*sx_inv) )
 * Operands are passed with the contraction index contiguous:
 *   dyq [M,N], wqT [K,N]            for dx [M,K]   (N % 16 == 0, K % 8 == 0)
 *   dyqT [N,M], xqT [K,M]           for dw [N,K]   (M % 16 == 0, K % 8 == 0)
 * dx_bf16 or dw_bf16 may be NULL to skip that product (its operands may then
 * be NULL too).
 */
tweo_status tweo_fp8_linear_bwd(const uint8_t *dyq, const uint8_t *dyqT, const float *sdy_inv,
                                const uint8_t *wqT, const float *sw_inv, const uint8_t *xqT,
                                const float *sx_inv, int64_t M, int64_t N, int64_t K,
                                void *dx_bf16, void *dw_bf16, void *workspace,
                                size_t workspace_bytes, void *stream);

/*
 * The same backward GEMMs with the gradient in E5M2 (HYBRID recipe, Sec. 4.3):
 * dyq / dyqT hold E5M2 codes (tweo_quantize_e5m2), wqT / xqT E4M3 codes.
 * Arguments, layouts and errors as tweo_fp8_linear_bwd.
 */
tweo_status tweo_fp8_linear_bwd_hybrid(const uint8_t *dyq, const uint8_t *dyqT, const float *sdy_inv,
                                       const uint8_t *wqT, const float *sw_inv, const uint8_t *xqT,
                                       const float *sx_inv, int64_t M, int64_t N, int64_t K,
                                       void *dx_bf16, void *dw_bf16, void *workspace,
                                       size_t workspace_bytes, void *stream);

/*
 * Gradient of the TWEO penalty, added to the incoming output gradient before it
 * is cast for the backward GEMMs.  Not printed in the paper: it is the
 * derivative of the loss of Sec. 3.3 (lambda / L * mean (|a| / (tau+eps))^p)
 * with respect to the penalised activation a:
 *   out[i] = bf16( dy[i] + g * p * sign(a[i]) * (|a[i]| / (tau+eps))^(p-1) / (tau+eps) ),
 * g = lambda / (L * numel) chosen by the caller.  fp32 arithmetic.
 *   dy_bf16, a_bf16, out_bf16 [n] device, 16-byte aligned, n % 8 == 0; out may
 *   be dy (in place).  sign(0) = 0; a NaN activation gives a NaN gradient.
 * Errors: TWEO_ERR_INVALID_ARG (null, misaligned, tau <= 0, eps < 0, NaN g),
 * TWEO_ERR_UNSUPPORTED (n % 8 != 0, p outside 1..8).
 */
tweo_status tweo_penalty_grad_inject(const void *dy_bf16, const void *a_bf16, int64_t n,
                                     const tweo_penalty_cfg *pen, float g, void *out_bf16,
                                     void *stream);

/*
 * Static per-tensor INT8 quantisation (Sec. 4.4 Eq. 4 with b = 8, Q_8 = 127):
 *   out[i] = clamp( rne( fp32(x[i]) * inv_step ), -127, 127 ),  inv_step = 127 / s
 * computed once by the caller from the calibration amax.  NaN -> 0.
 *   x_bf16 [n], n % 8 == 0.
 */
tweo_status tweo_quantize_i8(const void *x_bf16, int64_t n, float inv_step, int8_t *out,
                             void *stream);

/*
 * W8A8 per-tensor static INT8 linear (Sec. 4.4): exact int32 accumulation,
 *   y[m,n] = bf16( fp32( sum_k xq[m,k] wq[n,k] ) * alpha ),  alpha = step_x * step_w.
 *   xq [M,K], wq [N,K] int8, K % 16 == 0; y_bf16 [M,N], N % 8 == 0.
 * Bit-exact for every M (including the weight-streaming path used for small M).
 */
tweo_status tweo_w8a8_linear(const int8_t *xq, const int8_t *wq, int64_t M, int64_t N, int64_t K,
                             float alpha, void *y_bf16, void *workspace, size_t workspace_bytes,
                             void *stream);

/*
 * AbsMax INT8 quantisation with one s per row (Sec. 4.4 Eq. 4 at the "per-token"
 * granularity for activations [tokens, features] and at the "per-channel"
 * granularity for weights [out, in]), computed from the data in the same call:
 *   s_r = max_c |x[r,c]| + eps            (fp32)
 *   q[r,c] = clamp( rne( fp32(x[r,c]) * (127 / s_r) ), -127, 127 )
 *   step_out[r] = s_r / 127               (the factor X_deq applies to q)
 * 127 / s_r and s_r / 127 are single fp32 divisions.  A NaN in a row gives that
 * row step NaN and codes 0; a row of zeros with eps = 0 gives step 0 and codes 0.
 *   x_bf16 [rows, cols] device, 16-byte aligned, cols % 8 == 0; q int8
 *   [rows, cols] device, 16-byte aligned; step_out fp32 [rows] device.
 * Errors: TWEO_ERR_INVALID_ARG (null, misaligned, eps negative or NaN),
 * TWEO_ERR_UNSUPPORTED (cols % 8 != 0, a dimension above 2^24).
 */
tweo_status tweo_quantize_i8_rows(const void *x_bf16, int64_t rows, int64_t cols, float eps,
                                  int8_t *q, float *step_out, void *stream);

/*
 * W8A8 linear with finer step granularities (Sec. 4.4: per-token activations
 * "K", per-channel weights "C", combined freely with per-tensor "T"):
 *   y[m,n] = bf16( ( fp32( sum_k xq[m,k] wq[n,k] ) * x_step[m or 0] ) * w_step[n or 0] )
 * exact int32 accumulation, then two fp32 multiplies in this order.
 *   x_step: device fp32 [M] when x_step_per_token = 1, [1] when 0;
 *   w_step: device fp32 [N] when w_step_per_channel = 1, [1] when 0.
 *   xq [M,K], wq [N,K] int8 device, 16-byte aligned, K % 16 == 0; y_bf16 [M,N]
 *   device, 16-byte aligned, N % 8 == 0.  Needs no workspace.
 * Bit-exact for every M.  Large shapes run on the general tiled kernels, not on
 * the fastest per-tensor one: finer granularity costs throughput, as the paper
 * says of it.
 * Errors: TWEO_ERR_INVALID_ARG (null, misaligned, a flag other than 0 / 1),
 * TWEO_ERR_UNSUPPORTED (shape rules above).
 */
tweo_status tweo_w8a8_linear_scaled(const int8_t *xq, const int8_t *wq, int64_t M, int64_t N,
                                    int64_t K, const float *x_step, int x_step_per_token,
                                    const float *w_step, int w_step_per_channel, void *y_bf16,
                                    void *stream);

/*
 * The same linear with an INT8 result, for a pipeline whose residual stream is
 * itself quantised (Sec. 4.4, the "Res.? Yes" rows of the residual-stream
 * table): Eq. 4 with a static per-tensor s_out applied to the fp32 result,
 *   yq[m,n] = clamp( rne( ((fp32(acc) * x_step[m or 0]) * w_step[n or 0]) * inv_step_out ), -127, 127 ),
 * inv_step_out = 127 / s_out computed once by the caller; the fp32 value is not
 * rounded to bf16 in between; NaN -> 0.  yq int8 [M,N] device, 16-byte aligned;
 * everything else as tweo_w8a8_linear_scaled.  Errors as there, plus
 * TWEO_ERR_INVALID_ARG for a NaN inv_step_out.
 */
tweo_status tweo_w8a8_linear_scaled_i8out(const int8_t *xq, const int8_t *wq, int64_t M, int64_t N,
                                          int64_t K, const float *x_step, int x_step_per_token,
                                          const float *w_step, int w_step_per_channel,
                                          float inv_step_out, int8_t *yq, void *stream);

/*
 * State a forward pass leaves for the backward pass: the quantized operands,
 * their transposes and the per-tensor scalars.  All members are device
 * pointers to caller-owned buffers.
 *   xq [M,K], xqT [K,M], wq [N,K], wqT [K,N]
 *   scalars: 16 fp32: [0] amax_x [1] sx [2] sx_inv [3] amax_w [4] sw [5] sw_inv
 *                     [6] amax_dy [7] sdy [8] sdy_inv, rest reserved.
 */
typedef struct {
    uint8_t *xq;
    uint8_t *xqT;
    uint8_t *wq;
    uint8_t *wqT;
    float *scalars;
} tweo_fp8_saved;

/*
 * Whole forward path from bf16 operands: amax(x), amax(w), both quantize-casts
 * (with transposes, kept in `saved`), the FP8 GEMM and the fused penalty -
 * i.e. every step of a per-tensor FP8 linear under current scaling (Sec. 4.3)
 * plus Sec. 3.3's penalty.  M % 16 == 0, N % 16 == 0, K % 16 == 0.
 * workspace: required, 16-byte aligned, at least the first 4 KB of
 * tweo_workspace_bytes(TWEO_OP_FP8_LINEAR_FWD_BF16, ...) (plus the penalty part
 * when a penalty is asked for), else TWEO_ERR_WORKSPACE.
 */
tweo_status tweo_fp8_linear_fwd_bf16(const void *x_bf16, const void *w_bf16,
                                     const void *residual_bf16, int64_t M, int64_t N, int64_t K,
                                     void *y_bf16, const tweo_penalty_cfg *pen,
                                     double *penalty_sum, const tweo_fp8_saved *saved,
                                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * Whole backward path from a bf16 output gradient: amax(dy), quantize-cast of
 * dy (and its transpose) into dyq [M,N] / dyqT [N,M], then dgrad and wgrad on
 * the operands saved by the forward pass.  workspace: required, 16-byte
 * aligned, at least 4 KB (tweo_workspace_bytes(TWEO_OP_FP8_LINEAR_BWD_BF16, ...)),
 * else TWEO_ERR_WORKSPACE.
 */
tweo_status tweo_fp8_linear_bwd_bf16(const void *dy_bf16, const tweo_fp8_saved *saved, int64_t M,
                                     int64_t N, int64_t K, uint8_t *dyq, uint8_t *dyqT,
                                     void *dx_bf16, void *dw_bf16, void *workspace,
                                     size_t workspace_bytes, void *stream);

/* The same with dy cast to E5M2 (HYBRID recipe, Sec. 4.3). */
tweo_status tweo_fp8_linear_bwd_bf16_hybrid(const void *dy_bf16, const tweo_fp8_saved *saved, int64_t M,
                                            int64_t N, int64_t K, uint8_t *dyq, uint8_t *dyqT,
                                            void *dx_bf16, void *dw_bf16, void *workspace,
                                            size_t workspace_bytes, void *stream);

/*
 * The two whole paths under the recipe the paper trained with (Sec. 4.3: per-tensor
 * delayed scaling, amax history of 16, HYBRID formats): every tensor is read once,
 * cast with the scale its history fixed beforehand, and its own amax joins the
 * history (tweo_quantize_e4m3_delayed).  state_x, state_w, state_dy: one
 * delayed-scaling state per scaled tensor (tweo_delayed_state_init), distinct;
 * bootstrap != 0 on the first call on those states.  The activation and the weight
 * share one cast launch and one state-update launch.  saved->scalars receives, as
 * under current scaling, amax / scale used / its inverse of x (words 0-2), w (3-5)
 * and, by the backward call, dy (6-8).  dy_e5m2 = 1 casts the gradient to E5M2
 * (HYBRID), 0 to E4M3.  Shapes, workspace (that of tweo_fp8_linear_fwd /
 * tweo_fp8_linear_bwd, optional unless a penalty or a K split needs it) and errors
 * as tweo_fp8_linear_fwd_bf16 / tweo_fp8_linear_bwd_bf16.
 */
tweo_status tweo_fp8_linear_fwd_bf16_delayed(const void *x_bf16, const void *w_bf16,
                                             const void *residual_bf16, int64_t M, int64_t N, int64_t K,
                                             void *y_bf16, const tweo_penalty_cfg *pen,
                                             double *penalty_sum, const tweo_fp8_saved *saved,
                                             void *state_x, void *state_w, int bootstrap,
                                             void *workspace, size_t workspace_bytes, void *stream);
tweo_status tweo_fp8_linear_bwd_bf16_delayed(const void *dy_bf16, const tweo_fp8_saved *saved,
                                             void *state_dy, int bootstrap, int dy_e5m2, int64_t M,
                                             int64_t N, int64_t K, uint8_t *dyq, uint8_t *dyqT,
                                             void *dx_bf16, void *dw_bf16, void *workspace,
                                             size_t workspace_bytes, void *stream);

/*
 * The backward path with the penalty-gradient injection (tweo_penalty_grad_inject)
 * as a prologue of the gradient's amax and cast: dy' = bf16(dy + g * p * sign(a) *
 * (|a| / (tau+eps))^(p-1) / (tau+eps)) is formed on the way into both passes and
 * never stored; everything downstream (amax, scale, codes, GEMMs) is what
 * tweo_penalty_grad_inject followed by tweo_fp8_linear_bwd_bf16 (dy_e5m2 = 0) or
 * tweo_fp8_linear_bwd_bf16_hybrid (dy_e5m2 = 1) gives, bit for bit.  a_bf16
 * [M,N]: the penalised activation of the forward pass.  10 instead of 12 bytes
 * of traffic per gradient element, one launch less, no buffer for dy' (measured
 * on MI355X: the same time as the two calls, whose intermediate is re-read
 * from the memory-side cache).
 * Errors as the two calls it replaces.
 */
tweo_status tweo_fp8_linear_bwd_bf16_inject(const void *dy_bf16, const void *a_bf16,
                                            const tweo_penalty_cfg *pen, float g, int dy_e5m2,
                                            const tweo_fp8_saved *saved, int64_t M, int64_t N,
                                            int64_t K, uint8_t *dyq, uint8_t *dyqT, void *dx_bf16,
                                            void *dw_bf16, void *workspace, size_t workspace_bytes,
                                            void *stream);

/*
 * amax, scale and cast of one tensor in one call (Sec. 4.3, current scaling: the
 * scale comes from this tensor's own amax; E4M3 range +-448, Sec. 1; e5m2 != 0:
 * the gradient format of the HYBRID recipe, range +-57344).  The same results as
 * tweo_amax followed by tweo_quantize_e4m3 / tweo_quantize_e5m2; from 2^24
 * elements on it is one launch that keeps the tensor on chip between the two steps
 * (see tweo_set_fused_cast below), otherwise two launches.
 *   x_bf16 [rows, cols], rows % 16 == 0 and cols % 16 == 0.
 *   amax_out, scale_out, scale_inv_out: one fp32 each on the device, all required.
 *   q [rows, cols] and qT [cols, rows] codes, both required.
 *   workspace: at least 4096 bytes of device memory, 16-byte aligned, contents
 *   arbitrary (TWEO_ERR_WORKSPACE otherwise).
 */
tweo_status tweo_amax_quantize_f8(const void *x_bf16, int64_t rows, int64_t cols, int e5m2,
                                  float *amax_out, uint8_t *q, uint8_t *qT, float *scale_out,
                                  float *scale_inv_out, void *workspace, size_t workspace_bytes,
                                  void *stream);

/*
 * Sec. 4.3, current scaling.  tweo_amax_quantize_f8 and the bf16 entry points
 * (tweo_fp8_linear_fwd_bf16, tweo_fp8_linear_bwd_bf16 and its hybrid form) take the amax and cast their
 * tensors in ONE launch that holds the data in registers between the two steps
 * (4 instead of 6 bytes of traffic per element for what fits the chip).  That
 * kernel waits inside for all of its workgroups, one per CU, so all of them must be
 * able to run at the same time.  One stream, or several streams that do not run two
 * of these entry points at the same moment, need nothing.  A caller that lets them
 * overlap on one device (each launch could hold a part of the CUs and wait for the
 * rest) calls tweo_set_fused_cast(0) first: the entry points then use one amax and
 * one cast launch as before, with identical results.  Process-wide, not thread
 * safe, default 1.  Under stream capture the two-launch form is always used.
 * The wait is bounded (about 0.1 s): a launch that gives up makes the amax and the
 * scales it returns NaN and counts itself; tweo_fused_cast_timeouts copies that
 * per-device count to *count (host pointer; synchronises with the device; 0 in
 * any correct run).
 */
tweo_status tweo_set_fused_cast(int on);
tweo_status tweo_fused_cast_timeouts(unsigned *count);

/*
 * Tuning hook for benchmarks and tests: forces the GEMM kernel variant.
 * 0 = choose from the shape (the default).  1, 3, 4 = register-staged kernel, tiles
 * 256x256, 128x128, 64x64 (any K % 16 == 0).  6, 8 = DMA-pipelined kernel with
 * 64-byte stages (K % 64 == 0): 256x256 with 8 waves, 128x128.  11, 13, 14 =
 * persistent streaming kernel with 128-byte stages (K % 128 == 0): 256x256,
 * 128x128, 192x256.  15 = the deferred-epilogue persistent kernel (256x256 tiles, M
 * and N multiples of 256, K a multiple of 128 and at least 512, no residual, p in
 * {0, 4}); it falls back to variant 11 otherwise.  16 = the same kernel on 192x256
 * tiles (any M, N a multiple of 256, K a multiple of 128 and at least 2048); it
 * falls back to variant 14 otherwise.  17 (INT8 only, M <= 128, K % 64 == 0,
 * N % 4 == 0; M <= 256 when K >= 8192 and N <= 16 x the CU count) = the
 * weight-streaming kernel (what such shapes get anyway);
 * elsewhere it means variant 4.  A variant whose K requirement is not met falls
 * back to the nearest one that fits.  Results are identical up to the fp32
 * summation order.  Returns TWEO_ERR_INVALID_ARG for an unknown (or retired:
 * 2, 5, 7, 9, 10, 12) variant.
 * This setter, tweo_set_stream_k and tweo_profile_gemm_launches are test and
 * measurement knobs: process-wide, not thread safe; they change which kernel ANY
 * caller's next launch takes and what tweo_workspace_bytes() returns, so set them
 * before sizing workspaces, from one thread, and never in production code.
 */
tweo_status tweo_set_gemm_tile(int variant);

/*
 * Measurement hook for benchmarks: the next `pairs` GEMM kernels (FP8 or INT8, any
 * entry point) or reduction kernels of tweo_amax that the library launches record events[2i] when the
 * kernel starts and events[2i + 1] when it ends, i.e. the kernel's own duration
 * (events recorded on the stream around a call also time the gap that recording
 * them opens in front of the kernel).  `events`: host array of 2 * pairs
 * hipEvent_t handles created by the caller with timing enabled; at most 8
 * pairs; pairs = 0 cancels.  Process-wide, not thread safe.  Returns
 * TWEO_ERR_INVALID_ARG for a null handle, TWEO_ERR_UNSUPPORTED for more than 8
 * pairs.
 */
tweo_status tweo_profile_gemm_launches(void *const *events, int pairs);

/* Switch the K-splitting of a GEMM's last, partial round of tiles (see
 * tweo_workspace_bytes) on (non-zero) or off (0, the default: on MI355X the
 * plain schedule measured faster).  Process-wide, not thread safe. */
tweo_status tweo_set_stream_k(int on);

#ifdef __cplusplus
}
#endif
#endif /* TWEO_H */
