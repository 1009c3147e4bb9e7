// Host-side launchers of the HIP kernels (internal to the library; the public
// surface is include/tweo.h).  Every launcher enqueues on `s` and returns
// hipGetLastError().
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace tweo {

hipError_t launch_fill_u32(uint32_t *p, int n, uint32_t v, hipStream_t s);
hipError_t launch_amax(const void *x_bf16, int64_t n, float *amax_zeroed, hipStream_t s);
// two tensors (element counts multiples of 8) in one launch
hipError_t launch_amax2(const void *x0_bf16, int64_t n0, float *amax0_zeroed, const void *x1_bf16, int64_t n1,
                        float *amax1_zeroed, hipStream_t s);
// two tensors (rows and cols multiples of 16), each with its transposed copy, in one launch; with
// partials (from launch_amax2_partials) each workgroup first takes the maximum over them and
// workgroup 0 stores it to *amax, else *amax is read
hipError_t launch_quantize2_e4m3(const void *x0_bf16, int64_t rows0, int64_t cols0, float *amax0, uint8_t *q0,
                                 uint8_t *q0T, float *scale0, float *scale0_inv, const void *x1_bf16,
                                 int64_t rows1, int64_t cols1, float *amax1, uint8_t *q1, uint8_t *q1T,
                                 float *scale1, float *scale1_inv, hipStream_t s,
                                 const uint32_t *partials0 = nullptr, int n_partials0 = 0,
                                 const uint32_t *partials1 = nullptr, int n_partials1 = 0);
// amax without a cleared output and without atomics: one maximum (fp32 bit pattern) per workgroup
// into partials[0 .. *blocks), at most kAmaxPartialsMax of them per tensor
constexpr int kAmaxPartialsMax = 512;
hipError_t launch_amax_partials(const void *x_bf16, int64_t n, uint32_t *partials, int *blocks, hipStream_t s);
hipError_t launch_amax2_partials(const void *x0_bf16, int64_t n0, uint32_t *partials0, int *blocks0,
                                 const void *x1_bf16, int64_t n1, uint32_t *partials1, int *blocks1, hipStream_t s);
// the cast that consumes them (rows, cols multiples of 16); stores the maximum to *amax_out
// amax and cast of one or two tensors (x1 may be nullptr) in one launch that keeps the data on
// chip between the two; fused_cast_applies says whether a call can take it (shapes, capture, the
// switch); transposed_later: the transposed codes are not read before a later call (streaming stores); slots: kFusedMaxWorkgroups * 16 bytes of the caller's workspace, contents arbitrary.
constexpr int kFusedMaxWorkgroups = 256;
bool fused_cast_applies(int64_t rows0, int64_t cols0, int64_t rows1, int64_t cols1, hipStream_t s);
hipError_t launch_amax_cast_fused(const void *x0_bf16, int64_t rows0, int64_t cols0, float *amax0, uint8_t *q0,
                                  uint8_t *q0T, float *scale0, float *scale0_inv, const void *x1_bf16,
                                  int64_t rows1, int64_t cols1, float *amax1, uint8_t *q1, uint8_t *q1T,
                                  float *scale1, float *scale1_inv, bool e5m2, bool transposed_later, void *slots,
                                  hipStream_t s);
void set_fused_cast(bool on);
bool fused_cast_enabled();
hipError_t fused_cast_timeouts(uint32_t *count);
hipError_t launch_quantize_f8_from_partials(const void *x_bf16, int64_t rows, int64_t cols,
                                            const uint32_t *amax_partials, int n_partials, bool e5m2,
                                            float *amax_out, uint8_t *q, uint8_t *qT, float *scale_out,
                                            float *scale_inv_out, hipStream_t s);
hipError_t launch_quantize_e4m3(const void *x_bf16, int64_t rows, int64_t cols, const float *amax,
                                uint8_t *q, uint8_t *qT, float *scale_out, float *scale_inv_out,
                                hipStream_t s);
// the same cast into E5M2 (range +-57344), the gradient format of the HYBRID recipe
hipError_t launch_quantize_e5m2(const void *x_bf16, int64_t rows, int64_t cols, const float *amax,
                                uint8_t *q, uint8_t *qT, float *scale_out, float *scale_inv_out,
                                hipStream_t s);
hipError_t launch_delayed_state_init(void *state, hipStream_t s);
// sc_out (optional): three fp32 of the caller's - the tensor's amax, the scale its cast used, its inverse
hipError_t launch_quantize_e4m3_delayed(const void *x_bf16, int64_t rows, int64_t cols, void *state,
                                        int bootstrap, uint8_t *q, uint8_t *qT, hipStream_t s,
                                        float *sc_out = nullptr);
// the same for a tensor cast to E5M2 (gradients of the HYBRID recipe): scale = 57344 / max(history)
hipError_t launch_quantize_e5m2_delayed(const void *x_bf16, int64_t rows, int64_t cols, void *state,
                                        int bootstrap, uint8_t *q, uint8_t *qT, hipStream_t s,
                                        float *sc_out = nullptr);
// two tensors (rows, cols multiples of 16; transposed copies required) on their two states: one
// cast launch and one state-update launch
hipError_t launch_quantize2_e4m3_delayed(const void *x0_bf16, int64_t rows0, int64_t cols0, void *state0, uint8_t *q0,
                                         uint8_t *q0T, float *sc0, const void *x1_bf16, int64_t rows1, int64_t cols1,
                                         void *state1, uint8_t *q1, uint8_t *q1T, float *sc1, int bootstrap,
                                         hipStream_t s);
// LayerNorm of x (or of h = bf16(x + res), stored to h_out) followed by the per-tensor E4M3 cast of
// the normalised tensor; state == nullptr: current scaling (amax_out required), else delayed
// scaling on that state.  stats: 2 doubles per row, partials: kAmaxPartialsMax words of scratch.
hipError_t launch_layernorm_quantize(const void *x_bf16, const void *res_bf16, const void *gamma_bf16,
                                     const void *beta_bf16, int64_t rows, int64_t cols, double eps, void *h_out,
                                     void *y_out, uint8_t *q, uint8_t *qT, double *stats, uint32_t *partials,
                                     float *amax_out, float *scale_out, float *scale_inv_out, void *state,
                                     int bootstrap, hipStream_t s);
hipError_t launch_quantize_i8(const void *x_bf16, int64_t n, float inv_step, int8_t *out,
                              hipStream_t s);
// Row-granular AbsMax INT8: q [rows, cols] and one dequantisation step per row (cols % 8 == 0).
hipError_t launch_quantize_i8_rows(const void *x_bf16, int64_t rows, int64_t cols, float eps, int8_t *q,
                                   float *step, hipStream_t s);
hipError_t launch_penalty_finish(const float *partials, int n, double *out, hipStream_t s);
hipError_t launch_penalty_grad_inject(const void *dy_bf16, const void *a_bf16, int64_t n, float inv_tau,
                                      float coef, int p, void *out_bf16, hipStream_t s);
// the injection fused into the gradient's amax and cast launches (rows, cols multiples of 16;
// partials: kAmaxPartialsMax words of scratch)
hipError_t launch_amax_quantize_inject(const void *dy_bf16, const void *a_bf16, int64_t rows, int64_t cols,
                                       float inv_tau, float coef, int p, bool e5m2, uint32_t *partials,
                                       float *amax_out, uint8_t *q, uint8_t *qT, float *scale_out,
                                       float *scale_inv_out, hipStream_t s);

// C[M,N] = A[M,K] * B[N,K]^T on 8-bit operands, both K-contiguous.
struct GemmArgs {
    const uint8_t *A;
    const uint8_t *B;
    int64_t M, N, K;
    const float *s0;        // FP8: alpha = (*s0) * (*s1), device scalars
    const float *s1;
    float alpha;            // INT8: host scalar
    const void *residual;   // bf16 [M,N] or nullptr (FP8 only)
    void *out;              // bf16 [M,N]
    float inv_tau;          // 1 / (tau + eps)
    int p;                  // penalty power; 0 = no penalty
    float *partials;        // one fp32 per workgroup when p != 0
    bool a_e5m2;            // FP8 only: A holds E5M2 codes (B is always E4M3)
    void *sk_workspace;     // stream-K scratch (256-byte aligned) or nullptr: then no stream-K
    size_t sk_workspace_bytes;
    // INT8 only, both or neither: device vectors of dequantisation steps, per row of A (stride 1)
    // or one for all (stride 0), likewise per row of B; alpha is ignored when they are given
    const float *row_step, *col_step;
    int row_step_stride, col_step_stride;
    // with step vectors only: `out` is int8 [M,N], the fp32 result times out_inv_step rounded to INT8
    bool out_i8;
    float out_inv_step;
};

// Number of fp32 penalty partials the FP8 GEMM writes for these arguments.
int fp8_gemm_partials(const GemmArgs &a);
hipError_t launch_fp8_gemm(const GemmArgs &a, hipStream_t s);
hipError_t launch_i8_gemm(const GemmArgs &a, hipStream_t s);

// K split of tile-starved FP8 GEMMs (no penalty, no residual): number of runs (1 = none) and the
// fp32 scratch they need; given through sk_workspace like the stream-K scratch, which it shares.
int fp8_gemm_ksplit(int64_t M, int64_t N, int64_t K);
size_t fp8_gemm_ksplit_bytes(int64_t M, int64_t N, int64_t K);

// Bytes of stream-K scratch that let every shape use it on this device.
size_t stream_k_workspace_bytes();
void set_stream_k(bool on);
bool stream_k_enabled();

// Measurement hook: the next `pairs` GEMM kernel launches record events[2i] at their start and
// events[2i+1] at their end (hipEvent_t handles); false if pairs is out of range.
bool set_profile_events(void *const *events, int pairs);
// the next armed pair, if any (consumed): a launch that takes one records them at its start and end
bool take_profile_events(hipEvent_t *e0, hipEvent_t *e1);

// Tile-shape override for benchmarking sweeps: 0 = heuristic.
void set_gemm_tile_override(int variant);
int gemm_num_variants();
bool gemm_variant_exists(int v);

}  // namespace tweo
