// C ABI of the library (include/tweo.h): argument validation and dispatch.
// Nothing here allocates, frees or synchronises; everything is enqueued on the
// caller's stream.
#include <algorithm>
#include "../../include/tweo.h"
#include "kernels.h"

using namespace tweo;

namespace {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round256(size_t b) { return b == 0 ? 256 : (b + 255) / 256 * 256; }
inline tweo_status hip_status(hipError_t e) { return e == hipSuccess ? TWEO_OK : TWEO_ERR_HIP; }
constexpr int64_t kMaxDim = (int64_t)1 << 30;

inline bool dims_ok(int64_t M, int64_t N, int64_t K)
{
    // N <= 2^24 and K <= 2^24 keep the kernels' 32-bit row offsets (up to 256 rows) in range
    return M > 0 && N > 0 && K > 0 && M <= kMaxDim && N <= ((int64_t)1 << 24) &&
           K <= ((int64_t)1 << 24) && M * N < ((int64_t)1 << 40);
}

// upper bound on the number of penalty partials for any kernel (one per workgroup of the tiled
// kernels, whose tiles are at least 64x64; the persistent kernels write fewer)
inline size_t partial_slots(int64_t M, int64_t N) { return (size_t)(((M + 63) / 64) * ((N + 63) / 64)); }

tweo_status check_penalty(const tweo_penalty_cfg *pen, double *penalty_sum, float &inv_tau, int &p)
{
    p = 0;
    inv_tau = 0.0f;
    if (!pen || !penalty_sum)
        return TWEO_OK;
    if (!(pen->tau > 0.0f) || !(pen->eps >= 0.0f))
        return TWEO_ERR_INVALID_ARG;
    if (pen->p < 1 || pen->p > 8)
        return TWEO_ERR_UNSUPPORTED;
    inv_tau = (float)(1.0 / ((double)pen->tau + (double)pen->eps));
    p = pen->p;
    return TWEO_OK;
}

}  // namespace

extern "C" {

const char *tweo_status_string(tweo_status s)
{
    switch (s) {
    case TWEO_OK: return "ok";
    case TWEO_ERR_INVALID_ARG: return "invalid argument";
    case TWEO_ERR_UNSUPPORTED: return "unsupported shape or option";
    case TWEO_ERR_WORKSPACE: return "workspace missing or too small";
    case TWEO_ERR_HIP: return "HIP launch failed";
    }
    return "unknown status";
}

tweo_status tweo_set_stream_k(int on)
{
    set_stream_k(on != 0);
    return TWEO_OK;
}

tweo_status tweo_profile_gemm_launches(void *const *events, int pairs)
{
    if (pairs < 0 || (pairs > 0 && !events))
        return TWEO_ERR_INVALID_ARG;
    for (int i = 0; i < 2 * pairs; ++i)
        if (!events[i])
            return TWEO_ERR_INVALID_ARG;
    return set_profile_events(events, pairs) ? TWEO_OK : TWEO_ERR_UNSUPPORTED;
}

tweo_status tweo_set_fused_cast(int on)
{
    set_fused_cast(on != 0);
    return TWEO_OK;
}

tweo_status tweo_fused_cast_timeouts(unsigned *count)
{
    if (!count)
        return TWEO_ERR_INVALID_ARG;
    uint32_t c = 0;
    if (fused_cast_timeouts(&c) != hipSuccess)
        return TWEO_ERR_HIP;
    *count = c;
    return TWEO_OK;
}

tweo_status tweo_set_gemm_tile(int variant)
{
    if (!gemm_variant_exists(variant))
        return TWEO_ERR_INVALID_ARG;
    set_gemm_tile_override(variant);
    return TWEO_OK;
}

// Workspace layout: penalty partials (forward only), then the stream-K scratch.  The scratch is
// asked for only while stream-K is switched on and a contraction is long enough for it to be
// considered; a caller that passes less simply gets the plain schedule.
inline size_t penalty_bytes(int64_t M, int64_t N) { return round256(partial_slots(M, N) * sizeof(float)); }
inline bool stream_k_candidate(int64_t rows, int64_t cols, int64_t contraction)
{
    return stream_k_enabled() && contraction >= 2048 && rows >= 256 && cols >= 256;
}

// head of the workspace of the bf16 entry points: two runs of kAmaxPartialsMax workgroup maxima
constexpr size_t kAmaxScratchBytes = 2 * kAmaxPartialsMax * sizeof(uint32_t);

size_t tweo_workspace_bytes(int op, int64_t M, int64_t N, int64_t K)
{
    if (M <= 0 || N <= 0 || K <= 0)
        return 256;
    switch (op) {
    case TWEO_OP_FP8_LINEAR_FWD:
        return penalty_bytes(M, N) + round256(std::max(stream_k_candidate(M, N, K) ? stream_k_workspace_bytes() : 0,
                                                       fp8_gemm_ksplit_bytes(M, N, K)));
    case TWEO_OP_FP8_LINEAR_FWD_BF16:  // the workgroup maxima of the amax launch in front
        return kAmaxScratchBytes + tweo_workspace_bytes(TWEO_OP_FP8_LINEAR_FWD, M, N, K);
    case TWEO_OP_FP8_LINEAR_BWD:  // dgrad [M,K] over N, wgrad [N,K] over M
        return 256 + round256(std::max({stream_k_candidate(M, K, N) || stream_k_candidate(N, K, M)
                                            ? stream_k_workspace_bytes() : (size_t)0,
                                        fp8_gemm_ksplit_bytes(M, K, N), fp8_gemm_ksplit_bytes(N, K, M)}));
    case TWEO_OP_FP8_LINEAR_BWD_BF16:
        return kAmaxScratchBytes + tweo_workspace_bytes(TWEO_OP_FP8_LINEAR_BWD, M, N, K);
    case TWEO_OP_W8A8_LINEAR:
        return 256 + round256(std::max(stream_k_candidate(M, N, K) ? stream_k_workspace_bytes() : (size_t)0,
                                       fp8_gemm_ksplit_bytes(M, N, K)));
    case TWEO_OP_LAYERNORM_QUANTIZE:  // M rows (N, K unused)
        return kAmaxPartialsMax * sizeof(uint32_t) + 256 + round256((size_t)M * 2 * sizeof(double));
    default:
        return 256;
    }
}

namespace {
// the stream-K part of a caller's workspace that starts `skip` bytes in (or nothing)
inline void attach_stream_k(GemmArgs &a, void *workspace, size_t workspace_bytes, size_t skip)
{
    a.sk_workspace = nullptr;
    a.sk_workspace_bytes = 0;
    if (workspace && aligned16(workspace) && ((reinterpret_cast<uintptr_t>(workspace) + skip) & 255u) == 0 &&
        workspace_bytes > skip) {
        a.sk_workspace = (uint8_t *)workspace + skip;
        a.sk_workspace_bytes = workspace_bytes - skip;
    }
}
}  // namespace

tweo_status tweo_amax(const void *x_bf16, int64_t n, float *amax_out, void *stream)
{
    if (!x_bf16 || !amax_out || n <= 0 || !aligned16(x_bf16))
        return TWEO_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = launch_fill_u32((uint32_t *)amax_out, 1, 0u, s);
    if (e != hipSuccess)
        return TWEO_ERR_HIP;
    return hip_status(launch_amax(x_bf16, n, amax_out, s));
}

tweo_status tweo_quantize_e4m3(const void *x_bf16, int64_t rows, int64_t cols, const float *amax,
                               uint8_t *q, uint8_t *qT, float *scale_out, float *scale_inv_out,
                               void *stream)
{
    if (!x_bf16 || !amax || !q || rows <= 0 || cols <= 0 || !aligned16(x_bf16) || !aligned16(q) ||
        (qT && !aligned16(qT)))
        return TWEO_ERR_INVALID_ARG;
    if (cols % 8 != 0 || rows > kMaxDim || cols > kMaxDim)
        return TWEO_ERR_UNSUPPORTED;
    return hip_status(launch_quantize_e4m3(x_bf16, rows, cols, amax, q, qT, scale_out,
                                           scale_inv_out, (hipStream_t)stream));
}

tweo_status tweo_quantize_e5m2(const void *x_bf16, int64_t rows, int64_t cols, const float *amax,
                               uint8_t *q, uint8_t *qT, float *scale_out, float *scale_inv_out,
                               void *stream)
{
    if (!x_bf16 || !amax || !q || rows <= 0 || cols <= 0 || !aligned16(x_bf16) || !aligned16(q) ||
        (qT && !aligned16(qT)))
        return TWEO_ERR_INVALID_ARG;
    if (cols % 8 != 0 || rows > kMaxDim || cols > kMaxDim)
        return TWEO_ERR_UNSUPPORTED;
    return hip_status(launch_quantize_e5m2(x_bf16, rows, cols, amax, q, qT, scale_out,
                                           scale_inv_out, (hipStream_t)stream));
}

tweo_status tweo_amax_quantize_f8(const void *x_bf16, int64_t rows, int64_t cols, int e5m2,
                                  float *amax_out, uint8_t *q, uint8_t *qT, float *scale_out,
                                  float *scale_inv_out, void *workspace, size_t workspace_bytes,
                                  void *stream)
{
    if (!x_bf16 || !amax_out || !q || !qT || !scale_out || !scale_inv_out || rows <= 0 || cols <= 0 ||
        !aligned16(x_bf16) || !aligned16(q) || !aligned16(qT))
        return TWEO_ERR_INVALID_ARG;
    if (rows % 16 != 0 || cols % 16 != 0 || rows > kMaxDim || cols > kMaxDim)
        return TWEO_ERR_UNSUPPORTED;
    if (!workspace || !aligned16(workspace) || workspace_bytes < kAmaxScratchBytes)
        return TWEO_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    if (fused_cast_applies(rows, cols, 0, 0, s))
        return hip_status(launch_amax_cast_fused(x_bf16, rows, cols, amax_out, q, qT, scale_out, scale_inv_out, nullptr,
                                                 0, 0, nullptr, nullptr, nullptr, nullptr, nullptr, e5m2 != 0,
                                                 false, workspace, s));
    uint32_t *partials = (uint32_t *)workspace;
    int n = 0;
    hipError_t e = launch_amax_partials(x_bf16, rows * cols, partials, &n, s);
    if (e == hipSuccess)
        e = launch_quantize_f8_from_partials(x_bf16, rows, cols, partials, n, e5m2 != 0, amax_out, q, qT, scale_out,
                                             scale_inv_out, s);
    return hip_status(e);
}

size_t tweo_delayed_state_bytes(void) { return TWEO_DELAYED_STATE_WORDS * sizeof(float); }

tweo_status tweo_delayed_state_init(void *state, void *stream)
{
    if (!state || !aligned16(state))
        return TWEO_ERR_INVALID_ARG;
    return hip_status(launch_delayed_state_init(state, (hipStream_t)stream));
}

tweo_status tweo_quantize_e4m3_delayed(const void *x_bf16, int64_t rows, int64_t cols, void *state,
                                       int bootstrap, uint8_t *q, uint8_t *qT, void *stream)
{
    if (!x_bf16 || !state || !q || rows <= 0 || cols <= 0 || !aligned16(x_bf16) || !aligned16(q) ||
        !aligned16(state) || (qT && !aligned16(qT)))
        return TWEO_ERR_INVALID_ARG;
    if (cols % 8 != 0 || rows > kMaxDim || cols > kMaxDim)
        return TWEO_ERR_UNSUPPORTED;
    return hip_status(launch_quantize_e4m3_delayed(x_bf16, rows, cols, state, bootstrap != 0, q, qT,
                                                   (hipStream_t)stream));
}

tweo_status tweo_quantize_e5m2_delayed(const void *x_bf16, int64_t rows, int64_t cols, void *state,
                                       int bootstrap, uint8_t *q, uint8_t *qT, void *stream)
{
    if (!x_bf16 || !state || !q || rows <= 0 || cols <= 0 || !aligned16(x_bf16) || !aligned16(q) ||
        !aligned16(state) || (qT && !aligned16(qT)))
        return TWEO_ERR_INVALID_ARG;
    if (cols % 8 != 0 || rows > kMaxDim || cols > kMaxDim)
        return TWEO_ERR_UNSUPPORTED;
    return hip_status(launch_quantize_e5m2_delayed(x_bf16, rows, cols, state, bootstrap != 0, q, qT,
                                                   (hipStream_t)stream));
}

tweo_status tweo_fp8_linear_fwd(const uint8_t *xq, const float *sx_inv, const uint8_t *wq,
                                const float *sw_inv, const void *residual_bf16, int64_t M,
                                int64_t N, int64_t K, void *y_bf16, const tweo_penalty_cfg *pen,
                                double *penalty_sum, void *workspace, size_t workspace_bytes,
                                void *stream)
{
    if (!xq || !sx_inv || !wq || !sw_inv || !y_bf16 || M <= 0 || N <= 0 || K <= 0 ||
        !aligned16(xq) || !aligned16(wq) || !aligned16(y_bf16) ||
        (residual_bf16 && !aligned16(residual_bf16)))
        return TWEO_ERR_INVALID_ARG;
    if (!dims_ok(M, N, K) || K % 16 != 0 || N % 8 != 0)
        return TWEO_ERR_UNSUPPORTED;
    float inv_tau;
    int p;
    tweo_status st = check_penalty(pen, penalty_sum, inv_tau, p);
    if (st != TWEO_OK)
        return st;
    if (p != 0 && (!workspace || workspace_bytes < penalty_bytes(M, N) || !aligned16(workspace)))
        return TWEO_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    GemmArgs a{};
    a.A = xq;
    a.B = wq;
    a.M = M;
    a.N = N;
    a.K = K;
    a.s0 = sx_inv;
    a.s1 = sw_inv;
    a.residual = residual_bf16;
    a.out = y_bf16;
    a.inv_tau = inv_tau;
    a.p = p;
    a.partials = (float *)workspace;
    attach_stream_k(a, workspace, workspace_bytes, penalty_bytes(M, N));
    hipError_t e = launch_fp8_gemm(a, s);
    if (e != hipSuccess)
        return TWEO_ERR_HIP;
    if (p != 0)
        e = launch_penalty_finish((const float *)workspace, fp8_gemm_partials(a), penalty_sum, s);
    return hip_status(e);
}

// ---------------------------------------------------------------------------
// The forward entry point for callers that cannot allocate: the penalty partial sums live in a
// file-scope device array instead of a caller's workspace.  Each GPU holds its own copy of the
// array at its own address; the address is looked up once per device (with that device current)
// and kept.  Host code never uses the array's name for anything but that lookup.
constexpr size_t kStaticScratchBytes = (size_t)1 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};

tweo_status static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return TWEO_ERR_HIP;
    void *p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (p == nullptr) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr)
            return TWEO_ERR_HIP;
        __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE);  // every thread finds the same address
    }
    *out = p;
    return TWEO_OK;
}
}  // namespace

size_t tweo_static_scratch_bytes(void) { return kStaticScratchBytes; }

tweo_status tweo_fp8_linear_fwd_static(const uint8_t *xq, const float *sx_inv, const uint8_t *wq,
                                       const float *sw_inv, const void *residual_bf16, int64_t M,
                                       int64_t N, int64_t K, void *y_bf16, const tweo_penalty_cfg *pen,
                                       double *penalty_sum, void *stream)
{
    if (M <= 0 || N <= 0 || K <= 0)
        return TWEO_ERR_INVALID_ARG;
    if (!dims_ok(M, N, K))
        return TWEO_ERR_UNSUPPORTED;
    // the partial sums of this shape must fit the array (one fp32 per 64x64 block of the output)
    const size_t need = penalty_bytes(M, N);
    if (pen != nullptr && penalty_sum != nullptr && need > kStaticScratchBytes)
        return TWEO_ERR_UNSUPPORTED;
    void *ws = nullptr;
    tweo_status st = static_scratch(&ws);
    if (st != TWEO_OK)
        return st;
    // exactly the penalty part: no K-split or stream-K scratch is offered, so the plain schedule
    // runs.  Every slot the finishing kernel reads is written by this call's GEMM: nothing of a
    // previous call's contents is used and nothing needs clearing.
    return tweo_fp8_linear_fwd(xq, sx_inv, wq, sw_inv, residual_bf16, M, N, K, y_bf16, pen, penalty_sum, ws,
                               need < kStaticScratchBytes ? need : kStaticScratchBytes, stream);
}

static tweo_status fp8_linear_bwd_impl(const uint8_t *dyq, const uint8_t *dyqT, const float *sdy_inv,
                                       const uint8_t *wqT, const float *sw_inv, const uint8_t *xqT,
                                       const float *sx_inv, int64_t M, int64_t N, int64_t K,
                                       void *dx_bf16, void *dw_bf16, void *workspace,
                                       size_t workspace_bytes, void *stream, bool dy_e5m2)
{
    if (M <= 0 || N <= 0 || K <= 0 || !sdy_inv || (!dx_bf16 && !dw_bf16))
        return TWEO_ERR_INVALID_ARG;
    if (dx_bf16 && (!dyq || !wqT || !sw_inv || !aligned16(dyq) || !aligned16(wqT) || !aligned16(dx_bf16)))
        return TWEO_ERR_INVALID_ARG;
    if (dw_bf16 && (!dyqT || !xqT || !sx_inv || !aligned16(dyqT) || !aligned16(xqT) || !aligned16(dw_bf16)))
        return TWEO_ERR_INVALID_ARG;
    if (!dims_ok(M, N, K) || K % 8 != 0 || (dx_bf16 && N % 16 != 0) || (dw_bf16 && M % 16 != 0) ||
        M > ((int64_t)1 << 24) || N > ((int64_t)1 << 24))
        return TWEO_ERR_UNSUPPORTED;
    hipStream_t s = (hipStream_t)stream;
    if (dx_bf16) {  // dX[M,K] = dYq[M,N] * WqT[K,N]^T   (contraction over N)
        GemmArgs a{};
        a.A = dyq;
        a.B = wqT;
        a.M = M;
        a.N = K;
        a.K = N;
        a.s0 = sdy_inv;
        a.s1 = sw_inv;
        a.out = dx_bf16;
        a.a_e5m2 = dy_e5m2;
        attach_stream_k(a, workspace, workspace_bytes, 256);
        hipError_t e = launch_fp8_gemm(a, s);
        if (e != hipSuccess)
            return TWEO_ERR_HIP;
    }
    if (dw_bf16) {  // dW[N,K] = dYqT[N,M] * XqT[K,M]^T  (contraction over M)
        GemmArgs a{};
        a.A = dyqT;
        a.B = xqT;
        a.M = N;
        a.N = K;
        a.K = M;
        a.s0 = sdy_inv;
        a.s1 = sx_inv;
        a.out = dw_bf16;
        a.a_e5m2 = dy_e5m2;
        attach_stream_k(a, workspace, workspace_bytes, 256);
        hipError_t e = launch_fp8_gemm(a, s);
        if (e != hipSuccess)
            return TWEO_ERR_HIP;
    }
    return TWEO_OK;
}

tweo_status tweo_fp8_linear_bwd(const uint8_t *dyq, const uint8_t *dyqT, const float *sdy_inv,
                                const uint8_t *wqT, const float *sw_inv, const uint8_t *xqT,
                                const float *sx_inv, int64_t M, int64_t N, int64_t K,
                                void *dx_bf16, void *dw_bf16, void *workspace,
                                size_t workspace_bytes, void *stream)
{
    return fp8_linear_bwd_impl(dyq, dyqT, sdy_inv, wqT, sw_inv, xqT, sx_inv, M, N, K, dx_bf16, dw_bf16,
                               workspace, workspace_bytes, stream, false);
}

tweo_status tweo_fp8_linear_bwd_hybrid(const uint8_t *dyq, const uint8_t *dyqT, const float *sdy_inv,
                                       const uint8_t *wqT, const float *sw_inv, const uint8_t *xqT,
                                       const float *sx_inv, int64_t M, int64_t N, int64_t K,
                                       void *dx_bf16, void *dw_bf16, void *workspace,
                                       size_t workspace_bytes, void *stream)
{
    return fp8_linear_bwd_impl(dyq, dyqT, sdy_inv, wqT, sw_inv, xqT, sx_inv, M, N, K, dx_bf16, dw_bf16,
                               workspace, workspace_bytes, stream, true);
}

tweo_status tweo_penalty_grad_inject(const void *dy_bf16, const void *a_bf16, int64_t n,
                                     const tweo_penalty_cfg *pen, float g, void *out_bf16, void *stream)
{
    if (!dy_bf16 || !a_bf16 || !out_bf16 || !pen || n <= 0 || !aligned16(dy_bf16) || !aligned16(a_bf16) ||
        !aligned16(out_bf16) || !(g == g))
        return TWEO_ERR_INVALID_ARG;
    if (!(pen->tau > 0.0f) || !(pen->eps >= 0.0f))
        return TWEO_ERR_INVALID_ARG;
    if (n % 8 != 0 || pen->p < 1 || pen->p > 8)
        return TWEO_ERR_UNSUPPORTED;
    const double denom = (double)pen->tau + (double)pen->eps;
    return hip_status(launch_penalty_grad_inject(dy_bf16, a_bf16, n, (float)(1.0 / denom),
                                                 (float)((double)g * pen->p / denom), pen->p, out_bf16,
                                                 (hipStream_t)stream));
}

namespace {
// workspace of the LayerNorm entry points: the amax launch's workgroup maxima, one spare fp32 slot
// for the amax when the caller wants none, then two doubles per row
constexpr size_t kLnHeadBytes = kAmaxPartialsMax * sizeof(uint32_t) + 256;
inline size_t layernorm_bytes(int64_t rows) { return kLnHeadBytes + round256((size_t)rows * 2 * sizeof(double)); }

tweo_status layernorm_quantize_impl(const void *x_bf16, const void *residual_bf16, const void *gamma_bf16,
                                    const void *beta_bf16, int64_t rows, int64_t cols, float eps, void *state,
                                    int bootstrap, void *h_out_bf16, void *y_out_bf16, float *amax_out, uint8_t *q,
                                    uint8_t *qT, float *scale_out, float *scale_inv_out, void *workspace,
                                    size_t workspace_bytes, void *stream)
{
    if (!x_bf16 || !gamma_bf16 || !q || rows <= 0 || cols <= 0 || !aligned16(x_bf16) || !aligned16(gamma_bf16) ||
        !aligned16(q) || (beta_bf16 && !aligned16(beta_bf16)) || (qT && !aligned16(qT)) ||
        (y_out_bf16 && !aligned16(y_out_bf16)) || (state && !aligned16(state)) || !(eps >= 0.0f))
        return TWEO_ERR_INVALID_ARG;
    // a residual makes a new tensor h = x + r that the cast pass reads back: it needs a home
    if (residual_bf16 && (!h_out_bf16 || !aligned16(residual_bf16) || !aligned16(h_out_bf16)))
        return TWEO_ERR_INVALID_ARG;
    if (rows % 16 != 0 || cols % 16 != 0 || rows > kMaxDim || cols > ((int64_t)1 << 24))
        return TWEO_ERR_UNSUPPORTED;
    if (!workspace || !aligned16(workspace) || workspace_bytes < layernorm_bytes(rows))
        return TWEO_ERR_WORKSPACE;
    uint32_t *partials = (uint32_t *)workspace;
    float *spare = (float *)((uint8_t *)workspace + kAmaxPartialsMax * sizeof(uint32_t));
    double *stats = (double *)((uint8_t *)workspace + kLnHeadBytes);
    return hip_status(launch_layernorm_quantize(x_bf16, residual_bf16, gamma_bf16, beta_bf16, rows, cols, (double)eps,
                                                h_out_bf16, y_out_bf16, q, qT, stats, partials,
                                                amax_out ? amax_out : spare, scale_out, scale_inv_out, state,
                                                bootstrap != 0, (hipStream_t)stream));
}
}  // namespace

tweo_status tweo_layernorm_quantize_e4m3(const void *x_bf16, const void *residual_bf16, const void *gamma_bf16,
                                         const void *beta_bf16, int64_t rows, int64_t cols, float eps,
                                         void *h_out_bf16, void *y_out_bf16, float *amax_out, uint8_t *q, uint8_t *qT,
                                         float *scale_out, float *scale_inv_out, void *workspace,
                                         size_t workspace_bytes, void *stream)
{
    return layernorm_quantize_impl(x_bf16, residual_bf16, gamma_bf16, beta_bf16, rows, cols, eps, nullptr, 0, h_out_bf16,
                                   y_out_bf16, amax_out, q, qT, scale_out, scale_inv_out, workspace, workspace_bytes,
                                   stream);
}

tweo_status tweo_layernorm_quantize_e4m3_delayed(const void *x_bf16, const void *residual_bf16,
                                                 const void *gamma_bf16, const void *beta_bf16, int64_t rows,
                                                 int64_t cols, float eps, void *state, int bootstrap, void *h_out_bf16,
                                                 void *y_out_bf16, uint8_t *q, uint8_t *qT, void *workspace,
                                                 size_t workspace_bytes, void *stream)
{
    if (!state)
        return TWEO_ERR_INVALID_ARG;
    return layernorm_quantize_impl(x_bf16, residual_bf16, gamma_bf16, beta_bf16, rows, cols, eps, state, bootstrap,
                                   h_out_bf16, y_out_bf16, nullptr, q, qT, nullptr, nullptr, workspace, workspace_bytes,
                                   stream);
}

tweo_status tweo_quantize_i8(const void *x_bf16, int64_t n, float inv_step, int8_t *out,
                             void *stream)
{
    if (!x_bf16 || !out || n <= 0 || !aligned16(x_bf16) || !aligned16(out) || !(inv_step == inv_step))
        return TWEO_ERR_INVALID_ARG;
    if (n % 8 != 0)
        return TWEO_ERR_UNSUPPORTED;
    return hip_status(launch_quantize_i8(x_bf16, n, inv_step, out, (hipStream_t)stream));
}

tweo_status tweo_w8a8_linear(const int8_t *xq, const int8_t *wq, int64_t M, int64_t N, int64_t K,
                             float alpha, void *y_bf16, void *workspace, size_t workspace_bytes,
                             void *stream)
{
    if (!xq || !wq || !y_bf16 || M <= 0 || N <= 0 || K <= 0 || !aligned16(xq) || !aligned16(wq) ||
        !aligned16(y_bf16))
        return TWEO_ERR_INVALID_ARG;
    if (!dims_ok(M, N, K) || K % 16 != 0 || N % 8 != 0)
        return TWEO_ERR_UNSUPPORTED;
    GemmArgs a{};
    a.A = (const uint8_t *)xq;
    a.B = (const uint8_t *)wq;
    a.M = M;
    a.N = N;
    a.K = K;
    a.alpha = alpha;
    a.out = y_bf16;
    attach_stream_k(a, workspace, workspace_bytes, 256);
    return hip_status(launch_i8_gemm(a, (hipStream_t)stream));
}

tweo_status tweo_quantize_i8_rows(const void *x_bf16, int64_t rows, int64_t cols, float eps, int8_t *q,
                                  float *step_out, void *stream)
{
    if (!x_bf16 || !q || !step_out || rows <= 0 || cols <= 0 || !aligned16(x_bf16) || !aligned16(q) ||
        !(eps >= 0.0f))
        return TWEO_ERR_INVALID_ARG;
    if (cols % 8 != 0 || rows > kMaxDim || cols > kMaxDim)
        return TWEO_ERR_UNSUPPORTED;
    return hip_status(launch_quantize_i8_rows(x_bf16, rows, cols, eps, q, step_out, (hipStream_t)stream));
}

static tweo_status w8a8_linear_scaled_impl(const int8_t *xq, const int8_t *wq, int64_t M, int64_t N, int64_t K,
                                           const float *x_step, int x_step_per_token, const float *w_step,
                                           int w_step_per_channel, void *y_bf16, bool out_i8, float out_inv_step,
                                           void *stream)
{
    if (!xq || !wq || !y_bf16 || !x_step || !w_step || M <= 0 || N <= 0 || K <= 0 || !aligned16(xq) ||
        !aligned16(wq) || !aligned16(y_bf16) || (x_step_per_token != 0 && x_step_per_token != 1) ||
        (w_step_per_channel != 0 && w_step_per_channel != 1))
        return TWEO_ERR_INVALID_ARG;
    if (!dims_ok(M, N, K) || K % 16 != 0 || N % 8 != 0)
        return TWEO_ERR_UNSUPPORTED;
    GemmArgs a{};
    a.A = (const uint8_t *)xq;
    a.B = (const uint8_t *)wq;
    a.M = M;
    a.N = N;
    a.K = K;
    a.alpha = 1.0f;
    a.out = y_bf16;
    a.row_step = x_step;
    a.row_step_stride = x_step_per_token;
    a.col_step = w_step;
    a.col_step_stride = w_step_per_channel;
    a.out_i8 = out_i8;
    a.out_inv_step = out_inv_step;
    return hip_status(launch_i8_gemm(a, (hipStream_t)stream));
}

tweo_status tweo_w8a8_linear_scaled(const int8_t *xq, const int8_t *wq, int64_t M, int64_t N, int64_t K,
                                    const float *x_step, int x_step_per_token, const float *w_step,
                                    int w_step_per_channel, void *y_bf16, void *stream)
{
    return w8a8_linear_scaled_impl(xq, wq, M, N, K, x_step, x_step_per_token, w_step, w_step_per_channel, y_bf16,
                                   false, 0.0f, stream);
}

tweo_status tweo_w8a8_linear_scaled_i8out(const int8_t *xq, const int8_t *wq, int64_t M, int64_t N, int64_t K,
                                          const float *x_step, int x_step_per_token, const float *w_step,
                                          int w_step_per_channel, float inv_step_out, int8_t *yq, void *stream)
{
    if (!(inv_step_out == inv_step_out))
        return TWEO_ERR_INVALID_ARG;
    return w8a8_linear_scaled_impl(xq, wq, M, N, K, x_step, x_step_per_token, w_step, w_step_per_channel, yq, true,
                                   inv_step_out, stream);
}

tweo_status tweo_fp8_linear_fwd_bf16(const void *x_bf16, const void *w_bf16,
                                     const void *residual_bf16, int64_t M, int64_t N, int64_t K,
                                     void *y_bf16, const tweo_penalty_cfg *pen,
                                     double *penalty_sum, const tweo_fp8_saved *saved,
                                     void *workspace, size_t workspace_bytes, void *stream)
{
    if (!x_bf16 || !w_bf16 || !y_bf16 || !saved || !saved->xq || !saved->xqT || !saved->wq ||
        !saved->wqT || !saved->scalars || M <= 0 || N <= 0 || K <= 0 || !aligned16(x_bf16) ||
        !aligned16(w_bf16) || !aligned16(saved->xq) || !aligned16(saved->xqT) ||
        !aligned16(saved->wq) || !aligned16(saved->wqT) || !aligned16(saved->scalars))
        return TWEO_ERR_INVALID_ARG;
    if (!dims_ok(M, N, K) || M % 16 != 0 || N % 16 != 0 || K % 16 != 0)
        return TWEO_ERR_UNSUPPORTED;
    float inv_tau;
    int p;
    tweo_status st = check_penalty(pen, penalty_sum, inv_tau, p);
    if (st != TWEO_OK)
        return st;
    if (!workspace || !aligned16(workspace) ||
        workspace_bytes < kAmaxScratchBytes + (p != 0 ? penalty_bytes(M, N) : 0))
        return TWEO_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    float *sc = saved->scalars;
    // activation and weight share one amax launch and one cast launch (a kernel of its own for
    // the small weight tensor is mostly launch and tail latency); the amax launch leaves one
    // maximum per workgroup, the cast launch reduces them: nothing to clear, no atomics
    // (or, where it applies, one launch for both steps that keeps the tensors on chip in between)
    hipError_t e;
    if (fused_cast_applies(M, K, N, K, s)) {
        e = launch_amax_cast_fused(x_bf16, M, K, sc + 0, saved->xq, saved->xqT, sc + 1, sc + 2, w_bf16, N, K, sc + 3,
                                   saved->wq, saved->wqT, sc + 4, sc + 5, false, true, workspace, s);
    } else {
        uint32_t *px = (uint32_t *)workspace, *pw = px + kAmaxPartialsMax;
        int nx = 0, nw = 0;
        e = launch_amax2_partials(x_bf16, M * K, px, &nx, w_bf16, N * K, pw, &nw, s);
        if (e == hipSuccess)
            e = launch_quantize2_e4m3(x_bf16, M, K, sc + 0, saved->xq, saved->xqT, sc + 1, sc + 2, w_bf16, N, K,
                                      sc + 3, saved->wq, saved->wqT, sc + 4, sc + 5, s, px, nx, pw, nw);
    }
    if (e != hipSuccess)
        return TWEO_ERR_HIP;
    return tweo_fp8_linear_fwd(saved->xq, sc + 2, saved->wq, sc + 5, residual_bf16, M, N, K, y_bf16,
                               pen, penalty_sum, (uint8_t *)workspace + kAmaxScratchBytes,
                               workspace_bytes - kAmaxScratchBytes, stream);
}

static tweo_status fp8_linear_bwd_bf16_impl(const void *dy_bf16, const tweo_fp8_saved *saved, int64_t M,
                                            int64_t N, int64_t K, uint8_t *dyq, uint8_t *dyqT,
                                            void *dx_bf16, void *dw_bf16, void *workspace,
                                            size_t workspace_bytes, void *stream, bool dy_e5m2)
{
    if (!dy_bf16 || !saved || !saved->xqT || !saved->wqT || !saved->scalars || !dyq || !dyqT ||
        M <= 0 || N <= 0 || K <= 0 || !aligned16(dy_bf16) || !aligned16(dyq) || !aligned16(dyqT))
        return TWEO_ERR_INVALID_ARG;
    if (!dims_ok(M, N, K) || M % 16 != 0 || N % 16 != 0 || K % 16 != 0)
        return TWEO_ERR_UNSUPPORTED;
    if (!workspace || !aligned16(workspace) || workspace_bytes < kAmaxScratchBytes)
        return TWEO_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    float *sc = saved->scalars;
    hipError_t e;
    if (fused_cast_applies(M, N, 0, 0, s)) {
        e = launch_amax_cast_fused(dy_bf16, M, N, sc + 6, dyq, dyqT, sc + 7, sc + 8, nullptr, 0, 0, nullptr, nullptr,
                                   nullptr, nullptr, nullptr, dy_e5m2, false, workspace, s);
    } else {
        uint32_t *pdy = (uint32_t *)workspace;
        int ndy = 0;
        e = launch_amax_partials(dy_bf16, M * N, pdy, &ndy, s);
        if (e == hipSuccess)
            e = launch_quantize_f8_from_partials(dy_bf16, M, N, pdy, ndy, dy_e5m2, sc + 6, dyq, dyqT, sc + 7, sc + 8, s);
    }
    if (e != hipSuccess)
        return TWEO_ERR_HIP;
    return fp8_linear_bwd_impl(dyq, dyqT, sc + 8, saved->wqT, sc + 5, saved->xqT, sc + 2, M, N, K,
                               dx_bf16, dw_bf16, (uint8_t *)workspace + kAmaxScratchBytes,
                               workspace_bytes - kAmaxScratchBytes, stream, dy_e5m2);
}

tweo_status tweo_fp8_linear_bwd_bf16(const void *dy_bf16, const tweo_fp8_saved *saved, int64_t M,
                                     int64_t N, int64_t K, uint8_t *dyq, uint8_t *dyqT,
                                     void *dx_bf16, void *dw_bf16, void *workspace,
                                     size_t workspace_bytes, void *stream)
{
    return fp8_linear_bwd_bf16_impl(dy_bf16, saved, M, N, K, dyq, dyqT, dx_bf16, dw_bf16, workspace,
                                    workspace_bytes, stream, false);
}

tweo_status tweo_fp8_linear_bwd_bf16_hybrid(const void *dy_bf16, const tweo_fp8_saved *saved, int64_t M,
                                            int64_t N, int64_t K, uint8_t *dyq, uint8_t *dyqT,
                                            void *dx_bf16, void *dw_bf16, void *workspace,
                                            size_t workspace_bytes, void *stream)
{
    return fp8_linear_bwd_bf16_impl(dy_bf16, saved, M, N, K, dyq, dyqT, dx_bf16, dw_bf16, workspace,
                                    workspace_bytes, stream, true);
}

tweo_status tweo_fp8_linear_fwd_bf16_delayed(const void *x_bf16, const void *w_bf16, const void *residual_bf16,
                                             int64_t M, int64_t N, int64_t K, void *y_bf16,
                                             const tweo_penalty_cfg *pen, double *penalty_sum,
                                             const tweo_fp8_saved *saved, void *state_x, void *state_w,
                                             int bootstrap, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!x_bf16 || !w_bf16 || !y_bf16 || !saved || !saved->xq || !saved->xqT || !saved->wq || !saved->wqT ||
        !saved->scalars || !state_x || !state_w || state_x == state_w || M <= 0 || N <= 0 || K <= 0 ||
        !aligned16(x_bf16) || !aligned16(w_bf16) || !aligned16(saved->xq) || !aligned16(saved->xqT) ||
        !aligned16(saved->wq) || !aligned16(saved->wqT) || !aligned16(saved->scalars) || !aligned16(state_x) ||
        !aligned16(state_w))
        return TWEO_ERR_INVALID_ARG;
    if (!dims_ok(M, N, K) || M % 16 != 0 || N % 16 != 0 || K % 16 != 0)
        return TWEO_ERR_UNSUPPORTED;
    float *sc = saved->scalars;
    // x and w share one cast launch and one state-update launch; the update leaves each tensor's
    // amax, the scale its cast used and the inverse in the saved scalars (words 0-2 and 3-5)
    hipError_t e = launch_quantize2_e4m3_delayed(x_bf16, M, K, state_x, saved->xq, saved->xqT, sc + 0, w_bf16, N, K,
                                                 state_w, saved->wq, saved->wqT, sc + 3, bootstrap != 0,
                                                 (hipStream_t)stream);
    if (e != hipSuccess)
        return TWEO_ERR_HIP;
    return tweo_fp8_linear_fwd(saved->xq, sc + 2, saved->wq, sc + 5, residual_bf16, M, N, K, y_bf16, pen, penalty_sum,
                               workspace, workspace_bytes, stream);
}

tweo_status tweo_fp8_linear_bwd_bf16_delayed(const void *dy_bf16, const tweo_fp8_saved *saved, void *state_dy,
                                             int bootstrap, int dy_e5m2, int64_t M, int64_t N, int64_t K,
                                             uint8_t *dyq, uint8_t *dyqT, void *dx_bf16, void *dw_bf16,
                                             void *workspace, size_t workspace_bytes, void *stream)
{
    if (!dy_bf16 || !saved || !saved->xqT || !saved->wqT || !saved->scalars || !state_dy || !dyq || !dyqT ||
        M <= 0 || N <= 0 || K <= 0 || !aligned16(dy_bf16) || !aligned16(dyq) || !aligned16(dyqT) ||
        !aligned16(state_dy) || (dy_e5m2 != 0 && dy_e5m2 != 1))
        return TWEO_ERR_INVALID_ARG;
    if (!dims_ok(M, N, K) || M % 16 != 0 || N % 16 != 0 || K % 16 != 0)
        return TWEO_ERR_UNSUPPORTED;
    float *sc = saved->scalars;
    hipError_t e = dy_e5m2 ? launch_quantize_e5m2_delayed(dy_bf16, M, N, state_dy, bootstrap != 0, dyq, dyqT,
                                                          (hipStream_t)stream, sc + 6)
                           : launch_quantize_e4m3_delayed(dy_bf16, M, N, state_dy, bootstrap != 0, dyq, dyqT,
                                                          (hipStream_t)stream, sc + 6);
    if (e != hipSuccess)
        return TWEO_ERR_HIP;
    return fp8_linear_bwd_impl(dyq, dyqT, sc + 8, saved->wqT, sc + 5, saved->xqT, sc + 2, M, N, K, dx_bf16, dw_bf16,
                               workspace, workspace_bytes, stream, dy_e5m2 != 0);
}

tweo_status tweo_fp8_linear_bwd_bf16_inject(const void *dy_bf16, const void *a_bf16,
                                            const tweo_penalty_cfg *pen, float g, int dy_e5m2,
                                            const tweo_fp8_saved *saved, int64_t M, int64_t N, int64_t K,
                                            uint8_t *dyq, uint8_t *dyqT, void *dx_bf16, void *dw_bf16,
                                            void *workspace, size_t workspace_bytes, void *stream)
{
    if (!dy_bf16 || !a_bf16 || !pen || !saved || !saved->xqT || !saved->wqT || !saved->scalars || !dyq || !dyqT ||
        M <= 0 || N <= 0 || K <= 0 || !aligned16(dy_bf16) || !aligned16(a_bf16) || !aligned16(dyq) ||
        !aligned16(dyqT) || !(g == g) || !(pen->tau > 0.0f) || !(pen->eps >= 0.0f) ||
        (dy_e5m2 != 0 && dy_e5m2 != 1))
        return TWEO_ERR_INVALID_ARG;
    if (!dims_ok(M, N, K) || M % 16 != 0 || N % 16 != 0 || K % 16 != 0 || pen->p < 1 || pen->p > 8)
        return TWEO_ERR_UNSUPPORTED;
    if (!workspace || !aligned16(workspace) || workspace_bytes < kAmaxScratchBytes)
        return TWEO_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    float *sc = saved->scalars;
    const double denom = (double)pen->tau + (double)pen->eps;
    hipError_t e = launch_amax_quantize_inject(dy_bf16, a_bf16, M, N, (float)(1.0 / denom),
                                               (float)((double)g * pen->p / denom), pen->p, dy_e5m2 != 0,
                                               (uint32_t *)workspace, sc + 6, dyq, dyqT, sc + 7, sc + 8, s);
    if (e != hipSuccess)
        return TWEO_ERR_HIP;
    return fp8_linear_bwd_impl(dyq, dyqT, sc + 8, saved->wqT, sc + 5, saved->xqT, sc + 2, M, N, K, dx_bf16, dw_bf16,
                               (uint8_t *)workspace + kAmaxScratchBytes, workspace_bytes - kAmaxScratchBytes, stream,
                               dy_e5m2 != 0);
}

}  // extern "C"
