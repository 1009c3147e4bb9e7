/*
 * CPU oracle for the per-tensor FP8 linear layer with the TWEO penalty and for
 * the W8A8 per-tensor static INT8 linear layer.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a slow, plain, scalar statement of
 * what the GPU library must compute.  Only the tests, the smoke check and the
 * cpu_baseline leg of the benchmark may call it; the product path never does.
 * It shares no source, header, table or helper with the HIP kernels.
 *
 * Every function cites the passage of the TWEO paper (arXiv 2511.23225) that
 * defines it, or says that the paper is silent and which reading is taken.
 * Floating point is fp64 unless the method itself fixes a narrower type
 * (bf16 storage, the fp32 scale multiply in front of the E4M3 rounding, the
 * fp32 dequantisation multiply of the INT8 path).
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC (no fast-math: the
 * rounding steps rely on IEEE semantics and on the default round-to-nearest-
 * even mode).
 *
 * Parity pins (tests/test_oracle_*.py): E4M3 range +-448 (Sec. 1), brute-force
 * nearest-value search in exact rationals, a library cast for the in-range
 * part, the printed penalty values 0.0625 / 1 / 10000 (Sec. 3.3), integer
 * matmul by a library, adjoint identities between fwd/dgrad/wgrad, AbsMax
 * end points +-Q_8 (Sec. 4.4); for the row-granular INT8 functions exact
 * rationals, row independence, power-of-two steps and a library matmul
 * (tests/test_oracle_int8_rows.py); for LayerNorm closed forms (constant and
 * two-valued rows), invariances, exact rationals and a library layer norm in
 * fp64 (tests/test_oracle_layernorm.py).  No function here is "parity unpinned"; the
 * conventions the paper leaves open (NaN handling, zero amax, rounding mode of
 * "round") are listed where they are taken.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ bf16 */

/* bf16 is the top half of an IEEE binary32; widening is exact. */
float orc_bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* binary32 -> bf16, round to nearest, ties to even; NaN stays a (quiet) NaN. */
uint16_t orc_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if (isnan(f))
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t keep = u >> 16;
    uint32_t rest = u & 0xFFFFu;
    if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u)))
        keep += 1u; /* a carry out of the mantissa moves to the exponent; 0x7F7F+1 = inf */
    return (uint16_t)keep;
}

/* ------------------------------------------------------------------ E4M3 */

/*
 * E4M3 as used for FP8 training: 1 sign, 4 exponent (bias 7), 3 mantissa
 * bits, no infinities, one NaN code per sign (all ones), largest finite
 * magnitude 448 (Sec. 1: "E4M3 ranges within +-448").
 */
double orc_e4m3_decode(uint8_t b)
{
    int s = b >> 7, e = (b >> 3) & 15, m = b & 7;
    double mag;
    if (e == 15 && m == 7)
        return NAN;
    if (e == 0)
        mag = ldexp((double)m / 8.0, -6);
    else
        mag = ldexp(1.0 + (double)m / 8.0, e - 7);
    return s ? -mag : mag;
}

/*
 * Round a binary32 to the nearest E4M3 value, ties to the even mantissa,
 * saturating at +-448 (per-tensor FP8 casting never produces NaN from a finite
 * input).  NaN maps to the NaN code.  The paper only names the format and its
 * range; round-to-nearest-even with saturation is the reading taken here.
 *
 * The value grid inside the binade [2^E, 2^(E+1)) has spacing 2^(E-3); below
 * the smallest normal 2^-6 the spacing stays 2^-9 (subnormals).  So divide by
 * the spacing (exact in fp64: a power of two), round to an integer with the
 * default IEEE mode (ties to even integer == ties to even mantissa), and the
 * code is that integer offset by the binade's first code.
 */
uint8_t orc_e4m3_encode(float v)
{
    uint32_t u;
    memcpy(&u, &v, sizeof u);
    uint8_t sign = (u >> 31) ? 0x80 : 0x00;
    if (isnan(v))
        return sign | 0x7F;
    double a = fabs((double)v);
    if (a >= 448.0)
        return sign | 0x7E;
    if (a == 0.0)
        return sign;
    int ex;
    (void)frexp(a, &ex); /* a = f * 2^ex with f in [0.5,1)  =>  floor(log2 a) = ex-1 */
    int E = ex - 1;
    if (E < -6)
        E = -6;
    double spacing = ldexp(1.0, E - 3);
    double r = nearbyint(a / spacing); /* 0..8 in the subnormal band, 8..16 in a normal binade */
    /* first code of binade E is ((E+7)<<3) and corresponds to r = 8 */
    int code = ((E + 6) << 3) + (int)r;
    return sign | (uint8_t)code;
}

/*
 * E5M2, the gradient format of the HYBRID recipe the paper trained with
 * (Sec. 4.3: "Format.HYBRID (E4M3/E5M2)"): 1 sign, 5 exponent (bias 15), 2
 * mantissa bits, IEEE-like: exponent 31 is Inf (mantissa 0) or NaN; largest
 * finite magnitude 1.75 * 2^15 = 57344, smallest subnormal 2^-16.
 */
double orc_e5m2_decode(uint8_t b)
{
    int s = b >> 7, e = (b >> 2) & 31, m = b & 3;
    double mag;
    if (e == 31)
        mag = m == 0 ? INFINITY : NAN;
    else if (e == 0)
        mag = ldexp((double)m / 4.0, -14);
    else
        mag = ldexp(1.0 + (double)m / 4.0, e - 15);
    return s ? -mag : mag;
}

/*
 * Round a binary32 to the nearest E5M2 value, ties to the even mantissa,
 * saturating at +-57344 like the E4M3 cast (a training cast never produces Inf;
 * the paper is silent: same reading).  NaN maps to a NaN code.  Same grid
 * argument as for E4M3 with spacing 2^(E-2) and 2^-16 below 2^-14.
 */
uint8_t orc_e5m2_encode(float v)
{
    uint32_t u;
    memcpy(&u, &v, sizeof u);
    uint8_t sign = (u >> 31) ? 0x80 : 0x00;
    if (isnan(v))
        return sign | 0x7F;
    double a = fabs((double)v);
    if (a >= 57344.0)
        return sign | 0x7B;
    if (a == 0.0)
        return sign;
    int ex;
    (void)frexp(a, &ex);
    int E = ex - 1;
    if (E < -14)
        E = -14;
    double spacing = ldexp(1.0, E - 2);
    double r = nearbyint(a / spacing); /* 0..4 in the subnormal band, 4..8 in a normal binade */
    int code = ((E + 14) << 2) + (int)r;
    return sign | (uint8_t)code;
}

/* ------------------------------------------------------------------ amax */

/*
 * Per-tensor amax = max_i |x_i| over the whole tensor (Sec. 4.3: one scaling
 * factor for the entire tensor; Sec. 4.4 Eq. 4: max(|X|)).  bf16 magnitudes
 * order like their 15-bit patterns, so the maximum is taken on patterns; this
 * also fixes the open NaN/Inf case: Inf beats every finite value and a NaN
 * beats Inf, i.e. a NaN in the tensor is reported, not hidden.
 */
float orc_amax_bf16(const uint16_t *x, int64_t n)
{
    uint16_t best = 0;
    for (int64_t i = 0; i < n; ++i) {
        uint16_t mag = x[i] & 0x7FFF;
        if (mag > best)
            best = mag;
    }
    return orc_bf16_to_f32(best);
}

/*
 * scale maps [-amax, amax] onto the E4M3 range: scale = 448 / amax, one fp32
 * division; scale_inv = 1 / scale, one fp32 division.  The paper gives no
 * formula, margin or guard; reading: margin 0, no power-of-two rounding,
 * amax of 0 / Inf / NaN -> scale 1, an overflowing quotient -> FLT_MAX.
 */
void orc_scale_from_amax(float amax, float *scale, float *scale_inv)
{
    float s;
    if (!(amax > 0.0f) || isinf(amax) || isnan(amax)) {
        s = 1.0f;
    } else {
        s = 448.0f / amax;
        if (isinf(s))
            s = 3.402823466e+38f;
    }
    *scale = s;
    *scale_inv = 1.0f / s;
}

/* The same for the E5M2 range: scale = 57344 / amax. */
void orc_scale_from_amax_e5m2(float amax, float *scale, float *scale_inv)
{
    float s;
    if (!(amax > 0.0f) || isinf(amax) || isnan(amax)) {
        s = 1.0f;
    } else {
        s = 57344.0f / amax;
        if (isinf(s))
            s = 3.402823466e+38f;
    }
    *scale = s;
    *scale_inv = 1.0f / s;
}

void orc_quantize_e5m2(const uint16_t *x, int64_t rows, int64_t cols, float scale,
                       uint8_t *q, uint8_t *qT)
{
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            volatile float prod = orc_bf16_to_f32(x[r * cols + c]) * scale;
            uint8_t b = orc_e5m2_encode(prod);
            q[r * cols + c] = b;
            if (qT)
                qT[c * rows + r] = b;
        }
}

/*
 * q[r,c] = e4m3( fp32(x[r,c]) * scale ): one fp32 multiply, then the rounding
 * above.  qT (optional) is the same bytes transposed, qT[c,r] = q[r,c].
 */
void orc_quantize_e4m3(const uint16_t *x, int64_t rows, int64_t cols, float scale,
                       uint8_t *q, uint8_t *qT)
{
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            volatile float prod = orc_bf16_to_f32(x[r * cols + c]) * scale;
            uint8_t b = orc_e4m3_encode(prod);
            q[r * cols + c] = b;
            if (qT)
                qT[c * rows + r] = b;
        }
}

/* ------------------------------------------------------------- FP8 GEMMs */

static void decode_table(double *t)
{
    for (int b = 0; b < 256; ++b)
        t[b] = orc_e4m3_decode((uint8_t)b);
}

static void decode_table_fmt(double *t, int e5m2)
{
    for (int b = 0; b < 256; ++b)
        t[b] = e5m2 ? orc_e5m2_decode((uint8_t)b) : orc_e4m3_decode((uint8_t)b);
}

/*
 * Forward: Y[m,n] = (sum_k dec(Xq[m,k]) dec(Wq[n,k])) * sx_inv * sw_inv (+ R[m,n]).
 * A linear layer under per-tensor FP8 (Sec. 4.3); fp64 products of two E4M3
 * values are exact, the fp64 sum is the reference.
 * rows_idx (nullable) selects output rows m; row j of the outputs then holds
 * row rows_idx[j].  y64: fp64 result.  yabs (nullable): sum_k |x w| * sx_inv *
 * sw_inv (+|R|), the magnitude a rounding-error bound scales with.  ybf
 * (nullable): bf16 rounding (via fp32) of the fp64 result.
 */
void orc_fp8_linear_fwd(const uint8_t *xq, const uint8_t *wq, const uint16_t *residual,
                        int64_t M, int64_t N, int64_t K, float sx_inv, float sw_inv,
                        const int64_t *rows_idx, int64_t n_rows,
                        double *y64, double *yabs, uint16_t *ybf)
{
    double t[256];
    decode_table(t);
    int64_t R = rows_idx ? n_rows : M;
    double alpha = (double)sx_inv * (double)sw_inv;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < R; ++j) {
        int64_t m = rows_idx ? rows_idx[j] : j;
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0, aab = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double p = t[xq[m * K + k]] * t[wq[n * K + k]];
                acc += p;
                aab += fabs(p);
            }
            double y = acc * alpha, ya = aab * alpha;
            if (residual) {
                double r = (double)orc_bf16_to_f32(residual[m * N + n]);
                y += r;
                ya += fabs(r);
            }
            y64[j * N + n] = y;
            if (yabs)
                yabs[j * N + n] = ya;
            if (ybf)
                ybf[j * N + n] = orc_f32_to_bf16((float)y);
        }
    }
}

/*
 * Data gradient: dX[m,k] = (sum_n dec(dYq[m,n]) dec(Wq[n,k])) * sdy_inv * sw_inv.
 * Operands are the untransposed tensors; rows_idx selects rows m.
 */
void orc_fp8_linear_dgrad_fmt(const uint8_t *dyq, const uint8_t *wq,
                              int64_t M, int64_t N, int64_t K, float sdy_inv, float sw_inv,
                              const int64_t *rows_idx, int64_t n_rows,
                              double *dx64, double *dxabs, int dy_e5m2);

void orc_fp8_linear_dgrad(const uint8_t *dyq, const uint8_t *wq,
                          int64_t M, int64_t N, int64_t K, float sdy_inv, float sw_inv,
                          const int64_t *rows_idx, int64_t n_rows,
                          double *dx64, double *dxabs)
{
    orc_fp8_linear_dgrad_fmt(dyq, wq, M, N, K, sdy_inv, sw_inv, rows_idx, n_rows, dx64, dxabs, 0);
}

/* dy_e5m2 != 0: the output gradient is in E5M2 codes (HYBRID format), the weights stay E4M3. */
void orc_fp8_linear_dgrad_fmt(const uint8_t *dyq, const uint8_t *wq,
                              int64_t M, int64_t N, int64_t K, float sdy_inv, float sw_inv,
                              const int64_t *rows_idx, int64_t n_rows,
                              double *dx64, double *dxabs, int dy_e5m2)
{
    double t[256], tg[256];
    decode_table(t);
    decode_table_fmt(tg, dy_e5m2);
    int64_t R = rows_idx ? n_rows : M;
    double alpha = (double)sdy_inv * (double)sw_inv;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < R; ++j) {
        int64_t m = rows_idx ? rows_idx[j] : j;
        double *acc = dx64 + j * K;
        double *aab = dxabs ? dxabs + j * K : NULL;
        for (int64_t k = 0; k < K; ++k) {
            acc[k] = 0.0;
            if (aab)
                aab[k] = 0.0;
        }
        for (int64_t n = 0; n < N; ++n) { /* n ascending for every (m,k) */
            double g = tg[dyq[m * N + n]];
            for (int64_t k = 0; k < K; ++k) {
                double p = g * t[wq[n * K + k]];
                acc[k] += p;
                if (aab)
                    aab[k] += fabs(p);
            }
        }
        for (int64_t k = 0; k < K; ++k) {
            acc[k] *= alpha;
            if (aab)
                aab[k] *= alpha;
        }
    }
}

/*
 * Weight gradient: dW[n,k] = (sum_m dec(dYq[m,n]) dec(Xq[m,k])) * sdy_inv * sx_inv.
 * rows_idx selects rows n of dW.
 */
void orc_fp8_linear_wgrad_fmt(const uint8_t *dyq, const uint8_t *xq,
                              int64_t M, int64_t N, int64_t K, float sdy_inv, float sx_inv,
                              const int64_t *rows_idx, int64_t n_rows,
                              double *dw64, double *dwabs, int dy_e5m2);

void orc_fp8_linear_wgrad(const uint8_t *dyq, const uint8_t *xq,
                          int64_t M, int64_t N, int64_t K, float sdy_inv, float sx_inv,
                          const int64_t *rows_idx, int64_t n_rows,
                          double *dw64, double *dwabs)
{
    orc_fp8_linear_wgrad_fmt(dyq, xq, M, N, K, sdy_inv, sx_inv, rows_idx, n_rows, dw64, dwabs, 0);
}

void orc_fp8_linear_wgrad_fmt(const uint8_t *dyq, const uint8_t *xq,
                              int64_t M, int64_t N, int64_t K, float sdy_inv, float sx_inv,
                              const int64_t *rows_idx, int64_t n_rows,
                              double *dw64, double *dwabs, int dy_e5m2)
{
    double t[256], tg[256];
    decode_table(t);
    decode_table_fmt(tg, dy_e5m2);
    int64_t R = rows_idx ? n_rows : N;
    double alpha = (double)sdy_inv * (double)sx_inv;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < R; ++j) {
        int64_t n = rows_idx ? rows_idx[j] : j;
        double *acc = dw64 + j * K;
        double *aab = dwabs ? dwabs + j * K : NULL;
        for (int64_t k = 0; k < K; ++k) {
            acc[k] = 0.0;
            if (aab)
                aab[k] = 0.0;
        }
        for (int64_t m = 0; m < M; ++m) { /* m ascending for every (n,k) */
            double g = tg[dyq[m * N + n]];
            for (int64_t k = 0; k < K; ++k) {
                double p = g * t[xq[m * K + k]];
                acc[k] += p;
                if (aab)
                    aab[k] += fabs(p);
            }
        }
        for (int64_t k = 0; k < K; ++k) {
            acc[k] *= alpha;
            if (aab)
                aab[k] *= alpha;
        }
    }
}

/* ---------------------------------------------------------- TWEO penalty */

/*
 * S = sum_i ( |a_i| / (tau + eps) )^p over a bf16 activation tensor
 * (Sec. 3.3, the TWEO loss: the expectation is S divided by the element
 * count; the 1/L layer average and lambda(t) of the total loss belong to the
 * caller).  The paper leaves open whether the activation is taken before or
 * after its bf16 rounding; the stored (rounded) tensor is what the model sees,
 * so that is what is summed.
 */
double orc_penalty_sum(const uint16_t *a, int64_t n, double tau, double eps, int p)
{
    double denom = tau + eps, s = 0.0;
    for (int64_t i = 0; i < n; ++i)
        s += pow(fabs((double)orc_bf16_to_f32(a[i])) / denom, (double)p);
    return s;
}

/*
 * d/da of the summand above, times an outer factor g (the caller's
 * lambda / (L * numel)): g * p * sign(a) |a|^(p-1) / (tau+eps)^p.  Not printed
 * in the paper; it is the derivative of the loss of Sec. 3.3.
 */
void orc_penalty_grad(const uint16_t *a, int64_t n, double tau, double eps, int p, double g,
                      double *out)
{
    double denom = tau + eps;
    for (int64_t i = 0; i < n; ++i) {
        double v = (double)orc_bf16_to_f32(a[i]);
        double sgn = (v > 0) - (v < 0);
        out[i] = g * p * sgn * pow(fabs(v) / denom, (double)(p - 1)) / denom;
    }
}

/*
 * The same gradient added to the incoming output gradient, as the backward pass
 * sees it (bf16 in, bf16 out): out = bf16( dy + d(penalty)/da ), evaluated in
 * fp64 and rounded fp32 -> bf16 like every stored result in this file.  Also
 * returns the unrounded sums (may be NULL).
 */
void orc_penalty_grad_inject(const uint16_t *dy, const uint16_t *a, int64_t n, double tau, double eps,
                             int p, double g, uint16_t *out, double *exact)
{
    double denom = tau + eps;
    for (int64_t i = 0; i < n; ++i) {
        double v = (double)orc_bf16_to_f32(a[i]);
        double sgn = (v > 0) - (v < 0);
        double t = (double)orc_bf16_to_f32(dy[i]) + g * p * sgn * pow(fabs(v) / denom, (double)(p - 1)) / denom;
        if (exact)
            exact[i] = t;
        out[i] = orc_f32_to_bf16((float)t);
    }
}

/* ------------------------------------------------------------- INT8 W8A8 */

/*
 * Symmetric AbsMax quantisation with b = 8 (Sec. 4.4, Eq. 4): Q_8 = 127,
 * X_q = round(X / s * Q_8).  Static per-tensor: inv_step = 127 / s is computed
 * once by the caller.  Readings: "round" is round-to-nearest-even; the product
 * is a single fp32 multiply by inv_step; a static scale can be exceeded at run
 * time, so the result saturates to +-127 (-128 is never produced: the scheme
 * is symmetric); NaN maps to 0.
 */
void orc_quantize_i8(const uint16_t *x, int64_t n, float inv_step, int8_t *q)
{
    for (int64_t i = 0; i < n; ++i) {
        volatile float prod = orc_bf16_to_f32(x[i]) * inv_step;
        float r = nearbyintf(prod);
        int v;
        if (isnan(r))
            v = 0;
        else if (r > 127.0f)
            v = 127;
        else if (r < -127.0f)
            v = -127;
        else
            v = (int)r;
        q[i] = (int8_t)v;
    }
}

/*
 * W8A8 linear: acc[m,n] = sum_k xq[m,k] wq[n,k] in exact int32;
 * y = bf16( fp32(acc) * alpha ), alpha = step_x * step_w (the X_deq factors of
 * Eq. 4 for both operands, multiplied once by the caller).  fp32(acc) is the
 * IEEE int->float conversion (rounds above 2^24), then one fp32 multiply, then
 * bf16 round-to-nearest-even.  acc_out (nullable) receives the int32 sums.
 */
void orc_w8a8_linear(const int8_t *xq, const int8_t *wq, int64_t M, int64_t N, int64_t K,
                     float alpha, uint16_t *y, int32_t *acc_out)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int32_t acc = 0;
            for (int64_t k = 0; k < K; ++k)
                acc += (int32_t)xq[m * K + k] * (int32_t)wq[n * K + k];
            volatile float prod = (float)acc * alpha;
            y[m * N + n] = orc_f32_to_bf16(prod);
            if (acc_out)
                acc_out[m * N + n] = acc;
        }
}

/* Column-parallel variant for tiny M (same arithmetic, threads split n). */
void orc_w8a8_linear_small_m(const int8_t *xq, const int8_t *wq, int64_t M, int64_t N, int64_t K,
                             float alpha, uint16_t *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t m = 0; m < M; ++m) {
            int32_t acc = 0;
            for (int64_t k = 0; k < K; ++k)
                acc += (int32_t)xq[m * K + k] * (int32_t)wq[n * K + k];
            volatile float prod = (float)acc * alpha;
            y[m * N + n] = orc_f32_to_bf16(prod);
        }
}

/*
 * AbsMax quantisation at row granularity (Sec. 4.4, Eq. 4 with the "per-token"
 * and "per-channel" choices of s): every row of a [rows, cols] matrix gets its
 * own s_r = max_c |x_rc| + eps.  For activations a row is a token vector; for a
 * weight stored [out, in] a row is an output channel.  As in the per-tensor
 * case the division and the product with Q_8 are folded into one fp32 factor:
 * inv_r = 127 / s_r (one fp32 division), X_q = round(x * inv_r) (one fp32
 * multiply, round to nearest even), and the dequantisation step that Eq. 4
 * applies afterwards is step_r = s_r / 127 (one fp32 division).  The maximum is
 * taken on magnitude patterns (a NaN in a row poisons that row only: its step
 * is NaN and its codes are 0).  A row of zeros with eps = 0 gives inv = inf,
 * products NaN, codes 0 and step 0.
 */
void orc_quantize_i8_rows(const uint16_t *x, int64_t rows, int64_t cols, float eps, int8_t *q,
                          float *step)
{
    for (int64_t r = 0; r < rows; ++r) {
        volatile float s = orc_amax_bf16(x + r * cols, cols) + eps;
        volatile float inv = 127.0f / s;
        volatile float st = s / 127.0f;
        orc_quantize_i8(x + r * cols, cols, inv, q + r * cols);
        step[r] = st;
    }
}

/*
 * W8A8 linear with row-granular steps: acc[m,n] as above, then the two X_deq
 * factors of Eq. 4 one after the other, y = bf16( (fp32(acc) * sx[m]) * sw[n] ):
 * sx is per token (stride 1) or per tensor (stride 0), sw per output channel
 * (stride 1) or per tensor (stride 0).  Two fp32 multiplies in this order.
 */
void orc_w8a8_linear_scaled(const int8_t *xq, const int8_t *wq, int64_t M, int64_t N, int64_t K,
                            const float *sx, int64_t sx_stride, const float *sw,
                            int64_t sw_stride, uint16_t *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t m = 0; m < M; ++m) {
            int32_t acc = 0;
            for (int64_t k = 0; k < K; ++k)
                acc += (int32_t)xq[m * K + k] * (int32_t)wq[n * K + k];
            volatile float t = (float)acc * sx[m * sx_stride];
            volatile float u = t * sw[n * sw_stride];
            y[m * N + n] = orc_f32_to_bf16(u);
        }
}

/*
 * The same linear with an INT8 output for a quantised residual stream (Sec. 4.4, Table 4 "Res.?
 * Yes": the activation that leaves the layer is itself stored in 8 bits, with a static
 * per-tensor s): Eq. 4 applied to the fp32 result, X_q = round(y / s_out * Q_8) with the two
 * factors folded into inv_step_out = 127 / s_out by the caller.  Readings: the fp32 value
 * (fp32(acc) * sx[m]) * sw[n] is quantised directly, without rounding it to bf16 first; one more
 * fp32 multiply, round to nearest even, saturation to +-127, NaN -> 0, as in orc_quantize_i8.
 */
void orc_w8a8_linear_scaled_i8out(const int8_t *xq, const int8_t *wq, int64_t M, int64_t N, int64_t K,
                                  const float *sx, int64_t sx_stride, const float *sw,
                                  int64_t sw_stride, float inv_step_out, int8_t *yq)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t m = 0; m < M; ++m) {
            int32_t acc = 0;
            for (int64_t k = 0; k < K; ++k)
                acc += (int32_t)xq[m * K + k] * (int32_t)wq[n * K + k];
            volatile float t = (float)acc * sx[m * sx_stride];
            volatile float u = t * sw[n * sw_stride];
            volatile float prod = u * inv_step_out;
            float r = nearbyintf(prod);
            int v;
            if (isnan(r))
                v = 0;
            else if (r > 127.0f)
                v = 127;
            else if (r < -127.0f)
                v = -127;
            else
                v = (int)r;
            yq[m * N + n] = (int8_t)v;
        }
}

/* ------------------------------------------------- LayerNorm under FP8 */

/*
 * binary64 -> bf16 in ONE rounding (to nearest, ties to even), so that a value
 * computed in fp64 is not rounded twice on its way to bf16.  The bf16 grid in
 * the binade [2^E, 2^(E+1)) has spacing 2^(E-7); below the smallest normal
 * 2^-126 the spacing stays 2^-133.  A result of 2^128 or more is +-Inf.
 */
uint16_t orc_f64_to_bf16(double v)
{
    if (isnan(v))
        return 0x7FC0;
    uint16_t sign = signbit(v) ? 0x8000 : 0;
    double a = fabs(v);
    if (a == 0.0)
        return sign;
    if (isinf(a))
        return sign | 0x7F80;
    int ex;
    (void)frexp(a, &ex);
    int E = ex - 1; /* floor(log2 a) */
    if (E < -126)
        E = -126;
    double r = nearbyint(ldexp(a, 7 - E)); /* 128..256 in a normal binade, 0..128 below */
    if (E > 127 || (E == 127 && r >= 256.0))
        return sign | 0x7F80;
    /* first pattern of binade E is (E+127)<<7 and corresponds to r = 128; a carry to r = 256
     * lands on the next binade's first pattern by the same formula */
    uint32_t pattern = (uint32_t)((E + 126) << 7) + (uint32_t)r;
    return sign | (uint16_t)pattern;
}

/*
 * The residual-stream update in front of a normalisation: h = bf16(x + r).
 * The sum of two bf16 values is exact in fp64; it is rounded to bf16 once.
 */
void orc_residual_add_bf16(const uint16_t *x, const uint16_t *r, int64_t n, uint16_t *h)
{
    for (int64_t i = 0; i < n; ++i)
        h[i] = orc_f64_to_bf16((double)orc_bf16_to_f32(x[i]) + (double)orc_bf16_to_f32(r[i]));
}

/*
 * LayerNorm of each row of h[rows, cols] (Sec. 4.3: the paper runs the
 * LayerNorm components under FP8 as well, i.e. the normalised activation is
 * what the per-tensor cast of the next linear layer consumes).  The paper gives
 * no formula; the standard definition is taken:
 *   mu = mean_c h[r,c],  var = mean_c (h[r,c] - mu)^2   (biased),
 *   y[r,c] = (h[r,c] - mu) / sqrt(var + eps) * gamma[c] + beta[c],
 * everything in fp64; gamma, beta are bf16 parameters (beta may be NULL = 0).
 * y64 receives the fp64 values, y_bf16 their single rounding to bf16 (the
 * activation as the model stores it and as the FP8 cast reads it).
 */
void orc_layernorm(const uint16_t *h, const uint16_t *gamma, const uint16_t *beta, int64_t rows,
                   int64_t cols, double eps, double *y64, uint16_t *y_bf16)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const uint16_t *hr = h + r * cols;
        double sum = 0.0;
        for (int64_t c = 0; c < cols; ++c)
            sum += (double)orc_bf16_to_f32(hr[c]);
        double mu = sum / (double)cols;
        double ss = 0.0;
        for (int64_t c = 0; c < cols; ++c) {
            double d = (double)orc_bf16_to_f32(hr[c]) - mu;
            ss += d * d;
        }
        double var = ss / (double)cols;
        double rstd = 1.0 / sqrt(var + eps);
        for (int64_t c = 0; c < cols; ++c) {
            double d = (double)orc_bf16_to_f32(hr[c]) - mu;
            double y = d * rstd * (double)orc_bf16_to_f32(gamma[c]);
            if (beta)
                y += (double)orc_bf16_to_f32(beta[c]);
            if (y64)
                y64[r * cols + c] = y;
            if (y_bf16)
                y_bf16[r * cols + c] = orc_f64_to_bf16(y);
        }
    }
}

int orc_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
