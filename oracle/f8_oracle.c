/*
 * CPU oracle for the Float8 linear layer (forward + backward).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the HIP path, and
 * nothing in the product path may call it: only tests, the smoke check and the
 * cpu_baseline leg of the benchmark do.
 *
 * What it follows: the paper's section "Boosting throughput with mixed
 * precision training and Float8 support" (Float8 applied to linear layers,
 * dynamic per-tensor scaling: the scale comes from the abs-max of the tensor
 * being cast), the experiments section's remark that FP8 tensor-core matmuls
 * run beside BF16 ones (so: fp8 operands, higher-precision accumulate), the
 * FSDP mixed-precision appendix (layer inputs are bf16), and, for the two
 * number formats, the OCP FP8 definition the paper cites (Micikevicius et al.,
 * "FP8 formats for deep learning"): E4M3 (bias 7, no infinities, one NaN
 * mantissa pattern, max 448) and E5M2 (bias 15, IEEE-like, max 57344).
 *
 * Readings where the paper is silent (all "parity unpinned" by the paper; they
 * are pinned only by closed forms in the tests):
 *   - scale = FMAX / max(amax, 1e-12f) in fp32; quantise by multiplying with
 *     scale; de-quantise with inv_scale = 1.0f / scale.
 *   - the product x*scale is rounded to fp32 first, then clamped to +-FMAX,
 *     then rounded to fp8 with round-to-nearest, ties to even (saturating).
 *   - NaN input to the cast gives a NaN code (0x7F or 0xFF; the sign is not specified).
 *   - rowwise scaling: each GEMM operand has one scale per index of its
 *     non-contracted dimension, amax taken along the contracted dimension.
 *   - delayed scaling (f8o_history_push): the scale of a step is FMAX over the
 *     maximum of the amax values recorded at earlier steps (a window of `len`),
 *     the step's own amax is recorded after its cast.  Static scaling: a
 *     constant scale.  The paper only names the two strategies.
 *
 * Every function takes host pointers.  Matrices are row-major with a leading
 * dimension in elements.  bf16 values travel as uint16_t bit patterns, fp8
 * values as uint8_t codes.
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define F8O_E4M3 0
#define F8O_E5M2 1

#define F8O_TENSORWISE 0
#define F8O_ROWWISE 1
#define F8O_COLWISE 2

#define F8O_NT 0 /* A[M,K], B[N,K] */
#define F8O_NN 1 /* A[M,K], B[K,N] */
#define F8O_TN 2 /* A[K,M], B[K,N] */

/* ---- format parameters (OCP FP8) ---------------------------------------- */

static int mant_bits(int fmt) { return fmt == F8O_E4M3 ? 3 : 2; }
static int exp_bias(int fmt) { return fmt == F8O_E4M3 ? 7 : 15; }

/* Largest finite value: E4M3 1.75 * 2^8, E5M2 1.75 * 2^15. */
float f8o_fmax(int fmt) { return fmt == F8O_E4M3 ? 448.0f : 57344.0f; }

/* ---- bf16 <-> fp32 -------------------------------------------------------- */

/* A bf16 is the upper half of an fp32: widening is exact. */
float f8o_bf16_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* fp32 -> bf16, round to nearest, ties to even, written with real arithmetic:
 * pick the nearer of the two neighbouring bf16 values; on a tie the one whose
 * last mantissa bit is 0. */
uint16_t f8o_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if (isnan(f)) return (uint16_t)((u >> 16) | 0x0040u);
    if (isinf(f)) return (uint16_t)(u >> 16);
    uint16_t lo = (uint16_t)(u >> 16);          /* truncation: toward zero   */
    uint16_t hi = (uint16_t)(lo + 1);           /* next one away from zero   */
    double x = fabs((double)f);
    double vlo = fabs((double)f8o_bf16_to_f32(lo));
    double vhi = ((hi & 0x7F80u) == 0x7F80u) ? ldexp(1.0, 128) /* one step past the largest finite */
                                             : fabs((double)f8o_bf16_to_f32(hi));
    double dlo = x - vlo, dhi = vhi - x;
    if (dlo < dhi) return lo;
    if (dhi < dlo) return hi;
    return (lo & 1u) ? hi : lo;
}

/* ---- fp8 decode ----------------------------------------------------------- */

/* Value of an fp8 code, from the format definition:
 *   E == 0      : (-1)^S * 2^(1-bias) * (M / 2^m)          (subnormal / zero)
 *   otherwise   : (-1)^S * 2^(E-bias) * (1 + M / 2^m)
 * E4M3: S.1111.111 is NaN, there is no infinity.
 * E5M2: E == 31 is infinity (M == 0) or NaN (M != 0). */
float f8o_decode(uint8_t code, int fmt)
{
    int m = mant_bits(fmt), bias = exp_bias(fmt);
    int S = code >> 7;
    int E = (code & 0x7F) >> m;
    int M = code & ((1 << m) - 1);
    double v;
    if (fmt == F8O_E4M3) {
        if (E == 15 && M == 7) return S ? -NAN : NAN;
    } else {
        if (E == 31) {
            if (M == 0) return S ? -INFINITY : INFINITY;
            return S ? -NAN : NAN;
        }
    }
    if (E == 0)
        v = ldexp((double)M / (double)(1 << m), 1 - bias);
    else
        v = ldexp(1.0 + (double)M / (double)(1 << m), E - bias);
    return (float)(S ? -v : v); /* exact: every fp8 value is an fp32 value */
}

/* ---- fp8 encode ----------------------------------------------------------- */

/* Round a finite y with |y| <= FMAX to the nearest fp8 value, ties to the
 * even mantissa, and return its code.  Written as the definition of rounding
 * on the format's grid: in the binade of |y| (or the subnormal range) the
 * representable values are the multiples of one quantum q; divide by q, round
 * to the nearest integer with ties to even, multiply back.  Every step is
 * exact in double.  NaN gives 0x7F with the sign kept. */
uint8_t f8o_encode(float y, int fmt)
{
    int m = mant_bits(fmt), bias = exp_bias(fmt);
    uint32_t u;
    memcpy(&u, &y, 4);
    uint8_t sign = (uint8_t)((u >> 31) << 7);
    if (isnan(y)) return (uint8_t)(sign | 0x7F);
    double a = fabs((double)y);
    if (a == 0.0) return sign;

    int e;                       /* a = f * 2^e, f in [0.5, 1)  =>  binade exponent e-1 */
    (void)frexp(a, &e);
    int binade = e - 1;
    int emin = 1 - bias;         /* exponent of the smallest normal */
    if (binade < emin) binade = emin;   /* subnormals share the quantum of the first binade */
    double q = ldexp(1.0, binade - m);  /* spacing of representable values here */
    double n = rint(a / q);             /* default rounding mode: nearest, ties to even */
    /* n is in [0, 2^(m+1)]; n == 2^(m+1) is the first value of the next binade. */
    double r = n * q;                   /* the rounded magnitude, representable */

    if (r == 0.0) return sign;
    int er;
    double fr = frexp(r, &er);          /* r = fr * 2^er, fr in [0.5,1) */
    int E, M;
    if (er - 1 < emin) {                /* subnormal result: M = r / 2^(emin-m) */
        E = 0;
        M = (int)ldexp(r, -(emin - m));
    } else {
        E = (er - 1) + bias;
        M = (int)ldexp(fr * 2.0 - 1.0, m); /* fraction bits of 1.xxx */
    }
    return (uint8_t)(sign | (E << m) | M);
}

/* ---- step a1: amax -------------------------------------------------------- */

/* Largest magnitude of a bf16 matrix: over everything (tensorwise, 1 output),
 * per row over its columns (rowwise, `rows` outputs) or per column over its
 * rows (colwise, `cols` outputs).  Starts from 0. */
void f8o_amax(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, int gran, float* out)
{
    int64_t nout = gran == F8O_TENSORWISE ? 1 : (gran == F8O_ROWWISE ? rows : cols);
    for (int64_t i = 0; i < nout; ++i) out[i] = 0.0f;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            float a = fabsf(f8o_bf16_to_f32(x[r * ld + c]));
            int64_t o = gran == F8O_TENSORWISE ? 0 : (gran == F8O_ROWWISE ? r : c);
            if (a > out[o]) out[o] = a;
        }
}

/* ---- step a2: scale ------------------------------------------------------- */

/* scale = FMAX / max(amax, 1e-12), inv_scale = 1 / scale; fp32 divisions. */
void f8o_scale(const float* amax, int64_t n, int fmt, float* scale, float* inv_scale)
{
    for (int64_t i = 0; i < n; ++i) {
        float den = fmaxf(amax[i], 1e-12f);
        float s = f8o_fmax(fmt) / den;
        float inv = 1.0f / s;
        scale[i] = s;
        if (inv_scale) inv_scale[i] = inv;
    }
}

/* ---- step a3: cast -------------------------------------------------------- */

/* One element: fp32 product (rounded once to fp32), clamp, encode. */
uint8_t f8o_cast_one(uint16_t x_bf16, float scale, int fmt)
{
    float y = f8o_bf16_to_f32(x_bf16) * scale; /* one fp32 multiply, rounded to nearest */
    float fm = f8o_fmax(fmt);
    float c = y;
    if (c > fm) c = fm;      /* NaN compares false and passes through */
    if (c < -fm) c = -fm;
    return f8o_encode(c, fmt);
}

/* bf16 [rows, cols] -> fp8 codes.  scale has 1, rows or cols entries according
 * to gran.  out [rows, cols] and/or out_t [cols, rows] (the same codes,
 * transposed); either may be NULL. */
void f8o_cast(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, const float* scale,
              int gran, int fmt, uint8_t* out, int64_t ld_out, uint8_t* out_t, int64_t ld_out_t)
{
#pragma omp parallel for schedule(static)   /* rows are independent */
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            float s = gran == F8O_TENSORWISE ? scale[0] : (gran == F8O_ROWWISE ? scale[r] : scale[c]);
            uint8_t code = f8o_cast_one(x[r * ld + c], s, fmt);
            if (out) out[r * ld_out + c] = code;
            if (out_t) out_t[c * ld_out_t + r] = code;
        }
}

/* ---- steps a4-a6: GEMM ---------------------------------------------------- */

/* decode() of all 256 codes of a format, filled by the function above; the
 * inner loops read this instead of calling ldexp per element. */
static float dec_table[2][256];
static int dec_table_ready = 0;
static void fill_dec_table(void)
{
    if (dec_table_ready) return;
    for (int f = 0; f < 2; ++f)
        for (int c = 0; c < 256; ++c) dec_table[f][c] = f8o_decode((uint8_t)c, f);
    dec_table_ready = 1;
}

static inline uint8_t a_at(int layout, const uint8_t* A, int64_t lda, int64_t m, int64_t k)
{
    return layout == F8O_TN ? A[k * lda + m] : A[m * lda + k];
}
static inline uint8_t b_at(int layout, const uint8_t* B, int64_t ldb, int64_t n, int64_t k)
{
    return layout == F8O_NT ? B[n * ldb + k] : B[k * ldb + n];
}

/* One output element, fp32 accumulation in ascending k, then the scales, then
 * bf16.  Tensorwise: acc * (inv_sa * inv_sb).  Otherwise (rowwise GEMM):
 * (acc * inv_sa[m]) * inv_sb[n]. */
uint16_t f8o_gemm_elem(int layout, int64_t K, const uint8_t* A, int fa, int64_t lda,
                       const uint8_t* B, int fb, int64_t ldb, const float* inv_sa,
                       const float* inv_sb, int gran, int64_t m, int64_t n)
{
    float acc = 0.0f;
    fill_dec_table();
    for (int64_t k = 0; k < K; ++k) {
        float p = dec_table[fa][a_at(layout, A, lda, m, k)] * dec_table[fb][b_at(layout, B, ldb, n, k)];
        acc = acc + p; /* the product of two fp8 values is exact in fp32 */
    }
    float r;
    if (gran == F8O_TENSORWISE) {
        float s = inv_sa[0] * inv_sb[0];
        r = acc * s;
    } else {
        float t = acc * inv_sa[m];
        r = t * inv_sb[n];
    }
    return f8o_f32_to_bf16(r);
}

/* The same element in fp64 with no final rounding, plus sum |a||b| scaled the
 * same way (for the accumulation error bound). */
void f8o_gemm_elem_f64(int layout, int64_t K, const uint8_t* A, int fa, int64_t lda,
                       const uint8_t* B, int fb, int64_t ldb, const float* inv_sa,
                       const float* inv_sb, int gran, int64_t m, int64_t n, double* val,
                       double* abs_sum)
{
    double acc = 0.0, aacc = 0.0;
    fill_dec_table();
    for (int64_t k = 0; k < K; ++k) {
        double p = (double)dec_table[fa][a_at(layout, A, lda, m, k)] *
                   (double)dec_table[fb][b_at(layout, B, ldb, n, k)];
        acc += p;
        aacc += fabs(p);
    }
    double s = gran == F8O_TENSORWISE ? (double)inv_sa[0] * (double)inv_sb[0]
                                      : (double)inv_sa[m] * (double)inv_sb[n];
    *val = acc * s;
    if (abs_sum) *abs_sum = aacc * fabs(s);
}

/* Full D[M,N] (bf16 bits). */
void f8o_gemm(int layout, int64_t M, int64_t N, int64_t K, const uint8_t* A, int fa, int64_t lda,
              const uint8_t* B, int fb, int64_t ldb, const float* inv_sa, const float* inv_sb,
              int gran, uint16_t* D, int64_t ldd)
{
    fill_dec_table();
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n)
            D[m * ldd + n] = f8o_gemm_elem(layout, K, A, fa, lda, B, fb, ldb, inv_sa, inv_sb, gran, m, n);
}

/* Full D[M,N] in fp64 (no rounding) and, if asked, the matching sum |a||b|. */
void f8o_gemm_f64(int layout, int64_t M, int64_t N, int64_t K, const uint8_t* A, int fa,
                  int64_t lda, const uint8_t* B, int fb, int64_t ldb, const float* inv_sa,
                  const float* inv_sb, int gran, double* D, double* Dabs, int64_t ldd)
{
    fill_dec_table();
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n)
            f8o_gemm_elem_f64(layout, K, A, fa, lda, B, fb, ldb, inv_sa, inv_sb, gran, m, n,
                              &D[m * ldd + n], Dabs ? &Dabs[m * ldd + n] : NULL);
}

/* `count` chosen output elements (ms[i], ns[i]) -> out[i]; for the big shapes
 * where the full product is too slow on a CPU. */
void f8o_gemm_points(int layout, int64_t K, const uint8_t* A, int fa, int64_t lda,
                     const uint8_t* B, int fb, int64_t ldb, const float* inv_sa,
                     const float* inv_sb, int gran, const int64_t* ms, const int64_t* ns,
                     int64_t count, uint16_t* out)
{
    fill_dec_table();
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < count; ++i)
        out[i] = f8o_gemm_elem(layout, K, A, fa, lda, B, fb, ldb, inv_sa, inv_sb, gran, ms[i], ns[i]);
}

/* ---- step a7: the linear layer ------------------------------------------- */

/* Everything a Float8 linear keeps between forward and backward, all host
 * memory owned by the caller.  Tensorwise: one scale per tensor and the *_c
 * members are unused.  Rowwise: q is scaled per row of the tensor, q_c per
 * column of the tensor (both stored untransposed here; the oracle's GEMM
 * indexes either layout directly). */
typedef struct {
    uint8_t* q;      /* [rows, cols] codes, tensorwise or per-row scales  */
    float* amax;     /* 1 or rows */
    float* scale;
    float* inv_scale;
    uint8_t* q_c;    /* [rows, cols] codes with per-column scales (rowwise mode) */
    float* amax_c;   /* cols */
    float* scale_c;
    float* inv_scale_c;
} f8o_qtensor;

static void quantise(const uint16_t* x, int64_t rows, int64_t cols, int gran, int fmt,
                     uint8_t* q, float* amax, float* scale, float* inv_scale)
{
    int64_t n = gran == F8O_TENSORWISE ? 1 : (gran == F8O_ROWWISE ? rows : cols);
    f8o_amax(x, rows, cols, cols, gran, amax);
    f8o_scale(amax, n, fmt, scale, inv_scale);
    f8o_cast(x, rows, cols, cols, scale, gran, fmt, q, cols, NULL, 0);
}

/* Forward: Y[M,N] = X[M,K] * W[N,K]^T.  rowwise == 0: tensorwise scaling.
 * rowwise == 1: X per row m, W per row n for Y; additionally the per-column
 * casts of X and W (needed by backward) are produced here, as a training step
 * would save them. */
void f8o_linear_fwd(int64_t M, int64_t K, int64_t N, int rowwise, const uint16_t* X,
                    const uint16_t* W, uint16_t* Y, f8o_qtensor* xq, f8o_qtensor* wq)
{
    if (!rowwise) {
        quantise(X, M, K, F8O_TENSORWISE, F8O_E4M3, xq->q, xq->amax, xq->scale, xq->inv_scale);
        quantise(W, N, K, F8O_TENSORWISE, F8O_E4M3, wq->q, wq->amax, wq->scale, wq->inv_scale);
        f8o_gemm(F8O_NT, M, N, K, xq->q, F8O_E4M3, K, wq->q, F8O_E4M3, K, xq->inv_scale,
                 wq->inv_scale, F8O_TENSORWISE, Y, N);
    } else {
        quantise(X, M, K, F8O_ROWWISE, F8O_E4M3, xq->q, xq->amax, xq->scale, xq->inv_scale);
        quantise(W, N, K, F8O_ROWWISE, F8O_E4M3, wq->q, wq->amax, wq->scale, wq->inv_scale);
        quantise(X, M, K, F8O_COLWISE, F8O_E4M3, xq->q_c, xq->amax_c, xq->scale_c, xq->inv_scale_c);
        quantise(W, N, K, F8O_COLWISE, F8O_E4M3, wq->q_c, wq->amax_c, wq->scale_c, wq->inv_scale_c);
        f8o_gemm(F8O_NT, M, N, K, xq->q, F8O_E4M3, K, wq->q, F8O_E4M3, K, xq->inv_scale,
                 wq->inv_scale, F8O_ROWWISE, Y, N);
    }
}

/* Backward: dX[M,K] = dY[M,N] * W[N,K];  dW[N,K] = dY[M,N]^T * X[M,K].
 * grad_fmt is the fp8 format of dY.  Rowwise: dX uses dY per row m and W per
 * column k; dW uses dY per column n and X per column k. */
void f8o_linear_bwd(int64_t M, int64_t K, int64_t N, int rowwise, int grad_fmt,
                    const uint16_t* dY, const f8o_qtensor* xq, const f8o_qtensor* wq,
                    f8o_qtensor* dyq, uint16_t* dX, uint16_t* dW)
{
    if (!rowwise) {
        quantise(dY, M, N, F8O_TENSORWISE, grad_fmt, dyq->q, dyq->amax, dyq->scale, dyq->inv_scale);
        f8o_gemm(F8O_NN, M, K, N, dyq->q, grad_fmt, N, wq->q, F8O_E4M3, K, dyq->inv_scale,
                 wq->inv_scale, F8O_TENSORWISE, dX, K);
        f8o_gemm(F8O_TN, N, K, M, dyq->q, grad_fmt, N, xq->q, F8O_E4M3, K, dyq->inv_scale,
                 xq->inv_scale, F8O_TENSORWISE, dW, K);
    } else {
        quantise(dY, M, N, F8O_ROWWISE, grad_fmt, dyq->q, dyq->amax, dyq->scale, dyq->inv_scale);
        quantise(dY, M, N, F8O_COLWISE, grad_fmt, dyq->q_c, dyq->amax_c, dyq->scale_c, dyq->inv_scale_c);
        f8o_gemm(F8O_NN, M, K, N, dyq->q, grad_fmt, N, wq->q_c, F8O_E4M3, K, dyq->inv_scale,
                 wq->inv_scale_c, F8O_ROWWISE, dX, K);
        f8o_gemm(F8O_TN, N, K, M, dyq->q_c, grad_fmt, N, xq->q_c, F8O_E4M3, K, dyq->inv_scale_c,
                 xq->inv_scale_c, F8O_ROWWISE, dW, K);
    }
}

/* ---- delayed and static scaling --------------------------------------------
 * The paper's Float8 section names three per-tensor scaling strategies: dynamic,
 * delayed and static, without spelling out the last two.  The reading used
 * here:
 *   static  - the scale is a constant chosen beforehand; the cast is
 *             f8o_cast with that scale, nothing else changes.
 *   delayed - the scale used at a step comes from the amax values recorded at
 *             EARLIER steps: FMAX / max(max(history), 1e-12) over a window of
 *             the last `len` recorded values.  The tensor of the current step is
 *             cast with that scale (values beyond its range saturate) and its
 *             own amax is recorded afterwards, for later steps.
 * history[0] is the newest entry, history[len-1] the oldest. */

/* Record amax_new (dropping the oldest entry), then derive the scale of the
 * next step from the updated window. */
void f8o_history_push(float* history, int64_t len, float amax_new, int fmt, float* scale,
                      float* inv_scale)
{
    for (int64_t i = len - 1; i >= 1; --i) history[i] = history[i - 1];
    history[0] = amax_new;
    float window_max = 0.0f;
    for (int64_t i = 0; i < len; ++i)
        if (history[i] > window_max) window_max = history[i];
    f8o_scale(&window_max, 1, fmt, scale, inv_scale);
}

/* ---- the feed-forward glue between two Float8 linears ------------------------
 * Llama's feed-forward block is  Y = W2 ( silu(W1 x) * (W3 x) ),  silu(t) = t / (1 + e^-t).
 * With W1 and W3 stacked into one linear its output row is [a | b] (H values each) and the
 * next linear's input is h = silu(a) * b.  The paper does not spell this out (it trains
 * Llama 3.1 models); it is the textbook definition, evaluated here in double precision and
 * rounded to fp32 and from there to bf16 (two roundings to nearest even: within half a bf16
 * unit plus one part in 2^16 of the single rounding).  The backward formulas are its derivatives:
 *   dh/da = b * s'(a),  s'(t) = sig(t) * (1 + t * (1 - sig(t))),  sig(t) = 1 / (1 + e^-t)
 *   dh/db = silu(a).
 * Each function also returns the amax of what it wrote (the next cast's input). */
static double sigmoid64(double t) { return 1.0 / (1.0 + exp(-t)); }

void f8o_silu_mul(const uint16_t* ab, int64_t M, int64_t H, uint16_t* h, float* amax_h)
{
    float amax = 0.0f;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t j = 0; j < H; ++j) {
            double a = (double)f8o_bf16_to_f32(ab[m * 2 * H + j]);
            double b = (double)f8o_bf16_to_f32(ab[m * 2 * H + H + j]);
            uint16_t o = f8o_f32_to_bf16((float)(a * sigmoid64(a) * b));
            h[m * H + j] = o;
            float v = fabsf(f8o_bf16_to_f32(o));
            if (v > amax) amax = v;
        }
    if (amax_h) *amax_h = amax;
}

void f8o_silu_mul_bwd(const uint16_t* ab, const uint16_t* dh, int64_t M, int64_t H, uint16_t* dab,
                      float* amax_dab)
{
    float amax = 0.0f;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t j = 0; j < H; ++j) {
            double a = (double)f8o_bf16_to_f32(ab[m * 2 * H + j]);
            double b = (double)f8o_bf16_to_f32(ab[m * 2 * H + H + j]);
            double g = (double)f8o_bf16_to_f32(dh[m * H + j]);
            double sg = sigmoid64(a);
            uint16_t da = f8o_f32_to_bf16((float)(g * b * (sg * (1.0 + a * (1.0 - sg)))));
            uint16_t db = f8o_f32_to_bf16((float)(g * (a * sg)));
            dab[m * 2 * H + j] = da;
            dab[m * 2 * H + H + j] = db;
            float v = fabsf(f8o_bf16_to_f32(da)), w = fabsf(f8o_bf16_to_f32(db));
            if (v > amax) amax = v;
            if (w > amax) amax = w;
        }
    if (amax_dab) *amax_dab = amax;
}

/* RMS normalisation in front of the attention and feed-forward linears of a Llama block:
 *   y[m, :] = x[m, :] * rstd[m] * g,   rstd[m] = 1 / sqrt(mean_d x[m, d]^2 + eps)
 * The textbook definition, in double precision, rounded to fp32 and from there to bf16 (y), or
 * once to fp32 (rstd).  Only
 * the forward is here: it is the producer of a Float8 linear's input; the backward of the
 * normalisation does not touch the Float8 path. */
void f8o_rmsnorm(const uint16_t* x, const uint16_t* g, int64_t M, int64_t D, double eps, uint16_t* y,
                 float* rstd, float* amax_y)
{
    float amax = 0.0f;
    for (int64_t m = 0; m < M; ++m) {
        double ss = 0.0;
        for (int64_t d = 0; d < D; ++d) {
            double v = (double)f8o_bf16_to_f32(x[m * D + d]);
            ss += v * v;
        }
        double r = 1.0 / sqrt(ss / (double)D + eps);
        if (rstd) rstd[m] = (float)r;
        for (int64_t d = 0; d < D; ++d) {
            double v = (double)f8o_bf16_to_f32(x[m * D + d]) * r * (double)f8o_bf16_to_f32(g[d]);
            uint16_t o = f8o_f32_to_bf16((float)v);
            y[m * D + d] = o;
            float a = fabsf(f8o_bf16_to_f32(o));
            if (a > amax) amax = a;
        }
    }
    if (amax_y) *amax_y = amax;
}

int f8o_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
