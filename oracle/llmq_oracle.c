/*
 * CPU oracle for the FP8 linear-layer path of LLMQ's 8-bit training pipeline.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the GPU library and
 * must never be called from the product path; only the test-suite, the smoke
 * check and the benchmark's cpu_baseline leg load it.
 *
 * What it follows (paper sections):
 *   - Section 3, "Overview": just-in-time tensor-level absmax scaling -- find
 *     the largest absolute value of the tensor, rescale so that it lands on
 *     the largest representable FP8 value (no clipping), convert BF16 -> FP8;
 *     the main transformer matmuls (forward and backward) run in FP8, their
 *     results stay in BF16.
 *   - Section 2: the two FP8 types E4M3 and E5M2 (OCP 8-bit floating point
 *     formats, the specification the paper cites for FP8).
 *   - Section 3, paragraph on kernel fusion: FP8 GEMM is TN-only, so the
 *     transposed copies are produced by a fused transpose+quantize step.
 *
 * Readings where the paper is silent (listed in the design notes as well):
 *   scale  s = min(fl32(FMAX / amax), FLT_MAX): one IEEE binary32 division, whose
 *          overflow (a tiny amax) is clamped to the largest finite binary32;
 *          s = 1 for amax == 0, where "map the absmax onto FMAX" defines no
 *          scale and every scale gives the same codes (all +-0);
 *   value  p = fl32(fl32(x) * s), one binary32 multiplication, not fused;
 *   cast   round-to-nearest-even onto the FP8 grid, saturating to +-FMAX
 *          (never produces an Inf or NaN code from a finite p); NaN -> S.1111111;
 *   amax   of a tensor holding a NaN is the canonical quiet NaN (0x7FC00000),
 *          otherwise max |x| (which is +Inf if an Inf is present);
 *   GEMM   fp64 accumulation of exact products of the decoded FP8 values,
 *          divided by (double)sA * (double)sB.
 *
 *   - Section 3, kernel-fusion paragraph and "Activation checkpointing": the
 *     non-linearity (SwiGLU) also returns the absmax of its result, and under
 *     recomputation, with the absmax known, emits the FP8 bytes directly.
 *
 * Parity status: every function below is pinned by tests/test_oracle_*.py
 * (closed forms of the formats, an independent library cast, brute force on
 * small integer inputs, algebraic invariants; for SwiGLU the binary64
 * definition, a library SiLU, identities of the logistic function and finite
 * differences for the backward pass; for RMSNorm a library rms_norm in
 * binary64, scaling invariance, constant rows and a library BF16 addition).
 */
#include <float.h>
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define ORACLE_E4M3 0
#define ORACLE_E5M2 1

/* ---- format constants (OCP FP8) ----------------------------------------- */

static int fmt_mbits(int fmt) { return fmt == ORACLE_E4M3 ? 3 : 2; }
static int fmt_bias(int fmt) { return fmt == ORACLE_E4M3 ? 7 : 15; }

/* Largest finite magnitude: E4M3 S.1111.110 = 1.75 * 2^8, E5M2 S.11110.11 = 1.75 * 2^15. */
double oracle_fp8_max(int fmt) { return fmt == ORACLE_E4M3 ? 448.0 : 57344.0; }

/* ---- BF16 ------------------------------------------------------------------ */

/* A BF16 number is the upper half of the binary32 with the same value. */
float oracle_bf16_to_f32(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* binary64 -> BF16 with round-to-nearest-even (used by tests to form expected
 * outputs; overflow goes to Inf as IEEE rounding prescribes). */
uint16_t oracle_f64_to_bf16(double v) {
    if (isnan(v)) return 0x7FC0;
    uint16_t sign = signbit(v) ? 0x8000 : 0;
    double a = fabs(v);
    if (a == 0.0) return sign;
    if (isinf(a)) return sign | 0x7F80;
    int ex;
    frexp(a, &ex);               /* a = m * 2^ex, m in [0.5, 1) */
    int e = ex - 1;              /* a in [2^e, 2^(e+1)) */
    if (e < -126) e = -126;      /* subnormal range shares the quantum of e = -126 */
    double u = ldexp(1.0, e - 7);
    double t = a / u;            /* exact: division by a power of two */
    double f = floor(t), d = t - f;
    if (d > 0.5 || (d == 0.5 && fmod(f, 2.0) == 1.0)) f += 1.0;
    if (f >= 256.0) { f = 128.0; e += 1; }
    if (e > 127) return sign | 0x7F80;
    uint32_t n = (uint32_t)f;
    if (n < 128) return sign | (uint16_t)n;              /* subnormal, exponent field 0 */
    return sign | (uint16_t)(((e + 127) << 7) | (n - 128));
}

/* ---- FP8 decode: the closed form of the format ------------------------------ */

double oracle_fp8_decode(uint8_t code, int fmt) {
    const int m = fmt_mbits(fmt), bias = fmt_bias(fmt);
    const int sign = code >> 7;
    const int E = (code & 0x7F) >> m;
    const int M = code & ((1 << m) - 1);
    double v;
    if (fmt == ORACLE_E4M3) {
        if (E == 15 && M == 7) return NAN;               /* only NaN, no infinities */
    } else {
        if (E == 31) {
            if (M == 0) return sign ? -INFINITY : INFINITY;
            return NAN;
        }
    }
    if (E == 0)
        v = ldexp((double)M / (double)(1 << m), 1 - bias);          /* subnormal */
    else
        v = ldexp(1.0 + (double)M / (double)(1 << m), E - bias);    /* normal */
    return sign ? -v : v;
}

/* ---- FP8 encode: saturating round-to-nearest-even ---------------------------- */

uint8_t oracle_fp8_encode(float p, int fmt) {
    const int m = fmt_mbits(fmt), bias = fmt_bias(fmt);
    const int emin = 1 - bias;
    const uint8_t sign = signbit(p) ? 0x80 : 0x00;
    if (isnan(p)) return sign | 0x7F;
    const double a = fabs((double)p);
    const double fmax = oracle_fp8_max(fmt);
    if (a > fmax) return sign | (fmt == ORACLE_E4M3 ? 0x7E : 0x7B);   /* saturate, +-Inf too */
    if (a == 0.0) return sign;
    int ex;
    frexp(a, &ex);
    int e = ex - 1;                       /* a in [2^e, 2^(e+1)) */
    if (e < emin) e = emin;               /* below the smallest normal the quantum is fixed */
    const double u = ldexp(1.0, e - m);   /* spacing of the grid in this binade */
    const double t = a / u;               /* exact */
    double f = floor(t);
    const double d = t - f;
    if (d > 0.5 || (d == 0.5 && fmod(f, 2.0) == 1.0)) f += 1.0;   /* ties to even */
    int n = (int)f;                       /* 0 .. 2^(m+1) */
    if (n == (2 << m)) { n = 1 << m; e += 1; }                    /* carried into next binade */
    if (n < (1 << m)) return sign | (uint8_t)n;                   /* zero or subnormal */
    return sign | (uint8_t)(((e + bias) << m) | (n - (1 << m)));
}

/* Element-wise application of the encoder to an array (no other arithmetic). */
void oracle_fp8_encode_array(const float* p, size_t n, int fmt, uint8_t* out) {
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) out[i] = oracle_fp8_encode(p[i], fmt);
}

/* ---- absmax and scale --------------------------------------------------------- */

float oracle_amax_bf16(const uint16_t* x, size_t n) {
    float a = 0.0f;
    int saw_nan = 0;
#pragma omp parallel for reduction(max : a) reduction(| : saw_nan) schedule(static)
    for (size_t i = 0; i < n; ++i) {
        float v = fabsf(oracle_bf16_to_f32(x[i]));
        if (isnan(v)) saw_nan = 1;
        else if (v > a) a = v;
    }
    if (saw_nan) {
        uint32_t q = 0x7FC00000u;
        memcpy(&a, &q, sizeof a);
    }
    return a;
}

float oracle_scale(float amax, int fmt) {
    volatile float num = (float)oracle_fp8_max(fmt);
    volatile float den = amax;
    volatile float s;
    if (amax == 0.0f) return 1.0f;         /* all-zero tensor: the rule defines no scale, every code is +-0 */
    s = num / den;                         /* one binary32 division */
    if (isinf(s)) s = FLT_MAX;             /* a tiny absmax: the quotient overflows */
    return s;
}

/* ---- quantize (+ transposed copy) --------------------------------------------- */

/* q[i*cols + j] = cast(fl32(x[i,j] * scale)); qt[j*rows + i] = q[i*cols + j]; qt may be NULL. */
void oracle_quantize(const uint16_t* x, int64_t rows, int64_t cols, float scale, int fmt,
                     uint8_t* q, uint8_t* qt) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        for (int64_t j = 0; j < cols; ++j) {
            volatile float p = oracle_bf16_to_f32(x[i * cols + j]) * scale;   /* rounded to binary32 */
            uint8_t c = oracle_fp8_encode(p, fmt);
            q[i * cols + j] = c;
            if (qt) qt[j * rows + i] = c;
        }
    }
}

/* ---- the contraction shared by forward, dgrad and wgrad ----------------------- */

/*
 * y[r,c] = ( sum_t dec(A[r,t]) * dec(B[c,t]) ) / (sA*sB),   S[r,c] = ( sum_t |dec(A)*dec(B)| ) / (sA*sB)
 * A is [R,T], B is [C,T], both row-major with the contraction index contiguous.
 *   forward: A = Xq  [M,K],  B = Wq  [N,K]   ->  Y  [M,N]
 *   dgrad  : A = dYq [M,N],  B = Wq^T [K,N]  ->  dX [M,K]
 *   wgrad  : A = dYq^T [N,M], B = Xq^T [K,M] ->  dW [N,K]
 * S is the quantity the GEMM tolerance is stated in.  Either output may be NULL.
 */
static void dot_tn(const uint8_t* a, const double* da, const uint8_t* b, const double* db,
                   int64_t T, double den, double* y, double* S) {
    double acc = 0.0, mag = 0.0;
    for (int64_t t = 0; t < T; ++t) {
        double prod = da[a[t]] * db[b[t]];   /* exact in binary64 */
        acc += prod;
        mag += fabs(prod);
    }
    if (y) *y = acc / den;
    if (S) *S = mag / den;
}

static void decode_table(int fmt, double* tab) {
    for (int c = 0; c < 256; ++c) tab[c] = oracle_fp8_decode((uint8_t)c, fmt);
}

void oracle_gemm_tn(const uint8_t* A, int fmtA, const uint8_t* B, int fmtB,
                    int64_t R, int64_t C, int64_t T, float sA, float sB,
                    double* y, double* S) {
    double da[256], db[256];
    decode_table(fmtA, da);
    decode_table(fmtB, db);
    const double den = (double)sA * (double)sB;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < R; ++r)
        for (int64_t c = 0; c < C; ++c)
            dot_tn(A + r * T, da, B + c * T, db, T, den,
                   y ? y + r * C + c : NULL, S ? S + r * C + c : NULL);
}

/* Same contraction for a list of (row, col) output positions only. */
void oracle_gemm_tn_sampled(const uint8_t* A, int fmtA, const uint8_t* B, int fmtB,
                            int64_t R, int64_t C, int64_t T, float sA, float sB,
                            const int64_t* rr, const int64_t* cc, int64_t n,
                            double* y, double* S) {
    (void)R; (void)C;
    double da[256], db[256];
    decode_table(fmtA, da);
    decode_table(fmtB, db);
    const double den = (double)sA * (double)sB;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        dot_tn(A + rr[i] * T, da, B + cc[i] * T, db, T, den, y ? y + i : NULL, S ? S + i : NULL);
}

/* ---- SwiGLU with its extra outputs (Section 3, kernel-fusion paragraph) ----------- */

/*
 * The paper keeps the non-linearities in BF16 and gives each of them an extra output, the absmax of
 * its result, so that the FP8 conversion of the next matmul's input needs no reduction pass of its
 * own; when the absmax is already known (recomputation during backward, Section 3 "Activation
 * checkpointing") the conversion itself is fused into the non-linearity.  Neither changes a value:
 * the absmax is oracle_amax_bf16 of the BF16 result and the fused bytes are oracle_quantize of it,
 * so the oracle only needs the non-linearity; the callers compose.
 *
 * Layout reading: the gate+up projection writes GU [M, 2I]; columns [0, I) are the gate g, columns
 * [I, 2I) are the up branch u; h[m,i] = silu(g) * u with silu(g) = g * sigma(g), sigma(g) = 1/(1+e^-g).
 * The backward pass maps dh [M, I] to dGU [M, 2I] in the same layout:
 *   d/du = dh * silu(g),   d/dg = dh * u * sigma(g) * (1 + g * (1 - sigma(g))).
 *
 * Two versions of each:
 *   *_exact  the definition in binary64 (what the result approximates);
 *   the plain names: the binary32 evaluation whose BF16 rounding decides the stored bits (and through
 *   them the absmax and the FP8 codes).  The paper does not fix the arithmetic of the non-linearity
 *   beyond "BF16 in, BF16 out", so it is fixed here, in IEEE binary32 operations only (each rounded to
 *   nearest even, nothing contracted except the fused multiply-adds written out), which any machine
 *   reproduces bit for bit:
 *     1. a  = -min(max(g, -100), 86)
 *     2. n  = rint(a * LOG2E)                        ties to even
 *     3. r  = fma(n, -LN2_HI, a);  r = fma(n, -LN2_LO, r)
 *     4. p  = 1 + r(1 + r(1/2 + r(1/6 + r(1/24 + r(1/120 + r/720)))))     Horner, one fma per level
 *     5. e  = p * 2^n                                exact scaling; overflows to +Inf for g <= -89, which
 *                                                    makes sg and h zero where |silu(g)| < 2^-121
 *     6. sg = 1 / (1 + e)                            one addition, one division
 *     7. h  = bf16( (g * sg) * u )                   two multiplications, one rounding to BF16
 *   backward, with sg as above:
 *     du = bf16( dh * (g * sg) ),   dg = bf16( ((dh * u) * sg) * fma(g, 1 - sg, 1) ).
 *   The constants are the binary32 numbers nearest to log2(e), ln 2 (HI), ln 2 - HI (LO) and 1/k!.
 *   Non-finite inputs are outside the contract.
 */
static const float SW_LOG2E = 0x1.715476p+0f;
static const float SW_LN2_HI = 0x1.62e430p-1f;
static const float SW_LN2_LO = -0x1.05c610p-29f;
static const float SW_C2 = 0x1.000000p-1f, SW_C3 = 0x1.555556p-3f, SW_C4 = 0x1.555556p-5f,
                   SW_C5 = 0x1.111112p-7f, SW_C6 = 0x1.6c16c2p-10f;

double oracle_sigmoid_exact(double g) { return 1.0 / (1.0 + exp(-g)); }

float oracle_sigmoid_f32(float g) {
    float a = -fminf(fmaxf(g, -100.0f), 86.0f);
    float n = rintf(a * SW_LOG2E);
    float r = fmaf(n, -SW_LN2_HI, a);
    r = fmaf(n, -SW_LN2_LO, r);
    float p = SW_C6;
    p = fmaf(p, r, SW_C5);
    p = fmaf(p, r, SW_C4);
    p = fmaf(p, r, SW_C3);
    p = fmaf(p, r, SW_C2);
    p = fmaf(p, r, 1.0f);
    p = fmaf(p, r, 1.0f);
    float e = ldexpf(p, (int)n);
    float d = 1.0f + e;
    return 1.0f / d;
}

/* h [M, I] (BF16 bit patterns) from GU [M, 2I]. */
void oracle_swiglu_fwd(const uint16_t* gu, int64_t M, int64_t I, uint16_t* h) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t i = 0; i < I; ++i) {
            float g = oracle_bf16_to_f32(gu[m * 2 * I + i]);
            float u = oracle_bf16_to_f32(gu[m * 2 * I + I + i]);
            float silu = g * oracle_sigmoid_f32(g);
            float v = silu * u;
            h[m * I + i] = oracle_f64_to_bf16((double)v);
        }
}

void oracle_swiglu_fwd_exact(const uint16_t* gu, int64_t M, int64_t I, double* h) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t i = 0; i < I; ++i) {
            double g = oracle_bf16_to_f32(gu[m * 2 * I + i]);
            double u = oracle_bf16_to_f32(gu[m * 2 * I + I + i]);
            h[m * I + i] = g * oracle_sigmoid_exact(g) * u;
        }
}

/* dGU [M, 2I] (BF16 bit patterns) from dh [M, I] and GU [M, 2I]. */
void oracle_swiglu_bwd(const uint16_t* dh, const uint16_t* gu, int64_t M, int64_t I, uint16_t* dgu) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t i = 0; i < I; ++i) {
            float g = oracle_bf16_to_f32(gu[m * 2 * I + i]);
            float u = oracle_bf16_to_f32(gu[m * 2 * I + I + i]);
            float d = oracle_bf16_to_f32(dh[m * I + i]);
            float sg = oracle_sigmoid_f32(g);
            float silu = g * sg;
            float du = d * silu;
            float one_minus = 1.0f - sg;
            float t = fmaf(g, one_minus, 1.0f);
            float dg = d * u;
            dg = dg * sg;
            dg = dg * t;
            dgu[m * 2 * I + i] = oracle_f64_to_bf16((double)dg);
            dgu[m * 2 * I + I + i] = oracle_f64_to_bf16((double)du);
        }
}

void oracle_swiglu_bwd_exact(const uint16_t* dh, const uint16_t* gu, int64_t M, int64_t I, double* dgu) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t i = 0; i < I; ++i) {
            double g = oracle_bf16_to_f32(gu[m * 2 * I + i]);
            double u = oracle_bf16_to_f32(gu[m * 2 * I + I + i]);
            double d = oracle_bf16_to_f32(dh[m * I + i]);
            double sg = oracle_sigmoid_exact(g);
            dgu[m * 2 * I + i] = d * u * sg * (1.0 + g * (1.0 - sg));
            dgu[m * 2 * I + I + i] = d * g * sg;
        }
}

/* ---- RMSNorm joined with the residual addition (Section 3, kernel-fusion paragraph) -------- */

/*
 * The paper handles RMS-norm and the residual-stream addition in one kernel that also returns the absmax
 * of the normalised output (the input of the next FP8 matmul); with the statistics kept from the forward
 * pass the FP8 conversion is fused in under recomputation (Section 3 "Activation checkpointing").
 *
 *   res'[m,c] = bf16( res[m,c] + x[m,c] )                         residual stream, stored in BF16
 *   ms[m]     = (1/C) sum_c res'[m,c]^2,   rstd[m] = 1 / sqrt(ms[m] + eps)
 *   y[m,c]    = bf16( res'[m,c] * rstd[m] * w[c] )                w [C] BF16, the norm's weight
 *
 * Readings: the norm is taken of the BF16-rounded residual (what is stored, so that recomputing from the
 * stored stream gives the same result); the addition is one binary32 addition of the two BF16 values,
 * then one RNE rounding; rstd is a per-row statistic kept in binary32 alongside the absmax.
 * The row reduction has no prescribed order, so it is not reproducible bit for bit: the oracle gives it
 * in binary64 (oracle_rms_rstd) and the exact output in binary64 (oracle_rmsnorm_exact); the GPU's rstd
 * is compared within a tolerance.  GIVEN a binary32 rstd, the normalisation is fixed operation by
 * operation, y = bf16( (res' * rstd) * w ) with two binary32 multiplications (oracle_rmsnorm_apply), and
 * is reproducible bit for bit; that is the recompute path (statistics in, FP8 bytes out).
 */
void oracle_residual_add(const uint16_t* res, const uint16_t* x, size_t n, uint16_t* out) {
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        float sum = oracle_bf16_to_f32(res[i]) + oracle_bf16_to_f32(x[i]);
        out[i] = oracle_f64_to_bf16((double)sum);
    }
}

void oracle_rms_rstd(const uint16_t* res, int64_t M, int64_t C, double eps, double* rstd) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        double ss = 0.0;
        for (int64_t c = 0; c < C; ++c) {
            double v = oracle_bf16_to_f32(res[m * C + c]);
            ss += v * v;
        }
        rstd[m] = 1.0 / sqrt(ss / (double)C + eps);
    }
}

void oracle_rmsnorm_exact(const uint16_t* res, const uint16_t* w, int64_t M, int64_t C, double eps, double* y) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        double r;
        oracle_rms_rstd(res + m * C, 1, C, eps, &r);
        for (int64_t c = 0; c < C; ++c)
            y[m * C + c] = (double)oracle_bf16_to_f32(res[m * C + c]) * r * (double)oracle_bf16_to_f32(w[c]);
    }
}

void oracle_rmsnorm_apply(const uint16_t* res, const uint16_t* w, const float* rstd, int64_t M, int64_t C,
                          uint16_t* y) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t c = 0; c < C; ++c) {
            float t = oracle_bf16_to_f32(res[m * C + c]) * rstd[m];
            float v = t * oracle_bf16_to_f32(w[c]);
            y[m * C + c] = oracle_f64_to_bf16((double)v);
        }
}

/* ---- BF16 contraction: the baseline the FP8 path is compared with (Section 4, "Impact of FP8") ------ */

/*
 * The paper reports its FP8 results next to a pure BF16 run of the same model (speed-up column of
 * Table 1).  The baseline GEMM has the same form as the FP8 one, on BF16 operands and without scales:
 *   y[r,c] = sum_t A[r,t] * B[c,t],   S[r,c] = sum_t |A[r,t] * B[c,t]|,   A [R,T], B [C,T] BF16 bit patterns.
 * Products of two BF16 numbers are exact in binary64; the sum is taken in binary64.
 */
void oracle_gemm_bf16_tn(const uint16_t* A, const uint16_t* B, int64_t R, int64_t C, int64_t T,
                         double* y, double* S) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < R; ++r)
        for (int64_t c = 0; c < C; ++c) {
            double acc = 0.0, mag = 0.0;
            for (int64_t t = 0; t < T; ++t) {
                double prod = (double)oracle_bf16_to_f32(A[r * T + t]) * (double)oracle_bf16_to_f32(B[c * T + t]);
                acc += prod;
                mag += fabs(prod);
            }
            if (y) y[r * C + c] = acc;
            if (S) S[r * C + c] = mag;
        }
}

void oracle_gemm_bf16_tn_sampled(const uint16_t* A, const uint16_t* B, int64_t T,
                                 const int64_t* rr, const int64_t* cc, int64_t n, double* y, double* S) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double acc = 0.0, mag = 0.0;
        for (int64_t t = 0; t < T; ++t) {
            double prod = (double)oracle_bf16_to_f32(A[rr[i] * T + t]) * (double)oracle_bf16_to_f32(B[cc[i] * T + t]);
            acc += prod;
            mag += fabs(prod);
        }
        if (y) y[i] = acc;
        if (S) S[i] = mag;
    }
}

/* Threads the OpenMP loops above will use (reported by the benchmark). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
