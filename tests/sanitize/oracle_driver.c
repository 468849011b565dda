/* Host sanitizer run of the CPU oracle: every exported function on small, ragged and degenerate inputs.
 * Built by tests/test_host_sanitizers.py with -fsanitize=address,undefined together with oracle/llmq_oracle.c;
 * exit code 0 and no sanitizer report means no out-of-bounds access, no misaligned or overflowing
 * arithmetic on these inputs.  Checks only a few values: correctness is the pins' business. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double oracle_fp8_max(int fmt);
float oracle_bf16_to_f32(uint16_t b);
uint16_t oracle_f64_to_bf16(double v);
double oracle_fp8_decode(uint8_t code, int fmt);
uint8_t oracle_fp8_encode(float p, int fmt);
float oracle_amax_bf16(const uint16_t* x, size_t n);
float oracle_scale(float amax, int fmt);
void oracle_quantize(const uint16_t* x, int64_t rows, int64_t cols, float scale, int fmt, uint8_t* q, uint8_t* qt);
void oracle_gemm_tn(const uint8_t* A, int fmtA, const uint8_t* B, int fmtB, int64_t R, int64_t C, int64_t T,
                    float sA, float sB, double* y, double* S);
void oracle_gemm_tn_sampled(const uint8_t* A, int fmtA, const uint8_t* B, int fmtB, int64_t R, int64_t C, int64_t T,
                            float sA, float sB, const int64_t* rr, const int64_t* cc, int64_t n, double* y, double* S);
void oracle_swiglu_fwd(const uint16_t* gu, int64_t M, int64_t I, uint16_t* h);
void oracle_swiglu_fwd_exact(const uint16_t* gu, int64_t M, int64_t I, double* h);
void oracle_swiglu_bwd(const uint16_t* dh, const uint16_t* gu, int64_t M, int64_t I, uint16_t* dgu);
void oracle_swiglu_bwd_exact(const uint16_t* dh, const uint16_t* gu, int64_t M, int64_t I, double* dgu);
void oracle_residual_add(const uint16_t* res, const uint16_t* x, size_t n, uint16_t* out);
void oracle_rms_rstd(const uint16_t* res, int64_t M, int64_t C, double eps, double* rstd);
void oracle_rmsnorm_exact(const uint16_t* res, const uint16_t* w, int64_t M, int64_t C, double eps, double* y);
void oracle_rmsnorm_apply(const uint16_t* res, const uint16_t* w, const float* rstd, int64_t M, int64_t C, uint16_t* y);
void oracle_gemm_bf16_tn(const uint16_t* A, const uint16_t* B, int64_t R, int64_t C, int64_t T, double* y, double* S);
void oracle_gemm_bf16_tn_sampled(const uint16_t* A, const uint16_t* B, int64_t T, const int64_t* rr, const int64_t* cc,
                                 int64_t n, double* y, double* S);

static uint32_t rng = 12345u;
static uint32_t next(void) { rng = rng * 1664525u + 1013904223u; return rng >> 8; }

int main(void) {
    const int shapes[][2] = {{1, 1}, {3, 5}, {16, 8}, {33, 17}, {64, 130}};
    for (int fmt = 0; fmt < 2; ++fmt) {
        for (int c = 0; c < 256; ++c) {
            const double v = oracle_fp8_decode((uint8_t)c, fmt);
            if (v == v && fabs(v) <= oracle_fp8_max(fmt) && oracle_fp8_encode((float)v, fmt) != (uint8_t)c) return 2;
        }
        const float specials[] = {0.0f, -0.0f, 1e-45f, -1e-40f, 1e30f, -1e30f, INFINITY, -INFINITY, NAN, 448.0f, 57344.0f};
        for (unsigned i = 0; i < sizeof specials / sizeof specials[0]; ++i) (void)oracle_fp8_encode(specials[i], fmt);
        for (unsigned s = 0; s < sizeof shapes / sizeof shapes[0]; ++s) {
            const int64_t rows = shapes[s][0], cols = shapes[s][1], n = rows * cols;
            uint16_t* x = malloc((size_t)n * 2);
            uint8_t* q = malloc((size_t)n);
            uint8_t* qt = malloc((size_t)n);
            for (int64_t i = 0; i < n; ++i) x[i] = (uint16_t)(0x3C00 + (next() & 0x7FF) + ((next() & 1) << 15));
            const float a = oracle_amax_bf16(x, n);
            const float sc = oracle_scale(a, fmt);
            oracle_quantize(x, rows, cols, sc, fmt, q, qt);
            oracle_quantize(x, rows, cols, sc, fmt, q, NULL);
            for (int64_t i = 0; i < rows; ++i)
                for (int64_t j = 0; j < cols; ++j)
                    if (qt[j * rows + i] != q[i * cols + j]) return 3;
            /* contraction of the tensor with itself: [rows, cols] x [rows, cols]^T */
            double* y = malloc((size_t)(rows * rows) * sizeof(double));
            double* S = malloc((size_t)(rows * rows) * sizeof(double));
            oracle_gemm_tn(q, fmt, q, fmt, rows, rows, cols, sc, sc, y, S);
            for (int64_t i = 0; i < rows * rows; ++i)
                if (!(fabs(y[i]) <= S[i] * (1.0 + 1e-12))) return 4;
            /* the same at the last output position only, and the BF16 contraction */
            const int64_t rr = rows - 1, cc = rows - 1;
            double ys, Ss;
            oracle_gemm_tn_sampled(q, fmt, q, fmt, rows, rows, cols, sc, sc, &rr, &cc, 1, &ys, &Ss);
            if (ys != y[rows * rows - 1]) return 7;
            oracle_gemm_bf16_tn(x, x, rows, rows, cols, y, S);
            oracle_gemm_bf16_tn_sampled(x, x, cols, &rr, &cc, 1, &ys, &Ss);
            if (ys != y[rows * rows - 1]) return 8;
            /* the element-wise kernels around the linears: [rows, cols] as res / x / GU [rows, 2 I] when cols is even */
            uint16_t* o16 = malloc((size_t)n * 2);
            double* o64 = malloc((size_t)n * sizeof(double));
            double* rstd = malloc((size_t)rows * sizeof(double));
            float* rstd32 = malloc((size_t)rows * sizeof(float));
            oracle_residual_add(x, x, (size_t)n, o16);
            oracle_rms_rstd(x, rows, cols, 1e-6, rstd);
            for (int64_t i = 0; i < rows; ++i) rstd32[i] = (float)rstd[i];
            oracle_rmsnorm_exact(x, x, rows, cols, 1e-6, o64);
            oracle_rmsnorm_apply(x, x, rstd32, rows, cols, o16);
            if (cols % 2 == 0) {                       /* the tensor as GU [rows, 2 I] */
                const int64_t I = cols / 2;
                uint16_t* dgu = malloc((size_t)n * 2);
                double* dgu64 = malloc((size_t)n * sizeof(double));
                oracle_swiglu_fwd(x, rows, I, o16);            /* h [rows, I], then used as dh */
                oracle_swiglu_fwd_exact(x, rows, I, o64);
                oracle_swiglu_bwd(o16, x, rows, I, dgu);
                oracle_swiglu_bwd_exact(o16, x, rows, I, dgu64);
                free(dgu); free(dgu64);
            }
            free(o16); free(o64); free(rstd); free(rstd32);
            free(y); free(S); free(x); free(q); free(qt);
        }
        uint16_t z[5] = {0, 0x8000, 0, 0, 0};
        if (oracle_scale(oracle_amax_bf16(z, 5), fmt) != 1.0f) return 5;
        uint16_t nanv[3] = {0x3F80, 0x7FC1, 0xFF80};
        const float an = oracle_amax_bf16(nanv, 3);
        if (an == an) return 6;
    }
    (void)oracle_bf16_to_f32(0x7F80);
    (void)oracle_f64_to_bf16(1e300);
    (void)oracle_f64_to_bf16(-4.9e-324);
    puts("oracle sanitizer driver ok");
    return 0;
}
