/*
 * llmq.h -- C ABI of the MI355X (gfx950) FP8 linear-layer path of LLMQ's 8-bit training pipeline.
 *
 * What the path computes (paper, Section 3 "Overview" and the kernel-fusion paragraph of Section 3):
 *   1. just-in-time tensor-level absmax scaling: find the largest |x| of a BF16 tensor and choose the
 *      scale that maps it onto the largest finite FP8 value, so that nothing is clipped;
 *   2. convert BF16 -> FP8 (E4M3 or E5M2, Section 2) with that scale, fused with the transposed copy,
 *      because the FP8 GEMM takes both operands with the contraction index contiguous ("TN");
 *   3. the transformer-block matmuls in FP8 with BF16 results: forward Y = X W^T, and in the backward
 *      pass dX = dY W and dW = dY^T X.
 *
 * Conventions for every entry point
 *   - Tensors are row-major with the last index contiguous.  X is [M,K], W is [N,K], Y and dY are
 *     [M,N], dX is [M,K], dW is [N,K].  BF16 tensors are arrays of 16-bit patterns, FP8 tensors are
 *     arrays of 8-bit OCP codes.
 *   - Every pointer is DEVICE memory owned by the caller, except `stream`, which is a hipStream_t
 *     passed as void* (NULL = the default stream).  The library allocates nothing, frees nothing and
 *     keeps no pointer after a call returns (Section 3 "Overview": all allocation happens at start-up).
 *   - Calls only enqueue work on `stream` and return; nothing synchronises with the host.  Scales and
 *     absmax values are read from and written to device memory.  The calls enqueue kernels only (no memory
 *     set or copy commands), so a stream that is being captured into a HIP graph can take them, and replays
 *     compute from what the buffers hold then.  Several host threads may call at the same time on streams
 *     and buffers of their own; the one piece of state the library keeps on a GPU is the scratch array of
 *     llmq_amax_static (see there).
 *   - BF16 and FP8 tensor pointers must be 16-byte aligned, float pointers 4-byte aligned.
 *   - Return value: LLMQ_OK or a negative llmq_status.  Argument errors are found on the host before
 *     anything is launched and leave all outputs untouched.  LLMQ_ERR_DEVICE reports a launch failure.
 *   - Results are bitwise deterministic: same inputs, same bytes (Section 3 "Reproducibility").  The
 *     only atomic used is an integer max (fused output absmax), whose result does not depend on order.
 *   - Dimensions may be any positive value.  Shapes whose dimensions are multiples of 256 (GEMM) or of
 *     16 rows x 8 columns (quantize) take the tuned kernels; everything else takes slower generic ones.
 */
#ifndef LLMQ_H
#define LLMQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LLMQ_OK = 0,
    LLMQ_ERR_NULL = -1,       /* a required pointer is NULL */
    LLMQ_ERR_SHAPE = -2,      /* a dimension is < 1 or too large */
    LLMQ_ERR_ALIGN = -3,      /* a pointer is not aligned as required */
    LLMQ_ERR_FORMAT = -4,     /* not an llmq_fp8_format */
    LLMQ_ERR_WORKSPACE = -5,  /* workspace missing or smaller than llmq_fp8_linear_workspace_bytes() */
    LLMQ_ERR_DEVICE = -6,     /* the HIP runtime reported an error at launch */
    LLMQ_ERR_FLAGS = -7       /* unknown bits in `flags` */
} llmq_status;

/* OCP 8-bit floating point formats (Section 2): E4M3 has bias 7 and max 448 (no Inf, NaN = S.1111.111),
 * E5M2 has bias 15 and max 57344 (IEEE-like Inf/NaN). */
typedef enum { LLMQ_E4M3 = 0, LLMQ_E5M2 = 1 } llmq_fp8_format;

const char* llmq_status_string(int status);
int llmq_version(void);

/*
 * Absmax and scale of a BF16 tensor (Section 3 "Overview": tensor-level absmax scaling, the scale maps the
 * tensor's largest magnitude onto the largest finite value of the FP8 format).
 *   x_bf16   [n] BF16, device, 16-byte aligned; n >= 1.
 *   fmt      target FP8 format, selects FMAX (448 or 57344) for the scale.
 *   d_amax   [1] float, device, written: max_i |x_i| exactly; the canonical quiet NaN 0x7FC00000 if the
 *            tensor holds a NaN; +Inf if it holds an Inf and no NaN.
 *   d_scale  [1] float, device, written if not NULL: min(FMAX / amax, FLT_MAX) with one IEEE binary32
 *            division (FLT_MAX for an absmax so small that the quotient overflows); 1 for an all-zero
 *            tensor, where the rule defines no scale and every code is +-0 whatever the scale; 0 when amax
 *            is +Inf; NaN when amax is NaN.
 *   ws       device scratch of at least llmq_amax_workspace_bytes() bytes, 4-byte aligned; contents on
 *            entry do not matter, it holds per-block partial results between the two launches (a
 *            streaming reduction, then a one-block kernel that reduces the partial results and writes
 *            both outputs; no atomics: Section 3 "Reproducibility").  Calls that may overlap on the
 *            device (different streams) need different workspaces.
 */
size_t llmq_amax_workspace_bytes(void);
int llmq_amax(const void* x_bf16, size_t n, int fmt, float* d_amax, float* d_scale,
              void* ws, size_t ws_bytes, void* stream);

/*
 * llmq_amax for callers that cannot allocate device memory and have no workspace to hand over: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * bit-identical outputs, but the per-block partial results go to a 4 KB array inside the library's device
 * image (one copy per GPU, held until the process ends) instead of `ws`.  The call allocates and frees
 * nothing.  n: 1 <= n < 2^40 elements as for llmq_amax, LLMQ_ERR_SHAPE beyond; the array's size does not
 * depend on n.  It uses the copy of the device that is current when the call is made, which must be the
 * stream's device; LLMQ_ERR_DEVICE if the runtime cannot resolve the array.  Every call on a GPU shares that
 * GPU's array: calls that may overlap on one device (different streams, or graphs replayed side by side) race
 * on it and need llmq_amax with separate workspaces instead.  Nothing in the array has to be cleared between
 * calls: every word the second stage reads has been written by the first stage of the same call.
 */
int llmq_amax_static(const void* x_bf16, size_t n, int fmt, float* d_amax, float* d_scale, void* stream);

/*
 * Fused scale + FP8 cast + transposed copy (Section 3, kernel-fusion paragraph: quantization and the
 * transposition the backward GEMMs need are one kernel).
 *   q[i,j]   = cast( fl32( fl32(x[i,j]) * d_scale[0] ) ),  q_t[j,i] = q[i,j]
 * cast = round-to-nearest-even onto the FP8 grid, saturating at +-FMAX (a finite product never yields
 * an Inf or NaN code).  The result for NaN inputs is unspecified.
 *   x_bf16   [rows, cols] BF16;  d_scale [1] float (device);  q [rows, cols] FP8;
 *   q_t      [cols, rows] FP8, or NULL when no transposed copy is wanted.
 */
int llmq_quantize_fp8(const void* x_bf16, int64_t rows, int64_t cols, const float* d_scale, int fmt,
                      uint8_t* q, uint8_t* q_t, void* stream);
/*
 * The same with the transposed copy stored in slabs of 128 contraction bytes, the form the backward contractions
 * read fastest (LLMQ_LAYOUT_SLABS of llmq_fp8_gemm, there with rows = cols of x and T = rows of x):
 *   q_t byte of element (j, i) of the transposed tensor at (i / 128) * cols * 128 + j * 128 + i % 128.
 * A 128 x 256 tile of x is then one contiguous 32 KB piece of q_t instead of 256 pieces of 128 bytes.  rows must
 * be a multiple of 128 and cols a multiple of 256 (LLMQ_ERR_SHAPE otherwise); q_t must not be NULL.
 */
int llmq_quantize_fp8_slabs(const void* x_bf16, int64_t rows, int64_t cols, const float* d_scale, int fmt,
                            uint8_t* q, uint8_t* q_t, void* stream);

/*
 * The FP8 contraction that forward, dgrad and wgrad share (Section 3: FP8 GEMM is TN-only):
 *   c[r,cc] = bf16( ( sum_t A[r,t] * B[cc,t] ) / (sA * sB) )        accumulate == 0
 *   c[r,cc] = bf16( c[r,cc] + (sum ...) / (sA * sB) )                accumulate != 0 (BF16 gradient
 *                                                                    accumulation, Section 3 "Overview")
 *   A [R,T] FP8 in format fmtA, B [C,T] FP8 in format fmtB (any mix of E4M3 / E5M2), products exact,
 *   accumulation in binary32 on the matrix cores, de-scaling in binary32, one rounding to BF16 (RNE).
 *   d_scaleA, d_scaleB  [1] float each (device): the scales the operands were quantized with.
 *   c_bf16   [R,C] BF16, written (read first when accumulate != 0).
 *   d_amax_c [1] float (device) or NULL: if given, receives max |c| of the BF16 result, bit-identical to
 *            llmq_amax of c (the next layer's quantization then needs no separate reduction; Section 3,
 *            kernel-fusion paragraph).
 * Error of each element is bounded by 2^-7 * sum_t |A[r,t] B[cc,t]| / (sA sB).
 */
int llmq_fp8_gemm_tn(const uint8_t* A, int fmtA, const uint8_t* B, int fmtB,
                     int64_t R, int64_t C, int64_t T,
                     const float* d_scaleA, const float* d_scaleB,
                     void* c_bf16, int accumulate, float* d_amax_c, void* stream);

/*
 * The same contraction with either operand in another layout than [rows, T] (LLMQ_LAYOUT_ROWS = 0):
 *   LLMQ_LAYOUT_T_MAJOR = 1: stored [T, rows] (the contraction index runs down the rows, the rows index is
 *     contiguous);
 *   LLMQ_LAYOUT_SLABS = 2: stored K step by K step, byte (r, t) at (t / 128) * rows * 128 + r * 128 + t % 128
 *     (T a multiple of 128, else LLMQ_ERR_SHAPE): the 128 contraction bytes of all rows for one K step are one
 *     contiguous piece.  The arithmetic and its order are those of LLMQ_LAYOUT_ROWS: same result bytes.
 *   a_t_major: layout of A ([T,R] when T-major);   b_t_major: layout of B;   both 0: identical to
 *   llmq_fp8_gemm_tn.  Other values: LLMQ_ERR_FLAGS.
 * The paper keeps transposed FP8 copies of every quantized tensor because the FP8 GEMM it builds on only
 * takes contraction-contiguous operands, and names the extra transposes and buffers as the cost of FP8
 * (Section 3, kernel-fusion paragraph; Section 4 "Impact of FP8").  Here the tile kernel transposes a
 * T-major operand on its way from LDS to the matrix cores, so the backward GEMMs can read the row-major
 * copies the forward pass made:
 *   dX[m,k] = sum_n dYq[m,n] Wq[n,k]   : A = dYq [M,N],            B = Wq [N,K] T-major, T = N
 *   dW[n,k] = sum_m dYq[m,n] Xq[m,k]   : A = dYq [M,N] T-major,    B = Xq [M,K] T-major, T = M
 * Tuned for B in E4M3 with R, C multiples of 128, T a multiple of 128 and T-major operands below 2 GiB; other
 * cases take a slow generic kernel.  In the tuned kernel (and likewise in the generic one) every product lands in the same accumulator
 * position as with transposed copies, so the result is bit-identical to llmq_fp8_gemm_tn on those copies
 * whenever both calls run the same kind of kernel, which is the case for what the linear calls below launch
 * on operands below 2 GiB.  Arguments otherwise as above.
 */
#define LLMQ_LAYOUT_ROWS    0
#define LLMQ_LAYOUT_T_MAJOR 1
#define LLMQ_LAYOUT_SLABS   2
int llmq_fp8_gemm(const uint8_t* A, int fmtA, int a_t_major, const uint8_t* B, int fmtB, int b_t_major,
                  int64_t R, int64_t C, int64_t T,
                  const float* d_scaleA, const float* d_scaleB,
                  void* c_bf16, int accumulate, float* d_amax_c, void* stream);

/*
 * The same contraction with caller-owned scratch, which lets the library share out a ragged last round of
 * output tiles: the chip computes one tile per CU at a time, and when the number of tiles is not a multiple of
 * the number of CUs the last round leaves CUs idle (560 tiles on 256 CUs take three rounds, the third with 48
 * tiles).  With scratch, the left-over tiles are cut along the contraction index and dealt to all CUs; every
 * piece is written to the scratch as binary32 accumulators, and a second launch adds the pieces of a tile in
 * the fixed order of their contraction ranges and finishes the tile (de-scale, BF16, absmax).  No atomic
 * additions, no dependence on timing: same inputs, same bytes (Section 3 "Reproducibility": an intermediate
 * buffer and a second step instead of atomics).  The sums are grouped differently from a call without scratch,
 * so the two may differ in the last bit of an output; both are within the error bound above.
 *   scratch        device memory, 256-byte aligned, at least llmq_fp8_gemm_scratch_bytes(R, C, T) bytes for the
 *                  sharing to happen; NULL or a smaller buffer: every tile is computed whole (as llmq_fp8_gemm).
 *                  Contents on entry do not matter; calls that may overlap on the device need separate scratch.
 * llmq_fp8_gemm_scratch_bytes returns 0 for shapes the library computes whole anyway: whole rounds, small
 * problems, T-major operands, and every shape for which sharing was not measured to win.  The chip is
 * power-limited on real data, so CUs left idle by a ragged round let the busy ones clock higher and the round
 * costs less than a full one; sharing pays (3-7 % of one isolated GEMM) only for long contractions
 * (T >= 16384) whose left-over tiles all fit one group of pieces.  The linear calls below do not use it.
 */
size_t llmq_fp8_gemm_scratch_bytes(int64_t R, int64_t C, int64_t T);
int llmq_fp8_gemm_with_scratch(const uint8_t* A, int fmtA, int a_t_major, const uint8_t* B, int fmtB, int b_t_major,
                               int64_t R, int64_t C, int64_t T,
                               const float* d_scaleA, const float* d_scaleB,
                               void* c_bf16, int accumulate, float* d_amax_c,
                               void* scratch, size_t scratch_bytes, void* stream);

/*
 * BF16 baseline of the same contraction, for the FP8-versus-BF16 comparison the paper reports (Section 4,
 * "Impact of FP8", speed-up column of Table 1): no quantization, no scales,
 *   c[r,cc] = bf16( sum_t A[r,t] * B[cc,t] )   (+ c[r,cc] first when accumulate != 0)
 * A [R,T], B [C,T] BF16 with the contraction index contiguous, binary32 accumulation on the matrix cores
 * (v_mfma_f32_16x16x32_bf16 in the same tile kernel), one RNE rounding.  Error per element is bounded by
 * 2^-8 |c| + T 2^-24 sum_t |A[r,t] B[cc,t]|.  Shapes with R, C multiples of 128 and T a multiple of 64
 * take the tuned kernel, others a slow generic one.
 */
int llmq_bf16_gemm_tn(const void* A_bf16, const void* B_bf16, int64_t R, int64_t C, int64_t T,
                      void* c_bf16, int accumulate, void* stream);

/*
 * Workspace of the three linear-layer calls below, for one (M, N, K).  It holds the FP8 copies
 *   Xq [M,K], Wq [N,K], dYq [M,N], then 12 KB of scratch for the LLMQ_JIT_* flags, then
 *   Xq_t [K,M], Wq_t [K,N], dYq_t [N,M],
 * each starting at a multiple of 256 bytes.  llmq_fp8_linear_workspace_offsets() returns the byte offsets of
 * the copies in the order Xq, Xq_t, Wq, Wq_t, dYq, dYq_t.  Calls that carry LLMQ_NO_TRANSPOSE touch nothing
 * behind the scratch and accept a workspace of llmq_fp8_linear_workspace_bytes_no_transpose() bytes (half the
 * FP8 copies); calls that carry LLMQ_SHARE_TILES need llmq_fp8_linear_workspace_bytes_shared() bytes: the same
 * layout with a section for the binary32 pieces of shared tiles behind it (0-100 MB more, by the shapes).
 * The caller owns the workspace and may read the copies between calls.
 */
size_t llmq_fp8_linear_workspace_bytes(int64_t M, int64_t N, int64_t K);
size_t llmq_fp8_linear_workspace_bytes_no_transpose(int64_t M, int64_t N, int64_t K);
size_t llmq_fp8_linear_workspace_bytes_shared(int64_t M, int64_t N, int64_t K);
int llmq_fp8_linear_workspace_offsets(int64_t M, int64_t N, int64_t K, size_t offsets[6]);

/* `flags` of the linear calls: the named operand's FP8 copies are already in the workspace (written by
 * an earlier call with the same M, N, K and the same scale) and are not produced again.  The library takes the
 * caller's word for it: nothing in the workspace records what it holds, and a call that claims copies that are
 * not there computes on stale bytes and still returns LLMQ_OK.  Weights are
 * quantized once per optimizer step and reused across micro-steps and in the backward pass (Section 3,
 * weight caching), and the backward pass reuses the forward's copies of X. */
#define LLMQ_REUSE_X  1
#define LLMQ_REUSE_W  2
#define LLMQ_REUSE_DY 4
/* Just-in-time scaling inside the call (Section 3 "Overview": the scale is found right before the conversion,
 * at the price of one extra kernel for the global reduction): the named operand's d_scale_* is then an OUTPUT.
 * The call runs the first stage of the absmax reduction over the operand and the quantize kernel finishes it,
 * so the scale, the FP8 bytes and everything downstream are bit-identical to llmq_amax followed by the call
 * with the scale given, with one launch less.  Not together with the operand's REUSE flag. */
#define LLMQ_JIT_X   8
#define LLMQ_JIT_W  16
#define LLMQ_JIT_DY 32
/* No transposed copies: the call writes only the row-major FP8 copies (Xq, Wq, dYq) and the backward GEMMs
 * read those T-major (see llmq_fp8_gemm), which saves one byte written per quantized element and half the
 * workspace: the sections Xq_t, Wq_t, dYq_t are neither written nor read and need not exist.  Copies made
 * under this flag can only be reused (LLMQ_REUSE_*) by calls that carry it too, copies made without it by
 * any call; results are bit-identical either way. */
#define LLMQ_NO_TRANSPOSE 64
/* The call's contraction may share the output tiles of a ragged last round among all compute units, as
 * llmq_fp8_gemm_with_scratch does (pieces along the contraction index, added in a fixed order by a second
 * launch: Section 3 "Reproducibility"; run to run the same bytes).  The planner shares only where it was
 * measured to win (long contractions with few left-over tiles), so most shapes are not affected at all; where it
 * shares, the binary32 sums are taken in another order than with whole tiles, so the BF16 results may differ in
 * the last bit from those of a call without the flag (both within the error bound of llmq_fp8_gemm_tn).  In a
 * block's sequence of contractions it measured +1 % (32B- and 14B-class shapes).  Not together with LLMQ_NO_TRANSPOSE
 * (LLMQ_ERR_FLAGS); the workspace must hold llmq_fp8_linear_workspace_bytes_shared() bytes. */
#define LLMQ_SHARE_TILES 128
/* The transposed copies Xq_t, Wq_t, dYq_t are stored in slabs of 128 contraction bytes (LLMQ_LAYOUT_SLABS of the
 * contraction that reads them) instead of as plain transposed tensors, wherever the quantizer can write them so
 * (the untransposed tensor has a multiple of 128 rows and of 256 columns, less than 0x70000000 elements; other
 * tensors keep the plain form): a 128 x 256 tile of a tensor then lands as one contiguous 32 KB piece of its
 * transposed copy instead of 256 pieces of 128 bytes, and every K step of a backward contraction reads one
 * contiguous piece per operand.  Results are the same bytes as without the flag.  Copies made under this flag can
 * only be reused (LLMQ_REUSE_*) by calls that carry it too (the producers that write FP8 directly make such
 * copies with llmq_swiglu_fwd_fp8_slabs and llmq_rmsnorm_apply_fp8_slabs), and copies made without it (or by
 * llmq_swiglu_fwd_fp8 and llmq_rmsnorm_apply_fp8) only by calls without it.  Not together with
 * LLMQ_NO_TRANSPOSE (LLMQ_ERR_FLAGS). */
#define LLMQ_SLAB_COPIES 256

/*
 * Forward: Y[M,N] = X[M,K] W[N,K]^T in FP8 (E4M3 x E4M3), BF16 out.
 * Quantizes X and W (both layouts each, unless LLMQ_REUSE_X / LLMQ_REUSE_W; row-major only under
 * LLMQ_NO_TRANSPOSE) with the given scales, then
 * runs the contraction on Xq and Wq.  d_amax_y may be NULL.
 */
int llmq_fp8_linear_fwd(const void* X, const void* W, int64_t M, int64_t N, int64_t K,
                        float* d_scale_x, float* d_scale_w,
                        void* Y, float* d_amax_y, void* ws, size_t ws_bytes, int flags, void* stream);

/*
 * Input gradient: dX[M,K] = dY[M,N] W[N,K].  dY is quantized to fmt_dy (E5M2 or E4M3; the paper tried
 * both, Section 5 Scenario 1) unless LLMQ_REUSE_DY; W unless LLMQ_REUSE_W.  Contraction over N on dYq and
 * Wq_t (on Wq read T-major under LLMQ_NO_TRANSPOSE).  W and dY pointers are not read for operands whose REUSE flag is set (and may then be NULL).
 */
int llmq_fp8_linear_dgrad(const void* dY, const void* W, int64_t M, int64_t N, int64_t K,
                          float* d_scale_dy, float* d_scale_w, int fmt_dy,
                          void* dX, float* d_amax_dx, void* ws, size_t ws_bytes, int flags, void* stream);

/*
 * Weight gradient: dW[N,K] = dY[M,N]^T X[M,K] (accumulate != 0: dW += ..., in BF16).  Contraction over M on
 * dYq_t and Xq_t (on dYq and Xq read T-major under LLMQ_NO_TRANSPOSE).
 */
int llmq_fp8_linear_wgrad(const void* dY, const void* X, int64_t M, int64_t N, int64_t K,
                          float* d_scale_dy, float* d_scale_x, int fmt_dy,
                          void* dW, int accumulate, void* ws, size_t ws_bytes, int flags, void* stream);

/*
 * Scale from an absmax that a fused producer left on the device (the d_amax_* outputs of the calls above):
 *   d_scale[0] = min(FMAX(fmt) / d_amax[0], FLT_MAX), 1 if d_amax[0] == 0: the same rule and rounding as llmq_amax.
 */
int llmq_scale_from_amax(const float* d_amax, int fmt, float* d_scale, void* stream);

/*
 * SwiGLU with the extra outputs of the FP8 pipeline (Section 3, kernel-fusion paragraph: every
 * non-linearity also returns the absmax of its result; Section 3 "Activation checkpointing": with the
 * absmax known, as in recomputation during backward, the FP8 conversion is fused into the non-linearity).
 *
 *   GU [M, 2I] BF16, the output of the gate+up projection: columns [0, I) are the gate g, columns
 *   [I, 2I) the up branch u.   h[m,i] = bf16( silu(g) * u ),  silu(g) = g * sg,  sg = 1 / (1 + e^-g).
 *   The value is evaluated in IEEE binary32, operation by operation (so that the BF16 bits, and with them
 *   the absmax and the FP8 codes, are reproducible anywhere):
 *     a = -min(max(g, -100), 86);  n = rint(a * LOG2E);  r = fma(n, -LN2_HI, a);  r = fma(n, -LN2_LO, r);
 *     p = 1 + r(1 + r(1/2 + r(1/6 + r(1/24 + r(1/120 + r/720)))))  (Horner, one fma per level);
 *     e = p * 2^n;  sg = 1 / (1 + e);  h = bf16( (g * sg) * u ),  one RNE rounding to BF16.
 *   LOG2E, LN2_HI, LN2_LO, 1/k! are the binary32 numbers nearest to log2 e, ln 2, ln 2 - LN2_HI, 1/k!.
 *   Against the exact function the result is within half a BF16 ulp (+ 2^-20 relative); for g <= -89,
 *   where |silu(g)| < 2^-121, it is +-0.  Non-finite inputs are outside the contract.
 *
 * llmq_swiglu_fwd: writes h [M, I] (BF16), d_amax_h[0] = max |h| and, if d_scale_h is not NULL, the scale of
 *   h for format fmt (as llmq_amax would for h, bit for bit).  ws: device scratch of at least
 *   llmq_swiglu_workspace_bytes(M, I) bytes, 16-byte aligned, contents irrelevant on entry (per-workgroup
 *   partial results, reduced by a second kernel: no atomics).
 * llmq_swiglu_fwd_fp8: the scale is known (kept from the forward pass): writes q [M, I] = the FP8 codes
 *   llmq_quantize_fp8 would produce from h with *d_scale_h, q_t [I, M] their transposed copy if not NULL,
 *   and h itself only if h_bf16 is not NULL.  With q and q_t pointing at the Xq / Xq_t sections of a linear
 *   workspace, the down projection then runs with LLMQ_REUSE_X.
 * llmq_swiglu_fwd_fp8_slabs: the same with q_t (required) in slabs of 128 contraction bytes, exactly what
 *   llmq_quantize_fp8_slabs writes from h (byte (i, m) of the transposed tensor at (m / 128) I 128 + i 128 + m % 128),
 *   for a down projection that runs with LLMQ_REUSE_X | LLMQ_SLAB_COPIES.  M % 128 == 0, I % 256 == 0 and
 *   M I < 0x70000000 (the tensors such a linear call keeps in slabs), else LLMQ_ERR_SHAPE.
 * llmq_swiglu_bwd: dh [M, I], GU [M, 2I] -> dGU [M, 2I] (same column layout):
 *     dGU[m, I+i] = bf16( dh * (g * sg) ),   dGU[m, i] = bf16( ((dh * u) * sg) * fma(g, 1 - sg, 1) ),
 *   plus absmax and, if wanted, scale (format fmt) of dGU, which is the dY of the gate+up projection.
 * M, I >= 1, I < 2^24; GU, h, dh, dGU 16-byte aligned and I % 8 == 0 for that to hold for every row (other
 * I, and M not a multiple of 4, or of 16 with q_t, take a slower generic kernel; with q_t, M % 128 == 0 and
 * I % 256 == 0 take the fastest one).
 */
size_t llmq_swiglu_workspace_bytes(int64_t M, int64_t I);
int llmq_swiglu_fwd(const void* gu_bf16, int64_t M, int64_t I, void* h_bf16, int fmt,
                    float* d_amax_h, float* d_scale_h, void* ws, size_t ws_bytes, void* stream);
int llmq_swiglu_fwd_fp8(const void* gu_bf16, int64_t M, int64_t I, const float* d_scale_h, int fmt,
                        uint8_t* q, uint8_t* q_t, void* h_bf16, void* stream);
int llmq_swiglu_fwd_fp8_slabs(const void* gu_bf16, int64_t M, int64_t I, const float* d_scale_h, int fmt,
                              uint8_t* q, uint8_t* q_t, void* h_bf16, void* stream);
int llmq_swiglu_bwd(const void* dh_bf16, const void* gu_bf16, int64_t M, int64_t I, void* dgu_bf16, int fmt,
                    float* d_amax_dgu, float* d_scale_dgu, void* ws, size_t ws_bytes, void* stream);

/*
 * RMSNorm joined with the residual addition, with the extra outputs of the FP8 pipeline (Section 3,
 * kernel-fusion paragraph: one kernel for both, which also returns the absmax of the normalised output;
 * Section 3 "Activation checkpointing": statistics kept from the forward pass let the recomputation emit
 * FP8 directly).
 *
 *   res'[m,c] = bf16( res[m,c] + x[m,c] )       one binary32 addition, one RNE rounding; the stored stream
 *   rstd[m]   = 1 / sqrt( (1/C) sum_c res'[m,c]^2 + eps )     of the BF16-rounded res'; binary32
 *   y[m,c]    = bf16( (res'[m,c] * rstd[m]) * w[c] )          two binary32 multiplications, one rounding
 *   res, x, res', y [M, C] BF16; w [C] BF16; rstd [M] float.
 *
 * llmq_rmsnorm_fwd: x may be NULL (no addition: res is normalised as it is and res_out is ignored);
 *   otherwise res_out receives res' and may be the same buffer as res (in place).  Writes y, rstd (kept for
 *   the backward pass / recomputation), d_amax_y = max |y| and, if not NULL, d_scale_y for format fmt, both
 *   bit-identical to llmq_amax of y.  The row sum runs in binary32 in an order of the kernel's choosing, so
 *   rstd is reproducible run to run but only equal to the exact value within 2^-20 relative; y then is the
 *   formula above evaluated with that rstd.  ws: at least llmq_rmsnorm_workspace_bytes(M) bytes, 16-byte
 *   aligned, contents irrelevant (per-workgroup partial absmax; no atomics).
 * llmq_rmsnorm_apply_fp8: the recompute path.  res (the stored stream), w, rstd and the scale of y are
 *   given; writes q [M, C] = the FP8 codes llmq_quantize_fp8 would produce from y with *d_scale_y, their
 *   transposed copy q_t [C, M] if not NULL, and y itself only if y_bf16 is not NULL.  Element-wise, hence
 *   reproducible bit for bit from its inputs.  rstd must be 16-byte aligned.
 * llmq_rmsnorm_apply_fp8_slabs: the same with q_t (required) in slabs of 128 contraction bytes, as
 *   llmq_quantize_fp8_slabs writes it from y, for a linear call with LLMQ_REUSE_X | LLMQ_SLAB_COPIES.
 *   M % 128 == 0, C % 256 == 0 and M C < 0x70000000, else LLMQ_ERR_SHAPE.
 * M, C >= 1, C < 2^24.  C % 8 == 0 and C <= 8192 take the single-pass forward kernel; M % 16 == 0 (M % 4
 * without q_t) and C % 8 == 0 the tuned recompute kernels (with q_t, M % 128 == 0 and C % 256 == 0 the fastest
 * one); other shapes slower generic ones.
 */
size_t llmq_rmsnorm_workspace_bytes(int64_t M);
int llmq_rmsnorm_fwd(const void* res_bf16, const void* x_bf16, const void* w_bf16, int64_t M, int64_t C,
                     float eps, void* res_out_bf16, void* y_bf16, float* rstd, int fmt, float* d_amax_y,
                     float* d_scale_y, void* ws, size_t ws_bytes, void* stream);
int llmq_rmsnorm_apply_fp8(const void* res_bf16, const void* w_bf16, const float* rstd, int64_t M, int64_t C,
                           const float* d_scale_y, int fmt, uint8_t* q, uint8_t* q_t, void* y_bf16,
                           void* stream);
int llmq_rmsnorm_apply_fp8_slabs(const void* res_bf16, const void* w_bf16, const float* rstd, int64_t M,
                                 int64_t C, const float* d_scale_y, int fmt, uint8_t* q, uint8_t* q_t,
                                 void* y_bf16, void* stream);

/*
 * Peak calibration (the paper's appendix "A note on MFU" measures the attainable peak with a large-matmul
 * micro-benchmark instead of trusting the spec sheet).  Both calls only enqueue; the caller times them.
 *
 * llmq_calibrate_mfma: a register-only loop of the GEMM's FP8 MFMA instruction (v_mfma_f32_16x16x128_f8f6f4 in
 *   the 8 x 8 block pattern of a wave tile, one workgroup of 4 waves per CU, `iters` passes of 64 MFMAs per wave;
 *   the 32x32x64 form of the instruction sustains about a tenth less on random bits) with operand registers holding
 *   constants (random_bits == 0) or random FP8 bits (random_bits != 0; the matrix cores are power-limited and
 *   sustain a lower clock on random bits, as on real quantized data).  d_sink: [1] float, device, practically
 *   never written.  *flops (host pointer, may be NULL) receives the FLOP count of the launch.
 * llmq_calibrate_copy: plain device copy of `bytes` (multiple of 16, 16-byte aligned pointers): 2 * bytes of
 *   HBM traffic.
 */
/*
 * llmq_calibrate_gemm_phases: one E4M3 x E4M3 contraction (arguments as llmq_fp8_gemm_tn; R, C multiples of 256,
 *   T a multiple of 128) by the 256 x 256 tile kernel built with phase stamps: wave 0 of every workgroup writes
 *   the cycle counter into d_stamps[16 * workgroup + s] and the 100 MHz clock into d_stamps[16 * workgroup + 8 + s]
 *   (64-bit words) for s = 0 start, 1 first operand fragments in registers (end of the prologue), 2 end of the
 *   contraction loop, 4 last output store issued, 5 absmax done, 3 all stores completed.  Workgroup ids beyond the
 *   number of tiles leave their words untouched.  d_stamps: device, 8-byte aligned, at least
 *   llmq_calibrate_gemm_phases_bytes(R, C) bytes.  ieee_maximum != 0: the fused absmax as the library computes
 *   it (IEEE 754-2019 maximum); 0: the maxNum form it replaced, for comparison.  The results c and d_amax_c are
 *   those of llmq_fp8_gemm_tn.
 */
size_t llmq_calibrate_gemm_phases_bytes(int64_t R, int64_t C);
int llmq_calibrate_gemm_phases(const uint8_t* A, const uint8_t* B, int64_t R, int64_t C, int64_t T,
                               const float* d_scaleA, const float* d_scaleB, void* c_bf16, float* d_amax_c,
                               void* d_stamps, size_t stamps_bytes, int ieee_maximum, void* stream);
int llmq_calibrate_mfma(int fmtA, int fmtB, int random_bits, int iters, float* d_sink, double* flops,
                        void* stream);
int llmq_calibrate_copy(const void* src, void* dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LLMQ_H */
