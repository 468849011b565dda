// Host-side launchers of the gfx950 kernels (internal to the library; the public ABI is llmq.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

namespace llmq {

// Tuning overrides come from the environment, for tests and tuning runs only: they are looked at when the
// process started with LLMQ_TUNING=1 (read once) and ignored otherwise, so the product path never calls
// getenv at launch.
inline const char* tuning_env(const char* name) {
    static const bool enabled = [] { const char* e = getenv("LLMQ_TUNING"); return e && e[0] == '1'; }();
    return enabled ? getenv(name) : nullptr;
}

// The workgroup tile of the kernels that write FP8 codes in both layouts (quantize, and the SwiGLU and RMSNorm
// kernels that emit FP8 directly): tensors made of whole tiles take the tile kernels, and only those can write
// the transposed copy in slabs.
constexpr int kTileRows = 128, kTileCols = 256;
inline bool tile_shape_ok(int64_t rows, int64_t cols) { return rows % kTileRows == 0 && cols % kTileCols == 0; }

// Each returns 0 or LLMQ_ERR_DEVICE (-6).  Arguments are validated by the callers in api.hip.
constexpr int kAmaxMaxPartials = 1024;      // the absmax workspace holds one 32-bit word per block
int launch_amax(const void* x, size_t n, int fmt, float* d_amax, float* d_scale, void* ws,
                hipStream_t stream, int num_cus);
// The same with the partial results in the library's own file-scope device array (no workspace, no allocation).
int launch_amax_static(const void* x, size_t n, int fmt, float* d_amax, float* d_scale, hipStream_t stream,
                       int num_cus);
// Second stage of every absmax reduction: the maximum of n_partial BF16 magnitude patterns (one per
// workgroup of the first stage) becomes d_amax and, if d_scale is not NULL, the scale for fmt.
int launch_amax_final(const unsigned* partial, int n_partial, int fmt, float* d_amax, float* d_scale,
                      hipStream_t stream);
// BF16 x BF16 -> BF16 contraction without scales (T in elements), the baseline of the FP8 GEMM.
int launch_gemm_bf16_tn(const void* A, const void* B, int64_t R, int64_t C, int64_t T, void* c_bf16,
                        int accumulate, hipStream_t stream, int num_cus);
int launch_scale_from_amax(const float* d_amax, int fmt, float* d_scale, hipStream_t stream);
// zero_word: if not NULL, one 32-bit word the kernel also clears (the absmax accumulator of the GEMM
// that follows in the same call, which saves a launch).
// qt_slabs: the transposed copy is written in slabs of 128 contraction bytes (kLayoutSlabs of the contraction that
// reads it: [cols, rows] with rows the contraction index), which only the tile kernel does: ask
// quantize_can_write_slabs() first (else -2).
int launch_quantize(const void* x, int64_t rows, int64_t cols, const float* d_scale, int fmt,
                    uint8_t* q, uint8_t* q_t, unsigned* zero_word, hipStream_t stream, bool qt_slabs = false);
bool quantize_can_write_slabs(int64_t rows, int64_t cols);
// Where a quantizing kernel gets its scale from: a scale on the device, or the per-workgroup results of
// the first stage of an absmax reduction over the same tensor, in which case every workgroup finishes the
// reduction itself (at most 1024 words) and the first one also stores the scale: the second-stage launch of
// the absmax is saved.
struct ScaleSource {
    const float* d_scale;        // used when partial == nullptr
    const unsigned* partial;     // BF16 magnitude patterns, one per workgroup of the first stage
    int n_partial;
    float fmax;                  // largest finite value of the target format
    float* d_scale_out;          // written (by one workgroup) when partial != nullptr
};

// The same with the scale taken from a ScaleSource (a given scale, or the first-stage results of an absmax).
int launch_quantize_from(const void* x, int64_t rows, int64_t cols, const ScaleSource& src, int fmt,
                         uint8_t* q, uint8_t* q_t, unsigned* zero_word, hipStream_t stream, bool qt_slabs = false);
// First stage of the absmax only: one BF16 magnitude pattern per workgroup into partial; returns the number
// of workgroups (<= kAmaxMaxPartials) through n_partial.
int launch_amax_partial(const void* x, size_t n, unsigned* partial, int* n_partial, hipStream_t stream, int num_cus);
// Caller-owned device scratch for the binary32 pieces of output tiles whose contraction is shared among
// several workgroups (a ragged last round of tiles); {nullptr, 0}: every tile is computed by one workgroup.
struct GemmScratch {
    float* ptr;
    size_t bytes;
};
// What a contraction of this shape would use of it (0: nothing).
size_t gemm_scratch_bytes(int64_t R, int64_t C, int64_t T, int num_cus);
// How an operand [rows, T] of a contraction sits in memory: its rows of T contiguous bytes one after the other;
// the transposed tensor [T, rows]; or K step by K step ("slabs": byte (r, t) at (t / 128) rows 128 + r 128 + t % 128,
// T a multiple of 128), which is how the quantizer's tile kernel can write a transposed copy in contiguous pieces.
enum OperandLayout { kLayoutRows = 0, kLayoutTMajor = 1, kLayoutSlabs = 2 };
// Both operands kLayoutRows or kLayoutSlabs (slabs_a, slabs_b).
int launch_gemm_tn(const uint8_t* A, int fmtA, const uint8_t* B, int fmtB, int64_t R, int64_t C,
                   int64_t T, const float* d_scaleA, const float* d_scaleB, void* c_bf16,
                   int accumulate, float* d_amax_c, bool amax_is_zeroed, hipStream_t stream, int num_cus,
                   GemmScratch scratch, bool slabs_a = false, bool slabs_b = false);

// The 256 x 256 tile kernel with phase stamps: 16 words of 64 bits per workgroup id, gemm_phase_stamp_blocks() ids.
int gemm_phase_stamp_blocks(int64_t R, int64_t C);
int launch_gemm_phase_stamps(const uint8_t* A, const uint8_t* B, int64_t R, int64_t C, int64_t T, const float* sA,
                             const float* sB, void* c_bf16, float* d_amax_c, long long* stamps, int ieee_maximum,
                             hipStream_t stream, int num_cus);

// The same contraction with either operand in any OperandLayout: kLayoutTMajor: A is [T, R], B is [T, C] (the
// contraction index runs down the rows), so the backward GEMMs can read the untransposed quantized tensors.
int launch_gemm_fp8(const uint8_t* A, int fmtA, int layout_a, const uint8_t* B, int fmtB, int layout_b, int64_t R, int64_t C,
                    int64_t T, const float* d_scaleA, const float* d_scaleB, void* c_bf16, int accumulate,
                    float* d_amax_c, bool amax_is_zeroed, hipStream_t stream, int num_cus, GemmScratch scratch);

// SwiGLU with its extra outputs.  h, d_amax (with partial, the per-workgroup scratch), q and q_t are
// optional; q_fmt is only read when q is given.  swiglu_blocks() is the number of scratch words.
// qt_slabs (here and in the RMSNorm recompute launch): q_t in slabs of 128 contraction bytes, as in
// launch_quantize; needs q_t and tile_shape_ok(M, columns), else -2.
int64_t swiglu_blocks(int64_t M, int64_t I);
int launch_swiglu_fwd(const void* gu, int64_t M, int64_t I, void* h, unsigned* partial, int amax_fmt,
                      float* d_amax, float* d_scale, const float* d_qscale, int q_fmt, uint8_t* q, uint8_t* q_t,
                      hipStream_t stream, bool qt_slabs = false);
int launch_swiglu_bwd(const void* dh, const void* gu, int64_t M, int64_t I, void* dgu, unsigned* partial,
                      int amax_fmt, float* d_amax, float* d_scale, hipStream_t stream);

// RMSNorm + residual addition with absmax of the output (x, res_out optional together), and the
// element-wise recompute path that turns res, rstd and a known scale into FP8 codes (q_t, y optional).
// rmsnorm_blocks() is the number of scratch words of the forward launch.
int64_t rmsnorm_blocks(int64_t M);
int launch_rmsnorm_fwd(const void* res, const void* x, const void* w, int64_t M, int64_t C, float eps,
                       void* res_out, void* y, float* rstd, unsigned* partial, int fmt, float* d_amax,
                       float* d_scale, hipStream_t stream);
int launch_rmsnorm_apply_fp8(const void* res, const void* w, const float* rstd, int64_t M, int64_t C,
                             const float* d_qscale, int fmt, uint8_t* q, uint8_t* q_t, void* y, hipStream_t stream,
                             bool qt_slabs = false);

int launch_calibrate_mfma(int fmtA, int fmtB, int random_bits, int iters, float* d_sink, hipStream_t stream,
                          int num_cus);
int launch_calibrate_copy(const void* src, void* dst, size_t bytes, hipStream_t stream);

}  // namespace llmq
