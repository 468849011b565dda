// C ABI of the FP8 linear path: argument checks and launch sequencing only; all arithmetic is in
// the kernels (amax.hip, quantize.hip, gemm.hip, swiglu.hip, rmsnorm.hip).  Declarations and contracts: include/llmq.h.
#include <hip/hip_runtime.h>

#include "../../include/llmq.h"
#include "llmq_kernels.h"

namespace {

constexpr int64_t kMaxDim = (int64_t)1 << 31;        // per dimension
constexpr int64_t kMaxElems = (int64_t)1 << 40;      // per tensor

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline bool fmt_ok(int f) { return f == LLMQ_E4M3 || f == LLMQ_E5M2; }
inline bool dim_ok(int64_t d) { return d >= 1 && d < kMaxDim; }
inline size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

int num_cus() {
    static int cached = 0;                              // benign race: every thread computes the same value
    if (cached == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cached = n;
    }
    return cached;
}

struct WsLayout {
    size_t xq, xqt, wq, wqt, dyq, dyqt, part;     // part: three absmax scratch areas (X, W, dY)
    size_t compact, total;                        // bytes needed without / with the transposed copies
    size_t pieces, pieces_bytes, shared_total;    // LLMQ_SHARE_TILES: binary32 pieces of shared tiles behind everything else
};

// Row-major copies and the scratch first, the transposed copies behind them: a workspace that ends after the
// scratch serves every call that carries LLMQ_NO_TRANSPOSE.
WsLayout ws_layout(int64_t M, int64_t N, int64_t K) {
    WsLayout l;
    size_t off = 0;
    l.xq = off;   off += round256((size_t)M * K);
    l.wq = off;   off += round256((size_t)N * K);
    l.dyq = off;  off += round256((size_t)M * N);
    l.part = off; off += 3 * round256((size_t)llmq::kAmaxMaxPartials * sizeof(unsigned));
    l.compact = off;
    l.xqt = off;  off += round256((size_t)M * K);
    l.wqt = off;  off += round256((size_t)N * K);
    l.dyqt = off; off += round256((size_t)M * N);
    l.total = off;
    // what the largest of the three contractions may write when its ragged last round of tiles is shared out
    size_t need = llmq::gemm_scratch_bytes(M, N, K, num_cus());
    const size_t dgrad = llmq::gemm_scratch_bytes(M, K, N, num_cus()), wgrad = llmq::gemm_scratch_bytes(N, K, M, num_cus());
    if (dgrad > need) need = dgrad;
    if (wgrad > need) need = wgrad;
    l.pieces = off; l.pieces_bytes = round256(need); off += l.pieces_bytes;
    l.shared_total = off;
    return l;
}

// The scratch a linear call hands to its contraction: the pieces section under LLMQ_SHARE_TILES, nothing otherwise
// (every output tile is then computed whole).
llmq::GemmScratch pieces_of(const WsLayout& l, void* ws, int flags) {
    if (!(flags & LLMQ_SHARE_TILES) || l.pieces_bytes == 0) return llmq::GemmScratch{nullptr, 0};
    return llmq::GemmScratch{reinterpret_cast<float*>(static_cast<uint8_t*>(ws) + l.pieces), l.pieces_bytes};
}

int check_linear(int64_t M, int64_t N, int64_t K, const void* ws, size_t ws_bytes, int flags) {
    if (!dim_ok(M) || !dim_ok(N) || !dim_ok(K)) return LLMQ_ERR_SHAPE;
    if (M * K >= kMaxElems || N * K >= kMaxElems || M * N >= kMaxElems) return LLMQ_ERR_SHAPE;
    if (flags & ~(LLMQ_REUSE_X | LLMQ_REUSE_W | LLMQ_REUSE_DY | LLMQ_JIT_X | LLMQ_JIT_W | LLMQ_JIT_DY | LLMQ_NO_TRANSPOSE | LLMQ_SHARE_TILES | LLMQ_SLAB_COPIES)) return LLMQ_ERR_FLAGS;
    if ((flags & LLMQ_SLAB_COPIES) && (flags & LLMQ_NO_TRANSPOSE)) return LLMQ_ERR_FLAGS;       // no transposed copies to lay out
    // tiles are shared only by the kernels for contraction-contiguous operands
    if ((flags & LLMQ_SHARE_TILES) && (flags & LLMQ_NO_TRANSPOSE)) return LLMQ_ERR_FLAGS;
    // an operand is either reused or scaled just in time, not both
    if (((flags & LLMQ_REUSE_X) && (flags & LLMQ_JIT_X)) || ((flags & LLMQ_REUSE_W) && (flags & LLMQ_JIT_W)) ||
        ((flags & LLMQ_REUSE_DY) && (flags & LLMQ_JIT_DY)))
        return LLMQ_ERR_FLAGS;
    if (!ws) return LLMQ_ERR_NULL;
    if (!aligned(ws, 256)) return LLMQ_ERR_ALIGN;
    const WsLayout l = ws_layout(M, N, K);
    if (ws_bytes < ((flags & LLMQ_NO_TRANSPOSE) ? l.compact : (flags & LLMQ_SHARE_TILES) ? l.shared_total : l.total)) return LLMQ_ERR_WORKSPACE;
    return LLMQ_OK;
}

int check_swiglu_shape(int64_t M, int64_t I) {
    if (!dim_ok(M) || !dim_ok(I) || I >= ((int64_t)1 << 24) || M * I >= kMaxElems / 2) return LLMQ_ERR_SHAPE;
    return LLMQ_OK;
}

// Quantize one operand of a linear call into its two workspace sections.  jit: the scale is not given but
// found here: the first absmax stage runs over the tensor, the quantize kernel finishes the reduction and
// stores the scale in d_scale (saving the launch of the second stage).
int quantize_operand(const void* t, int64_t rows, int64_t cols, float* d_scale, int fmt, uint8_t* q, uint8_t* q_t,
                     bool jit, unsigned* partial, unsigned* zero, hipStream_t s, bool qt_slabs) {
    if (!jit) return llmq::launch_quantize(t, rows, cols, d_scale, fmt, q, q_t, zero, s, qt_slabs);
    int n_partial = 0;
    int st = llmq::launch_amax_partial(t, (size_t)rows * (size_t)cols, partial, &n_partial, s, num_cus());
    if (st) return st;
    const llmq::ScaleSource src{nullptr, partial, n_partial, fmt == LLMQ_E4M3 ? 448.0f : 57344.0f, d_scale};
    return llmq::launch_quantize_from(t, rows, cols, src, fmt, q, q_t, zero, s, qt_slabs);
}

// Under LLMQ_SLAB_COPIES the transposed copy of a tensor [rows, cols] is stored in slabs of 128 contraction bytes
// whenever the quantizer's tile kernel takes the tensor (a pure function of the shape, so that the call that
// writes a copy and the calls that reuse it agree); otherwise as the plain transposed tensor.
constexpr int64_t kMaxSlabElems = 0x70000000;      // tensors kept in slabs stay below this many elements

bool slab_copy(int flags, int64_t rows, int64_t cols) {
    return (flags & LLMQ_SLAB_COPIES) && llmq::quantize_can_write_slabs(rows, cols) && rows * cols < kMaxSlabElems;
}

}  // namespace

extern "C" {

const char* llmq_status_string(int status) {
    switch (status) {
        case LLMQ_OK: return "ok";
        case LLMQ_ERR_NULL: return "a required pointer is NULL";
        case LLMQ_ERR_SHAPE: return "a dimension is out of range";
        case LLMQ_ERR_ALIGN: return "a pointer is not aligned as required";
        case LLMQ_ERR_FORMAT: return "unknown FP8 format";
        case LLMQ_ERR_WORKSPACE: return "workspace too small";
        case LLMQ_ERR_DEVICE: return "HIP launch failed";
        case LLMQ_ERR_FLAGS: return "unknown flag bits";
        default: return "unknown status";
    }
}

int llmq_version(void) { return 212; }

size_t llmq_amax_workspace_bytes(void) { return (size_t)llmq::kAmaxMaxPartials * sizeof(unsigned); }

int llmq_amax(const void* x_bf16, size_t n, int fmt, float* d_amax, float* d_scale, void* ws, size_t ws_bytes,
              void* stream) {
    if (!x_bf16 || !d_amax || !ws) return LLMQ_ERR_NULL;
    if (n < 1 || n >= (size_t)kMaxElems) return LLMQ_ERR_SHAPE;
    if (!fmt_ok(fmt)) return LLMQ_ERR_FORMAT;
    if (!aligned(x_bf16, 16) || !aligned(d_amax, 4) || !aligned(d_scale, 4) || !aligned(ws, 4)) return LLMQ_ERR_ALIGN;
    if (ws_bytes < llmq_amax_workspace_bytes()) return LLMQ_ERR_WORKSPACE;
    return llmq::launch_amax(x_bf16, n, fmt, d_amax, d_scale, ws, static_cast<hipStream_t>(stream), num_cus());
}

int llmq_amax_static(const void* x_bf16, size_t n, int fmt, float* d_amax, float* d_scale, void* stream) {
    if (!x_bf16 || !d_amax) return LLMQ_ERR_NULL;
    if (n < 1 || n >= (size_t)kMaxElems) return LLMQ_ERR_SHAPE;      // the largest tensor llmq_amax takes
    if (!fmt_ok(fmt)) return LLMQ_ERR_FORMAT;
    if (!aligned(x_bf16, 16) || !aligned(d_amax, 4) || !aligned(d_scale, 4)) return LLMQ_ERR_ALIGN;
    return llmq::launch_amax_static(x_bf16, n, fmt, d_amax, d_scale, static_cast<hipStream_t>(stream), num_cus());
}

int llmq_quantize_fp8(const void* x_bf16, int64_t rows, int64_t cols, const float* d_scale, int fmt,
                      uint8_t* q, uint8_t* q_t, void* stream) {
    if (!x_bf16 || !d_scale || !q) return LLMQ_ERR_NULL;
    if (!dim_ok(rows) || !dim_ok(cols) || rows * cols >= kMaxElems) return LLMQ_ERR_SHAPE;
    if (!fmt_ok(fmt)) return LLMQ_ERR_FORMAT;
    if (!aligned(x_bf16, 16) || !aligned(q, 16) || !aligned(q_t, 16) || !aligned(d_scale, 4)) return LLMQ_ERR_ALIGN;
    return llmq::launch_quantize(x_bf16, rows, cols, d_scale, fmt, q, q_t, nullptr, static_cast<hipStream_t>(stream));
}

int llmq_quantize_fp8_slabs(const void* x_bf16, int64_t rows, int64_t cols, const float* d_scale, int fmt,
                            uint8_t* q, uint8_t* q_t, void* stream) {
    if (!x_bf16 || !d_scale || !q || !q_t) return LLMQ_ERR_NULL;
    if (!dim_ok(rows) || !dim_ok(cols) || rows * cols >= kMaxElems) return LLMQ_ERR_SHAPE;
    if (rows % 128 != 0 || cols % 256 != 0) return LLMQ_ERR_SHAPE;
    if (!fmt_ok(fmt)) return LLMQ_ERR_FORMAT;
    if (!aligned(x_bf16, 16) || !aligned(q, 16) || !aligned(q_t, 16) || !aligned(d_scale, 4)) return LLMQ_ERR_ALIGN;
    if (!llmq::quantize_can_write_slabs(rows, cols)) return LLMQ_ERR_SHAPE;
    return llmq::launch_quantize(x_bf16, rows, cols, d_scale, fmt, q, q_t, nullptr, static_cast<hipStream_t>(stream), true);
}

int llmq_fp8_gemm_tn(const uint8_t* A, int fmtA, const uint8_t* B, int fmtB, int64_t R, int64_t C, int64_t T,
                     const float* d_scaleA, const float* d_scaleB, void* c_bf16, int accumulate,
                     float* d_amax_c, void* stream) {
    if (!A || !B || !d_scaleA || !d_scaleB || !c_bf16) return LLMQ_ERR_NULL;
    if (!dim_ok(R) || !dim_ok(C) || !dim_ok(T)) return LLMQ_ERR_SHAPE;
    if (R * T >= kMaxElems || C * T >= kMaxElems || R * C >= kMaxElems) return LLMQ_ERR_SHAPE;
    if (!fmt_ok(fmtA) || !fmt_ok(fmtB)) return LLMQ_ERR_FORMAT;
    if (!aligned(A, 16) || !aligned(B, 16) || !aligned(c_bf16, 16) || !aligned(d_scaleA, 4) ||
        !aligned(d_scaleB, 4) || !aligned(d_amax_c, 4))
        return LLMQ_ERR_ALIGN;
    return llmq::launch_gemm_tn(A, fmtA, B, fmtB, R, C, T, d_scaleA, d_scaleB, c_bf16, accumulate, d_amax_c, false,
                                static_cast<hipStream_t>(stream), num_cus(), llmq::GemmScratch{nullptr, 0});
}

int llmq_fp8_gemm(const uint8_t* A, int fmtA, int a_t_major, const uint8_t* B, int fmtB, int b_t_major, int64_t R,
                  int64_t C, int64_t T, const float* d_scaleA, const float* d_scaleB, void* c_bf16, int accumulate,
                  float* d_amax_c, void* stream) {
    return llmq_fp8_gemm_with_scratch(A, fmtA, a_t_major, B, fmtB, b_t_major, R, C, T, d_scaleA, d_scaleB, c_bf16,
                                      accumulate, d_amax_c, nullptr, 0, stream);
}

size_t llmq_fp8_gemm_scratch_bytes(int64_t R, int64_t C, int64_t T) {
    if (!dim_ok(R) || !dim_ok(C) || !dim_ok(T)) return 0;
    return llmq::gemm_scratch_bytes(R, C, T, num_cus());
}

int llmq_fp8_gemm_with_scratch(const uint8_t* A, int fmtA, int a_t_major, const uint8_t* B, int fmtB, int b_t_major,
                               int64_t R, int64_t C, int64_t T, const float* d_scaleA, const float* d_scaleB,
                               void* c_bf16, int accumulate, float* d_amax_c, void* scratch, size_t scratch_bytes,
                               void* stream) {
    if (!A || !B || !d_scaleA || !d_scaleB || !c_bf16) return LLMQ_ERR_NULL;
    if (!dim_ok(R) || !dim_ok(C) || !dim_ok(T)) return LLMQ_ERR_SHAPE;
    if (R * T >= kMaxElems || C * T >= kMaxElems || R * C >= kMaxElems) return LLMQ_ERR_SHAPE;
    if (!fmt_ok(fmtA) || !fmt_ok(fmtB)) return LLMQ_ERR_FORMAT;
    if (!aligned(A, 16) || !aligned(B, 16) || !aligned(c_bf16, 16) || !aligned(d_scaleA, 4) ||
        !aligned(d_scaleB, 4) || !aligned(d_amax_c, 4) || !aligned(scratch, 256))
        return LLMQ_ERR_ALIGN;
    // operand layouts: 0 rows, 1 T-major, 2 slabs of 128 contraction bytes
    if (a_t_major < 0 || a_t_major > LLMQ_LAYOUT_SLABS || b_t_major < 0 || b_t_major > LLMQ_LAYOUT_SLABS) return LLMQ_ERR_FLAGS;
    if ((a_t_major == LLMQ_LAYOUT_SLABS || b_t_major == LLMQ_LAYOUT_SLABS) && T % 128 != 0) return LLMQ_ERR_SHAPE;
    const llmq::GemmScratch sc{scratch ? static_cast<float*>(scratch) : nullptr, scratch ? scratch_bytes : 0};
    return llmq::launch_gemm_fp8(A, fmtA, a_t_major, B, fmtB, b_t_major, R, C, T, d_scaleA, d_scaleB, c_bf16,
                                 accumulate, d_amax_c, false, static_cast<hipStream_t>(stream), num_cus(), sc);
}

int llmq_bf16_gemm_tn(const void* A_bf16, const void* B_bf16, int64_t R, int64_t C, int64_t T, void* c_bf16,
                      int accumulate, void* stream) {
    if (!A_bf16 || !B_bf16 || !c_bf16) return LLMQ_ERR_NULL;
    if (!dim_ok(R) || !dim_ok(C) || !dim_ok(T)) return LLMQ_ERR_SHAPE;
    if (R * T >= kMaxElems || C * T >= kMaxElems || R * C >= kMaxElems) return LLMQ_ERR_SHAPE;
    if (!aligned(A_bf16, 16) || !aligned(B_bf16, 16) || !aligned(c_bf16, 16)) return LLMQ_ERR_ALIGN;
    return llmq::launch_gemm_bf16_tn(A_bf16, B_bf16, R, C, T, c_bf16, accumulate, static_cast<hipStream_t>(stream),
                                     num_cus());
}

size_t llmq_fp8_linear_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    if (!dim_ok(M) || !dim_ok(N) || !dim_ok(K)) return 0;
    return ws_layout(M, N, K).total;
}

size_t llmq_fp8_linear_workspace_bytes_no_transpose(int64_t M, int64_t N, int64_t K) {
    if (!dim_ok(M) || !dim_ok(N) || !dim_ok(K)) return 0;
    return ws_layout(M, N, K).compact;
}

size_t llmq_fp8_linear_workspace_bytes_shared(int64_t M, int64_t N, int64_t K) {
    if (!dim_ok(M) || !dim_ok(N) || !dim_ok(K)) return 0;
    return ws_layout(M, N, K).shared_total;
}

int llmq_fp8_linear_workspace_offsets(int64_t M, int64_t N, int64_t K, size_t offsets[6]) {
    if (!offsets) return LLMQ_ERR_NULL;
    if (!dim_ok(M) || !dim_ok(N) || !dim_ok(K)) return LLMQ_ERR_SHAPE;
    const WsLayout l = ws_layout(M, N, K);
    offsets[0] = l.xq; offsets[1] = l.xqt; offsets[2] = l.wq; offsets[3] = l.wqt; offsets[4] = l.dyq; offsets[5] = l.dyqt;
    return LLMQ_OK;
}

int llmq_fp8_linear_fwd(const void* X, const void* W, int64_t M, int64_t N, int64_t K,
                        float* d_scale_x, float* d_scale_w, void* Y, float* d_amax_y,
                        void* ws, size_t ws_bytes, int flags, void* stream) {
    int st = check_linear(M, N, K, ws, ws_bytes, flags);
    if (st != LLMQ_OK) return st;
    if (flags & (LLMQ_REUSE_DY | LLMQ_JIT_DY)) return LLMQ_ERR_FLAGS;
    const bool qx = !(flags & LLMQ_REUSE_X), qw = !(flags & LLMQ_REUSE_W);
    if ((qx && !X) || (qw && !W) || !d_scale_x || !d_scale_w || !Y) return LLMQ_ERR_NULL;
    if ((qx && !aligned(X, 16)) || (qw && !aligned(W, 16)) || !aligned(Y, 16) || !aligned(d_scale_x, 4) ||
        !aligned(d_scale_w, 4) || !aligned(d_amax_y, 4))
        return LLMQ_ERR_ALIGN;
    const WsLayout l = ws_layout(M, N, K);
    uint8_t* base = static_cast<uint8_t*>(ws);
    hipStream_t s = static_cast<hipStream_t>(stream);
    // the first quantize kernel of the call also clears the absmax accumulator of the GEMM
    unsigned* zero = reinterpret_cast<unsigned*>(d_amax_y);
    const bool zeroed = zero && (qx || qw);
    unsigned* part = reinterpret_cast<unsigned*>(base + l.part);
    constexpr size_t kPartWords = 256 * ((llmq::kAmaxMaxPartials * sizeof(unsigned) + 255) / 256) / sizeof(unsigned);
    const bool nt = (flags & LLMQ_NO_TRANSPOSE) != 0;
    if (qx && (st = quantize_operand(X, M, K, d_scale_x, LLMQ_E4M3, base + l.xq, nt ? nullptr : base + l.xqt, (flags & LLMQ_JIT_X) != 0, part, zero, s, slab_copy(flags, M, K)))) return st;
    if (qw && (st = quantize_operand(W, N, K, d_scale_w, LLMQ_E4M3, base + l.wq, nt ? nullptr : base + l.wqt, (flags & LLMQ_JIT_W) != 0, part + kPartWords, qx ? nullptr : zero, s, slab_copy(flags, N, K)))) return st;
    return llmq::launch_gemm_tn(base + l.xq, LLMQ_E4M3, base + l.wq, LLMQ_E4M3, M, N, K, d_scale_x, d_scale_w,
                                Y, 0, d_amax_y, zeroed, s, num_cus(), pieces_of(l, ws, flags));
}

int llmq_fp8_linear_dgrad(const void* dY, const void* W, int64_t M, int64_t N, int64_t K,
                          float* d_scale_dy, float* d_scale_w, int fmt_dy, void* dX,
                          float* d_amax_dx, void* ws, size_t ws_bytes, int flags, void* stream) {
    int st = check_linear(M, N, K, ws, ws_bytes, flags);
    if (st != LLMQ_OK) return st;
    if (flags & (LLMQ_REUSE_X | LLMQ_JIT_X)) return LLMQ_ERR_FLAGS;
    if (!fmt_ok(fmt_dy)) return LLMQ_ERR_FORMAT;
    const bool qd = !(flags & LLMQ_REUSE_DY), qw = !(flags & LLMQ_REUSE_W);
    if ((qd && !dY) || (qw && !W) || !d_scale_dy || !d_scale_w || !dX) return LLMQ_ERR_NULL;
    if ((qd && !aligned(dY, 16)) || (qw && !aligned(W, 16)) || !aligned(dX, 16) || !aligned(d_scale_dy, 4) ||
        !aligned(d_scale_w, 4) || !aligned(d_amax_dx, 4))
        return LLMQ_ERR_ALIGN;
    const WsLayout l = ws_layout(M, N, K);
    uint8_t* base = static_cast<uint8_t*>(ws);
    hipStream_t s = static_cast<hipStream_t>(stream);
    unsigned* zero = reinterpret_cast<unsigned*>(d_amax_dx);
    const bool zeroed = zero && (qd || qw);
    unsigned* part = reinterpret_cast<unsigned*>(base + l.part);
    constexpr size_t kPartWords = 256 * ((llmq::kAmaxMaxPartials * sizeof(unsigned) + 255) / 256) / sizeof(unsigned);
    const bool nt = (flags & LLMQ_NO_TRANSPOSE) != 0;
    if (qd && (st = quantize_operand(dY, M, N, d_scale_dy, fmt_dy, base + l.dyq, nt ? nullptr : base + l.dyqt, (flags & LLMQ_JIT_DY) != 0, part + 2 * kPartWords, zero, s, slab_copy(flags, M, N)))) return st;
    if (qw && (st = quantize_operand(W, N, K, d_scale_w, LLMQ_E4M3, base + l.wq, nt ? nullptr : base + l.wqt, (flags & LLMQ_JIT_W) != 0, part + kPartWords, qd ? nullptr : zero, s, slab_copy(flags, N, K)))) return st;
    // dX[m,k] = sum_n dYq[m,n] * Wq_t[k,n] = sum_n dYq[m,n] * Wq[n,k]
    const int w_layout = nt ? llmq::kLayoutTMajor : slab_copy(flags, N, K) ? llmq::kLayoutSlabs : llmq::kLayoutRows;
    return llmq::launch_gemm_fp8(base + l.dyq, fmt_dy, llmq::kLayoutRows, nt ? base + l.wq : base + l.wqt, LLMQ_E4M3, w_layout, M, K, N,
                                 d_scale_dy, d_scale_w, dX, 0, d_amax_dx, zeroed, s, num_cus(), pieces_of(l, ws, flags));
}

int llmq_fp8_linear_wgrad(const void* dY, const void* X, int64_t M, int64_t N, int64_t K,
                          float* d_scale_dy, float* d_scale_x, int fmt_dy, void* dW,
                          int accumulate, void* ws, size_t ws_bytes, int flags, void* stream) {
    int st = check_linear(M, N, K, ws, ws_bytes, flags);
    if (st != LLMQ_OK) return st;
    if (flags & (LLMQ_REUSE_W | LLMQ_JIT_W)) return LLMQ_ERR_FLAGS;
    if (!fmt_ok(fmt_dy)) return LLMQ_ERR_FORMAT;
    const bool qd = !(flags & LLMQ_REUSE_DY), qx = !(flags & LLMQ_REUSE_X);
    if ((qd && !dY) || (qx && !X) || !d_scale_dy || !d_scale_x || !dW) return LLMQ_ERR_NULL;
    if ((qd && !aligned(dY, 16)) || (qx && !aligned(X, 16)) || !aligned(dW, 16) || !aligned(d_scale_dy, 4) ||
        !aligned(d_scale_x, 4))
        return LLMQ_ERR_ALIGN;
    const WsLayout l = ws_layout(M, N, K);
    uint8_t* base = static_cast<uint8_t*>(ws);
    hipStream_t s = static_cast<hipStream_t>(stream);
    unsigned* part = reinterpret_cast<unsigned*>(base + l.part);
    constexpr size_t kPartWords = 256 * ((llmq::kAmaxMaxPartials * sizeof(unsigned) + 255) / 256) / sizeof(unsigned);
    const bool nt = (flags & LLMQ_NO_TRANSPOSE) != 0;
    if (qd && (st = quantize_operand(dY, M, N, d_scale_dy, fmt_dy, base + l.dyq, nt ? nullptr : base + l.dyqt, (flags & LLMQ_JIT_DY) != 0, part + 2 * kPartWords, nullptr, s, slab_copy(flags, M, N)))) return st;
    if (qx && (st = quantize_operand(X, M, K, d_scale_x, LLMQ_E4M3, base + l.xq, nt ? nullptr : base + l.xqt, (flags & LLMQ_JIT_X) != 0, part, nullptr, s, slab_copy(flags, M, K)))) return st;
    // dW[n,k] = sum_m dYq_t[n,m] * Xq_t[k,m] = sum_m dYq[m,n] * Xq[m,k]
    const int dy_layout = nt ? llmq::kLayoutTMajor : slab_copy(flags, M, N) ? llmq::kLayoutSlabs : llmq::kLayoutRows;
    const int x_layout = nt ? llmq::kLayoutTMajor : slab_copy(flags, M, K) ? llmq::kLayoutSlabs : llmq::kLayoutRows;
    return llmq::launch_gemm_fp8(nt ? base + l.dyq : base + l.dyqt, fmt_dy, dy_layout, nt ? base + l.xq : base + l.xqt, LLMQ_E4M3, x_layout,
                                 N, K, M, d_scale_dy, d_scale_x, dW, accumulate, nullptr, false, s, num_cus(), pieces_of(l, ws, flags));
}

int llmq_scale_from_amax(const float* d_amax, int fmt, float* d_scale, void* stream) {
    if (!d_amax || !d_scale) return LLMQ_ERR_NULL;
    if (!fmt_ok(fmt)) return LLMQ_ERR_FORMAT;
    if (!aligned(d_amax, 4) || !aligned(d_scale, 4)) return LLMQ_ERR_ALIGN;
    return llmq::launch_scale_from_amax(d_amax, fmt, d_scale, static_cast<hipStream_t>(stream));
}

size_t llmq_swiglu_workspace_bytes(int64_t M, int64_t I) {
    if (check_swiglu_shape(M, I) != LLMQ_OK) return 0;
    return (size_t)llmq::swiglu_blocks(M, I) * sizeof(unsigned);
}

int llmq_swiglu_fwd(const void* gu_bf16, int64_t M, int64_t I, void* h_bf16, int fmt, float* d_amax_h,
                    float* d_scale_h, void* ws, size_t ws_bytes, void* stream) {
    if (!gu_bf16 || !h_bf16 || !d_amax_h || !ws) return LLMQ_ERR_NULL;
    int st = check_swiglu_shape(M, I);
    if (st != LLMQ_OK) return st;
    if (!fmt_ok(fmt)) return LLMQ_ERR_FORMAT;
    if (!aligned(gu_bf16, 16) || !aligned(h_bf16, 16) || !aligned(d_amax_h, 4) || !aligned(d_scale_h, 4) ||
        !aligned(ws, 16))
        return LLMQ_ERR_ALIGN;
    if (ws_bytes < llmq_swiglu_workspace_bytes(M, I)) return LLMQ_ERR_WORKSPACE;
    return llmq::launch_swiglu_fwd(gu_bf16, M, I, h_bf16, static_cast<unsigned*>(ws), fmt, d_amax_h, d_scale_h,
                                   nullptr, 0, nullptr, nullptr, static_cast<hipStream_t>(stream));
}

int llmq_swiglu_fwd_fp8(const void* gu_bf16, int64_t M, int64_t I, const float* d_scale_h, int fmt, uint8_t* q,
                        uint8_t* q_t, void* h_bf16, void* stream) {
    if (!gu_bf16 || !d_scale_h || !q) return LLMQ_ERR_NULL;
    int st = check_swiglu_shape(M, I);
    if (st != LLMQ_OK) return st;
    if (!fmt_ok(fmt)) return LLMQ_ERR_FORMAT;
    if (!aligned(gu_bf16, 16) || !aligned(h_bf16, 16) || !aligned(q, 16) || !aligned(q_t, 16) || !aligned(d_scale_h, 4))
        return LLMQ_ERR_ALIGN;
    return llmq::launch_swiglu_fwd(gu_bf16, M, I, h_bf16, nullptr, fmt, nullptr, nullptr, d_scale_h, fmt, q, q_t,
                                   static_cast<hipStream_t>(stream));
}

int llmq_swiglu_fwd_fp8_slabs(const void* gu_bf16, int64_t M, int64_t I, const float* d_scale_h, int fmt, uint8_t* q,
                              uint8_t* q_t, void* h_bf16, void* stream) {
    if (!gu_bf16 || !d_scale_h || !q || !q_t) return LLMQ_ERR_NULL;
    int st = check_swiglu_shape(M, I);
    if (st != LLMQ_OK) return st;
    if (!llmq::tile_shape_ok(M, I) || M * I >= kMaxSlabElems) return LLMQ_ERR_SHAPE;
    if (!fmt_ok(fmt)) return LLMQ_ERR_FORMAT;
    if (!aligned(gu_bf16, 16) || !aligned(h_bf16, 16) || !aligned(q, 16) || !aligned(q_t, 16) || !aligned(d_scale_h, 4))
        return LLMQ_ERR_ALIGN;
    return llmq::launch_swiglu_fwd(gu_bf16, M, I, h_bf16, nullptr, fmt, nullptr, nullptr, d_scale_h, fmt, q, q_t,
                                   static_cast<hipStream_t>(stream), true);
}

int llmq_swiglu_bwd(const void* dh_bf16, const void* gu_bf16, int64_t M, int64_t I, void* dgu_bf16, int fmt,
                    float* d_amax_dgu, float* d_scale_dgu, void* ws, size_t ws_bytes, void* stream) {
    if (!dh_bf16 || !gu_bf16 || !dgu_bf16 || !d_amax_dgu || !ws) return LLMQ_ERR_NULL;
    int st = check_swiglu_shape(M, I);
    if (st != LLMQ_OK) return st;
    if (!fmt_ok(fmt)) return LLMQ_ERR_FORMAT;
    if (!aligned(dh_bf16, 16) || !aligned(gu_bf16, 16) || !aligned(dgu_bf16, 16) || !aligned(d_amax_dgu, 4) ||
        !aligned(d_scale_dgu, 4) || !aligned(ws, 16))
        return LLMQ_ERR_ALIGN;
    if (ws_bytes < llmq_swiglu_workspace_bytes(M, I)) return LLMQ_ERR_WORKSPACE;
    return llmq::launch_swiglu_bwd(dh_bf16, gu_bf16, M, I, dgu_bf16, static_cast<unsigned*>(ws), fmt, d_amax_dgu,
                                   d_scale_dgu, static_cast<hipStream_t>(stream));
}

size_t llmq_rmsnorm_workspace_bytes(int64_t M) {
    if (!dim_ok(M)) return 0;
    return (size_t)llmq::rmsnorm_blocks(M) * sizeof(unsigned);
}

int llmq_rmsnorm_fwd(const void* res_bf16, const void* x_bf16, const void* w_bf16, int64_t M, int64_t C, float eps,
                     void* res_out_bf16, void* y_bf16, float* rstd, int fmt, float* d_amax_y, float* d_scale_y,
                     void* ws, size_t ws_bytes, void* stream) {
    if (!res_bf16 || !w_bf16 || !y_bf16 || !rstd || !d_amax_y || !ws || (x_bf16 && !res_out_bf16)) return LLMQ_ERR_NULL;
    if (!dim_ok(M) || !dim_ok(C) || C >= ((int64_t)1 << 24) || M * C >= kMaxElems) return LLMQ_ERR_SHAPE;
    if (!(eps >= 0.0f) || eps > 3.402823466e+38f) return LLMQ_ERR_SHAPE;
    if (!fmt_ok(fmt)) return LLMQ_ERR_FORMAT;
    if (!aligned(res_bf16, 16) || !aligned(x_bf16, 16) || !aligned(w_bf16, 16) || !aligned(y_bf16, 16) ||
        (x_bf16 && !aligned(res_out_bf16, 16)) || !aligned(rstd, 4) || !aligned(d_amax_y, 4) ||
        !aligned(d_scale_y, 4) || !aligned(ws, 16))
        return LLMQ_ERR_ALIGN;
    if (ws_bytes < llmq_rmsnorm_workspace_bytes(M)) return LLMQ_ERR_WORKSPACE;
    return llmq::launch_rmsnorm_fwd(res_bf16, x_bf16, w_bf16, M, C, eps, x_bf16 ? res_out_bf16 : nullptr, y_bf16, rstd,
                                    static_cast<unsigned*>(ws), fmt, d_amax_y, d_scale_y,
                                    static_cast<hipStream_t>(stream));
}

int llmq_rmsnorm_apply_fp8(const void* res_bf16, const void* w_bf16, const float* rstd, int64_t M, int64_t C,
                           const float* d_scale_y, int fmt, uint8_t* q, uint8_t* q_t, void* y_bf16, void* stream) {
    if (!res_bf16 || !w_bf16 || !rstd || !d_scale_y || !q) return LLMQ_ERR_NULL;
    if (!dim_ok(M) || !dim_ok(C) || C >= ((int64_t)1 << 24) || M * C >= kMaxElems) return LLMQ_ERR_SHAPE;
    if (!fmt_ok(fmt)) return LLMQ_ERR_FORMAT;
    if (!aligned(res_bf16, 16) || !aligned(w_bf16, 16) || !aligned(rstd, 16) || !aligned(d_scale_y, 4) ||
        !aligned(q, 16) || !aligned(q_t, 16) || !aligned(y_bf16, 16))
        return LLMQ_ERR_ALIGN;
    return llmq::launch_rmsnorm_apply_fp8(res_bf16, w_bf16, rstd, M, C, d_scale_y, fmt, q, q_t, y_bf16,
                                          static_cast<hipStream_t>(stream));
}

int llmq_rmsnorm_apply_fp8_slabs(const void* res_bf16, const void* w_bf16, const float* rstd, int64_t M, int64_t C,
                                 const float* d_scale_y, int fmt, uint8_t* q, uint8_t* q_t, void* y_bf16,
                                 void* stream) {
    if (!res_bf16 || !w_bf16 || !rstd || !d_scale_y || !q || !q_t) return LLMQ_ERR_NULL;
    if (!dim_ok(M) || !dim_ok(C) || C >= ((int64_t)1 << 24) || M * C >= kMaxElems) return LLMQ_ERR_SHAPE;
    if (!llmq::tile_shape_ok(M, C) || M * C >= kMaxSlabElems) return LLMQ_ERR_SHAPE;
    if (!fmt_ok(fmt)) return LLMQ_ERR_FORMAT;
    if (!aligned(res_bf16, 16) || !aligned(w_bf16, 16) || !aligned(rstd, 16) || !aligned(d_scale_y, 4) ||
        !aligned(q, 16) || !aligned(q_t, 16) || !aligned(y_bf16, 16))
        return LLMQ_ERR_ALIGN;
    return llmq::launch_rmsnorm_apply_fp8(res_bf16, w_bf16, rstd, M, C, d_scale_y, fmt, q, q_t, y_bf16,
                                          static_cast<hipStream_t>(stream), true);
}

int llmq_calibrate_mfma(int fmtA, int fmtB, int random_bits, int iters, float* d_sink, double* flops,
                        void* stream) {
    if (!d_sink) return LLMQ_ERR_NULL;
    if (!fmt_ok(fmtA) || !fmt_ok(fmtB)) return LLMQ_ERR_FORMAT;
    if (iters < 1 || iters > (1 << 24)) return LLMQ_ERR_SHAPE;
    if (!aligned(d_sink, 4)) return LLMQ_ERR_ALIGN;
    // workgroups x waves x iterations x 64 MFMAs x 2 * 16 * 16 * 128 FLOP
    if (flops) *flops = (double)num_cus() * 4.0 * iters * 64.0 * 2.0 * 16 * 16 * 128;
    return llmq::launch_calibrate_mfma(fmtA, fmtB, random_bits != 0, iters, d_sink, static_cast<hipStream_t>(stream),
                                       num_cus());
}

size_t llmq_calibrate_gemm_phases_bytes(int64_t R, int64_t C) {
    if (!dim_ok(R) || !dim_ok(C) || R % 256 != 0 || C % 256 != 0) return 0;
    return (size_t)llmq::gemm_phase_stamp_blocks(R, C) * 16 * sizeof(long long);
}

int llmq_calibrate_gemm_phases(const uint8_t* A, const uint8_t* B, int64_t R, int64_t C, int64_t T, const float* d_scaleA,
                               const float* d_scaleB, void* c_bf16, float* d_amax_c, void* d_stamps, size_t stamps_bytes,
                               int ieee_maximum, void* stream) {
    if (!A || !B || !d_scaleA || !d_scaleB || !c_bf16 || !d_amax_c || !d_stamps) return LLMQ_ERR_NULL;
    if (!dim_ok(R) || !dim_ok(C) || !dim_ok(T) || R % 256 != 0 || C % 256 != 0 || T % 128 != 0 || T >= ((int64_t)1 << 23) ||
        (R / 256) * (C / 256) >= ((int64_t)1 << 30))
        return LLMQ_ERR_SHAPE;
    if (!aligned(A, 16) || !aligned(B, 16) || !aligned(c_bf16, 16) || !aligned(d_scaleA, 4) || !aligned(d_scaleB, 4) ||
        !aligned(d_amax_c, 4) || !aligned(d_stamps, 8))
        return LLMQ_ERR_ALIGN;
    if (stamps_bytes < llmq_calibrate_gemm_phases_bytes(R, C)) return LLMQ_ERR_WORKSPACE;
    return llmq::launch_gemm_phase_stamps(A, B, R, C, T, d_scaleA, d_scaleB, c_bf16, d_amax_c,
                                          static_cast<long long*>(d_stamps), ieee_maximum, static_cast<hipStream_t>(stream),
                                          num_cus());
}

int llmq_calibrate_copy(const void* src, void* dst, size_t bytes, void* stream) {
    if (!src || !dst) return LLMQ_ERR_NULL;
    if (bytes < 16 || bytes % 16 != 0 || bytes >= ((size_t)1 << 40)) return LLMQ_ERR_SHAPE;
    if (!aligned(src, 16) || !aligned(dst, 16)) return LLMQ_ERR_ALIGN;
    return llmq::launch_calibrate_copy(src, dst, bytes, static_cast<hipStream_t>(stream));
}

}  // extern "C"
