// Host sanitizer run of the C ABI's argument checks and launch sequencing (csrc/api.hip), without a GPU: the
// kernel launchers are replaced by stubs that only count calls, api.hip is compiled for the host with
// -fsanitize=address,undefined (tests/test_host_sanitizers.py), and every entry point is called with bad and
// with good arguments.  Pointers are made-up addresses: the host code must never dereference a device pointer.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/llmq.h"
#include "../../paper_2512_15306_amd/csrc/llmq_kernels.h"

static int g_launches = 0;
static size_t g_scratch_seen = 0;
namespace llmq {
int launch_amax(const void*, size_t, int, float*, float*, void*, hipStream_t, int) { ++g_launches; return 0; }
int launch_amax_static(const void*, size_t, int, float*, float*, hipStream_t, int) { ++g_launches; return 0; }
int launch_amax_final(const unsigned*, int, int, float*, float*, hipStream_t) { ++g_launches; return 0; }
int launch_gemm_bf16_tn(const void*, const void*, int64_t, int64_t, int64_t, void*, int, hipStream_t, int) { ++g_launches; return 0; }
int launch_scale_from_amax(const float*, int, float*, hipStream_t) { ++g_launches; return 0; }
int launch_quantize(const void*, int64_t, int64_t, const float*, int, uint8_t*, uint8_t*, unsigned*, hipStream_t, bool) { ++g_launches; return 0; }
bool quantize_can_write_slabs(int64_t rows, int64_t cols) { return rows % 128 == 0 && cols % 256 == 0; }
int launch_quantize_from(const void*, int64_t, int64_t, const ScaleSource&, int, uint8_t*, uint8_t*, unsigned*, hipStream_t, bool) { ++g_launches; return 0; }
int launch_amax_partial(const void*, size_t, unsigned*, int* n_partial, hipStream_t, int) { ++g_launches; *n_partial = 7; return 0; }
size_t gemm_scratch_bytes(int64_t R, int64_t C, int64_t, int) { return (size_t)((R / 256) * (C / 256) % 7) * 262144; }
int launch_gemm_tn(const uint8_t*, int, const uint8_t*, int, int64_t, int64_t, int64_t, const float*, const float*, void*, int, float*, bool, hipStream_t, int, GemmScratch sc, bool, bool) { ++g_launches; g_scratch_seen = sc.ptr ? sc.bytes : 0; return 0; }
int launch_gemm_fp8(const uint8_t*, int, int, const uint8_t*, int, int, int64_t, int64_t, int64_t, const float*, const float*, void*, int, float*, bool, hipStream_t, int, GemmScratch sc) { ++g_launches; g_scratch_seen = sc.ptr ? sc.bytes : 0; return 0; }
int gemm_phase_stamp_blocks(int64_t R, int64_t C) { return (int)((R / 256) * (C / 256)); }
int launch_gemm_phase_stamps(const uint8_t*, const uint8_t*, int64_t, int64_t, int64_t, const float*, const float*, void*, float*, long long*, int, hipStream_t, int) { ++g_launches; return 0; }
int64_t swiglu_blocks(int64_t M, int64_t I) { return (M + 31) / 32 * ((I + 255) / 256); }
int launch_swiglu_fwd(const void*, int64_t, int64_t, void*, unsigned*, int, float*, float*, const float*, int, uint8_t*, uint8_t*, hipStream_t, bool) { ++g_launches; return 0; }
int launch_swiglu_bwd(const void*, const void*, int64_t, int64_t, void*, unsigned*, int, float*, float*, hipStream_t) { ++g_launches; return 0; }
int64_t rmsnorm_blocks(int64_t M) { return (M + 3) / 4; }
int launch_rmsnorm_fwd(const void*, const void*, const void*, int64_t, int64_t, float, void*, void*, float*, unsigned*, int, float*, float*, hipStream_t) { ++g_launches; return 0; }
int launch_rmsnorm_apply_fp8(const void*, const void*, const float*, int64_t, int64_t, const float*, int, uint8_t*, uint8_t*, void*, hipStream_t, bool) { ++g_launches; return 0; }
int launch_calibrate_mfma(int, int, int, int, float*, hipStream_t, int) { ++g_launches; return 0; }
int launch_calibrate_copy(const void*, void*, size_t, hipStream_t) { ++g_launches; return 0; }
}  // namespace llmq

static int g_fail = 0;
#define EXPECT(call, status, launches)                                                                   \
    do {                                                                                                 \
        const int before = g_launches;                                                                   \
        const int st = (call);                                                                           \
        if (st != (status) || g_launches - before != (launches)) {                                       \
            std::printf("line %d: status %d (want %d), launches %d (want %d)\n", __LINE__, st, (status), \
                        g_launches - before, (launches));                                                \
            ++g_fail;                                                                                    \
        }                                                                                                \
    } while (0)

int main() {
    void* P = reinterpret_cast<void*>(0x7f0000001000ull);       // "device" pointers, 256-byte aligned
    uint8_t* B8 = static_cast<uint8_t*>(P);
    float* F = reinterpret_cast<float*>(0x7f0000002000ull);
    void* odd = reinterpret_cast<void*>(0x7f0000001008ull);
    const int64_t M = 256, N = 1024, K = 512;
    const size_t ws = llmq_fp8_linear_workspace_bytes(M, N, K), ws_nt = llmq_fp8_linear_workspace_bytes_no_transpose(M, N, K);
    size_t offs[6];
    EXPECT(llmq_fp8_linear_workspace_offsets(M, N, K, offs), LLMQ_OK, 0);
    EXPECT(llmq_fp8_linear_workspace_offsets(M, N, K, nullptr), LLMQ_ERR_NULL, 0);
    for (int st = -9; st <= 1; ++st) if (!llmq_status_string(st)) ++g_fail;
    // absmax, with workspace and with the static scratch
    EXPECT(llmq_amax(P, 1000, 0, F, F, P, llmq_amax_workspace_bytes(), nullptr), LLMQ_OK, 1);
    EXPECT(llmq_amax(P, 1000, 0, F, F, P, llmq_amax_workspace_bytes() - 1, nullptr), LLMQ_ERR_WORKSPACE, 0);
    EXPECT(llmq_amax(P, 0, 0, F, F, P, 4096, nullptr), LLMQ_ERR_SHAPE, 0);
    EXPECT(llmq_amax(odd, 8, 0, F, F, P, 4096, nullptr), LLMQ_ERR_ALIGN, 0);
    EXPECT(llmq_amax_static(P, 1000, 1, F, nullptr, nullptr), LLMQ_OK, 1);
    EXPECT(llmq_amax_static(P, (size_t)1 << 40, 1, F, nullptr, nullptr), LLMQ_ERR_SHAPE, 0);
    EXPECT(llmq_amax_static(P, 8, 2, F, nullptr, nullptr), LLMQ_ERR_FORMAT, 0);
    // quantize and the contractions
    EXPECT(llmq_quantize_fp8(P, 16, 8, F, 0, B8, B8, nullptr), LLMQ_OK, 1);
    EXPECT(llmq_quantize_fp8(P, 16, 8, F, 0, B8, nullptr, nullptr), LLMQ_OK, 1);
    EXPECT(llmq_quantize_fp8(P, -1, 8, F, 0, B8, B8, nullptr), LLMQ_ERR_SHAPE, 0);
    EXPECT(llmq_quantize_fp8(P, 16, 8, nullptr, 0, B8, B8, nullptr), LLMQ_ERR_NULL, 0);
    EXPECT(llmq_fp8_gemm_tn(B8, 0, B8, 1, 256, 256, 128, F, F, P, 0, F, nullptr), LLMQ_OK, 1);
    EXPECT(llmq_fp8_gemm_tn(B8, 0, B8, 3, 256, 256, 128, F, F, P, 0, F, nullptr), LLMQ_ERR_FORMAT, 0);
    EXPECT(llmq_fp8_gemm(B8, 1, 1, B8, 0, 1, 256, 256, 128, F, F, P, 1, nullptr, nullptr), LLMQ_OK, 1);
    EXPECT(llmq_fp8_gemm(B8, 1, 1, B8, 0, 1, 256, 0, 128, F, F, P, 1, nullptr, nullptr), LLMQ_ERR_SHAPE, 0);
    EXPECT(llmq_fp8_gemm_with_scratch(B8, 1, 0, B8, 0, 1, 256, 256, 128, F, F, P, 0, nullptr, P, 1 << 20, nullptr), LLMQ_OK, 1);
    if (g_scratch_seen != (1u << 20)) ++g_fail;
    EXPECT(llmq_fp8_gemm_with_scratch(B8, 1, 0, B8, 0, 1, 256, 256, 128, F, F, P, 0, nullptr, nullptr, 1 << 20, nullptr), LLMQ_OK, 1);
    if (g_scratch_seen != 0) ++g_fail;
    EXPECT(llmq_fp8_gemm_with_scratch(B8, 1, 0, B8, 0, 1, 256, 256, 128, F, F, P, 0, nullptr, odd, 1 << 20, nullptr), LLMQ_ERR_ALIGN, 0);
    if (llmq_fp8_gemm_scratch_bytes(0, 256, 128) != 0) ++g_fail;
    EXPECT(llmq_bf16_gemm_tn(P, P, 256, 256, 64, P, 0, nullptr), LLMQ_OK, 1);
    EXPECT(llmq_bf16_gemm_tn(P, nullptr, 256, 256, 64, P, 0, nullptr), LLMQ_ERR_NULL, 0);
    // the three linear calls: explicit scales (quantize x2 + GEMM), just-in-time scaling (first absmax stage +
    // quantize per operand, then the GEMM), reuse (GEMM only)
    EXPECT(llmq_fp8_linear_fwd(P, P, M, N, K, F, F, P, F, P, ws, 0, nullptr), LLMQ_OK, 3);
    EXPECT(llmq_fp8_linear_fwd(P, P, M, N, K, F, F, P, F, P, ws, LLMQ_JIT_X | LLMQ_JIT_W, nullptr), LLMQ_OK, 5);
    EXPECT(llmq_fp8_linear_fwd(nullptr, nullptr, M, N, K, F, F, P, nullptr, P, ws, LLMQ_REUSE_X | LLMQ_REUSE_W, nullptr), LLMQ_OK, 1);
    EXPECT(llmq_fp8_linear_fwd(P, P, M, N, K, F, F, P, F, P, ws_nt, LLMQ_NO_TRANSPOSE, nullptr), LLMQ_OK, 3);
    EXPECT(llmq_fp8_linear_fwd(P, P, M, N, K, F, F, P, F, P, ws_nt, 0, nullptr), LLMQ_ERR_WORKSPACE, 0);
    EXPECT(llmq_fp8_linear_fwd(P, P, M, N, K, F, F, P, F, P, ws, LLMQ_JIT_X | LLMQ_REUSE_X, nullptr), LLMQ_ERR_FLAGS, 0);
    EXPECT(llmq_fp8_linear_fwd(P, P, M, N, K, F, F, P, F, P, ws, 1 << 20, nullptr), LLMQ_ERR_FLAGS, 0);
    EXPECT(llmq_fp8_linear_fwd(P, P, M, N, K, F, F, P, F, odd, ws, 0, nullptr), LLMQ_ERR_ALIGN, 0);
    EXPECT(llmq_fp8_linear_fwd(nullptr, P, M, N, K, F, F, P, F, P, ws, 0, nullptr), LLMQ_ERR_NULL, 0);
    EXPECT(llmq_fp8_linear_dgrad(P, nullptr, M, N, K, F, F, 1, P, F, P, ws, LLMQ_JIT_DY | LLMQ_REUSE_W, nullptr), LLMQ_OK, 3);
    EXPECT(llmq_fp8_linear_dgrad(P, nullptr, M, N, K, F, F, 1, P, nullptr, P, ws, LLMQ_REUSE_DY | LLMQ_REUSE_W, nullptr), LLMQ_OK, 1);
    EXPECT(llmq_fp8_linear_dgrad(P, P, M, N, K, F, F, 2, P, F, P, ws, 0, nullptr), LLMQ_ERR_FORMAT, 0);
    EXPECT(llmq_fp8_linear_dgrad(P, P, M, N, K, F, F, 1, P, F, P, ws, LLMQ_JIT_X, nullptr), LLMQ_ERR_FLAGS, 0);
    EXPECT(llmq_fp8_linear_wgrad(nullptr, nullptr, M, N, K, F, F, 1, P, 1, P, ws, LLMQ_REUSE_X | LLMQ_REUSE_DY, nullptr), LLMQ_OK, 1);
    EXPECT(llmq_fp8_linear_wgrad(P, P, M, N, K, F, F, 0, P, 0, P, ws, LLMQ_JIT_X | LLMQ_JIT_DY, nullptr), LLMQ_OK, 5);
    EXPECT(llmq_fp8_linear_wgrad(P, P, M, (int64_t)1 << 31, K, F, F, 0, P, 0, P, ws, 0, nullptr), LLMQ_ERR_SHAPE, 0);
    // the kernels around the linears
    EXPECT(llmq_scale_from_amax(F, 0, F, nullptr), LLMQ_OK, 1);
    EXPECT(llmq_scale_from_amax(F, 5, F, nullptr), LLMQ_ERR_FORMAT, 0);
    EXPECT(llmq_swiglu_fwd(P, 64, 256, P, 0, F, F, P, llmq_swiglu_workspace_bytes(64, 256), nullptr), LLMQ_OK, 1);
    EXPECT(llmq_swiglu_fwd(P, 64, 256, P, 0, F, F, P, 0, nullptr), LLMQ_ERR_WORKSPACE, 0);
    EXPECT(llmq_swiglu_fwd_fp8(P, 64, 256, F, 0, B8, B8, nullptr, nullptr), LLMQ_OK, 1);
    EXPECT(llmq_swiglu_fwd_fp8_slabs(P, 128, 256, F, 0, B8, B8, nullptr, nullptr), LLMQ_OK, 1);
    EXPECT(llmq_swiglu_fwd_fp8_slabs(P, 64, 256, F, 0, B8, B8, nullptr, nullptr), LLMQ_ERR_SHAPE, 0);     // whole 128 x 256 tiles only
    EXPECT(llmq_swiglu_fwd_fp8_slabs(P, 128, 256, F, 0, B8, nullptr, nullptr, nullptr), LLMQ_ERR_NULL, 0);
    EXPECT(llmq_swiglu_bwd(P, P, 64, (int64_t)1 << 24, P, 1, F, F, P, 1 << 20, nullptr), LLMQ_ERR_SHAPE, 0);
    EXPECT(llmq_swiglu_bwd(P, P, 64, 256, P, 1, F, F, P, llmq_swiglu_workspace_bytes(64, 256), nullptr), LLMQ_OK, 1);
    EXPECT(llmq_rmsnorm_fwd(P, P, P, 32, 384, 1e-6f, P, P, F, 0, F, F, P, llmq_rmsnorm_workspace_bytes(32), nullptr), LLMQ_OK, 1);
    EXPECT(llmq_rmsnorm_fwd(P, P, P, 32, 384, -1.0f, P, P, F, 0, F, F, P, llmq_rmsnorm_workspace_bytes(32), nullptr), LLMQ_ERR_SHAPE, 0);
    EXPECT(llmq_rmsnorm_fwd(P, P, P, 32, 384, 1e-6f, nullptr, P, F, 0, F, F, P, llmq_rmsnorm_workspace_bytes(32), nullptr), LLMQ_ERR_NULL, 0);
    EXPECT(llmq_rmsnorm_apply_fp8(P, P, F, 32, 384, F, 0, B8, B8, nullptr, nullptr), LLMQ_OK, 1);
    EXPECT(llmq_rmsnorm_apply_fp8(P, P, F + 1, 32, 384, F, 0, B8, B8, nullptr, nullptr), LLMQ_ERR_ALIGN, 0);   // rstd: 16-byte aligned
    EXPECT(llmq_rmsnorm_apply_fp8_slabs(P, P, F, 128, 512, F, 0, B8, B8, nullptr, nullptr), LLMQ_OK, 1);
    EXPECT(llmq_rmsnorm_apply_fp8_slabs(P, P, F, 128, 384, F, 0, B8, B8, nullptr, nullptr), LLMQ_ERR_SHAPE, 0);
    EXPECT(llmq_rmsnorm_apply_fp8_slabs(P, P, F, 128, 512, F, 0, B8, nullptr, nullptr, nullptr), LLMQ_ERR_NULL, 0);
    double flops = 0;
    EXPECT(llmq_calibrate_mfma(0, 1, 1, 100, F, &flops, nullptr), LLMQ_OK, 1);
    EXPECT(llmq_calibrate_mfma(0, 1, 1, 0, F, &flops, nullptr), LLMQ_ERR_SHAPE, 0);
    EXPECT(llmq_calibrate_gemm_phases(B8, B8, 512, 256, 128, F, F, P, F, P, llmq_calibrate_gemm_phases_bytes(512, 256), 1, nullptr), LLMQ_OK, 1);
    EXPECT(llmq_calibrate_gemm_phases(B8, B8, 512, 256, 128, F, F, P, F, P, 8, 1, nullptr), LLMQ_ERR_WORKSPACE, 0);
    EXPECT(llmq_calibrate_gemm_phases(B8, B8, 500, 256, 128, F, F, P, F, P, 1 << 20, 1, nullptr), LLMQ_ERR_SHAPE, 0);
    EXPECT(llmq_calibrate_copy(P, P, 4096, nullptr), LLMQ_OK, 1);
    EXPECT(llmq_calibrate_copy(P, P, 4097, nullptr), LLMQ_ERR_SHAPE, 0);
    if (llmq_version() < 100 || ws <= ws_nt || !(flops > 0)) ++g_fail;
    if (g_fail) { std::printf("%d checks failed\n", g_fail); return 1; }
    std::puts("abi sanitizer driver ok");
    return 0;
}
