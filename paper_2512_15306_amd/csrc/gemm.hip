// FP8 contraction on the gfx950 matrix cores (paper Section 3: the transformer-block matmuls of
// forward and backward run in FP8, results stay in BF16; the FP8 GEMM is "TN", i.e. both operands
// have the contraction index contiguous).
//
//   C[r,c] = bf16( (sum_t A[r,t] * B[c,t]) / (sA * sB) ),   A [R,T] fp8, B [Cn,T] fp8.
//
// Tuned kernel (R, Cn multiples of 256; T a multiple of 128)
//   - one workgroup of 4 wavefronts per 256x256 output tile, each wavefront owns 128x128 of it
//     as 4x4 blocks of v_mfma_f32_32x32x64_f8f6f4 (fp32 accumulators, 256 registers per lane);
//   - K advances 128 bytes per step; the A and B slabs (256 rows x 128 B each) go from global memory
//     straight into LDS with buffer_load ... lds (16 bytes per lane, no VGPR staging), double
//     buffered: 2 x 64 KB of the 160 KB LDS;
//   - LDS rows are 128 B; the 16-byte chunk index is XOR-ed with (row & 7), applied on the global
//     side of the load, so that the ds_read_b128 fragment reads of 8 consecutive rows hit all banks;
//   - the order of the contraction index inside one MFMA does not matter as long as A and B use
//     the same order, so every lane simply reads 32 contiguous bytes of its row;
//   - the MFMA takes the B rows as its first operand, which leaves every lane with 4 consecutive
//     output columns of one row: the epilogue de-scales in fp32, rounds to BF16 with the hardware
//     conversion and stores 8 bytes per lane; the output absmax is taken on the rounded BF16 bits;
//   - workgroup ids are dealt round-robin to the 8 XCDs by the hardware, so ids are remapped to give
//     each XCD (own L2) a contiguous range of tiles, walked in bands 8 tile-rows high.
// Generic kernel: any shape, one wavefront per 16x16 outputs, guarded loads; slow, for tests and
// odd sizes.
#include "llmq_device.h"
#include "llmq_kernels.h"

namespace llmq {

typedef __attribute__((address_space(3))) void lds_void;
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 256, BN = 256, BK = 128;
constexpr int kGemmThreads = 256;
constexpr int kSlabBytes = BM * BK;                 // 32 KB per operand per stage
constexpr int kXcds = 8;
constexpr int kBandRows = 8;

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
    // raw buffer, no stride; out-of-range reads return zero instead of faulting
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

__device__ inline unsigned bf16_mag_max4(unsigned m, bf16x4 v) {
    v2u w = __builtin_bit_cast(v2u, v);
    unsigned a = w[0] & 0x7FFF7FFFu, b = w[1] & 0x7FFF7FFFu;
    unsigned x = (a & 0xFFFFu) > (a >> 16) ? (a & 0xFFFFu) : (a >> 16);
    unsigned y = (b & 0xFFFFu) > (b >> 16) ? (b & 0xFFFFu) : (b >> 16);
    x = x > y ? x : y;
    return m > x ? m : x;
}

// Linear workgroup id -> output tile, XCD-aware.  Returns false for the padding ids.
__device__ inline bool tile_of_block(int pid, int tiles_r, int tiles_c, int& tr, int& tc) {
    const int nt = tiles_r * tiles_c;
    const int per_xcd = (nt + kXcds - 1) / kXcds;
    const int id = (pid % kXcds) * per_xcd + pid / kXcds;
    if (id >= nt) return false;
    const int band = kBandRows * tiles_c;
    const int first = (id / band) * kBandRows;
    const int h = tiles_r - first < kBandRows ? tiles_r - first : kBandRows;
    const int in_band = id % band;
    tr = first + in_band % h;
    tc = in_band / h;
    return true;
}

// MFMA scheduling masks of __builtin_amdgcn_sched_group_barrier
constexpr int kSchedMfma = 0x008, kSchedVmemRead = 0x020, kSchedDsRead = 0x100;

template <int FA, int FB>
__device__ inline void mma_4x4(v16f (&acc)[4][4], const v8i (&a)[4], const v8i (&b)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b[j], a[i], acc[i][j], FB, FA, 0, 0, 0, 0);
}

// Tuning knobs of the tuned kernel.
struct GemmTuning {
    // K steps ahead of the direct-to-LDS loads at which each wave touches one dword per 128-byte
    // line of its share of the slabs, to pull them into L2 early (0 = no touching).
    static constexpr int kTouchAhead = 2;
    // Development aid: a tuning struct with kProfile = true also provides
    //   static __device__ void record(int block, int slot, long long value)
    // and gets cycle stamps of the phases of wave 0 of every workgroup.
    static constexpr bool kProfile = false;
    // LDS swizzle of the operand slabs: the 16-byte chunk index of a row is XOR-ed with
    // (row >> kSwizzleShift) & 7.
    static constexpr int kSwizzleShift = 1;
};

template <int N>
__device__ inline void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Workgroup barrier that orders LDS traffic only: the caller has already waited for the
// direct-to-LDS loads it needs with wait_vmcnt<>, other global loads may stay in flight.
__device__ inline void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int FA, int FB, class V = GemmTuning>
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_tn_256_kernel(
    const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, uint16_t* __restrict__ C,
    int Cn, int T, const float* __restrict__ d_sA, const float* __restrict__ d_sB,
    int accumulate, unsigned* __restrict__ amax_bits, int tiles_r, int tiles_c) {
    // One array per stage and operand: distinct LDS objects let the compiler see that the
    // direct-to-LDS loads of one stage do not alias the fragment reads of the other, so it does
    // not make the reads wait for the loads in flight.
    __shared__ __attribute__((aligned(1024))) uint8_t ldsA0[kSlabBytes];
    __shared__ __attribute__((aligned(1024))) uint8_t ldsB0[kSlabBytes];
    __shared__ __attribute__((aligned(1024))) uint8_t ldsA1[kSlabBytes];
    __shared__ __attribute__((aligned(1024))) uint8_t ldsB1[kSlabBytes];
    __shared__ unsigned s_amax[kGemmThreads / kWave];
    int tr, tc;
    if (!tile_of_block(blockIdx.x, tiles_r, tiles_c, tr, tc)) return;   // uniform over the workgroup

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int wr = wave >> 1, wc = wave & 1;
    auto stamp = [&](int slot) {
        if constexpr (V::kProfile) {
            if (threadIdx.x == 0) {
                V::record(blockIdx.x, slot, (long long)__builtin_readcyclecounter());
                V::record(blockIdx.x, slot + 8, (long long)__builtin_amdgcn_s_memrealtime());
            }
        }
    };
    stamp(0);

    // ---- global -> LDS: one instruction moves 8 rows x 128 B; wave w moves rows [64w, 64w+64) of A and B
    const __amdgpu_buffer_rsrc_t rsA = make_rsrc(A + (size_t)tr * BM * T, (unsigned)((size_t)BM * T));
    const __amdgpu_buffer_rsrc_t rsB = make_rsrc(B + (size_t)tc * BN * T, (unsigned)((size_t)BN * T));
    // Instruction j of a wave covers rows 64*wave + 8*j + (lane >> 3); the swizzle of those rows only
    // depends on the parity of j.
    constexpr int kSw = V::kSwizzleShift;
    const int ld_row = lane >> 3;                                   // row inside the group of 8
    const int ld_voff0 = ld_row * T + (((lane & 7) ^ ((ld_row >> kSw) & 7)) << 4);
    const int ld_voff1 = ld_row * T + (((lane & 7) ^ (((8 + ld_row) >> kSw) & 7)) << 4);
    const int ld_soff = wave * 64 * T;
    auto issue_loads = [&](uint8_t* slabA, uint8_t* slabB, int k0) {
        uint8_t* sa = slabA + wave * 64 * BK;
        uint8_t* sb = slabB + wave * 64 * BK;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int voff = (j & 1) ? ld_voff1 : ld_voff0;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsA, (lds_void*)(sa + j * 8 * BK), 16, voff, ld_soff + k0 + j * 8 * T, 0, 0);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB, (lds_void*)(sb + j * 8 * BK), 16, voff, ld_soff + k0 + j * 8 * T, 0, 0);
        }
    };

    // ---- LDS -> registers: lane reads 32 contiguous bytes (two swizzled 16-byte chunks) of its row
    const int fr_row = lane & 31;
    const int fr_half = lane >> 5;                                  // which 32 bytes of the 64-byte K half
    const int swz = (fr_row >> kSw) & 7;                            // same for every row this lane reads
    // byte offsets inside a slab for K-half 0 and 1, first and second chunk
    const int offA = (wr * 128 + fr_row) * BK, offB = (wc * 128 + fr_row) * BK;
    const int ch00 = ((fr_half * 2) ^ swz) << 4, ch01 = ((fr_half * 2 + 1) ^ swz) << 4;
    const int ch10 = ((4 + fr_half * 2) ^ swz) << 4, ch11 = ((4 + fr_half * 2 + 1) ^ swz) << 4;
    auto read_frags = [&](const uint8_t* slab, int off, int ks, v8i (&f)[4]) {
        const int c0 = ks ? ch10 : ch00, c1 = ks ? ch11 : ch01;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint8_t* p = slab + off + i * 32 * BK;
            v4i lo = *reinterpret_cast<const v4i*>(p + c0);
            v4i hi = *reinterpret_cast<const v4i*>(p + c1);
            f[i] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
    };

    v16f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    v8i a0[4], b0[4], a1[4], b1[4];        // fragment sets of the two 64-byte halves of a K step
    const int nk = T / BK;

    // L2 touch loads: lane l of wave w reads the first dword of row 64w + l of a slab still V::kTouchAhead
    // steps ahead of the direct-to-LDS loads.  All CUs of an XCD walk K in lock-step, so without this
    // every slab is first requested only ~1.5 steps before it is needed, less than an L2 miss takes.
    constexpr int kTouch = V::kTouchAhead;
    const int touch_voff = lane * T;
    int touchA[2] = {0, 0}, touchB[2] = {0, 0};   // results are only kept so that the loads stay tracked
    int touch_sink = 0;

    // One K step on the stage (curA, curB) while the other stage (nxtA, nxtB) is being filled:
    //   first half : read the second-half fragments            | 16 MFMAs on the first-half fragments
    //   barrier    : the next slab has landed, everybody is done reading the current one
    //   second half: start loading slab kt+2 into the current stage, read the first-half
    //                fragments of slab kt+1                     | 16 MFMAs on the second-half fragments
    // Loads that would start beyond the last slab are pointed outside the buffer range instead:
    // the hardware then fetches nothing, and the stage they would fill is never read.
    constexpr int kOutOfRange = 0x7FFFFF00;
    auto k_step = [&](uint8_t* curA, uint8_t* curB, uint8_t* nxtA, uint8_t* nxtB, int kt, int parity) {
        read_frags(curA, offA, 1, a1);
        read_frags(curB, offB, 1, b1);
        mma_4x4<FA, FB>(acc, a0, b0);
        // fragment reads ride along with the first 8 MFMAs, so that they have landed by the 16th
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(kSchedMfma, 1, 0);
            __builtin_amdgcn_sched_group_barrier(kSchedDsRead, 2, 0);
        }
        __builtin_amdgcn_sched_group_barrier(kSchedMfma, 8, 0);
        // the 16 direct-to-LDS loads of the previous step must have landed; its two touch loads, issued
        // after them, may still be in flight
        if constexpr (kTouch > 0) wait_vmcnt<2>(); else wait_vmcnt<0>();
        lds_barrier();
        __builtin_amdgcn_sched_barrier(0);
        issue_loads(curA, curB, kt + 2 < nk ? (kt + 2) * BK : kOutOfRange);
        read_frags(nxtA, offA, 0, a0);          // past the last slab this reads stale bytes that are never used
        read_frags(nxtB, offB, 0, b0);
        mma_4x4<FA, FB>(acc, a1, b1);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(kSchedMfma, 1, 1);
            __builtin_amdgcn_sched_group_barrier(kSchedDsRead, 2, 1);
            __builtin_amdgcn_sched_group_barrier(kSchedVmemRead, 1, 1);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(kSchedMfma, 1, 1);
            __builtin_amdgcn_sched_group_barrier(kSchedVmemRead, 1, 1);
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (kTouch > 0) {
            const int kp = kt + 2 + kTouch;
            const int off = kp < nk ? ld_soff + kp * BK : kOutOfRange;
            touch_sink ^= touchA[parity] ^ touchB[parity];          // issued two steps ago: long landed
            touchA[parity] = __builtin_amdgcn_raw_buffer_load_b32(rsA, touch_voff, off, 0);
            touchB[parity] = __builtin_amdgcn_raw_buffer_load_b32(rsB, touch_voff, off, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    issue_loads(ldsA0, ldsB0, 0);
    wait_vmcnt<0>();
    lds_barrier();
    issue_loads(ldsA1, ldsB1, nk > 1 ? BK : kOutOfRange);
    if constexpr (kTouch > 0) {                   // keep "two touch loads are the newest" true from the start
        touchA[1] = __builtin_amdgcn_raw_buffer_load_b32(rsA, touch_voff, 2 < nk ? ld_soff + 2 * BK : kOutOfRange, 0);
        touchB[1] = __builtin_amdgcn_raw_buffer_load_b32(rsB, touch_voff, 2 < nk ? ld_soff + 2 * BK : kOutOfRange, 0);
    }
    read_frags(ldsA0, offA, 0, a0);
    read_frags(ldsB0, offB, 0, b0);
    stamp(1);
    int kt = 0;
    for (; kt + 1 < nk; kt += 2) {
        k_step(ldsA0, ldsB0, ldsA1, ldsB1, kt, 0);
        k_step(ldsA1, ldsB1, ldsA0, ldsB0, kt + 1, 1);
    }
    if (kt < nk) k_step(ldsA0, ldsB0, ldsA1, ldsB1, kt, 0);
    wait_vmcnt<0>();                               // nothing may still be landing in LDS when the wave ends
    if constexpr (kTouch > 0) {
        touch_sink ^= touchA[0] ^ touchB[0] ^ touchA[1] ^ touchB[1];
        asm volatile("" ::"v"(touch_sink));
    }
    stamp(2);

    // ---- epilogue.  Per 32x32 block a lane holds 4 groups of 4 consecutive columns of row (lane % 32).
    // Storing those 8-byte pieces directly scatters every store over 32 rows; instead each wave
    // stages its 128x128 BF16 quadrant (32 KB) in one of the four slabs, which nobody reads any more,
    // and writes it out as full 256-byte row segments, 16 bytes per lane.  Rows are 256 B in LDS with
    // the 16-byte slot index XOR-ed with (row & 15), so both the 8-byte writes and the 16-byte reads
    // spread over all banks.  The region is private to the wave and LDS executes a wave's accesses
    // in order, so no barrier is needed.
    const float inv_a = 1.0f / *d_sA, inv_b = 1.0f / *d_sB;
    unsigned mag = 0;
    if (!accumulate) {
        uint8_t* stage = wave == 0 ? ldsA0 : wave == 1 ? ldsB0 : wave == 2 ? ldsA1 : ldsB1;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = i * 32 + fr_row;
            uint8_t* srow = stage + row * 256;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int col = j * 32 + g * 8 + fr_half * 4;            // multiple of 4
                    v4f y;
#pragma unroll
                    for (int e = 0; e < 4; ++e) y[e] = acc[i][j][4 * g + e] * inv_a * inv_b;
                    bf16x4 o = __builtin_convertvector(y, bf16x4);
                    mag = bf16_mag_max4(mag, o);
                    *reinterpret_cast<bf16x4*>(srow + ((((col >> 3) ^ (row & 15)) << 4) | ((col & 7) << 1))) = o;
                }
            }
        }
        const int slot = lane & 15, sub = lane >> 4;                          // 16 lanes per row, 4 rows per pass
        uint16_t* cbase = C + (size_t)(tr * BM + wr * 128) * Cn + tc * BN + wc * 128 + slot * 8;
#pragma unroll 8
        for (int it = 0; it < 32; ++it) {
            const int row = it * 4 + sub;
            v4u v = *reinterpret_cast<const v4u*>(stage + row * 256 + ((slot ^ (row & 15)) << 4));
            *reinterpret_cast<v4u*>(cbase + (size_t)row * Cn) = v;
        }
    } else {
        // BF16 accumulation needs the old value before the single rounding: straight from the registers.
        const int row_base = tr * BM + wr * 128 + fr_row;
        const int col_base = tc * BN + wc * 128 + fr_half * 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint16_t* crow = C + (size_t)(row_base + i * 32) * Cn + col_base;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    uint16_t* dst = crow + j * 32 + g * 8;
                    v4f y;
#pragma unroll
                    for (int e = 0; e < 4; ++e) y[e] = acc[i][j][4 * g + e] * inv_a * inv_b;
                    v2u old = *reinterpret_cast<const v2u*>(dst);
                    y[0] += __uint_as_float(old[0] << 16);
                    y[1] += __uint_as_float(old[0] & 0xFFFF0000u);
                    y[2] += __uint_as_float(old[1] << 16);
                    y[3] += __uint_as_float(old[1] & 0xFFFF0000u);
                    bf16x4 o = __builtin_convertvector(y, bf16x4);
                    mag = bf16_mag_max4(mag, o);
                    *reinterpret_cast<bf16x4*>(dst) = o;
                }
            }
        }
    }
    if (amax_bits) {
        mag = wave_max_u32(mag);
        if (lane == 0) s_amax[wave] = mag;
        __syncthreads();
        if (threadIdx.x == 0) {
#pragma unroll
            for (int w = 1; w < kGemmThreads / kWave; ++w) mag = mag > s_amax[w] ? mag : s_amax[w];
            // same-address atomics of many workgroups serialise; a stale read never exceeds the true maximum
            const unsigned bits = amax_bits_from_bf16_mag(mag);
            if (bits > __hip_atomic_load(amax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(amax_bits, bits);
        }
    }
    if constexpr (V::kProfile) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        stamp(3);
    }
}

// ---- generic kernel: one wavefront per 16x16 outputs, v_mfma_f32_16x16x128_f8f6f4, guarded loads
template <int FA, int FB>
__global__ __launch_bounds__(256) void gemm_tn_generic_kernel(
    const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, uint16_t* __restrict__ C,
    int64_t R, int64_t Cn, int64_t T, const float* __restrict__ d_sA, const float* __restrict__ d_sB,
    int accumulate, unsigned* __restrict__ amax_bits) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int64_t r0 = ((int64_t)blockIdx.y * 2 + (wave >> 1)) * 16;
    const int64_t c0 = ((int64_t)blockIdx.x * 2 + (wave & 1)) * 16;
    const int64_t ar = r0 + (lane & 15), bc = c0 + (lane & 15);
    const bool a_ok = ar < R, b_ok = bc < Cn;
    const bool vec_ok = (T % 16) == 0;
    auto load32 = [&](const uint8_t* base, bool ok, int64_t row, int64_t k) -> v8i {
        v8i v = {0, 0, 0, 0, 0, 0, 0, 0};
        if (!ok || k >= T) return v;
        const uint8_t* p = base + row * T + k;
        if (vec_ok && k + 32 <= T) {
            v4i lo = *reinterpret_cast<const v4i*>(p), hi = *reinterpret_cast<const v4i*>(p + 16);
            return v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
        for (int w = 0; w < 8; ++w) {
            unsigned word = 0;
            for (int e = 0; e < 4; ++e) {
                int64_t kk = k + w * 4 + e;
                if (kk < T) word |= (unsigned)p[w * 4 + e] << (8 * e);   // beyond T: code 0x00 = +0
            }
            v[w] = (int)word;
        }
        return v;
    };
    v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int64_t k0 = 0; k0 < T; k0 += 128) {
        const int64_t k = k0 + (lane >> 4) * 32;
        v8i a = load32(A, a_ok, ar, k);
        v8i b = load32(B, b_ok, bc, k);
        acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(b, a, acc, FB, FA, 0, 0, 0, 0);
    }
    // lane holds row r0 + lane % 16, columns c0 + 4 * (lane / 16) + 0..3
    const float inv_a = 1.0f / *d_sA, inv_b = 1.0f / *d_sB;
    unsigned mag = 0;
    const int64_t r = r0 + (lane & 15);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int64_t c = c0 + (lane >> 4) * 4 + e;
        if (r < R && c < Cn) {
            float y = acc[e] * inv_a * inv_b;
            uint16_t* dst = C + r * Cn + c;
            if (accumulate) y += __uint_as_float((unsigned)*dst << 16);
            __bf16 o = (__bf16)y;
            unsigned bits = __builtin_bit_cast(uint16_t, o);
            *dst = (uint16_t)bits;
            bits &= 0x7FFFu;
            mag = mag > bits ? mag : bits;
        }
    }
    if (amax_bits) {
        mag = wave_max_u32(mag);
        if (lane == 0) atomicMax(amax_bits, amax_bits_from_bf16_mag(mag));
    }
}

__global__ void gemm_amax_reset_kernel(unsigned* amax_bits) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *amax_bits = 0u;
}

template <int FA, int FB>
static void launch_one(const uint8_t* A, const uint8_t* B, int64_t R, int64_t C, int64_t T,
                       const float* sA, const float* sB, void* c, int accumulate, unsigned* amax,
                       hipStream_t stream) {
    const bool tuned = R % BM == 0 && C % BN == 0 && T % BK == 0 &&
                       (size_t)BM * T < (1ull << 31) && R * T < (1ll << 40) && C * T < (1ll << 40);
    if (tuned) {
        const int tiles_r = (int)(R / BM), tiles_c = (int)(C / BN);
        const int nt = tiles_r * tiles_c;
        const int grid = ((nt + kXcds - 1) / kXcds) * kXcds;
        hipLaunchKernelGGL((gemm_tn_256_kernel<FA, FB>), dim3(grid), dim3(kGemmThreads), 0, stream,
                           A, B, reinterpret_cast<uint16_t*>(c), (int)C, (int)T, sA, sB,
                           accumulate, amax, tiles_r, tiles_c);
    } else {
        dim3 grid((unsigned)((C + 31) / 32), (unsigned)((R + 31) / 32));
        hipLaunchKernelGGL((gemm_tn_generic_kernel<FA, FB>), grid, dim3(256), 0, stream,
                           A, B, reinterpret_cast<uint16_t*>(c), R, C, T, sA, sB, accumulate, amax);
    }
}

int launch_gemm_tn(const uint8_t* A, int fmtA, const uint8_t* B, int fmtB, int64_t R, int64_t C,
                   int64_t T, const float* d_scaleA, const float* d_scaleB, void* c_bf16,
                   int accumulate, float* d_amax_c, hipStream_t stream, int num_cus) {
    (void)num_cus;
    unsigned* amax = reinterpret_cast<unsigned*>(d_amax_c);
    if (amax) hipLaunchKernelGGL(gemm_amax_reset_kernel, dim3(1), dim3(64), 0, stream, amax);
    if (fmtA == 0 && fmtB == 0) launch_one<0, 0>(A, B, R, C, T, d_scaleA, d_scaleB, c_bf16, accumulate, amax, stream);
    else if (fmtA == 1 && fmtB == 0) launch_one<1, 0>(A, B, R, C, T, d_scaleA, d_scaleB, c_bf16, accumulate, amax, stream);
    else if (fmtA == 0 && fmtB == 1) launch_one<0, 1>(A, B, R, C, T, d_scaleA, d_scaleB, c_bf16, accumulate, amax, stream);
    else launch_one<1, 1>(A, B, R, C, T, d_scaleA, d_scaleB, c_bf16, accumulate, amax, stream);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace llmq
