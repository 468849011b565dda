// Tile kernel of the FP8 contraction on the gfx950 matrix cores (paper Section 3: the transformer-block matmuls of
// forward and backward run in FP8, results stay in BF16; the FP8 GEMM is "TN", i.e. both operands
// have the contraction index contiguous).
//
//   C[r,c] = bf16( (sum_t A[r,t] * B[c,t]) / (sA * sB) ),   A [R,T] fp8, B [Cn,T] fp8.
//
// Tuned kernel (template on the wave tile NI x NJ in units of 32: workgroup tile BM x BN with
// BM = 64 NI, BN = 64 NJ, both in {128, 192, 256}; R % BM == 0, Cn % BN == 0, T % 128 == 0)
//   - one workgroup of 4 wavefronts (2 x 2) per output tile, one workgroup per CU; a wavefront owns
//     2 NI x 2 NJ blocks of v_mfma_f32_16x16x128_f8f6f4 with fp32 accumulators (256 registers per lane at
//     4 x 4: the whole accumulator file);
//   - K advances 128 bytes per step, one MFMA deep; the A and B slabs (BM / BN rows x 128 B) go from global
//     memory straight into LDS with buffer_load ... lds (16 bytes per lane, no VGPR staging), double buffered;
//   - LDS rows are 128 B; the 16-byte chunk index is XOR-ed with a function of the row (row_swizzle), applied
//     on the global side of the load, so that the ds_read_b128 fragment reads run without bank conflicts;
//   - the order of the contraction index inside one MFMA does not matter as long as A and B use
//     the same order, so lane L simply reads the 32 contiguous bytes [32 (L / 16), +32) of row L % 16;
//   - every step is software pipelined in four quarters (half the block rows x half the block columns): the MFMAs
//     of one quarter run while the one fragment set that is free by then is read for the next quarter but one,
//     and the slab after next is requested during the second half; one barrier per step;
//   - the MFMA takes the B rows as its first operand, which leaves every lane with 4 consecutive
//     output columns of one row; the epilogue de-scales in fp32, rounds to BF16 with the hardware
//     conversion, takes the output absmax on the rounded bits, stages the wave's quadrant in LDS
//     and stores full row segments, 16 bytes per lane;
//   - workgroup ids are dealt round-robin to the 8 XCDs by the hardware, so ids are remapped to give
//     each XCD (own L2) a contiguous range of tiles, walked in bands 4 tile-rows high;
//   - the host picks NI x NJ per problem so that the tiles fill the 256 CUs in whole rounds.
// Generic kernel: any shape, one wavefront per 16x16 outputs, guarded loads; slow, for tests and
// odd sizes.
//
// An operand may also be given "T-major", [T, rows] with the contraction index running down the rows (the
// untransposed quantized tensor where the backward pass contracts over what is the row index of the
// forward pass): see SlabShape below.  This header holds the kernel and its launcher; the translation
// units that include it instantiate the operand layouts they serve.
#pragma once
#include <stdlib.h>

#include "llmq_device.h"
#include "llmq_kernels.h"

namespace llmq {

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(3))) v2i lds_v2i;
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 128;
constexpr int kGemmThreads = 256;
constexpr int kXcds = 8;
constexpr int kBandRows = 4;

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
    // raw buffer, no stride; out-of-range reads return zero instead of faulting
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// Workgroup id -> position in a walk of n items, XCD-aware: the hardware deals workgroup ids round-robin to
// the XCDs, and every XCD gets a contiguous range of positions.  -1 for the padding ids.
__host__ __device__ inline int walk_position(int pid, int n) {
    const int per_xcd = (n + kXcds - 1) / kXcds;
    const int pos = (pid % kXcds) * per_xcd + pid / kXcds;
    return pos < n ? pos : -1;
}

// Position in the walk of tiles -> output tile: bands band_rows tile rows high, walked down the rows first.
__host__ __device__ inline void tile_of_position(int pos, int tiles_r, int tiles_c, int band_rows, int& tr, int& tc) {
    const int band = band_rows * tiles_c;
    const int first = (pos / band) * band_rows;
    const int h = tiles_r - first < band_rows ? tiles_r - first : band_rows;
    const int in_band = pos % band;
    tr = first + in_band % h;
    tc = in_band / h;
}

// How a launch shares out its tiles: a deterministic split of the contraction for a ragged last round of tiles
// (paper Section 3 "Reproducibility": partial results go to an intermediate buffer and are added in a fixed
// order by a second step, never with atomic additions).
//   Positions [0, n_whole) of the walk are computed whole, one workgroup per tile, by a launch of the plain
//   kernel (n_whole is a multiple of the number of workgroups the chip holds: whole rounds).  The remaining
//   positions are served by a launch of the kSharePieces instantiation, which comes first; they come in up to
//   kMaxSplitGroups groups; the tiles of a group are each cut into `pieces` pieces of `steps` K steps (the last
//   piece takes what is left), one workgroup per piece, and a group never has more workgroups than the chip holds
//   at once, so the groups run one after the other like rounds of ever shorter pieces: 192 left-over tiles on
//   256 CUs are 128 tiles in halves, then 64 tiles in quarters, 3/4 of a round instead of a whole one.
//   A piece's accumulators go, as binary32, to slot (wg_begin + tile_in_group * pieces + piece) of `partials`
//   (also those of a tile left whole, pieces == 1, in a last group: the kernel of the pieces has no other way
//   out), and a launch of the kShareFixup instantiation, one workgroup per shared tile, adds the pieces of a tile
//   in the order of their K ranges and runs the usual epilogue on the sums.
constexpr int kMaxSplitGroups = 4;
struct SplitGroup {
    int tile_begin;      // first tile of the group, counted from n_whole
    int tiles;
    int pieces;          // per tile
    int steps;           // K steps per piece
    int wg_begin;        // first workgroup of the group in the sharing launch; also its first slot
    int wgs;             // workgroups of the group, padded to a multiple of the XCD count
};
struct SplitPlan {
    int n_whole;         // the plain kernel walks positions [0, n_whole); the shared tiles follow
    int n_groups;        // 0: nothing is shared
    SplitGroup group[kMaxSplitGroups];
    float* partials;
};

// Tuning knobs of the tuned kernel.
struct GemmTuning {
    // Whether the kernel contains the L2 touch loads at all (their distance is a run-time argument).
    static constexpr bool kTouch = true;
    // Fragment reads ride along with the first 1 / kDsSpread of a quarter step's MFMAs (4 x 4 tiles) or
    // 1 / kDsSpreadSmall (smaller tiles: fewer MFMAs per read); on the 4 x 4 tile spreading them over the whole
    // quarter measured the same.
    static constexpr int kDsSpread = 2, kDsSpreadSmall = 1;
    // The direct-to-LDS loads of a step travel with the third quarter's MFMAs (1) or the third and fourth (2).
    // An MFMA of this shape occupies the matrix pipe for 32 cycles only: with a fragment read, a load and its
    // address arithmetic behind every MFMA of the third quarter the wave cannot issue the next MFMA in time
    // (measured on 8192^3: 3.6 PFLOP/s on all-zero operands with 1, 4.04 with 2; 2.77 and 2.89 on random codes).
    static constexpr int kLoadQuarters = 2;
    static constexpr bool kNtStoreC = false;     // streaming hint on the output stores
    // Scheduling fences between the 32-row blocks of the epilogue: without them the compiler hoists every
    // de-scale multiply to the front and parks the products in accumulator registers.
    static constexpr bool kEpilogueFence = true;
    // Phase stamps (llmq_calibrate_gemm_phases): a tuning struct with kProfile = true also provides
    //   static __device__ void record(float* buf, int block, int slot, long long value)
    // and wave 0 of every workgroup stamps the cycle counter and the 100 MHz clock at the start (slots 0, 8),
    // after the first fragments are in registers (1, 9), after the K loop (2, 10), after the last output store
    // is issued (4, 12), after the absmax (5, 13) and after all stores have completed (3, 11); buf is the
    // `partials` pointer of the plan, which the plain kernel does not use otherwise.
    static constexpr bool kProfile = false;
    // The fused output absmax with the IEEE 754-2019 maximum (v_maximum3_f32: two elements per instruction, NaN
    // propagates) or, for comparison in the phase stamps only, with maxNum (v_max_f32 per element, NaN dropped).
    static constexpr bool kIeeeMaximum = true;
};

template <bool B>
struct BoolTag { static constexpr bool value = B; };
template <int N>
struct IntTag { static constexpr int value = N; };

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

// Operand kinds of the tuned kernel: 0 = E4M3, 1 = E5M2 (one byte per element, any mix), 2 = BF16 (both
// operands; the baseline the FP8 path is compared with).  The kernel itself moves bytes: T is the length of
// a row in bytes, and a lane's 32-byte fragment holds 32 FP8 or 16 BF16 contraction elements.
constexpr int kFmtBf16 = 2;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// The accumulators of a wave tile of MI x MJ blocks of 16 x 16, four registers per block and lane.
template <int MI, int MJ>
struct BlockAcc {
    v4f t[MI][MJ];
    __device__ inline v4f get(int i, int j) const { return t[i][j]; }
    __device__ inline void set(int i, int j, const v4f& v) { t[i][j] = v; }
};

// Calls f(IntTag<0>{}), ..., f(IntTag<N - 1>{}).
template <int N, int I = 0, class F>
__device__ inline void static_for(F&& f) {
    if constexpr (I < N) {
        f(IntTag<I>{});
        static_for<N, I + 1>(f);
    }
}

// One 16 x 16 block update: acc(16 x 16) += a(16 x 128 bytes) b(16 x 128 bytes)^T.
// v_mfma_f32_16x16x128_f8f6f4 rather than 32x32x64: on random FP8 bits, where the board's power cap and not the
// issue rate sets the speed, a register-only loop of the 16x16x128 form sustains 4.22 PFLOP/s against 3.83-3.85
// for 32x32x64 (both 4.98 on constant bits): it adds 128 products per accumulator update instead of 64.
template <int FA, int FB>
__device__ inline void mma_block(v4f& c, const v8i& a, const v8i& b) {
    static_assert((FA == kFmtBf16) == (FB == kFmtBf16), "BF16 operands come in pairs");
    // The instructions are written out so that the accumulator can be constrained to the accumulator register file
    // and tied to the result.  Given the builtin, whose accumulators may sit in either file, the register
    // allocator moves the 4-register blocks between the files inside the K loop (hundreds of copies and a
    // handful of spills per K step, which made the kernel issue-bound at half its speed).  The compiler does
    // not know what the statement is, so it adds none of the MFMA wait states; the kernel needs none: fragments
    // come from LDS reads (waited for by counter), a block is updated again 16 or more MFMAs later, and
    // the epilogue starts behind wait states of its own, a counter wait and a barrier.
    if constexpr (FA == kFmtBf16) {
        // two v_mfma_f32_16x16x32_bf16, one per 16-byte half of the fragments
        const v4i a_lo = {a[0], a[1], a[2], a[3]}, a_hi = {a[4], a[5], a[6], a[7]};
        const v4i b_lo = {b[0], b[1], b[2], b[3]}, b_hi = {b[4], b[5], b[6], b[7]};
        asm("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(b_lo), "v"(a_lo));
        asm("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(b_hi), "v"(a_hi));
    } else {
        // cbsz / blgp: formats of the first / second operand
        asm("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0 cbsz:%3 blgp:%4" : "+a"(c) : "v"(b), "v"(a), "n"(FB), "n"(FA));
    }
}

// One quarter of a wave tile's MFMAs of a K step: the 16 x 16 blocks (I0 + i, J0 + j) of the accumulators from HI
// fragments of A and HJ fragments of B (32 bytes per lane each: the 128-byte K step of 16 operand rows), i running
// slowest (or j with J_OUTER: the set that was read last is then needed one fragment at a time).  After block update
// number m the caller's side(IntTag<m>) issues whatever memory instructions are to travel with it; scheduling fences
// keep that order (the written-out MFMA is invisible to the scheduler's instruction classes, so the order is fixed
// here rather than asked for with group barriers).
template <int FA, int FB, int I0, int J0, bool J_OUTER, int MI, int MJ, int HI, int HJ, class Side>
__device__ inline void mma_quadrant(BlockAcc<MI, MJ>& acc, const v8i (&a)[HI], const v8i (&b)[HJ], Side&& side) {
    static_for<HI * HJ>([&](auto tag) {
        constexpr int m = decltype(tag)::value;
        constexpr int i = J_OUTER ? m % HI : m / HJ, j = J_OUTER ? m / HI : m % HJ;
        mma_block<FA, FB>(acc.t[I0 + i][J0 + j], a[i], b[j]);
        side(tag);
        __builtin_amdgcn_sched_barrier(0);
    });
}

// LDS swizzle of a row-wise slab: the 16-byte chunk index of a row (row index modulo 16) is XOR-ed with this.
// A fragment read has lane L fetch chunks 2 (L / 16) and 2 (L / 16) + 1 of row L % 16 with ds_read_b128, which the
// LDS serves 16 lanes (256 B) per cycle when their bank groups differ; which 16 lanes share a cycle was not
// established, only what each candidate costs with four waves reading back to back: this function 4.0 cycles per
// instruction (the same as a linear pattern), (row >> 1) & 7 and row & 7 8.0, no swizzle 16.0.  The GEMM itself runs
// the same with 4 or 8 cycles per read (the LDS is a quarter or half busy), within 1 %.
__device__ constexpr int row_swizzle(int row) { return (((row >> 1) & 3) << 1) | ((row >> 3) & 1); }

// How an operand [rows, T] may sit in memory (OperandLayout of the launchers):
//   rows    : row r at r T, its T contraction bytes contiguous;
//   t_major : the transposed tensor [T, rows] (see TMAJOR below);
//   slabs   : K step by K step, byte (r, t) at (t / 128) rows 128 + r 128 + t % 128: each K step of all rows is one
//             contiguous piece (T a multiple of 128).  The kernel reads it like `rows` with a row pitch of 128 bytes
//             and rows x 128 bytes from one K step to the next; the tile kernel of the quantizer writes its transposed
//             copy that way, a whole tile's transposed bytes as one contiguous 32 KB piece.
// How one operand slab sits in memory and in LDS, and how its MFMA fragments are read.
//   TMAJOR = false: the operand is [rows, T], a slab is 64 NX rows of 128 B; LDS keeps the rows, 128 B
//     each, the 16-byte chunk index XOR-ed with row_swizzle(row); a lane reads the 32 contiguous
//     bytes of its row with two ds_read_b128.
//   TMAJOR = true: the operand is [T, rows] (the contraction index runs down the rows, `ld` bytes apart),
//     a slab is 128 rows of 64 NX bytes and LDS keeps it that way.  A lane's 32 contraction bytes then sit
//     in 32 different LDS rows; four ds_read_b64_tr_b8 fetch them: within 16 lanes, lane s points at 8
//     bytes of row k0 + s / 2 (the two lanes of a pair at the two halves of 16 consecutive bytes), and the
//     hardware hands lane i the byte of column i of each of the eight rows, in row order.  So lane i holds
//     contraction bytes k0 .. k0 + 7 of operand row r0 + i, the same order as in the other layout, and the
//     two layouts mix freely in one MFMA.  The 16-byte unit index of an LDS row is XOR-ed with a mask that
//     depends on the row (swizzle_of_row), again on the global side of the load, so that the rows one
//     transposing read touches lie in different banks.
template <int NX, bool TMAJOR>
struct SlabShape {
    static constexpr int kRows = 64 * NX;                     // operand rows (output rows or columns) of the tile
    static constexpr int kUnits = kRows / 16;                 // T-major: 16-byte units per LDS row
    static constexpr int kPeriod = NX == 4 ? 2 : NX == 2 ? 1 : 3;       // T-major: load instructions per pattern
    static constexpr int kPeriodRows = 64 * kPeriod / kUnits;           // T-major: slab rows per pattern
    static constexpr int kReadsPerFrag = TMAJOR ? 4 : 2;
    static constexpr int kLines = TMAJOR ? (kRows + 127) / 128 : 1;     // 128-byte lines per memory row of a slab
    // XOR mask of the 16-byte unit index of LDS row k.  One transposing read of 32 lanes touches 8 consecutive
    // rows x 2 neighbouring units (x 2 halves); the mask moves in steps of two units so that these 16 units fall
    // into 16 different groups of four banks: rows are 64 / 48 / 32 banks long for NX = 4 / 3 / 2.
    // The two halves of 16 lanes of such a read sit 32 LDS rows apart (K quarters of the 16x16x128 fragment), i.e. a
    // multiple of 64 banks: bit 5 of the row goes into the lowest bit of the mask to separate them.
    __device__ static int swizzle_of_row(int k) { return ((NX == 4 ? k & 7 : NX == 2 ? (k >> 1) & 3 : (k >> 2) & 1) << 1) | ((k >> 5) & 1); }
};

// MODE: kWholeTiles ignores the plan and computes one whole tile per workgroup, with nothing of the sharing logic
// in the code; kSharePieces computes the pieces of shared tiles; kShareFixup adds them up and has no K loop.  Three
// kernels rather than branches of one: the accumulators fill the accumulator file, and code that reaches them from
// two sides (loaded sums or MFMA results) made the register allocator spill them around the K loop.
constexpr int kWholeTiles = 0, kSharePieces = 1, kShareFixup = 2;
template <int FA, int FB, int NI, int NJ, bool ACCUM, class V = GemmTuning, bool TA = false, bool TB = false, int MODE = kWholeTiles>
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_tile_kernel(
    const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, uint16_t* __restrict__ C,
    int Cn, int T, const float* __restrict__ d_sA, const float* __restrict__ d_sB,
    unsigned* __restrict__ amax_bits, int tiles_r, int tiles_c, int touch_ahead, int band_rows, int next_stride,
    int ldA, int ldB, int ks_a, int ks_b, int share_a, int share_b, const SplitPlan plan) {
    static_assert(!(TA || TB) || (FA != kFmtBf16 && FB != kFmtBf16), "the transposing reads move single bytes");
    // Bytes from one K step of an operand to the next: 128 rows of a T-major operand, else what the host says
    // (128 for rows of T contiguous bytes; rows x 128 when the operand is stored slab by slab, see OperandLayout).
    const int ksA = TA ? BK * ldA : ks_a, ksB = TB ? BK * ldB : ks_b;
    constexpr int BM = 64 * NI, BN = 64 * NJ;
    typedef SlabShape<NI, TA> SA;
    typedef SlabShape<NJ, TB> SB;
    constexpr int kOutOfRange = 0x7FFFFF00;     // a buffer offset beyond every operand: such loads fetch nothing
    constexpr int kSlabA = BM * BK, kSlabB = BN * BK;
    // One array per stage and operand: distinct LDS objects let the compiler see that the
    // direct-to-LDS loads of one stage do not alias the fragment reads of the other, so it does
    // not make the reads wait for the loads in flight.
    __shared__ __attribute__((aligned(1024))) uint8_t ldsA0[kSlabA];
    __shared__ __attribute__((aligned(1024))) uint8_t ldsB0[kSlabB];
    __shared__ __attribute__((aligned(1024))) uint8_t ldsA1[kSlabA];
    __shared__ __attribute__((aligned(1024))) uint8_t ldsB1[kSlabB];
    // Four words for the workgroup's output absmax.  The epilogue stages 2048 NJ bytes per wave at the start
    // of the slabs (8192 NJ bytes in the case of this one), so the end of the last slab is free by then; the
    // kernel's LDS is exactly its slabs.
    unsigned* s_amax = reinterpret_cast<unsigned*>(ldsB1 + kSlabB - 16);
    // What this workgroup computes (uniform over the workgroup): the tile at position `pos` of the walk, K steps
    // [kb, kb + nk), written as a whole tile (slot < 0) or as one piece of a shared tile.  In the fix-up launch
    // slot is the first slot of the tile's pieces and nk their number.
    int pos, kb = 0, nk = T / BK, slot = -1;
    constexpr bool SPLIT = MODE != kWholeTiles, fixup = MODE == kShareFixup;
    if constexpr (!SPLIT) {
        pos = walk_position(blockIdx.x, plan.n_whole);
        if (pos < 0) return;
    } else {
        const int q = (int)blockIdx.x;                     // shared tile (fix-up launch) or sharing workgroup
        int gi = 0;
        while (gi + 1 < plan.n_groups && q >= (fixup ? plan.group[gi + 1].tile_begin : plan.group[gi + 1].wg_begin)) ++gi;
        const SplitGroup grp = plan.group[gi];
        if constexpr (fixup) {
            const int j = q - grp.tile_begin;
            pos = plan.n_whole + q;
            slot = grp.wg_begin + j * grp.pieces;
            nk = grp.pieces;
        } else {
            const int w = walk_position(q - grp.wg_begin, grp.tiles * grp.pieces);   // neighbours on an XCD: neighbouring tiles, same K range
            if (w < 0) return;
            const int piece = w / grp.tiles, j = w - piece * grp.tiles;
            pos = plan.n_whole + grp.tile_begin + j;
            kb = piece * grp.steps;
            nk = nk - kb < grp.steps ? nk - kb : grp.steps;
            if (nk <= 0) return;                           // cannot happen with steps = ceil(K steps / pieces)
            slot = grp.wg_begin + j * grp.pieces + piece;
        }
    }
    int tr, tc;
    tile_of_position(pos, tiles_r, tiles_c, band_rows, tr, tc);

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int wr = wave >> 1, wc = wave & 1;
    auto stamp = [&](int slot) {
        if constexpr (V::kProfile) {
            if (threadIdx.x == 0) {
                V::record(plan.partials, blockIdx.x, slot, (long long)__builtin_readcyclecounter());
                V::record(plan.partials, blockIdx.x, slot + 8, (long long)__builtin_amdgcn_s_memrealtime());
            }
        }
    };
    stamp(0);
    // requested now, needed in the epilogue; BF16 operands carry no scales
    const float scale_a = FA == kFmtBf16 ? 1.0f : *d_sA, scale_b = FB == kFmtBf16 ? 1.0f : *d_sB;

    // ---- global -> LDS.  Row-wise operand: one instruction moves 8 rows x 128 B; wave w moves rows
    // [16 NX w, 16 NX (w+1)) of the slab with 2 NX instructions; instruction j covers rows 8 j + (lane >> 3)
    // of the wave's share, and the swizzle of those rows only depends on the parity of j (the share starts
    // at a multiple of 16 rows).  T-major operand: an instruction moves 1 KB = 64 units of consecutive LDS
    // rows (64 NX bytes each); wave w moves slab rows [32 w, 32 w + 32), again 2 NX instructions, whose
    // lane pattern repeats every kPeriod instructions (kPeriodRows slab rows).
    const __amdgpu_buffer_rsrc_t rsA = TA ? make_rsrc(A + (size_t)tr * BM, (unsigned)((size_t)T * ldA - (size_t)tr * BM))
                                          : make_rsrc(A + (size_t)tr * BM * ldA, (unsigned)((size_t)(T / BK - 1) * ksA + (size_t)(BM - 1) * ldA + BK));
    const __amdgpu_buffer_rsrc_t rsB = TB ? make_rsrc(B + (size_t)tc * BN, (unsigned)((size_t)T * ldB - (size_t)tc * BN))
                                          : make_rsrc(B + (size_t)tc * BN * ldB, (unsigned)((size_t)(T / BK - 1) * ksB + (size_t)(BN - 1) * ldB + BK));
    const int ld_row = lane >> 3;                                   // row inside the group of 8
    auto rows_voff = [&](int m, int ld) {                           // rows 8 m + ld_row of a row-wise operand, `ld` bytes apart
        return ld_row * ld + (((lane & 7) ^ row_swizzle(8 * m + ld_row)) << 4);
    };
    auto tmajor_voff = [&](auto shape, int m, int ld) {             // pattern m of a T-major operand
        typedef decltype(shape) S;
        const int unit = 64 * m + lane, row = unit / S::kUnits, col = unit % S::kUnits;
        return row * ld + ((col ^ S::swizzle_of_row(row + 32 * wave)) << 4);      // the wave moves slab rows [32 wave, 32 wave + 32)
    };
    int ld_voffA[3], ld_voffB[3];
#pragma unroll
    for (int m = 0; m < 3; ++m) {
        ld_voffA[m] = TA ? (m < SA::kPeriod ? tmajor_voff(SA{}, m, ldA) : 0) : rows_voff(m & 1, ldA);
        ld_voffB[m] = TB ? (m < SB::kPeriod ? tmajor_voff(SB{}, m, ldB) : 0) : rows_voff(m & 1, ldB);
    }
    const int ld_soffA = TA ? wave * 32 * ldA : wave * 16 * NI * ldA, ld_soffB = TB ? wave * 32 * ldB : wave * 16 * NJ * ldB;
    // The direct-to-LDS loads of one slab pair: pieces 0 .. 2 NI - 1 fill the wave's share of the A slab, the
    // next 2 NJ that of the B slab.  step: K step of the slab, or a negative value for "no slab"
    // (nothing is fetched).
    auto load_base = [&](int step, int& baseA, int& baseB) {
        baseA = step < 0 ? kOutOfRange : ld_soffA + step * ksA;
        baseB = step < 0 ? kOutOfRange : ld_soffB + step * ksB;
    };
    auto issue_load = [&](uint8_t* slabA, uint8_t* slabB, int baseA, int baseB, auto piece) {
        constexpr int p = decltype(piece)::value;
        if constexpr (p < 2 * NI) {
            constexpr int j = p;
            const int voff = TA ? ld_voffA[j % SA::kPeriod] : ld_voffA[j & 1];
            const int soff = TA ? (j / SA::kPeriod) * SA::kPeriodRows * ldA : j * 8 * ldA;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsA, (lds_void*)(slabA + wave * 16 * NI * BK + j * 8 * BK), 16, voff, baseA + soff, 0, 0);
        } else {
            constexpr int j = p - 2 * NI;
            const int voff = TB ? ld_voffB[j % SB::kPeriod] : ld_voffB[j & 1];
            const int soff = TB ? (j / SB::kPeriod) * SB::kPeriodRows * ldB : j * 8 * ldB;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB, (lds_void*)(slabB + wave * 16 * NJ * BK + j * 8 * BK), 16, voff, baseB + soff, 0, 0);
        }
    };
    constexpr int kLoadsPerStep = 2 * (NI + NJ);
    auto issue_loads = [&](uint8_t* slabA, uint8_t* slabB, int step) {
        int baseA, baseB;
        load_base(step, baseA, baseB);
        static_for<kLoadsPerStep>([&](auto piece) { issue_load(slabA, slabB, baseA, baseB, piece); });
    };
    // The wave tile as 16 x 16 blocks: MI x MJ of them, handled in halves of HI block rows / HJ block columns.
    constexpr int MI = 2 * NI, MJ = 2 * NJ, HI = NI, HJ = NJ;
    constexpr int kReadsA = SA::kReadsPerFrag * HI, kReadsB = SB::kReadsPerFrag * HJ;   // LDS reads of one fragment set
    constexpr int kSlots = HI * HJ;                // block updates of one quarter: the slots its side work is spread over
    // T-major operands take twice as many (half as wide) LDS reads: spread over the whole phase they cost
    // nothing, bunched into its first half the both-T-major 4 x 4 kernel measured 4-8 % slower
    constexpr int kDsSpread = (TA || TB) ? 1 : NI * NJ >= 16 ? V::kDsSpread : V::kDsSpreadSmall;

    // ---- LDS -> registers.  The fragment of a 16-row block for v_mfma_f32_16x16x128: lane L holds the 32
    // contiguous bytes [32 (L / 16), 32 (L / 16) + 32) of the K step of operand row L % 16 (two swizzled 16-byte
    // chunks of its LDS row).
    const int fr_row = lane & 15;
    const int fr_q = lane >> 4;                                     // which 32 bytes of the 128-byte K step
    const int swz = row_swizzle(fr_row);                            // same for every row this lane reads
    const int offA = (wr * 32 * NI + fr_row) * BK, offB = (wc * 32 * NJ + fr_row) * BK;
    const int ch0 = ((fr_q * 2) ^ swz) << 4, ch1 = ((fr_q * 2 + 1) ^ swz) << 4;
    // read number p of a fragment set: 16-byte half p % 2 of fragment p / 2
    auto read_piece_rows = [&](const uint8_t* slab, int off, int first_block, auto& f, auto piece) {
        constexpr int p = decltype(piece)::value, i = p >> 1, h = (p & 1) * 4;
        const v4i v = *reinterpret_cast<const v4i*>(slab + off + (first_block + i) * 16 * BK + ((p & 1) ? ch1 : ch0));
        f[i][h] = v[0], f[i][h + 1] = v[1], f[i][h + 2] = v[2], f[i][h + 3] = v[3];
    };
    // T-major: byte offset of this lane's first transposing read of the wave's 16-row block 0: LDS row
    // 32 fr_q + (lane & 15) / 2, 16-byte unit (first unit of the wave) swizzled, half (lane & 1) of the unit; block i
    // is unit + i, read q of a fragment is 8 LDS rows further down.
    const int tm_row = fr_q * 32 + ((lane & 15) >> 1);
    int tm_offA[MI], tm_offB[MJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
        tm_offA[i] = tm_row * BM + (((MI * wr + i) ^ SA::swizzle_of_row(tm_row)) << 4) + ((lane & 1) << 3);
#pragma unroll
    for (int i = 0; i < MJ; ++i)
        tm_offB[i] = tm_row * BN + (((MJ * wc + i) ^ SB::swizzle_of_row(tm_row)) << 4) + ((lane & 1) << 3);
    // read number p of a fragment set: 8-byte quarter p % 4 of fragment p / 4
    auto read_piece_tmajor = [&](const uint8_t* slab, const int* offs, int pitch, auto& f, auto piece) {
        constexpr int p = decltype(piece)::value, i = p >> 2, q = p & 3;
        const v2i r = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i*)(slab + offs[i] + 8 * q * pitch));
        f[i][2 * q] = r[0], f[i][2 * q + 1] = r[1];
    };
    // first_block: 0 or HI / HJ, the half of the wave tile's block rows / columns the set f is for
    auto read_pieceA = [&](uint8_t* slab, auto first_block, auto& f, auto piece) {
        constexpr int kFirst = decltype(first_block)::value;
        if constexpr (TA) read_piece_tmajor(slab, tm_offA + kFirst, BM, f, piece); else read_piece_rows(slab, offA, kFirst, f, piece);
    };
    auto read_pieceB = [&](uint8_t* slab, auto first_block, auto& f, auto piece) {
        constexpr int kFirst = decltype(first_block)::value;
        if constexpr (TB) read_piece_tmajor(slab, tm_offB + kFirst, BN, f, piece); else read_piece_rows(slab, offB, kFirst, f, piece);
    };

    // The accumulators start from a zero the compiler cannot see through: a known constant it would re-create
    // wherever it likes (also by copying one zeroed accumulator register to the next), and the build checks that
    // nothing but MFMAs reads accumulator registers while MFMAs are under way.
    BlockAcc<MI, MJ> acc;
    float zero;
    asm("v_mov_b32 %0, 0" : "=v"(zero));
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < MJ; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc.t[i][j][e] = zero;

    // Fragment sets: the low and high halves of the wave tile's block rows (A) and block columns (B).
    v8i aL[HI], aH[HI], bL[HJ], bH[HJ];

    // L2 touch loads: a wave reads the first dword of some rows of a slab that is still touch_ahead
    // steps ahead of the direct-to-LDS loads (touch_ahead <= 0: nothing is fetched).  The CUs of an XCD
    // start their tiles together and walk K at about the same pace, so without this every slab is first
    // requested only ~1.5 steps before it is needed, less than a miss to HBM takes when the operands are
    // not in the last-level cache.
    // The workgroups that run side by side on an XCD (band_rows tile rows x the tile columns that fit) share
    // each slab: a workgroup touches the lines [g * n / share, (g + 1) * n / share) of the n lines of its A slab,
    // g = tile column mod share_a, and likewise of its B slab with the tile row and share_b (the host picks the
    // shares); each wave takes a quarter of that.
    constexpr bool kTouch = V::kTouch;
    // (T-major operand: the slab is 128 memory rows of kLines lines each, shared out the same way.)
    constexpr int kLinesOfA = TA ? BK * SA::kLines : BM, kLinesOfB = TB ? BK * SB::kLines : BN;
    const int per_wave_a = (kLinesOfA + share_a * 4 - 1) / (share_a * 4), per_wave_b = (kLinesOfB + share_b * 4 - 1) / (share_b * 4);
    const int touch_lineA = ((tc % share_a) * 4 + wave) * per_wave_a + lane, touch_lineB = ((tr % share_b) * 4 + wave) * per_wave_b + lane;
    const int touch_voffA = (lane >= per_wave_a || touch_lineA >= kLinesOfA) ? kOutOfRange
                            : TA ? (touch_lineA / SA::kLines) * ldA + (touch_lineA % SA::kLines) * 128 : touch_lineA * ldA;
    const int touch_voffB = (lane >= per_wave_b || touch_lineB >= kLinesOfB) ? kOutOfRange
                            : TB ? (touch_lineB / SB::kLines) * ldB + (touch_lineB % SB::kLines) * 128 : touch_lineB * ldB;
    int touchA[2] = {0, 0}, touchB[2] = {0, 0};   // results are only kept so that the loads stay tracked
    int touch_sink = 0;

    // The side work of slot m of a quarter: its share of the LDS reads of a fragment set, spread evenly over the
    // first kSlots / kDsSpread slots so that they have landed when the quarter ends, and its share of the step's
    // direct-to-LDS loads, spread over the third quarter or (kLoadQuarters = 2) the third and fourth.  Of n pieces
    // spread over `span` slots, slot m takes the pieces [ceil(m n / span), ceil((m + 1) n / span)).
    constexpr int kDsSpan = (kSlots + kDsSpread - 1) / kDsSpread;
    constexpr int kVmSpan = kSlots * V::kLoadQuarters;
    auto pieces_of_slot = [&](auto n_pieces, auto span, auto m, auto&& issue) {
        constexpr int n = decltype(n_pieces)::value, sp = decltype(span)::value, mm = decltype(m)::value;
        constexpr int first = (mm * n + sp - 1) / sp, last = ((mm + 1) * n + sp - 1) / sp;
        static_for<(last < n ? last : n) - (first < n ? first : n)>([&](auto u) { issue(IntTag<first + decltype(u)::value>{}); });
    };
    auto readsA_of_slot = [&](uint8_t* slab, auto first_block, auto& f, auto m) {
        pieces_of_slot(IntTag<kReadsA>{}, IntTag<kDsSpan>{}, m, [&](auto piece) { read_pieceA(slab, first_block, f, piece); });
    };
    auto readsB_of_slot = [&](uint8_t* slab, auto first_block, auto& f, auto m) {
        pieces_of_slot(IntTag<kReadsB>{}, IntTag<kDsSpan>{}, m, [&](auto piece) { read_pieceB(slab, first_block, f, piece); });
    };
    auto loads_of_slot = [&](uint8_t* slabA, uint8_t* slabB, int baseA, int baseB, auto m) {
        pieces_of_slot(IntTag<kLoadsPerStep>{}, IntTag<kVmSpan>{}, m, [&](auto piece) { issue_load(slabA, slabB, baseA, baseB, piece); });
    };
    auto read_fragsA = [&](uint8_t* slab, auto first_block, auto& f) {
        static_for<kReadsA>([&](auto piece) { read_pieceA(slab, first_block, f, piece); });
    };
    auto read_fragsB = [&](uint8_t* slab, auto first_block, auto& f) {
        static_for<kReadsB>([&](auto piece) { read_pieceB(slab, first_block, f, piece); });
    };

    // One K step on the stage (curA, curB) while the other stage (nxtA, nxtB) is being filled.  The wave tile's
    // MFMAs of the step run as four quarters (half of the block rows x half of the block columns), and each
    // quarter covers the LDS reads of the one fragment set that is free by then.  On entry the sets aX (one half
    // of the block rows: the low one on even steps, the high one on odd steps) and bL hold the current slab:
    //   quarter 0: MFMAs (aX, bL) | read aY of the current slab
    //   quarter 1: MFMAs (aY, bL) | read bH of the current slab
    //   barrier  : the next slab has landed, everybody is done reading the current one
    //   quarter 2: MFMAs (aY, bH) | start loading slab kt+2 into the current stage, read bL of the next slab
    //   quarter 3: MFMAs (aX, bH) | read aY of the next slab, which is the next step's aX
    // Loads that would start beyond the last slab are pointed outside the buffer range instead:
    // the hardware then fetches nothing (LDS receives zeros), and that stage is never used.
    auto k_step = [&](uint8_t* curA, uint8_t* curB, uint8_t* nxtA, uint8_t* nxtB, int kt, int parity, auto x_is_high) {
        constexpr bool XH = decltype(x_is_high)::value;
        constexpr int X0 = XH ? HI : 0, Y0 = XH ? 0 : HI;
        auto& aX = *(XH ? &aH : &aL);
        auto& aY = *(XH ? &aL : &aH);
        mma_quadrant<FA, FB, X0, 0, false>(acc, aX, bL, [&](auto m) { readsA_of_slot(curA, IntTag<Y0>{}, aY, m); });
        mma_quadrant<FA, FB, Y0, 0, false>(acc, aY, bL, [&](auto m) { readsB_of_slot(curB, IntTag<HJ>{}, bH, m); });
        // the direct-to-LDS loads of the previous step must have landed; its two touch loads, issued
        // after them, may still be in flight
        if constexpr (kTouch) wait_vmcnt<2>(); else wait_vmcnt<0>();
        lds_barrier();
        __builtin_amdgcn_sched_barrier(0);
        int baseA, baseB;
        load_base(kt + 2 < nk ? kb + kt + 2 : -1, baseA, baseB);
        mma_quadrant<FA, FB, Y0, HJ, true>(acc, aY, bH, [&](auto m) {
            readsB_of_slot(nxtB, IntTag<0>{}, bL, m);     // past the last slab this reads bytes that are never used
            loads_of_slot(curA, curB, baseA, baseB, m);
        });
        mma_quadrant<FA, FB, X0, HJ, false>(acc, aX, bH, [&](auto m) {
            readsA_of_slot(nxtA, IntTag<Y0>{}, aY, m);
            loads_of_slot(curA, curB, baseA, baseB, IntTag<kSlots + decltype(m)::value>{});
        });
        if constexpr (kTouch) {
            const int kp = kt + 2 + touch_ahead;
            const bool on = touch_ahead > 0 && kp < nk;
            touch_sink ^= touchA[parity] ^ touchB[parity];          // issued two steps ago: long landed
            touchA[parity] = __builtin_amdgcn_raw_buffer_load_b32(rsA, touch_voffA, on ? (kb + kp) * ksA : kOutOfRange, 0);
            touchB[parity] = __builtin_amdgcn_raw_buffer_load_b32(rsB, touch_voffB, on ? (kb + kp) * ksB : kOutOfRange, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    if constexpr (!fixup) {
    // both stages are requested at once; only the first has to have landed before the first fragments
    issue_loads(ldsA0, ldsB0, kb);
    issue_loads(ldsA1, ldsB1, nk > 1 ? kb + 1 : -1);
    if constexpr (kTouch) {                       // keep "two touch loads are the newest" true from the start
        const bool on = touch_ahead > 0 && 2 < nk;
        touchA[1] = __builtin_amdgcn_raw_buffer_load_b32(rsA, touch_voffA, on ? (kb + 2) * ksA : kOutOfRange, 0);
        touchB[1] = __builtin_amdgcn_raw_buffer_load_b32(rsB, touch_voffB, on ? (kb + 2) * ksB : kOutOfRange, 0);
    }
    wait_vmcnt<kLoadsPerStep + (kTouch ? 2 : 0)>();
    lds_barrier();
    read_fragsA(ldsA0, IntTag<0>{}, aL);
    read_fragsB(ldsB0, IntTag<0>{}, bL);
    stamp(1);
    int kt = 0;
    for (; kt + 1 < nk; kt += 2) {
        k_step(ldsA0, ldsB0, ldsA1, ldsB1, kt, 0, BoolTag<false>{});
        k_step(ldsA1, ldsB1, ldsA0, ldsB0, kt + 1, 1, BoolTag<true>{});
    }
    if (kt < nk) k_step(ldsA0, ldsB0, ldsA1, ldsB1, kt, 0, BoolTag<false>{});
    // The last block updates must have left the matrix pipeline before ordinary instructions read the accumulators
    // (the compiler cannot count these wait states for a written-out MFMA).
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    // Every wave waits for its own direct-to-LDS loads (the out-of-range ones of the last two steps
    // still write zeros into the slabs), then all meet: after this barrier nothing lands in LDS any
    // more and nobody reads the slabs, so the epilogue may reuse them.
    wait_vmcnt<0>();
    lds_barrier();
    if constexpr (kTouch) {
        touch_sink ^= touchA[0] ^ touchB[0] ^ touchA[1] ^ touchB[1];
        asm volatile("" ::"v"(touch_sink));
    }
    stamp(2);
    } else {
        // Fix-up launch: the accumulators are the sums of the pieces the sharing workgroups left, added in the
        // order of their K ranges; two rows of 16 x 16 blocks at a time (4 NJ loads of 16 bytes in flight per lane:
        // the launch has one workgroup per shared tile and is bound by the latency of these loads).
        constexpr int kTileFloats = BM * BN;
        for (int c = 0; c < nk; ++c) {
            const v4f* src = reinterpret_cast<const v4f*>(plan.partials + (size_t)(slot + c) * kTileFloats);
#pragma unroll
            for (int i = 0; i < MI; i += 2) {
                v4f v[2][MJ];
#pragma unroll
                for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                    for (int j = 0; j < MJ; ++j) v[ii][j] = __builtin_nontemporal_load(src + ((i + ii) * MJ + j) * kGemmThreads + threadIdx.x);
#pragma unroll
                for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                    for (int j = 0; j < MJ; ++j) {
                        v4f c = acc.get(i + ii, j);
#pragma unroll
                        for (int e = 0; e < 4; ++e) c[e] += v[ii][j][e];
                        acc.set(i + ii, j, c);
                    }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    if constexpr (MODE == kSharePieces) {
        // a piece of a shared tile: the accumulators as they are, 16 bytes per lane and store, 4 KB per store
        // of the workgroup; the fix-up launch reads them back in the same arrangement
        // (uniform base + lane index per store: one address register pair instead of one per store)
        v4f* dst = reinterpret_cast<v4f*>(plan.partials + (size_t)slot * (BM * BN));
#pragma unroll
        for (int i = 0; i < MI; ++i) {
#pragma unroll
            for (int j = 0; j < MJ; ++j) (dst + (i * MJ + j) * kGemmThreads)[threadIdx.x] = acc.get(i, j);
            if ((i & 1) == 1) __builtin_amdgcn_sched_barrier(0);
        }
        return;
    }
    // The workgroup that follows on this XCD (id + next_stride: same XCD, and dispatched about when this
    // one retires) starts with two slabs of its own operands; one dword per 128-byte line of them is
    // requested here, so that they reach the L2 while this workgroup is busy with its epilogue.
    int next_touch[4] = {0, 0, 0, 0};
    if constexpr (kTouch) {
        int ntr, ntc;
        // (plain kernel only: the workgroups that share tiles have no such successor)
        const int next_pid = (int)blockIdx.x + next_stride;
        const int next_pos = (!SPLIT && next_stride > 0 && T >= 2 * BK) ? walk_position(next_pid, plan.n_whole) : -1;
        if (next_pos >= 0) {
            tile_of_position(next_pos, tiles_r, tiles_c, band_rows, ntr, ntc);
            if constexpr (TA) {                   // memory rows 0 .. 255, one per thread, kLines lines each
                const uint8_t* na = A + (size_t)threadIdx.x * ldA + (size_t)ntr * BM;
                next_touch[0] = *reinterpret_cast<const int*>(na);
                if (SA::kLines > 1) next_touch[1] = *reinterpret_cast<const int*>(na + 128);
            } else {
                const uint8_t* na = A + ((size_t)ntr * BM + wave * (BM / 4) + lane) * ldA;
                if (lane < BM / 4) {
                    next_touch[0] = *reinterpret_cast<const int*>(na);
                    next_touch[1] = *reinterpret_cast<const int*>(na + ksA);
                }
            }
            if constexpr (TB) {
                const uint8_t* nb = B + (size_t)threadIdx.x * ldB + (size_t)ntc * BN;
                next_touch[2] = *reinterpret_cast<const int*>(nb);
                if (SB::kLines > 1) next_touch[3] = *reinterpret_cast<const int*>(nb + 128);
            } else {
                const uint8_t* nb = B + ((size_t)ntc * BN + wave * (BN / 4) + lane) * ldB;
                if (lane < BN / 4) {
                    next_touch[2] = *reinterpret_cast<const int*>(nb);
                    next_touch[3] = *reinterpret_cast<const int*>(nb + ksB);
                }
            }
        }
    }

    // ---- epilogue.  Per 16 x 16 block a lane holds 4 consecutive columns of row (lane % 16).
    // Storing those 8-byte pieces directly scatters every store over 16 rows; instead each wave
    // stages 32 rows of its quadrant at a time (32 rows x 32 NJ BF16 columns) at the start of one
    // of the four slabs, which nobody reads any more, and writes it out as full row segments, 16 bytes per lane.  The
    // 16-byte slot index of a staged row is rotated by the row number, so that the 8-byte writes of
    // 32 rows and the 16-byte reads spread over the banks.  The region is private to the wave and LDS
    // executes a wave's accesses in order, so no further barrier is needed.
    // De-scale with one multiply by 1 / (sA sB) unless that product leaves the normal range (degenerate
    // scales such as FLT_MAX for an all-zero tensor), in which case the two factors are applied in turn
    // (a second copy of the epilogue, so that the usual path carries no trace of it).
    const float inv_a = 1.0f / scale_a, inv_b = 1.0f / scale_b;
    const float inv_ab = inv_a * inv_b;
    const bool one_mul = inv_ab >= 1.17549435e-38f && inv_ab <= 3.402823466e+38f;
    const float m1 = one_mul ? inv_ab : inv_a;
    // The output absmax is taken in fp32 before rounding: rounding to BF16 is monotonic, so the BF16
    // rounding of the largest |y| is the largest rounded magnitude.  The maximum is the IEEE 754-2019 one
    // (v_maximum3_f32, two elements per instruction): a NaN output makes the absmax NaN, as it does for the
    // absmax kernel run over the stored tensor.
    float maxabs = 0.0f;
    auto track4 = [&](const v4f& y) {
        if constexpr (V::kIeeeMaximum) {
            maxabs = __builtin_elementwise_maximum(__builtin_elementwise_maximum(maxabs, __builtin_fabsf(y[0])), __builtin_fabsf(y[1]));
            maxabs = __builtin_elementwise_maximum(__builtin_elementwise_maximum(maxabs, __builtin_fabsf(y[2])), __builtin_fabsf(y[3]));
        } else {
            maxabs = __builtin_fmaxf(__builtin_fmaxf(maxabs, __builtin_fabsf(y[0])), __builtin_fabsf(y[1]));
            maxabs = __builtin_fmaxf(__builtin_fmaxf(maxabs, __builtin_fabsf(y[2])), __builtin_fabsf(y[3]));
        }
    };
    // The body exists twice, for one and for two de-scale multiplies; the choice is uniform over the grid.
    // A lane holds, of the 16 x 16 block (i, j), the four consecutive columns 16 j + 4 (lane / 16) .. of row
    // 16 i + lane % 16.
    auto write_out = [&](auto two_mul) {
    auto descale4 = [&](const v4f& block) -> v4f {
        v4f y;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            y[e] = block[e] * m1;
            if constexpr (decltype(two_mul)::value) y[e] *= inv_b;
        }
        return y;
    };
    if constexpr (!ACCUM) {
        constexpr int kSlots = 4 * NJ;                                       // 16-byte slots per staged row
        constexpr int kPitch = 16 * kSlots;
        uint8_t* stage = wave == 0 ? ldsA0 : wave == 1 ? ldsB0 : wave == 2 ? ldsA1 : ldsB1;
        // 8 bytes per block: columns 16 j + 4 fr_q .. are slot 2 j + fr_q / 2 of the staged row, half fr_q % 2
        const int slot0 = fr_q >> 1, half_off = (fr_q & 1) << 3;
        uint16_t* cbase = C + (size_t)(tr * BM + wr * 32 * NI) * Cn + tc * BN + wc * 32 * NJ;
        constexpr int kBlockPieces = 32 * kSlots;                            // 16-byte pieces of 32 staged rows
        // 32 rows (two rows of blocks) at a time: while their stores are in flight the next ones are converted
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            if constexpr (V::kEpilogueFence) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ii = 0; ii < 2; ++ii) {
                const int row = 16 * ii + fr_row;     // the 32 staged rows are reused every time: LDS runs a wave's accesses in order
                uint8_t* srow = stage + row * kPitch;
#pragma unroll
                for (int j = 0; j < MJ; ++j) {
                    const v4f y = descale4(acc.get(2 * i + ii, j));
                    track4(y);
                    bf16x4 o = __builtin_convertvector(y, bf16x4);
                    const int off = (((2 * j + slot0 + row) % kSlots) << 4) | half_off;
                    *reinterpret_cast<bf16x4*>(srow + off) = o;
                }
            }
            // all pieces of the 32 rows are read back before the first is stored, so that the LDS round
            // trips overlap instead of each store waiting for its own read
            constexpr int kPiecesPerLane = kBlockPieces / kWave;
            v4u piece[kPiecesPerLane];
#pragma unroll
            for (int k = 0; k < kPiecesPerLane; ++k) {
                const int p = lane + k * kWave;
                const int r = p / kSlots, sl = p % kSlots;
                piece[k] = *reinterpret_cast<const v4u*>(stage + r * kPitch + (((sl + r) % kSlots) << 4));
            }
            if constexpr (V::kEpilogueFence) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < kPiecesPerLane; ++k) {
                const int p = lane + k * kWave;
                const int r = i * 32 + p / kSlots, sl = p % kSlots;      // row inside the wave's quadrant
                if constexpr (V::kNtStoreC) __builtin_nontemporal_store(piece[k], reinterpret_cast<v4u*>(cbase + (size_t)r * Cn + sl * 8));
                else *reinterpret_cast<v4u*>(cbase + (size_t)r * Cn + sl * 8) = piece[k];
            }
        }
        if constexpr (V::kProfile) stamp(4);
    } else {
        // BF16 accumulation: C = bf16(C + y), one rounding, so the old values are needed in binary32 arithmetic
        // before the conversion.  The de-scaled binary32 results take the same way through LDS as the BF16
        // values above (32 rows of the wave's quadrant at a time, 16 bytes per block and lane), so that the old
        // values are loaded, and the sums stored, as full row segments of 16 bytes per lane as well; read and
        // written 8 bytes per lane straight from the accumulator layout (32-byte runs of 16 rows per instruction)
        // this epilogue took 15-20 % of a contraction of 64 K steps.  A staged row holds 4 NJ 16-byte pieces of
        // BF16 output = 8 NJ units of four binary32 values: the first units of all pieces, then the second
        // units; the piece index is rotated by the row number, which keeps the 16-byte writes of 8 rows and the
        // 16-byte reads of 8 neighbouring pieces in different banks.
        constexpr int kSlots = 4 * NJ;                                       // 16-byte pieces of output per row
        constexpr int kPitch = 32 * kSlots;                                  // bytes of a staged binary32 row
        uint8_t* stage = wave == 0 ? ldsA0 : wave == 1 ? ldsB0 : wave == 2 ? ldsA1 : ldsB1;
        static_assert(32 * kPitch <= kSlabA && 32 * kPitch <= kSlabB - 16, "32 staged rows fit the start of any slab");
        uint16_t* cbase = C + (size_t)(tr * BM + wr * 32 * NI) * Cn + tc * BN + wc * 32 * NJ;
        constexpr int kPiecesPerLane = 32 * kSlots / kWave;
        const int piece0 = fr_q >> 1, unit_off = (fr_q & 1) * (16 * kSlots);
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            if constexpr (V::kEpilogueFence) __builtin_amdgcn_sched_barrier(0);
            v4u old[kPiecesPerLane];               // requested first: their way from memory hides behind the staging
#pragma unroll
            for (int k = 0; k < kPiecesPerLane; ++k) {
                const int p = lane + k * kWave;
                const int r = i * 32 + p / kSlots, sl = p % kSlots;
                old[k] = *reinterpret_cast<const v4u*>(cbase + (size_t)r * Cn + sl * 8);
            }
#pragma unroll
            for (int ii = 0; ii < 2; ++ii) {
                const int row = 16 * ii + fr_row;
                uint8_t* srow = stage + row * kPitch + unit_off;
#pragma unroll
                for (int j = 0; j < MJ; ++j)
                    *reinterpret_cast<v4f*>(srow + (((2 * j + piece0 + row) % kSlots) << 4)) = descale4(acc.get(2 * i + ii, j));
            }
            v4f lo[kPiecesPerLane], hi[kPiecesPerLane];
#pragma unroll
            for (int k = 0; k < kPiecesPerLane; ++k) {
                const int p = lane + k * kWave;
                const int r = p / kSlots, sl = p % kSlots;
                const uint8_t* src = stage + r * kPitch + (((sl + r) % kSlots) << 4);
                lo[k] = *reinterpret_cast<const v4f*>(src);
                hi[k] = *reinterpret_cast<const v4f*>(src + 16 * kSlots);
            }
            if constexpr (V::kEpilogueFence) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < kPiecesPerLane; ++k) {
                const int p = lane + k * kWave;
                const int r = i * 32 + p / kSlots, sl = p % kSlots;
                v4f y0 = lo[k], y1 = hi[k];
                y0[0] += __uint_as_float(old[k][0] << 16);
                y0[1] += __uint_as_float(old[k][0] & 0xFFFF0000u);
                y0[2] += __uint_as_float(old[k][1] << 16);
                y0[3] += __uint_as_float(old[k][1] & 0xFFFF0000u);
                y1[0] += __uint_as_float(old[k][2] << 16);
                y1[1] += __uint_as_float(old[k][2] & 0xFFFF0000u);
                y1[2] += __uint_as_float(old[k][3] << 16);
                y1[3] += __uint_as_float(old[k][3] & 0xFFFF0000u);
                track4(y0);
                track4(y1);
                const bf16x4 o0 = __builtin_convertvector(y0, bf16x4), o1 = __builtin_convertvector(y1, bf16x4);
                const v2u w0 = __builtin_bit_cast(v2u, o0), w1 = __builtin_bit_cast(v2u, o1);
                *reinterpret_cast<v4u*>(cbase + (size_t)r * Cn + sl * 8) = v4u{w0[0], w0[1], w1[0], w1[1]};
            }
        }
        if constexpr (V::kProfile) stamp(4);
    }
    };
    if (one_mul) {
        write_out(BoolTag<false>{});
    } else {
        write_out(BoolTag<true>{});
    }
    if constexpr (kTouch) asm volatile("" ::"v"(next_touch[0] ^ next_touch[1] ^ next_touch[2] ^ next_touch[3]));
    unsigned mag = (unsigned)__builtin_bit_cast(uint16_t, (__bf16)maxabs);   // non-negative: magnitude bits
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
        stamp(5);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        stamp(3);
    }
}

// ---- host side: tile choice and launch
struct TileChoice {
    int ni, nj;       // 0, 0: no tuned tile divides the problem, use the generic kernel
};
// scratch_bytes: what the launch may use for the pieces of shared tiles (0: every tile is computed whole)
TileChoice choose_tile(int64_t R, int64_t C, int64_t T, int num_cus, size_t scratch_bytes);

// Distance of the L2 touch loads in K steps beyond the slab the direct-to-LDS loads are fetching (measured with
// bands 4 high on the block configurations: 1 is 0.5-0.8 % faster than 2, 3 and 4 lose 1.5 % and 4 %);
// LLMQ_GEMM_TOUCH overrides it for tuning.
inline int touch_ahead() {
    if (const char* e = tuning_env("LLMQ_GEMM_TOUCH")) return atoi(e);
    return 1;
}

// Height of the bands of tiles, in tile rows; LLMQ_GEMM_BAND overrides it for tuning.
inline int band_rows() {
    if (const char* e = tuning_env("LLMQ_GEMM_BAND")) { const int v = atoi(e); if (v >= 1 && v <= 64) return v; }
    return kBandRows;
}

// The same for 2 x 2 tiles, where two workgroups share a CU and already cover each other's waits.
inline int touch_ahead_pair() {
    if (const char* e = tuning_env("LLMQ_GEMM_TOUCH_PAIR")) return atoi(e);
    return 0;
}

// Whether a workgroup requests the first slabs of its successor; LLMQ_GEMM_TOUCH_NEXT=0 / 1 overrides it.
inline bool touch_next(bool by_default) {
    if (const char* e = tuning_env("LLMQ_GEMM_TOUCH_NEXT")) return atoi(e) != 0;
    return by_default;
}

// Workgroups of the tile kernel resident on the chip at once (a multiple of the XCD count);
// LLMQ_GEMM_SLOTS overrides it for tests, so that small problems meet the many-rounds code paths.
inline int resident_slots(int num_cus, int ni, int nj) {
    if (const char* e = tuning_env("LLMQ_GEMM_SLOTS")) { const int v = atoi(e); if (v >= kXcds && v % kXcds == 0) return v; }
    return (num_cus / kXcds) * kXcds * ((ni == 2 && nj == 2) ? 2 : 1);
}

// The tile shape whose kernels exist in the tile-sharing form (for contraction-contiguous operands only): the
// largest one, which is what problems big enough to have a ragged last round worth sharing get.
constexpr bool split_supported(int ni, int nj) { return ni == 4 && nj == 4; }

// How a problem of nt tiles x nk K steps is shared out (see SplitPlan), and what it is expected to cost.
struct SplitChoice {
    int n_whole;             // tiles computed whole by the leading workgroups
    int n_groups;            // 0: nothing is shared
    SplitGroup group[kMaxSplitGroups];
    int shared_tiles;        // tiles in the groups
    int share_wgs;           // workgroups of the groups (padded)
    size_t slots;            // binary32 tiles of scratch the launch may write (0: nothing is shared)
    double cost_us;          // model time of the whole launch
    double whole_cost_us;    // the same with every tile computed whole
};

// The r tiles of a ragged last round are served in groups: as long as at least half the chip's worth of tiles is
// left, half a chip's worth is cut in two; what is left below that is cut into as many pieces as fill the chip
// once (r = 192 on 256 CUs: 128 tiles in halves, 64 in quarters).  cost_us is a rough time model in microseconds
// (~1.25 us per K step of a 256 x 256 tile, ~7 us of prologue + epilogue per tile or piece, ~4 TB/s for the
// partial results written and read back, ~4 us for the extra launches); it only scales the tile choice.
// Whether sharing is used at all is decided by what was measured on the chip, which is power-limited on real
// data: CUs left idle by a ragged round let the busy ones clock higher, so a round a fifth to a half full costs
// 0.4-0.9 of a full one, while the pieces launch costs its K steps + ~30 us and the fix-up launch 45-70 us.
// Sharing wins 1-13 % of the GEMM for contractions of 64 K steps or more (T >= 8192) with all left-over tiles in
// one group (pieces of 8 K steps at least); it loses 4-30 % on shorter contractions and with several groups.
inline SplitChoice choose_split(int nt, int nk, int slots, int ni, int nj, size_t scratch_bytes) {
    const double unit = 1.25 * ni * nj / 16.0, ovh = 7.0;
    const double tile_f32 = 4.0 * 4096 * ni * nj, tile_out = 2.0 * 4096 * ni * nj;
    const int rounds = (nt + slots - 1) / slots;
    SplitChoice whole{};
    whole.n_whole = nt;
    whole.cost_us = whole.whole_cost_us = rounds * (nk * unit + ovh);
    const int full = nt / slots, r = nt - full * slots;
    const char* force = tuning_env("LLMQ_GEMM_SPLIT");
    if (r == 0 || nk < 2 || !split_supported(ni, nj) || (force && force[0] == '0')) return whole;
    int min_steps = 8;                             // shorter pieces are all overhead
    int forced_pieces = 0;                         // tests: LLMQ_GEMM_SPLIT=a<n> cuts every left-over tile into n pieces
    if (force && force[0] == 'a') { forced_pieces = atoi(force + 1); min_steps = 1; }
    SplitChoice c{};
    c.n_whole = full * slots;
    c.whole_cost_us = whole.whole_cost_us;
    c.cost_us = full * (nk * unit + ovh);
    int left = r, tile_at = 0, wg_at = 0;
    double pieces_total = 0;
    while (left > 0 && c.n_groups < kMaxSplitGroups) {
        int pieces = forced_pieces > 0 ? forced_pieces : left * 2 >= slots ? 2 : slots / left;
        if (pieces > nk / min_steps) pieces = nk / min_steps;
        if (pieces < 1) pieces = 1;
        if (c.n_groups == kMaxSplitGroups - 1 && forced_pieces == 0 && pieces * left > slots) pieces = 1;   // last group takes all that is left
        int tiles = pieces > 1 ? slots / pieces : left;
        if (tiles > left) tiles = left;
        if (tiles < 1) { tiles = left; pieces = 1; }
        const int steps = (nk + pieces - 1) / pieces;
        pieces = (nk + steps - 1) / steps;         // no empty last piece
        SplitGroup& g = c.group[c.n_groups++];
        g.tile_begin = tile_at; g.tiles = tiles; g.pieces = pieces; g.steps = steps; g.wg_begin = wg_at;
        g.wgs = ((tiles * pieces + kXcds - 1) / kXcds) * kXcds;
        tile_at += tiles; wg_at += g.wgs; left -= tiles;
        c.cost_us += ((tiles * pieces + slots - 1) / slots) * (steps * unit + ovh);
        if (pieces > 1) pieces_total += (double)tiles * pieces;
    }
    if (left > 0) return whole;                    // does not fit the groups
    c.shared_tiles = r;
    c.share_wgs = wg_at;
    c.slots = (size_t)wg_at;
    if (pieces_total == 0) return whole;
    c.cost_us += 4.0 + (2.0 * pieces_total * tile_f32 + r * tile_out) / 4.0e6;
    if ((double)c.slots * tile_f32 > (double)scratch_bytes) return whole;
    // LLMQ_GEMM_SPLIT=1 or a<n>: whenever possible; otherwise only where it was measured to win
    if (!force && !(nk >= 64 && c.n_groups == 1)) return whole;
    if (c.cost_us > whole.cost_us) c.cost_us = whole.cost_us;
    return c;
}

template <int FA, int FB, int NI, int NJ, bool TA = false, bool TB = false>
static void launch_tile(const uint8_t* A, const uint8_t* B, int64_t R, int64_t C, int64_t T,
                        const float* sA, const float* sB, void* c, int accumulate, unsigned* amax,
                        hipStream_t stream, int num_cus, GemmScratch scratch, bool slabs_a, bool slabs_b) {
    // row pitch and K-step stride of the operands (OperandLayout)
    const int ldA = TA ? (int)R : slabs_a ? BK : (int)T, ldB = TB ? (int)C : slabs_b ? BK : (int)T;
    const int ksA = slabs_a ? (int)(R * BK) : BK, ksB = slabs_b ? (int)(C * BK) : BK;
    const int tiles_r = (int)(R / (64 * NI)), tiles_c = (int)(C / (64 * NJ));
    const int nt = tiles_r * tiles_c;
    const int touch = (NI == 2 && NJ == 2) ? touch_ahead_pair() : touch_ahead();
    // workgroups resident on the chip at once: the distance to the workgroup that takes over a slot
    // (measured: +3 % on a GEMM of 19 rounds of tiles, whose later workgroups otherwise start on cold
    // operands; nothing or slightly less on GEMMs of 2-4 rounds, so it is used from 6 rounds on)
    const int slots = resident_slots(num_cus, NI, NJ);
    const SplitChoice sc = choose_split(nt, (int)(T / BK), slots, NI, NJ, (scratch.ptr && !TA && !TB && FA != kFmtBf16) ? scratch.bytes : 0);
    SplitPlan plan{};
    plan.n_whole = sc.n_whole;
    plan.n_groups = sc.n_groups;
    for (int g = 0; g < sc.n_groups; ++g) plan.group[g] = sc.group[g];
    plan.partials = scratch.ptr;
    const int grid = ((sc.n_whole + kXcds - 1) / kXcds) * kXcds;        // of the plain kernel
    // Touch shares (LLMQ_GEMM_SHARE_A / _B override them): the band_rows tile rows that run side by side on an
    // XCD cover a B slab together, each a different part.  Of the tile columns side by side (the XCD's workgroups
    // / band_rows: 8 at band height 4) four cover an A slab together, so every A line is requested by two
    // workgroups: they are not in lock step, and a line that only a straggler would request comes late.
    const int band = band_rows();
    int share_b = band < tiles_r ? band : tiles_r;
    int share_a = 4 < tiles_c ? 4 : tiles_c;
    if (const char* e = tuning_env("LLMQ_GEMM_SHARE_A")) { const int v = atoi(e); if (v >= 1 && v <= 64) share_a = v; }
    if (const char* e = tuning_env("LLMQ_GEMM_SHARE_B")) { const int v = atoi(e); if (v >= 1 && v <= 64) share_b = v; }
    const int next_stride = touch_next(nt >= 6 * slots) ? slots : 0;
    auto launch = [&](auto kernel, int blocks, const SplitPlan& pl) {
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(kGemmThreads), 0, stream,
                           A, B, reinterpret_cast<uint16_t*>(c), (int)C, (int)T, sA, sB, amax, tiles_r, tiles_c,
                           touch, band, next_stride, ldA, ldB, ksA, ksB, share_a, share_b, pl);
    };
    // The pieces first (all CUs start and end them together), their sums next, the whole rounds last.
    if constexpr (split_supported(NI, NJ) && FA != kFmtBf16 && !TA && !TB) {
        if (sc.n_groups) {
            launch(gemm_tile_kernel<FA, FB, NI, NJ, false, GemmTuning, TA, TB, kSharePieces>, sc.share_wgs, plan);
            if (accumulate) launch(gemm_tile_kernel<FA, FB, NI, NJ, true, GemmTuning, TA, TB, kShareFixup>, sc.shared_tiles, plan);
            else launch(gemm_tile_kernel<FA, FB, NI, NJ, false, GemmTuning, TA, TB, kShareFixup>, sc.shared_tiles, plan);
        }
    }
    if (sc.n_whole == 0) return;
    if (accumulate) launch(gemm_tile_kernel<FA, FB, NI, NJ, true, GemmTuning, TA, TB>, grid, plan);
    else launch(gemm_tile_kernel<FA, FB, NI, NJ, false, GemmTuning, TA, TB>, grid, plan);
}


// Dispatch on the tile chosen for the problem; false if none divides it.  One translation unit per operand kinds and
// layout instantiates this (gemm_tiles_*.hip: each holds the kernels of all tile shapes for its case, and the files
// compile side by side); everybody else sees the declarations below.
#define LLMQ_TILE_LAUNCH_PARAMS                                                                                   \
    const uint8_t *A, const uint8_t *B, int64_t R, int64_t C, int64_t T, const float *sA, const float *sB, void *c, \
        int accumulate, unsigned *amax, hipStream_t stream, int num_cus, GemmScratch scratch, bool slabs_a, bool slabs_b
template <int FA, int FB, bool TA, bool TB>
bool launch_chosen_tile(LLMQ_TILE_LAUNCH_PARAMS) {
    const TileChoice tc = choose_tile(R, C, T, num_cus, (scratch.ptr && !TA && !TB && FA != kFmtBf16) ? scratch.bytes : 0);
#define LLMQ_TILE_CASE(I, J)                                                                              \
    case I * 8 + J:                                                                                       \
        launch_tile<FA, FB, I, J, TA, TB>(A, B, R, C, T, sA, sB, c, accumulate, amax, stream, num_cus, scratch, slabs_a, slabs_b); \
        return true;
    switch (tc.ni * 8 + tc.nj) {
        LLMQ_TILE_CASE(4, 4) LLMQ_TILE_CASE(4, 3) LLMQ_TILE_CASE(4, 2)
        LLMQ_TILE_CASE(3, 4) LLMQ_TILE_CASE(3, 3) LLMQ_TILE_CASE(3, 2)
        LLMQ_TILE_CASE(2, 4) LLMQ_TILE_CASE(2, 3) LLMQ_TILE_CASE(2, 2)
        default: break;
    }
#undef LLMQ_TILE_CASE
    return false;
}
// contraction-contiguous operands: every mix of E4M3 and E5M2, and BF16 pairs
extern template bool launch_chosen_tile<0, 0, false, false>(LLMQ_TILE_LAUNCH_PARAMS);
extern template bool launch_chosen_tile<1, 0, false, false>(LLMQ_TILE_LAUNCH_PARAMS);
extern template bool launch_chosen_tile<0, 1, false, false>(LLMQ_TILE_LAUNCH_PARAMS);
extern template bool launch_chosen_tile<1, 1, false, false>(LLMQ_TILE_LAUNCH_PARAMS);
extern template bool launch_chosen_tile<kFmtBf16, kFmtBf16, false, false>(LLMQ_TILE_LAUNCH_PARAMS);
// T-major operands: B is E4M3 (weights and activations), A either format
extern template bool launch_chosen_tile<0, 0, true, true>(LLMQ_TILE_LAUNCH_PARAMS);
extern template bool launch_chosen_tile<0, 0, false, true>(LLMQ_TILE_LAUNCH_PARAMS);
extern template bool launch_chosen_tile<0, 0, true, false>(LLMQ_TILE_LAUNCH_PARAMS);
extern template bool launch_chosen_tile<1, 0, true, true>(LLMQ_TILE_LAUNCH_PARAMS);
extern template bool launch_chosen_tile<1, 0, false, true>(LLMQ_TILE_LAUNCH_PARAMS);
extern template bool launch_chosen_tile<1, 0, true, false>(LLMQ_TILE_LAUNCH_PARAMS);

}  // namespace llmq
