// LDS-tiled MFMA GEMMs for gfx950: INT8, packed INT4 (widened to INT8 in registers) and the
// bf16 baseline from one kernel template, and the 4-bit GEMM on the 6-bit matrix pipe (operands
// stored as E3M2 codes; its own kernels and layout, described where they are defined).
//
// arXiv 2402.17985 Sec. 5.1: the quantized linear layer is an INT8 / INT4 GEMM with int32
// accumulation whose result is scaled back by s_x * s_w (the inverse of Eq. 1); Table 5 compares
// it with a 16-bit floating-point GEMM of the same shape.
//
// Both operands are K-contiguous ("NT" product):  C[i,n] = sum_k A[i,k] * B[n,k].
// Everything is expressed in 16-byte chunks of a row, which is exactly one lane's MFMA operand:
//   INT8  v_mfma_i32_32x32x32_i8     a chunk = 16 k-values
//   INT4  same instruction; a chunk = 32 packed nibbles, split in registers into the 16 low and
//         the 16 high nibbles, each moved to the top of its byte (value * 16), two MFMAs per
//         chunk; the accumulator then holds 256 * sum and is shifted right by 8 (exact)
//   BF16  v_mfma_f32_32x32x16_bf16   a chunk = 8 k-values
// The instruction's lane->k assignment is the same for its A and B operands, and a dot product
// does not depend on the order of its terms, so lane l simply takes chunk (l / 32) of the
// 32-byte k-slice for both operands.
//
// Tile: BM x BN outputs per workgroup, BKB bytes of every row per pipeline stage, two LDS stages.
// LDS rows are BKB bytes; the 16-byte chunk index is XOR-swizzled with the row so that the 16
// lanes that read the same chunk column of 16 consecutive rows hit 16 different bank groups.
// Workgroup ids are remapped so that each XCD (ids are dealt round-robin to the 8 XCDs) works on
// a contiguous band of tiles, walked in groups of GROUP_M tile-rows for L2 reuse.
//
// Kernels of the int8 / bf16 family:
//   gemm_dma_kernel   global -> LDS directly (global_load_lds_dwordx4: a wave fills one contiguous
//                     1 KiB block of the stage per instruction, each lane fetching the global chunk
//                     that belongs at its LDS position), stage t+1 in flight while stage t is
//                     multiplied.  Three schedules of the multiply (template parameter PIPE): the
//                     ping-pong of two wave groups (large problems), and two schedules that interleave
//                     the LDS reads of k-slice s+1 with the MFMAs of k-slice s in every wave.  With
//                     the ping-pong schedule one workgroup per CU walks its tiles and fetches the next
//                     tile's first stage while it stores the current one.  Batched products put the
//                     batch index in the grid's y dimension.
//   gemm_wide_kernel  INT8 and bf16: four waves with 128 x 128 wave tiles, reads and copies dealt out
//                     per MFMA slot (default for large bf16 problems).
//   gemm_reg_kernel   global -> registers -> LDS, 128x128 tile; a selectable variant.
// 6-bit pipe: gemm_f6_wide_kernel (four waves with 128 x 128 wave tiles).
// This file is compiled once per operand mode (see the end of the file).
#include <atomic>
#include <type_traits>

#include "fq_internal.h"

namespace fq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v2i __attribute__((ext_vector_type(2)));

enum { MODE_I8 = 0, MODE_I4 = 1, MODE_BF16 = 2, MODE_F6 = 3 };   // F6: 4-bit values stored as 6-bit E3M2 codes

#define FQ_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define FQ_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// Direct global -> LDS copy of 16 bytes per lane (global_load_lds_dwordx4): lane i of the wave
// writes LDS bytes [lds_base + 16 i, +16).  lds_base is wave-uniform and travels in M0.
// Written as inline assembly so that the outstanding-copy count (vmcnt) is managed by the kernel
// itself: several stages stay in flight across barriers, which the compiler's conservative
// "wait for every LDS DMA before any LDS read" rule would forbid.
__device__ __forceinline__ void dma16(const uint8_t* uniform_base, uint32_t lane_offset, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0"
                 :
                 : "s"(uniform_base), "v"(lane_offset), "s"(lds_base)
                 : "memory");
}
__device__ __forceinline__ void dma16_addr(const uint8_t* lane_address, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(lane_address), "s"(lds_base)
                 : "memory");
}

// 16 zero bytes in device memory: the source of DMA lanes that fall beyond the end of a row.
__device__ const int g_zero_chunk[4] = {0, 0, 0, 0};

// Clock probe (measurement hook): with a non-null counter pair, the first wave of the workgroup adds the shader-clock
// and the constant-rate ticks between construction and finish().  Both reads are scalar instructions.
struct ClockProbe {
    unsigned long long t0, r0;
    __device__ __forceinline__ explicit ClockProbe(const unsigned long long* ticks)
    {
        t0 = r0 = 0;
        if (ticks) {
            t0 = __builtin_amdgcn_s_memtime();
            r0 = __builtin_amdgcn_s_memrealtime();
        }
    }
    __device__ __forceinline__ void finish(unsigned long long* ticks) const
    {
        if (ticks) {
            const unsigned long long t1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
            if (threadIdx.x == 0) {
                atomicAdd(&ticks[0], t1 - t0);
                atomicAdd(&ticks[1], r1 - r0);
            }
        }
    }
};

template <int MODE> struct Acc { typedef v16i type; };
template <> struct Acc<MODE_BF16> { typedef v16f type; };
template <> struct Acc<MODE_F6> { typedef v16f type; };      // exact integers below 2^24 held in fp32

__device__ __forceinline__ void tile_of_logical(int logical, int tiles_m, int tiles_n, int& tile_m, int& tile_n);

// Workgroup id -> output tile.  Ids are dealt round-robin to the 8 XCDs; each XCD gets a contiguous
// band of the logical tile sequence, which walks GROUP_M tile-rows at a time.
__device__ __forceinline__ void tile_of_workgroup(int wg, int nwg, int tiles_m, int tiles_n, int& tile_m,
                                                  int& tile_n)
{
    const int q = nwg >> 3, rem = nwg & 7;
    const int xcd = wg & 7, idx = wg >> 3;
    const int logical = (xcd < rem) ? xcd * (q + 1) + idx : rem * (q + 1) + (xcd - rem) * q + idx;
    tile_of_logical(logical, tiles_m, tiles_n, tile_m, tile_n);
}
__device__ __forceinline__ void tile_of_logical(int logical, int tiles_m, int tiles_n, int& tile_m, int& tile_n)
{
    constexpr int GROUP_M = 8;     // 2, 4, 16, 32 measured 1-7 % slower on the 6-bit kernel
    const int group = GROUP_M * tiles_n;
    const int gidx = logical / group;
    const int first_m = gidx * GROUP_M;
    const int gsz = min(tiles_m - first_m, GROUP_M);
    const int in_group = logical - gidx * group;
    tile_m = first_m + in_group % gsz;
    tile_n = in_group / gsz;
}

// Epilogue of one wave.  The MFMAs are issued with the W fragment as the first operand and the X
// fragment as the second, so in the 32x32 accumulator block (i, j) lane l holds output row
// 32 i + l%32 and, in registers 4g..4g+3, the four consecutive output columns
// 32 j + 8 g + 4 (l/32) + 0..3: they are scaled, converted and written as one 8- or 16-byte store.
template <int YDT> struct OutVec;
template <> struct OutVec<FQ_I32> { typedef int type __attribute__((ext_vector_type(4))); };
template <> struct OutVec<FQ_F32> { typedef float type __attribute__((ext_vector_type(4))); };
template <> struct OutVec<FQ_F16> { typedef _Float16 type __attribute__((ext_vector_type(4))); };
template <> struct OutVec<FQ_BF16> { typedef __bf16 type __attribute__((ext_vector_type(4))); };

// fp32 -> half of a value that has already been rounded to fp32.  The empty asm keeps the compiler from folding
// the preceding fp32 multiply (or bias add) into a mixed-precision instruction that rounds the exact product only
// once, straight to half: the interface defines the output as the fp32 result rounded again to the output type.
__device__ __forceinline__ _Float16 half_of_rounded_fp32(float f)
{
    asm("" : "+v"(f));
    return (_Float16)f;
}

// One output element: the accumulator scaled by s_x * s_w, plus (optionally) the column's bias, both
// in fp32 as two separately rounded operations, then rounded to the output type.
template <int MODE, int YDT> __device__ __forceinline__ auto convert_out(typename Acc<MODE>::type const& acc, int r, float scale,
                                                                         bool has_bias = false, float b = 0.0f)
{
    if constexpr (MODE == MODE_BF16) {
        return (__bf16)acc[r];
    } else if constexpr (MODE == MODE_F6) {
        // the fp32 accumulator holds the integer result exactly (|acc| < 2^24): it is fl32(acc) already
        if constexpr (YDT == FQ_I32) {
            return (int)acc[r];
        } else {
            float f = acc[r] * scale;
            if (has_bias) f += b;
            if constexpr (YDT == FQ_F32) return f;
            else if constexpr (YDT == FQ_BF16) return (__bf16)f;
            else return half_of_rounded_fp32(f);
        }
    } else {
        int v = acc[r];
        if (MODE == MODE_I4) v >>= 8;
        if constexpr (YDT == FQ_I32) {
            return v;
        } else {
            float f = (float)v * scale;
            if (has_bias) f += b;
            if constexpr (YDT == FQ_F32) return f;
            else if constexpr (YDT == FQ_BF16) return (__bf16)f;
            else return half_of_rounded_fp32(f);
        }
    }
}

// The lane index as the epilogue sees it: an opaque copy, so that the per-lane addresses of the epilogue are computed
// after the main loop.  Derived from the plain lane index they are loop invariants the compiler computes at kernel
// start and keeps live across the main loop, where every register is taken: they were spilled, and their reloads
// (vector memory operations, waited for with vmcnt) had each tile's epilogue wait for everything in flight.
__device__ __forceinline__ int epilogue_lane()
{
    int lane = threadIdx.x & 63;
    asm volatile("" : "+v"(lane));
    return lane;
}

// The four bias values of the columns col .. col + 3 (zeros when there is no bias).
__device__ __forceinline__ v4f bias4(const float* __restrict__ bias, int col)
{
    v4f b = {0.0f, 0.0f, 0.0f, 0.0f};
    if (bias) b = *reinterpret_cast<const v4f*>(bias + col);
    return b;
}

template <int MODE, int YDT, int FM, int FN, bool hb = false, typename acc_t>
__device__ __forceinline__ void store_tile_as(acc_t (&acc)[FM][FN], int row0, int col0, int M, int N, float scale,
                                              void* __restrict__ Y, int ldy, bool fast,
                                              const float* __restrict__ bias = nullptr)
{
    typedef typename OutVec<YDT>::type vec_t;
    typedef decltype(convert_out<MODE, YDT>(acc[0][0], 0, scale)) elem_t;
    const int lane = epilogue_lane();
    const int frow = lane & 31, fhalf = lane >> 5;
    elem_t* Yt = static_cast<elem_t*>(Y);
    if (fast) {
        // whole wave tile inside the matrix, rows aligned for vector stores
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            elem_t* yrow = Yt + (size_t)(row0 + i * 32 + frow) * ldy + col0 + 4 * fhalf;
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const v4f b4 = bias4(hb ? bias : nullptr, col0 + 4 * fhalf + j * 32 + 8 * g);
                    vec_t v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = convert_out<MODE, YDT>(acc[i][j], 4 * g + e, scale, hb, b4[e]);
                    *reinterpret_cast<vec_t*>(yrow + j * 32 + 8 * g) = v;
                }
        }
    } else {
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            const int row = row0 + i * 32 + frow;
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int col = col0 + j * 32 + 8 * (r >> 2) + 4 * fhalf + (r & 3);
                    if (row < M && col < N)
                        Yt[(size_t)row * ldy + col] = convert_out<MODE, YDT>(acc[i][j], r, scale, hb, hb ? bias[col] : 0.0f);
                }
        }
    }
}

// 2-byte outputs of an interior tile go through a wave-private LDS staging area so that global
// memory sees full 128-byte row segments: the wave writes its tile as [row][column] (16-byte units
// XOR-swizzled with the row to spread banks), reads it back 16 bytes per lane, and stores 16 bytes
// per lane with 64/UNITS complete rows per instruction.  `stage` must hold FM*32 x FN*32 x 2 bytes.
template <int MODE, int YDT, int FM, int FN, bool hb = false, int CH = FM, typename acc_t>
__device__ __forceinline__ void store_tile_via_lds(acc_t (&acc)[FM][FN], int row0, int col0, float scale,
                                                   void* __restrict__ Y, int ldy, uint8_t* stage,
                                                   const float* __restrict__ bias = nullptr)
{
    // CH = 32-row blocks staged at a time: `stage` holds CH*32 rows and is reused FM/CH times (the
    // LDS operations of one wave execute in order, so a chunk's reads precede the next chunk's writes)
    typedef typename OutVec<YDT>::type vec_t;              // 4 x 2 bytes
    constexpr int ROWB = FN * 32 * 2;                      // bytes per staged row
    constexpr int UNITS = ROWB / 16;
    constexpr int SW = (UNITS >= 8 ? 8 : UNITS) - 1;
    // the swizzle advances once per 256 bytes of staged rows, so that the 8-byte writes of 32 lanes (one
    // row each) spread over all 16-byte units of the 64 banks
    constexpr int SWS = (ROWB >= 256) ? 0 : (ROWB == 128 ? 1 : 2);
    constexpr int ROWS_PER_INSTR = 64 / UNITS;
    static_assert(sizeof(vec_t) == 8 && (CH * 32) % ROWS_PER_INSTR == 0 && FM % CH == 0, "staging layout");
    const int lane = epilogue_lane();
    const int frow = lane & 31, fhalf = lane >> 5;
    uint8_t* Yb = static_cast<uint8_t*>(Y);
    const int mr = lane / UNITS, us = lane % UNITS;
    const bool whole_lines = (ldy & 63) == 0 && (col0 & 63) == 0 && (reinterpret_cast<uintptr_t>(Y) & 127) == 0;
#pragma unroll
    for (int c = 0; c < FM / CH; ++c) {
#pragma unroll
        for (int ic = 0; ic < CH; ++ic) {
            const int i = c * CH + ic;
            const int m = ic * 32 + frow;
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const v4f b4 = bias4(hb ? bias : nullptr, col0 + 4 * fhalf + j * 32 + 8 * g);
                    vec_t v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = convert_out<MODE, YDT>(acc[i][j], 4 * g + e, scale, hb, b4[e]);
                    const int u = g + 4 * j;
                    *reinterpret_cast<vec_t*>(stage + m * ROWB + ((u ^ ((m >> SWS) & SW)) << 4) + 8 * fhalf) = v;
                }
        }
        // The output is written once and not read by this kernel: a streaming store keeps it from
        // displacing the operand panels in L2 -- but only when the 128-byte row segments are whole cache
        // lines; partial-line streaming stores are several times slower than ordinary ones.  (Two loops
        // kept apart: merged, they become one ordinary store.)
        uint8_t* ybase = Yb + ((size_t)(row0 + c * CH * 32) * ldy + col0) * 2;
        if (whole_lines) {
            asm volatile("; streaming stores begin");    // the markers keep the two arms from being merged
#pragma unroll
            for (int t = 0; t < CH * 32 / ROWS_PER_INSTR; ++t) {
                const int m = t * ROWS_PER_INSTR + mr;
                const int u = us ^ ((m >> SWS) & SW);
                const v4i d = *reinterpret_cast<const v4i*>(stage + m * ROWB + (us << 4));
                __builtin_nontemporal_store(d, reinterpret_cast<v4i*>(ybase + (size_t)m * ldy * 2 + (u << 4)));
            }
            asm volatile("; streaming stores end");
        } else {
#pragma unroll
            for (int t = 0; t < CH * 32 / ROWS_PER_INSTR; ++t) {
                const int m = t * ROWS_PER_INSTR + mr;
                const int u = us ^ ((m >> SWS) & SW);
                const v4i d = *reinterpret_cast<const v4i*>(stage + m * ROWB + (us << 4));
                *reinterpret_cast<v4i*>(ybase + (size_t)m * ldy * 2 + (u << 4)) = d;
            }
        }
    }
}

// The product of the two per-tensor scales, read at the start of a tile so that the epilogue does not wait for two
// scalar loads (raw accumulator output passes null pointers: no scale).
template <int MODE> __device__ __forceinline__ float tile_scale(const float* __restrict__ s_x, const float* __restrict__ s_w)
{
    if constexpr (MODE == MODE_BF16) return 1.0f;
    else return (s_x && s_w) ? (*s_x) * (*s_w) : 1.0f;
}

// ONLY_BF16: the caller guarantees y_dtype == FQ_BF16 and no bias, and only that path is compiled (a kernel
// that carries every output type keeps more live state across its main loop and spills in the epilogue).
template <int MODE, int FM, int FN, int CH = FM, bool ONLY_BF16 = false, typename acc_t>
__device__ __forceinline__ void store_tile(acc_t (&acc)[FM][FN], int row0, int col0, int M, int N, float scale,
                                           void* __restrict__ Y, int y_dtype, int ldy, uint8_t* stage = nullptr,
                                           const float* __restrict__ bias = nullptr)
{
    const bool fast = row0 + FM * 32 <= M && col0 + FN * 32 <= N && (ldy & 3) == 0 &&
                      (reinterpret_cast<uintptr_t>(Y) & 15) == 0;
    const bool staged = fast && stage != nullptr && (ldy & 7) == 0 && (col0 & 7) == 0;
    if constexpr (MODE == MODE_BF16) {
        if (staged) store_tile_via_lds<MODE, FQ_BF16, FM, FN, false, CH>(acc, row0, col0, 1.0f, Y, ldy, stage);
        else store_tile_as<MODE, FQ_BF16, FM, FN>(acc, row0, col0, M, N, 1.0f, Y, ldy, fast);
    } else {
        if constexpr (ONLY_BF16) {
            if (staged) store_tile_via_lds<MODE, FQ_BF16, FM, FN, false, CH>(acc, row0, col0, scale, Y, ldy, stage);
            else store_tile_as<MODE, FQ_BF16, FM, FN>(acc, row0, col0, M, N, scale, Y, ldy, fast);
            return;
        }
        if (y_dtype == FQ_I32) {
            store_tile_as<MODE, FQ_I32, FM, FN>(acc, row0, col0, M, N, 1.0f, Y, ldy, fast);
            return;
        }
        if (bias) {
            // the biased epilogue is a separate instantiation so that the plain one carries none of it
            if (staged && y_dtype == FQ_BF16) store_tile_via_lds<MODE, FQ_BF16, FM, FN, true, CH>(acc, row0, col0, scale, Y, ldy, stage, bias);
            else if (staged && y_dtype == FQ_F16) store_tile_via_lds<MODE, FQ_F16, FM, FN, true, CH>(acc, row0, col0, scale, Y, ldy, stage, bias);
            else if (y_dtype == FQ_BF16) store_tile_as<MODE, FQ_BF16, FM, FN, true>(acc, row0, col0, M, N, scale, Y, ldy, fast, bias);
            else if (y_dtype == FQ_F16) store_tile_as<MODE, FQ_F16, FM, FN, true>(acc, row0, col0, M, N, scale, Y, ldy, fast, bias);
            else store_tile_as<MODE, FQ_F32, FM, FN, true>(acc, row0, col0, M, N, scale, Y, ldy, fast, bias);
            return;
        }
        if (staged && y_dtype == FQ_BF16) store_tile_via_lds<MODE, FQ_BF16, FM, FN, false, CH>(acc, row0, col0, scale, Y, ldy, stage);
        else if (staged && y_dtype == FQ_F16) store_tile_via_lds<MODE, FQ_F16, FM, FN, false, CH>(acc, row0, col0, scale, Y, ldy, stage);
        else if (y_dtype == FQ_BF16) store_tile_as<MODE, FQ_BF16, FM, FN>(acc, row0, col0, M, N, scale, Y, ldy, fast);
        else if (y_dtype == FQ_F16) store_tile_as<MODE, FQ_F16, FM, FN>(acc, row0, col0, M, N, scale, Y, ldy, fast);
        else store_tile_as<MODE, FQ_F32, FM, FN>(acc, row0, col0, M, N, scale, Y, ldy, fast);
    }
}

// The MFMAs of one 32-byte k-slice for a wave: FM x FN blocks.
template <int MODE, int FM, int FN, typename acc_t>
__device__ __forceinline__ void mfma_slice(const v4i (&a)[FM], const v4i (&b)[FN], acc_t (&acc)[FM][FN])
{
    if constexpr (MODE == MODE_I8) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b[j], a[i], acc[i][j], 0, 0, 0);
    } else if constexpr (MODE == MODE_I4) {
        v4i alo[FM], ahi[FM], blo[FN], bhi[FN];
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            alo[i] = (a[i] << 4) & (int)0xf0f0f0f0;
            ahi[i] = a[i] & (int)0xf0f0f0f0;
        }
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            blo[j] = (b[j] << 4) & (int)0xf0f0f0f0;
            bhi[j] = b[j] & (int)0xf0f0f0f0;
        }
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(blo[j], alo[i], acc[i][j], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bhi[j], ahi[i], acc[i][j], 0, 0, 0);
    } else {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, b[j]),
                                                                   __builtin_bit_cast(v8bf, a[i]), acc[i][j], 0, 0, 0);
    }
}

// =============================================================================================
// gemm_dma_kernel: direct global -> LDS stages, register double-buffered MFMA operands
// =============================================================================================
template <int MODE, int BM, int BN, int BKB, int WM, int WN, int NSTAGE, int PIPE, int PP_SLICES = 2, bool ONLY_BF16 = false>
__device__ __forceinline__ void gemm_dma_tile(uint8_t* smem, int m0, int n0, const uint8_t* __restrict__ A,
                                              const uint8_t* __restrict__ B, int M, int N, int rowbytes,
                                              const float* __restrict__ s_x, const float* __restrict__ s_w,
                                              void* __restrict__ Y, int y_dtype, int ldy,
                                              const float* __restrict__ bias, bool prefetched = false,
                                              bool has_next = false, int m0_next = 0, int n0_next = 0)
{
    // prefetched / has_next (two-buffer ping-pong pipeline only): a workgroup that walks several tiles
    // issues the first stage of its next tile before it stores the current one, and then skips that
    // issue when it starts the next tile.
    constexpr int NW = WM * WN;
    constexpr int CPR = BKB / 16;              // chunks per row per stage
    constexpr int RPB = 64 / CPR;              // rows of one 1 KiB DMA block (one wave instruction)
    constexpr int A_BLOCKS = BM / RPB / NW;    // DMA blocks per wave per stage
    constexpr int B_BLOCKS = BN / RPB / NW;
    constexpr int LPS = A_BLOCKS + B_BLOCKS;   // DMA instructions per wave per stage
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int FM = TM / 32, FN = TN / 32;
    constexpr int KS = BKB / 32;               // 32-byte k-slices per stage
    constexpr int STAGE = (BM + BN) * BKB;
    constexpr int SWZ_SHIFT = (CPR == 8) ? 1 : 2;
    constexpr int SWZ_MASK = CPR - 1;
    // s_waitcnt immediate that leaves at most (NSTAGE-2) stages of this wave's DMA outstanding
    constexpr int VM_KEEP = (NSTAGE - 2) * LPS;
    constexpr int WAIT_KEEP = (VM_KEEP & 0xf) | ((VM_KEEP >> 4) << 14) | 0x0f70;
    constexpr int WAIT_ALL = 0x0f70;           // vmcnt(0)
    static_assert(NSTAGE >= 2 && VM_KEEP < 64, "stage count");
    static_assert(BM % (RPB * NW) == 0 && BN % (RPB * NW) == 0, "DMA blocks do not tile the stage");
    static_assert((RPB * NW) % 16 == 0, "swizzle must repeat across a wave's DMA blocks");
    static_assert(CPR == 4 || CPR == 8, "BKB must be 64 or 128");
    typedef typename Acc<MODE>::type acc_t;
    const float scale = tile_scale<MODE>(s_x, s_w);
    // next-tile prefetch across the epilogue: every DMA wait of the two-buffer pipeline is vmcnt(0), so
    // the epilogue's stores in the same counter cannot be mistaken for a landed stage
    constexpr bool OVERLAP = PIPE == 2 && NSTAGE == 2;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // ---- DMA mapping.  Block b of a tile covers rows b*RPB .. b*RPB+RPB-1; lane i lands at
    //      (row b*RPB + i/CPR, stored chunk i%CPR), which must hold global chunk (i%CPR) ^ swz(row).
    //      Wave w owns blocks w, w+NW, ...  Rows beyond the matrix re-read its last row. ----
    const int drow = lane / CPR;                                   // row within the block
    const int dsw = ((wave * RPB + drow) >> SWZ_SHIFT) & SWZ_MASK;    // same for all of the wave's blocks
    const int dchunk = (lane % CPR) ^ dsw;                          // global chunk this lane fetches
    const int nk_full = rowbytes / BKB;
    const int nk = nk_full + ((rowbytes % BKB) ? 1 : 0);
    uint32_t offA[A_BLOCKS], offB[B_BLOCKS];
    auto set_offsets = [&](int mt, int nt) {
#pragma unroll
        for (int j = 0; j < A_BLOCKS; ++j)
            offA[j] = (uint32_t)min(mt + (wave + j * NW) * RPB + drow, M - 1) * (uint32_t)rowbytes + dchunk * 16;
#pragma unroll
        for (int j = 0; j < B_BLOCKS; ++j)
            offB[j] = (uint32_t)min(nt + (wave + j * NW) * RPB + drow, N - 1) * (uint32_t)rowbytes + dchunk * 16;
    };
    set_offsets(m0, n0);

    const uint32_t lds0 = (uint32_t)(size_t)FQ_LDS_PTR(smem) + wave * 1024;
    auto issue_stage = [&](int buf, int kb, auto tail_tag) {
        constexpr bool TAIL = decltype(tail_tag)::value;
        const uint32_t sA = lds0 + buf * STAGE;
        const uint32_t sB = sA + BM * BKB;
        const uint8_t* gA = A + kb;
        const uint8_t* gB = B + kb;
        if constexpr (!TAIL) {
#pragma unroll
            for (int j = 0; j < A_BLOCKS; ++j) dma16(gA, offA[j], sA + j * NW * 1024);
#pragma unroll
            for (int j = 0; j < B_BLOCKS; ++j) dma16(gB, offB[j], sB + j * NW * 1024);
        } else {
            // last, partial stage: lanes whose chunk lies at or beyond the row end fetch 16 zero bytes
            // instead, so that every stage issues the same number of DMA instructions per wave
            const bool ok = kb + dchunk * 16 < rowbytes;
            const uint8_t* z = reinterpret_cast<const uint8_t*>(g_zero_chunk);
#pragma unroll
            for (int j = 0; j < A_BLOCKS; ++j) dma16_addr(ok ? gA + offA[j] : z, sA + j * NW * 1024);
#pragma unroll
            for (int j = 0; j < B_BLOCKS; ++j) dma16_addr(ok ? gB + offB[j] : z, sB + j * NW * 1024);
        }
    };
    auto issue_any = [&](int stage_index) {
        if (stage_index < nk_full) issue_stage(stage_index % NSTAGE, stage_index * BKB, std::false_type{});
        else issue_stage(stage_index % NSTAGE, stage_index * BKB, std::true_type{});
    };

    // ---- fragment read offsets ----
    const int frow = lane & 31, fhalf = lane >> 5;
    const int fsw = (frow >> SWZ_SHIFT) & SWZ_MASK;
    int kofs[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kofs[ks] = ((2 * ks + fhalf) ^ fsw) << 4;
    const int a_rd = (wm * TM + frow) * BKB;
    const int b_rd = BM * BKB + (wn * TN + frow) * BKB;

    acc_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // MFMA operands, double-buffered in registers.  slice(cur, rs, rks, rd): the MFMAs of the k-slice
    // held in buffer `cur`; when `rd`, the operands of k-slice `rks` of the LDS stage at `rs` are read
    // into the other buffer, two after each of the first MFMAs, in the order they will be needed
    // (a0, b0, b1.., a1..).  Scheduling barriers pin that interleaving.
    v4i a[2][FM], b[2][FN];
    constexpr int NR = FM + FN;
    auto read_frag = [&](const uint8_t* rs, int buf, int ks, int r) {
        if (r == 0) a[buf][0] = *reinterpret_cast<const v4i*>(rs + a_rd + kofs[ks]);
        else if (r <= FN) b[buf][r - 1] = *reinterpret_cast<const v4i*>(rs + b_rd + (r - 1) * 32 * BKB + kofs[ks]);
        else a[buf][r - FN] = *reinterpret_cast<const v4i*>(rs + a_rd + (r - FN) * 32 * BKB + kofs[ks]);
    };
    auto slice = [&](int cur, const uint8_t* rs, int rks, bool rd) {
        const int nxt = cur ^ 1;
        if constexpr (MODE == MODE_I4) {
            v4i alo[FM], ahi[FM], blo[FN], bhi[FN];
#pragma unroll
            for (int t = 0; t < 2 * FM * FN; ++t) {
                const int sub = t / (FM * FN), idx = t % (FM * FN), i = idx / FN, j = idx % FN;
                // widen an operand the first time it is needed
                if (sub == 0) {
                    if (j == 0) alo[i] = (a[cur][i] << 4) & (int)0xf0f0f0f0;
                    if (i == 0) blo[j] = (b[cur][j] << 4) & (int)0xf0f0f0f0;
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(blo[j], alo[i], acc[i][j], 0, 0, 0);
                } else {
                    if (j == 0) ahi[i] = a[cur][i] & (int)0xf0f0f0f0;
                    if (i == 0) bhi[j] = b[cur][j] & (int)0xf0f0f0f0;
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bhi[j], ahi[i], acc[i][j], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (rd && 2 * t < NR) {
                    read_frag(rs, nxt, rks, 2 * t);
                    if (2 * t + 1 < NR) read_frag(rs, nxt, rks, 2 * t + 1);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        } else {
#pragma unroll
            for (int t = 0; t < FM * FN; ++t) {
                const int i = t / FN, j = t % FN;
                if constexpr (MODE == MODE_I8)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b[cur][j], a[cur][i], acc[i][j], 0, 0, 0);
                else
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, b[cur][j]),
                                                                       __builtin_bit_cast(v8bf, a[cur][i]), acc[i][j],
                                                                       0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (rd && 2 * t < NR) {
                    read_frag(rs, nxt, rks, 2 * t);
                    if (2 * t + 1 < NR) read_frag(rs, nxt, rks, 2 * t + 1);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    };

    if constexpr (PIPE == 2) {
        // ---- ping-pong.  The 8 waves form two groups (waves 0-3 and 4-7; wave w and w+4 share a SIMD).
        //      Every wave alternates a memory phase (LDS operand reads of SPP k-slices, for INT4 also
        //      the widening to int8, and once per stage the DMA of a later stage) and a compute phase
        //      (the MFMAs on those operands), with a workgroup barrier after each phase.  Group B runs
        //      one barrier interval behind group A, so on every SIMD one wave issues nothing but MFMAs
        //      while its partner issues nothing but memory instructions.
        //
        //      Barrier events e = 1, 2, ...; L = 2 * NPH * nk loop barriers per wave.  Group A passes its
        //      loop barriers at e = 1..L and one balancing barrier at e = L+1; group B one staggering
        //      barrier at e = 1 and its loop barriers at e = 2..L+1.  Buffer of stage t-1 is last read
        //      in B's final memory phase of stage t-1, which ends at e = 2 NPH t; A issues the DMA of
        //      stage t+1 into it in its first memory phase of stage t, which begins after that event
        //      (B later still).  Stage t+1 is first read by A after e = 2 NPH (t+1); A waits for its own
        //      DMA before that barrier (end of its last compute phase of stage t), B before the barrier
        //      closing its last memory phase of stage t, which is the same event. ----
        //      With more than two buffers, NSTAGE-1 stages are in flight and the waits leave NSTAGE-2 of
        //      them outstanding (all of them once no further stage is issued).
        static_assert(PIPE != 2 || NW == 8, "ping-pong pipeline: 8 waves");
        // PP_SLICES = MFMA k-steps (operand sets) per phase; a packed INT4 slice yields two of them
        constexpr int SPP = (MODE == MODE_I4) ? (PP_SLICES >= 2 ? PP_SLICES / 2 : 1) : PP_SLICES;   // LDS k-slices per phase
        constexpr int NPH = KS / SPP;
        constexpr int NOP = (MODE == MODE_I4) ? 2 * SPP : SPP;     // operand sets per phase
        static_assert(KS % SPP == 0, "phases must tile the stage");
        const bool group_b = wave >= 4;
        v4i pa[NOP][FM], pb[NOP][FN];

        if (!(OVERLAP && prefetched)) {
#pragma unroll
            for (int st = 0; st < NSTAGE - 1; ++st)
                if (st < nk) issue_any(st);
        }
        if (nk >= NSTAGE - 1) __builtin_amdgcn_s_waitcnt(WAIT_KEEP);
        else __builtin_amdgcn_s_waitcnt(WAIT_ALL);
        __builtin_amdgcn_s_barrier();
        if (group_b) __builtin_amdgcn_s_barrier();
        int buf = 0;
        for (int kt = 0; kt < nk; ++kt) {
            const uint8_t* s = smem + buf * STAGE;
            buf = (buf + 1 == NSTAGE) ? 0 : buf + 1;
            const bool steady = kt + NSTAGE - 1 < nk;
#pragma unroll
            for (int ph = 0; ph < NPH; ++ph) {
                // ---------------- memory phase ----------------
                if (ph == 0 && steady) issue_any(kt + NSTAGE - 1);
#pragma unroll
                for (int q = 0; q < SPP; ++q) {
                    const int ks = ph * SPP + q;
                    v4i ra[FM], rb[FN];
#pragma unroll
                    for (int i = 0; i < FM; ++i) ra[i] = *reinterpret_cast<const v4i*>(s + a_rd + i * 32 * BKB + kofs[ks]);
#pragma unroll
                    for (int j = 0; j < FN; ++j) rb[j] = *reinterpret_cast<const v4i*>(s + b_rd + j * 32 * BKB + kofs[ks]);
                    if constexpr (MODE == MODE_I4) {
                        // INT4: only the operands of the first MFMA are widened here; the rest is
                        // widened in the compute phase, in the shadow of the MFMAs (see below)
#pragma unroll
                        for (int i = 0; i < FM; ++i) pa[2 * q + 1][i] = ra[i];
#pragma unroll
                        for (int j = 0; j < FN; ++j) pb[2 * q + 1][j] = rb[j];
                        pa[2 * q][0] = (ra[0] << 4) & (int)0xf0f0f0f0;
                        pb[2 * q][0] = (rb[0] << 4) & (int)0xf0f0f0f0;
                    } else {
#pragma unroll
                        for (int i = 0; i < FM; ++i) pa[q][i] = ra[i];
#pragma unroll
                        for (int j = 0; j < FN; ++j) pb[q][j] = rb[j];
                    }
                }
                __builtin_amdgcn_s_waitcnt(0xc07f);                                 // lgkmcnt(0)
                if (ph == NPH - 1 && group_b) {                                     // B: my DMA of stage kt+1 landed
                    if (steady) __builtin_amdgcn_s_waitcnt(WAIT_KEEP);
                    else __builtin_amdgcn_s_waitcnt(WAIT_ALL);
                }
                __builtin_amdgcn_sched_barrier(0);
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
                // ---------------- compute phase ----------------
                __builtin_amdgcn_s_setprio(1);
                if constexpr (MODE == MODE_I4) {
                    // For packed slice q, pa[2q+1] / pb[2q+1] hold the packed operands.  Low nibbles
                    // (x << 4) & 0xf0.. go to pa[2q] / pb[2q] and feed the first FM*FN MFMAs; the high
                    // nibbles x & 0xf0.. are formed in place for the second FM*FN.  Each widening is
                    // issued right after an earlier MFMA, so it executes while that MFMA occupies the
                    // matrix pipe, and at least one MFMA before its first use.
                    constexpr int NM = FM * FN;
                    static_assert((FN - 1) + (FM - 1) + (FM > FN ? FM : FN) <= NM, "widening must finish within the low half");
#pragma unroll
                    for (int q = 0; q < SPP; ++q) {
                        auto widen_after = [&](int t) {
                            // after MFMA t of the low half: production order b[1..FN-1], a[1..FM-1] as the
                            // (i, j) walk needs them, then the high halves, two operands per slot
                            if (t < FN - 1) pb[2 * q][t + 1] = (pb[2 * q + 1][t + 1] << 4) & (int)0xf0f0f0f0;
                            else if (t - (FN - 1) < FM - 1) {
                                const int i = t - (FN - 1) + 1;
                                pa[2 * q][i] = (pa[2 * q + 1][i] << 4) & (int)0xf0f0f0f0;
                            } else {
                                const int u = t - (FN - 1) - (FM - 1);          // 0, 1, ...
                                if (u < FM) pa[2 * q + 1][u] = pa[2 * q + 1][u] & (int)0xf0f0f0f0;
                                if (u < FN) pb[2 * q + 1][u] = pb[2 * q + 1][u] & (int)0xf0f0f0f0;
                            }
                        };
#pragma unroll
                        for (int t = 0; t < NM; ++t) {
                            const int i = t / FN, j = t % FN;
                            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(pb[2 * q][j], pa[2 * q][i], acc[i][j], 0, 0, 0);
                            widen_after(t);
                            __builtin_amdgcn_sched_barrier(0);
                        }
#pragma unroll
                        for (int t = 0; t < NM; ++t) {
                            const int i = t / FN, j = t % FN;
                            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(pb[2 * q + 1][j], pa[2 * q + 1][i], acc[i][j], 0, 0, 0);
                        }
                    }
                } else {
#pragma unroll
                    for (int o = 0; o < NOP; ++o)
#pragma unroll
                        for (int i = 0; i < FM; ++i)
#pragma unroll
                            for (int j = 0; j < FN; ++j) {
                                if constexpr (MODE == MODE_BF16)
                                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, pb[o][j]),
                                                                                       __builtin_bit_cast(v8bf, pa[o][i]),
                                                                                       acc[i][j], 0, 0, 0);
                                else
                                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(pb[o][j], pa[o][i], acc[i][j], 0, 0, 0);
                            }
                }
                __builtin_amdgcn_s_setprio(0);
                if (ph == NPH - 1 && !group_b) {                                    // A: my DMA of stage kt+1 landed
                    if (steady) __builtin_amdgcn_s_waitcnt(WAIT_KEEP);
                    else __builtin_amdgcn_s_waitcnt(WAIT_ALL);
                }
                __builtin_amdgcn_sched_barrier(0);
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (!group_b) __builtin_amdgcn_s_barrier();
        // Every wave is past its last LDS operand read and has waited for all of its DMA: buffer 0 may
        // receive the next tile's first stage while this tile is stored from registers through the
        // other buffer.
        if (OVERLAP && has_next) {
            set_offsets(m0_next, n0_next);
            issue_any(0);
        }
    } else {
        // ---- two buffers, barrier before the LAST k-slice of a stage.  By then every wave holds the
        //      operands of that slice in registers, so the stage's buffer is free: the barrier both
        //      publishes stage kt+1 (each wave waited for its own DMA) and releases buffer kt for the
        //      DMA of stage kt+2, and the MFMAs of the last slice overlap the first LDS reads of
        //      stage kt+1, so no wave idles behind the barrier waiting for operands. ----
        static_assert(NSTAGE == 2 && KS % 2 == 0, "mid-stage barrier pipeline needs 2 buffers, even KS");
        issue_any(0);
        __builtin_amdgcn_s_waitcnt(0x0070);      // vmcnt(0) lgkmcnt(0)
        __syncthreads();
        if (nk > 1) issue_any(1);
#pragma unroll
        for (int r = 0; r < NR; ++r) read_frag(smem, 0, 0, r);
        __builtin_amdgcn_sched_barrier(0);
        for (int kt = 0; kt < nk; ++kt) {
            const uint8_t* s = smem + (kt & 1) * STAGE;
            const uint8_t* sn = smem + ((kt + 1) & 1) * STAGE;
#pragma unroll
            for (int ks = 0; ks < KS - 1; ++ks) slice(ks & 1, s, ks + 1, true);
            __builtin_amdgcn_s_waitcnt(0x0070);  // last slice's operands are in registers; my DMA of stage kt+1 landed
            __syncthreads();
            if (kt + 2 < nk) issue_any(kt + 2);
            __builtin_amdgcn_sched_barrier(0);
            slice((KS - 1) & 1, sn, 0, kt + 1 < nk);
        }
    }

    // After the last barrier of the loop no wave reads the stage buffers any more (the operands of
    // the final k-slice are in registers), so each wave may reuse its share of LDS to stage its output.
    if constexpr (OVERLAP) {
        // buffer 0 may be filling with the next tile's first stage: stage the output through this
        // wave's share of buffer 1, as many 32-row blocks at a time as fit
        constexpr int SHARE = STAGE / NW;
        constexpr int CH_FIT = SHARE / (32 * TN * 2);
        constexpr int CH = CH_FIT >= FM ? FM : (CH_FIT >= 2 ? 2 : CH_FIT);
        static_assert(CH >= 1 && FM % CH == 0, "output staging must fit the wave's share of a stage buffer");
        store_tile<MODE, FM, FN, CH, ONLY_BF16>(acc, m0 + wm * TM, n0 + wn * TN, M, N, scale, Y, y_dtype, ldy,
                                     smem + STAGE + wave * SHARE, bias);
    } else {
        constexpr bool CAN_STAGE = NW * TM * TN * 2 <= NSTAGE * STAGE;
        store_tile<MODE, FM, FN, FM, ONLY_BF16>(acc, m0 + wm * TM, n0 + wn * TN, M, N, scale, Y, y_dtype, ldy,
                                 CAN_STAGE ? smem + wave * (TM * TN * 2) : nullptr, bias);
    }
}

// The kernel.  Workgroups [0, n_main) compute full BM x BN tiles.  When the number of tiles leaves a
// last, partly filled round of at most half the CUs, those tiles are instead computed as two
// (BM/2) x BN halves by workgroups [n_main, n_main + 2 * n_tail), so that the last round takes about
// half as long.
template <int MODE, int BM, int BN, int BKB, int WM, int WN, int NSTAGE, int PIPE, int PP_SLICES = 2, bool ONLY_BF16 = false>
__global__ __launch_bounds__(WM* WN * 64) void gemm_dma_kernel(const uint8_t* __restrict__ A,
                                                                const uint8_t* __restrict__ B, int M, int N,
                                                                int rowbytes, const float* __restrict__ s_x,
                                                                const float* __restrict__ s_w,
                                                                void* __restrict__ Y, int y_dtype, int ldy,
                                                                int tiles_m, int tiles_n, int n_main, int n_tail, Batch bt)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const ClockProbe probe(bt.ticks);
    // batched launches: blockIdx.y selects the problem
    A += (size_t)blockIdx.y * bt.stride_a;
    B += (size_t)blockIdx.y * bt.stride_b;
    Y = static_cast<uint8_t*>(Y) + (size_t)blockIdx.y * bt.stride_y;
    // Workgroup w walks the virtual workgroup ids w, w + gridDim.x, ...: ids below n_main are full
    // tiles, the rest half tiles.  (With gridDim.x >= n_main + 2 n_tail each workgroup has one id.)
    constexpr bool CAN_PREFETCH = PIPE == 2 && NSTAGE == 2;     // see gemm_dma_tile
    const int n_ids = n_main + 2 * n_tail;
    int tile_m, tile_n;
    bool prefetched = false;
    for (int v = blockIdx.x; v < n_ids; v += gridDim.x) {
        if (v < n_main) {
            tile_of_workgroup(v, n_main, tiles_m, tiles_n, tile_m, tile_n);
            const int vn = v + gridDim.x;
            const bool has_next = vn < n_main;
            int next_m = 0, next_n = 0;
            if (has_next) tile_of_workgroup(vn, n_main, tiles_m, tiles_n, next_m, next_n);
            gemm_dma_tile<MODE, BM, BN, BKB, WM, WN, NSTAGE, PIPE, PP_SLICES, ONLY_BF16>(smem, tile_m * BM, tile_n * BN, A, B, M, N, rowbytes,
                                                                    s_x, s_w, Y, y_dtype, ldy, bt.bias, prefetched,
                                                                    has_next, next_m * BM, next_n * BN);
            prefetched = CAN_PREFETCH && has_next;
        } else {
            if constexpr (BM >= 128 && (BM / 2) % (64 / (BKB / 16) * WM * WN) == 0) {
                const int t = v - n_main;
                tile_of_logical(n_main + (t >> 1), tiles_m, tiles_n, tile_m, tile_n);
                gemm_dma_tile<MODE, BM / 2, BN, BKB, WM, WN, NSTAGE, PIPE, PP_SLICES, ONLY_BF16>(smem, tile_m * BM + (t & 1) * (BM / 2),
                                                                            tile_n * BN, A, B, M, N, rowbytes, s_x, s_w,
                                                                            Y, y_dtype, ldy, bt.bias);
            }
        }
        // the stage buffers are reused by the next tile: every wave must be done staging its output
        // (a tile that was prefetched synchronizes on its own first barrier instead, after its waits)
        if (v + (int)gridDim.x < n_ids && !prefetched) __syncthreads();
    }
    probe.finish(bt.ticks);
}

// =============================================================================================
// gemm_wide_kernel (INT8, bf16): four waves with 128 x 128 wave tiles
// =============================================================================================
// The ping-pong kernel's 128 x 64 wave tiles fetch 3/4 of an operand from LDS per MFMA; at the INT8 and
// bf16 rates that read stream plus the copies' writes keeps the LDS as busy as the matrix pipe.  Here a
// wave owns 128 x 128 of the output (256 accumulator registers per lane, in AGPRs; one wave per SIMD),
// which needs 1/2 operand per MFMA.  A single wave has to issue everything itself, so the work is dealt
// out by MFMA slot: one 16-byte LDS read of the next k-slice's operands after every second MFMA
// (operands double-buffered in registers) and, during a stage's last k-slice, one global->LDS copy
// instruction per MFMA for the stage after next.  Two stage buffers of 128 bytes per row; the barrier
// sits before the last k-slice of a stage, when every wave holds that slice in registers: it frees the
// stage's buffer for those copies and publishes the next stage (each wave has waited for its own
// copies), and the last slice's MFMAs overlap the first reads of the next stage.
// Rows must be whole 128-byte stages (checked at launch): a per-copy choice between the row and the zero
// chunk, as the ping-pong kernel makes once per stage, costs this kernel 15 % when it sits between the MFMAs.
// Measured against the ping-pong kernel, in the instantiation that carries the bf16 epilogue only (the
// generic one spills with 256 accumulators and loses 5 us per tile): per 128-byte stage of a tile both take
// 1.08-1.11 us at full clock, fixed cost per tile 7-11 us in both; INT8 +2 % and bf16 +2-4 % on live data,
// INT8 -2..-5 % on zero operands.  It is the default for large INT8 and bf16 problems with such rows and a
// plain bf16 output; variant 11 selects it for any output.
template <int MODE, int BM, int BN, bool ONLY_BF16>
__device__ __forceinline__ void gemm_wide_tile(uint8_t* smem, int m0, int n0, const uint8_t* __restrict__ A,
                                               const uint8_t* __restrict__ B, int M, int N, int rowbytes,
                                               const float* __restrict__ s_x, const float* __restrict__ s_w,
                                               void* __restrict__ Y, int y_dtype, int ldy,
                                               const float* __restrict__ bias)
{
    static_assert(MODE == MODE_I8 || MODE == MODE_BF16, "16-byte operands per lane");
    constexpr int WM = 2, WN = 2, NW = 4, NSTAGE = 2, BKB = 128;
    constexpr int CPR = BKB / 16, RPB = 64 / CPR;
    constexpr int A_BLOCKS = BM / RPB / NW, B_BLOCKS = BN / RPB / NW, LPS = A_BLOCKS + B_BLOCKS;
    constexpr int TM = BM / WM, TN = BN / WN, FM = TM / 32, FN = TN / 32;
    constexpr int KS = BKB / 32;                     // k-slices per stage
    constexpr int NR = FM + FN, NM = FM * FN;
    constexpr int STAGE = (BM + BN) * BKB;
    constexpr int SWZ_SHIFT = 1, SWZ_MASK = 7;
    static_assert(BM % (RPB * NW) == 0 && BN % (RPB * NW) == 0, "copy blocks must tile the stage");
    typedef typename Acc<MODE>::type acc_t;
    const float scale = tile_scale<MODE>(s_x, s_w);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int nk_full = rowbytes / BKB;
    const int nk = nk_full + ((rowbytes % BKB) ? 1 : 0);

    // copy mapping as in gemm_dma_tile: block b covers rows b RPB .. +RPB-1, lane i lands at
    // (row b RPB + i / CPR, stored chunk i % CPR) and fetches global chunk (i % CPR) ^ swz(row)
    const int drow = lane / CPR;
    const int dsw = ((wave * RPB + drow) >> SWZ_SHIFT) & SWZ_MASK;
    const int dchunk = (lane % CPR) ^ dsw;
    static_assert((RPB * NW) % 16 == 0, "swizzle must repeat across a wave's copy blocks");
    uint32_t offA[A_BLOCKS], offB[B_BLOCKS];
#pragma unroll
    for (int j = 0; j < A_BLOCKS; ++j)
        offA[j] = (uint32_t)min(m0 + (wave + j * NW) * RPB + drow, M - 1) * (uint32_t)rowbytes + dchunk * 16;
#pragma unroll
    for (int j = 0; j < B_BLOCKS; ++j)
        offB[j] = (uint32_t)min(n0 + (wave + j * NW) * RPB + drow, N - 1) * (uint32_t)rowbytes + dchunk * 16;
    const uint32_t lds0 = (uint32_t)(size_t)FQ_LDS_PTR(smem) + wave * 1024;
    const uint8_t* zero16 = reinterpret_cast<const uint8_t*>(g_zero_chunk);
    // copy instruction idx (0 .. LPS-1) of a stage: the A blocks, then the B blocks; in the last, partial
    // stage lanes whose chunk lies at or beyond the row end fetch 16 zero bytes instead
    auto issue_one = [&](int stage_index, int idx) {
        const uint32_t sA = lds0 + (stage_index % NSTAGE) * STAGE;
        const int kb = stage_index * BKB;
        const bool isA = idx < A_BLOCKS;
        const int j = isA ? idx : idx - A_BLOCKS;
        const uint8_t* g = (isA ? A : B) + kb;
        const uint32_t off = isA ? offA[j] : offB[j];
        const uint32_t dst = (isA ? sA : sA + BM * BKB) + j * NW * 1024;
        dma16(g, off, dst);                      // whole stages only: rowbytes is a multiple of BKB (checked at launch)
    };
    auto issue_all = [&](int stage_index) {
#pragma unroll
        for (int q = 0; q < LPS; ++q) issue_one(stage_index, q);
    };

    const int frow = lane & 31, fhalf = lane >> 5;
    const int fsw = (frow >> SWZ_SHIFT) & SWZ_MASK;
    int kofs[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kofs[ks] = ((2 * ks + fhalf) ^ fsw) << 4;
    const int a_rd = (wm * TM + frow) * BKB, b_rd = BM * BKB + (wn * TN + frow) * BKB;

    acc_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // operands in the order the MFMA walk (i outer, j inner) first needs them: a0, b0 .. b(FN-1), a1 ..
    v4i opa[2][FM], opb[2][FN];
    auto read_op = [&](const uint8_t* st, int ks, int buf, int r) {
        if (r == 0) opa[buf][0] = *reinterpret_cast<const v4i*>(st + a_rd + kofs[ks]);
        else if (r <= FN) opb[buf][r - 1] = *reinterpret_cast<const v4i*>(st + b_rd + (r - 1) * 32 * BKB + kofs[ks]);
        else opa[buf][r - FN] = *reinterpret_cast<const v4i*>(st + a_rd + (r - FN) * 32 * BKB + kofs[ks]);
    };
    // the MFMAs of the slice in buffer `cur`; the NR reads of slice `rks` of stage `rs` (into the other
    // buffer) and, when cp, the LPS copies of `copy_stage` are spread evenly over the NM slots
    auto slice = [&](int cur, const uint8_t* rs, int rks, auto rd_tag, auto copy_tag, int copy_stage) {
        constexpr bool rd = decltype(rd_tag)::value;
        constexpr bool cp = decltype(copy_tag)::value;
#pragma unroll
        for (int t = 0; t < NM; ++t) {
            const int i = t / FN, j = t % FN;
            if constexpr (MODE == MODE_I8)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(opb[cur][j], opa[cur][i], acc[i][j], 0, 0, 0);
            else
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, opb[cur][j]),
                                                                   __builtin_bit_cast(v8bf, opa[cur][i]), acc[i][j], 0, 0, 0);
            if constexpr (rd) {
#pragma unroll
                for (int q = t * NR / NM; q < (t + 1) * NR / NM; ++q) read_op(rs, rks, cur ^ 1, q);
            }
            if constexpr (cp) {
#pragma unroll
                for (int q = t * LPS / NM; q < (t + 1) * LPS / NM; ++q) issue_one(copy_stage, q);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    typedef std::true_type yes;
    typedef std::false_type no;

    // both buffers are free: issue the first two stages together, wait for the first
    issue_all(0);
    if (nk > 1) {
        issue_all(1);
        __builtin_amdgcn_s_waitcnt((LPS & 0xf) | ((LPS >> 4) << 14) | 0x0070);     // vmcnt(LPS) lgkmcnt(0)
    } else {
        __builtin_amdgcn_s_waitcnt(0x0070);          // vmcnt(0) lgkmcnt(0)
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < NR; ++r) read_op(smem, 0, 0, r);
    __builtin_amdgcn_sched_barrier(0);

    static_assert(KS % 2 == 0, "operand buffers alternate per slice");
    // one stage: slices 0 .. KS-2 (each reads the next slice of the stage), the barrier, the last slice
    // (reads slice 0 of the next stage; when copy_tag, copies stage kt+2 into the buffer just freed)
    auto stage = [&](int kt, auto next_tag, auto copy_tag) {
        const uint8_t* s = smem + (kt & 1) * STAGE;
        const uint8_t* sn = smem + ((kt + 1) & 1) * STAGE;
#pragma unroll
        for (int ks = 0; ks < KS - 1; ++ks) slice(ks & 1, s, ks + 1, yes{}, no{}, 0);
        // the last slice's operands are in registers; my copies of stage kt+1 (issued a stage ago) landed
        __builtin_amdgcn_s_waitcnt(0x0070);
        __syncthreads();
        slice((KS - 1) & 1, sn, 0, next_tag, copy_tag, kt + 2);
    };
    int kt = 0;
    for (; kt + 2 < nk; ++kt) stage(kt, yes{}, yes{});
    for (; kt + 1 < nk; ++kt) stage(kt, yes{}, no{});
    stage(kt, no{}, no{});
    __syncthreads();                                 // every wave is past its last LDS operand read

    store_tile<MODE, FM, FN, 2, ONLY_BF16>(acc, m0 + wm * TM, n0 + wn * TN, M, N, scale, Y, y_dtype, ldy,
                                smem + wave * (64 * TN * 2), bias);
}

// Workgroups [0, n_main) compute 256 x 256 tiles; a last, partly filled round of at most half the CUs is
// computed as 128 x 256 halves by workgroups [n_main, n_main + 2 n_tail).
template <int MODE, bool ONLY_BF16>
__global__ __launch_bounds__(256) void gemm_wide_kernel(const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, int M,
                                                        int N, int rowbytes, const float* __restrict__ s_x,
                                                        const float* __restrict__ s_w, void* __restrict__ Y, int y_dtype,
                                                        int ldy, int tiles_m, int tiles_n, int n_main, Batch bt)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const ClockProbe probe(bt.ticks);
    A += (size_t)blockIdx.y * bt.stride_a;
    B += (size_t)blockIdx.y * bt.stride_b;
    Y = static_cast<uint8_t*>(Y) + (size_t)blockIdx.y * bt.stride_y;
    int tile_m, tile_n;
    const int v = blockIdx.x;
    if (v < n_main) {
        tile_of_workgroup(v, n_main, tiles_m, tiles_n, tile_m, tile_n);
        gemm_wide_tile<MODE, 256, 256, ONLY_BF16>(smem, tile_m * 256, tile_n * 256, A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy,
                                       bt.bias);
    } else {
        const int t = v - n_main;
        tile_of_logical(n_main + (t >> 1), tiles_m, tiles_n, tile_m, tile_n);
        gemm_wide_tile<MODE, 128, 256, ONLY_BF16>(smem, tile_m * 256 + (t & 1) * 128, tile_n * 256, A, B, M, N, rowbytes, s_x, s_w,
                                       Y, y_dtype, ldy, bt.bias);
    }
    probe.finish(bt.ticks);
}

// =============================================================================================
// gemm_deep_kernel (INT8, packed INT4, bf16): four waves with 128 x 128 wave tiles, A staged three deep, B two deep
// =============================================================================================
// What bounds gemm_wide_kernel: a global->LDS copy instruction moves 1 KiB and keeps the address unit of the CU busy
// for 16 cycles (64 bytes per cycle), so the 64 copies of a 128-byte stage take it 1024 cycles -- half of the stage's
// 2048 MFMA cycles.  With two stage buffers all of them have to be issued in the one slice after the barrier that
// frees a buffer, by all four waves at once: that slice's 16 MFMA slots then advance at the address unit's pace
// (64 cycles each instead of 32; measured 1050 cycles for the slice against 512).  Here the whole of LDS is used to
// give the copies room: three A buffers and two B buffers of 32 KiB (A = the tile's rows of X, B = its rows of W).
// A's copies may then be issued a stage earlier than B's, and the 16 copies a wave issues per stage are dealt out
// over all four slices, four per slice, the waves staggered (wave w in the MFMA slots t = w mod 4): every MFMA slot
// carries exactly one copy instruction of one wave, which the address unit finishes within that slot.
//   stage kt:  slice 0   second half of B(kt+1)   (into the B buffer freed by the barrier of stage kt-1)
//              slice 1,2 A(kt+2)                  (into the A buffer freed by the barrier of stage kt-1)
//              wait for the stage kt+1 (all but the copies of A(kt+2), the youngest), barrier
//              slice 3   first half of B(kt+2)    (into the B buffer this barrier frees)
// The wave index is a template parameter (four instantiations of the tile, selected once per workgroup): the stagger
// costs no branches inside the loop.  Rows must be whole 128-byte stages, as for gemm_wide_kernel.
// Widening steps of a packed-nibble slice of gemm_deep_tile: the (at most two) steps issued after MFMA slot `sl`
// (low pass = slots [0, NM), high pass = [NM, 2 NM), NM = 4 FM).  A step is kind * 8 + operand, operand 0..3 = a0..a3,
// 4..7 = b0..b3.  Low pass: the low halves of a1.. (a0 and every b come in ready), then every high half, in the order
// the high pass first uses them.  High pass (its slots t = 0.. also issue the LDS reads of the next slice, a0 b0 b1 b2
// b3 a1.. one per slot): the low halves of the next slice's a0, b0..b3, each at least three slots after its read.
enum { W_NONE = 0, W_SH = 1, W_AN = 2, W_HI = 3, W_SHN = 4 };
template <int FM> constexpr int widen_plan(int sl, int which)
{
    constexpr int NM = 4 * FM;
    constexpr int carry[5] = {0, 4, 5, 6, 7};                       // a0, b0, b1, b2, b3
    if (FM == 4) {
        constexpr int hi_order[8] = {4, 0, 5, 6, 7, 1, 2, 3};       // b0 a0 b1 b2 b3 a1 a2 a3
        if (which != 0) return 0;
        if (sl < 6) return ((sl & 1) ? W_AN : W_SH) * 8 + 1 + sl / 2;
        if (sl < 14) return W_HI * 8 + hi_order[sl - 6];
        if (sl < NM + 6) return 0;
        return (((sl - NM) & 1) ? W_AN : W_SHN) * 8 + carry[(sl - NM - 6) / 2];
    } else {
        constexpr int hi_order[6] = {4, 0, 5, 6, 7, 1};
        if (sl < 2) return which ? 0 : (sl ? W_AN : W_SH) * 8 + 1;
        if (sl < NM) return which ? 0 : W_HI * 8 + hi_order[sl - 2];
        if (sl < NM + 3) return 0;
        return (which ? W_AN : W_SHN) * 8 + carry[sl - NM - 3];
    }
}

template <int MODE, int BM, int BN, bool ONLY_BF16, int W>
__device__ __forceinline__ void gemm_deep_tile(uint8_t* smem, int m0, int n0, const uint8_t* __restrict__ A,
                                               const uint8_t* __restrict__ B, int M, int N, int rowbytes,
                                               const float* __restrict__ s_x, const float* __restrict__ s_w,
                                               void* __restrict__ Y, int y_dtype, int ldy,
                                               const float* __restrict__ bias)
{
    static_assert(MODE == MODE_I8 || MODE == MODE_BF16 || MODE == MODE_I4, "16-byte operands per lane");
    constexpr int WM = 2, WN = 2, NW = 4, BKB = 128;
    constexpr int CPR = BKB / 16, RPB = 64 / CPR;
    constexpr int A_BLOCKS = BM / RPB / NW, B_BLOCKS = BN / RPB / NW;
    constexpr int TM = BM / WM, TN = BN / WN, FM = TM / 32, FN = TN / 32;
    constexpr int KS = BKB / 32, NR = FM + FN, NM = FM * FN;
    constexpr int A_UNIT = BM * BKB, B_UNIT = BN * BKB, B_BASE = 3 * A_UNIT;
    constexpr int SWZ_SHIFT = 1, SWZ_MASK = 7;
    constexpr int wm = W / WN, wn = W % WN;
    static_assert(KS == 4 && A_BLOCKS % 2 == 0 && B_BLOCKS % 2 == 0, "schedule written for four slices and halves");
    static_assert((RPB * NW) % 16 == 0, "swizzle must repeat across a wave's copy blocks");
    typedef typename Acc<MODE>::type acc_t;
    const float scale = tile_scale<MODE>(s_x, s_w);

    const int lane = threadIdx.x & 63;
    const int nk = rowbytes / BKB;                  // whole stages only (checked at launch)

    // copy mapping as in gemm_dma_tile: block b covers rows b RPB .. +RPB-1, lane i lands at
    // (row b RPB + i / CPR, stored chunk i % CPR) and fetches global chunk (i % CPR) ^ swz(row)
    const int drow = lane / CPR;
    const int dsw = ((W * RPB + drow) >> SWZ_SHIFT) & SWZ_MASK;
    const int dchunk = (lane % CPR) ^ dsw;
    uint32_t offA[A_BLOCKS], offB[B_BLOCKS];
#pragma unroll
    for (int j = 0; j < A_BLOCKS; ++j)
        offA[j] = (uint32_t)min(m0 + (W + j * NW) * RPB + drow, M - 1) * (uint32_t)rowbytes + dchunk * 16;
#pragma unroll
    for (int j = 0; j < B_BLOCKS; ++j)
        offB[j] = (uint32_t)min(n0 + (W + j * NW) * RPB + drow, N - 1) * (uint32_t)rowbytes + dchunk * 16;
    const uint32_t lds0 = (uint32_t)(size_t)FQ_LDS_PTR(smem) + W * 1024;
    // copy instruction j of A / B of a stage into ring slot `slot`
    auto issue_a = [&](int stage_index, int slot, int j) {
        dma16(A + stage_index * BKB, offA[j], lds0 + slot * A_UNIT + j * NW * 1024);
    };
    auto issue_b = [&](int stage_index, int slot, int j) {
        dma16(B + stage_index * BKB, offB[j], lds0 + B_BASE + slot * B_UNIT + j * NW * 1024);
    };

    const int frow = lane & 31, fhalf = lane >> 5;
    const int fsw = (frow >> SWZ_SHIFT) & SWZ_MASK;
    int kofs[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kofs[ks] = ((2 * ks + fhalf) ^ fsw) << 4;
    const int a_rd = (wm * TM + frow) * BKB, b_rd = (wn * TN + frow) * BKB;

    acc_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // operands in the order the MFMA walk (i outer, j inner) first needs them: a0, b0 .. b(FN-1), a1 ..
    v4i opa[2][FM], opb[2][FN];
    auto read_op = [&](const uint8_t* sa, const uint8_t* sb, int ks, int buf, int r) {
        if (r == 0) opa[buf][0] = *reinterpret_cast<const v4i*>(sa + a_rd + kofs[ks]);
        else if (r <= FN) opb[buf][r - 1] = *reinterpret_cast<const v4i*>(sb + b_rd + (r - 1) * 32 * BKB + kofs[ks]);
        else opa[buf][r - FN] = *reinterpret_cast<const v4i*>(sa + a_rd + (r - FN) * 32 * BKB + kofs[ks]);
    };
    // The MFMAs of the slice in operand buffer `cur`; the NR reads of slice `rks` of the stage at (ra, rb) into the
    // other buffer; and this wave's copies of the slice.  kind: 0 none, 1 = B blocks [B_BLOCKS/2, B_BLOCKS),
    // 2 = A blocks [0, A_BLOCKS/2), 3 = A blocks [A_BLOCKS/2, A_BLOCKS), 4 = B blocks [0, B_BLOCKS/2); C copies in
    // NM slots, one every S = NM / C slots, this wave's at offset W mod S.
    // Packed nibbles (MODE_I4): a slice is 32 packed bytes of k = two MFMA k-steps, a low pass over the NM
    // accumulators with the low nibbles (x << 4) & 0xf0.. (alo / blo) and a high pass with the high nibbles
    // x & 0xf0.., formed in place in the packed registers.  The LDS reads of the next slice are issued in the high
    // pass (issued in the low pass, with their results waiting a whole pass, they cost a quarter of the MFMA rate:
    // measured).  The widening runs in the shadow of the MFMAs, at most widen_plan's steps per MFMA slot, each at
    // least one slot before its first use; a slice enters with alo[0] and blo[0..3] ready: formed during the high
    // pass of the slice before (in the prologue for the first).
    v4i alo[FM], blo[FN];
    auto widen_lo = [](const v4i& x) -> v4i { return (x << 4) & (int)0xf0f0f0f0; };
    // One widening step = 4 VALU instructions on one operand vector: W_SH lo = packed << 4 (W_SHN: of the NEXT slice's
    // packed vector), W_AN lo &= 0xf0.., W_HI packed &= 0xf0.. in place (after the vector's W_SH).
    auto widen_step = [&](int code, int cur) {
        const int kind = code >> 3, x = code & 7, src = (kind == W_SHN) ? (cur ^ 1) : cur;
        if (kind == W_SH || kind == W_SHN) {
            if (x < 4) alo[x] = opa[src][x] << 4;
            else blo[x - 4] = opb[src][x - 4] << 4;
        } else if (kind == W_AN) {
            if (x < 4) alo[x] = alo[x] & (int)0xf0f0f0f0;
            else blo[x - 4] = blo[x - 4] & (int)0xf0f0f0f0;
        } else if (kind == W_HI) {
            if (x < 4) opa[cur][x] = opa[cur][x] & (int)0xf0f0f0f0;
            else opb[cur][x - 4] = opb[cur][x - 4] & (int)0xf0f0f0f0;
        }
    };
    auto slice = [&](int cur, const uint8_t* ra, const uint8_t* rb, int rks, auto rd_tag, auto kind_tag, int copy_stage,
                     int copy_slot) {
        constexpr bool rd = decltype(rd_tag)::value;
        constexpr int kind = decltype(kind_tag)::value;
        constexpr int C = (kind == 0) ? 0 : ((kind == 2 || kind == 3) ? A_BLOCKS / 2 : B_BLOCKS / 2);
        constexpr int SLOTS = (MODE == MODE_I4) ? 2 * NM : NM;        // MFMA slots of the slice
        constexpr int S = SLOTS / (C == 0 ? SLOTS : C);
        static_assert(C == 0 || (SLOTS % C == 0 && S >= 1), "copies must tile the MFMA slots");
        static_assert(MODE != MODE_I4 || (FN == 4 && (FM == 4 || FM == 2)), "widening plans exist for these tiles");
#pragma unroll
        for (int sl = 0; sl < SLOTS; ++sl) {
            const int t = sl % NM, i = t / FN, j = t % FN;
            if constexpr (MODE == MODE_I8) {
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(opb[cur][j], opa[cur][i], acc[i][j], 0, 0, 0);
            } else if constexpr (MODE == MODE_I4) {
                if (sl < NM) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(blo[j], alo[i], acc[i][j], 0, 0, 0);
                else acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(opb[cur][j], opa[cur][i], acc[i][j], 0, 0, 0);
                if (sl < NM || rd) {
                    widen_step(widen_plan<FM>(sl, 0), cur);
                    widen_step(widen_plan<FM>(sl, 1), cur);
                }
            } else {
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, opb[cur][j]),
                                                                   __builtin_bit_cast(v8bf, opa[cur][i]), acc[i][j], 0, 0, 0);
            }
            if constexpr (rd) {
                if constexpr (MODE == MODE_I4) {
                    if (sl >= NM && t < NR) read_op(ra, rb, rks, cur ^ 1, t);     // one read per slot from the high pass on
                } else {
#pragma unroll
                    for (int q = t * NR / NM; q < (t + 1) * NR / NM; ++q) read_op(ra, rb, rks, cur ^ 1, q);
                }
            }
            if constexpr (C != 0) {
                if (sl % S == (W * (S / 4 > 0 ? S / 4 : 1)) % S) {
                    const int q = sl / S;
                    if constexpr (kind == 1) issue_b(copy_stage, copy_slot, B_BLOCKS / 2 + q);
                    else if constexpr (kind == 2) issue_a(copy_stage, copy_slot, q);
                    else if constexpr (kind == 3) issue_a(copy_stage, copy_slot, A_BLOCKS / 2 + q);
                    else issue_b(copy_stage, copy_slot, q);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    typedef std::true_type yes;
    typedef std::false_type no;
    typedef std::integral_constant<int, 0> k0;
    typedef std::integral_constant<int, 1> k1;
    typedef std::integral_constant<int, 2> k2;
    typedef std::integral_constant<int, 3> k3;
    typedef std::integral_constant<int, 4> k4;

    // prologue: stages 0 and 1 entire (A ring slots 0, 1; B ring slots 0, 1), wait for stage 0
#pragma unroll
    for (int j = 0; j < A_BLOCKS; ++j) issue_a(0, 0, j);
#pragma unroll
    for (int j = 0; j < B_BLOCKS; ++j) issue_b(0, 0, j);
    if (nk > 1) {
#pragma unroll
        for (int j = 0; j < A_BLOCKS; ++j) issue_a(1, 1, j);
#pragma unroll
        for (int j = 0; j < B_BLOCKS; ++j) issue_b(1, 1, j);
        constexpr int KEEP = A_BLOCKS + B_BLOCKS;
        __builtin_amdgcn_s_waitcnt((KEEP & 0xf) | ((KEEP >> 4) << 14) | 0x0070);
    } else {
        __builtin_amdgcn_s_waitcnt(0x0070);
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < NR; ++r) read_op(smem, smem + B_BASE, 0, 0, r);
    if constexpr (MODE == MODE_I4) {
        alo[0] = widen_lo(opa[0][0]);
#pragma unroll
        for (int j = 0; j < FN; ++j) blo[j] = widen_lo(opb[0][j]);
    }
    __builtin_amdgcn_sched_barrier(0);

    int ia = 0, ib = 0;                              // ring slots of the stage being multiplied
    // One stage, straight-line for its three compile-time flags: MB = the second half of B(kt+1) is still to be
    // issued (every stage but the first and the last), MA = stage kt+2 exists, NEXT = stage kt+1 exists.
    auto stage = [&](int kt, auto mb_tag, auto ma_tag, auto next_tag) {
        constexpr bool MB = decltype(mb_tag)::value, MA = decltype(ma_tag)::value;
        const int ia1 = (ia == 2) ? 0 : ia + 1, ia2 = (ia1 == 2) ? 0 : ia1 + 1;
        const uint8_t* sa = smem + ia * A_UNIT;
        const uint8_t* sb = smem + B_BASE + ib * B_UNIT;
        const uint8_t* sa_next = smem + ia1 * A_UNIT;
        const uint8_t* sb_next = smem + B_BASE + (ib ^ 1) * B_UNIT;
        slice(0, sa, sb, 1, yes{}, std::integral_constant<int, MB ? 1 : 0>{}, kt + 1, ib ^ 1);
        slice(1, sa, sb, 2, yes{}, std::integral_constant<int, MA ? 2 : 0>{}, kt + 2, ia2);
        slice(0, sa, sb, 3, yes{}, std::integral_constant<int, MA ? 3 : 0>{}, kt + 2, ia2);
        // slice 3 is in registers; stage kt+1 has landed: everything but the copies of A(kt+2), the youngest
        if constexpr (MA) __builtin_amdgcn_s_waitcnt((A_BLOCKS & 0xf) | ((A_BLOCKS >> 4) << 14) | 0x0070);
        else __builtin_amdgcn_s_waitcnt(0x0070);
        __syncthreads();
        slice(1, sa_next, sb_next, 0, next_tag, std::integral_constant<int, MA ? 4 : 0>{}, kt + 2, ib);
        ia = ia1;
        ib ^= 1;
    };
    int kt = 0;
    for (; kt < 1 && kt + 2 < nk; ++kt) stage(kt, no{}, yes{}, yes{});      // the first stage of three or more
    for (; kt < 1 && kt + 1 < nk; ++kt) stage(kt, no{}, no{}, yes{});       // the first stage of two
    for (; kt + 2 < nk; ++kt) stage(kt, yes{}, yes{}, yes{});               // the steady state
    for (; kt + 1 < nk; ++kt) stage(kt, yes{}, no{}, yes{});                // the last but one
    for (; kt < nk; ++kt) stage(kt, no{}, no{}, no{});                      // the last stage
    __syncthreads();                                 // every wave is past its last LDS operand read

    store_tile<MODE, FM, FN, 2, ONLY_BF16>(acc, m0 + wm * TM, n0 + wn * TN, M, N, scale, Y, y_dtype, ldy,
                                smem + W * (64 * TN * 2), bias);
}

// Workgroups [0, n_main) compute 256 x 256 tiles; a last, partly filled round of at most half the CUs is
// computed as 128 x 256 halves by workgroups [n_main, n_main + 2 n_tail).
template <int MODE, bool ONLY_BF16>
__global__ __launch_bounds__(256) void gemm_deep_kernel(const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, int M,
                                                        int N, int rowbytes, const float* __restrict__ s_x,
                                                        const float* __restrict__ s_w, void* __restrict__ Y, int y_dtype,
                                                        int ldy, int tiles_m, int tiles_n, int n_main, Batch bt)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const ClockProbe probe(bt.ticks);
    A += (size_t)blockIdx.y * bt.stride_a;
    B += (size_t)blockIdx.y * bt.stride_b;
    Y = static_cast<uint8_t*>(Y) + (size_t)blockIdx.y * bt.stride_y;
    int tile_m, tile_n;
    const int v = blockIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (v < n_main) {
        tile_of_workgroup(v, n_main, tiles_m, tiles_n, tile_m, tile_n);
        const int m0 = tile_m * 256, n0 = tile_n * 256;
        switch (wave) {
        case 0: gemm_deep_tile<MODE, 256, 256, ONLY_BF16, 0>(smem, m0, n0, A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt.bias); break;
        case 1: gemm_deep_tile<MODE, 256, 256, ONLY_BF16, 1>(smem, m0, n0, A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt.bias); break;
        case 2: gemm_deep_tile<MODE, 256, 256, ONLY_BF16, 2>(smem, m0, n0, A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt.bias); break;
        default: gemm_deep_tile<MODE, 256, 256, ONLY_BF16, 3>(smem, m0, n0, A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt.bias); break;
        }
    } else {
        const int t = v - n_main;
        tile_of_logical(n_main + (t >> 1), tiles_m, tiles_n, tile_m, tile_n);
        const int m0 = tile_m * 256 + (t & 1) * 128, n0 = tile_n * 256;
        switch (wave) {
        case 0: gemm_deep_tile<MODE, 128, 256, ONLY_BF16, 0>(smem, m0, n0, A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt.bias); break;
        case 1: gemm_deep_tile<MODE, 128, 256, ONLY_BF16, 1>(smem, m0, n0, A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt.bias); break;
        case 2: gemm_deep_tile<MODE, 128, 256, ONLY_BF16, 2>(smem, m0, n0, A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt.bias); break;
        default: gemm_deep_tile<MODE, 128, 256, ONLY_BF16, 3>(smem, m0, n0, A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt.bias); break;
        }
    }
    probe.finish(bt.ticks);
}

#if FQ_GEMM_MODE == 3
// =============================================================================================
// gemm_f6_wide_kernel: 4-bit operands stored as 6-bit E3M2 codes, multiplied on the 6-bit matrix pipe
// =============================================================================================
// v_mfma_scale_f32_32x32x64_f8f6f4 with both operands in the E3M2 format runs at twice the INT8 rate.
// E3M2 represents every integer in [-8, 8] exactly, products are integers of magnitude <= 64 and
// the fp32 accumulator stays exact below 2^24 (Kpad < 131072 is enforced), so the result equals the
// integer GEMM bit for bit.  A lane's operand is 32 consecutive k-values = 24 bytes (6 VGPRs); lane l
// holds row (l % 32), k-values 32 (l / 32) .. +31 of the 64-deep k-slice.
//
// Storage (written by the quantizer) is shaped by three facts measured on this chip:
//   - blocked along k: block t holds, for every row in turn, the 96 bytes of its codes 128 t .. 128 t + 127
//     (address (t * rows + row) * 96), so one k-stage of a tile operand is one contiguous run of 256 * 96
//     bytes of whole cache lines.  Row-major rows make every 96-byte piece straddle 128-byte lines, which
//     more than doubled the traffic between L2 and the compute units and capped the kernel there.
//   - a 48-byte group (one k-slice of a row) is stored X_a Y_a Y_b X_b, X / Y = first 16 / last 8 bytes of
//     a 32-code unit's bit stream: each lane finds its 24 bytes as one aligned 16-byte and one aligned
//     8-byte piece, in register order, whichever k-half it serves (no selects).
//   - (a, b) = (0, 1) in rows with bit 4 clear, (1, 0) otherwise.  LDS has 64 banks of 4 bytes; an 8-byte
//     read serves 32 lanes per pass, and rows 16 apart (1536 bytes) share their banks: the exchange moves
//     the 8-byte pieces of rows 16..31 of a fragment to the other half of the 16-byte bank pair.
// In LDS rows stay 96 bytes apart, which repeats the bank alignment every 8 rows; rows with
// (bit 2 ^ bit 3) set hold their two groups in swapped order (done by the copy: each lane of a direct
// global->LDS copy fetches the 16-byte chunk that belongs at its LDS position).  Among the layouts of
// this family, this pair of rules is one of those for which a probe kernel measured both reads at full
// rate (4 cycles per 16-byte, 2.5 per 8-byte wave-read).
//
// Four waves (2 x 2) with wave tiles of 128 x 128: every operand fetched from LDS feeds four MFMAs, i.e. 1/2
// of an operand per MFMA (an eight-wave ping-pong schedule with 128 x 64 wave tiles needs 3/4, was bound by
// those reads at this pipe's rate and measured 25 % slower).  One wave per SIMD: the LDS reads of the next
// k-slice and their selects are issued between the MFMAs of the current one (operands double-buffered
// in registers).  Three stage buffers; the barrier sits in the middle of a stage, after the reads of
// its second slice: it publishes stage kt+1 (each wave waited for its own copies), frees stage kt's
// buffer for the copy of stage kt+3, and lets the MFMAs of the second slice overlap the first reads
// of stage kt+1.
template <int BM, int BN, bool ONLY_BF16>
__device__ __forceinline__ void gemm_f6_wide_tile(uint8_t* smem, int m0, int n0, const uint8_t* __restrict__ A,
                                                  const uint8_t* __restrict__ B, int M, int N, int rowbytes,
                                                  const float* __restrict__ s_x, const float* __restrict__ s_w,
                                                  void* __restrict__ Y, int y_dtype, int ldy,
                                                  const float* __restrict__ bias)
{
    constexpr int WM = 2, WN = 2, NW = 4, NSTAGE = 3;
    constexpr int SB = 96, CPR = SB / 16;
    constexpr int STAGE = (BM + BN) * SB;
    constexpr int A_BLOCKS = BM * CPR / 64 / NW, B_BLOCKS = BN * CPR / 64 / NW;
    constexpr int LPS = A_BLOCKS + B_BLOCKS;
    constexpr int TM = BM / WM, TN = BN / WN, FM = TM / 32, FN = TN / 32;
    constexpr int NR = FM + FN;                      // operands of one k-slice
    constexpr int NM = FM * FN;                      // MFMAs of one k-slice
    constexpr int WAIT_ONE = (LPS & 0xf) | ((LPS >> 4) << 14) | 0x0f70;          // vmcnt(LPS): one stage may be in flight
    constexpr int WAIT_TWO = ((2 * LPS) & 0xf) | (((2 * LPS) >> 4) << 14) | 0x0f70;
    constexpr int WAIT_ALL = 0x0f70;
    static_assert((BM * CPR) % (64 * NW) == 0 && (BN * CPR) % (64 * NW) == 0, "copy blocks must tile the stage");
    static_assert(2 * LPS < 64 && 2 * NR <= 2 * NM && LPS <= 2 * NM, "pipeline shape");
    typedef v16f acc_t;
    const float scale = tile_scale<MODE_F6>(s_x, s_w);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int nk = rowbytes / SB;
    const size_t blockA = (size_t)M * SB, blockB = (size_t)N * SB;

    uint32_t offA[A_BLOCKS], offB[B_BLOCKS];
#pragma unroll
    for (int j = 0; j < A_BLOCKS; ++j) {
        const int c = 64 * (wave + j * NW) + lane, row = c / CPR, pos = c % CPR;
        const int gc = (((row >> 2) ^ (row >> 3)) & 1) ? (pos + 3) % CPR : pos;
        offA[j] = (uint32_t)min(m0 + row, M - 1) * (uint32_t)SB + gc * 16;
    }
#pragma unroll
    for (int j = 0; j < B_BLOCKS; ++j) {
        const int c = 64 * (wave + j * NW) + lane, row = c / CPR, pos = c % CPR;
        const int gc = (((row >> 2) ^ (row >> 3)) & 1) ? (pos + 3) % CPR : pos;
        offB[j] = (uint32_t)min(n0 + row, N - 1) * (uint32_t)SB + gc * 16;
    }
    const uint32_t lds0 = (uint32_t)(size_t)FQ_LDS_PTR(smem) + wave * 1024;
    auto issue_any = [&](int stage_index) {
        const uint32_t sA = lds0 + (stage_index % NSTAGE) * STAGE;
        const uint32_t sB = sA + BM * SB;
        const uint8_t* gA = A + stage_index * blockA;
        const uint8_t* gB = B + stage_index * blockB;
#pragma unroll
        for (int j = 0; j < A_BLOCKS; ++j) dma16(gA, offA[j], sA + j * NW * 1024);
#pragma unroll
        for (int j = 0; j < B_BLOCKS; ++j) dma16(gB, offB[j], sB + j * NW * 1024);
    };

    // copy instruction `idx` (0 .. LPS-1) of a stage: the A blocks, then the B blocks
    auto issue_one = [&](int stage_index, int idx) {
        const uint32_t sA = lds0 + (stage_index % NSTAGE) * STAGE;
        if (idx < A_BLOCKS) dma16(A + stage_index * blockA, offA[idx], sA + idx * NW * 1024);
        else dma16(B + stage_index * blockB, offB[idx - A_BLOCKS], sA + BM * SB + (idx - A_BLOCKS) * NW * 1024);
    };

    // operand read offsets.  A 48-byte group is stored X_a Y_a Y_b X_b (X: first 16, Y: last 8 bytes of a 32-code
    // unit's stream) with (a, b) = (0, 1) in rows with bit 4 clear, (1, 0) otherwise: the lane of k-half h takes
    // X at 0 / Y at 16 or X at 32 / Y at 24, both reads naturally aligned
    const int frow = lane & 31, fhalf = lane >> 5;
    const int swp = ((frow >> 2) ^ (frow >> 3)) & 1;
    const int mirrored = (fhalf ^ (frow >> 4)) & 1;      // the lane's unit is the second one stored in its group
    const int a_rd = (wm * TM + frow) * SB, b_rd = BM * SB + (wn * TN + frow) * SB;
    int xofs[2], yofs[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        xofs[ks] = 48 * (ks ^ swp) + (mirrored ? 32 : 0);
        yofs[ks] = 48 * (ks ^ swp) + (mirrored ? 24 : 16);
    }

    acc_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // operands of a k-slice in the order the MFMA walk (i outer, j inner) first needs them: a0, b0..b3, a1..a3
    v8i opa[2][FM], opb[2][FN];
    auto op_addr = [&](const uint8_t* st, int r) -> const uint8_t* {
        return (r == 0) ? st + a_rd : (r <= FN ? st + b_rd + (r - 1) * 32 * SB : st + a_rd + (r - FN) * 32 * SB);
    };
    // operand r of a slice, read in two steps (the 16-byte piece, then the 8-byte piece)
    auto set_op = [&](int buf, int r) -> v8i& {
        return (r == 0) ? opa[buf][0] : (r <= FN ? opb[buf][r - 1] : opa[buf][r - FN]);
    };
    auto read_x = [&](const uint8_t* st, int ks, int buf, int r) {
        const v4i x = *reinterpret_cast<const v4i*>(op_addr(st, r) + xofs[ks]);
        v8i& o = set_op(buf, r);
        o[0] = x[0]; o[1] = x[1]; o[2] = x[2]; o[3] = x[3];
    };
    auto read_y = [&](const uint8_t* st, int ks, int buf, int r) {
        const v2i y = *reinterpret_cast<const v2i*>(op_addr(st, r) + yofs[ks]);
        v8i& o = set_op(buf, r);
        o[4] = y[0]; o[5] = y[1]; o[6] = 0; o[7] = 0;
    };
    auto read_op = [&](const uint8_t* st, int ks, int buf, int r) {
        read_x(st, ks, buf, r);
        read_y(st, ks, buf, r);
    };
    // `copy_stage` >= 0: the copy instructions of that stage are issued one per MFMA, after the reads
    auto slice = [&](int cur, const uint8_t* rs, int rks, auto rd_tag, auto copy_tag, int copy_stage) {
        constexpr bool rd = decltype(rd_tag)::value;
        constexpr bool cp = decltype(copy_tag)::value;
#pragma unroll
        for (int t = 0; t < NM; ++t) {
            const int i = t / FN, j = t % FN;
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(opb[cur][j], opa[cur][i], acc[i][j], 3, 3, 0, 127, 0, 127);
            // The 2 NR LDS reads of the next slice's operands (16-byte, then 8-byte piece of operand 0, 1, ...)
            // and the LPS copy instructions are spread evenly over the NM MFMA slots.  An operand is needed
            // by the next slice's MFMA 0 (operands 0, 1), MFMA j (operand 1 + j) or MFMA FN i (operand FN + i):
            // always a full slice after its read.
            if constexpr (rd) {
#pragma unroll
                for (int q = t * (2 * NR) / NM; q < (t + 1) * (2 * NR) / NM; ++q) {
                    if (q & 1) read_y(rs, rks, cur ^ 1, q >> 1);
                    else read_x(rs, rks, cur ^ 1, q >> 1);
                }
            }
            if constexpr (cp) {
#pragma unroll
                for (int q = t * LPS / NM; q < (t + 1) * LPS / NM; ++q) issue_one(copy_stage, q);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

#pragma unroll
    for (int st = 0; st < NSTAGE; ++st)
        if (st < nk) issue_any(st);
    if (nk >= 3) __builtin_amdgcn_s_waitcnt(WAIT_TWO);
    else if (nk == 2) __builtin_amdgcn_s_waitcnt(WAIT_ONE);
    else __builtin_amdgcn_s_waitcnt(WAIT_ALL);
    __syncthreads();
#pragma unroll
    for (int r = 0; r < NR; ++r) read_op(smem, 0, 0, r);
    __builtin_amdgcn_sched_barrier(0);

    typedef std::true_type yes;
    typedef std::false_type no;
    int buf = 0;
    // one stage: slice 0 (reads slice 1 of the stage), the barrier, slice 1 (reads slice 0 of the next
    // stage and, when `copy_tag`, copies stage kt+3 into the buffer the barrier freed)
    auto stage = [&](int kt, auto copy_tag) {
        const uint8_t* s = smem + buf * STAGE;
        buf = (buf + 1 == NSTAGE) ? 0 : buf + 1;
        const uint8_t* sn = smem + buf * STAGE;
        slice(0, s, 1, yes{}, no{}, 0);
        // slice 1 of stage kt is in registers: its buffer is free, and stage kt+1 must be complete
        if (kt + 2 < nk) __builtin_amdgcn_s_waitcnt(WAIT_ONE & 0xc07f);     // + lgkmcnt(0)
        else __builtin_amdgcn_s_waitcnt(WAIT_ALL & 0xc07f);
        __syncthreads();
        slice(1, sn, 0, yes{}, copy_tag, kt + NSTAGE);
    };
    int kt = 0;
    for (; kt + NSTAGE < nk; ++kt) stage(kt, yes{});
    for (; kt + 1 < nk; ++kt) stage(kt, no{});
    {   // last stage: nothing further to read
        const uint8_t* s = smem + buf * STAGE;
        slice(0, s, 1, yes{}, no{}, 0);
        slice(1, s, 0, no{}, no{}, 0);
    }
    __syncthreads();                                // every wave is past its last LDS operand read

    store_tile<MODE_F6, FM, FN, 2, ONLY_BF16>(acc, m0 + wm * TM, n0 + wn * TN, M, N, scale, Y, y_dtype, ldy,
                                   smem + wave * (64 * TN * 2), bias);
}

// Workgroups [0, n_main) compute 256 x 256 tiles; a last, partly filled round of at most half the CUs is
// computed as 128 x 256 halves by workgroups [n_main, n_main + 2 n_tail), so that it takes about half as long.
template <bool ONLY_BF16>
__global__ __launch_bounds__(256) void gemm_f6_wide_kernel(const uint8_t* __restrict__ A, const uint8_t* __restrict__ B,
                                                           int M, int N, int rowbytes, const float* __restrict__ s_x,
                                                           const float* __restrict__ s_w, void* __restrict__ Y,
                                                           int y_dtype, int ldy, int tiles_m, int tiles_n, int n_main,
                                                           Batch bt)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const ClockProbe probe(bt.ticks);
    A += (size_t)blockIdx.y * bt.stride_a;
    B += (size_t)blockIdx.y * bt.stride_b;
    Y = static_cast<uint8_t*>(Y) + (size_t)blockIdx.y * bt.stride_y;
    int tile_m, tile_n;
    const int v = blockIdx.x;
    if (v < n_main) {
        tile_of_workgroup(v, n_main, tiles_m, tiles_n, tile_m, tile_n);
        gemm_f6_wide_tile<256, 256, ONLY_BF16>(smem, tile_m * 256, tile_n * 256, A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy,
                                    bt.bias);
    } else {
        const int t = v - n_main;
        tile_of_logical(n_main + (t >> 1), tiles_m, tiles_n, tile_m, tile_n);
        gemm_f6_wide_tile<128, 256, ONLY_BF16>(smem, tile_m * 256 + (t & 1) * 128, tile_n * 256, A, B, M, N, rowbytes, s_x, s_w, Y,
                                    y_dtype, ldy, bt.bias);
    }
    probe.finish(bt.ticks);
}

#endif  // FQ_GEMM_MODE == 3

// =============================================================================================
// gemm_reg_kernel: global -> registers -> LDS
// =============================================================================================
template <int MODE, int BM, int BN, int BKB, int WM, int WN>
__global__ __launch_bounds__(WM* WN * 64) void gemm_reg_kernel(const uint8_t* __restrict__ A,
                                                                const uint8_t* __restrict__ B, int M, int N,
                                                                int rowbytes, const float* __restrict__ s_x,
                                                                const float* __restrict__ s_w,
                                                                void* __restrict__ Y, int y_dtype, int ldy,
                                                                int tiles_m, int tiles_n, Batch bt)
{
    const ClockProbe probe(bt.ticks);
    A += (size_t)blockIdx.y * bt.stride_a;
    B += (size_t)blockIdx.y * bt.stride_b;
    Y = static_cast<uint8_t*>(Y) + (size_t)blockIdx.y * bt.stride_y;
    constexpr int NT = WM * WN * 64;
    constexpr int CPR = BKB / 16;          // chunks per row per stage
    constexpr int RPP = NT / CPR;          // rows covered by one pass of the loader
    constexpr int A_LOADS = BM / RPP;
    constexpr int B_LOADS = BN / RPP;
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int FM = TM / 32, FN = TN / 32;
    constexpr int KS = BKB / 32;           // 32-byte k-slices per stage
    constexpr int STAGE = (BM + BN) * BKB;
    constexpr int SWZ_SHIFT = (CPR == 8) ? 1 : 2;
    constexpr int SWZ_MASK = CPR - 1;
    static_assert(BM % RPP == 0 && BN % RPP == 0, "loader does not tile the block");
    static_assert(RPP % 16 == 0, "swizzle must repeat across loader passes");
    static_assert(CPR == 4 || CPR == 8, "BKB must be 64 or 128");
    typedef typename Acc<MODE>::type acc_t;
    const float scale = tile_scale<MODE>(s_x, s_w);

    extern __shared__ __align__(16) uint8_t smem[];

    int tile_m, tile_n;
    tile_of_workgroup(blockIdx.x, gridDim.x, tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // ---- loader mapping: thread -> (row lr + i*RPP, chunk lc) ----
    const int lc = tid % CPR, lr = tid / CPR;
    const uint8_t* gA[A_LOADS];
    const uint8_t* gB[B_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) gA[i] = A + (size_t)min(m0 + lr + i * RPP, M - 1) * rowbytes + lc * 16;
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) gB[i] = B + (size_t)min(n0 + lr + i * RPP, N - 1) * rowbytes + lc * 16;
    const int wofs = lr * BKB + ((lc ^ ((lr >> SWZ_SHIFT) & SWZ_MASK)) << 4);

    // ---- fragment read offsets ----
    const int frow = lane & 31, fhalf = lane >> 5;
    const int fsw = (frow >> SWZ_SHIFT) & SWZ_MASK;
    int kofs[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kofs[ks] = ((2 * ks + fhalf) ^ fsw) << 4;
    const int a_rd = (wm * TM + frow) * BKB;
    const int b_rd = BM * BKB + (wn * TN + frow) * BKB;

    acc_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    const int nk = (rowbytes + BKB - 1) / BKB;
    v4i ra[A_LOADS], rb[B_LOADS];

    auto load_global = [&](int kt) {
        const int kb = kt * BKB;
        const bool ok = kb + lc * 16 < rowbytes;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i)
            ra[i] = ok ? *reinterpret_cast<const v4i*>(gA[i] + kb) : v4i{0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i)
            rb[i] = ok ? *reinterpret_cast<const v4i*>(gB[i] + kb) : v4i{0, 0, 0, 0};
    };
    auto store_lds = [&](int stage) {
        uint8_t* s = smem + stage * STAGE;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) *reinterpret_cast<v4i*>(s + wofs + i * RPP * BKB) = ra[i];
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i) *reinterpret_cast<v4i*>(s + BM * BKB + wofs + i * RPP * BKB) = rb[i];
    };

    load_global(0);
    store_lds(0);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const uint8_t* s = smem + (kt & 1) * STAGE;
        if (kt + 1 < nk) load_global(kt + 1);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            v4i a[FM], b[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) a[i] = *reinterpret_cast<const v4i*>(s + a_rd + i * 32 * BKB + kofs[ks]);
#pragma unroll
            for (int j = 0; j < FN; ++j) b[j] = *reinterpret_cast<const v4i*>(s + b_rd + j * 32 * BKB + kofs[ks]);
            mfma_slice<MODE, FM, FN>(a, b, acc);
        }
        if (kt + 1 < nk) store_lds((kt + 1) & 1);
        __syncthreads();
    }

    store_tile<MODE, FM, FN>(acc, m0 + wm * TM, n0 + wn * TN, M, N, scale, Y, y_dtype, ldy, nullptr, bt.bias);
    probe.finish(bt.ticks);
}

// Raises a kernel's dynamic-LDS limit once per device.  `done` holds one bit per device ordinal (mod 64); a race
// between two threads only repeats the idempotent call.
int set_lds_limit(const void* kern, int smem, std::atomic<unsigned long long>& done)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(FQ_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    const unsigned long long bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return FQ_OK;
    e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return fail(FQ_ERR_HIP, "hipFuncSetAttribute(%d bytes LDS): %s", smem, hipGetErrorString(e));
    done.fetch_or(bit, std::memory_order_release);
    return FQ_OK;
}

// Compute units of the current device (cached per device ordinal).
int compute_units()
{
    static std::atomic<int> cus[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    std::atomic<int>& slot = cus[dev & 63];
    int n = slot.load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        slot.store(n, std::memory_order_relaxed);
    }
    return n;
}

template <int MODE, int BM, int BN, int BKB, int WM, int WN, int NSTAGE, int PIPE, int PP_SLICES = 2, bool ONLY_BF16 = false>
int launch_dma(const void* A, const void* B, int M, int N, int rowbytes, const float* s_x, const float* s_w,
               void* Y, int y_dtype, int ldy, Batch bt, hipStream_t stream)
{
    // the DMA kernel addresses rows with 32-bit byte offsets
    if ((unsigned long long)M * rowbytes >= (1ull << 32) || (unsigned long long)N * rowbytes >= (1ull << 32))
        return fail(FQ_ERR_RANGE, "operand larger than 4 GiB");
    auto kern = gemm_dma_kernel<MODE, BM, BN, BKB, WM, WN, NSTAGE, PIPE, PP_SLICES, ONLY_BF16>;
    constexpr int smem = NSTAGE * (BM + BN) * BKB;
    static std::atomic<unsigned long long> attr_set{0};
    if (int rc = set_lds_limit(reinterpret_cast<const void*>(kern), smem, attr_set)) return rc;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const long long tiles = (long long)tiles_m * tiles_n;
    if (tiles > 0x3fffffffLL) return fail(FQ_ERR_RANGE, "too many tiles");
    // a last round that would occupy at most half of the CUs is run as half-height tiles instead
    constexpr bool HALF_OK = BM >= 128 && (BM / 2) % (64 / (BKB / 16) * WM * WN) == 0;
    const int cus = compute_units();
    const int r = (int)(tiles % cus);
    int n_main = (int)tiles, n_tail = 0;
    if (HALF_OK && bt.count == 1 && r > 0 && 2 * r <= cus) {
        n_tail = r;
        n_main = (int)tiles - r;
    }
    // The two-buffer ping-pong kernel runs one workgroup per CU that walks its tiles in rounds and
    // prefetches across tile boundaries; the others get one workgroup per tile.
    constexpr bool PERSISTENT = PIPE == 2 && NSTAGE == 2;
    int grid_x = n_main + 2 * n_tail;
    if (PERSISTENT && bt.count == 1 && grid_x > cus) grid_x = cus;
    kern<<<dim3((unsigned)grid_x, (unsigned)bt.count), dim3(WM * WN * 64), smem, stream>>>(
        static_cast<const uint8_t*>(A), static_cast<const uint8_t*>(B), M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy,
        tiles_m, tiles_n, n_main, n_tail, bt);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FQ_ERR_HIP, "GEMM launch failed: %s", hipGetErrorString(e));
    return FQ_OK;
}

template <int MODE, int BM, int BN, int BKB, int WM, int WN>
int launch_reg(const void* A, const void* B, int M, int N, int rowbytes, const float* s_x, const float* s_w,
               void* Y, int y_dtype, int ldy, Batch bt, hipStream_t stream)
{
    auto kern = gemm_reg_kernel<MODE, BM, BN, BKB, WM, WN>;
    constexpr int smem = 2 * (BM + BN) * BKB;
    static std::atomic<unsigned long long> attr_set{0};
    if (int rc = set_lds_limit(reinterpret_cast<const void*>(kern), smem, attr_set)) return rc;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const long long tiles = (long long)tiles_m * tiles_n;
    if (tiles > 0x7fffffffLL) return fail(FQ_ERR_RANGE, "too many tiles");
    kern<<<dim3((unsigned)tiles, (unsigned)bt.count), dim3(WM * WN * 64), smem, stream>>>(
        static_cast<const uint8_t*>(A), static_cast<const uint8_t*>(B), M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy,
        tiles_m, tiles_n, bt);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FQ_ERR_HIP, "GEMM launch failed: %s", hipGetErrorString(e));
    return FQ_OK;
}

// gemm_wide_kernel has no packed-nibble form: only the deep kernel is instantiated for MODE_I4
template <int MODE, bool DEEP>
auto pick_wide_kernel(bool only_bf16)
{
    if constexpr (DEEP) return only_bf16 ? gemm_deep_kernel<MODE, true> : gemm_deep_kernel<MODE, false>;
    else return only_bf16 ? gemm_wide_kernel<MODE, true> : gemm_wide_kernel<MODE, false>;
}

template <int MODE, bool DEEP = false>
int launch_wide(const void* A, const void* B, int M, int N, int rowbytes, const float* s_x, const float* s_w, void* Y,
                int y_dtype, int ldy, Batch bt, hipStream_t stream)
{
    if constexpr (MODE == MODE_I8 || MODE == MODE_BF16 || (MODE == MODE_I4 && DEEP)) {
        if ((unsigned long long)M * rowbytes >= (1ull << 32) || (unsigned long long)N * rowbytes >= (1ull << 32))
            return fail(FQ_ERR_RANGE, "operand larger than 4 GiB");
        if (rowbytes % 128) return fail(FQ_ERR_SHAPE, "GEMM variants 11 and 12 need rows of whole 128-byte stages");
        // the common case (bf16 output, no bias) has an instantiation with that epilogue only
        const bool only_bf16 = y_dtype == FQ_BF16 && !bt.bias;
        auto kern = pick_wide_kernel<MODE, DEEP>(only_bf16);
        // two stage buffers of 64 KiB, or (deep) three A and two B buffers of 32 KiB: all of the CU's LDS
        constexpr int smem = DEEP ? 5 * 256 * 128 : 2 * 512 * 128;
        static std::atomic<unsigned long long> attr_set[2];
        if (int rc = set_lds_limit(reinterpret_cast<const void*>(kern), smem, attr_set[only_bf16 ? 1 : 0])) return rc;
        const int tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256;
        const long long tiles = (long long)tiles_m * tiles_n;
        if (tiles > 0x3fffffffLL) return fail(FQ_ERR_RANGE, "too many tiles");
        // a last round that would occupy at most half of the CUs is run as half-height tiles instead
        const int cus = compute_units();
        const int r = (int)(tiles % cus);
        int n_main = (int)tiles, n_tail = 0;
        if (bt.count == 1 && r > 0 && 2 * r <= cus) {
            n_tail = r;
            n_main = (int)tiles - r;
        }
        kern<<<dim3((unsigned)(n_main + 2 * n_tail), (unsigned)bt.count), dim3(256), smem, stream>>>(
            static_cast<const uint8_t*>(A), static_cast<const uint8_t*>(B), M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy,
            tiles_m, tiles_n, n_main, bt);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(FQ_ERR_HIP, "GEMM launch failed: %s", hipGetErrorString(e));
        return FQ_OK;
    } else {
        return fail(FQ_ERR_RANGE, "GEMM variant 11 exists for INT8 and bf16 operands only, 12 also for packed nibbles");
    }
}

template <int MODE>
int dispatch(const void* A, const void* B, int M, int N, int rowbytes, const float* s_x, const float* s_w,
             void* Y, int y_dtype, int ldy, Batch bt, hipStream_t stream)
{
    if (bt.count < 1 || bt.count > 65535) return fail(FQ_ERR_RANGE, "batch = %d must lie in [1, 65535]", bt.count);
    int v = forced_gemm_variant();
    if (v < 0) {
        const long long big_tiles = (long long)((M + 255) / 256) * ((N + 255) / 256) * bt.count;
        // The four-wave kernel with the deep staging (12) needs rows of whole 128-byte stages and exists with the
        // plain bf16 epilogue as its spill-free instantiation: taken for that output, without bias, unbatched.  On
        // large problems it gains +14 % over the ping-pong kernel at full clock for INT8 and bf16 (+3-5 % at the
        // clock the power limit leaves on live operands) and +1-5 % for packed nibbles.  Thresholds measured at
        // N = 4096 in steps of one tile row: INT8 takes it from 80 tiles on (its partly filled rounds run as
        // half-height tiles on twice as many CUs: 20 % faster than the 128 x 128 tile at 144-176 tiles), nibbles from
        // 176; otherwise the ping-pong kernel (long phases, 10, where the operand registers allow it: packed nibbles
        // with at least four k-stages; INT8 and bf16 would hold four unpacked k-slices per phase and spill, so they
        // keep two per phase, 7) from 144 / 112 tiles on; narrow outputs (N <= 128, the P V product of attention) and
        // small problems use the 128 x 128 tile (6).
        const bool deep_ok = MODE != MODE_F6 && rowbytes % 128 == 0 && bt.count == 1 && y_dtype == FQ_BF16 && !bt.bias;
        v = 6;
        if (N > 128) {
            if (MODE == MODE_I4 && rowbytes >= 512) {
                if (big_tiles >= 112) v = (big_tiles >= 176 && deep_ok) ? 12 : 10;
            } else if (MODE == MODE_I4) {
                if (big_tiles >= 192) v = 7;
            } else {
                if (big_tiles >= 80 && deep_ok) v = 12;
                else if (big_tiles >= 144) v = 7;
            }
        }
    }
    switch (v) {
    case 2: return launch_reg<MODE, 128, 128, 64, 2, 2>(A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt, stream);
    case 6: return launch_dma<MODE, 128, 128, 128, 2, 2, 2, 1>(A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt, stream);
    case 7:
        // the large-problem kernels have an instantiation with the plain bf16 epilogue only (no spills)
        if (MODE != MODE_BF16 && y_dtype == FQ_BF16 && !bt.bias)
            return launch_dma<MODE, 256, 256, 128, 2, 4, 2, 2, 2, true>(A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt, stream);
        return launch_dma<MODE, 256, 256, 128, 2, 4, 2, 2, 2>(A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt, stream);
    case 10:
        if (MODE != MODE_BF16 && y_dtype == FQ_BF16 && !bt.bias)
            return launch_dma<MODE, 256, 256, 128, 2, 4, 2, 2, 4, true>(A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt, stream);
        return launch_dma<MODE, 256, 256, 128, 2, 4, 2, 2, 4>(A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt, stream);
    case 11: return launch_wide<MODE>(A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt, stream);
    case 12: return launch_wide<MODE, true>(A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt, stream);
    default: return fail(FQ_ERR_RANGE, "unknown GEMM variant %d", v);
    }
}

}  // namespace

// This file is compiled once per operand mode (FQ_GEMM_MODE = 0 INT8, 1 packed INT4, 2 bf16, 3 E3M2), each
// translation unit holding that mode's kernels and exporting its dispatcher.
#ifndef FQ_GEMM_MODE
#error "compile with -DFQ_GEMM_MODE=0, 1, 2 or 3"
#endif
#if FQ_GEMM_MODE == 3
int gemm_dispatch_f6(const void* A, const void* B, int M, int N, int rowbytes, const float* s_x, const float* s_w,
                     void* Y, int y_dtype, int ldy, Batch bt, hipStream_t stream)
{
    if (bt.count < 1 || bt.count > 65535) return fail(FQ_ERR_RANGE, "batch = %d must lie in [1, 65535]", bt.count);
    if ((unsigned long long)M * rowbytes >= (1ull << 32) || (unsigned long long)N * rowbytes >= (1ull << 32))
        return fail(FQ_ERR_RANGE, "operand larger than 4 GiB");
    if (rowbytes % 96) return fail(FQ_ERR_SHAPE, "E3M2 rows must be whole 96-byte blocks");
    constexpr int smem = 3 * 512 * 96;
    const int tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256;
    const long long tiles = (long long)tiles_m * tiles_n;
    if (tiles > 0x3fffffffLL) return fail(FQ_ERR_RANGE, "too many tiles");
    // the common case (bf16 output, no bias) has an instantiation with that epilogue only
    const bool only_bf16 = y_dtype == FQ_BF16 && !bt.bias;
    auto kern = only_bf16 ? gemm_f6_wide_kernel<true> : gemm_f6_wide_kernel<false>;
    static std::atomic<unsigned long long> attr_set[2];
    if (int rc = set_lds_limit(reinterpret_cast<const void*>(kern), smem, attr_set[only_bf16 ? 1 : 0])) return rc;
    // a last round that would occupy at most half of the CUs is run as half-height tiles instead
    const int cus = compute_units();
    const int r = (int)(tiles % cus);
    int n_main = (int)tiles, n_tail = 0;
    if (bt.count == 1 && r > 0 && 2 * r <= cus) {
        n_tail = r;
        n_main = (int)tiles - r;
    }
    kern<<<dim3((unsigned)(n_main + 2 * n_tail), (unsigned)bt.count), dim3(256), smem, stream>>>(
        static_cast<const uint8_t*>(A), static_cast<const uint8_t*>(B), M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy,
        tiles_m, tiles_n, n_main, bt);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FQ_ERR_HIP, "GEMM launch failed: %s", hipGetErrorString(e));
    return FQ_OK;
}
#elif FQ_GEMM_MODE == 0
// =============================================================================================
// gemm_fused_a_kernel: flatten-quantize fused into the A-operand load (Sec. 6, the paper's future work)
// =============================================================================================
// gemm_reg_kernel (128 x 128 tile, 64-byte k-stages, four waves, operands staged through registers) with the
// loader of A replaced: a thread's 16-byte chunk of a quantized row is 16 flattened slots p0 .. p0 + 15, which it
// forms itself from X -- two 16-byte loads of bf16 when the group is 16 consecutive channels (gflag), 16 gathered
// elements X[row, src[p]] otherwise -- times the slots' multipliers, rounded half-to-even and clamped exactly as
// the separate quantizer does (one fp32 multiply per element), packed and written to the same LDS position.
// X'q never exists in memory.  Every column tile of the output converts its rows of X again.
namespace {
__device__ __forceinline__ int quantize_i8(float x, float m)
{
    float r = rintf(x * m);
    r = fminf(fmaxf(r, -128.0f), 127.0f);
    return (int)r;
}

template <int BM, int BN, int BKB, int WM, int WN>
__global__ __launch_bounds__(WM* WN * 64) void gemm_fused_a_kernel(const uint16_t* __restrict__ X, int ldx, int K,
                                                                    const int32_t* __restrict__ src,
                                                                    const float* __restrict__ mslot,
                                                                    const uint8_t* __restrict__ gflag,
                                                                    const uint8_t* __restrict__ B, int M, int N, int rowbytes,
                                                                    const float* __restrict__ s_x,
                                                                    const float* __restrict__ s_w, void* __restrict__ Y,
                                                                    int y_dtype, int ldy, int tiles_m, int tiles_n,
                                                                    const float* __restrict__ bias)
{
    constexpr int MODE = MODE_I8;
    constexpr int NT = WM * WN * 64;
    constexpr int CPR = BKB / 16, RPP = NT / CPR;
    constexpr int A_LOADS = BM / RPP, B_LOADS = BN / RPP;
    constexpr int TM = BM / WM, TN = BN / WN, FM = TM / 32, FN = TN / 32;
    constexpr int KS = BKB / 32;
    constexpr int STAGE = (BM + BN) * BKB;
    constexpr int SWZ_SHIFT = (CPR == 8) ? 1 : 2, SWZ_MASK = CPR - 1;
    static_assert(BM % RPP == 0 && BN % RPP == 0 && RPP % 16 == 0 && (CPR == 4 || CPR == 8), "loader layout");
    typedef typename Acc<MODE>::type acc_t;
    const float scale = tile_scale<MODE>(s_x, s_w);

    extern __shared__ __align__(16) uint8_t smem[];
    int tile_m, tile_n;
    tile_of_workgroup(blockIdx.x, gridDim.x, tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    const int lc = tid % CPR, lr = tid / CPR;
    const uint16_t* gX[A_LOADS];
    const uint8_t* gB[B_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) gX[i] = X + (size_t)min(m0 + lr + i * RPP, M - 1) * ldx;
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) gB[i] = B + (size_t)min(n0 + lr + i * RPP, N - 1) * rowbytes + lc * 16;
    const int wofs = lr * BKB + ((lc ^ ((lr >> SWZ_SHIFT) & SWZ_MASK)) << 4);

    const int frow = lane & 31, fhalf = lane >> 5;
    const int fsw = (frow >> SWZ_SHIFT) & SWZ_MASK;
    int kofs[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kofs[ks] = ((2 * ks + fhalf) ^ fsw) << 4;
    const int a_rd = (wm * TM + frow) * BKB;
    const int b_rd = BM * BKB + (wn * TN + frow) * BKB;

    acc_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    const int nk = (rowbytes + BKB - 1) / BKB;
    v4i rb[B_LOADS];
    uint32_t xa[A_LOADS][8];                     // 16 bf16 elements per row, two per register
    float mv[16];
    bool ok = false;

    auto load_global = [&](int kt) {
        const int p0 = kt * BKB + lc * 16;       // first of this thread's 16 slots
        ok = p0 < rowbytes;
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i)
            rb[i] = ok ? *reinterpret_cast<const v4i*>(gB[i] + kt * BKB) : v4i{0, 0, 0, 0};
        if (!ok) return;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const v4f m4 = *reinterpret_cast<const v4f*>(mslot + p0 + 4 * q);
#pragma unroll
            for (int e = 0; e < 4; ++e) mv[4 * q + e] = m4[e];
        }
        if (gflag[p0 >> 4]) {                    // 16 consecutive channels p0 .. p0 + 15
#pragma unroll
            for (int i = 0; i < A_LOADS; ++i) {
                const v4u lo = *reinterpret_cast<const v4u*>(gX[i] + p0), hi = *reinterpret_cast<const v4u*>(gX[i] + p0 + 8);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    xa[i][e] = lo[e];
                    xa[i][4 + e] = hi[e];
                }
            }
        } else {
            int sp[16];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const v4i s4 = *reinterpret_cast<const v4i*>(src + p0 + 4 * q);
#pragma unroll
                for (int e = 0; e < 4; ++e) sp[4 * q + e] = s4[e];
            }
#pragma unroll
            for (int i = 0; i < A_LOADS; ++i)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int c0 = sp[2 * e], c1 = sp[2 * e + 1];
                    const uint32_t v0 = ((unsigned)c0 < (unsigned)K) ? gX[i][c0] : 0u;
                    const uint32_t v1 = ((unsigned)c1 < (unsigned)K) ? gX[i][c1] : 0u;
                    xa[i][e] = v0 | (v1 << 16);
                }
        }
    };
    auto store_lds = [&](int stage) {
        uint8_t* s = smem + stage * STAGE;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) {
            v4i packed = {0, 0, 0, 0};
            if (ok) {
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    uint32_t word = 0;
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const int e = 4 * w + b;
                        const uint32_t raw = xa[i][e >> 1];
                        const float x = __uint_as_float((e & 1) ? (raw & 0xffff0000u) : (raw << 16));
                        word |= (uint32_t)(quantize_i8(x, mv[e]) & 0xff) << (8 * b);
                    }
                    packed[w] = (int)word;
                }
            }
            *reinterpret_cast<v4i*>(s + wofs + i * RPP * BKB) = packed;
        }
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i) *reinterpret_cast<v4i*>(s + BM * BKB + wofs + i * RPP * BKB) = rb[i];
    };

    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const uint8_t* s = smem + (kt & 1) * STAGE;
        if (kt + 1 < nk) load_global(kt + 1);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            v4i a[FM], b[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) a[i] = *reinterpret_cast<const v4i*>(s + a_rd + i * 32 * BKB + kofs[ks]);
#pragma unroll
            for (int j = 0; j < FN; ++j) b[j] = *reinterpret_cast<const v4i*>(s + b_rd + j * 32 * BKB + kofs[ks]);
            mfma_slice<MODE, FM, FN>(a, b, acc);
        }
        if (kt + 1 < nk) store_lds((kt + 1) & 1);
        __syncthreads();
    }
    store_tile<MODE, FM, FN>(acc, m0 + wm * TM, n0 + wn * TN, M, N, scale, Y, y_dtype, ldy, nullptr, bias);
}
}  // namespace

int launch_gemm_fused_a_i8(const void* X, int ldx, int K, const int32_t* src, const float* mslot, const uint8_t* gflag,
                           const void* Wq, int M, int N, int Kpad, const float* s_x, const float* s_w, void* Y,
                           int y_dtype, int ldy, const float* bias, hipStream_t stream)
{
    constexpr int BM = 128, BN = 128, BKB = 64;
    auto kern = gemm_fused_a_kernel<BM, BN, BKB, 2, 2>;
    constexpr int smem = 2 * (BM + BN) * BKB;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const long long tiles = (long long)tiles_m * tiles_n;
    if (tiles > 0x7fffffffLL) return fail(FQ_ERR_RANGE, "too many tiles");
    kern<<<dim3((unsigned)tiles), dim3(256), smem, stream>>>(static_cast<const uint16_t*>(X), ldx, K, src, mslot, gflag,
                                                            static_cast<const uint8_t*>(Wq), M, N, Kpad, s_x, s_w, Y,
                                                            y_dtype, ldy, tiles_m, tiles_n, bias);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FQ_ERR_HIP, "fused GEMM launch failed: %s", hipGetErrorString(e));
    return FQ_OK;
}

int gemm_dispatch_i8(const void* A, const void* B, int M, int N, int rowbytes, const float* s_x, const float* s_w,
                     void* Y, int y_dtype, int ldy, Batch bt, hipStream_t stream)
{
    return dispatch<MODE_I8>(A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt, stream);
}
#elif FQ_GEMM_MODE == 1
int gemm_dispatch_i4(const void* A, const void* B, int M, int N, int rowbytes, const float* s_x, const float* s_w,
                     void* Y, int y_dtype, int ldy, Batch bt, hipStream_t stream)
{
    return dispatch<MODE_I4>(A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt, stream);
}
#else
int gemm_dispatch_bf16(const void* A, const void* B, int M, int N, int rowbytes, const float* s_x, const float* s_w,
                       void* Y, int y_dtype, int ldy, Batch bt, hipStream_t stream)
{
    return dispatch<MODE_BF16>(A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, bt, stream);
}
#endif

}  // namespace fq
