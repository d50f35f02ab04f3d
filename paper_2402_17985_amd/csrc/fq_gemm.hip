// LDS-tiled MFMA GEMMs for gfx950: INT8, packed INT4 (widened to INT8 in registers) and the
// bf16 baseline, one kernel template.
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
// Global -> registers -> LDS for stage t+1 is issued before the MFMAs of stage t.
// LDS rows are BKB bytes; the 16-byte chunk index is XOR-swizzled with the row so that the 16
// lanes that read the same chunk column of 16 consecutive rows hit 16 different bank groups.
// Workgroup ids are remapped so that each XCD (ids are dealt round-robin to the 8 XCDs) works on
// a contiguous band of tiles, walked in groups of GROUP_M tile-rows for L2 reuse.
#include "fq_internal.h"

namespace fq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned short v4us __attribute__((ext_vector_type(4)));

enum { MODE_I8 = 0, MODE_I4 = 1, MODE_BF16 = 2 };

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <int MODE> struct Acc { typedef v16i type; };
template <> struct Acc<MODE_BF16> { typedef v16f type; };

template <int MODE, int BM, int BN, int BKB, int WM, int WN>
__global__ __launch_bounds__(WM* WN * 64) void gemm_kernel(const uint8_t* __restrict__ A,
                                                            const uint8_t* __restrict__ B, int M, int N,
                                                            int rowbytes, const float* __restrict__ s_x,
                                                            const float* __restrict__ s_w, void* __restrict__ Y,
                                                            int y_dtype, int ldy, int tiles_m, int tiles_n)
{
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
    constexpr int GROUP_M = 8;
    static_assert(BM % RPP == 0 && BN % RPP == 0, "loader does not tile the block");
    static_assert(RPP % 16 == 0, "swizzle must repeat across loader passes");
    static_assert(CPR == 4 || CPR == 8, "BKB must be 64 or 128");
    typedef typename Acc<MODE>::type acc_t;

    extern __shared__ __align__(16) uint8_t smem[];

    // ---- workgroup -> tile ----
    int tile_m, tile_n;
    {
        const int nwg = gridDim.x;
        const int wg = blockIdx.x;
        const int q = nwg >> 3, rem = nwg & 7;
        const int xcd = wg & 7, idx = wg >> 3;
        const int logical = (xcd < rem) ? xcd * (q + 1) + idx : rem * (q + 1) + (xcd - rem) * q + idx;
        const int group = GROUP_M * tiles_n;
        const int gidx = logical / group;
        const int first_m = gidx * GROUP_M;
        const int gsz = min(tiles_m - first_m, GROUP_M);
        const int in_group = logical - gidx * group;
        tile_m = first_m + in_group % gsz;
        tile_n = in_group / gsz;
    }
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
            if constexpr (MODE == MODE_I8) {
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
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
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(alo[i], blo[j], acc[i][j], 0, 0, 0);
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ahi[i], bhi[j], acc[i][j], 0, 0, 0);
            } else {
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(v8bf, a[i]), __builtin_bit_cast(v8bf, b[j]), acc[i][j], 0, 0, 0);
            }
        }
        if (kt + 1 < nk) store_lds((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue: accumulator layout of the 32x32 MFMA: lane -> column lane%32,
    //      register r -> row 8*(r/4) + 4*(lane/32) + r%4 ----
    float scale = 1.0f;
    if (MODE != MODE_BF16 && y_dtype != FQ_I32) scale = (*s_x) * (*s_w);
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int col = n0 + wn * TN + j * 32 + frow;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * TM + i * 32 + 8 * (r >> 2) + 4 * fhalf + (r & 3);
                if (row < M && col < N) {
                    const size_t o = (size_t)row * ldy + col;
                    if constexpr (MODE == MODE_BF16) {
                        static_cast<uint16_t*>(Y)[o] = f32_to_bf16_rne(acc[i][j][r]);
                    } else {
                        int v = acc[i][j][r];
                        if (MODE == MODE_I4) v >>= 8;
                        if (y_dtype == FQ_I32) {
                            static_cast<int32_t*>(Y)[o] = v;
                        } else {
                            const float f = (float)v * scale;
                            if (y_dtype == FQ_F32) static_cast<float*>(Y)[o] = f;
                            else if (y_dtype == FQ_BF16) static_cast<uint16_t*>(Y)[o] = f32_to_bf16_rne(f);
                            else static_cast<_Float16*>(Y)[o] = (_Float16)f;
                        }
                    }
                }
            }
        }
}

// Forced kernel variant (-1 = automatic); a tuning hook, see fq_gemm_select().
int g_variant = -1;

template <int MODE, int BM, int BN, int BKB, int WM, int WN>
int launch_variant(const void* A, const void* B, int M, int N, int rowbytes, const float* s_x,
                   const float* s_w, void* Y, int y_dtype, int ldy, hipStream_t stream)
{
    auto kern = gemm_kernel<MODE, BM, BN, BKB, WM, WN>;
    constexpr int smem = 2 * (BM + BN) * BKB;
    static bool attr_set = false;       // one per instantiation
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return fail(FQ_ERR_HIP, "hipFuncSetAttribute(%d bytes LDS): %s", smem, hipGetErrorString(e));
        attr_set = true;
    }
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const long long nwg = (long long)tiles_m * tiles_n;
    if (nwg > 0x7fffffffLL) return fail(FQ_ERR_RANGE, "too many tiles");
    kern<<<dim3((unsigned)nwg), dim3(WM * WN * 64), smem, stream>>>(
        static_cast<const uint8_t*>(A), static_cast<const uint8_t*>(B), M, N, rowbytes, s_x, s_w, Y, y_dtype,
        ldy, tiles_m, tiles_n);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FQ_ERR_HIP, "GEMM launch failed: %s", hipGetErrorString(e));
    return FQ_OK;
}

// variant 0: 256x256 tile, 128-byte stages, 8 waves (2x4)   — large problems
// variant 1: 256x256 tile,  64-byte stages, 8 waves (2x4)
// variant 2: 128x128 tile,  64-byte stages, 4 waves (2x2)   — small problems
// variant 3: 256x128 tile, 128-byte stages, 8 waves (4x2)
template <int MODE>
int dispatch(const void* A, const void* B, int M, int N, int rowbytes, const float* s_x, const float* s_w,
             void* Y, int y_dtype, int ldy, hipStream_t stream)
{
    int v = g_variant;
    if (v < 0) {
        const long long big_tiles = (long long)((M + 255) / 256) * ((N + 255) / 256);
        v = (big_tiles >= 192) ? 0 : 2;
    }
    switch (v) {
    case 0: return launch_variant<MODE, 256, 256, 128, 2, 4>(A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, stream);
    case 1: return launch_variant<MODE, 256, 256, 64, 2, 4>(A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, stream);
    case 2: return launch_variant<MODE, 128, 128, 64, 2, 2>(A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, stream);
    case 3: return launch_variant<MODE, 256, 128, 128, 4, 2>(A, B, M, N, rowbytes, s_x, s_w, Y, y_dtype, ldy, stream);
    default: return fail(FQ_ERR_RANGE, "unknown GEMM variant %d", v);
    }
}

}  // namespace

int set_gemm_variant(int v)
{
    if (v < -1 || v > 3) return fail(FQ_ERR_RANGE, "unknown GEMM variant %d", v);
    g_variant = v;
    return FQ_OK;
}

int launch_gemm_int(const void* Xq, const void* Wq, int M, int N, int Kpad, int bits, const float* s_x,
                    const float* s_w, void* Y, int y_dtype, int ldy, hipStream_t stream)
{
    if (bits == 8) return dispatch<MODE_I8>(Xq, Wq, M, N, Kpad, s_x, s_w, Y, y_dtype, ldy, stream);
    return dispatch<MODE_I4>(Xq, Wq, M, N, Kpad / 2, s_x, s_w, Y, y_dtype, ldy, stream);
}

int launch_gemm_bf16(const void* X, const void* W, int M, int N, int K, void* Y, int ldy, hipStream_t stream)
{
    return dispatch<MODE_BF16>(X, W, M, N, K * 2, nullptr, nullptr, Y, FQ_BF16, ldy, stream);
}

}  // namespace fq
