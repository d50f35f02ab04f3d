// Measurement hooks (include/fq_peak.h): an MFMA-only issue loop per matrix-pipe format and a plain copy.
#include "fq_internal.h"
#include "../../include/fq_peak.h"

namespace fq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

template <int KIND> struct PeakAcc { typedef v16f type; };
template <> struct PeakAcc<FQ_PEAK_I8> { typedef v16i type; };
template <> struct PeakAcc<FQ_PEAK_I8_NIBBLES> { typedef v16i type; };

// One operand vector of the lane: 16 bytes (24 for E3M2, in a v8i whose last two words are unused).
template <int KIND> __device__ __forceinline__ v8i load_operand(const uint8_t* base, size_t size, size_t index)
{
    v8i o = {0, 0, 0, 0, 0, 0, 0, 0};
    if (!base) return o;
    constexpr size_t BYTES = (KIND == FQ_PEAK_E3M2) ? 32 : 16;        // 32-byte slots keep E3M2 loads aligned
    const size_t off = (index * BYTES) % (size - 32 + 1) & ~(size_t)15;
    const v4i lo = *reinterpret_cast<const v4i*>(base + off);
    o[0] = lo[0]; o[1] = lo[1]; o[2] = lo[2]; o[3] = lo[3];
    if (KIND == FQ_PEAK_E3M2) {
        const v4i hi = *reinterpret_cast<const v4i*>(base + off + 16);
        o[4] = hi[0]; o[5] = hi[1];
    }
    if (KIND == FQ_PEAK_I8_NIBBLES) {
        // low nibbles moved to the top of their bytes, as the INT4 GEMM feeds them to the int8 MFMA
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = (o[i] << 4) & (int)0xf0f0f0f0;
    }
    return o;
}

template <int KIND>
__global__ __launch_bounds__(256) void peak_mfma_kernel(const uint8_t* __restrict__ operands, size_t operand_bytes,
                                                        long long iters, unsigned long long* __restrict__ ticks,
                                                        float* __restrict__ sink)
{
    typedef typename PeakAcc<KIND>::type acc_t;
    const size_t wave_id = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const size_t lane = threadIdx.x & 63;
    v8i a[2][4], b[2][4];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a[s][i] = load_operand<KIND>(operands, operand_bytes, ((wave_id * 16 + s * 8 + i) * 64 + lane));
            b[s][i] = load_operand<KIND>(operands, operand_bytes, ((wave_id * 16 + s * 8 + 4 + i) * 64 + lane));
        }
    acc_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    auto slice = [&](int s) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (KIND == FQ_PEAK_I8 || KIND == FQ_PEAK_I8_NIBBLES) {
                    const v4i x = {a[s][i][0], a[s][i][1], a[s][i][2], a[s][i][3]};
                    const v4i y = {b[s][j][0], b[s][j][1], b[s][j][2], b[s][j][3]};
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(y, x, acc[i][j], 0, 0, 0);
                } else if constexpr (KIND == FQ_PEAK_BF16) {
                    const v4i x = {a[s][i][0], a[s][i][1], a[s][i][2], a[s][i][3]};
                    const v4i y = {b[s][j][0], b[s][j][1], b[s][j][2], b[s][j][3]};
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, y), __builtin_bit_cast(v8bf, x),
                                                                       acc[i][j], 0, 0, 0);
                } else {
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b[s][j], a[s][i], acc[i][j], 3, 3, 0, 127, 0, 127);
                }
            }
    };

    __syncthreads();
    const unsigned long long t0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
    for (long long it = 0; it < iters; it += 2) {
        slice(0);
        __builtin_amdgcn_sched_barrier(0);
        slice(1);
        __builtin_amdgcn_sched_barrier(0);
    }
    // the loop's MFMAs have been issued; wait for the last results before reading the clocks
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) s += (float)acc[i][j][r];
    const unsigned long long t1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
    if (ticks && threadIdx.x == 0) {
        ticks[2 * (size_t)blockIdx.x] = t1 - t0;
        ticks[2 * (size_t)blockIdx.x + 1] = r1 - r0;
    }
}

__global__ __launch_bounds__(256) void peak_copy_kernel(const v4i* __restrict__ src, v4i* __restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

template <int KIND>
int launch_peak(const void* operands, size_t operand_bytes, int blocks, long long iters, unsigned long long* ticks,
                float* sink, hipStream_t stream)
{
    peak_mfma_kernel<KIND><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(static_cast<const uint8_t*>(operands), operand_bytes,
                                                                             iters, ticks, sink);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FQ_ERR_HIP, "peak kernel launch failed: %s", hipGetErrorString(e));
    return FQ_OK;
}

}  // namespace
}  // namespace fq

using namespace fq;

extern "C" {

int fq_peak_mfma(int kind, const void* operands, size_t operand_bytes, int blocks, long long iters,
                 unsigned long long* ticks_out, float* sink, void* stream)
{
    clear_error();
    if (!sink) return fail(FQ_ERR_NULL, "sink is NULL");
    if (blocks < 1 || blocks > (1 << 20) || iters < 1) return fail(FQ_ERR_SHAPE, "blocks = %d, iters = %lld", blocks, iters);
    if (operands && operand_bytes < 65536) return fail(FQ_ERR_SHAPE, "operand buffer of %zu bytes < 65536", operand_bytes);
    if (operands && !aligned16(operands)) return fail(FQ_ERR_ALIGN, "operands is not 16-byte aligned");
    if (ticks_out && (reinterpret_cast<uintptr_t>(ticks_out) & 7u)) return fail(FQ_ERR_ALIGN, "ticks_out is not 8-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    iters = (iters + 1) & ~1LL;                       // the loop issues both operand sets per pass
    switch (kind) {
    case FQ_PEAK_I8: return launch_peak<FQ_PEAK_I8>(operands, operand_bytes, blocks, iters, ticks_out, sink, st);
    case FQ_PEAK_BF16: return launch_peak<FQ_PEAK_BF16>(operands, operand_bytes, blocks, iters, ticks_out, sink, st);
    case FQ_PEAK_E3M2: return launch_peak<FQ_PEAK_E3M2>(operands, operand_bytes, blocks, iters, ticks_out, sink, st);
    case FQ_PEAK_I8_NIBBLES: return launch_peak<FQ_PEAK_I8_NIBBLES>(operands, operand_bytes, blocks, iters, ticks_out, sink, st);
    default: return fail(FQ_ERR_DTYPE, "unknown pipe kind %d", kind);
    }
}

int fq_peak_copy(const void* src, void* dst, size_t bytes, void* stream)
{
    clear_error();
    if (!src || !dst) return fail(FQ_ERR_NULL, "src or dst is NULL");
    if (bytes == 0 || bytes % 16) return fail(FQ_ERR_SHAPE, "bytes = %zu must be a positive multiple of 16", bytes);
    if (!aligned16(src) || !aligned16(dst)) return fail(FQ_ERR_ALIGN, "src or dst is not 16-byte aligned");
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    peak_copy_kernel<<<dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const v4i*>(src), static_cast<v4i*>(dst), n16);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FQ_ERR_HIP, "copy launch failed: %s", hipGetErrorString(e));
    return FQ_OK;
}

}  // extern "C"
