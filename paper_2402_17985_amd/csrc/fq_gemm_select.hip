// Kernel-variant selection and the entry points of the GEMM family: they forward to the per-mode
// dispatchers, which live in the four translation units built from fq_gemm.hip.
#include "fq_internal.h"
#include "../../include/fq_peak.h"

namespace fq {

namespace {
// Forced kernel variant of the calling thread (-1 = automatic); a tuning and test hook, see fq_gemm_select().
// Thread-local, so concurrent callers of the GEMM entry points never see each other's choice.
thread_local int g_variant = -1;
// Measurement hook of the calling thread (fq_peak_gemm_ticks): where the GEMM kernels add their clock ticks.
thread_local unsigned long long* g_ticks = nullptr;
}  // namespace

unsigned long long* gemm_ticks_pointer() { return g_ticks; }
void g_ticks_set(unsigned long long* p) { g_ticks = p; }

int forced_gemm_variant() { return g_variant; }

int set_gemm_variant(int v)
{
    if (v != -1 && v != 2 && v != 6 && v != 7 && v != 10 && v != 11 && v != 12)
        return fail(FQ_ERR_RANGE, "unknown GEMM variant %d (valid: -1, 2, 6, 7, 10, 11, 12)", v);
    g_variant = v;
    return FQ_OK;
}

// What a forced variant cannot run, checked before anything is enqueued (rowbytes = bytes of a quantized row).
int check_forced_variant(int bits, int rowbytes)
{
    if (g_variant != 11 && g_variant != 12) return FQ_OK;
    if (bits == FQ_BITS_I4_E3M2) return FQ_OK;              // the 6-bit GEMM has one kernel and ignores the hook
    if (bits != 8 && g_variant == 11) return fail(FQ_ERR_RANGE, "GEMM variant 11 exists for INT8 and bf16 operands only");
    if (rowbytes % 128) return fail(FQ_ERR_SHAPE, "GEMM variants 11 and 12 need rows of whole 128-byte stages");
    return FQ_OK;
}

int launch_gemm_int(const void* Xq, const void* Wq, int M, int N, int Kpad, int bits, const float* s_x,
                    const float* s_w, void* Y, int y_dtype, int ldy, hipStream_t stream, const float* bias)
{
    const Batch one = {1, 0, 0, 0, bias, g_ticks};
    if (bits == 8) return gemm_dispatch_i8(Xq, Wq, M, N, Kpad, s_x, s_w, Y, y_dtype, ldy, one, stream);
    if (bits == FQ_BITS_I4_E3M2) return gemm_dispatch_f6(Xq, Wq, M, N, Kpad / 4 * 3, s_x, s_w, Y, y_dtype, ldy, one, stream);
    return gemm_dispatch_i4(Xq, Wq, M, N, Kpad / 2, s_x, s_w, Y, y_dtype, ldy, one, stream);
}

int launch_bmm_int(const void* Aq, const void* Bq, int batch, int M, int N, int Kpad, int bits, size_t stride_a,
                   size_t stride_b, const float* s_a, const float* s_b, void* Y, int y_dtype, int ldy,
                   size_t stride_y_bytes, hipStream_t stream)
{
    const Batch bt = {batch, stride_a, stride_b, stride_y_bytes, nullptr, g_ticks};
    if (bits == 8) return gemm_dispatch_i8(Aq, Bq, M, N, Kpad, s_a, s_b, Y, y_dtype, ldy, bt, stream);
    return gemm_dispatch_i4(Aq, Bq, M, N, Kpad / 2, s_a, s_b, Y, y_dtype, ldy, bt, stream);
}

int launch_gemm_bf16(const void* X, const void* W, int M, int N, int K, void* Y, int ldy, hipStream_t stream)
{
    const Batch one = {1, 0, 0, 0, nullptr, g_ticks};
    return gemm_dispatch_bf16(X, W, M, N, K * 2, nullptr, nullptr, Y, FQ_BF16, ldy, one, stream);
}

}  // namespace fq

extern "C" int fq_peak_gemm_ticks(unsigned long long* ticks_dev)
{
    fq::clear_error();
    if (reinterpret_cast<uintptr_t>(ticks_dev) & 7u) return fq::fail(FQ_ERR_ALIGN, "ticks is not 8-byte aligned");
    fq::g_ticks_set(ticks_dev);
    return FQ_OK;
}

extern "C" int fq_peak_wall_clock_khz(void)
{
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess)
        return 0;
    return khz;
}
