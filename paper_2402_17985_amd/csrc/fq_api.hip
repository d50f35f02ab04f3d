// C-ABI layer of libfq: argument validation, the host-side flatten plan, and the composition
// of the kernels into the calls declared in include/fq.h.  Nothing here allocates or synchronizes.
#include <algorithm>
#include <cmath>
#include <memory>
#include <new>
#include <cstdarg>
#include <cstdio>
#include <mutex>

#include "fq_internal.h"

namespace fq {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}
void clear_error() { g_err[0] = '\0'; }


namespace {

bool float_dtype(int d) { return d == FQ_F32 || d == FQ_F16 || d == FQ_BF16; }

// Checks shared by the calls that read a floating-point matrix [rows, K] with stride ld.
int check_matrix(const char* what, const void* p, int dtype, int rows, int K, int ld)
{
    if (!p) return fail(FQ_ERR_NULL, "%s is NULL", what);
    if (!float_dtype(dtype)) return fail(FQ_ERR_DTYPE, "%s: dtype %d is not F32/F16/BF16", what, dtype);
    if (rows <= 0 || K <= 0) return fail(FQ_ERR_SHAPE, "%s: non-positive shape %d x %d", what, rows, K);
    if (ld < K) return fail(FQ_ERR_SHAPE, "%s: row stride %d < K = %d", what, ld, K);
    if (((size_t)ld * elem_size(dtype)) % 16 != 0)
        return fail(FQ_ERR_SHAPE, "%s: row stride of %d elements is not a multiple of 16 bytes", what, ld);
    if (!aligned16(p)) return fail(FQ_ERR_ALIGN, "%s is not 16-byte aligned", what);
    return FQ_OK;
}

// bytes of one row of a quantized array: a byte, a nibble or a 6-bit code per slot
size_t quantized_row_bytes(int Kpad, int bits)
{
    return bits == 8 ? (size_t)Kpad : (bits == 4 ? (size_t)Kpad / 2 : (size_t)Kpad / 4 * 3);
}

int check_map(const int32_t* src_idx, int Kpad, int bits)
{
    if (!src_idx) return fail(FQ_ERR_NULL, "src_idx is NULL");
    if (bits != 8 && bits != 4 && bits != FQ_BITS_I4_E3M2)
        return fail(FQ_ERR_DTYPE, "bits = %d, must be 8, 4 or %d (4-bit values in E3M2 storage)", bits, FQ_BITS_I4_E3M2);
    if (Kpad <= 0 || Kpad % 32 != 0) return fail(FQ_ERR_SHAPE, "Kpad = %d must be a positive multiple of 32", Kpad);
    if (bits == FQ_BITS_I4_E3M2 && Kpad % 128 != 0)
        return fail(FQ_ERR_SHAPE, "Kpad = %d must be a multiple of 128 for E3M2 storage", Kpad);
    if (Kpad >= 131072) return fail(FQ_ERR_RANGE, "Kpad = %d: int32 accumulators could overflow (needs Kpad < 131072)", Kpad);
    if (!aligned16(src_idx)) return fail(FQ_ERR_ALIGN, "src_idx is not 16-byte aligned");
    return FQ_OK;
}

int check_gemm(const void* Xq, const void* Wq, int M, int N, int Kpad, int bits, const float* s_x, const float* s_w,
               const void* Y, int y_dtype, int ldy)
{
    if (!Xq || !Wq || !Y) return fail(FQ_ERR_NULL, "Xq, Wq or Y is NULL");
    if (y_dtype != FQ_F32 && y_dtype != FQ_F16 && y_dtype != FQ_BF16 && y_dtype != FQ_I32)
        return fail(FQ_ERR_DTYPE, "unsupported output dtype %d", y_dtype);
    if (y_dtype != FQ_I32 && (!s_x || !s_w)) return fail(FQ_ERR_NULL, "s_x or s_w is NULL");
    if (M <= 0 || N <= 0) return fail(FQ_ERR_SHAPE, "non-positive shape M = %d, N = %d", M, N);
    if (Kpad <= 0 || Kpad % 32 != 0) return fail(FQ_ERR_SHAPE, "Kpad = %d must be a positive multiple of 32", Kpad);
    if (Kpad >= 131072) return fail(FQ_ERR_RANGE, "Kpad = %d: int32 accumulators could overflow (needs Kpad < 131072)", Kpad);
    if (ldy < N) return fail(FQ_ERR_SHAPE, "ldy = %d < N = %d", ldy, N);
    if (!aligned16(Xq) || !aligned16(Wq)) return fail(FQ_ERR_ALIGN, "Xq or Wq is not 16-byte aligned");
    // the GEMM kernels address an operand with 32-bit byte offsets
    const unsigned long long rowbytes = quantized_row_bytes(Kpad, bits);
    if ((unsigned long long)M * rowbytes >= (1ull << 32) || (unsigned long long)N * rowbytes >= (1ull << 32))
        return fail(FQ_ERR_RANGE, "a quantized operand of 4 GiB or more (M or N times %llu bytes per row)", rowbytes);
    return check_forced_variant(bits, (int)rowbytes);
}

}  // namespace
}  // namespace fq

using namespace fq;

extern "C" {

const char* fq_last_error_string(void) { return g_err; }

int fq_version(void) { return 100; }

int fq_gemm_select(int variant)
{
    clear_error();
    return set_gemm_variant(variant);
}

int fq_flatten_plan(const float* chmax_host, int K, float T, int align, int32_t* src_idx_host,
                    int32_t* rep_host, int cap, int* Kprime_out, int* Kpad_out)
{
    clear_error();
    if (!chmax_host) return fail(FQ_ERR_NULL, "chmax is NULL");
    if (K <= 0 || align <= 0 || cap < 0) return fail(FQ_ERR_SHAPE, "K = %d, align = %d, cap = %d", K, align, cap);
    if (!(T > 0.0f) || std::isinf(T)) return fail(FQ_ERR_RANGE, "T = %g must be positive and finite", (double)T);
    // pass 1: copies per channel and the total
    const double Td = (double)T;
    long long extra = 0;
    for (int j = 0; j < K; ++j) {
        const float c = chmax_host[j];
        if (!(c >= 0.0f) || std::isinf(c))
            return fail(FQ_ERR_RANGE, "chmax[%d] = %g must be finite and >= 0", j, (double)c);
        const double n = std::ceil((double)c / Td);
        if (n > 1.0e9) return fail(FQ_ERR_RANGE, "chmax[%d] / T = %g: more than 10^9 copies of one channel", j, n);
        if (n > 1.0) extra += (long long)n - 1;
        if (extra > (1LL << 30)) return fail(FQ_ERR_RANGE, "flattened width exceeds 2^30 channels");
    }
    const long long Kprime = (long long)K + extra;
    const long long Kpad = (Kprime + align - 1) / align * align;
    if (Kpad > 0x7fffffffLL) return fail(FQ_ERR_RANGE, "padded width exceeds int32");
    if (Kprime_out) *Kprime_out = (int)Kprime;
    if (Kpad_out) *Kpad_out = (int)Kpad;
    if (cap == 0) return FQ_OK;
    if (!src_idx_host || !rep_host) return fail(FQ_ERR_NULL, "src_idx / rep is NULL with cap > 0");
    if (cap < Kpad) return fail(FQ_ERR_SHAPE, "cap = %d < Kpad = %lld", cap, Kpad);
    // pass 2: originals stay in place, extras go to the appended block in channel order
    int tail = K;
    for (int j = 0; j < K; ++j) {
        double nd = std::ceil((double)chmax_host[j] / Td);
        const int n = nd > 1.0 ? (int)nd : 1;
        src_idx_host[j] = j;
        rep_host[j] = n;
        for (int e = 1; e < n; ++e, ++tail) {
            src_idx_host[tail] = j;
            rep_host[tail] = n;
        }
    }
    for (; tail < (int)Kpad; ++tail) {
        src_idx_host[tail] = -1;
        rep_host[tail] = 0;
    }
    return FQ_OK;
}

int fq_flatten_plan_xw(const float* chmax_x_host, float T_x, const float* chmax_w_host, float T_w, int K, int align,
                       int32_t* src_idx_host, int32_t* rep_x_host, int32_t* rep_w_host, int32_t* ord_host, int cap,
                       int* Kprime_out, int* Kpad_out)
{
    clear_error();
    if (!chmax_x_host) return fail(FQ_ERR_NULL, "chmax_x is NULL");
    if (K <= 0 || align <= 0 || cap < 0) return fail(FQ_ERR_SHAPE, "K = %d, align = %d, cap = %d", K, align, cap);
    if (!(T_x > 0.0f) || std::isinf(T_x)) return fail(FQ_ERR_RANGE, "T_x = %g must be positive and finite", (double)T_x);
    if (chmax_w_host && (!(T_w > 0.0f) || std::isinf(T_w)))
        return fail(FQ_ERR_RANGE, "T_w = %g must be positive and finite", (double)T_w);
    // shares of channel j on either side; 0 reports an invalid maximum
    auto shares = [](float c, float T) -> long long {
        if (!(c >= 0.0f) || std::isinf(c)) return 0;
        const double n = std::ceil((double)c / (double)T);
        return n > 1.0 ? (n > 1.0e9 ? (long long)1e9 : (long long)n) : 1;
    };
    long long total = 0;
    for (int j = 0; j < K; ++j) {
        const long long nx = shares(chmax_x_host[j], T_x), nw = chmax_w_host ? shares(chmax_w_host[j], T_w) : 1;
        if (nx == 0 || nw == 0) return fail(FQ_ERR_RANGE, "channel maximum %d must be finite and >= 0", j);
        total += nx * nw;
        if (total > (1LL << 30)) return fail(FQ_ERR_RANGE, "flattened width exceeds 2^30 channels");
    }
    const long long Kpad = (total + align - 1) / align * align;
    if (Kpad > 0x7fffffffLL) return fail(FQ_ERR_RANGE, "padded width exceeds int32");
    if (Kprime_out) *Kprime_out = (int)total;
    if (Kpad_out) *Kpad_out = (int)Kpad;
    if (cap == 0) return FQ_OK;
    if (!src_idx_host || !rep_x_host) return fail(FQ_ERR_NULL, "src_idx / rep_x is NULL with cap > 0");
    if (cap < Kpad) return fail(FQ_ERR_SHAPE, "cap = %d < Kpad = %lld", cap, Kpad);
    auto put = [&](int p, int j, int nx, int nw, int e) {
        src_idx_host[p] = j;
        rep_x_host[p] = nx;
        if (rep_w_host) rep_w_host[p] = nw;
        if (ord_host) ord_host[p] = e;
    };
    int tail = K;
    for (int j = 0; j < K; ++j) {
        const int nx = (int)shares(chmax_x_host[j], T_x), nw = chmax_w_host ? (int)shares(chmax_w_host[j], T_w) : 1;
        put(j, j, nx, nw, 0);
        for (int e = 1; e < nx * nw; ++e) put(tail++, j, nx, nw, e);
    }
    for (; tail < (int)Kpad; ++tail) put(tail, -1, 0, 0, 0);
    return FQ_OK;
}

int fq_threshold_boxplot(const float* chmax_host, int K, float beta, float* T_out_host)
{
    clear_error();
    if (!chmax_host || !T_out_host) return fail(FQ_ERR_NULL, "chmax or T_out is NULL");
    if (K <= 0) return fail(FQ_ERR_SHAPE, "K = %d", K);
    if (!(beta > 0.0f) || std::isinf(beta)) return fail(FQ_ERR_RANGE, "beta = %g must be positive and finite", (double)beta);
    // sorted copy of the maxima; the allocation must not throw across the C boundary
    std::unique_ptr<double[]> v(new (std::nothrow) double[(size_t)K]);
    if (!v) return fail(FQ_ERR_NOMEM, "out of host memory for %d channel maxima", K);
    for (int j = 0; j < K; ++j) {
        v[j] = (double)chmax_host[j];
        if (!(v[j] >= 0.0) || std::isinf(v[j])) return fail(FQ_ERR_RANGE, "chmax[%d] = %g must be finite and >= 0", j, v[j]);
    }
    std::sort(v.get(), v.get() + K);
    // quartiles by linear interpolation at position q * (K - 1)
    auto quartile = [&](double q) {
        const double pos = q * (double)(K - 1);
        const int lo = (int)std::floor(pos), hi = std::min(lo + 1, K - 1);
        return v[lo] + (v[hi] - v[lo]) * (pos - (double)lo);
    };
    const double q1 = quartile(0.25), q3 = quartile(0.75);
    const double fence_lo = q1 - 1.5 * (q3 - q1), fence_hi = q3 + 1.5 * (q3 - q1);
    double sum = 0.0;
    for (int j = 0; j < K; ++j) sum += std::min(std::max(v[j], fence_lo), fence_hi);
    *T_out_host = (float)((double)beta * (sum / (double)K));
    return FQ_OK;
}

int fq_smooth_scales(const float* chmax_x_host, const float* chmax_w_host, int K, float alpha, float* s_out_host)
{
    clear_error();
    if (!chmax_x_host || !chmax_w_host || !s_out_host) return fail(FQ_ERR_NULL, "chmax_x, chmax_w or s_out is NULL");
    if (K <= 0) return fail(FQ_ERR_SHAPE, "K = %d", K);
    if (!(alpha >= 0.0f) || !(alpha <= 1.0f)) return fail(FQ_ERR_RANGE, "alpha = %g must lie in [0, 1]", (double)alpha);
    double mean = 0.0;
    for (int j = 0; j < K; ++j) {
        const float a = chmax_x_host[j], b = chmax_w_host[j];
        if (!(a >= 0.0f) || std::isinf(a) || !(b >= 0.0f) || std::isinf(b))
            return fail(FQ_ERR_RANGE, "channel maximum %d must be finite and >= 0", j);
        mean += (double)a;
    }
    mean /= (double)K;
    double ss = 0.0;
    for (int j = 0; j < K; ++j) ss += ((double)chmax_x_host[j] - mean) * ((double)chmax_x_host[j] - mean);
    const double sd = std::sqrt(ss / (double)K);
    const double a = (double)alpha;
    for (int j = 0; j < K; ++j) {
        if (sd == 0.0) {
            s_out_host[j] = 1.0f;
            continue;
        }
        const double gx = 1.0 / (1.0 + std::exp(-((double)chmax_x_host[j] - mean) / sd));
        const double gw = 1.0 / (1.0 + std::exp(-((double)chmax_w_host[j] - mean) / sd));
        s_out_host[j] = (float)(std::pow(gx, a) / std::pow(gw, 1.0 - a));
    }
    return FQ_OK;
}

int fq_channel_absmax(const void* X, int x_dtype, int M, int K, int ldx, int accumulate, float* chmax_dev,
                      void* stream)
{
    clear_error();
    if (int rc = check_matrix("X", X, x_dtype, M, K, ldx)) return rc;
    if (!chmax_dev) return fail(FQ_ERR_NULL, "chmax is NULL");
    if ((reinterpret_cast<uintptr_t>(chmax_dev) & 3u) != 0) return fail(FQ_ERR_ALIGN, "chmax is not 4-byte aligned");
    return launch_channel_absmax(X, x_dtype, M, K, ldx, accumulate, chmax_dev, static_cast<hipStream_t>(stream));
}

size_t fq_act_workspace_bytes(int K, int Kpad)
{
    if (K <= 0 || Kpad <= 0) return 0;
    return carve_act_workspace(nullptr, K, Kpad).bytes;
}

size_t fq_weights_workspace_bytes(int K, int Kpad) { return fq_act_workspace_bytes(K, Kpad); }

size_t fq_linear_workspace_bytes(int M, int K, int Kpad, int bits)
{
    if (M <= 0 || K <= 0 || Kpad <= 0 || (bits != 8 && bits != 4 && bits != FQ_BITS_I4_E3M2)) return 0;
    const size_t xq = round_up((size_t)M * quantized_row_bytes(Kpad, bits), 256);
    return xq + fq_act_workspace_bytes(K, Kpad);
}

int fq_flatten_weights(const void* W, int w_dtype, int N, int K, int ldw, const int32_t* src_idx, int Kpad,
                       int bits, void* Wq_out, float* s_w_out, void* workspace, size_t workspace_bytes,
                       void* stream)
{
    clear_error();
    int rc = check_matrix("W", W, w_dtype, N, K, ldw);
    if (rc) return rc;
    rc = check_map(src_idx, Kpad, bits);
    if (rc) return rc;
    if (!Wq_out || !s_w_out || !workspace) return fail(FQ_ERR_NULL, "Wq_out, s_w_out or workspace is NULL");
    if (!aligned16(Wq_out) || !aligned16(workspace)) return fail(FQ_ERR_ALIGN, "Wq_out or workspace is not 16-byte aligned");
    if (workspace_bytes < fq_weights_workspace_bytes(K, Kpad))
        return fail(FQ_ERR_WORKSPACE, "workspace of %zu bytes < %zu required", workspace_bytes,
                    fq_weights_workspace_bytes(K, Kpad));
    ActWorkspace ws = carve_act_workspace(workspace, K, Kpad);
    return launch_flatten_quant(W, w_dtype, N, K, ldw, src_idx, nullptr, Kpad, bits, /*mode=*/2, nullptr, Wq_out,
                                s_w_out, ws, static_cast<hipStream_t>(stream));
}

int fq_flatten_quant_act(const void* X, int x_dtype, int M, int K, int ldx, const int32_t* src_idx,
                         const int32_t* rep, int Kpad, int bits, const float* absmax_in, void* Xq_out,
                         float* s_x_out, void* workspace, size_t workspace_bytes, void* stream)
{
    clear_error();
    int rc = check_matrix("X", X, x_dtype, M, K, ldx);
    if (rc) return rc;
    rc = check_map(src_idx, Kpad, bits);
    if (rc) return rc;
    if (!rep || !Xq_out || !s_x_out || !workspace) return fail(FQ_ERR_NULL, "rep, Xq_out, s_x_out or workspace is NULL");
    if (!aligned16(Xq_out) || !aligned16(workspace)) return fail(FQ_ERR_ALIGN, "Xq_out or workspace is not 16-byte aligned");
    if (workspace_bytes < fq_act_workspace_bytes(K, Kpad))
        return fail(FQ_ERR_WORKSPACE, "workspace of %zu bytes < %zu required", workspace_bytes,
                    fq_act_workspace_bytes(K, Kpad));
    ActWorkspace ws = carve_act_workspace(workspace, K, Kpad);
    return launch_flatten_quant(X, x_dtype, M, K, ldx, src_idx, rep, Kpad, bits, absmax_in ? 1 : 0, absmax_in,
                                Xq_out, s_x_out, ws, static_cast<hipStream_t>(stream));
}

// ---------------------------------------------------------------------------------------------
// fq_flatten_quant_act_noalloc: the workspace of fq_flatten_quant_act held in device memory that belongs
// to the library's code object, for callers that cannot allocate.
// ---------------------------------------------------------------------------------------------
}  // extern "C"

namespace {
constexpr size_t NOALLOC_SCRATCH_BYTES = FQ_NOALLOC_SCRATCH_BYTES;
// One copy per GPU that loads the library, at that GPU's own address, held until the process ends.  In host
// code this name is only a handle for hipGetSymbolAddress; kernels receive the address that call returns.
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[NOALLOC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};

// Device address of `scratch` on the current device (looked up once per device).
int scratch_of_current_device(void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(FQ_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(FQ_ERR_RANGE, "device ordinal %d beyond %d", dev, MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(FQ_ERR_HIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return FQ_OK;
}
}  // namespace

extern "C" {

size_t fq_noalloc_scratch_bytes(void) { return NOALLOC_SCRATCH_BYTES; }

int fq_flatten_quant_act_noalloc(const void* X, int x_dtype, int M, int K, int ldx, const int32_t* src_idx,
                                 const int32_t* rep, int Kpad, int bits, const float* absmax_in, void* Xq_out,
                                 float* s_x_out, void* stream)
{
    clear_error();
    int rc = check_matrix("X", X, x_dtype, M, K, ldx);
    if (rc) return rc;
    rc = check_map(src_idx, Kpad, bits);
    if (rc) return rc;
    if (!rep || !Xq_out || !s_x_out) return fail(FQ_ERR_NULL, "rep, Xq_out or s_x_out is NULL");
    if (!aligned16(Xq_out)) return fail(FQ_ERR_ALIGN, "Xq_out is not 16-byte aligned");
    const size_t need = fq_act_workspace_bytes(K, Kpad);
    if (need > NOALLOC_SCRATCH_BYTES)
        return fail(FQ_ERR_WORKSPACE, "K = %d, Kpad = %d need %zu bytes of scratch, beyond the built-in %zu: use "
                                      "fq_flatten_quant_act with a caller-owned workspace", K, Kpad, need,
                    NOALLOC_SCRATCH_BYTES);
    void* base = nullptr;
    rc = scratch_of_current_device(&base);
    if (rc) return rc;
    // cmax, the part of the scratch that must start at zero, is cleared by a fill kernel inside the launch
    ActWorkspace ws = carve_act_workspace(base, K, Kpad);
    return launch_flatten_quant(X, x_dtype, M, K, ldx, src_idx, rep, Kpad, bits, absmax_in ? 1 : 0, absmax_in,
                                Xq_out, s_x_out, ws, static_cast<hipStream_t>(stream));
}

int fq_flatten_weights_split(const void* W, int w_dtype, int N, int K, int ldw, const int32_t* src_idx,
                             const int32_t* rep_w, int Kpad, int bits, void* Wq_out, float* s_w_out, void* workspace,
                             size_t workspace_bytes, void* stream)
{
    // the equal split applied to the weight array: the activation path with the weights' share counts
    return fq_flatten_quant_act(W, w_dtype, N, K, ldw, src_idx, rep_w, Kpad, bits, nullptr, Wq_out, s_w_out, workspace,
                                workspace_bytes, stream);
}

int fq_flatten_quant_act_peel(const void* X, int x_dtype, int M, int K, int ldx, const int32_t* src_idx,
                              const int32_t* ord, int Kpad, int bits, float T, const float* absmax_in, void* Xq_out,
                              float* s_x_out, void* workspace, size_t workspace_bytes, void* stream)
{
    clear_error();
    int rc = check_matrix("X", X, x_dtype, M, K, ldx);
    if (rc) return rc;
    rc = check_map(src_idx, Kpad, bits);
    if (rc) return rc;
    if (!(T > 0.0f) || std::isinf(T)) return fail(FQ_ERR_RANGE, "T = %g must be positive and finite", (double)T);
    if (!ord || !Xq_out || !s_x_out || !workspace) return fail(FQ_ERR_NULL, "ord, Xq_out, s_x_out or workspace is NULL");
    if (!aligned16(Xq_out) || !aligned16(workspace)) return fail(FQ_ERR_ALIGN, "Xq_out or workspace is not 16-byte aligned");
    if (workspace_bytes < fq_act_workspace_bytes(K, Kpad))
        return fail(FQ_ERR_WORKSPACE, "workspace of %zu bytes < %zu required", workspace_bytes,
                    fq_act_workspace_bytes(K, Kpad));
    ActWorkspace ws = carve_act_workspace(workspace, K, Kpad);
    return launch_flatten_quant(X, x_dtype, M, K, ldx, src_idx, ord, Kpad, bits, absmax_in ? 4 : 3, absmax_in, Xq_out,
                                s_x_out, ws, static_cast<hipStream_t>(stream), T);
}

namespace {
int check_bias(const float* bias, int y_dtype)
{
    if (!bias) return FQ_OK;
    if (y_dtype == FQ_I32) return fail(FQ_ERR_DTYPE, "a bias cannot be added to raw int32 accumulators");
    if (!aligned16(bias)) return fail(FQ_ERR_ALIGN, "bias is not 16-byte aligned");
    return FQ_OK;
}

int gemm_common(const void* Xq, const void* Wq, int M, int N, int Kpad, int bits, const float* s_x, const float* s_w,
                const float* bias, void* Y, int y_dtype, int ldy, void* stream)
{
    clear_error();
    int rc = check_gemm(Xq, Wq, M, N, Kpad, bits, s_x, s_w, Y, y_dtype, ldy);
    if (rc) return rc;
    rc = check_bias(bias, y_dtype);
    if (rc) return rc;
    return launch_gemm_int(Xq, Wq, M, N, Kpad, bits, s_x, s_w, Y, y_dtype, ldy, static_cast<hipStream_t>(stream), bias);
}
}  // namespace

int fq_gemm_i8(const int8_t* Xq, const int8_t* Wq, int M, int N, int Kpad, const float* s_x, const float* s_w,
               void* Y, int y_dtype, int ldy, void* stream)
{
    return gemm_common(Xq, Wq, M, N, Kpad, 8, s_x, s_w, nullptr, Y, y_dtype, ldy, stream);
}

int fq_gemm_i4(const uint8_t* Xq, const uint8_t* Wq, int M, int N, int Kpad, const float* s_x, const float* s_w,
               void* Y, int y_dtype, int ldy, void* stream)
{
    return gemm_common(Xq, Wq, M, N, Kpad, 4, s_x, s_w, nullptr, Y, y_dtype, ldy, stream);
}

int fq_gemm_i4_e3m2(const uint8_t* Xq, const uint8_t* Wq, int M, int N, int Kpad, const float* s_x, const float* s_w,
                    const float* bias, void* Y, int y_dtype, int ldy, void* stream)
{
    if (Kpad > 0 && Kpad % 128 != 0) {
        clear_error();
        return fail(FQ_ERR_SHAPE, "Kpad = %d must be a multiple of 128 for E3M2 storage", Kpad);
    }
    return gemm_common(Xq, Wq, M, N, Kpad, FQ_BITS_I4_E3M2, s_x, s_w, bias, Y, y_dtype, ldy, stream);
}

int fq_gemm_i8_bias(const int8_t* Xq, const int8_t* Wq, int M, int N, int Kpad, const float* s_x, const float* s_w,
                    const float* bias, void* Y, int y_dtype, int ldy, void* stream)
{
    return gemm_common(Xq, Wq, M, N, Kpad, 8, s_x, s_w, bias, Y, y_dtype, ldy, stream);
}

int fq_gemm_i4_bias(const uint8_t* Xq, const uint8_t* Wq, int M, int N, int Kpad, const float* s_x, const float* s_w,
                    const float* bias, void* Y, int y_dtype, int ldy, void* stream)
{
    return gemm_common(Xq, Wq, M, N, Kpad, 4, s_x, s_w, bias, Y, y_dtype, ldy, stream);
}

namespace {
int bmm_common(const void* Aq, const void* Bq, int batch, int M, int N, int Kpad, int bits, long long stride_a,
               long long stride_b, const float* s_a, const float* s_b, void* Y, int y_dtype, int ldy, long long stride_y,
               void* stream)
{
    clear_error();
    if (int rc = check_gemm(Aq, Bq, M, N, Kpad, bits, s_a, s_b, Y, y_dtype, ldy)) return rc;
    if (batch < 1 || batch > 65535) return fail(FQ_ERR_RANGE, "batch = %d must lie in [1, 65535]", batch);
    const long long rowbytes = (long long)quantized_row_bytes(Kpad, bits);
    if (stride_a < (long long)M * rowbytes || stride_b < (long long)N * rowbytes)
        return fail(FQ_ERR_SHAPE, "operand batch stride smaller than one matrix (%lld, %lld bytes)", stride_a, stride_b);
    if (stride_a % 16 != 0 || stride_b % 16 != 0)
        return fail(FQ_ERR_ALIGN, "operand batch strides must be multiples of 16 bytes");
    if (stride_y < (long long)(M - 1) * ldy + N) return fail(FQ_ERR_SHAPE, "output batch stride %lld too small", stride_y);
    return launch_bmm_int(Aq, Bq, batch, M, N, Kpad, bits, (size_t)stride_a, (size_t)stride_b, s_a, s_b, Y, y_dtype, ldy,
                          (size_t)stride_y * elem_size(y_dtype), static_cast<hipStream_t>(stream));
}
}  // namespace

int fq_bmm_i8(const int8_t* Aq, const int8_t* Bq, int batch, int M, int N, int Kpad, long long stride_a,
              long long stride_b, const float* s_a, const float* s_b, void* Y, int y_dtype, int ldy, long long stride_y,
              void* stream)
{
    return bmm_common(Aq, Bq, batch, M, N, Kpad, 8, stride_a, stride_b, s_a, s_b, Y, y_dtype, ldy, stride_y, stream);
}

int fq_bmm_i4(const uint8_t* Aq, const uint8_t* Bq, int batch, int M, int N, int Kpad, long long stride_a,
              long long stride_b, const float* s_a, const float* s_b, void* Y, int y_dtype, int ldy, long long stride_y,
              void* stream)
{
    return bmm_common(Aq, Bq, batch, M, N, Kpad, 4, stride_a, stride_b, s_a, s_b, Y, y_dtype, ldy, stride_y, stream);
}

int fq_linear(const void* X, int x_dtype, int M, int K, int ldx, const int32_t* src_idx, const int32_t* rep,
              int Kpad, const void* Wq, const float* s_w, int N, int bits, const float* absmax_in, void* Y,
              int y_dtype, int ldy, void* workspace, size_t workspace_bytes, void* stream)
{
    return fq_linear_bias(X, x_dtype, M, K, ldx, src_idx, rep, Kpad, Wq, s_w, nullptr, N, bits, absmax_in, Y, y_dtype, ldy,
                          workspace, workspace_bytes, stream);
}

int fq_linear_bias(const void* X, int x_dtype, int M, int K, int ldx, const int32_t* src_idx, const int32_t* rep,
                   int Kpad, const void* Wq, const float* s_w, const float* bias, int N, int bits,
                   const float* absmax_in, void* Y, int y_dtype, int ldy, void* workspace, size_t workspace_bytes,
                   void* stream)
{
    clear_error();
    int rc = check_matrix("X", X, x_dtype, M, K, ldx);
    if (rc) return rc;
    rc = check_map(src_idx, Kpad, bits);
    if (rc) return rc;
    if (!rep || !workspace) return fail(FQ_ERR_NULL, "rep or workspace is NULL");
    if (!aligned16(workspace)) return fail(FQ_ERR_ALIGN, "workspace is not 16-byte aligned");
    if (workspace_bytes < fq_linear_workspace_bytes(M, K, Kpad, bits))
        return fail(FQ_ERR_WORKSPACE, "workspace of %zu bytes < %zu required", workspace_bytes,
                    fq_linear_workspace_bytes(M, K, Kpad, bits));
    uint8_t* base = static_cast<uint8_t*>(workspace);
    const size_t xq_bytes = round_up((size_t)M * quantized_row_bytes(Kpad, bits), 256);
    void* Xq = base;
    ActWorkspace ws = carve_act_workspace(base + xq_bytes, K, Kpad);
    float* s_x = ws.scalars + 1;
    rc = check_gemm(Xq, Wq, M, N, Kpad, bits, s_x, s_w, Y, y_dtype, ldy);
    if (rc) return rc;
    rc = check_bias(bias, y_dtype);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = launch_flatten_quant(X, x_dtype, M, K, ldx, src_idx, rep, Kpad, bits, absmax_in ? 1 : 0, absmax_in, Xq,
                              s_x, ws, st);
    if (rc) return rc;
    return launch_gemm_int(Xq, Wq, M, N, Kpad, bits, s_x, s_w, Y, y_dtype, ldy, st, bias);
}

int fq_linear_fused_a_i8(const void* X, int x_dtype, int M, int K, int ldx, const int32_t* src_idx, const int32_t* rep,
                         int Kpad, const void* Wq, const float* s_w, const float* bias, int N, const float* absmax_in,
                         void* Y, int y_dtype, int ldy, void* workspace, size_t workspace_bytes, void* stream)
{
    clear_error();
    int rc = check_matrix("X", X, x_dtype, M, K, ldx);
    if (rc) return rc;
    if (x_dtype != FQ_BF16) return fail(FQ_ERR_DTYPE, "the fused A-operand path reads bf16 activations only");
    rc = check_map(src_idx, Kpad, 8);
    if (rc) return rc;
    if (!rep || !workspace) return fail(FQ_ERR_NULL, "rep or workspace is NULL");
    if (!aligned16(workspace)) return fail(FQ_ERR_ALIGN, "workspace is not 16-byte aligned");
    if (workspace_bytes < fq_act_workspace_bytes(K, Kpad))
        return fail(FQ_ERR_WORKSPACE, "workspace of %zu bytes < %zu required", workspace_bytes, fq_act_workspace_bytes(K, Kpad));
    if (!Wq || !Y) return fail(FQ_ERR_NULL, "Wq or Y is NULL");
    if (y_dtype != FQ_F32 && y_dtype != FQ_F16 && y_dtype != FQ_BF16 && y_dtype != FQ_I32)
        return fail(FQ_ERR_DTYPE, "unsupported output dtype %d", y_dtype);
    if (y_dtype != FQ_I32 && !s_w) return fail(FQ_ERR_NULL, "s_w is NULL");
    if (N <= 0) return fail(FQ_ERR_SHAPE, "non-positive N = %d", N);
    if (ldy < N) return fail(FQ_ERR_SHAPE, "ldy = %d < N = %d", ldy, N);
    if (!aligned16(Wq)) return fail(FQ_ERR_ALIGN, "Wq is not 16-byte aligned");
    if ((unsigned long long)N * (unsigned long long)Kpad >= (1ull << 32))
        return fail(FQ_ERR_RANGE, "a quantized operand of 4 GiB or more");
    rc = check_bias(bias, y_dtype);
    if (rc) return rc;
    ActWorkspace ws = carve_act_workspace(workspace, K, Kpad);
    float* s_x = ws.scalars + 1;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // the scale, the per-slot multipliers and the group flags; nothing is quantized here
    rc = launch_flatten_quant(X, x_dtype, M, K, ldx, src_idx, rep, Kpad, 8, absmax_in ? 1 : 0, absmax_in, nullptr, s_x, ws, st);
    if (rc) return rc;
    return launch_gemm_fused_a_i8(X, ldx, K, src_idx, ws.mslot, ws.gflag, Wq, M, N, Kpad, s_x, s_w, Y, y_dtype, ldy, bias, st);
}

int fq_gemm_bf16(const void* X, const void* W, int M, int N, int K, void* Y, int ldy, void* stream)
{
    clear_error();
    if (!X || !W || !Y) return fail(FQ_ERR_NULL, "X, W or Y is NULL");
    if (M <= 0 || N <= 0 || K <= 0) return fail(FQ_ERR_SHAPE, "non-positive shape %d x %d x %d", M, N, K);
    if (K % 8 != 0) return fail(FQ_ERR_SHAPE, "K = %d must be a multiple of 8", K);
    if (ldy < N) return fail(FQ_ERR_SHAPE, "ldy = %d < N = %d", ldy, N);
    if (!aligned16(X) || !aligned16(W)) return fail(FQ_ERR_ALIGN, "X or W is not 16-byte aligned");
    return launch_gemm_bf16(X, W, M, N, K, Y, ldy, static_cast<hipStream_t>(stream));
}

}  // extern "C"
