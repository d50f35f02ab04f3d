// Internal declarations shared by the translation units of libfq (GPU library only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/fq.h"

namespace fq {

// Records the reason of a failure for fq_last_error_string() and returns `code`.
int fail(int code, const char* fmt, ...);
void clear_error();

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int elem_size(int dtype)
{
    switch (dtype) {
    case FQ_F32: return 4;
    case FQ_F16: return 2;
    case FQ_BF16: return 2;
    case FQ_I32: return 4;
    default: return 0;
    }
}

// Workspace layout of the activation path: [cmax: K u32][mslot: Kpad f32][scalars: 4 f32][gflag: Kpad/16 u8]
struct ActWorkspace {
    uint32_t* cmax;   // per input channel max|x| as fp32 bit patterns
    float* mslot;     // per flattened slot multiplier m_p
    float* scalars;   // [0] = a'
    uint8_t* gflag;   // per group of 16 slots: 1 = the 16 channels at the same indices; then, Kpad/16 + 1
                      // bytes further, cflag: 1 = every slot repeats an identity slot's value or holds 0
    size_t bytes;
};
ActWorkspace carve_act_workspace(void* base, int K, int Kpad);

// ---- launchers (each validates nothing: the C-ABI layer has already done so) ----
// mode 0: equal split, dynamic absmax; 1: equal split, static absmax (*absmax_in); 2: weights (rep
// ignored, every slot a plain copy); 3 / 4: the printed peel split with threshold T, dynamic / static
// absmax, `rep` then carrying the slot ordinals.  out == nullptr: only the scale, the per-slot multipliers and
// the group flags are produced (in ws), nothing is quantized
int launch_flatten_quant(const void* X, int x_dtype, int M, int K, int ld,
                         const int32_t* src_idx, const int32_t* rep, int Kpad, int bits,
                         int mode, const float* absmax_in, void* out, float* scale_out,
                         const ActWorkspace& ws, hipStream_t stream, float T = 0.0f);

// chmax[j] = max(start, max_i |X[i, j]|), start = 0 or (accumulate) the non-negative value held on entry
int launch_channel_absmax(const void* X, int x_dtype, int M, int K, int ld, int accumulate, float* chmax,
                          hipStream_t stream);

// Batched launches: `count` independent problems, operand and output base addresses advancing by these
// byte strides (count = 1, strides 0 for a single GEMM); also carries the epilogue's optional bias.
struct Batch {
    int count;
    size_t stride_a, stride_b, stride_y;
    const float* bias;   // optional fp32 [N] added to the scaled accumulators (shared by the batch), or null
    unsigned long long* ticks;   // measurement hook (fq_peak_gemm_ticks): null, or two counters every workgroup adds
                                 // the shader-clock and constant-rate ticks of its first wave to
};
unsigned long long* gemm_ticks_pointer();   // the calling thread's hook value
void g_ticks_set(unsigned long long* p);

// Per-mode dispatchers (one translation unit each): A [M, rowbytes], B [N, rowbytes] bytes
int gemm_dispatch_i8(const void* A, const void* B, int M, int N, int rowbytes, const float* s_x, const float* s_w,
                     void* Y, int y_dtype, int ldy, Batch bt, hipStream_t stream);
int gemm_dispatch_i4(const void* A, const void* B, int M, int N, int rowbytes, const float* s_x, const float* s_w,
                     void* Y, int y_dtype, int ldy, Batch bt, hipStream_t stream);
int gemm_dispatch_bf16(const void* A, const void* B, int M, int N, int rowbytes, const float* s_x, const float* s_w,
                       void* Y, int y_dtype, int ldy, Batch bt, hipStream_t stream);
int gemm_dispatch_f6(const void* A, const void* B, int M, int N, int rowbytes, const float* s_x, const float* s_w,
                       void* Y, int y_dtype, int ldy, Batch bt, hipStream_t stream);
int forced_gemm_variant();   // -1 = choose from the shape
int set_gemm_variant(int v);
int check_forced_variant(int bits, int rowbytes);   // FQ_OK unless the forced variant cannot run this operand

// bias: optional fp32 [N] (16-byte aligned) added after scaling; must be null for FQ_I32 output
int launch_gemm_int(const void* Xq, const void* Wq, int M, int N, int Kpad, int bits,
                    const float* s_x, const float* s_w, void* Y, int y_dtype, int ldy,
                    hipStream_t stream, const float* bias = nullptr);

// `batch` independent products; operand strides in bytes, stride_y_bytes in bytes
int launch_bmm_int(const void* Aq, const void* Bq, int batch, int M, int N, int Kpad, int bits, size_t stride_a,
                   size_t stride_b, const float* s_a, const float* s_b, void* Y, int y_dtype, int ldy,
                   size_t stride_y_bytes, hipStream_t stream);

int launch_gemm_bf16(const void* X, const void* W, int M, int N, int K, void* Y, int ldy,
                     hipStream_t stream);
// INT8 GEMM whose A operand is X itself (bf16, row stride ldx elements): slot p of a row is quantized from
// X[row, src[p]] * mslot[p] on the way into LDS (gflag marks the 16-slot groups that are 16 consecutive channels)
int launch_gemm_fused_a_i8(const void* X, int ldx, int K, const int32_t* src, const float* mslot, const uint8_t* gflag,
                           const void* Wq, int M, int N, int Kpad, const float* s_x, const float* s_w, void* Y,
                           int y_dtype, int ldy, const float* bias, hipStream_t stream);

}  // namespace fq
