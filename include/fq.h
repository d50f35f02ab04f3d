/*
 * fq.h — C ABI of the FlattenQuant per-tensor-quantized linear layer for AMD MI355X (gfx950).
 *
 * The layer (arXiv 2402.17985):
 *   1. flatten the activation: an input channel j whose calibrated max|x| exceeds the
 *      truncation threshold T is spread over n_j channels and the matching weight channel is
 *      repeated n_j times, so that X'W' = XW (Sec. 4.1, Eq. 2-4);
 *   2. quantize X' and W' per tensor to INT8 or INT4 (Sec. 2.1, Eq. 1);
 *   3. multiply in integers with int32 accumulation and scale the result back by s_x * s_w
 *      (Sec. 5.1 "Implementation": quantized linear layers on INT8 / INT4 GEMM kernels).
 *
 * Shapes and layouts
 *   X    activations  [M, K]      row-major, K contiguous, row stride ldx elements
 *   W    weights      [N, K]      row-major (the nn.Linear storage layout).  The paper writes
 *                                 Y = X W; its "weight channel j" is column j of this array.
 *   map  src_idx[p], rep[p], p in [0, Kpad): flattened slot p reads input channel src_idx[p]
 *        (-1 = padding slot, value 0) and that channel has rep[p] = n_j copies in total.
 *   Xq   [M, Kpad] int8, or [M, Kpad/2] bytes for INT4 (two's-complement nibbles, even slot in
 *        the low nibble); Wq likewise [N, Kpad] / [N, Kpad/2].  Rows are densely packed.
 *   Y    [M, N] row-major, row stride ldy elements.
 *   Kpad must be a multiple of 32 (Sec. 5.1 pads the flattened channel count to a multiple of 32).
 *   The GEMMs run fastest when every quantized row starts on a 128-byte boundary, i.e. when the plan
 *   is made with align = 128 for INT8 and 256 for INT4 (the extra zero columns cost no MFMA work:
 *   a k-stage is 128 bytes of a row in any case).
 *
 * Conventions common to every call
 *   - Returns FQ_OK (0) or an FQ_ERR_* code; fq_last_error_string() (thread-local) says why.
 *   - Pointers are DEVICE pointers unless the parameter name ends in _host.
 *   - All buffers are caller-owned.  The library allocates nothing, frees nothing and never
 *     synchronizes: every kernel is enqueued on `stream` (a hipStream_t passed as void*;
 *     NULL = the default stream) and the call returns immediately.
 *   - Arguments are validated on the host before anything is launched: on error nothing has
 *     been enqueued.  Device-resident maps cannot be validated from the host; kernels treat
 *     any src_idx outside [0, K) as a padding slot, so a bad map cannot cause an
 *     out-of-bounds access.
 *   - Inputs must be finite.  Results are deterministic (bit-identical from run to run).
 *   - Device pointers must be 16-byte aligned (anything from hipMalloc is).
 */
#ifndef FQ_H
#define FQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FQ_F32 = 0,
    FQ_F16 = 1,
    FQ_BF16 = 2,
    FQ_I32 = 3   /* raw int32 accumulators (GEMM output only; for verification) */
} fq_dtype;

enum {
    FQ_OK = 0,
    FQ_ERR_NULL = 1,       /* a required pointer is NULL */
    FQ_ERR_SHAPE = 2,      /* non-positive size, Kpad not a multiple of 32, stride too small, capacity too small */
    FQ_ERR_DTYPE = 3,      /* dtype / bit width not supported by this call */
    FQ_ERR_RANGE = 4,      /* T <= 0 or not finite, channel maximum negative / NaN / Inf, size beyond int32 or accumulator bounds */
    FQ_ERR_ALIGN = 5,      /* a device pointer is not 16-byte aligned */
    FQ_ERR_HIP = 6,        /* a HIP launch failed */
    FQ_ERR_WORKSPACE = 7,  /* workspace_bytes smaller than the matching *_workspace_bytes() */
    FQ_ERR_NOMEM = 8       /* a host-side helper could not allocate its temporary (host functions only) */
};

/* Human-readable reason of the last error on the calling thread ("" if none). */
const char* fq_last_error_string(void);

/* Library version: major*10000 + minor*100 + patch. */
int fq_version(void);

/* ---------------------------------------------------------------------------------------------
 * fq_flatten_plan — channel maxima and T -> the channel index / repeat map.   HOST function.
 * Sec. 4.1 Eq. 2 (number of channels per input channel), Eq. 3 (index layout), Sec. 5.1 (padding).
 *
 *   n_j = max(1, ceil(chmax_j / T))  (ratio in float64), E_j = n_j - 1 extra channels,
 *   Kprime = K + sum_j E_j,  Kpad = Kprime rounded up to a multiple of `align`.
 *   Slots 0..K-1 keep the original channels (src_idx[p] = p).  The E_j extras of channel j occupy
 *   slots K + sum_{k<j} E_k ... in increasing j.  Slots Kprime..Kpad-1 are padding (src -1, rep 0).
 *   (Eq. 2 prints floor(max/T) extra channels; that equals n_j - 1 except when max is an exact
 *   multiple of T, where the printed form would add one channel that is always zero.)
 *
 * chmax_host  [K] fp32, host; each >= 0 and finite.       T > 0, finite.
 * align       > 0; must be a multiple of 32 for the map to be usable by the device calls.
 * src_idx_host, rep_host  [cap] int32, host, written up to Kpad entries.
 * cap = 0: size query only (src/rep may be NULL); Kprime_out / Kpad_out (either may be NULL)
 *          are written.  cap > 0 and cap < Kpad: FQ_ERR_SHAPE, sizes still written.
 * ------------------------------------------------------------------------------------------- */
int fq_flatten_plan(const float* chmax_host, int K, float T, int align,
                    int32_t* src_idx_host, int32_t* rep_host, int cap,
                    int* Kprime_out, int* Kpad_out);

/* ---------------------------------------------------------------------------------------------
 * fq_channel_absmax, fq_threshold_boxplot, fq_smooth_scales — the paper's offline policy for the
 * plan's inputs.  The latter two are HOST functions.
 *
 * fq_threshold_boxplot (Sec. 4.2 Eq. 6-7): the channel maxima are clipped to the box-plot fences
 *   [Q1 - 1.5 IQR, Q3 + 1.5 IQR] (quartiles by linear interpolation) and
 *   T = beta * mean(clipped maxima); the paper uses beta = 1.3.  chmax_host [K] >= 0, finite.
 * fq_smooth_scales (Sec. 4.2 Eq. 5):
 *   s_j = Sigmoid((max|X_j| - mu)/sigma)^alpha / Sigmoid((max|W_j| - mu)/sigma)^(1 - alpha),
 *   mu / sigma = mean / population standard deviation of the activation channel maxima (the weight
 *   term uses the same mu and sigma, as printed); alpha in [0, 1], the paper uses 0.5.  The smoothed
 *   layer is X diag(s)^-1 and diag(s) W (to be folded into the producer of X and into W offline).
 *   sigma = 0 gives s_j = 1.  chmax_w_host[j] = max_n |W[n, j]|.
 * Both evaluate in float64 and round the results to fp32.
 * ------------------------------------------------------------------------------------------- */
/* fq_channel_absmax — calibration statistic on the device (Sec. 4.2: the per-channel maxima that
 *   Eq. 2, Eq. 5 and Eq. 6 consume).  chmax_dev[j] = max(start_j, max_i |X[i, j]|) with start_j = 0,
 *   or, with accumulate != 0, the value chmax_dev[j] holds on entry (a running maximum over
 *   calibration batches; it must be a non-negative, non-NaN fp32).  NaN elements of X are ignored.
 *   X [M, K] DEVICE, F32 / F16 / BF16, row stride ldx elements (ldx * element size a multiple of 16,
 *   X 16-byte aligned); chmax_dev fp32 [K] DEVICE; asynchronous on `stream`; no workspace. */
int fq_channel_absmax(const void* X, int x_dtype, int M, int K, int ldx, int accumulate, float* chmax_dev,
                      void* stream);
int fq_threshold_boxplot(const float* chmax_host, int K, float beta, float* T_out_host);
int fq_smooth_scales(const float* chmax_x_host, const float* chmax_w_host, int K, float alpha, float* s_out_host);

/* ---------------------------------------------------------------------------------------------
 * fq_flatten_weights — offline: quantize W per tensor and repeat its channels by the map.
 * Eq. 1 (s_w = max|W| / qmax, qmax = 2^(bits-1) - 1), Eq. 4 (repeat); an offline step that belongs to
 * quantizing the model, not to inference (Fig. 3).
 *
 *   m_w = fl32(qmax / max|W|) (quotient in float64),  Wq[n,j] = clamp(rne(W[n,j] * m_w), qmin, qmax),
 *   Wq_out[n,p] = Wq[n, src_idx[p]], 0 in padding slots; bits = 4 packs two slots per byte.
 *   All-zero W: Wq_out = 0, s_w = 1.
 *
 * W        [N, K] device, w_dtype in {FQ_F32, FQ_F16, FQ_BF16}, row stride ldw >= K elements.
 * Wq_out   [N, Kpad] int8 (bits 8) or [N, Kpad/2] uint8 (bits 4), device.  bits = FQ_BITS_I4_E3M2 (6): the
 *          4-bit quantizer with its values stored as E3M2 codes, N * 3 Kpad / 4 bytes in the blocked layout
 *          described at fq_gemm_i4_e3m2 (Kpad a multiple of 128); likewise for Xq_out of the activation calls.
 * s_w_out  one fp32, device.
 * workspace  fq_weights_workspace_bytes(K, Kpad) bytes, device, 16-byte aligned; contents undefined after.
 * ------------------------------------------------------------------------------------------- */
int fq_flatten_weights(const void* W, int w_dtype, int N, int K, int ldw,
                       const int32_t* src_idx, int Kpad, int bits,
                       void* Wq_out, float* s_w_out,
                       void* workspace, size_t workspace_bytes, void* stream);
size_t fq_weights_workspace_bytes(int K, int Kpad);

/* ---------------------------------------------------------------------------------------------
 * fq_flatten_quant_act — inference time: fused flatten (gather + equal split) and per-tensor
 * quantization of the activation.  Eq. 3 in its equal-split form (each of the n_j copies of
 * channel j holds x / n_j), then Eq. 1.
 *
 *   a' = absmax of the flattened tensor:
 *        static  (absmax_in != NULL): *absmax_in, e.g. the calibrated bound T — the paper's
 *                 setting (Table 2: per-tensor static);
 *        dynamic (absmax_in == NULL): max_p fl32( max_i |X[i,src_idx[p]]| / rep[p] ), taken from X.
 *   s_x = fl32(a' / qmax),  m_p = fl32(qmax / (rep[p] * a'))  (both formed in float64),
 *   Xq_out[i,p] = clamp(rne(X[i,src_idx[p]] * m_p), qmin, qmax); 0 in padding slots;
 *   bits = 4 packs two slots per byte.   a' = 0: Xq_out = 0, s_x = 1.
 *
 * X         [M, K] device, x_dtype in {FQ_F32, FQ_F16, FQ_BF16}, row stride ldx >= K elements;
 *           ldx * sizeof(element) must be a multiple of 16.
 * Xq_out    [M, Kpad] int8 or [M, Kpad/2] uint8, device.
 * s_x_out   one fp32, device.
 * workspace fq_act_workspace_bytes(K, Kpad) bytes, device, 16-byte aligned.
 * ------------------------------------------------------------------------------------------- */
int fq_flatten_quant_act(const void* X, int x_dtype, int M, int K, int ldx,
                         const int32_t* src_idx, const int32_t* rep, int Kpad, int bits,
                         const float* absmax_in, void* Xq_out, float* s_x_out,
                         void* workspace, size_t workspace_bytes, void* stream);
size_t fq_act_workspace_bytes(int K, int Kpad);

/* ---------------------------------------------------------------------------------------------
 * fq_flatten_quant_act_noalloc — fq_flatten_quant_act for callers that cannot allocate device memory
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the workspace is
 * a fixed array of FQ_NOALLOC_SCRATCH_BYTES that is part of the library's device image (one copy on every
 * GPU that loads the library, held until the process ends), so the caller passes inputs and outputs only.
 * The call allocates and frees nothing, and computes exactly what fq_flatten_quant_act computes (same
 * kernels, same bytes).
 *
 * Limit: fq_act_workspace_bytes(K, Kpad) <= FQ_NOALLOC_SCRATCH_BYTES (e.g. K = 32768 with Kpad = 65536),
 * else FQ_ERR_WORKSPACE and nothing is enqueued.  The first call on a device looks the array's address up
 * (hipGetSymbolAddress; FQ_ERR_HIP if that fails).
 * All calls on one GPU share that GPU's array and it keeps the previous call's contents; what has to start
 * at zero is cleared by a kernel inside every call (no memset node, so the call may be captured).  Calls
 * that overlap on one GPU (different streams, or threads without ordering) race on the array: order them.
 * ------------------------------------------------------------------------------------------- */
#define FQ_NOALLOC_SCRATCH_BYTES (1u << 20)
int fq_flatten_quant_act_noalloc(const void* X, int x_dtype, int M, int K, int ldx,
                                 const int32_t* src_idx, const int32_t* rep, int Kpad, int bits,
                                 const float* absmax_in, void* Xq_out, float* s_x_out, void* stream);
size_t fq_noalloc_scratch_bytes(void);

/* ---------------------------------------------------------------------------------------------
 * Eq. 3 as printed ("peel" split) and flattening of the weights' own channels (Sec. 4.1, last
 * paragraph).  The map layout, the GEMM and its epilogue are the ones above.
 *
 * fq_flatten_plan_xw — HOST.  Channel j is split into nx_j = max(1, ceil(chmax_x[j] / T_x)) shares on
 *   the activation side and, when chmax_w_host != NULL (chmax_w[j] = max_n |W[n, j]|), into
 *   nw_j = max(1, ceil(chmax_w[j] / T_w)) shares on the weight side; x*w is then the sum over
 *   nx_j * nw_j slots of (x / nx_j)(w / nw_j), so channel j occupies that many slots: index j plus
 *   appended slots, channels in increasing j (Eq. 3's index rule).  Per slot: src_idx, rep_x = nx,
 *   rep_w = nw (may be NULL), ord = the slot's ordinal within its channel, 0 at the original position
 *   (may be NULL).  Padding: -1, 0, 0, 0.  With chmax_w_host == NULL, src_idx / rep_x equal
 *   fq_flatten_plan's.  cap = 0 queries the sizes, as in fq_flatten_plan.
 *
 * fq_flatten_weights_split — weights with their own large channels split into equal shares:
 *   slot p of row n holds W[n, src_idx[p]] / rep_w[p], quantized per tensor with
 *   a_w = max_p fl32(max_n |W[n, src_idx[p]]| / rep_w[p]) exactly as fq_flatten_quant_act does for the
 *   activation (dynamic).  Pair it with fq_flatten_quant_act(X, src_idx, rep_x).
 *
 * fq_flatten_quant_act_peel — the split Eq. 3 prints: the slot with ordinal e of channel j holds
 *   v = sign(x) * min(max(|x| - fl32(e * T), 0), T)  (floor(|x| / T) slots of T, the remainder, zeros;
 *   negative values through |x|), then Eq. 1 with a single multiplier:
 *   Xq = clamp(rne(fl32(v * m)), qmin, qmax), m = fl32(qmax / a'), s_x = fl32(a' / qmax);
 *   a' = *absmax_in when given (the paper's static setting: a' = T), else min(T, max |X|).
 *   The weights are plainly repeated (fq_flatten_weights) for this split; ord comes from
 *   fq_flatten_plan_xw with chmax_w_host = NULL.  Buffers, workspace and limits as fq_flatten_quant_act.
 * ------------------------------------------------------------------------------------------- */
int fq_flatten_plan_xw(const float* chmax_x_host, float T_x, const float* chmax_w_host, float T_w, int K, int align,
                       int32_t* src_idx_host, int32_t* rep_x_host, int32_t* rep_w_host, int32_t* ord_host,
                       int cap, int* Kprime_out, int* Kpad_out);
int fq_flatten_weights_split(const void* W, int w_dtype, int N, int K, int ldw,
                             const int32_t* src_idx, const int32_t* rep_w, int Kpad, int bits,
                             void* Wq_out, float* s_w_out, void* workspace, size_t workspace_bytes, void* stream);
int fq_flatten_quant_act_peel(const void* X, int x_dtype, int M, int K, int ldx,
                              const int32_t* src_idx, const int32_t* ord, int Kpad, int bits, float T,
                              const float* absmax_in, void* Xq_out, float* s_x_out,
                              void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * fq_gemm_i8 / fq_gemm_i4 — integer GEMM with int32 accumulation and the fused per-tensor
 * dequantize epilogue (Sec. 5.1; the inverse of Eq. 1 applied to the product).
 *
 *   acc[i,n] = sum_{p < Kpad} Xq[i,p] * Wq[n,p]                      (exact, int32)
 *   Y[i,n]   = round_to_y_dtype( fl32( fl32(acc[i,n]) * fl32(*s_x * *s_w) ) )   for F32 / F16 / BF16
 *   Y[i,n]   = acc[i,n]                                                for FQ_I32 (scales may be NULL)
 * Two roundings for 2-byte outputs: the product is rounded to fp32 first and that value is rounded (half to
 * even; halves overflow to infinity and go subnormal as IEEE prescribes) to the output type.  Every stored bit
 * is defined by this and is what the tests compare.
 *
 * fq_gemm_i4 takes both operands packed two per byte ([M, Kpad/2], [N, Kpad/2]); they stay
 * packed in HBM and LDS and are widened to int8 in registers (gfx950 has no 4-bit MFMA).
 * M, N >= 1; Kpad a multiple of 32 with Kpad * 128 * 128 < 2^31; each quantized operand smaller than
 * 4 GiB (M, N times the bytes of a quantized row; FQ_ERR_RANGE otherwise: rows are addressed with 32-bit
 * byte offsets).
 * s_x, s_w  device scalars read by the kernel (no host synchronization).
 * Y         device, row stride ldy >= N elements.  2-byte outputs leave fastest when Y is 128-byte aligned
 *           and ldy is a multiple of 64 elements (whole cache lines per row segment).
 * ------------------------------------------------------------------------------------------- */
int fq_gemm_i8(const int8_t* Xq, const int8_t* Wq, int M, int N, int Kpad,
               const float* s_x, const float* s_w, void* Y, int y_dtype, int ldy, void* stream);
int fq_gemm_i4(const uint8_t* Xq, const uint8_t* Wq, int M, int N, int Kpad,
               const float* s_x, const float* s_w, void* Y, int y_dtype, int ldy, void* stream);

/* fq_gemm_i8_bias / fq_gemm_i4_bias / fq_linear_bias — the same calls with the layer's bias folded
 * into the epilogue (the paper's quantized layer replaces OPT's linear layers, which carry one; it
 * does not spell the bias out, the reading taken: added in floating point after dequantization):
 *   Y[i,n] = round_to_y_dtype( fl32( fl32(fl32(acc[i,n]) * fl32(*s_x * *s_w)) + bias[n] ) ).
 * bias  fp32 [N], device, 16-byte aligned; NULL gives exactly the calls above.  Not allowed with
 *       FQ_I32 output (FQ_ERR_DTYPE). */
int fq_gemm_i8_bias(const int8_t* Xq, const int8_t* Wq, int M, int N, int Kpad,
                    const float* s_x, const float* s_w, const float* bias,
                    void* Y, int y_dtype, int ldy, void* stream);
int fq_gemm_i4_bias(const uint8_t* Xq, const uint8_t* Wq, int M, int N, int Kpad,
                    const float* s_x, const float* s_w, const float* bias,
                    void* Y, int y_dtype, int ldy, void* stream);

/* ---------------------------------------------------------------------------------------------
 * fq_gemm_i4_e3m2 — the 4-bit layer's integer GEMM on operands stored as 6-bit codes.
 * Sec. 5.1 (4-bit GEMM of the quantized linear layer), Eq. 1 with k = 4.  What is computed is exactly
 * fq_gemm_i4_bias: the quantized values are the same integers in [-8, 7].  Only their storage differs,
 * which lets the product run on gfx950's 6-bit matrix pipe at twice the INT8 rate (there is no 4-bit
 * integer MFMA; the nibble path widens to int8):
 *
 *   storage  the value q of slot p is held as the 6-bit E3M2 floating-point code of the integer q
 *            (sign, 3 exponent bits with bias 3, 2 mantissa bits; every integer in [-8, 8] is exactly
 *            representable: 0 -> 0, |q| -> exponent floor(log2|q|) + 3, top two fraction bits of |q|).
 *            Layout: blocked along the flattened-channel axis.  Block t holds, for row 0, 1, ... in turn,
 *            96 bytes with that row's codes p = 128 t .. 128 t + 127; byte address of a row's piece:
 *            (t * rows + row) * 96; total size rows * 3 Kpad / 4 bytes.  The piece is two 48-byte groups of
 *            64 codes, each group two units of 32 codes.  A unit's codes form a little-endian bit stream of
 *            24 bytes (code u of the unit in bits 6u .. 6u+5; bit b is bit b%8 of byte b/8), split into
 *            its first 16 bytes X and last 8 bytes Y.  A group is stored X_a Y_a Y_b X_b, with (a, b) =
 *            (0, 1) in rows whose index has bit 4 clear and (1, 0) in rows with bit 4 set.
 *            (Why: a k-stage of a GEMM tile is one contiguous run of whole cache lines, every lane of the
 *            matrix instruction finds its 24 bytes as one aligned 16-byte and one aligned 8-byte piece,
 *            and the LDS reads of 32 consecutive rows are free of bank conflicts.)
 *   product  every product of two codes is an integer of magnitude <= 64 and the fp32 accumulator of
 *            the MFMA is exact below 2^24 > 64 Kpad, so acc[i,n] equals the int32 accumulator of
 *            fq_gemm_i4 bit for bit; the epilogue (scales, bias, rounding, FQ_I32 output) is the same.
 *
 * Produced by fq_flatten_weights / fq_flatten_quant_act / fq_flatten_weights_split / fq_linear[_bias]
 * when called with bits = FQ_BITS_I4_E3M2 (the 4-bit quantizer of Eq. 1, E3M2 storage; Wq then has to be
 * in this storage too).  Kpad must be a multiple of 128 (whole blocks; a plan made with align = 128).
 * The peel split has no E3M2 form (FQ_ERR_DTYPE).  bias may be NULL.
 * ------------------------------------------------------------------------------------------- */
#define FQ_BITS_I4_E3M2 6
int fq_gemm_i4_e3m2(const uint8_t* Xq, const uint8_t* Wq, int M, int N, int Kpad,
                    const float* s_x, const float* s_w, const float* bias,
                    void* Y, int y_dtype, int ldy, void* stream);

/* ---------------------------------------------------------------------------------------------
 * fq_bmm_i8 / fq_bmm_i4 — the batched form of the integer GEMM (Sec. 5.1: the quantized BMM function
 * that stands beside the quantized linear layer, for attention's two products).  The paper gives
 * no detail beyond INT8 / INT4 operands; the reading taken: per-tensor scales over the whole batched
 * tensors, no flattening of these operands.
 *
 *   acc[b,i,n] = sum_{p < Kpad} Aq[b,i,p] * Bq[b,n,p],   b < batch            (exact, int32)
 *   Y[b,i,n]   = the epilogue of fq_gemm_i8 with *s_a, *s_b.
 *
 * Aq  batch matrices [M, Kpad] int8 (fq_bmm_i4: [M, Kpad/2] packed), rows dense, matrix b at byte
 *     offset b * stride_a; Bq likewise [N, Kpad] with stride_b.  Strides are in bytes, multiples of
 *     16, at least one matrix.  Both operands have the reduction index last: for P V pass V^T.
 * Y   matrix b at element offset b * stride_y, row stride ldy >= N elements.
 * batch in [1, 65535]; other limits as fq_gemm_i8.  To quantize an operand per tensor, call
 * fq_flatten_quant_act on its [batch * rows, K] view with an identity map (T above every channel maximum).
 * ------------------------------------------------------------------------------------------- */
int fq_bmm_i8(const int8_t* Aq, const int8_t* Bq, int batch, int M, int N, int Kpad,
              long long stride_a, long long stride_b, const float* s_a, const float* s_b,
              void* Y, int y_dtype, int ldy, long long stride_y, void* stream);
int fq_bmm_i4(const uint8_t* Aq, const uint8_t* Bq, int batch, int M, int N, int Kpad,
              long long stride_a, long long stride_b, const float* s_a, const float* s_b,
              void* Y, int y_dtype, int ldy, long long stride_y, void* stream);

/* ---------------------------------------------------------------------------------------------
 * fq_linear — the end-to-end inference call: fq_flatten_quant_act followed by fq_gemm_i8 /
 * fq_gemm_i4 (fq_gemm_i4_e3m2 for bits = FQ_BITS_I4_E3M2) on one stream.  Wq / s_w come from
 * fq_flatten_weights with the same map and bits.
 * workspace  fq_linear_workspace_bytes(M, K, Kpad, bits) bytes, device, 16-byte aligned; holds
 *            the quantized activation, the per-slot multipliers and s_x.
 * ------------------------------------------------------------------------------------------- */
int fq_linear(const void* X, int x_dtype, int M, int K, int ldx,
              const int32_t* src_idx, const int32_t* rep, int Kpad,
              const void* Wq, const float* s_w, int N, int bits,
              const float* absmax_in, void* Y, int y_dtype, int ldy,
              void* workspace, size_t workspace_bytes, void* stream);
int fq_linear_bias(const void* X, int x_dtype, int M, int K, int ldx,
                   const int32_t* src_idx, const int32_t* rep, int Kpad,
                   const void* Wq, const float* s_w, const float* bias, int N, int bits,
                   const float* absmax_in, void* Y, int y_dtype, int ldy,
                   void* workspace, size_t workspace_bytes, void* stream);
size_t fq_linear_workspace_bytes(int M, int K, int Kpad, int bits);

/* ---------------------------------------------------------------------------------------------
 * fq_linear_fused_a_i8 — the INT8 layer with flatten + quantize fused into the GEMM's A-operand load (Sec. 6,
 * named there as future work): fq_linear_bias for bits = 8 without the quantized activation ever being written to
 * memory.  The scale (static *absmax_in, or NULL = dynamic: one absmax pass over X) and the per-slot multipliers
 * are formed first; the GEMM then reads X itself and quantizes slot p of a row from X[row, src_idx[p]] on the way
 * into LDS, with the arithmetic of fq_flatten_quant_act.  Results are identical to fq_linear_bias, bit for bit,
 * for every output type.  Every 128-column tile of the output converts its rows of X again, inside the MFMA loop:
 * measured 2.4 to 4.8 times slower than fq_linear_bias at every shape tried (narrow outputs included).  It is
 * the measured answer to that future-work item, not a path to prefer.
 * X bf16 only (FQ_ERR_DTYPE otherwise); workspace >= fq_act_workspace_bytes(K, Kpad); other arguments, layouts,
 * ownership and errors as fq_linear_bias.  fq_gemm_select does not apply (one kernel).
 * ------------------------------------------------------------------------------------------- */
int fq_linear_fused_a_i8(const void* X, int x_dtype, int M, int K, int ldx, const int32_t* src_idx, const int32_t* rep,
                         int Kpad, const void* Wq, const float* s_w, const float* bias, int N, const float* absmax_in,
                         void* Y, int y_dtype, int ldy, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * fq_gemm_bf16 — the unquantized baseline the paper compares against (Table 5, "Gemm (FP16)"):
 * Y = X W^T with bf16 operands, fp32 accumulation on the bf16 MFMA, bf16 output.
 * X [M, K], W [N, K] device bf16, dense rows; K a multiple of 8.  Y [M, N] bf16, row stride ldy.
 * ------------------------------------------------------------------------------------------- */
int fq_gemm_bf16(const void* X, const void* W, int M, int N, int K, void* Y, int ldy, void* stream);

/* ---------------------------------------------------------------------------------------------
 * fq_gemm_select — tuning and test hook: force the kernel variant that fq_gemm_i8 / fq_gemm_i4 / fq_gemm_bf16 /
 * fq_bmm_* / fq_linear use ON THE CALLING THREAD (thread-local; other threads keep their own choice, so the
 * GEMM entry points stay re-entrant).  -1 (default) = chosen from the shape.
 *   7:  256x256 tile, 128-byte k-stages, 8 waves, direct global->LDS copies, ping-pong schedule: the two
 *       waves of a SIMD alternate LDS-read and MFMA phases, two MFMA k-steps per phase.  One workgroup per
 *       CU walks its tiles and fetches the first stage of the next tile before it stores the current one.
 *   10: as 7 with phases twice as long (four MFMA k-steps per phase); large INT4 problems that 12 cannot run.
 *   11: INT8 and bf16 only, rows of whole 128-byte stages only (FQ_ERR_SHAPE otherwise, before anything is
 *       enqueued): 256x256 tile, 4 waves with 128x128 wave tiles (one wave per SIMD), two stage buffers, LDS
 *       reads and copies dealt out per MFMA slot.
 *   12: as 11 with all of LDS as stage buffers (A three deep, B two deep) so that the global->LDS copies are
 *       spread over the whole stage, one copy instruction of one wave per MFMA slot; also for packed INT4, whose
 *       nibble widening is dealt out over the MFMA slots as well.  The choice for problems of 80 (INT8, bf16) or
 *       176 (INT4) tiles and more with such rows and a bf16 output without bias; other outputs keep 7 (INT8,
 *       bf16) or 10 (INT4).
 *   6:  128x128 tile, 4 waves, direct global->LDS copies (small problems, narrow outputs).
 *   2:  128x128 tile, 64-byte k-stages, 4 waves, operands staged through registers.
 * fq_gemm_i4_e3m2 has a single kernel and ignores the hook.
 * Every variant computes the same values.  Returns FQ_ERR_RANGE for an unknown variant.
 * ------------------------------------------------------------------------------------------- */
int fq_gemm_select(int variant);

#ifdef __cplusplus
}
#endif
#endif /* FQ_H */
