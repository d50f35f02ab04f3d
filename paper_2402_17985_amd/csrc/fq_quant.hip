// Flatten + per-tensor quantize kernels (activation path at inference time, weight path offline).
//
// arXiv 2402.17985: Sec. 4.1 Eq. 3 (flatten, equal-split form: each of the n copies of a
// channel holds x/n), Eq. 4 (weight channel repeated), Sec. 2.1 Eq. 1 (per-tensor scale
// s = max|.| / qmax, round, here round-half-even, then clamp).
//
// The kernels, all bandwidth or latency bound:
//   colabsmax           per input channel max|x| over the rows (64-wide wave reads 1 KiB of a row per
//                       instruction; per-thread running max; one atomic max per column per block;
//                       the max of non-negative floats is taken on their bit patterns, so the
//                       result does not depend on the order of the updates)
//   scale               per-tensor absmax a' by wavefront reductions, the scale s, the per-slot
//                       multiplier m_p = fl32(qmax / (n_p * a')) (float64 quotient), and two flags
//                       per group of 16 slots that tell the quantizer which path a group may take
//   flatten_quant_rows  the quantizer of the equal split: a workgroup owns a strip of rows, reads the
//                       head of the map with vector loads, keeps the quantized bytes in LDS and lets
//                       the appended copies take their values from there
//   flatten_quant       the general form (one thread per 16 slots and strip of rows, every slot
//                       gathered from global memory): the peel split of Eq. 3 as printed, and layers
//                       too wide for the row-strip kernel's LDS budget
#include <atomic>

#include "fq_internal.h"

namespace fq {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
// 12 bytes at 4-byte alignment (a 3-element vector type would claim 16)
struct __attribute__((aligned(4))) u3 { uint32_t a, b, c; };

// 6-bit E3M2 code (sign, 3 exponent bits with bias 3, 2 mantissa bits) of an integer-valued float r in
// [-8, 8]: the fp32 form of |r| already holds the exponent and, in its top mantissa bits, the two
// mantissa bits (exponent field 127 + e -> 3 + e: subtract 124 << 2 after the shift); 0 -> 0.
__device__ __forceinline__ int e3m2_code_of_float(float r)
{
    const uint32_t bits = __float_as_uint(r + 0.0f);                   // -0 -> +0
    const int mag = max((int)((bits & 0x7fffffffu) >> 21) - (124 << 2), 0);
    return mag | (int)((bits >> 26) & 0x20u);
}
// 16 codes as a 96-bit little-endian bit stream (code i in bits 6 i .. 6 i + 5)
__device__ __forceinline__ u3 pack16_e3m2(const int (&c)[16])
{
    uint32_t g[4];                                                     // four codes = 24 bits
#pragma unroll
    for (int i = 0; i < 4; ++i)
        g[i] = (uint32_t)c[4 * i] | ((uint32_t)c[4 * i + 1] << 6) | ((uint32_t)c[4 * i + 2] << 12) | ((uint32_t)c[4 * i + 3] << 18);
    return u3{g[0] | (g[1] << 24), (g[1] >> 8) | (g[2] << 16), (g[2] >> 16) | (g[3] << 8)};
}

template <int DT> struct Elem;
template <> struct Elem<FQ_F32> {
    typedef float type;
    static constexpr int VEC = 4;   // elements per 16 bytes
    static __device__ __forceinline__ float widen(float v) { return v; }
};
template <> struct Elem<FQ_F16> {
    typedef _Float16 type;
    static constexpr int VEC = 8;
    static __device__ __forceinline__ float widen(_Float16 v) { return (float)v; }
};
template <> struct Elem<FQ_BF16> {
    typedef uint16_t type;
    static constexpr int VEC = 8;
    static __device__ __forceinline__ float widen(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
};

// Widen one 16-byte vector of storage elements to floats.
template <int DT> __device__ __forceinline__ void widen16(const v4u raw, float* out);
template <> __device__ __forceinline__ void widen16<FQ_F32>(const v4u raw, float* out)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) out[i] = __uint_as_float(raw[i]);
}
template <> __device__ __forceinline__ void widen16<FQ_BF16>(const v4u raw, float* out)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        out[2 * i] = __uint_as_float(raw[i] << 16);
        out[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u);
    }
}
template <> __device__ __forceinline__ void widen16<FQ_F16>(const v4u raw, float* out)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        union { uint32_t u; _Float16 h[2]; } cv;
        cv.u = raw[i];
        out[2 * i] = (float)cv.h[0];
        out[2 * i + 1] = (float)cv.h[1];
    }
}

__global__ void fill_u32_kernel(uint32_t* p, int count, uint32_t v)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = v;
}

// ---------------------------------------------------------------------------------------------
// per input channel absmax
// ---------------------------------------------------------------------------------------------
// Workgroup = 4 waves.  The 64 lanes of a wave cover 64 adjacent 16-byte column groups (1 KiB of a
// row per load); the 4 waves take interleaved rows of the block's row strip, each lane keeping
// sixteen loads in flight.  The 4 partial maxima
// of a column meet in LDS and one lane issues the atomic max, and only if its value exceeds what the
// column already holds (the stored value only grows, so a stale read can only cause a redundant
// atomic, never a missed one).
template <int DT>
__global__ __launch_bounds__(256) void colabsmax_kernel(const void* __restrict__ Xv, int M, int K, int ld,
                                                        int rows_per_block, uint32_t* __restrict__ cmax)
{
    typedef typename Elem<DT>::type T;
    constexpr int VEC = Elem<DT>::VEC;
    __shared__ float part[4][64 * VEC];
    const T* X = static_cast<const T*>(Xv);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col0 = (blockIdx.x * 64 + lane) * VEC;
    const int r0 = blockIdx.y * rows_per_block;
    const int r1 = min(M, r0 + rows_per_block);
    float mx[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) mx[v] = 0.0f;
    if (col0 + VEC <= K) {
        // wave w takes rows r0 + w, r0 + w + 4, ...; sixteen 16-byte loads in flight per lane
        const T* p = X + (size_t)(r0 + wave) * ld + col0;
        const size_t step = (size_t)4 * ld;
        int r = r0 + wave;
        for (; r + 60 < r1; r += 64, p += 16 * step) {
            v4u raw[16];
#pragma unroll
            for (int q = 0; q < 16; ++q) raw[q] = *reinterpret_cast<const v4u*>(p + q * step);
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                float f[VEC];
                widen16<DT>(raw[q], f);
#pragma unroll
                for (int v = 0; v < VEC; ++v) mx[v] = fmaxf(mx[v], fabsf(f[v]));
            }
        }
        for (; r + 12 < r1; r += 16, p += 4 * step) {
            v4u raw[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) raw[q] = *reinterpret_cast<const v4u*>(p + q * step);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float f[VEC];
                widen16<DT>(raw[q], f);
#pragma unroll
                for (int v = 0; v < VEC; ++v) mx[v] = fmaxf(mx[v], fabsf(f[v]));
            }
        }
        for (; r < r1; r += 4, p += step) {
            float f[VEC];
            widen16<DT>(*reinterpret_cast<const v4u*>(p), f);
#pragma unroll
            for (int v = 0; v < VEC; ++v) mx[v] = fmaxf(mx[v], fabsf(f[v]));
        }
    } else if (col0 < K) {                                       // ragged last column group
        for (int v = 0; col0 + v < K; ++v)
            for (int r = r0 + wave; r < r1; r += 4)
                mx[v] = fmaxf(mx[v], fabsf(Elem<DT>::widen(X[(size_t)r * ld + col0 + v])));
    }
#pragma unroll
    for (int v = 0; v < VEC; ++v) part[wave][lane * VEC + v] = mx[v];
    __syncthreads();
    // 256 threads finish 64*VEC columns
    for (int c = threadIdx.x; c < 64 * VEC; c += 256) {
        const int col = blockIdx.x * 64 * VEC + c;
        if (col < K) {
            const float m = fmaxf(fmaxf(part[0][c], part[1][c]), fmaxf(part[2][c], part[3][c]));
            const uint32_t bits = __float_as_uint(m);
            if (bits > __hip_atomic_load(&cmax[col], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(&cmax[col], bits);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// per-tensor absmax, scale and per-slot multipliers (one workgroup)
// ---------------------------------------------------------------------------------------------
// The per-tensor absmax of the flattened tensor is max_p fl32(c_p / n_p) with c_p the channel
// maximum behind slot p and n_p its copy count.  Rounding is monotonic, so it equals
// fl32(c* / n*) for the pair with the largest exact quotient; pairs are compared exactly by cross
// multiplication in float64 (24-bit x n products, exact for n < 2^29), leaving a single division at
// the end.
struct Quot {
    float c;
    int n;
};
__device__ __forceinline__ Quot quot_max(Quot a, Quot b)
{
    return ((double)b.c * (double)a.n > (double)a.c * (double)b.n) ? b : a;
}
__device__ __forceinline__ Quot wave_quot_max(Quot q)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        Quot o;
        o.c = __shfl_xor(q.c, off, 64);
        o.n = __shfl_xor(q.n, off, 64);
        q = quot_max(q, o);
    }
    return q;
}

// Every workgroup recomputes the absmax a' (a cheap reduction over the map), tabulates the
// multipliers m(n) = fl32(qmax / (n * a')) for n < 1024 in LDS (one float64 division per thread),
// and fills its own 1024 slots of mslot.  Workgroup 0 also writes the scale.
__global__ __launch_bounds__(1024) void scale_kernel(const uint32_t* __restrict__ cmax, int K,
                                                     const int32_t* __restrict__ src,
                                                     const int32_t* __restrict__ rep, int Kpad, int qmax,
                                                     int mode, const float* __restrict__ absmax_in, float T,
                                                     float* __restrict__ mslot, float* __restrict__ scale_out,
                                                     float* __restrict__ scalars, uint8_t* __restrict__ gflag)
{
    // Peel split (modes 3 dynamic / 4 static): `rep` carries the slot ordinals e; mslot[p] receives the
    // offset fl32(e * T) that the slot subtracts from |x| (+inf in padding, which clamps to 0), and the
    // single multiplier m = fl32(qmax / a') goes to scalars[2].  a' = min(T, max_j cmax[j]) when dynamic.
    if (mode >= 3) {
        __shared__ float redf[16];
        __shared__ float a_peel;
        const int tid = threadIdx.x;
        float a;
        if (mode == 3) {
            float best = 0.0f;
#pragma unroll 8
            for (int j = tid; j < K; j += 1024) best = fmaxf(best, __uint_as_float(cmax[j]));
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) best = fmaxf(best, __shfl_xor(best, off, 64));
            if ((tid & 63) == 0) redf[tid >> 6] = best;
            __syncthreads();
            if (tid == 0) {
                float t = 0.0f;
                for (int w = 0; w < 16; ++w) t = fmaxf(t, redf[w]);
                a_peel = fminf(t, T);
            }
            __syncthreads();
            a = a_peel;
        } else {
            a = *absmax_in;
            if (!(a >= 0.0f) || a > 3.0e38f) a = 0.0f;
        }
        if (blockIdx.x == 0 && tid == 0) {
            *scale_out = (a == 0.0f) ? 1.0f : (float)((double)a / (double)qmax);
            scalars[0] = a;
            scalars[2] = (a == 0.0f) ? 0.0f : (float)((double)qmax / (double)a);
        }
        const int p = blockIdx.x * 1024 + tid;
        if (p < Kpad) {
            const int sp = src[p], e = rep[p];
            const bool valid = (unsigned)sp < (unsigned)K && e >= 0;
            mslot[p] = valid ? (float)e * T : __builtin_inff();
        }
        return;
    }
    __shared__ Quot red[16];
    __shared__ float a_shared;
    __shared__ float table[1024];
    const int tid = threadIdx.x;
    float a;
    if (mode != 1) {
        Quot best = {0.0f, 1};
        if (mode == 0) {
            // eight slots per thread at a time: all map loads, then all gathers of the channel maxima, so
            // that a pass costs two memory latencies instead of two per slot
            for (int base = tid; base < Kpad; base += 8 * 1024) {
                int s[8], n[8];
                float c[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int p = base + u * 1024;
                    s[u] = (p < Kpad) ? src[p] : -1;
                    n[u] = (p < Kpad) ? rep[p] : 0;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const bool ok = (unsigned)s[u] < (unsigned)K && n[u] > 0;
                    c[u] = ok ? __uint_as_float(cmax[s[u]]) : 0.0f;
                    if (!ok) n[u] = 1;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) best = quot_max(best, Quot{c[u], n[u]});
            }
        } else {
#pragma unroll 8
            for (int j = tid; j < K; j += 1024) best = quot_max(best, Quot{__uint_as_float(cmax[j]), 1});
        }
        best = wave_quot_max(best);
        if ((tid & 63) == 0) red[tid >> 6] = best;
        __syncthreads();
        if (tid < 64) {
            Quot t = (tid < 16) ? red[tid] : Quot{0.0f, 1};
            t = wave_quot_max(t);
            // the float64 quotient rounded to fp32 is the correctly rounded fp32 quotient
            if (tid == 0) a_shared = (float)((double)t.c / (double)t.n);
        }
        __syncthreads();
        a = a_shared;
    } else {
        a = *absmax_in;
        if (!(a >= 0.0f) || a > 3.0e38f) a = 0.0f;     // negative / NaN / Inf static bound: treated as 0
    }
    const double ad = (double)a;
    if (blockIdx.x == 0 && tid == 0) {
        *scale_out = (a == 0.0f) ? 1.0f : (float)(ad / (double)qmax);
        scalars[0] = a;
    }
    table[tid] = (tid > 0 && a != 0.0f) ? (float)((double)qmax / ((double)tid * ad)) : 0.0f;
    __syncthreads();
    const int p = blockIdx.x * 1024 + tid;
    if (p < Kpad) {
        const int s = src[p];
        const int n = (mode == 2) ? 1 : rep[p];
        const bool valid = (unsigned)s < (unsigned)K && n > 0 && a != 0.0f;
        float m = 0.0f;
        if (valid) m = (n < 1024) ? table[n] : (float)((double)qmax / ((double)n * ad));
        mslot[p] = m;
    }
    // gflag[g] = 1 when the 16 slots of group g are the 16 channels at the same indices (the head of
    // the map): such a group is read with vector loads and its quantized values can be copied by the
    // appended slots that repeat its channels
    const bool ident = p < Kpad && p < K && src[p] == p;
    const unsigned long long bal = __ballot(ident);
    if (p < Kpad && (tid & 15) == 0) gflag[p >> 4] = (((bal >> (tid & 48)) & 0xffffull) == 0xffffull) ? 1 : 0;
    // cflag[g] = 1 when every slot of group g either holds 0 whatever the input (padding) or repeats a
    // channel j < 16 * (K / 16) whose own slot j is the identity slot with the same copy count: the
    // slot's quantized value then equals slot j's and can be copied instead of recomputed
    bool copyable = false;
    if (p < Kpad) {
        const int j = src[p];
        if ((unsigned)j >= (unsigned)K) copyable = true;
        else if (j < ((K >> 4) << 4) && src[j] == j) copyable = (mode == 2) || (rep[p] > 0 && rep[j] == rep[p]);
    }
    const unsigned long long balc = __ballot(copyable);
    // ... and 2 when, in addition, all 16 slots repeat the same channel (the long runs of a large
    // outlier's copies): one value then fills the group
    const int sp = (p < Kpad) ? src[p] : -1;
    const int s0 = __shfl(sp, (tid & 63) & ~15, 64);
    const unsigned long long balu = __ballot(sp == s0 && (unsigned)sp < (unsigned)K);
    uint8_t* cflag = gflag + ((Kpad >> 4) + 1);
    if (p < Kpad && (tid & 15) == 0) {
        const bool all_copy = ((balc >> (tid & 48)) & 0xffffull) == 0xffffull;
        const bool all_same = ((balu >> (tid & 48)) & 0xffffull) == 0xffffull;
        cflag[p >> 4] = all_copy ? (all_same ? 2 : 1) : 0;
    }
}

// ---------------------------------------------------------------------------------------------
// flatten + quantize
// ---------------------------------------------------------------------------------------------
// BITS = 8, 4, or 6 = the 4-bit quantizer with its values stored as 6-bit E3M2 codes (k-blocked layout);
// for 6 the result is the code itself, which is also what the row strip keeps in LDS
template <int BITS> __device__ __forceinline__ int quant1(float x, float m)
{
    constexpr int QB = (BITS == 6) ? 4 : BITS;
    constexpr float hi = (float)((1 << (QB - 1)) - 1);
    constexpr float lo = -(float)(1 << (QB - 1));
    float r = rintf(x * m);                 // one fp32 multiply, then round-half-even
    r = fminf(fmaxf(r, lo), hi);
    if constexpr (BITS == 6) return e3m2_code_of_float(r);
    else return (int)r;
}

// PEEL = false: slot value x * m_p (equal split; m_p from mslot).  PEEL = true: the printed split of
// Eq. 3, slot value sign(x) * clamp(|x| - t_p, 0, thr) times the single multiplier scalars[2], with the
// offsets t_p in mslot.
template <int DT, int BITS, bool PEEL = false>
__global__ __launch_bounds__(256) void flatten_quant_kernel(const void* __restrict__ Xv, int M, int K, int ld,
                                                            const int32_t* __restrict__ src,
                                                            const float* __restrict__ mslot, int Kpad,
                                                            int rows_per_thread, uint8_t* __restrict__ out,
                                                            const float* __restrict__ scalars = nullptr,
                                                            float thr = 0.0f)
{
    typedef typename Elem<DT>::type T;
    constexpr int VEC = Elem<DT>::VEC;
    const T* X = static_cast<const T*>(Xv);
    const int G = Kpad >> 4;                                   // groups of 16 slots per row
    // Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  Remap them so that
    // consecutive logical workgroups (the head and the gathered tail of the same rows) share an XCD:
    // the tail's gathers then hit the lines the head has just brought into that L2.
    const unsigned nwg = gridDim.x, wg = blockIdx.x;
    const unsigned q = nwg >> 3, rem = nwg & 7, xcd = wg & 7, idx = wg >> 3;
    const unsigned lwg = (xcd < rem) ? xcd * (q + 1) + idx : rem * (q + 1) + (xcd - rem) * q + idx;
    const long long gid = (long long)lwg * 256 + threadIdx.x;
    const int g = (int)(gid % G);
    const long long rt = gid / G;
    const long long r0l = rt * rows_per_thread;
    if (r0l >= M) return;
    const int r0 = (int)r0l;
    const int r1 = min(M, r0 + rows_per_thread);
    const int p0 = g << 4;

    int s[16];
    float m[16];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v4i sv = *reinterpret_cast<const v4i*>(src + p0 + 4 * i);
        v4f mv = *reinterpret_cast<const v4f*>(mslot + p0 + 4 * i);
#pragma unroll
        for (int j = 0; j < 4; ++j) { s[4 * i + j] = sv[j]; m[4 * i + j] = mv[j]; }
    }
    bool contig = (s[0] >= 0) && (s[0] % VEC == 0) && (s[0] + 15 < K);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        if ((unsigned)s[i] >= (unsigned)K) {                                            // padding / invalid
            s[i] = 0;
            m[i] = PEEL ? __builtin_inff() : 0.0f;
            contig = false;
        }
        if (s[i] != s[0] + i) contig = false;
    }

    float mq = 0.0f;
    if constexpr (PEEL) mq = scalars[2];
    const size_t orow_bytes = (BITS == 8) ? (size_t)Kpad : (size_t)(Kpad >> 1);
    uint8_t* o = out + (size_t)r0 * orow_bytes + ((BITS == 8) ? p0 : (p0 >> 1));
    const T* row = X + (size_t)r0 * ld;

#pragma unroll 4
    for (int r = r0; r < r1; ++r, row += ld, o += orow_bytes) {
        float x[16];
        if (contig) {
            const v4u* vp = reinterpret_cast<const v4u*>(row + s[0]);
#pragma unroll
            for (int i = 0; i < 16 / VEC; ++i) {
                v4u raw = vp[i];
                widen16<DT>(raw, x + i * VEC);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = Elem<DT>::widen(row[s[i]]);
        }
        int q[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if constexpr (PEEL) {
                const float mag = fminf(fmaxf(fabsf(x[i]) - m[i], 0.0f), thr);
                q[i] = quant1<BITS>(x[i] < 0.0f ? -mag : mag, mq);
            } else {
                q[i] = quant1<BITS>(x[i], m[i]);
            }
        }
        if (BITS == 8) {
            v4u w;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                w[i] = (uint32_t)(q[4 * i] & 0xff) | ((uint32_t)(q[4 * i + 1] & 0xff) << 8) |
                       ((uint32_t)(q[4 * i + 2] & 0xff) << 16) | ((uint32_t)(q[4 * i + 3] & 0xff) << 24);
            *reinterpret_cast<v4u*>(o) = w;
        } else {
            v2u w;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                uint32_t acc = 0;
#pragma unroll
                for (int j = 0; j < 8; ++j) acc |= (uint32_t)(q[8 * i + j] & 0xf) << (4 * j);
                w[i] = acc;
            }
            *reinterpret_cast<v2u*>(o) = w;
        }
    }
}


// ---------------------------------------------------------------------------------------------
// flatten + quantize, row-strip form (the equal split)
// ---------------------------------------------------------------------------------------------
// A workgroup owns a strip of R rows.  Phase 1: each thread takes groups among the first K/16 (the
// head of the map): a group whose 16 slots are the 16 channels at the same indices (gflag) is read
// with vector loads, otherwise gathered; multiply, round, clamp, pack, store, and the quantized value
// of every identity slot also goes to LDS as a byte, q[row][channel].  Phase 2: the remaining groups
// (appended copies and padding), one (group, row) item at a time over all threads.  An appended slot
// with the same copy count as its channel's identity slot holds the same quantized value, so a group
// made of such slots and padding (cflag) is copied from LDS; any other group is gathered from global
// memory and quantized with its own multipliers.
template <int DT, int BITS>
__global__ __launch_bounds__(BITS == 6 ? 512 : 256) void flatten_quant_rows_kernel(const void* __restrict__ Xv, int M, int K, int ld,
                                                                 const int32_t* __restrict__ src,
                                                                 const float* __restrict__ mslot,
                                                                 const uint8_t* __restrict__ gflag, int Kpad, int R,
                                                                 uint8_t* __restrict__ out)
{
    typedef typename Elem<DT>::type T;
    constexpr int VEC = Elem<DT>::VEC;
    extern __shared__ __align__(16) uint8_t lds[];
    const T* X = static_cast<const T*>(Xv);
    const int NH = K >> 4;                                     // groups of the head
    const int KQ = NH << 4;
    const int G = Kpad >> 4;
    const int NT = G - NH;                                     // groups of phase 2
    uint8_t* qs = lds;                                         // [R][KQ] int8
    uint16_t* ts = reinterpret_cast<uint16_t*>(lds + (size_t)R * KQ);   // sources of the phase-2 slots
    uint8_t* tf = lds + (size_t)R * KQ + (size_t)NT * 32;               // copy flags of the phase-2 groups
    const uint8_t* cflag = gflag + (G + 1);
    const int r0 = blockIdx.x * R;
    const int nthr = blockDim.x;
    const int nr = min(M - r0, R);
    // bytes of an output row and of one group of 16 slots: 16 (INT8), 8 (INT4 nibbles), 12 (E3M2 codes)
    constexpr int GB = (BITS == 8) ? 16 : (BITS == 4 ? 8 : 12);
    // INT8 / INT4 rows are dense (E3M2 output has its own addressing, see store_e3m2)
    const size_t orow_bytes = (size_t)(Kpad >> 4) * GB;
    auto group_ofs = [&](int g) -> size_t { return (size_t)g * GB; };

    // sources of the phase-2 slots as 16-bit channel numbers (0xffff: the slot holds 0); eight slots per
    // thread and pass, loaded before any is stored, so that the passes do not each wait a round trip
    for (int t = threadIdx.x * 8; t < NT * 16; t += nthr * 8) {
        const v4i a = *reinterpret_cast<const v4i*>(src + KQ + t);
        const v4i b = *reinterpret_cast<const v4i*>(src + KQ + t + 4);
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int j0 = (i < 2) ? a[2 * i] : b[2 * i - 4], j1 = (i < 2) ? a[2 * i + 1] : b[2 * i - 3];
            const uint32_t lo = ((unsigned)j0 < (unsigned)KQ) ? (uint32_t)j0 : 0xffffu;
            const uint32_t hi = ((unsigned)j1 < (unsigned)KQ) ? (uint32_t)j1 : 0xffffu;
            w[i] = lo | (hi << 16);
        }
        *reinterpret_cast<v4u*>(ts + t) = v4u{w[0], w[1], w[2], w[3]};
    }
    for (int t = threadIdx.x; t < NT; t += nthr) tf[t] = cflag[NH + t];

    auto pack_store = [&](const int (&q)[16], uint8_t* o) {
        if (BITS == 8) {
            v4u w;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                w[i] = (uint32_t)(q[4 * i] & 0xff) | ((uint32_t)(q[4 * i + 1] & 0xff) << 8) |
                       ((uint32_t)(q[4 * i + 2] & 0xff) << 16) | ((uint32_t)(q[4 * i + 3] & 0xff) << 24);
            *reinterpret_cast<v4u*>(o) = w;
        } else if (BITS == 6) {
            (void)o;                                // E3M2 output goes through store_e3m2
        } else {
            v2u w;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                uint32_t acc = 0;
#pragma unroll
                for (int j = 0; j < 8; ++j) acc |= (uint32_t)(q[8 * i + j] & 0xf) << (4 * j);
                w[i] = acc;
            }
            *reinterpret_cast<v2u*>(o) = w;
        }
    };
    // E3M2 output, blocked along k: block t (codes 128 t .. 128 t + 127) holds 96 bytes of every row in turn.
    // A row's 96 bytes are two 48-byte groups of 64 codes; the 24-byte bit stream of each 32-code unit a is
    // split into its first 16 bytes X_a and last 8 bytes Y_a, and the group is stored X_a Y_a Y_b X_b with
    // (a, b) = (0, 1) in rows whose index has bit 4 clear and (1, 0) in the others (what the GEMM's LDS reads
    // want).  A thread's 16 codes are half a unit: stream bytes 0..11 (e = 0) or 12..23 (e = 1).
    auto store_e3m2 = [&](const int (&q)[16], int row, int g) {
        const u3 v = pack16_e3m2(q);
        const int gi = g & 7, e = gi & 1;
        uint8_t* grp = out + ((size_t)(g >> 3) * (size_t)M + (size_t)row) * 96 + 48 * (gi >> 2);
        const bool mirrored = (((gi >> 1) ^ (row >> 4)) & 1) != 0;
        if (!mirrored) {
            *reinterpret_cast<u3*>(grp + 12 * e) = v;                 // X at 0, Y at 16: the plain stream
        } else if (e == 0) {
            *reinterpret_cast<u3*>(grp + 32) = v;                     // X at 32
        } else {
            *reinterpret_cast<uint32_t*>(grp + 44) = v.a;             // the last 4 bytes of X
            *reinterpret_cast<v2u*>(grp + 24) = v2u{v.b, v.c};        // Y at 24
        }
    };
    // the general form of one group over rows [ra, rb) of the strip: every slot's source element is
    // gathered from global memory; identity slots of the head also leave their value in LDS
    auto gather_group = [&](int g, int ra, int rb, bool to_lds) {
        const int p0 = g << 4;
        int s[16];
        float m[16];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v4i sv = *reinterpret_cast<const v4i*>(src + p0 + 4 * i);
            v4f mv = *reinterpret_cast<const v4f*>(mslot + p0 + 4 * i);
#pragma unroll
            for (int j = 0; j < 4; ++j) { s[4 * i + j] = sv[j]; m[4 * i + j] = mv[j]; }
        }
        bool ident[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            ident[i] = to_lds && s[i] == p0 + i;
            if ((unsigned)s[i] >= (unsigned)K) { s[i] = 0; m[i] = 0.0f; }
        }
        uint8_t* o = out + (size_t)(r0 + ra) * orow_bytes + group_ofs(g);
        const T* row = X + (size_t)(r0 + ra) * ld;
        for (int r = ra; r < rb; ++r, row += ld, o += orow_bytes) {
            int q[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) q[i] = quant1<BITS>(Elem<DT>::widen(row[s[i]]), m[i]);
            if constexpr (BITS == 6) store_e3m2(q, r0 + r, g);
            else pack_store(q, o);
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (ident[i]) qs[(size_t)r * KQ + p0 + i] = (uint8_t)q[i];
        }
    };

    // ---- phase 1: the head ----
    for (int g = threadIdx.x; g < NH; g += nthr) {
        if (!gflag[g]) {
            gather_group(g, 0, nr, true);
            continue;
        }
        const int p0 = g << 4;
        float m[16];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v4f mv = *reinterpret_cast<const v4f*>(mslot + p0 + 4 * i);
#pragma unroll
            for (int j = 0; j < 4; ++j) m[4 * i + j] = mv[j];
        }
        uint8_t* o = out + (size_t)r0 * orow_bytes + group_ofs(g);
        const T* row = X + (size_t)r0 * ld + p0;
        uint8_t* ql = qs + p0;
#pragma unroll 4
        for (int r = 0; r < nr; ++r, row += ld, o += orow_bytes, ql += KQ) {
            float x[16];
            const v4u* vp = reinterpret_cast<const v4u*>(row);
#pragma unroll
            for (int i = 0; i < 16 / VEC; ++i) widen16<DT>(vp[i], x + i * VEC);
            int q[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) q[i] = quant1<BITS>(x[i], m[i]);
            if constexpr (BITS == 6) store_e3m2(q, r0 + r, g);
            else pack_store(q, o);
            v4u w;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                w[i] = (uint32_t)(q[4 * i] & 0xff) | ((uint32_t)(q[4 * i + 1] & 0xff) << 8) |
                       ((uint32_t)(q[4 * i + 2] & 0xff) << 16) | ((uint32_t)(q[4 * i + 3] & 0xff) << 24);
            *reinterpret_cast<v4u*>(ql) = w;
        }
    }
    __syncthreads();

    // ---- phase 2: appended copies and padding, (group, row) items over all threads, two per thread
    //      and pass with the LDS reads of both issued before either is packed ----
    constexpr int U = 2;
    const int items = NT * nr;
    for (int it0 = threadIdx.x; it0 < items; it0 += nthr * U) {
        int gt[U], rr[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int it = it0 + u * nthr;
            const bool valid = it < items;
            gt[u] = valid ? it % NT : 0;
            rr[u] = valid ? it / NT : 0;
            const uint8_t cf = valid ? tf[gt[u]] : (uint8_t)1;
            ok[u] = valid && cf != 0;
            if (valid && cf == 0) gather_group(NH + gt[u], rr[u], rr[u] + 1, false);
        }
        v4u t0[U], t1[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const v4u* tp = reinterpret_cast<const v4u*>(ts + gt[u] * 16);
            t0[u] = tp[0];
            t1[u] = tp[1];
        }
        int q[U][16];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int8_t* ql = reinterpret_cast<const int8_t*>(qs) + (size_t)rr[u] * KQ;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const uint32_t word = (i < 8) ? t0[u][i >> 1] : t1[u][(i - 8) >> 1];
                const uint32_t j = (i & 1) ? (word >> 16) : (word & 0xffffu);
                q[u][i] = (j == 0xffffu) ? 0 : (int)ql[j];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (ok[u]) {
                const int g = NH + gt[u];
                if constexpr (BITS == 6) store_e3m2(q[u], r0 + rr[u], g);
                else pack_store(q[u], out + (size_t)(r0 + rr[u]) * orow_bytes + group_ofs(g));
            }
    }
}

// Per input channel max|x| into cmax (fp32 bit patterns, which order like the non-negative floats
// they hold); accumulate keeps what cmax holds on entry as the starting value.
template <int DT>
void launch_colabsmax(const void* X, int M, int K, int ld, bool accumulate, uint32_t* cmax, hipStream_t stream)
{
    constexpr int VEC = Elem<DT>::VEC;
    if (!accumulate) fill_u32_kernel<<<(K + 255) / 256, 256, 0, stream>>>(cmax, K, 0u);
    const int bx = (K + 64 * VEC - 1) / (64 * VEC);
    // A workgroup takes a multiple of 64 rows (16 loads in flight for each of its 4 waves).  Measured:
    // long strips (a few hundred workgroups in all, each wave streaming 100+ rows) beat many short ones,
    // and the strip height must not be a power of two: with power-of-two row strides (K = 4096 bf16)
    // workgroups that start a power-of-two number of rows apart hit the same memory channels
    // (3.1 TB/s at 128 or 512 rows, 4.6 TB/s at 448).  So: an odd multiple of 64, 448..704 rows,
    // fewer when the matrix is too small to give about 64 workgroups.
    long long rpb = ((long long)M * bx + 399) / 400;
    rpb = (rpb + 63) / 64 * 64;
    if (rpb < 448) rpb = 448;
    if (rpb > 704) rpb = 704;
    long long cap = ((long long)M * bx / 64 + 63) / 64 * 64;
    if (cap < 64) cap = 64;
    if (rpb > cap) rpb = cap;
    if ((rpb / 64) % 2 == 0) rpb += 64;
    dim3 grid(bx, (unsigned)((M + rpb - 1) / rpb));
    colabsmax_kernel<DT><<<grid, 256, 0, stream>>>(X, M, K, ld, (int)rpb, cmax);
}

template <int DT>
int launch_for_dtype(const void* X, int M, int K, int ld, const int32_t* src_idx, const int32_t* rep,
                     int Kpad, int bits, int mode, const float* absmax_in, float T, void* out, float* scale_out,
                     const ActWorkspace& ws, hipStream_t stream)
{
    const int qmax = (bits == 6) ? 7 : (1 << (bits - 1)) - 1;       // 6: the 4-bit quantizer, E3M2 storage
    const bool peel = mode >= 3;
    if (bits == 6) {
        // E3M2 storage exists in the row-strip kernel only: refuse before anything is enqueued
        const size_t kq1 = (size_t)(K & ~15), tail1 = 2 * ((size_t)Kpad - kq1) + ((size_t)Kpad - kq1) / 16;
        if (peel || K < 16 || kq1 + tail1 > 64u * 1024u)
            return fail(FQ_ERR_DTYPE, "E3M2 storage (bits = 6) needs K >= 16 and a layer narrow enough for the "
                                      "row-strip kernel, and is not available for the peel split");
        // very wide layers launch this kernel with up to 128 KiB of LDS: raise its limit once per device
        static std::atomic<unsigned long long> raised{0};
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return fail(FQ_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
        const unsigned long long bit = 1ull << (dev & 63);
        if (!(raised.load(std::memory_order_acquire) & bit)) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(flatten_quant_rows_kernel<DT, 6>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
            if (e != hipSuccess) return fail(FQ_ERR_HIP, "hipFuncSetAttribute(128 KiB LDS): %s", hipGetErrorString(e));
            raised.fetch_or(bit, std::memory_order_release);
        }
    }
    if (mode != 1 && mode != 4) launch_colabsmax<DT>(X, M, K, ld, /*accumulate=*/false, ws.cmax, stream);
    scale_kernel<<<(Kpad + 1023) / 1024, 1024, 0, stream>>>(ws.cmax, K, src_idx, rep, Kpad, qmax, mode, absmax_in, T,
                                                            ws.mslot, scale_out, ws.scalars, ws.gflag);
    if (!out) {
        // scales only: the caller quantizes elsewhere (the GEMM that converts its A operand on the way into LDS)
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(FQ_ERR_HIP, "activation scale launch failed: %s", hipGetErrorString(e));
        return FQ_OK;
    }
    uint8_t* o8 = static_cast<uint8_t*>(out);
    if (!peel && K >= 16) {
        // row-strip kernel: R rows per workgroup with R * K bytes of LDS plus 2 bytes per appended slot
        // (at most 64 KiB, so that two workgroups fit a CU); wider layers use the general kernel below
        // per appended slot 2 bytes (its source) and per appended group 1 byte (its flag)
        const size_t kq = (size_t)(K & ~15), tail_src = 2 * ((size_t)Kpad - kq) + ((size_t)Kpad - kq) / 16;
        int R = 8;
        while (R > 1 && (size_t)R * kq + tail_src > 64u * 1024u) R >>= 1;
        const size_t lds = (size_t)R * kq + tail_src;
        if (lds <= 64u * 1024u) {
            const unsigned nblk = (unsigned)((M + R - 1) / R);
            // 256 threads walk the strip's groups (larger workgroups, one thread per head group, measured slower)
            const int nthr = 256;
            if (bits == 8)
                flatten_quant_rows_kernel<DT, 8><<<nblk, nthr, lds, stream>>>(X, M, K, ld, src_idx, ws.mslot, ws.gflag, Kpad, R, o8);
            else if (bits == 6) {
                // Very wide layers (strips cut to two rows or one): the blocked E3M2 layout then gets runs of only
                // 192 or 96 bytes per block.  A strip twice as high in a 512-thread workgroup with up to 128 KiB of
                // LDS (one workgroup per CU) measured 11 % faster at K = 22016; at K = 11008 (four rows -> eight)
                // the same change was 16 % slower, so it stops there.
                int R6 = R;
                size_t lds6 = lds;
                int nthr6 = nthr;
                if (R <= 2 && (size_t)(2 * R) * kq + tail_src <= 128u * 1024u) {
                    R6 = 2 * R;
                    lds6 = (size_t)R6 * kq + tail_src;
                    nthr6 = 512;
                    // (the kernel's LDS limit was raised above, before anything of this call was enqueued)
                }
                flatten_quant_rows_kernel<DT, 6><<<(unsigned)((M + R6 - 1) / R6), nthr6, lds6, stream>>>(X, M, K, ld, src_idx, ws.mslot, ws.gflag, Kpad, R6, o8);
            }
            else
                flatten_quant_rows_kernel<DT, 4><<<nblk, nthr, lds, stream>>>(X, M, K, ld, src_idx, ws.mslot, ws.gflag, Kpad, R, o8);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return fail(FQ_ERR_HIP, "flatten-quantize launch failed: %s", hipGetErrorString(e));
            return FQ_OK;
        }
    }
    const int G = Kpad / 16;
    // rows per thread: as many as 8 while the launch still has >= 2048 waves
    int rpt = 8;
    while (rpt > 1 && ((long long)G * ((M + rpt - 1) / rpt)) < 2048LL * 64) rpt >>= 1;
    const long long threads = (long long)G * ((M + rpt - 1) / rpt);
    const unsigned blocks = (unsigned)((threads + 255) / 256);
    if (peel && bits == 8)
        flatten_quant_kernel<DT, 8, true><<<blocks, 256, 0, stream>>>(X, M, K, ld, src_idx, ws.mslot, Kpad, rpt, o8, ws.scalars, T);
    else if (peel)
        flatten_quant_kernel<DT, 4, true><<<blocks, 256, 0, stream>>>(X, M, K, ld, src_idx, ws.mslot, Kpad, rpt, o8, ws.scalars, T);
    else if (bits == 8)
        flatten_quant_kernel<DT, 8><<<blocks, 256, 0, stream>>>(X, M, K, ld, src_idx, ws.mslot, Kpad, rpt, o8);
    else
        flatten_quant_kernel<DT, 4><<<blocks, 256, 0, stream>>>(X, M, K, ld, src_idx, ws.mslot, Kpad, rpt, o8);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FQ_ERR_HIP, "flatten-quantize launch failed: %s", hipGetErrorString(e));
    return FQ_OK;
}

}  // namespace

ActWorkspace carve_act_workspace(void* base, int K, int Kpad)
{
    ActWorkspace ws;
    uint8_t* p = static_cast<uint8_t*>(base);
    size_t off = 0;
    ws.cmax = reinterpret_cast<uint32_t*>(p + off);
    off += round_up((size_t)K * 4, 256);
    ws.mslot = reinterpret_cast<float*>(p + off);
    off += round_up((size_t)Kpad * 4, 256);
    ws.scalars = reinterpret_cast<float*>(p + off);
    off += 256;
    ws.gflag = p + off;
    off += round_up(2 * (size_t)(Kpad / 16 + 1), 256);       // gflag, then cflag
    ws.bytes = off;
    return ws;
}

int launch_flatten_quant(const void* X, int x_dtype, int M, int K, int ld, const int32_t* src_idx,
                         const int32_t* rep, int Kpad, int bits, int mode, const float* absmax_in,
                         void* out, float* scale_out, const ActWorkspace& ws, hipStream_t stream, float T)
{
    switch (x_dtype) {
    case FQ_F32:
        return launch_for_dtype<FQ_F32>(X, M, K, ld, src_idx, rep, Kpad, bits, mode, absmax_in, T, out, scale_out, ws, stream);
    case FQ_F16:
        return launch_for_dtype<FQ_F16>(X, M, K, ld, src_idx, rep, Kpad, bits, mode, absmax_in, T, out, scale_out, ws, stream);
    case FQ_BF16:
        return launch_for_dtype<FQ_BF16>(X, M, K, ld, src_idx, rep, Kpad, bits, mode, absmax_in, T, out, scale_out, ws, stream);
    default:
        return fail(FQ_ERR_DTYPE, "unsupported input dtype %d", x_dtype);
    }
}

int launch_channel_absmax(const void* X, int x_dtype, int M, int K, int ld, int accumulate, float* chmax,
                          hipStream_t stream)
{
    uint32_t* cmax = reinterpret_cast<uint32_t*>(chmax);
    switch (x_dtype) {
    case FQ_F32: launch_colabsmax<FQ_F32>(X, M, K, ld, accumulate != 0, cmax, stream); break;
    case FQ_F16: launch_colabsmax<FQ_F16>(X, M, K, ld, accumulate != 0, cmax, stream); break;
    case FQ_BF16: launch_colabsmax<FQ_BF16>(X, M, K, ld, accumulate != 0, cmax, stream); break;
    default: return fail(FQ_ERR_DTYPE, "unsupported input dtype %d", x_dtype);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FQ_ERR_HIP, "channel absmax launch failed: %s", hipGetErrorString(e));
    return FQ_OK;
}

}  // namespace fq
