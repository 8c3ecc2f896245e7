// Shared device helpers of the draft-verification kernels (gfx950, wave64).
//
// Everything is in base 2: with k = log2(e) / T and y(x) = logit(x) * k the softmax is
// p(x) = exp2(y(x) - L), L = log2 sum_x exp2(y(x)).  All reductions have a fixed order, so
// results are bit-reproducible from run to run.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>

namespace sv {

constexpr int kThreads = 256;             // threads per workgroup: 4 wavefronts of 64
constexpr int kWaves = kThreads / 64;
// log2 of the ratio r_i never goes below this: a drafted token whose target logit is -inf (masked out by
// top-k / top-p warping) has r_i = 0, and exp2 of this is exactly 0 in double while sums of it stay finite
constexpr double kLog2RatioFloor = -1.0e6;
constexpr int kChunk = 8192;              // logits of one row handled by one workgroup
constexpr int kWaveChunk = kChunk / kWaves;   // contiguous logits of one row handled by one wavefront
constexpr int kPerThread = kChunk / kThreads; // logits of one row held by one thread

enum Algo : int { kBlock = 0, kToken = 1, kGreedy = 2 };

struct bf16_t { uint16_t bits; };

template <typename T> struct ElemTraits;
template <> struct ElemTraits<float>  { static constexpr int kVec = 4; };   // logits per 16 bytes
template <> struct ElemTraits<bf16_t> { static constexpr int kVec = 8; };

// Row-level constants of one (sequence, position) for evaluating residual weights:
// w_i p_i(x) = cq * c * exp2(y_p(x) - sh_p) and q_i(x) = cq * exp2(y_q(x) - sh_q).  The float
// shifts take the large part of the exponent exactly; c and cq carry what rounding the shifts
// to float left over, so no systematic error of size ulp(shift) enters the weights.
struct RowCoef {
    float sh_p;      // float(L_p - log2 w)
    float sh_q;      // float(L_q)
    float c;         // exp2(sh_p - (L_p - log2 w)) / exp2(sh_q - L_q)
    float cq;        // exp2(sh_q - L_q)
};

__host__ __device__ inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ RowCoef make_row_coef(double alpha_p, double alpha_q)
{
    RowCoef rc;
    rc.sh_p = (float)alpha_p;
    rc.sh_q = (float)alpha_q;
    const double cp = exp2((double)rc.sh_p - alpha_p), cq = exp2((double)rc.sh_q - alpha_q);
    rc.c = (float)(cp / cq);
    rc.cq = (float)cq;
    return rc;
}

// w p - q for one token, in units of cq.
__device__ __forceinline__ float residual_term(float xp, float xq, float k, const RowCoef &rc)
{
    const float ep = fast_exp2(__builtin_fmaf(xp, k, -rc.sh_p));
    const float eq = fast_exp2(__builtin_fmaf(xq, k, -rc.sh_q));
    return __builtin_fmaf(ep, rc.c, -eq);
}

__device__ __forceinline__ float bf16_lo(uint32_t word) { return __uint_as_float(word << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t word) { return __uint_as_float(word & 0xffff0000u); }

template <typename T>
__device__ __forceinline__ float logit_as_float(const T *p)
{
    if constexpr (ElemTraits<T>::kVec == 4) return *reinterpret_cast<const float *>(p);
    else return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t *>(p)[0] << 16);
}
// The same in two steps, for a caller that must not wait for the load where it asks: the logit's bits as loaded ...
template <typename T>
__device__ __forceinline__ uint32_t logit_bits(const T *p)
{
    if constexpr (ElemTraits<T>::kVec == 4) return *reinterpret_cast<const uint32_t *>(p);
    else return (uint32_t)reinterpret_cast<const uint16_t *>(p)[0];
}
// ... and the float they stand for
template <typename T>
__device__ __forceinline__ float logit_bits_as_float(uint32_t bits)
{
    if constexpr (ElemTraits<T>::kVec == 4) return __uint_as_float(bits);
    else return __uint_as_float(bits << 16);
}
template <typename T>
__device__ __forceinline__ double logit_as_double(const T *p) { return (double)logit_as_float(p); }

// Sixteen bytes of a row that is read once: a non-temporal load, which leaves the caches to what is used again (the words
// that cross workgroups, the kernel's arguments): 55.9 -> 54.5 us at B = 64, gamma = 8, V = 128256.
__device__ __forceinline__ uint4 load_streamed(const void *p)
{
    typedef unsigned v4u __attribute__((ext_vector_type(4)));
    const v4u t = __builtin_nontemporal_load(static_cast<const v4u *>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}

// kVec consecutive logits starting at element `idx` of a row of V logits, as floats.
// Elements at or beyond V come back as -inf (weight zero everywhere downstream).  The aligned
// form needs idx % kVec == 0, V % kVec == 0 and a 16-byte aligned row.
template <typename T, bool ALIGNED>
__device__ __forceinline__ void load_vec(const T *row, int V, int idx, float *out)
{
    constexpr int kVec = ElemTraits<T>::kVec;
    if constexpr (ALIGNED) {
        if (idx < V) {
            const uint4 v = load_streamed(row + idx);
            if constexpr (kVec == 4) {
                out[0] = __uint_as_float(v.x); out[1] = __uint_as_float(v.y);
                out[2] = __uint_as_float(v.z); out[3] = __uint_as_float(v.w);
            } else {
                out[0] = bf16_lo(v.x); out[1] = bf16_hi(v.x);
                out[2] = bf16_lo(v.y); out[3] = bf16_hi(v.y);
                out[4] = bf16_lo(v.z); out[5] = bf16_hi(v.z);
                out[6] = bf16_lo(v.w); out[7] = bf16_hi(v.w);
            }
        } else {
#pragma unroll
            for (int e = 0; e < kVec; ++e) out[e] = -INFINITY;
        }
    } else {
#pragma unroll
        for (int e = 0; e < kVec; ++e) {
            float val = -INFINITY;
            if (idx + e < V) {
                if constexpr (kVec == 4) val = reinterpret_cast<const float *>(row)[idx + e];
                else val = __uint_as_float((uint32_t)reinterpret_cast<const uint16_t *>(row)[idx + e] << 16);
            }
            out[e] = val;
        }
    }
}

// ------------------------------------------------------------------ wavefront reductions
// All cross-lane moves go through DPP (no LDS crossbar): four steps inside each row of 16 lanes,
// two row broadcasts that leave the result in lane 63, one readlane.  Every lane gets the same
// value; the order of the operations is fixed.  Each step is ONE instruction, v = op(dpp(v), v)
// in place: lanes that a broadcast step does not address keep their value.  The compiler does not
// form these from the DPP builtin for max nor for the broadcast steps, hence the assembly; the
// s_nop before each step covers the two wait states a DPP read needs after a VALU write.
#define SV_DPP_REDUCE(OP)                                                                       \
    "s_nop 1\n\t" OP " %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"          \
    "s_nop 1\n\t" OP " %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"          \
    "s_nop 1\n\t" OP " %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"              \
    "s_nop 1\n\t" OP " %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"                   \
    "s_nop 1\n\t" OP " %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"                 \
    "s_nop 1\n\t" OP " %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"                 \
    "s_nop 1"

__device__ __forceinline__ float wave_sum(float v)
{
    asm volatile(SV_DPP_REDUCE("v_add_f32_dpp") : "+v"(v));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__device__ __forceinline__ float wave_max(float v)
{
    asm volatile(SV_DPP_REDUCE("v_max_f32_dpp") : "+v"(v));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// The same over each half of the wave (lanes 0..31 and 32..63) at once: five steps; lane 31 ends up with
// the first half's result, lane 63 with the second half's.
#define SV_DPP_REDUCE_HALVES(OP)                                                                \
    "s_nop 1\n\t" OP " %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"          \
    "s_nop 1\n\t" OP " %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"          \
    "s_nop 1\n\t" OP " %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"              \
    "s_nop 1\n\t" OP " %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"                   \
    "s_nop 1\n\t" OP " %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"                 \
    "s_nop 1"
__device__ __forceinline__ void halves_sum(float v, float &first, float &second)
{
    asm volatile(SV_DPP_REDUCE_HALVES("v_add_f32_dpp") : "+v"(v));
    first = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 31));
    second = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ void halves_max(float v, float &first, float &second)
{
    asm volatile(SV_DPP_REDUCE_HALVES("v_max_f32_dpp") : "+v"(v));
    first = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 31));
    second = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
#undef SV_DPP_REDUCE_HALVES
#undef SV_DPP_REDUCE

__device__ __forceinline__ double wave_sum_double(double v)
{
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// ------------------------------------------------------------------ workgroup reductions
// `lds` must hold kWaves values.  Every thread gets the result.
__device__ __forceinline__ float block_sum(float v, float *lds)
{
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = lds[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) t += lds[w];
    return t;
}

__device__ __forceinline__ float block_max(float v, float *lds)
{
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = lds[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) t = fmaxf(t, lds[w]);
    return t;
}

__device__ __forceinline__ double block_sum_double(double v, double *lds)
{
    v = wave_sum_double(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = lds[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) t += lds[w];
    return t;
}

// Inclusive scan over the workgroup in thread order.  `exclusive` is bit-identical to the
// inclusive value of the previous thread (0 for thread 0); `total` is the sum of all threads.
__device__ __forceinline__ float block_inclusive_scan(float v, float *lds, float &exclusive, float &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const float up = __shfl_up(v, off, 64);
        if (lane >= off) v += up;
    }
    const float prev = __shfl_up(v, 1, 64);
    __syncthreads();
    if (lane == 63) lds[wave] = v;
    __syncthreads();
    float base = 0.f, tot = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        if (w < wave) base += lds[w];
        tot += lds[w];
    }
    total = tot;
    exclusive = lane ? prev + base : base;
    return v + base;
}

// ------------------------------------------------------------------ inverse-CDF walk
// The workgroup walks `nsub` consecutive sub-ranges of kThreads * 8 logits of one row pair,
// starting at element `start`, in vocabulary order, and returns (to every thread) the first
// token whose running weight exceeds t.  Weights: residual (`residual` true): max(w p - q, 0)
// in units of rc.cq; otherwise exp2(y_p - shift) * scale.  If rounding leaves t beyond the
// range's total, the last token of positive weight in the range is returned (0 if none).
// `lds` holds kWaves floats, `ints` two ints.
template <typename T, bool ALIGNED>
__device__ int walk_range(const T *prow, const T *qrow, int V, int start, int nsub, float k,
                          bool residual, const RowCoef &rc, float shift, float scale, float t,
                          float *lds, int *ints)
{
    constexpr int kVec = ElemTraits<T>::kVec;
    constexpr int kPer = 8;                           // logits per thread and sub-range
    const int tid = threadIdx.x;
    int last_positive = -1;
    int result = -1;
    for (int sub = 0; sub < nsub; ++sub) {
        const int idx = start + (sub * kThreads + tid) * kPer;
        float wgt[kPer];
        {
            float xp[kPer], xq[kPer];
#pragma unroll
            for (int v = 0; v < kPer / kVec; ++v) load_vec<T, ALIGNED>(prow, V, idx + v * kVec, xp + v * kVec);
            if (residual) {
#pragma unroll
                for (int v = 0; v < kPer / kVec; ++v) load_vec<T, ALIGNED>(qrow, V, idx + v * kVec, xq + v * kVec);
#pragma unroll
                for (int e = 0; e < kPer; ++e) wgt[e] = fmaxf(residual_term(xp[e], xq[e], k, rc), 0.f);
            } else {
#pragma unroll
                for (int e = 0; e < kPer; ++e) wgt[e] = fast_exp2(__builtin_fmaf(xp[e], k, -shift)) * scale;
            }
        }
        float mine = 0.f;
#pragma unroll
        for (int e = 0; e < kPer; ++e) {
            mine += wgt[e];
            if (wgt[e] > 0.f) last_positive = idx + e;
        }
        float exc, total;
        const float inc = block_inclusive_scan(mine, lds, exc, total);
        // the first thread whose running sum exceeds t: per wave by a ballot, then the first wave that has one
        // (one atomic operation per thread on one LDS word took microseconds here); `lds` is free after the scan
        const unsigned long long hits = __ballot(inc > t);
        int *wave_first = reinterpret_cast<int *>(lds);
        __syncthreads();
        if ((tid & 63) == 0) wave_first[tid >> 6] = hits ? (tid | (__ffsll((long long)hits) - 1)) : kThreads;
        __syncthreads();
        int first = kThreads;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) first = wave_first[w] < first ? wave_first[w] : first;
        __syncthreads();
        if (first < kThreads) {
            if (tid == first) {
                float run = exc;
                int y = -1, lastpos = 0;
#pragma unroll
                for (int e = 0; e < kPer; ++e) {
                    run += wgt[e];
                    if (wgt[e] > 0.f) lastpos = e;
                    if (y < 0 && run > t) y = e;
                }
                if (y < 0) y = lastpos;   // scan and walk rounded differently: last positive weight
                ints[1] = idx + y;
            }
            __syncthreads();
            result = ints[1];
            break;
        }
        t -= total;
        __syncthreads();
    }
    if (result < 0) {
        if (tid == 0) ints[1] = -1;
        __syncthreads();
        atomicMax(&ints[1], last_positive);
        __syncthreads();
        result = ints[1] < 0 ? 0 : ints[1];
    }
    __syncthreads();
    return result;
}

}  // namespace sv
