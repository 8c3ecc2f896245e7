// Draft verification for speculative decoding on gfx950: kernels and the C ABI.
//
// Path of one call (Alg. 1 / Alg. 2 / Alg. 4 of the block-verification paper):
//   1. row_stats_kernel     every logit row, cut into chunks of CHUNK elements: the chunk's
//                           maximum and sum of exp2((a - max) * k), k = log2(e) / T
//   2. prefix_weights_kernel per sequence: row log-normalisers, the ratios of the drafted
//                           tokens, the recursion w_i = min(w_{i-1} r_i, 1) (in double, in the
//                           log domain), and the per-row constants of step 3
//   3. residual_kernel      every (target row i, draft row i) pair: chunk partial sums of
//                           max(w_i p_i(x) - q_i(x), 0)
//   4. finalize_kernel      per sequence: S_i, h_i, tau, then the inverse-CDF draw of Y
//                           (pick the chunk from the partial sums, re-read that one chunk)
//
// Everything is in base 2: with y(x) = a(x) * k the softmax is p(x) = exp2(y(x) - L),
// L = log2 sum_x exp2(y(x)).  All reductions have a fixed order, so results are
// bit-reproducible from run to run.

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>

#include "../../include/specverify.h"

namespace {

constexpr int kThreads = 256;            // threads per workgroup (4 wavefronts of 64)
constexpr int kWaves = kThreads / 64;
constexpr int kChunk = 8192;             // logits of one row handled by one workgroup

enum Algo : int { kBlock = 0, kToken = 1, kGreedy = 2 };

struct bf16_t { uint16_t bits; };

template <typename T> struct ElemTraits;
template <> struct ElemTraits<float>  { static constexpr int kVec = 4; };
template <> struct ElemTraits<bf16_t> { static constexpr int kVec = 8; };

// Per (sequence, position) constants produced by step 2 and consumed by steps 3 and 4.
// w_i p_i(x) = cq * c * exp2(y_p(x) - sh_p) and q_i(x) = cq * exp2(y_q(x) - sh_q): the float
// shifts sh_* absorb the large part of the exponent exactly, c and cq carry what the
// rounding of the shifts left over.
struct RowCoef {
    float sh_p;      // float(L_p,i - log2 w_i)
    float sh_q;      // float(L_q,i)
    float c;         // exp2(sh_p - (L_p,i - log2 w_i)) / exp2(sh_q - L_q,i)
    float cq;        // exp2(sh_q - L_q,i)
    double w;        // w_i
    double one_minus_w;
    double log2r;    // log2 r_i (ratio of draft token i, judged with rows i-1); 0 at i = 0
    float row_max;   // M_i: maximum over the target row's chunks of (chunk max * k)
    float pad;
};

__host__ __device__ inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float bf16_lo(uint32_t word) { return __uint_as_float(word << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t word) { return __uint_as_float(word & 0xffff0000u); }

// kVec consecutive logits starting at element `idx` of a row of V logits, as floats.
// Elements at or beyond V come back as -inf (weight zero everywhere downstream).
template <typename T, bool ALIGNED>
__device__ __forceinline__ void load_vec(const T *row, int V, int idx, float (&out)[ElemTraits<T>::kVec])
{
    constexpr int kVec = ElemTraits<T>::kVec;
    if constexpr (ALIGNED) {
        if (idx < V) {
            const uint4 v = *reinterpret_cast<const uint4 *>(row + idx);
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

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// Workgroup reductions with a fixed combination order; every thread gets the result.
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

// ---------------------------------------------------------------------------- step 1
template <typename T, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void row_stats_kernel(
    const T *__restrict__ target, const T *__restrict__ draft,
    int B, int gamma, int V, float k, int nchunks, float2 *__restrict__ stats)
{
    constexpr int kVec = ElemTraits<T>::kVec;
    constexpr int kU = kChunk / (kThreads * kVec);
    __shared__ float lds[kWaves];
    const int r = blockIdx.x / nchunks, c = blockIdx.x - r * nchunks, tid = threadIdx.x;
    const int n_target_rows = B * (gamma + 1);
    const T *row = r < n_target_rows ? target + (size_t)r * V : draft + (size_t)(r - n_target_rows) * V;

    float x[kU][kVec];
#pragma unroll
    for (int u = 0; u < kU; ++u) load_vec<T, ALIGNED>(row, V, c * kChunk + (u * kThreads + tid) * kVec, x[u]);

    float m = -INFINITY;
#pragma unroll
    for (int u = 0; u < kU; ++u)
#pragma unroll
        for (int e = 0; e < kVec; ++e) m = fmaxf(m, x[u][e]);
    m = block_max(m, lds);
    const float mk = m * k;

    float s = 0.f;
#pragma unroll
    for (int u = 0; u < kU; ++u)
#pragma unroll
        for (int e = 0; e < kVec; ++e) s += fast_exp2(__builtin_fmaf(x[u][e], k, -mk));
    s = block_sum(s, lds);
    if (tid == 0) stats[(size_t)r * nchunks + c] = make_float2(mk, s);
}

// ---------------------------------------------------------------------------- step 2
template <typename T>
__device__ __forceinline__ double logit_as_double(const T *p)
{
    if constexpr (ElemTraits<T>::kVec == 4) return (double)*reinterpret_cast<const float *>(p);
    else return (double)__uint_as_float((uint32_t)reinterpret_cast<const uint16_t *>(p)[0] << 16);
}

template <typename T>
__global__ __launch_bounds__(64) void prefix_weights_kernel(
    const T *__restrict__ target, const T *__restrict__ draft, const int32_t *__restrict__ tokens,
    int gamma, int V, float k, int nchunks, int n_target_rows, int algo,
    const float2 *__restrict__ stats, RowCoef *__restrict__ coef)
{
    extern __shared__ double sm[];          // [2*(gamma+1)] log2-normalisers, then row maxima
    double *L_p = sm, *L_q = sm + (gamma + 1);
    float *M_p = reinterpret_cast<float *>(sm + 2 * (gamma + 1));
    const int b = blockIdx.x, tid = threadIdx.x;

    // log2-normaliser of every row of this sequence: L = M + log2 sum_c s_c exp2(mk_c - M)
    for (int j = tid; j < 2 * gamma + 1; j += 64) {
        const bool is_target = j <= gamma;
        const int i = is_target ? j : j - (gamma + 1);
        const size_t r = is_target ? (size_t)b * (gamma + 1) + i : (size_t)n_target_rows + (size_t)b * gamma + i;
        const float2 *st = stats + r * nchunks;
        float M = -INFINITY;
        for (int c = 0; c < nchunks; ++c) M = fmaxf(M, st[c].x);
        double z = 0.0;
        for (int c = 0; c < nchunks; ++c) z += (double)st[c].y * exp2((double)(st[c].x - M));
        const double L = (double)M + log2(z);
        if (is_target) { L_p[i] = L; M_p[i] = M; } else L_q[i] = L;
    }
    __syncthreads();
    if (tid != 0) return;

    // Alg. 2, the recursion for w_i (its p_i), carried as log2 w_i so that products of
    // ratios neither overflow nor lose 1 - w_i when w_i is close to 1.
    const double kd = (double)k;
    double log2w = 0.0, log2r = 0.0;
    for (int i = 0; i <= gamma; ++i) {
        RowCoef rc;
        const double lw = (algo == kToken) ? 0.0 : log2w;     // token verification: residual is p - q
        const double alpha_p = L_p[i] - lw;
        const double alpha_q = i < gamma ? L_q[i] : 0.0;
        rc.sh_p = (float)alpha_p;
        rc.sh_q = (float)alpha_q;
        const double cp = exp2((double)rc.sh_p - alpha_p), cq = exp2((double)rc.sh_q - alpha_q);
        rc.c = (float)(cp / cq);
        rc.cq = (float)cq;
        rc.w = exp2(lw);
        rc.one_minus_w = -expm1(lw * 0.69314718055994530942);
        rc.log2r = log2r;
        rc.row_max = M_p[i];
        rc.pad = 0.f;
        coef[(size_t)b * (gamma + 1) + i] = rc;
        if (i < gamma) {
            // r_{i+1} = p_i(X_{i+1}) / q_i(X_{i+1}) from the two gathered logits
            const int tok = tokens[(size_t)b * gamma + i];
            const double ya = logit_as_double(target + ((size_t)b * (gamma + 1) + i) * V + tok) * kd;
            const double yb = logit_as_double(draft + ((size_t)b * gamma + i) * V + tok) * kd;
            log2r = (ya - L_p[i]) - (yb - L_q[i]);
            log2w += log2r;
            if (algo != kGreedy && log2w > 0.0) log2w = 0.0;  // the min{., 1}; greedy block verification omits it
        }
    }
}

// ---------------------------------------------------------------------------- step 3
// One residual weight: max(w p - q, 0) in units of cq; `neg` receives max(q - w p, 0).
__device__ __forceinline__ float residual_term(float xp, float xq, float k, const RowCoef &rc)
{
    const float ep = fast_exp2(__builtin_fmaf(xp, k, -rc.sh_p));
    const float eq = fast_exp2(__builtin_fmaf(xq, k, -rc.sh_q));
    return __builtin_fmaf(ep, rc.c, -eq);
}

template <typename T, bool ALIGNED, bool GREEDY>
__global__ __launch_bounds__(kThreads) void residual_kernel(
    const T *__restrict__ target, const T *__restrict__ draft,
    int gamma, int V, float k, int nchunks, const RowCoef *__restrict__ coef,
    float *__restrict__ spart, float *__restrict__ rpart)
{
    constexpr int kVec = ElemTraits<T>::kVec;
    constexpr int kU = kChunk / (kThreads * kVec);
    __shared__ float lds[kWaves];
    const int pr = blockIdx.x / nchunks, c = blockIdx.x - pr * nchunks, tid = threadIdx.x;
    const int b = pr / gamma, i = pr - b * gamma;
    const RowCoef rc = coef[(size_t)b * (gamma + 1) + i];
    const T *prow = target + ((size_t)b * (gamma + 1) + i) * V;
    const T *qrow = draft + ((size_t)b * gamma + i) * V;

    float xp[kU][kVec], xq[kU][kVec];
#pragma unroll
    for (int u = 0; u < kU; ++u) {
        const int idx = c * kChunk + (u * kThreads + tid) * kVec;
        load_vec<T, ALIGNED>(prow, V, idx, xp[u]);
        load_vec<T, ALIGNED>(qrow, V, idx, xq[u]);
    }
    float acc = 0.f, rej = 0.f;
#pragma unroll
    for (int u = 0; u < kU; ++u)
#pragma unroll
        for (int e = 0; e < kVec; ++e) {
            const float d = residual_term(xp[u][e], xq[u][e], k, rc);
            acc += fmaxf(d, 0.f);
            if constexpr (GREEDY) rej += fmaxf(-d, 0.f);
        }
    acc = block_sum(acc, lds);
    if constexpr (GREEDY) rej = block_sum(rej, lds);
    if (tid == 0) {
        spart[(size_t)pr * nchunks + c] = acc;
        if constexpr (GREEDY) rpart[(size_t)pr * nchunks + c] = rej;
    }
}

// ---------------------------------------------------------------------------- step 4
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

template <typename T, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void finalize_kernel(
    const T *__restrict__ target, const T *__restrict__ draft, const float *__restrict__ uniforms,
    int gamma, int V, float k, int nchunks, int n_target_rows, int algo,
    const float2 *__restrict__ stats, const RowCoef *__restrict__ coef,
    const float *__restrict__ spart, const float *__restrict__ rpart,
    int32_t *__restrict__ accept_len, int32_t *__restrict__ next_token, float *__restrict__ debug_out)
{
    constexpr int kVec = ElemTraits<T>::kVec;
    constexpr int kU = kChunk / (kThreads * kVec);
    extern __shared__ double smd[];                     // [gamma+1] S_i, [gamma+1] rejected mass
    __shared__ float lds[kWaves];
    __shared__ int s_tau, s_chunk, s_mode, s_hit, s_first, s_last;
    __shared__ float s_t;
    double *S = smd, *R = smd + (gamma + 1);
    const int b = blockIdx.x, tid = threadIdx.x;
    const RowCoef *rcb = coef + (size_t)b * (gamma + 1);

    // S_i = cq_i * sum_c spart[b, i, c], chunks added in index order
    for (int i = tid; i <= gamma; i += kThreads) {
        if (i < gamma) {
            double acc = 0.0, rej = 0.0;
            const float *sp = spart + ((size_t)b * gamma + i) * nchunks;
            for (int c = 0; c < nchunks; ++c) acc += (double)sp[c];
            if (algo == kGreedy) {
                const float *rp = rpart + ((size_t)b * gamma + i) * nchunks;
                for (int c = 0; c < nchunks; ++c) rej += (double)rp[c];
            }
            S[i] = acc * (double)rcb[i].cq;
            R[i] = rej * (double)rcb[i].cq;
        } else {
            S[i] = rcb[i].w;       // q_gamma == 0: the residual mass of the last row is w_gamma
            R[i] = 0.0;
        }
    }
    __syncthreads();

    if (tid == 0) {
        // accept tests: eta_i < h_i
        int tau = 0;
        const float *eta = uniforms + (size_t)b * (gamma + 1);
        for (int i = 0; i <= gamma; ++i) {
            double h;
            if (i == 0) h = 1.0;
            else if (algo == kToken) h = exp2(fmin(rcb[i].log2r, 0.0));                 // min(r_i, 1)
            else if (i == gamma) h = fmin(rcb[i].w, 1.0);                               // h_gamma = w_gamma
            else if (algo == kGreedy) h = R[i] > 0.0 ? fmin(S[i] / R[i], 1.0) : 1.0;    // p_remain / p_rej
            else h = rcb[i].w >= 1.0 ? 1.0 : S[i] / (S[i] + rcb[i].one_minus_w);        // block acceptance formula
            if (i >= 1) {
                const bool pass = (double)eta[i - 1] < h;
                if (algo == kToken) { if (pass && tau == i - 1) tau = i; }              // stops at the first failure
                else if (pass) tau = i;                                                 // last passing sub-block
            }
            if (debug_out) {
                float *d = debug_out + ((size_t)b * (gamma + 1) + i) * 3;
                d[0] = (float)rcb[i].w; d[1] = (float)S[i]; d[2] = (float)h;
            }
        }
        accept_len[b] = tau;

        // pick the chunk of row tau that holds t = u * (total weight)
        const float u = eta[gamma];
        int mode = (tau == gamma) ? 1 : 0;              // 1: weights are p_tau; 0: residual weights
        double total = 0.0;
        if (mode == 0) {
            const float *sp = spart + ((size_t)b * gamma + tau) * nchunks;
            for (int c = 0; c < nchunks; ++c) total += (double)sp[c];
            if (!(total > 0.0)) mode = 1;               // no residual mass at all: fall back to p_tau
        }
        const float2 *st = stats + ((size_t)b * (gamma + 1) + tau) * nchunks;
        const float M = rcb[tau].row_max;
        if (mode == 1) {
            total = 0.0;
            for (int c = 0; c < nchunks; ++c) total += (double)(st[c].y * fast_exp2(st[c].x - M));
        }
        const double t = (double)u * total;
        double cum = 0.0;
        int chunk = -1, last_nonzero = 0;
        for (int c = 0; c < nchunks; ++c) {
            const double part = mode == 0 ? (double)spart[((size_t)b * gamma + tau) * nchunks + c]
                                          : (double)(st[c].y * fast_exp2(st[c].x - M));
            if (part > 0.0) last_nonzero = c;
            if (cum + part > t) { chunk = c; break; }
            cum += part;
        }
        float t_in = (float)(t - cum);
        if (chunk < 0) { chunk = last_nonzero; t_in = INFINITY; }   // rounding pushed t past the end
        s_tau = tau; s_chunk = chunk; s_mode = mode; s_t = t_in; s_hit = -1;
    }
    __syncthreads();
    const int tau = s_tau, chunk = s_chunk, mode = s_mode;
    float t_in = s_t;

    // weights of the chosen chunk, recomputed exactly as the partial sums were
    const T *prow = target + ((size_t)b * (gamma + 1) + tau) * V;
    float wgt[kU][kVec];
    if (mode == 0) {
        const RowCoef rc = rcb[tau];
        const T *qrow = draft + ((size_t)b * gamma + tau) * V;
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            float xp[kVec], xq[kVec];
            const int idx = chunk * kChunk + (u * kThreads + tid) * kVec;
            load_vec<T, ALIGNED>(prow, V, idx, xp);
            load_vec<T, ALIGNED>(qrow, V, idx, xq);
#pragma unroll
            for (int e = 0; e < kVec; ++e) wgt[u][e] = fmaxf(residual_term(xp[e], xq[e], k, rc), 0.f);
        }
    } else {
        const float2 st = stats[((size_t)b * (gamma + 1) + tau) * nchunks + chunk];
        const float scale = fast_exp2(st.x - rcb[tau].row_max);
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            float xp[kVec];
            load_vec<T, ALIGNED>(prow, V, chunk * kChunk + (u * kThreads + tid) * kVec, xp);
#pragma unroll
            for (int e = 0; e < kVec; ++e) wgt[u][e] = fast_exp2(__builtin_fmaf(xp[e], k, -st.x)) * scale;
        }
    }

    // walk the chunk in vocabulary order: sub-chunk u, then thread, then element
    int last_positive = -1;
    bool found = false;
#pragma unroll
    for (int u = 0; u < kU; ++u) {
        float mine = 0.f;
#pragma unroll
        for (int e = 0; e < kVec; ++e) {
            mine += wgt[u][e];
            if (wgt[u][e] > 0.f) last_positive = chunk * kChunk + (u * kThreads + tid) * kVec + e;
        }
        float exc, total;
        const float inc = block_inclusive_scan(mine, lds, exc, total);
        if (tid == 0) s_first = kThreads;
        __syncthreads();
        if (inc > t_in) atomicMin(&s_first, tid);       // first thread whose running sum exceeds t
        __syncthreads();
        const int first = s_first;
        if (first < kThreads) {
            if (tid == first) {
                float run = exc;
                int y = -1, lastpos = 0;
#pragma unroll
                for (int e = 0; e < kVec; ++e) {
                    run += wgt[u][e];
                    if (wgt[u][e] > 0.f) lastpos = e;
                    if (y < 0 && run > t_in) y = e;
                }
                if (y < 0) y = lastpos;     // scan and walk rounded differently: last positive weight
                s_hit = chunk * kChunk + (u * kThreads + tid) * kVec + y;
            }
            found = true;
            break;
        }
        t_in -= total;
    }
    if (!found) {
        // t lies beyond the chunk's recomputed total: the last token of positive weight
        if (tid == 0) s_last = -1;
        __syncthreads();
        atomicMax(&s_last, last_positive);
        __syncthreads();
        if (tid == 0) s_hit = s_last < 0 ? 0 : s_last;
    }
    __syncthreads();
    if (tid == 0) next_token[b] = s_hit;
}

// ---------------------------------------------------------------------------- host side
struct Layout {
    int nchunks;
    size_t rows_total;
    size_t off_stats, off_coef, off_spart, off_rpart, total;
};

bool make_layout(int32_t B, int32_t gamma, int32_t V, Layout &L)
{
    if (B < 1 || gamma < 1 || V < 1 || gamma > SV_MAX_GAMMA) return false;
    L.nchunks = (V + kChunk - 1) / kChunk;
    L.rows_total = (size_t)B * (2 * (size_t)gamma + 1);
    if (L.rows_total * (size_t)L.nchunks > 0x7fffffffull) return false;     // 1-D grids of 32-bit size
    size_t off = 0;
    L.off_stats = off; off = align_up(off + L.rows_total * L.nchunks * sizeof(float2), 256);
    L.off_coef = off;  off = align_up(off + (size_t)B * (gamma + 1) * sizeof(RowCoef), 256);
    L.off_spart = off; off = align_up(off + (size_t)B * gamma * L.nchunks * sizeof(float), 256);
    L.off_rpart = off; off = align_up(off + (size_t)B * gamma * L.nchunks * sizeof(float), 256);
    L.total = off;
    return true;
}

template <typename T, bool ALIGNED>
sv_status_t launch_all(int algo, const void *target_v, const void *draft_v, const int32_t *tokens,
                       const float *uniforms, int B, int gamma, int V, float k, const Layout &L,
                       char *ws, int32_t *accept_len, int32_t *next_token, float *debug_out,
                       hipStream_t stream)
{
    const T *target = static_cast<const T *>(target_v);
    const T *draft = static_cast<const T *>(draft_v);
    float2 *stats = reinterpret_cast<float2 *>(ws + L.off_stats);
    RowCoef *coef = reinterpret_cast<RowCoef *>(ws + L.off_coef);
    float *spart = reinterpret_cast<float *>(ws + L.off_spart);
    float *rpart = reinterpret_cast<float *>(ws + L.off_rpart);
    const int n_target_rows = B * (gamma + 1);

    row_stats_kernel<T, ALIGNED><<<(unsigned)(L.rows_total * L.nchunks), kThreads, 0, stream>>>(
        target, draft, B, gamma, V, k, L.nchunks, stats);
    const size_t sm2 = 2 * (gamma + 1) * sizeof(double) + (gamma + 1) * sizeof(float);
    prefix_weights_kernel<T><<<B, 64, sm2, stream>>>(target, draft, tokens, gamma, V, k, L.nchunks,
                                                    n_target_rows, algo, stats, coef);
    const unsigned pair_blocks = (unsigned)((size_t)B * gamma * L.nchunks);
    if (algo == kGreedy)
        residual_kernel<T, ALIGNED, true><<<pair_blocks, kThreads, 0, stream>>>(
            target, draft, gamma, V, k, L.nchunks, coef, spart, rpart);
    else
        residual_kernel<T, ALIGNED, false><<<pair_blocks, kThreads, 0, stream>>>(
            target, draft, gamma, V, k, L.nchunks, coef, spart, rpart);
    const size_t sm4 = 2 * (gamma + 1) * sizeof(double);
    finalize_kernel<T, ALIGNED><<<B, kThreads, sm4, stream>>>(
        target, draft, uniforms, gamma, V, k, L.nchunks, n_target_rows, algo, stats, coef, spart, rpart,
        accept_len, next_token, debug_out);
    return hipGetLastError() == hipSuccess ? SV_OK : SV_ERR_HIP;
}

sv_status_t verify_entry(int algo, const void *target, const void *draft, const int32_t *tokens,
                         const float *uniforms, int32_t B, int32_t gamma, int32_t V, sv_dtype_t dtype,
                         float temperature, void *workspace, size_t workspace_bytes,
                         int32_t *accept_len, int32_t *next_token, float *debug_out, void *stream_v)
{
    if (!target || !draft || !tokens || !uniforms || !workspace || !accept_len || !next_token)
        return SV_ERR_INVALID_ARG;
    if (B < 1 || gamma < 1 || V < 1) return SV_ERR_INVALID_ARG;
    if (!(temperature > 0.f) || !isfinite(temperature)) return SV_ERR_INVALID_ARG;
    if (dtype != SV_DTYPE_F32 && dtype != SV_DTYPE_BF16) return SV_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return SV_ERR_INVALID_ARG;
    Layout L;
    if (!make_layout(B, gamma, V, L)) return SV_ERR_UNSUPPORTED;
    if (workspace_bytes < L.total) return SV_ERR_WORKSPACE_TOO_SMALL;

    const float k = (float)(1.4426950408889634074 / (double)temperature);
    const size_t esize = dtype == SV_DTYPE_F32 ? 4 : 2;
    const bool aligned = ((reinterpret_cast<uintptr_t>(target) | reinterpret_cast<uintptr_t>(draft)) & 15u) == 0 &&
                         ((size_t)V * esize) % 16 == 0;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char *ws = static_cast<char *>(workspace);
    if (dtype == SV_DTYPE_F32) {
        return aligned ? launch_all<float, true>(algo, target, draft, tokens, uniforms, B, gamma, V, k, L, ws,
                                                 accept_len, next_token, debug_out, stream)
                       : launch_all<float, false>(algo, target, draft, tokens, uniforms, B, gamma, V, k, L, ws,
                                                  accept_len, next_token, debug_out, stream);
    }
    return aligned ? launch_all<bf16_t, true>(algo, target, draft, tokens, uniforms, B, gamma, V, k, L, ws,
                                              accept_len, next_token, debug_out, stream)
                   : launch_all<bf16_t, false>(algo, target, draft, tokens, uniforms, B, gamma, V, k, L, ws,
                                               accept_len, next_token, debug_out, stream);
}

}  // namespace

extern "C" {

size_t spec_verify_workspace_bytes(int32_t B, int32_t gamma, int32_t V)
{
    Layout L;
    return make_layout(B, gamma, V, L) ? L.total : 0;
}

sv_status_t spec_verify_block(const void *target_logits, const void *draft_logits,
                              const int32_t *draft_tokens, const float *uniforms,
                              int32_t B, int32_t gamma, int32_t V, sv_dtype_t dtype,
                              float temperature, void *workspace, size_t workspace_bytes,
                              int32_t *accept_len, int32_t *next_token, float *debug_out, void *stream)
{
    return verify_entry(kBlock, target_logits, draft_logits, draft_tokens, uniforms, B, gamma, V, dtype,
                        temperature, workspace, workspace_bytes, accept_len, next_token, debug_out, stream);
}

sv_status_t spec_verify_token(const void *target_logits, const void *draft_logits,
                              const int32_t *draft_tokens, const float *uniforms,
                              int32_t B, int32_t gamma, int32_t V, sv_dtype_t dtype,
                              float temperature, void *workspace, size_t workspace_bytes,
                              int32_t *accept_len, int32_t *next_token, float *debug_out, void *stream)
{
    return verify_entry(kToken, target_logits, draft_logits, draft_tokens, uniforms, B, gamma, V, dtype,
                        temperature, workspace, workspace_bytes, accept_len, next_token, debug_out, stream);
}

sv_status_t spec_verify_greedy(const void *target_logits, const void *draft_logits,
                               const int32_t *draft_tokens, const float *uniforms,
                               int32_t B, int32_t gamma, int32_t V, sv_dtype_t dtype,
                               float temperature, void *workspace, size_t workspace_bytes,
                               int32_t *accept_len, int32_t *next_token, float *debug_out, void *stream)
{
    return verify_entry(kGreedy, target_logits, draft_logits, draft_tokens, uniforms, B, gamma, V, dtype,
                        temperature, workspace, workspace_bytes, accept_len, next_token, debug_out, stream);
}

const char *spec_verify_status_string(sv_status_t status)
{
    switch (status) {
    case SV_OK: return "ok";
    case SV_ERR_INVALID_ARG: return "invalid argument";
    case SV_ERR_UNSUPPORTED: return "unsupported size";
    case SV_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case SV_ERR_HIP: return "HIP launch failed";
    }
    return "unknown status";
}

}  // extern "C"
