// Staged path: four launches, each logit read from HBM twice.  It has no limit on the
// vocabulary size and needs no cross-workgroup waiting, so the library uses it for shapes
// the fused kernel does not take; it is also the simplest statement of the method on the GPU.
//
//   1. row_stats_kernel      every logit row, cut into chunks of kChunk logits: the chunk's
//                            maximum (times k) and the sum of exp2(y - that)
//   2. prefix_weights_kernel per sequence: row log2-normalisers, the ratios of the drafted
//                            tokens, the recursion w_i = min(w_{i-1} r_i, 1) of Alg. 2 (in
//                            double, in the log domain), and the row constants of step 3
//   3. residual_kernel       every (target row i, draft row i) pair: chunk partial sums of
//                            max(w_i p_i(x) - q_i(x), 0)
//   4. finalize_kernel       per sequence: S_i, h_i, tau, then the inverse-CDF draw of Y
//                            (pick the chunk from the partial sums, re-read that one chunk)
#pragma once

#include "common.hpp"

namespace sv {

struct SeqCoef {
    RowCoef rc;
    double w;            // w_i
    double one_minus_w;
    double log2r;        // log2 r_i (ratio of draft token i, judged with rows i-1); 0 at i = 0
    float row_max;       // maximum over the target row's chunks of (chunk max * k)
    int needed;          // whether S_i can matter (see prefix_weights_kernel); where not, no partial sums are formed
};

template <typename T, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void row_stats_kernel(
    const T *__restrict__ target, const T *__restrict__ draft, size_t tstride, size_t dstride,
    int B, int gamma, int V, float k, int nchunks, float2 *__restrict__ stats)
{
    constexpr int kVec = ElemTraits<T>::kVec;
    constexpr int kU = kChunk / (kThreads * kVec);
    __shared__ float lds[kWaves];
    const int r = blockIdx.x / nchunks, c = blockIdx.x - r * nchunks, tid = threadIdx.x;
    const int n_target_rows = B * (gamma + 1);
    const T *row = r < n_target_rows ? target + (size_t)r * tstride : draft + (size_t)(r - n_target_rows) * dstride;

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
    const float shift = m > -INFINITY ? mk : 0.f;       // a chunk without a finite logit (masked out, or beyond the row)

    float s = 0.f;
#pragma unroll
    for (int u = 0; u < kU; ++u)
#pragma unroll
        for (int e = 0; e < kVec; ++e) s += fast_exp2(__builtin_fmaf(x[u][e], k, -shift));
    s = block_sum(s, lds);
    if (tid == 0) stats[(size_t)r * nchunks + c] = make_float2(mk, s);
}

template <typename T>
__global__ __launch_bounds__(64) void prefix_weights_kernel(
    const T *__restrict__ target, const T *__restrict__ draft, size_t tstride, size_t dstride,
    const int32_t *__restrict__ tokens,
    int gamma, int V, float k, double kd, double k_eps, int nchunks, int n_target_rows, int algo,
    const float2 *__restrict__ stats, SeqCoef *__restrict__ coef, const int32_t *__restrict__ draft_lens,
    const float *__restrict__ uniforms, int every_residual)
{
    extern __shared__ double sm[];          // [2*(gamma+1)] log2-normalisers, then row maxima
    double *L_p = sm, *L_q = sm + (gamma + 1);
    float *M_p = reinterpret_cast<float *>(sm + 2 * (gamma + 1));
    float *M_q = M_p + (gamma + 1);
    const int b = blockIdx.x, tid = threadIdx.x;
    // this sequence's draft length (kept in range whatever the caller wrote); gamma stays the stride
    const int gb = draft_lens ? (draft_lens[b] < 1 ? 1 : draft_lens[b] > gamma ? gamma : draft_lens[b]) : gamma;

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
        if (is_target) { L_p[i] = L; M_p[i] = M; } else { L_q[i] = L; M_q[i] = M; }
    }
    __syncthreads();
    if (tid != 0) return;

    // Alg. 2, the recursion for w_i (the paper's p_i), carried as log2 w_i so that products of
    // ratios neither overflow nor lose 1 - w_i when w_i is close to 1.
    // Which residual masses can matter: h_i = S_i / (S_i + 1 - w_i) <= w_i because S_i <= w_i, so a test with
    // eta_i >= w_i fails whatever S_i is and position i cannot become tau (margin far above the rounding of h_i);
    // Alg. 1 stops at the first failed test, so only positions that all earlier tests let through can.
    // Position 0 is where tau = 0 draws from.  `every_residual`: the caller wants every S_i reported.
    double log2w = 0.0, log2r = 0.0;
    bool prefix_pass = true;
    const float *eta = uniforms + (size_t)b * (gamma + 1);
    for (int i = 0; i <= gb; ++i) {
        SeqCoef sc;
        if (i >= 1) prefix_pass = prefix_pass && (double)eta[i - 1] < exp2(fmin(log2r, 0.0));
        sc.needed = (i == 0 || every_residual) ? 1
                  : algo == kToken ? (prefix_pass ? 1 : 0)
                  : (log2((double)eta[i - 1]) < log2w + 1.0e-3 ? 1 : 0);
        const double lw = (algo == kToken) ? 0.0 : log2w;     // token verification: residual is p - q
        sc.rc = make_row_coef(L_p[i] - lw, i < gb ? L_q[i] : 0.0);
        sc.w = exp2(lw);
        sc.one_minus_w = -expm1(lw * 0.69314718055994530942);
        sc.log2r = log2r;
        sc.row_max = M_p[i];
        coef[(size_t)b * (gamma + 1) + i] = sc;
        if (i < gb) {
            // r_{i+1} = p_i(X_{i+1}) / q_i(X_{i+1}) from the two gathered logits.  The sweeps scale
            // logits by the float k; the exact factor is kd = k (1 + k_eps).  To first order that moves
            // a row's log2-normaliser by k_eps * (the scaled logit where the mass sits, taken as the
            // row maximum); only this ratio, whose logs reach hundreds, is sensitive to it.
            const int tok = tokens[(size_t)b * gamma + i];
            const double ya = logit_as_double(target + ((size_t)b * (gamma + 1) + i) * tstride + tok) * kd;
            const double yb = logit_as_double(draft + ((size_t)b * gamma + i) * dstride + tok) * kd;
            log2r = (ya - (L_p[i] + k_eps * (double)M_p[i])) - (yb - (L_q[i] + k_eps * (double)M_q[i]));
            log2r = fmax(log2r, kLog2RatioFloor);   // a drafted token the target masks out (logit -inf): r = 0, kept finite
            log2w += log2r;
            if (algo != kGreedy && log2w > 0.0) log2w = 0.0;  // the min{., 1}; greedy block verification omits it
        }
    }
}

template <typename T, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void residual_kernel(
    const T *__restrict__ target, const T *__restrict__ draft, size_t tstride, size_t dstride,
    int gamma, int V, float k, int nchunks, const SeqCoef *__restrict__ coef,
    float *__restrict__ spart)
{
    constexpr int kVec = ElemTraits<T>::kVec;
    constexpr int kU = kChunk / (kThreads * kVec);
    __shared__ float lds[kWaves];
    const int pr = blockIdx.x / nchunks, c = blockIdx.x - pr * nchunks, tid = threadIdx.x;
    const int b = pr / gamma, i = pr - b * gamma;
    if (!coef[(size_t)b * (gamma + 1) + i].needed) return;      // this position's residual mass cannot matter (whole workgroup)
    const RowCoef rc = coef[(size_t)b * (gamma + 1) + i].rc;
    const T *prow = target + ((size_t)b * (gamma + 1) + i) * tstride;
    const T *qrow = draft + ((size_t)b * gamma + i) * dstride;

    float xp[kU][kVec], xq[kU][kVec];
#pragma unroll
    for (int u = 0; u < kU; ++u) {
        const int idx = c * kChunk + (u * kThreads + tid) * kVec;
        load_vec<T, ALIGNED>(prow, V, idx, xp[u]);
        load_vec<T, ALIGNED>(qrow, V, idx, xq[u]);
    }
    float acc = 0.f;
#pragma unroll
    for (int u = 0; u < kU; ++u)
#pragma unroll
        for (int e = 0; e < kVec; ++e) acc += fmaxf(residual_term(xp[u][e], xq[u][e], k, rc), 0.f);
    acc = block_sum(acc, lds);
    if (tid == 0) spart[(size_t)pr * nchunks + c] = acc;
}

template <typename T, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void finalize_kernel(
    const T *__restrict__ target, const T *__restrict__ draft, size_t tstride, size_t dstride,
    const float *__restrict__ uniforms,
    int gamma, int V, float k, int nchunks, int algo,
    const float2 *__restrict__ stats, const SeqCoef *__restrict__ coef,
    const float *__restrict__ spart,
    int32_t *__restrict__ accept_len, int32_t *__restrict__ next_token, float *__restrict__ debug_out,
    const int32_t *__restrict__ draft_lens)
{
    extern __shared__ double smd[];                     // [gamma+1] S_i
    __shared__ float lds[kWaves];
    __shared__ int s_tau, s_chunk, s_mode, s_ints[2];
    __shared__ float s_t;
    double *S = smd;
    const int b = blockIdx.x, tid = threadIdx.x;
    const SeqCoef *scb = coef + (size_t)b * (gamma + 1);
    // this sequence's draft length (kept in range whatever the caller wrote); gamma stays the stride
    const int gb = draft_lens ? (draft_lens[b] < 1 ? 1 : draft_lens[b] > gamma ? gamma : draft_lens[b]) : gamma;

    // S_i = cq_i * sum_c spart[b, i, c], chunks added in index order
    for (int i = tid; i <= gb; i += kThreads) {
        if (i < gb) {
            double acc = 0.0;
            const float *sp = spart + ((size_t)b * gamma + i) * nchunks;
            if (scb[i].needed)                      // otherwise no partial sums were formed: the test fails whatever S_i is
                for (int c = 0; c < nchunks; ++c) acc += (double)sp[c];
            S[i] = acc * (double)scb[i].rc.cq;
        } else {
            S[i] = scb[i].w;       // q_gamma == 0: the residual mass of the last row is w_gamma
        }
    }
    __syncthreads();

    if (tid == 0) {
        // accept tests: eta_i < h_i
        int tau = 0;
        const float *eta = uniforms + (size_t)b * (gamma + 1);
        for (int i = 0; i <= gb; ++i) {
            double h;
            if (i == 0) h = 1.0;
            else if (algo == kToken) h = exp2(fmin(scb[i].log2r, 0.0));                 // min(r_i, 1)
            else if (i == gb) h = fmin(scb[i].w, 1.0);                               // h_gamma = w_gamma
            // block acceptance formula.  Greedy block verification (Alg. 4) divides by the rejected mass
            // sum_x max(q - w p, 0) instead: the same number, S - sum_x (w p - q) = S + 1 - w for rows that sum to
            // one (w unclipped; at w >= 1 the ratio is >= 1 and every eta in [0, 1) passes)
            else h = scb[i].w >= 1.0 ? 1.0 : S[i] / (S[i] + scb[i].one_minus_w);
            if (i >= 1) {
                const bool pass = (double)eta[i - 1] < h && (i == gb || scb[i].needed);
                if (algo == kToken) { if (pass && tau == i - 1) tau = i; }              // stops at the first failure
                else if (pass) tau = i;                                                 // last passing sub-block
            }
            if (debug_out) {
                float *d = debug_out + ((size_t)b * (gamma + 1) + i) * 3;
                d[0] = (float)scb[i].w; d[1] = (float)S[i]; d[2] = (float)h;
            }
        }
        accept_len[b] = tau;

        // pick the chunk of row tau that holds t = u * (total weight)
        const float u = eta[gb];
        int mode = (tau == gb) ? 1 : 0;              // 1: weights are p_tau; 0: residual weights
        double total = 0.0;
        if (mode == 0) {
            const float *sp = spart + ((size_t)b * gamma + tau) * nchunks;
            for (int c = 0; c < nchunks; ++c) total += (double)sp[c];
            if (!(total > 0.0)) mode = 1;               // no residual mass at all: fall back to p_tau
        }
        const float2 *st = stats + ((size_t)b * (gamma + 1) + tau) * nchunks;
        const float M = scb[tau].row_max;
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
        s_tau = tau; s_chunk = chunk; s_mode = mode; s_t = t_in;
    }
    __syncthreads();
    const int tau = s_tau, chunk = s_chunk;
    const bool residual = s_mode == 0;
    const T *prow = target + ((size_t)b * (gamma + 1) + tau) * tstride;
    const T *qrow = draft + ((size_t)b * gamma + (tau < gb ? tau : 0)) * dstride;
    const float2 st = stats[((size_t)b * (gamma + 1) + tau) * nchunks + chunk];
    const int y = walk_range<T, ALIGNED>(prow, qrow, V, chunk * kChunk, kChunk / (kThreads * 8), k, residual,
                                         scb[tau].rc, st.x, fast_exp2(st.x - scb[tau].row_max), s_t, lds, s_ints);
    if (tid == 0) next_token[b] = y;
}

}  // namespace sv
