// Verification with the distributions themselves as inputs (the ps / qs arrays of App. A): target rows
// hold p_i(x), draft rows q_i(x), used as given - no temperature, no normalisation sweep.  The weight
// w_i of Alg. 2 needs only the two gathered probabilities of each earlier drafted token, so every
// element is read from HBM exactly once and no workgroup waits for another:
//
//   1. probs_weights_kernel   one wave per sequence: the ratios r_i of the drafted tokens and the
//                             recursion w_i = min(w_{i-1} r_i, 1) (in double, in the log domain)
//   2. probs_residual_kernel  one workgroup per (sequence, position, chunk of kChunk tokens): the
//                             chunk's share of S_i = sum_x max(w_i p_i(x) - q_i(x), 0)
//                             (numerator of the block acceptance formula; for greedy block verification,
//                             Alg. 4, also the rejected mass sum_x max(q_i - w_i p_i, 0)); at the
//                             sequence's last position the chunk's share of sum_x p(x)
//   3. probs_finalize_kernel  one workgroup per sequence: S_i, h_i, the accept tests of Alg. 1 / 2 / 4,
//                             then the inverse-CDF draw of Y (pick the chunk from the partial sums,
//                             re-read that one chunk)
#pragma once

#include "fused.hpp"

namespace sv {

constexpr int kProbsKeepMax = 8192;      // chunk sums of one sequence that the finishing kernel keeps in LDS (32 KB)

struct ProbWeight {
    double w;            // w_i (1 for token verification, whose residual is p - q)
    double one_minus_w;
    double h_token;      // min(r_i, 1), r_i the ratio of drafted token i judged with rows i-1; 1 at i = 0
    float w_hi, w_lo;    // w_i split into two floats
    int needed;          // whether the sums over rows i can matter (see probs_weights_kernel); where not, none are formed
};

// kVec consecutive probabilities of a row; elements at or beyond V count as 0
template <typename T, bool ALIGNED>
__device__ __forceinline__ void load_probs(const T *row, int V, int idx, float *out)
{
    load_vec<T, ALIGNED>(row, V, idx, out);
#pragma unroll
    for (int e = 0; e < ElemTraits<T>::kVec; ++e) out[e] = fmaxf(out[e], 0.f);
}

// w p - q with w = w_hi + w_lo (a double split into two floats): the products are exact inside the
// fused multiply-adds, so a small residual keeps its relative accuracy
__device__ __forceinline__ float prob_residual(float p, float q, float w_hi, float w_lo)
{
    return __builtin_fmaf(w_lo, p, __builtin_fmaf(w_hi, p, -q));
}

__device__ __forceinline__ int clamped_draft_len(const int32_t *draft_lens, int b, int gamma)
{
    if (!draft_lens) return gamma;
    const int g = draft_lens[b];
    return g < 1 ? 1 : g > gamma ? gamma : g;
}

// w_0 = 1, w_i = min(w_{i-1} r_i, 1) (Alg. 2; Alg. 4 omits the min), r_i = p_{i-1}(X_i) / q_{i-1}(X_i).
// One wave per sequence: lane j gathers the two probabilities of drafted token j + 1, every lane runs
// the recursion up to the position it carries in log2 (products of ratios neither overflow nor lose 1 - w_i
// next to 1), lane i writes the constants of position i.
template <typename T>
__global__ __launch_bounds__(64) void probs_weights_kernel(
    const T *__restrict__ target, const T *__restrict__ draft, size_t tstride, size_t dstride,
    const int32_t *__restrict__ tokens, const int32_t *__restrict__ draft_lens, int gamma, int algo,
    ProbWeight *__restrict__ weights, const float *__restrict__ uniforms, int every_sum)
{
    const int b = blockIdx.x, lane = threadIdx.x;
    const int gb = clamped_draft_len(draft_lens, b, gamma);
    double mine = 0.0;
    if (lane < gb) {
        const int tok = tokens[(size_t)b * gamma + lane];
        const double lp = log2(logit_as_double(target + ((size_t)b * (gamma + 1) + lane) * tstride + tok));
        const double lq = log2(logit_as_double(draft + ((size_t)b * gamma + lane) * dstride + tok));
        mine = fmax(lp - lq, kLog2RatioFloor);     // a drafted token outside the target's support: r = 0, kept finite
    }
    // lane l carries position l + 1 (positions 1 .. gb <= SV_MAX_GAMMA = 64); position 0 is w_0 = 1
    double log2w = 0.0, log2r = 0.0;
    for (int j = 0; j < gb; ++j) {
        const double r = __shfl(mine, j, 64);
        if (j <= lane) {
            log2r = r;
            log2w += r;
            if (algo != kGreedy && log2w > 0.0) log2w = 0.0;
        }
    }
    ProbWeight *wb = weights + (size_t)b * (gamma + 1);
    if (lane == 0) {
        ProbWeight first;
        first.w = 1.0; first.one_minus_w = 0.0; first.h_token = 1.0; first.w_hi = 1.f; first.w_lo = 0.f;
        first.needed = 1;                                  // tau = 0 draws from the residual of rows 0
        wb[0] = first;
    }
    const int i = lane + 1;
    const double w_block = exp2(log2w);
    if (algo == kToken) log2w = 0.0;
    ProbWeight pw;
    pw.w = exp2(log2w);
    pw.one_minus_w = -expm1(log2w * 0.69314718055994530942);
    pw.h_token = exp2(fmin(log2r, 0.0));
    pw.w_hi = (float)pw.w;
    pw.w_lo = (float)(pw.w - (double)pw.w_hi);
    // Which sums can matter (exact, whatever the rows sum to).  Alg. 1 stops at the first failed test, so only a
    // position that every earlier test let through can become tau; the last target row is summed (and drawn
    // from) only if tau = gamma: every test passed (Alg. 1), or the last one did (Alg. 2 / 4: eta < w_gamma).
    // The tests are evaluated with the expressions the finishing kernel uses, on the same stored values.
    const float eta_i = i <= gb ? uniforms[(size_t)b * (gamma + 1) + i - 1] : 1.f;
    const unsigned long long failed = __ballot(i <= gb && !((double)eta_i < pw.h_token));
    const bool prefix_pass = (failed & ((2ull << lane) - 1ull)) == 0;     // tests 1 .. i
    if (i > gb) return;
    if (every_sum) pw.needed = 1;
    else if (algo == kToken) pw.needed = prefix_pass ? 1 : 0;
    else pw.needed = (i < gb || (double)eta_i < fmin(w_block, 1.0)) ? 1 : 0;
    wb[i] = pw;
}

template <typename T, bool ALIGNED, bool GREEDY>
__global__ __launch_bounds__(kThreads) void probs_residual_kernel(
    const T *__restrict__ target, const T *__restrict__ draft, size_t tstride, size_t dstride,
    const int32_t *__restrict__ draft_lens,
    int gamma, int V, int nchunks, float2 *__restrict__ part, const ProbWeight *__restrict__ weights)
{
    constexpr int kVec = ElemTraits<T>::kVec;
    constexpr int kU = kChunk / (kThreads * kVec);
    __shared__ float lds[kWaves];
    const int pr = blockIdx.x / nchunks, c = blockIdx.x - pr * nchunks, tid = threadIdx.x;
    const int b = pr / (gamma + 1), i = pr - b * (gamma + 1);
    const int gb = clamped_draft_len(draft_lens, b, gamma);
    if (i > gb) return;                                          // a position this sequence does not use
    if (!weights[pr].needed) return;                             // sums that cannot matter (whole workgroup)
    const T *target_seq = target + (size_t)b * (gamma + 1) * tstride;
    const T *draft_seq = draft + (size_t)b * gamma * dstride;
    const T *prow = target_seq + (size_t)i * tstride;
    const bool last = i == gb;                                   // no draft row: q == 0
    const T *qrow = draft_seq + (size_t)(last ? 0 : i) * dstride;
    const float w_hi = weights[pr].w_hi, w_lo = weights[pr].w_lo;

    float xp[kU][kVec], xq[kU][kVec];
#pragma unroll
    for (int u = 0; u < kU; ++u) {
        const int idx = c * kChunk + (u * kThreads + tid) * kVec;
        load_probs<T, ALIGNED>(prow, V, idx, xp[u]);
        if (!last) load_probs<T, ALIGNED>(qrow, V, idx, xq[u]);
    }

    float acc = 0.f, rej = 0.f;
    if (last) {
#pragma unroll
        for (int u = 0; u < kU; ++u)
#pragma unroll
            for (int e = 0; e < kVec; ++e) acc += xp[u][e];
    } else {
#pragma unroll
        for (int u = 0; u < kU; ++u)
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                const float d = prob_residual(xp[u][e], xq[u][e], w_hi, w_lo);
                acc += fmaxf(d, 0.f);
                if constexpr (GREEDY) rej += fmaxf(-d, 0.f);
            }
    }
    acc = block_sum(acc, lds);
    if constexpr (GREEDY) rej = block_sum(rej, lds);
    if (tid == 0) part[(size_t)pr * nchunks + c] = make_float2(acc, rej);
}

// The workgroup's sum of the weights of chunk c of a row pair, thread t owning the kPerThread
// consecutive tokens from c * kChunk + t * kPerThread; every thread receives its own sum.
template <typename T, bool ALIGNED>
__device__ __forceinline__ float prob_thread_weights(const T *prow, const T *qrow, int V, int c, bool residual,
                                                     float w_hi, float w_lo, float *wgt)
{
    constexpr int kVec = ElemTraits<T>::kVec;
    const int start = c * kChunk + (int)threadIdx.x * kPerThread;
    float mine = 0.f;
#pragma unroll
    for (int v = 0; v < kPerThread / kVec; ++v) {
        float xp[kVec], xq[kVec];
        load_probs<T, ALIGNED>(prow, V, start + v * kVec, xp);
        if (residual) load_probs<T, ALIGNED>(qrow, V, start + v * kVec, xq);
#pragma unroll
        for (int e = 0; e < kVec; ++e) {
            const float g = residual ? fmaxf(prob_residual(xp[e], xq[e], w_hi, w_lo), 0.f) : xp[e];
            wgt[v * kVec + e] = g;
            mine += g;
        }
    }
    return mine;
}

// Sums and inclusive sums over the lanes of a wave in double, through DPP (fixed orders).
__device__ __forceinline__ double wave_total_double(double v)
{
    double first, second;
    halves_sum_f64(v, first, second);
    return first + second;
}
__device__ __forceinline__ double wave_inclusive_scan_double(double v) { return wave_scan(v); }

template <typename T, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void probs_finalize_kernel(
    const T *__restrict__ target, const T *__restrict__ draft, size_t tstride, size_t dstride,
    const float *__restrict__ uniforms, const int32_t *__restrict__ draft_lens,
    int gamma, int V, int nchunks, int algo, const float2 *__restrict__ part, const ProbWeight *__restrict__ weights,
    int32_t *__restrict__ accept_len, int32_t *__restrict__ next_token, float *__restrict__ debug_out)
{
    extern __shared__ double smd[];                     // [gamma+1] S_i, [gamma+1] rejected mass, then the kept partial sums
    __shared__ double wave_tot[kWaves];
    __shared__ int s_tau, s_chunk, s_mode, s_winner, wave_cand[kWaves];
    __shared__ double s_t, s_total;
    double *S = smd, *R = smd + (gamma + 1);
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int gb = clamped_draft_len(draft_lens, b, gamma);
    const float2 *pb = part + (size_t)b * (gamma + 1) * nchunks;
    const float *eta = uniforms + (size_t)b * (gamma + 1);
    // the chunk sums stay in LDS for the draw when they fit (the host sizes the dynamic LDS to match: one float per
    // sum, a second one per chunk for Alg. 4's rejected mass)
    const bool keep = (gamma + 1) * nchunks * (algo == kGreedy ? 2 : 1) <= kProbsKeepMax;
    float *kept = reinterpret_cast<float *>(smd + 2 * (gamma + 1));
    float *kept_rej = kept + (gamma + 1) * nchunks;
    __shared__ ProbWeight wbs[SV_MAX_GAMMA + 1];                 // the sequence's constants, read once

    // Everything that comes from memory is asked for at once - the sequence's constants, the uniforms, every chunk sum
    // of its positions (those of rows whose sums were not formed are stale and never used) - so that the kernel has
    // one trip to memory here and one for the chunk that holds the token.
    float eta_i = 0.f, u = 0.f;
    if (wave == 0) {
        if (lane + 1 <= gb) eta_i = eta[lane];
        u = eta[gb];
    }
    if (tid <= gb) wbs[tid] = weights[(size_t)b * (gamma + 1) + tid];
    if (keep) {
        const int n_words = (gb + 1) * nchunks;
        for (int w = tid; w < n_words; w += kThreads) {
            const float2 v = pb[w];
            kept[w] = v.x;
            if (algo == kGreedy) kept_rej[w] = v.y;
        }
    }
    __syncthreads();
    const ProbWeight *wb = wbs;
    ProbWeight pw = {};
    if (wave == 0 && lane + 1 <= gb) pw = wb[lane + 1];

    // S_i = sum over the chunks: wave (i mod 4) takes position i, lanes stride over the chunks
    for (int i = wave; i <= gb; i += kWaves) {
        double acc = 0.0, rej = 0.0;
        // (rows whose sums were not formed: S stays 0, their tests are decided without it and they cannot become tau)
        if (wb[i].needed) for (int c = lane; c < nchunks; c += 64) {
            if (keep) {
                acc += (double)kept[i * nchunks + c];
                if (algo == kGreedy) rej += (double)kept_rej[i * nchunks + c];
            } else {
                const float2 v = pb[(size_t)i * nchunks + c];
                acc += (double)v.x; rej += (double)v.y;
            }
        }
        acc = wave_total_double(acc);
        if (algo == kGreedy) rej = wave_total_double(rej);
        if (lane == 0) { S[i] = acc; R[i] = rej; }
    }
    __syncthreads();

    if (wave == 0) {
        // accept tests eta_i < h_i: lane l judges position l + 1 (positions 1 .. gb <= 64)
        const int i = lane + 1;
        bool pass = false;
        if (i <= gb) {
            double h;
            if (algo == kToken) h = pw.h_token;                                         // min(r_i, 1)
            else if (i == gb) h = fmin(pw.w, 1.0);                                      // h_gamma = w_gamma
            else if (algo == kGreedy) h = R[i] > 0.0 ? fmin(S[i] / R[i], 1.0) : 1.0;    // p_remain / p_rej
            else h = pw.w >= 1.0 ? 1.0 : S[i] / (S[i] + pw.one_minus_w);                // block acceptance formula
            pass = (double)eta_i < h;
            if (debug_out) {
                float *d = debug_out + ((size_t)b * (gamma + 1) + i) * 3;
                // q == 0 at the last position: the residual mass there is w times the row's own sum
                d[0] = (float)pw.w; d[1] = (float)(i == gb ? (algo == kBlock ? pw.w : pw.w * S[gb]) : S[i]); d[2] = (float)h;
            }
        }
        const unsigned long long passed = __ballot(pass);                               // bit l: position l + 1
        // token verification stops at the first failure; block / greedy keep the last passing sub-block
        const int tau = algo == kToken ? (~passed ? __ffsll((long long)~passed) - 1 : 64)
                                       : (passed ? 64 - __clzll((long long)passed) : 0);
        if (lane == 0) {
            if (debug_out) {
                float *d = debug_out + (size_t)b * (gamma + 1) * 3;
                d[0] = 1.f; d[1] = (float)S[0]; d[2] = 1.f;
            }
            accept_len[b] = tau;
            s_tau = tau;
            // weights of the draw: the residual of row tau, or p_tau when everything was accepted (its chunk
            // sums are then the partial sums of the last position) or when no residual mass is left at all
            s_mode = (tau < gb && S[tau] > 0.0) ? 0 : (tau == gb ? 1 : 2);
        }
    }
    __syncthreads();
    const int tau = s_tau, mode = s_mode;
    const bool residual = mode == 0;
    const T *prow = target + ((size_t)b * (gamma + 1) + tau) * tstride;
    const T *qrow = draft + ((size_t)b * gamma + (tau < gb ? tau : 0)) * dstride;
    float w_hi = 1.f, w_lo = 0.f;
    if (residual) { w_hi = wb[tau].w_hi; w_lo = wb[tau].w_lo; }
    float wgt[kPerThread];

    // the workgroup's chunk c: every thread's own sum, the sum of the threads before it, the chunk's total
    auto scan_chunk = [&](int c, bool res, float &mine, double &below, double &total) {
        mine = prob_thread_weights<T, ALIGNED>(prow, qrow, V, c, res, w_hi, w_lo, wgt);
        const double inc = wave_inclusive_scan_double((double)mine);
        __syncthreads();
        if (lane == 63) wave_tot[wave] = inc;
        __syncthreads();
        double base = 0.0, tot = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) { if (w < wave) base += wave_tot[w]; tot += wave_tot[w]; }
        below = base + inc - (double)mine;
        total = tot;
    };

    if (mode == 2) {
        // chunk sums of p_tau were never formed for this row: form the row total here (rare: rounding ate a residual)
        double row_total = 0.0;
        for (int c = 0; c < nchunks; ++c) {
            float mine; double below, total;
            scan_chunk(c, false, mine, below, total);
            row_total += total;
        }
        if (tid == 0) { s_total = (double)u * row_total; s_winner = -1; }
    } else if (wave == 0) {
        // pick the chunk of row tau that holds t = u * (total weight): 64 chunk sums at a time, scanned in order
        const double total = mode == 1 ? S[gb] : S[tau];
        const double t = (double)u * total;
        const float2 *pp = pb + (size_t)tau * nchunks;
        int chunk = -1, last_nonzero = 0;
        double carry = 0.0, t_in = INFINITY;
        for (int c0 = 0; c0 < nchunks && chunk < 0; c0 += 64) {
            const int c = c0 + lane;
            const double v = c < nchunks ? (double)(keep ? kept[tau * nchunks + c] : pp[c].x) : 0.0;
            const double inc = wave_inclusive_scan_double(v) + carry;
            const unsigned long long nz = __ballot(v > 0.0), hit = __ballot(c < nchunks && inc > t);
            if (nz) last_nonzero = c0 + 63 - __clzll((long long)nz);
            if (hit) {
                const int first = __ffsll((long long)hit) - 1;
                chunk = c0 + first;
                t_in = t - read_lane_double(inc - v, first);
            }
            carry = read_lane_double(inc, 63);
        }
        if (lane == 0) {
            s_chunk = chunk < 0 ? last_nonzero : chunk;      // rounding pushed t past the end: the last chunk with weight
            s_t = t_in;
            s_winner = -1;
        }
    }
    __syncthreads();

    // walk: the chosen chunk, or (mode 2) every chunk in turn until the one whose running sum passes t.
    // Inside that chunk the token lies with the last thread whose preceding sum does not exceed t (one
    // thread exactly, whatever the rounding of the scan); if rounding left t at or beyond the chunk's own
    // total, that thread is the last one with weight and the token its last one with weight.
    int c = mode == 2 ? 0 : s_chunk;
    double t_in = mode == 2 ? s_total : s_t;
    int last_positive = -1;
    for (;;) {
        float mine; double below, total;
        scan_chunk(c, residual, mine, below, total);
        const int start = c * kChunk + tid * kPerThread;
#pragma unroll
        for (int e = 0; e < kPerThread; ++e)
            if (wgt[e] > 0.f) last_positive = start + e;
        if (mode != 2 || t_in < total || c + 1 >= nchunks) {
            // the last thread with weight whose preceding sum does not exceed t: per wave by a ballot, then the last
            // wave that has one (hundreds of atomic operations on one LDS word took microseconds here)
            const unsigned long long cands = __ballot(mine > 0.f && below <= t_in);
            if (lane == 0) wave_cand[wave] = cands ? wave * kWave + 63 - __clzll((long long)cands) : -1;
            __syncthreads();
            int cand = -1;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) cand = wave_cand[w] > cand ? wave_cand[w] : cand;
            if (tid == cand) {
                double run = below;
                int y = -1, lastpos = 0;
#pragma unroll
                for (int e = 0; e < kPerThread; ++e) {
                    run += (double)wgt[e];
                    if (wgt[e] > 0.f) lastpos = e;
                    if (y < 0 && run > t_in) y = e;
                }
                s_winner = start + (y < 0 ? lastpos : y);
            }
            break;
        }
        t_in -= total;
        ++c;
    }
    __syncthreads();
    if (s_winner < 0) {
        // no weight at all in the chunk the walk ended in: the last token of positive weight seen before it
        atomicMax(&s_winner, last_positive);
        __syncthreads();
    }
    if (tid == 0) next_token[b] = s_winner < 0 ? 0 : s_winner;
}

}  // namespace sv
