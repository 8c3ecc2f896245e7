// Small sequences: ONE workgroup per sequence, nothing between workgroups.
//
// Where the 2 gamma + 1 rows of a sequence fit into LDS together ((2 gamma + 1) V <= kTinyMaxFloats logits: a few
// positions over a vocabulary of a thousand tokens, the shape of the worked example of Sec. 2 scaled up), the whole
// of Alg. 1 / Alg. 2 / Alg. 4 for that sequence is a handful of passes over LDS by one workgroup of sixteen waves, with
// barriers where the large kernel has words that travel through device memory: a call is one read of the logits and
// seven barriers long instead of six dependent round trips through memory.  The arithmetic is the large kernel's:
// base-2 exponentials in float against an integer shift per row, sums of them in double, log2 r_i, w_i, h_i in double,
// residual terms in float with the larger of the two row factors taken out, the draw of Y in vocabulary order.
#pragma once

#include "fused.hpp"

namespace sv {

constexpr int kTinyThreads = 1024, kTinyWaves = kTinyThreads / kWave;
constexpr int kTinyMaxFloats = 14336;               // logits of one sequence that the workgroup keeps in LDS (56 KB)
constexpr int kTinyMaxRows = 2 * SV_MAX_GAMMA + 1;
constexpr int kTinyMaxChunks = (kTinyMaxFloats / 3 + kWave - 1) / kWave;     // 64-token chunks of the widest row (gamma = 1)

// The sum over the wave in double, through DPP (no trip through LDS per step).
__device__ __forceinline__ double tiny_wave_sum(double v)
{
    double first, second;
    halves_sum_f64(v, first, second);
    return first + second;
}

// What turns a row pair's exponentials xa = 2^(y_p - shift_p), xb = 2^(y_q - shift_q) into residual terms
// max(w p - q, 0): with cp = 2^(shift_p - L_p + log2 w) and cq = 2^(shift_q - L_q) the term is max(xa cp - xb cq, 0);
// the larger factor is taken out (`scale`), so the other one, `f`, is a ratio <= 1 rounded once from double and
// every term lies in [0, 1].  A row without a draft row (the draw from p itself): xb == nullptr, the term is xa.
struct TinyCoef {
    float f;
    bool q_units;          // terms in units of cq: max(xa f - xb, 0); else in units of cp: max(xa - xb f, 0)
    double scale;
};
__device__ __forceinline__ TinyCoef tiny_coef(double log2_cp, double log2_cq)
{
    TinyCoef c;
    const double d = log2_cp - log2_cq;
    c.q_units = d <= 0.0;
    c.f = (float)exp2_precise(c.q_units ? d : -d);
    c.scale = exp2_precise(c.q_units ? log2_cq : log2_cp);
    return c;
}
__device__ __forceinline__ float tiny_term(const float *xa, const float *xb, int x, const TinyCoef &c)
{
    if (!xb) return xa[x];
    return c.q_units ? __builtin_amdgcn_fmed3f(__builtin_fmaf(xa[x], c.f, -xb[x]), 0.f, 1.f)
                     : __builtin_amdgcn_fmed3f(__builtin_fmaf(xb[x], -c.f, xa[x]), 0.f, 1.f);
}

// Uses of FusedParams: the inputs, shape, strides, k, kd, k_eps, algo, magic, header and the outputs; inv_wpr holds
// floor(2^32 / V) + 1 (V > 1), so that e / V = mulhi(e, .) for every element index e that occurs.
template <typename T>
__global__ __launch_bounds__(kTinyThreads)
void tiny_verify_kernel(const FusedParams P)
{
    __shared__ float x[kTinyMaxFloats];             // row r at r * V: target rows 0 .. gb, then draft rows 0 .. gb - 1
    __shared__ double L[kTinyMaxRows];              // log2-normaliser of each row
    __shared__ float Mk[kTinyMaxRows];              // k * the row's largest logit
    __shared__ float shift[kTinyMaxRows];           // the row's integer shift: after the first pass x holds 2^(y - shift)
    __shared__ float ytok[2][SV_MAX_GAMMA];         // the drafted token's target / draft logit per position
    __shared__ double lw[SV_MAX_GAMMA + 1];         // log2 w_i (Alg. 1: 0 while every test up to i has passed)
    __shared__ double S[SV_MAX_GAMMA];              // S_i
    __shared__ float eta_s[SV_MAX_GAMMA + 1];       // the sequence's uniforms
    __shared__ double chunk_total[kTinyMaxChunks];  // the draw: the weights' sums per 64 tokens
    __shared__ int draw_row[2];                     // the draw: tau; whether the weights are the residual's (1) or p's (0)
    static_assert(kTinyMaxFloats % kTinyThreads == 0, "whole rounds of the workgroup");

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b = blockIdx.x, gamma = P.gamma, V = P.V;
    const float k = P.k;
    long long *stamps = nullptr;
#ifdef SV_PROFILE
    if (P.prof && b == 0) stamps = P.prof;          // tuning builds: timestamps of the first sequence's workgroup
#endif
    SV_STAMP(0);
    int gb = gamma;
    if (P.draft_lens) { gb = load_uniform(P.draft_lens + b); gb = gb < 1 ? 1 : gb > gamma ? gamma : gb; }
    const int rows = 2 * gb + 1;
    const size_t seq_d = (size_t)b * gamma, seq_u = (size_t)b * (gamma + 1);
    const T *const target = static_cast<const T *>(P.target) + seq_u * P.tstride;
    const T *const draft = static_cast<const T *>(P.draft) + seq_d * P.dstride;

    // ---- everything the sequence needs from memory, asked for at once (the kernel is as long as its dependent round
    // trips to memory, and this is the only one).  The logits go into LDS as floats: thread t takes elements
    // t, t + 1024, ... of the rows laid end to end (an element beyond the end is read as the last one and not stored).
    {
        constexpr int kPer = kTinyMaxFloats / kTinyThreads;
        const int total = rows * V;
        const int tok = P.tokens[seq_d + (tid < gb ? tid : gb - 1)];
        const float eta = P.uniforms[seq_u + (tid <= gb ? tid : gb)];
        const int magic_word = load_uniform(P.header + kHdrMagic);
        float v[kPer];
        if (P.tstride == (size_t)V && P.dstride == (size_t)V) {
            // dense rows: the sequence's target rows are one stretch of memory, its draft rows another
            const int n_target = (gb + 1) * V;
#pragma unroll
            for (int n = 0; n < kPer; ++n) {
                const int e = min(tid + n * kTinyThreads, total - 1);
                v[n] = logit_as_float(e < n_target ? target + e : draft + (e - n_target));
            }
        } else {
#pragma unroll
            for (int n = 0; n < kPer; ++n) {
                const int e = min(tid + n * kTinyThreads, total - 1);
                const int r = V == 1 ? e : (int)__umulhi((unsigned)e, P.inv_wpr);       // e / V
                const int j = e - r * V;
                const T *row = r <= gb ? target + (size_t)r * P.tstride : draft + (size_t)(r - gb - 1) * P.dstride;
                v[n] = logit_as_float(row + j);
            }
        }
        if (magic_word != P.magic) {
            // the workspace was not initialised for this shape: this kernel needs none of it, but the contract is one
            if (tid == 0) { P.accept_len[b] = -1; P.next_token[b] = -1; }
            return;
        }
#pragma unroll
        for (int n = 0; n < kPer; ++n) {
            const int e = tid + n * kTinyThreads;
            if (e < total) x[e] = v[n];
        }
        if (tid <= gb) eta_s[tid] = eta;
        SV_STAMP(1);
        __syncthreads();
        // the drafted tokens' logits, before the rows become exponentials
        if (tid < gb) {
            ytok[0][tid] = x[tid * V + tok];
            ytok[1][tid] = x[(gb + 1 + tid) * V + tok];
        }
    }
    __syncthreads();
    SV_STAMP(2);
    // ---- per row (one wave each): largest logit, exponentials against the integer shift (kept in place), their sum
    for (int r = wave; r < rows; r += kTinyWaves) {
        float *xr = x + r * V;
        float m = -INFINITY;
#pragma unroll 4
        for (int j = lane; j < V; j += kWave) m = fmaxf(m, xr[j]);
        const float Mw = wave_max(m * k);
        const float sh = shift_of(Mw);
        double acc = 0.0;
#pragma unroll 4
        for (int j = lane; j < V; j += kWave) {
            const float e = fast_exp2(__builtin_fmaf(xr[j], k, -sh));
            xr[j] = e;
            acc += (double)e;
        }
        const double z = tiny_wave_sum(acc);
        if (lane == 0) { L[r] = (double)sh + log2_precise(z); Mk[r] = Mw; shift[r] = sh; }
    }
    __syncthreads();
    SV_STAMP(3);
    // ---- log2 r_{i+1} (lane i) and the weights: as the large kernel forms them for calls of one resident set
    u64 ratio_word = 0;
    if (wave == 0) {
        if (lane < gb) {
            const double lp = (double)ytok[0][lane] * P.kd - (L[lane] + P.k_eps * (double)Mk[lane]);
            const double lq = (double)ytok[1][lane] * P.kd - (L[gb + 1 + lane] + P.k_eps * (double)Mk[gb + 1 + lane]);
            const double lr = fmax(lp - lq, kLog2RatioFloor);
            const float eta = eta_s[lane];                                                 // eta_{i+1}
            ratio_word = pack_ratio(lr, P.algo == kToken && (double)eta < exp2_precise(fmin(lr, 0.0)));
        }
        const double lw_next = weights_from_ratios(P.algo, ratio_word, gb);                // lane i: log2 w_{i+1}
        if (lane < gb) lw[lane + 1] = lw_next;
        if (lane == 0) lw[0] = 0.0;
    }
    __syncthreads();
    SV_STAMP(4);
    // ---- S_i = sum_x max(w_i p_i(x) - q_i(x), 0), one wave per position
    for (int i = wave; i < gb; i += kTinyWaves) {
        double log2w = lw[i];
        if (P.algo == kToken) log2w = 0.0;                          // the residual of token verification is p - q
        if (P.algo == kGreedy) log2w = fmin(log2w, 100.0);
        const TinyCoef c = tiny_coef((double)shift[i] - (L[i] - log2w), (double)shift[gb + 1 + i] - L[gb + 1 + i]);
        const float *xa = x + i * V, *xb = x + (gb + 1 + i) * V;
        double acc = 0.0;
#pragma unroll 4
        for (int j = lane; j < V; j += kWave) acc += (double)tiny_term(xa, xb, j, c);
        const double s = tiny_wave_sum(acc) * c.scale;
        if (lane == 0) S[i] = s;
    }
    __syncthreads();
    SV_STAMP(5);

    // ---- the accept tests (first wave; lane l: position j = l + 1), tau
    const bool token_algo = P.algo == kToken;
    if (wave == 0) {
        const int j = lane + 1;
        double lw_j = j <= gb ? lw[j] : 0.0;
        if (P.algo == kGreedy) lw_j = fmin(lw_j, 100.0);
        if (token_algo) lw_j = 0.0;
        bool pass = false;
        if (j <= gb) {
            const float eta = eta_s[lane];
            const double w_j = exp2_precise(lw_j);
            const double S_j = j < gb ? S[j] : w_j;                     // q_gamma == 0: S_gamma = w_gamma
            double h;
            if (token_algo) h = exp2_precise(fmin(unpack_ratio(ratio_word), 0.0));             // min(r_j, 1)
            else if (j == gb) h = fmin(w_j, 1.0);
            else h = lw_j >= 0.0 ? 1.0 : S_j / (S_j + one_minus_exp2(fmin(lw_j, 0.0)));        // (Alg. 4: the same number, see AcceptTest)
            pass = token_algo ? ratio_passes(ratio_word) : (double)eta < h;
            if (P.debug_out) {
                float *d = P.debug_out + (seq_u + j) * 3;
                d[0] = (float)w_j; d[1] = (float)S_j; d[2] = (float)h;
            }
        }
        if (lane == 0 && P.debug_out) {
            float *d = P.debug_out + seq_u * 3;
            d[0] = 1.f; d[1] = (float)S[0]; d[2] = 1.f;
        }
        const u64 passed = __ballot(pass);
        int tau;
        if (token_algo) { tau = __ffsll((long long)~passed) - 1; if (tau < 0 || tau > gb) tau = gb; }   // leading run of passes
        else tau = passed ? 64 - __clzll((long long)passed) : 0;                                        // last passing sub-block
        if (lane == 0) {
            P.accept_len[b] = tau;
            draw_row[0] = tau;
            draw_row[1] = tau < gb && S[tau < gb ? tau : 0] > 0.0 ? 1 : 0;     // a residual without mass: Y comes from p_tau
        }
    }
    __syncthreads();
    SV_STAMP(6);

    // ---- Y: first token whose running weight exceeds u * total, in vocabulary order.  tau < gb: the residual of row
    // pair tau (p_tau itself if the residual has no mass); tau = gb: p_gb.  First the weights' sums per 64 tokens
    // (all waves), then the first wave finds the chunk and the token in it.
    const int tau = draw_row[0];
    const float *xa = x + tau * V;
    const float *xb = draw_row[1] ? x + (gb + 1 + tau) * V : nullptr;
    TinyCoef c = {1.f, true, 1.0};
    if (xb) {
        double log2w = lw[tau];
        if (token_algo) log2w = 0.0;
        if (P.algo == kGreedy) log2w = fmin(log2w, 100.0);
        c = tiny_coef((double)shift[tau] - (L[tau] - log2w), (double)shift[gb + 1 + tau] - L[gb + 1 + tau]);
    }
    const int chunks = (V + kWave - 1) / kWave;
    for (int ch = wave; ch < chunks; ch += kTinyWaves) {
        const int e = ch * kWave + lane;
        const double s = tiny_wave_sum(e < V ? (double)tiny_term(xa, xb, e, c) : 0.0);
        if (lane == 0) chunk_total[ch] = s;
    }
    __syncthreads();
    if (wave != 0) return;
    SV_STAMP(7);
    double total = 0.0;
    for (int c0 = 0; c0 < chunks; c0 += kWave) total += tiny_wave_sum(c0 + lane < chunks ? chunk_total[c0 + lane] : 0.0);
    const double t = (double)eta_s[gb] * total;
    // the chunk: the first whose running sum exceeds t (rounding may leave none: then the last with any weight)
    int chunk = -1, last_chunk = 0;
    double before = 0.0;
    for (int c0 = 0; c0 < chunks && chunk < 0; c0 += kWave) {
        const double mine = c0 + lane < chunks ? chunk_total[c0 + lane] : 0.0;
        const double inc = wave_scan(mine) + before;
        const u64 hit = __ballot(inc > t), nz = __ballot(mine > 0.0);
        if (nz) last_chunk = c0 + 63 - __clzll((long long)nz);
        if (hit) {
            const int first = __ffsll((long long)hit) - 1;
            chunk = c0 + first;
            before = read_lane_double(inc - mine, first);
        } else {
            before = read_lane_double(inc, kWave - 1);
        }
    }
    double t_in = t - before;
    if (chunk < 0) { chunk = last_chunk; t_in = INFINITY; }
    // the token in the chunk
    const int e = chunk * kWave + lane;
    const double wgt = e < V ? (double)tiny_term(xa, xb, e, c) : 0.0;
    const double inc = wave_scan(wgt);
    const u64 hit = __ballot(inc > t_in), nz = __ballot(wgt > 0.0);
    int y = hit ? __ffsll((long long)hit) - 1 : nz ? 63 - __clzll((long long)nz) : 0;
    y += chunk * kWave;
    if (lane == 0) P.next_token[b] = y;
    SV_STAMP(8);
}

}  // namespace sv
