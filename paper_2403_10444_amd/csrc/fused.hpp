// Fused path: ONE launch, every logit read from HBM once.
//
// The method needs two sweeps over each (target row i, draft row i) pair: the residual mass
// S_i = sum_x max(w_i p_i(x) - q_i(x), 0) of Alg. 2 depends on the rows' normalisers and on
// w_i, which depends on the normalisers of all earlier rows of the sequence.  Here the second
// sweep never touches memory: a workgroup owns kChunk logits of a row pair, turns them into
// exp2(y - shift) with a per-thread shift during the first sweep, KEEPS those 2 x 32 values
// per thread in registers, publishes its partial normalisers, waits until the rows it depends
// on are complete, and then forms its share of S_i from the registers.
//
// Workgroup g owns unit g in the order (sequence, position, chunk).  The hardware starts
// workgroups in index order (round-robin over the 8 XCDs, in order within each), so a unit
// only ever waits for units that started before it or that belong to its own row, and a row's
// units (at most 128) are far fewer than the workgroups one XCD holds: the grid always
// drains.  Every wait is also bounded by a spin limit; running into it sets the workspace's
// error word and goes on instead of hanging.
//
// Cross-workgroup protocol (all counters live in the workspace and are zero between calls):
//   rowcnt[b, i]   units of row i that have published their first-sweep partials; the unit
//                  that completes the count reduces them to the row's log2-normalisers, adds
//                  the ratio of draft token i+1, stores a RowRec and sets rowflag[b, i]
//   rowflag[b, i]  polled by the units of rows >= i of sequence b
//   seqcnt[b]      units of sequence b that are done; the unit that completes the count runs
//                  the accept tests and the inverse-CDF draw, writes tau and Y, and clears the
//                  sequence's counters
#pragma once

#include "common.hpp"

namespace sv {

// Word 0 of an initialised workspace: a constant mixed with the shape it was initialised for.
__host__ __device__ inline int workspace_magic(int B, int gamma, int V)
{
    return (int)(0x53564b31u ^ ((unsigned)B * 2654435761u + (unsigned)gamma * 40503u + (unsigned)V * 2246822519u));
}

enum HeaderWord : int { kHdrMagic = 0, kHdrError = 1, kHdrWords = 64 };

struct RowRec {
    double L_p;          // log2-normaliser of the target row
    double L_q;          // log2-normaliser of the draft row (0 for the last target row)
    double log2r_next;   // log2 [p_i(X_{i+1}) / q_i(X_{i+1})]  (0 for the last target row)
    double M_p;          // maximum of the target row's partial shifts
};

struct FusedParams {
    const void *target, *draft;
    const int32_t *tokens;
    const float *uniforms;
    int B, gamma, V;
    float k;              // float(log2(e) / T): the factor the sweeps multiply logits by
    double kd;            // log2(e) / T in double
    double k_eps;         // kd / k - 1: what rounding k to float left out (|k_eps| <= 2^-24)
    int algo;
    int nu;               // units per row pair = ceil(V / kChunk)
    int nuf;              // units of the last target row (two chunks each) = ceil(nu / 2)
    int units_per_seq;    // gamma * nu + nuf
    int nw;               // partial slots per row = 8 * nuf (one per wave chunk)
    int spin_limit;
    int magic;            // workspace_magic(B, gamma, V)
    int *header, *rowcnt, *rowflag, *seqcnt;
    RowRec *rowrec;
    unsigned long long *pstats;   // [B, gamma+1, nw] packed (shift, sum) of target wave chunks
    unsigned long long *qstats;   // [B, gamma,   nw] same for the draft rows
    float *spart;                 // [B, gamma, nw] residual partial sums
    float *rpart;                 // [B, gamma, nw] greedy only: partial sums of max(q - w p, 0)
    int32_t *accept_len, *next_token;
    float *debug_out;
    long long *prof;              // NULL, or [units, 8] timestamps (100 MHz ticks) for tuning
};

// ---- accessors for data that other workgroups (on any XCD) write or read.
// Everything that crosses workgroups is written and read with agent-scope atomic accesses, which
// go through to device memory instead of living in one XCD's L2.  Ordering between a payload and
// the flag or counter that announces it is kept by waiting for the payload's stores to complete
// (`drain_stores`) before the announcing access is issued, and by issuing the payload's loads only
// after the announcement was observed.  This avoids agent-scope release/acquire fences, which on
// this part write back and invalidate a whole L2 and cost more than the rest of the kernel.
__device__ __forceinline__ void drain_stores()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);            // vmcnt(0) expcnt(0) lgkmcnt(0): all stores of this wave are done
}
__device__ __forceinline__ int ld_flag(const int *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_flag(int *p, int v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ int add_count(int *p, int v) { return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float ld_f32(const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_f32(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ unsigned long long ld_u64(const unsigned long long *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_u64(unsigned long long *p, unsigned long long v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ double ld_f64(const double *p)
{
    return __longlong_as_double((long long)ld_u64(reinterpret_cast<const unsigned long long *>(p)));
}
__device__ __forceinline__ void st_f64(double *p, double v)
{
    st_u64(reinterpret_cast<unsigned long long *>(p), (unsigned long long)__double_as_longlong(v));
}
__device__ __forceinline__ unsigned long long pack_stat(float shift, float sum)
{
    return ((unsigned long long)__float_as_uint(sum) << 32) | (unsigned long long)__float_as_uint(shift);
}
__device__ __forceinline__ float stat_shift(unsigned long long v) { return __uint_as_float((unsigned)(v & 0xffffffffull)); }
__device__ __forceinline__ float stat_sum(unsigned long long v) { return __uint_as_float((unsigned)(v >> 32)); }

// First sweep over the 32 logits a thread holds of one row: x[j] becomes exp2(x[j] * k - shift)
// with shift = k * (largest of the 32), `mk` is that shift (-inf when all 32 lie beyond the row)
// and `s` the sum of the 32 exponentials.
__device__ __forceinline__ void exp_sum(float (&x)[kPerThread], float k, float &shift, float &mk, float &s)
{
    float m = x[0];
#pragma unroll
    for (int j = 1; j < kPerThread; ++j) m = fmaxf(m, x[j]);
    mk = m * k;
    shift = m > -INFINITY ? mk : 0.f;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};     // four partial sums: shorter chains, smaller rounding error
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
        x[j] = fast_exp2(__builtin_fmaf(x[j], k, -shift));
        acc[j & 3] += x[j];
    }
    s = (acc[0] + acc[1]) + (acc[2] + acc[3]);
}

// Wave-level combination of the per-thread (shift, sum) pairs: returns the packed partial.
__device__ __forceinline__ unsigned long long wave_stat(float mk, float s)
{
    const float Mw = wave_max(mk);
    const float scale = Mw > -INFINITY ? fast_exp2(mk - Mw) : 0.f;
    const float sw = wave_sum(s * scale);
    return pack_stat(Mw, sw);
}

template <typename T, bool ALIGNED>
__device__ __forceinline__ void load_slice(const T *row, int V, int first, float (&x)[kPerThread])
{
    constexpr int kVec = ElemTraits<T>::kVec;
#pragma unroll
    for (int v = 0; v < kPerThread / kVec; ++v) load_vec<T, ALIGNED>(row, V, first + v * 64 * kVec, x + v * kVec);
}

// log2-normaliser of a row from its n published partials: L = M + log2 sum_e s_e exp2(m_e - M).
// Workgroup-wide; every thread gets L and M.
__device__ __forceinline__ double reduce_row(const unsigned long long *stats, int n, float *lds_f, double *lds_d, float &M_out)
{
    const int tid = threadIdx.x;
    float m = -INFINITY;
    for (int e = tid; e < n; e += kThreads) m = fmaxf(m, stat_shift(ld_u64(stats + e)));
    const float M = block_max(m, lds_f);
    double z = 0.0;
    for (int e = tid; e < n; e += kThreads) {
        const unsigned long long v = ld_u64(stats + e);
        z += (double)stat_sum(v) * exp2((double)(stat_shift(v) - M));
    }
    z = block_sum_double(z, lds_d);
    M_out = M;
    return (double)M + log2(z);
}

template <typename T, bool ALIGNED, bool GREEDY>
__global__ __launch_bounds__(kThreads) void fused_verify_kernel(const FusedParams P)
{
    constexpr int kVec = ElemTraits<T>::kVec;
    __shared__ float lds_f[kWaves];
    __shared__ double lds_d[kWaves];
    __shared__ int s_int[4];
    __shared__ double s_alpha[2];
    __shared__ double s_S[SV_MAX_GAMMA + 1], s_R[SV_MAX_GAMMA + 1], s_Lp[SV_MAX_GAMMA + 1], s_Lq[SV_MAX_GAMMA + 1],
        s_lr[SV_MAX_GAMMA + 1], s_Mp[SV_MAX_GAMMA + 1], s_lw[SV_MAX_GAMMA + 1];
    __shared__ RowCoef s_rc;
    __shared__ float s_walk[3];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int gamma = P.gamma, V = P.V;
    const float k = P.k;
    const T *target = static_cast<const T *>(P.target);
    const T *draft = static_cast<const T *>(P.draft);

    // ---- the unit of this workgroup.  Workgroups start in the order of their index, so a unit
    // only ever waits for units that started before it or belong to its own row.
    if (__builtin_nontemporal_load(P.header + kHdrMagic) != P.magic) {
        // the workspace was not initialised for this shape: report it through the outputs and leave
        if (blockIdx.x == 0)
            for (int b = tid; b < P.B; b += kThreads) { P.accept_len[b] = -1; P.next_token[b] = -1; }
        return;
    }
    const int ticket = blockIdx.x;
#define SV_STAMP(slot) do { if (P.prof && tid == 0) P.prof[(size_t)blockIdx.x * 8 + (slot)] = wall_clock64(); } while (0)
    SV_STAMP(0);
    const int b = ticket / P.units_per_seq;
    const int r = ticket - b * P.units_per_seq;
    const bool last_row = r >= gamma * P.nu;            // a unit of target row gamma (no draft row)
    const int i = last_row ? gamma : r / P.nu;
    const int c = last_row ? r - gamma * P.nu : r - i * P.nu;
    const size_t trow = (size_t)b * (gamma + 1) + i;    // index of the target row
    const size_t drow = (size_t)b * gamma + i;          // index of the draft row (pair units only)

    // stream A: target row i, chunk c (last row: chunk 2c); stream B: draft row i, chunk c
    // (last row: target row gamma, chunk 2c+1)
    const T *rowA = target + trow * V;
    const T *rowB = last_row ? rowA : draft + drow * V;
    const int chunkA = last_row ? 2 * c : c;
    const int chunkB = last_row ? 2 * c + 1 : c;

    // the two logits of draft token X_{i+1}, needed only by the unit that completes the row
    double ya = 0.0, yb = 0.0;
    if (tid == 0 && !last_row) {
        const int tok = P.tokens[(size_t)b * gamma + i];
        ya = logit_as_double(rowA + tok);
        yb = logit_as_double(rowB + tok);
    }

    float xa[kPerThread], xb[kPerThread];
    load_slice<T, ALIGNED>(rowA, V, chunkA * kChunk + wave * kWaveChunk + lane * kVec, xa);
    load_slice<T, ALIGNED>(rowB, V, chunkB * kChunk + wave * kWaveChunk + lane * kVec, xb);

    // ---- first sweep: exponentials stay in xa / xb
    float shiftA, mkA, sA, shiftB, mkB, sB;
    exp_sum(xa, k, shiftA, mkA, sA);
    exp_sum(xb, k, shiftB, mkB, sB);
    SV_STAMP(1);
    {
        const unsigned long long stA = wave_stat(mkA, sA), stB = wave_stat(mkB, sB);
        if (lane == 0) {
            st_u64(P.pstats + trow * P.nw + chunkA * kWaves + wave, stA);
            if (last_row) st_u64(P.pstats + trow * P.nw + chunkB * kWaves + wave, stB);
            else st_u64(P.qstats + drow * P.nw + chunkB * kWaves + wave, stB);
        }
    }
    drain_stores();
    __syncthreads();
    if (tid == 0) s_int[0] = add_count(P.rowcnt + trow, 1) == (last_row ? P.nuf : P.nu) - 1;
    __syncthreads();
    SV_STAMP(2);
    if (s_int[0]) {
        // this unit completed the row: reduce the partials to the row's normalisers
        float Mp, Mq = 0.f;
        const double Lp = reduce_row(P.pstats + trow * P.nw, (last_row ? 2 * P.nuf : P.nu) * kWaves, lds_f, lds_d, Mp);
        double Lq = 0.0;
        if (!last_row) Lq = reduce_row(P.qstats + drow * P.nw, P.nu * kWaves, lds_f, lds_d, Mq);
        if (tid == 0) {
            RowRec *rec = P.rowrec + trow;
            st_f64(&rec->L_p, Lp);
            st_f64(&rec->L_q, Lq);
            // The sweeps scale logits by the float k; the exact factor is k (1 + k_eps).  To first order
            // in k_eps that moves a row's log2-normaliser by k_eps * (the scaled logit where the mass
            // sits, taken as the row maximum) and a token's scaled logit by k_eps * itself; only the
            // ratio below, whose logs reach hundreds, is sensitive to it.
            const double lp = ya * P.kd - (Lp + P.k_eps * (double)Mp);
            const double lq = yb * P.kd - (Lq + P.k_eps * (double)Mq);
            st_f64(&rec->log2r_next, last_row ? 0.0 : lp - lq);
            st_f64(&rec->M_p, (double)Mp);
            drain_stores();
            st_flag(P.rowflag + trow, 1);
        }
    }

    if (!last_row) {
        // ---- wait for rows 0..i of this sequence, then w_i (Alg. 2: w_i = min(w_{i-1} r_i, 1))
        if (wave == 0) {
            const int base = b * (gamma + 1);
            int spins = 0;
            bool ok;
            for (;;) {
                int f = 1;
                if (lane <= i) f = ld_flag(P.rowflag + base + lane);
                ok = __all(f != 0);
                if (ok || ++spins > P.spin_limit) break;
                __builtin_amdgcn_s_sleep(8);
            }
            if (!ok && lane == 0) atomicOr(P.header + kHdrError, 1);
            double lr = 0.0, Lp = 0.0, Lq = 0.0;
            if (lane <= i) {
                const RowRec *rec = P.rowrec + base + lane;
                lr = ld_f64(&rec->log2r_next);
                if (lane == i) { Lp = ld_f64(&rec->L_p); Lq = ld_f64(&rec->L_q); }
            }
            double log2w = 0.0;
            if (P.algo != kToken) {
                for (int j = 0; j < i; ++j) {
                    log2w += __shfl(lr, j, 64);
                    if (!GREEDY && log2w > 0.0) log2w = 0.0;
                }
                if (GREEDY) log2w = fmin(log2w, 100.0);     // keeps w p finite in float
            }
            if (lane == i) { s_alpha[0] = Lp - log2w; s_alpha[1] = Lq; }
        }
        __syncthreads();
        SV_STAMP(3);

        // ---- second sweep, from registers: w p(x) = xa * cp, q(x) = xb * cq
        const float cp = fast_exp2((float)((double)shiftA - s_alpha[0]));
        const float cq = fast_exp2((float)((double)shiftB - s_alpha[1]));
        float acc = 0.f, rej = 0.f;
#pragma unroll
        for (int j = 0; j < kPerThread; ++j) {
            const float d = __builtin_fmaf(xa[j], cp, -(xb[j] * cq));
            acc += fmaxf(d, 0.f);
            if constexpr (GREEDY) rej += fmaxf(-d, 0.f);
        }
        acc = wave_sum(acc);
        if constexpr (GREEDY) rej = wave_sum(rej);
        if (lane == 0) {
            st_f32(P.spart + drow * P.nw + c * kWaves + wave, acc);
            if constexpr (GREEDY) st_f32(P.rpart + drow * P.nw + c * kWaves + wave, rej);
        }
    }

    // ---- count this unit as done; the unit that completes the sequence finishes it
    SV_STAMP(4);
    drain_stores();
    __syncthreads();
    if (tid == 0) s_int[0] = add_count(P.seqcnt + b, 1) == P.units_per_seq - 1;
    __syncthreads();
    SV_STAMP(5);
    if (!s_int[0]) return;

    const int base = b * (gamma + 1);
    const int n_pair = P.nu * kWaves;                   // partial slots in use per pair row
    for (int j = tid; j <= gamma; j += kThreads) {
        const RowRec *rec = P.rowrec + base + j;
        s_Lp[j] = ld_f64(&rec->L_p); s_Lq[j] = ld_f64(&rec->L_q);
        s_lr[j] = ld_f64(&rec->log2r_next); s_Mp[j] = ld_f64(&rec->M_p);
    }
    // S_i = sum of the row's partials: lanes take entries e = lane, lane+64, ..., then a wave sum
    for (int j = wave; j < gamma; j += kWaves) {
        double acc = 0.0, rej = 0.0;
        for (int e = lane; e < n_pair; e += 64) {
            acc += (double)ld_f32(P.spart + ((size_t)b * gamma + j) * P.nw + e);
            if constexpr (GREEDY) rej += (double)ld_f32(P.rpart + ((size_t)b * gamma + j) * P.nw + e);
        }
        acc = wave_sum_double(acc);
        if constexpr (GREEDY) rej = wave_sum_double(rej);
        if (lane == 0) { s_S[j] = acc; s_R[j] = rej; }
    }
    __syncthreads();

    if (tid == 0) {
        // w_i, then the accept tests eta_i < h_i
        const int algo = P.algo;
        double log2w = 0.0;
        for (int j = 0; j <= gamma; ++j) {
            s_lw[j] = (algo == kToken) ? 0.0 : (GREEDY ? fmin(log2w, 100.0) : log2w);
            log2w += s_lr[j];
            if (!GREEDY && log2w > 0.0) log2w = 0.0;
        }
        int tau = 0;
        const float *eta = P.uniforms + (size_t)b * (gamma + 1);
        for (int j = 0; j <= gamma; ++j) {
            const double w = exp2(s_lw[j]);
            const double S = j < gamma ? s_S[j] : w;      // q_gamma == 0: S_gamma = w_gamma
            double h;
            if (j == 0) h = 1.0;
            else if (algo == kToken) h = exp2(fmin(s_lr[j - 1], 0.0));                       // min(r_j, 1)
            else if (j == gamma) h = fmin(w, 1.0);                                           // h_gamma = w_gamma
            else if (GREEDY) h = s_R[j] > 0.0 ? fmin(S / s_R[j], 1.0) : 1.0;                 // p_remain / p_rej
            else h = s_lw[j] >= 0.0 ? 1.0 : S / (S - expm1(s_lw[j] * 0.69314718055994530942)); // S / (S + 1 - w)
            if (j >= 1) {
                const bool pass = (double)eta[j - 1] < h;
                if (algo == kToken) { if (pass && tau == j - 1) tau = j; }                   // stops at the first failure
                else if (pass) tau = j;                                                      // last passing sub-block
            }
            if (P.debug_out) {
                float *d = P.debug_out + ((size_t)base + j) * 3;
                d[0] = (float)w; d[1] = (float)S; d[2] = (float)h;
            }
        }
        P.accept_len[b] = tau;
        s_int[1] = tau;
        if (tau < gamma) s_rc = make_row_coef(s_Lp[tau] - s_lw[tau], s_Lq[tau]);
    }
    __syncthreads();
    const int tau = s_int[1];
    SV_STAMP(6);

    // ---- inverse-CDF draw of Y, first over the row's wave-chunk partials (wave 0)
    if (wave == 0) {
        const float u = P.uniforms[(size_t)b * (gamma + 1) + gamma];
        const float Mrow = (float)s_Mp[tau];
        const unsigned long long *st = P.pstats + ((size_t)base + tau) * P.nw;
        const float *sp = P.spart + ((size_t)b * gamma + (tau < gamma ? tau : 0)) * P.nw;
        int mode = tau < gamma ? 0 : 1;                 // 0: residual weights; 1: p_tau itself
        int slot = -1, last_nonzero = 0;
        double t_in = 0.0;
        for (int attempt = 0; attempt < 2 && slot < 0; ++attempt) {
            const int n = mode == 0 ? n_pair : (tau < gamma ? n_pair : 2 * P.nuf * kWaves);
            // pass 0: total; pass 1: locate t = u * total
            double total = 0.0, t = 0.0;
            for (int pass = 0; pass < 2; ++pass) {
                double carry = 0.0;
                for (int e0 = 0; e0 < n; e0 += 64) {
                    const int e = e0 + lane;
                    double part = 0.0;
                    if (e < n) {
                        if (mode == 0) part = (double)ld_f32(sp + e);
                        else {
                            const unsigned long long v = ld_u64(st + e);
                            const float sh = stat_shift(v);
                            part = sh > -INFINITY ? (double)(stat_sum(v) * fast_exp2(sh - Mrow)) : 0.0;
                        }
                    }
                    double inc = part;
#pragma unroll
                    for (int off = 1; off < 64; off <<= 1) {
                        const double up = __shfl_up(inc, off, 64);
                        if (lane >= off) inc += up;
                    }
                    inc += carry;
                    if (pass == 1 && slot < 0) {
                        const unsigned long long hit = __ballot(e < n && inc > t);
                        const unsigned long long nz = __ballot(e < n && part > 0.0);
                        if (nz) last_nonzero = e0 + 63 - __clzll(nz);
                        if (hit) {
                            const int first = __ffsll((long long)hit) - 1;
                            slot = e0 + first;
                            const double before = __shfl(inc - part, first, 64);
                            t_in = t - before;
                        }
                    }
                    carry = __shfl(inc, 63, 64);
                }
                if (pass == 0) { total = carry; t = (double)u * total; }
            }
            if (slot < 0) {
                if (mode == 0 && !(total > 0.0)) { mode = 1; continue; }   // no residual mass: draw from p_tau
                slot = last_nonzero; t_in = INFINITY;                      // rounding pushed t past the end
            }
        }
        if (lane == 0) {
            s_int[2] = slot; s_int[3] = mode;
            const unsigned long long v = ld_u64(st + slot);
            s_walk[0] = mode == 0 ? (float)(t_in / (double)s_rc.cq) : (float)t_in;
            s_walk[1] = stat_shift(v);
            s_walk[2] = fast_exp2(stat_shift(v) - Mrow);
        }
    }
    __syncthreads();
    {
        const int slot = s_int[2];
        const bool residual = s_int[3] == 0;
        const T *prow = target + ((size_t)base + tau) * V;
        const T *qrow = draft + ((size_t)b * gamma + (tau < gamma ? tau : 0)) * V;
        const RowCoef rc = s_rc;
        const int y = walk_range<T, ALIGNED>(prow, qrow, V, slot * kWaveChunk, 1, k, residual, rc,
                                             s_walk[1], s_walk[2], s_walk[0], lds_f, s_int);
        if (tid == 0) P.next_token[b] = y;
    }

    // ---- leave the sequence's counters zero for the next call
    for (int j = tid; j <= gamma; j += kThreads) { P.rowcnt[base + j] = 0; P.rowflag[base + j] = 0; }
    if (tid == 0) P.seqcnt[b] = 0;
    SV_STAMP(7);
#undef SV_STAMP
}

// Clears the control words of a workspace and marks it initialised.
__global__ void workspace_init_kernel(int *words, size_t n, int magic)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < n) words[idx] = idx == kHdrMagic ? magic : 0;
}

}  // namespace sv
