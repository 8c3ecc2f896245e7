// Fused path: ONE launch, every logit read from HBM once.
//
// The method needs two sweeps over each (target row i, draft row i) pair: the residual mass
// S_i = sum_x max(w_i p_i(x) - q_i(x), 0) of Alg. 2 depends on the rows' normalisers and on
// w_i, which depends on the normalisers of all earlier rows of the sequence.  Here the second
// sweep never touches memory.  The kernel is a grid of independent, persistent WAVEFRONTS
// (workgroups of 64 threads; no LDS, no workgroup barrier).  A *unit* is 2048 contiguous logits
// of a row pair (or two such chunks of the last target row, which has no draft row).  A wave
//   1. unpacks its unit's 2 x 2048 logits (32 + 32 per lane) and at once issues the loads of its
//      NEXT unit into the freed registers, so that HBM stays busy during everything below,
//   2. turns the logits into exp2(y - shift) with per-lane shifts and KEEPS those 2 x 32 floats
//      per lane in registers; publishes the unit's partial normalisers (shift, sum) as two words,
//   3. waits for the words of the other units of its row, derives L_p and L_q, and, with the
//      ratios of the earlier rows (fetched a round ago), w_i (Alg. 2: w_i = min(w_{i-1} r_i, 1)),
//   4. forms its share of S_i from the registers, stores it, counts itself done, and goes on.
// Wave g handles units g, g+G, g+2G, ... where G is the number of waves the device keeps
// resident.  Units are ordered position-major inside groups of sequences (all row pairs of
// position 0, then position 1, ..., then the last target rows), so that the ratios of earlier
// positions were published a whole round before they are needed and a unit only ever waits for
// the other units of its own row.  A wave that has no unit left turns to whole sequences: it
// waits until a sequence's row pairs are counted done and runs the accept tests and the
// inverse-CDF draw.
//
// Everything that crosses waves is a self-announcing word: it is zero between calls and
// non-zero once written (a packed (shift, sum) pair always has a non-zero sum or a -inf shift;
// ratio words get their lowest mantissa bit set).  Words are written and read with agent-scope
// atomic accesses, which go through to device memory instead of living in one XCD's L2; no
// agent-scope fence is needed (on this part such a fence writes back / invalidates a whole L2
// and cost more than the rest of the kernel).  Where a counter announces other stores, the
// wave first waits for those stores to complete.
//
// Progress: a unit waits only for units of its own row (waves next to its own, same round) and
// of earlier rows of its sequence (earlier in the unit order), and publishing never waits, so by
// induction over the unit index every word gets written as long as all G waves are resident (G
// is taken from the occupancy query).  Every wait is also bounded by a spin limit; running into
// it sets the workspace's error word and goes on instead of hanging.
#pragma once

#include "common.hpp"

namespace sv {

constexpr int kWave = 64;
constexpr int kMaxUnitsPerRow = 512;     // wave chunks per row the fused kernel takes (V <= 1 Mi logits)

// Word 0 of an initialised workspace: a constant mixed with the shape it was initialised for.
__host__ __device__ inline int workspace_magic(int B, int gamma, int V)
{
    return (int)(0x53564b33u ^ ((unsigned)B * 2654435761u + (unsigned)gamma * 40503u + (unsigned)V * 2246822519u));
}

enum HeaderWord : int { kHdrMagic = 0, kHdrError = 1, kHdrWords = 64 };

typedef unsigned long long u64;

struct FusedParams {
    const void *target, *draft;
    const int32_t *tokens;
    const float *uniforms;
    int B, gamma, V;
    float k;              // float(log2(e) / T): the factor the sweeps multiply logits by
    double kd;            // log2(e) / T in double
    double k_eps;         // kd / k - 1: what rounding k to float left out (|k_eps| <= 2^-24)
    int algo;
    int nu;               // units (wave chunks) per row pair = ceil(V / kWaveChunk)
    int nuf;              // units of the last target row (two wave chunks each) = ceil(nu / 2)
    int units_per_seq;    // gamma * nu + nuf
    int total_units;      // B * units_per_seq
    int group_seqs;       // sequences per group of the unit order
    int n_waves;          // waves launched (all persistent)
    int spin_limit;
    int magic;            // workspace_magic(B, gamma, V)
    int *header;
    int *seqcnt;          // [B, 2]                   row-pair units / last-row units of the sequence that are done
    u64 *ratio;           // [B, gamma]               log2 r_{i+1} as double bits, lowest bit set
    u64 *pstat;           // [B, gamma+1, 2 * nuf]    packed (shift, sum) per wave chunk of a target row
    u64 *qstat;           // [B, gamma, nu]           same for the draft rows
    float *spart;         // [B, gamma, nu]           residual partial sums per wave chunk
    float *rpart;         // [B, gamma, nu]           greedy only: partial sums of max(q - w p, 0)
    int32_t *accept_len, *next_token;
    float *debug_out;
    long long *prof;      // NULL, or [units + B, 8] timestamps (100 MHz ticks) for tuning
};

// ---- agent-scope accessors for words that other waves (on any XCD) write or read
__device__ __forceinline__ void stores_done() { __builtin_amdgcn_s_waitcnt(0); }   // vmcnt(0): this wave's stores are out
__device__ __forceinline__ int ld_i32(const int *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_i32(int *p, int v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float ld_f32(const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_f32(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ u64 ld_u64(const u64 *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_u64(u64 *p, u64 v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ u64 pack_stat(float shift, float sum)
{
    return ((u64)__float_as_uint(sum) << 32) | (u64)__float_as_uint(shift);
}
__device__ __forceinline__ float stat_shift(u64 v) { return __uint_as_float((unsigned)(v & 0xffffffffull)); }
__device__ __forceinline__ float stat_sum(u64 v) { return __uint_as_float((unsigned)(v >> 32)); }
__device__ __forceinline__ u64 pack_ratio(double log2r) { return (u64)__double_as_longlong(log2r) | 1ull; }
__device__ __forceinline__ double unpack_ratio(u64 v) { return __longlong_as_double((long long)v); }

// A word that is zero until its producer has written it.  Gives up after `limit` polls.
__device__ __forceinline__ u64 wait_word(const u64 *p, int limit, bool &gave_up)
{
    u64 v = ld_u64(p);
    int spins = 0;
    while (v == 0) {
        if (++spins > limit) { gave_up = true; break; }
        __builtin_amdgcn_s_sleep(1);
        v = ld_u64(p);
    }
    return v;
}

// A counter that only grows.  Lane 0 polls; every lane gets the verdict.
__device__ __forceinline__ bool wait_count(const int *p, int target, int limit)
{
    int ok = 0;
    if ((threadIdx.x & 63) == 0) {
        int spins = 0;
        for (;;) {
            ok = ld_i32(p) >= target;
            if (ok || ++spins > limit) break;
            __builtin_amdgcn_s_sleep(4);
        }
    }
    return __builtin_amdgcn_readfirstlane(ok) != 0;
}

// log2 of a positive float with an absolute error of a few 1e-8: exponent + log2(mantissa in [1,2)).
__device__ __forceinline__ double log2_precise(float z)
{
    int e;
    const float m = frexpf(z, &e);            // z = m * 2^e, m in [0.5, 1)
    return (double)(e - 1) + (double)__builtin_amdgcn_logf(m * 2.0f);
}

// Running combination of (shift, sum) pairs: sum of exp2 relative to the largest shift so far.
struct StatAcc {
    float m = -INFINITY, z = 0.f;
    __device__ __forceinline__ void add(u64 word)
    {
        const float sh = stat_shift(word), s = stat_sum(word);
        if (sh > m) { z = z * fast_exp2(m - sh) + s; m = sh; }      // exp2(-inf) = 0 covers the first word
        else if (sh > -INFINITY) z += s * fast_exp2(sh - m);
    }
};

// Log2-normaliser of a row from the words of its n wave chunks: every lane polls entries lane,
// lane+64, ... (in that fixed order), then the wave combines.  Returns L; M_out is the largest shift.
__device__ __forceinline__ double row_normaliser(const u64 *words, int n, int limit, bool &gave_up, float &M_out)
{
    const int lane = threadIdx.x & 63;
    StatAcc acc;
    for (int e = lane; e < n; e += kWave) acc.add(wait_word(words + e, limit, gave_up));
    const float M = wave_max(acc.m);
    const float z = wave_sum(acc.m > -INFINITY ? acc.z * fast_exp2(acc.m - M) : 0.f);
    M_out = M;
    return (double)M + log2_precise(z);
}

struct Unit {
    int b, i, c;          // sequence, position, wave chunk (last row: unit index, chunks 2c and 2c+1)
    bool last_row;
};

// Unit order: groups of `group_seqs` sequences; inside a group first the row pairs position-major
// (position, sequence, chunk), then the units of the last target rows (sequence, chunk pair).
__device__ __forceinline__ Unit decode_unit(const FusedParams &P, int u)
{
    Unit U;
    const int per_group = P.group_seqs * P.units_per_seq;
    const int g = u / per_group;
    int r = u - g * per_group;
    const int b0 = g * P.group_seqs;
    const int nb = P.B - b0 < P.group_seqs ? P.B - b0 : P.group_seqs;   // sequences in this group
    const int pairs = P.gamma * nb * P.nu;
    U.last_row = r >= pairs;
    if (!U.last_row) {
        U.i = r / (nb * P.nu);
        r -= U.i * nb * P.nu;
        const int bl = r / P.nu;
        U.b = b0 + bl;
        U.c = r - bl * P.nu;
    } else {
        r -= pairs;
        const int bl = r / P.nuf;
        U.i = P.gamma;
        U.b = b0 + bl;
        U.c = r - bl * P.nuf;
    }
    return U;
}

// The 2 x 32 logits of one lane, as loaded: raw 16-byte vectors on the aligned path.
template <typename T, bool ALIGNED> struct RawSlice;
template <typename T> struct RawSlice<T, true> {
    static constexpr int kNV = kPerThread / ElemTraits<T>::kVec;
    uint4 a[kNV], b[kNV];
};
template <typename T> struct RawSlice<T, false> { };      // the element-wise path loads when it unpacks

template <typename T>
struct Stream {
    const T *rowA, *rowB;
    int firstA, firstB;       // element index of this lane's first vector in each row
};

// Stream A: target row i, wave chunk c (last row: chunk 2c); stream B: draft row i, chunk c
// (last row: target row gamma, chunk 2c+1).  Vector v of a lane starts at first + v * 64 * kVec,
// so one load instruction of the wave covers 1 KB of contiguous memory.
template <typename T>
__device__ __forceinline__ Stream<T> unit_streams(const FusedParams &P, const Unit &U)
{
    constexpr int kVec = ElemTraits<T>::kVec;
    const int lane = threadIdx.x & 63;
    const T *target = static_cast<const T *>(P.target);
    const T *draft = static_cast<const T *>(P.draft);
    Stream<T> S;
    S.rowA = target + ((size_t)U.b * (P.gamma + 1) + U.i) * P.V;
    S.rowB = U.last_row ? S.rowA : draft + ((size_t)U.b * P.gamma + U.i) * P.V;
    S.firstA = (U.last_row ? 2 * U.c : U.c) * kWaveChunk + lane * kVec;
    S.firstB = (U.last_row ? 2 * U.c + 1 : U.c) * kWaveChunk + lane * kVec;
    return S;
}

template <typename T, bool ALIGNED>
__device__ __forceinline__ void issue_loads(const Stream<T> &S, int V, RawSlice<T, ALIGNED> &raw)
{
    if constexpr (ALIGNED) {
        constexpr int kVec = ElemTraits<T>::kVec;
        constexpr int kNV = kPerThread / kVec;
#pragma unroll
        for (int v = 0; v < kNV; ++v) {
            const int ia = S.firstA + v * kWave * kVec, ib = S.firstB + v * kWave * kVec;
            // vectors beyond the row are recognised again when the slice is unpacked; load something valid
            raw.a[v] = *reinterpret_cast<const uint4 *>(S.rowA + (ia < V ? ia : 0));
            raw.b[v] = *reinterpret_cast<const uint4 *>(S.rowB + (ib < V ? ib : 0));
        }
        // the loads must be issued HERE (they are the prefetch that overlaps the work that follows);
        // without this the compiler is free to sink them to their first use
        asm volatile("" ::: "memory");
    }
}

template <typename T>
__device__ __forceinline__ void unpack_vec(const uint4 &v, bool valid, float *out)
{
    constexpr int kVec = ElemTraits<T>::kVec;
    if (!valid) {
#pragma unroll
        for (int e = 0; e < kVec; ++e) out[e] = -INFINITY;
        return;
    }
    if constexpr (kVec == 4) {
        out[0] = __uint_as_float(v.x); out[1] = __uint_as_float(v.y);
        out[2] = __uint_as_float(v.z); out[3] = __uint_as_float(v.w);
    } else {
        out[0] = bf16_lo(v.x); out[1] = bf16_hi(v.x); out[2] = bf16_lo(v.y); out[3] = bf16_hi(v.y);
        out[4] = bf16_lo(v.z); out[5] = bf16_hi(v.z); out[6] = bf16_lo(v.w); out[7] = bf16_hi(v.w);
    }
}

template <typename T, bool ALIGNED>
__device__ __forceinline__ void unpack_slice(const Stream<T> &S, int V, const RawSlice<T, ALIGNED> &raw,
                                             float (&xa)[kPerThread], float (&xb)[kPerThread])
{
    constexpr int kVec = ElemTraits<T>::kVec;
    constexpr int kNV = kPerThread / kVec;
#pragma unroll
    for (int v = 0; v < kNV; ++v) {
        const int ia = S.firstA + v * kWave * kVec, ib = S.firstB + v * kWave * kVec;
        if constexpr (ALIGNED) {
            unpack_vec<T>(raw.a[v], ia < V, xa + v * kVec);
            unpack_vec<T>(raw.b[v], ib < V, xb + v * kVec);
        } else {
            load_vec<T, false>(S.rowA, V, ia, xa + v * kVec);
            load_vec<T, false>(S.rowB, V, ib, xb + v * kVec);
        }
    }
}

// First sweep over the 32 logits a lane holds of one row: x[j] becomes exp2(x[j] * k - shift)
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

// Wave-level combination of the per-lane (shift, sum) pairs.
__device__ __forceinline__ u64 wave_stat(float mk, float s)
{
    const float Mw = wave_max(mk);
    const float scale = Mw > -INFINITY ? fast_exp2(mk - Mw) : 0.f;
    const float sw = wave_sum(s * scale);
    return pack_stat(Mw, sw);
}

// ------------------------------------------------------------------ whole sequences
// Inclusive scan over the 64 lanes; `total` is the wave's sum.  exclusive = inclusive of the lane before.
__device__ __forceinline__ float wave_inclusive_scan(float v, float &exclusive, float &total)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const float up = __shfl_up(v, off, kWave);
        if (lane >= off) v += up;
    }
    const float prev = __shfl_up(v, 1, kWave);
    exclusive = lane ? prev : 0.f;
    total = __shfl(v, kWave - 1, kWave);
    return v;
}

// Accept tests and inverse-CDF draw of one sequence (one wave), once its row pairs are counted done.
template <typename T, bool ALIGNED, bool GREEDY>
__device__ void finalize_sequence(const FusedParams &P, int b)
{
    constexpr int kVec = ElemTraits<T>::kVec;
    constexpr int kNV = kPerThread / kVec;
    const int lane = threadIdx.x & 63;
    const int gamma = P.gamma, V = P.V, nu = P.nu;
    const float k = P.k;
    const T *target = static_cast<const T *>(P.target);
    const T *draft = static_cast<const T *>(P.draft);
    const size_t base = (size_t)b * (gamma + 1);
    bool gave_up = !wait_count(P.seqcnt + 2 * b, gamma * nu, P.spin_limit);

    // Row results live in lane j's registers (gamma <= 64): L_p, L_q, M_p, S, rejected mass, log2 r_{j+1}.
    double my_Lp = 0.0, my_Lq = 0.0, my_S = 0.0, my_R = 0.0, my_lr = 0.0;
    float my_Mp = 0.f;
    for (int j = 0; j < gamma; ++j) {
        float Mp, Mq;
        const double Lp = row_normaliser(P.pstat + (base + j) * 2 * P.nuf, nu, P.spin_limit, gave_up, Mp);
        const double Lq = row_normaliser(P.qstat + ((size_t)b * gamma + j) * nu, nu, P.spin_limit, gave_up, Mq);
        double acc = 0.0, rej = 0.0;
        for (int e = lane; e < nu; e += kWave) {
            acc += (double)ld_f32(P.spart + ((size_t)b * gamma + j) * nu + e);
            if constexpr (GREEDY) rej += (double)ld_f32(P.rpart + ((size_t)b * gamma + j) * nu + e);
        }
        acc = wave_sum_double(acc);
        if constexpr (GREEDY) rej = wave_sum_double(rej);
        if (lane == j) { my_Lp = Lp; my_Lq = Lq; my_Mp = Mp; my_S = acc; my_R = rej; }
    }
    if (lane < gamma) my_lr = unpack_ratio(wait_word(P.ratio + (size_t)b * gamma + lane, P.spin_limit, gave_up));

    // log2 w_j for lane j (Alg. 2: w_j = min(w_{j-1} r_j, 1); Alg. 4 drops the min); lw_last is log2 w_gamma
    double my_lw = 0.0, lw_last = 0.0;
    {
        double cur = 0.0;
        for (int j = 0; j < gamma; ++j) {
            if (lane == j) my_lw = cur;
            cur += __shfl(my_lr, j, kWave);
            if (!GREEDY && cur > 0.0) cur = 0.0;
        }
        lw_last = cur;
        if (P.algo == kToken) { my_lw = 0.0; lw_last = 0.0; }
        if (GREEDY) { my_lw = fmin(my_lw, 100.0); lw_last = fmin(lw_last, 100.0); }
    }

    // accept tests eta_j < h_j: lane l tests position j = l + 1, whose row values sit in lane j
    const float *eta = P.uniforms + (size_t)b * (gamma + 1);
    const int j = lane + 1;
    const double lw_next = __shfl_down(my_lw, 1, kWave);
    const double lw_j = j < gamma ? lw_next : lw_last;
    const double S_row = __shfl_down(my_S, 1, kWave), R_row = __shfl_down(my_R, 1, kWave);
    bool pass = false;
    if (j <= gamma) {
        const double w = exp2(lw_j);
        const double S = j < gamma ? S_row : w;          // q_gamma == 0: S_gamma = w_gamma
        double h;
        if (P.algo == kToken) h = exp2(fmin(my_lr, 0.0));                                  // min(r_j, 1); lane l holds log2 r_{l+1}
        else if (j == gamma) h = fmin(w, 1.0);                                             // h_gamma = w_gamma
        else if (GREEDY) h = R_row > 0.0 ? fmin(S / R_row, 1.0) : 1.0;                     // p_remain / p_rej
        else h = lw_j >= 0.0 ? 1.0 : S / (S - expm1(lw_j * 0.69314718055994530942));       // S / (S + 1 - w)
        pass = (double)eta[j - 1] < h;
        if (P.debug_out) {
            float *d = P.debug_out + (base + j) * 3;
            d[0] = (float)w; d[1] = (float)S; d[2] = (float)h;
        }
    }
    if (lane == 0 && P.debug_out) {
        float *d = P.debug_out + base * 3;
        d[0] = 1.f; d[1] = (float)my_S; d[2] = 1.f;
    }
    const u64 passed = __ballot(pass);
    int tau;
    if (P.algo == kToken) tau = passed == ~0ull ? 64 : __ffsll((long long)~passed) - 1;    // leading run of passes
    else tau = passed ? 64 - __clzll((long long)passed) : 0;                               // last passing sub-block
    if (lane == 0) P.accept_len[b] = tau;

    // ---- inverse-CDF draw of Y: first the wave chunk of row tau that holds t = u * total ...
    const float u = eta[gamma];
    int mode = tau < gamma ? 0 : 1;                     // 0: residual weights; 1: p_tau itself
    float Mrow = 0.f;
    RowCoef rc = {};
    if (tau < gamma) {
        Mrow = __shfl(my_Mp, tau, kWave);
        rc = make_row_coef(__shfl(my_Lp, tau, kWave) - __shfl(my_lw, tau, kWave), __shfl(my_Lq, tau, kWave));
    } else {
        // everything accepted: Y comes from p_gamma, so the last target row must be complete too
        if (!wait_count(P.seqcnt + 2 * b + 1, P.nuf, P.spin_limit)) gave_up = true;
        row_normaliser(P.pstat + (base + gamma) * 2 * P.nuf, 2 * P.nuf, P.spin_limit, gave_up, Mrow);
    }
    const u64 *st = P.pstat + (base + tau) * 2 * P.nuf;
    const float *sp = P.spart + ((size_t)b * gamma + (tau < gamma ? tau : 0)) * nu;
    int slot = -1, last_nonzero = 0;
    double t_in = 0.0;
    for (int attempt = 0; attempt < 2 && slot < 0; ++attempt) {
        const int n = tau < gamma ? nu : 2 * P.nuf;
        double total = 0.0, t = 0.0;
        for (int pass_no = 0; pass_no < 2; ++pass_no) {           // pass 0: total; pass 1: locate t = u * total
            double carry = 0.0;
            for (int e0 = 0; e0 < n; e0 += kWave) {
                const int e = e0 + lane;
                double part = 0.0;
                if (e < n) {
                    if (mode == 0) part = (double)ld_f32(sp + e);
                    else {
                        const u64 v = ld_u64(st + e);
                        const float sh = stat_shift(v);
                        part = sh > -INFINITY ? (double)(stat_sum(v) * fast_exp2(sh - Mrow)) : 0.0;
                    }
                }
                double inc = part;
#pragma unroll
                for (int off = 1; off < kWave; off <<= 1) {
                    const double up = __shfl_up(inc, off, kWave);
                    if (lane >= off) inc += up;
                }
                inc += carry;
                if (pass_no == 1 && slot < 0) {
                    const u64 hit = __ballot(e < n && inc > t);
                    const u64 nz = __ballot(e < n && part > 0.0);
                    if (nz) last_nonzero = e0 + 63 - __clzll((long long)nz);
                    if (hit) {
                        const int first = __ffsll((long long)hit) - 1;
                        slot = e0 + first;
                        t_in = t - __shfl(inc - part, first, kWave);
                    }
                }
                carry = __shfl(inc, kWave - 1, kWave);
            }
            if (pass_no == 0) { total = carry; t = (double)u * total; }
        }
        if (slot < 0) {
            if (mode == 0 && !(total > 0.0)) { mode = 1; continue; }   // no residual mass: draw from p_tau
            slot = last_nonzero; t_in = INFINITY;                      // rounding pushed t past the end
        }
    }
    if (slot < 0) { slot = 0; t_in = INFINITY; }

    // ---- ... then the token inside that chunk: weights recomputed from the logits, walked in
    // vocabulary order (vector, lane, element)
    {
        const T *prow = target + (base + tau) * V;
        const T *qrow = draft + ((size_t)b * gamma + (tau < gamma ? tau : 0)) * V;
        const u64 sv = ld_u64(st + slot);
        const float shift = stat_shift(sv), scale = fast_exp2(shift - Mrow);
        float t = mode == 0 ? (float)(t_in / (double)rc.cq) : (float)t_in;
        const int first = slot * kWaveChunk + lane * kVec;
        int y = -1, last_positive = -1;
#pragma unroll
        for (int v = 0; v < kNV; ++v) {
            const int idx = first + v * kWave * kVec;
            float xp[kVec], xq[kVec], wgt[kVec];
            load_vec<T, ALIGNED>(prow, V, idx, xp);
            if (mode == 0) {
                load_vec<T, ALIGNED>(qrow, V, idx, xq);
#pragma unroll
                for (int e = 0; e < kVec; ++e) wgt[e] = fmaxf(residual_term(xp[e], xq[e], k, rc), 0.f);
            } else {
#pragma unroll
                for (int e = 0; e < kVec; ++e) wgt[e] = fast_exp2(__builtin_fmaf(xp[e], k, -shift)) * scale;
            }
            float mine = 0.f;
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                mine += wgt[e];
                if (wgt[e] > 0.f) last_positive = idx + e;
            }
            float exc, total;
            const float inc = wave_inclusive_scan(mine, exc, total);
            const u64 hit = __ballot(inc > t);
            if (y < 0 && hit) {
                const int first_lane = __ffsll((long long)hit) - 1;
                int cand = -1;
                if (lane == first_lane) {
                    float run = exc;
                    int lastpos = 0;
#pragma unroll
                    for (int e = 0; e < kVec; ++e) {
                        run += wgt[e];
                        if (wgt[e] > 0.f) lastpos = e;
                        if (cand < 0 && run > t) cand = e;
                    }
                    if (cand < 0) cand = lastpos;     // scan and walk rounded differently: last positive weight
                    cand += idx;
                }
                y = __shfl(cand, first_lane, kWave);
            }
            t -= total;
        }
        if (y < 0) {
            // t lies beyond the chunk's recomputed total: the last token of positive weight
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) last_positive = max(last_positive, __shfl_xor(last_positive, off, kWave));
            y = last_positive < 0 ? 0 : last_positive;
        }
        if (lane == 0) P.next_token[b] = y;
    }

    // ---- leave the sequence's words zero for the next call (the last row's units must be through first)
    if (!wait_count(P.seqcnt + 2 * b + 1, P.nuf, P.spin_limit)) gave_up = true;
    if (gave_up && lane == 0) atomicOr(P.header + kHdrError, 1);
    for (int e = lane; e < (gamma + 1) * 2 * P.nuf; e += kWave) st_u64(P.pstat + base * 2 * P.nuf + e, 0);
    for (int e = lane; e < gamma * nu; e += kWave) st_u64(P.qstat + (size_t)b * gamma * nu + e, 0);
    for (int e = lane; e < gamma; e += kWave) st_u64(P.ratio + (size_t)b * gamma + e, 0);
    if (lane < 2) st_i32(P.seqcnt + 2 * b + lane, 0);
}

// ------------------------------------------------------------------ the kernel
template <typename T, bool ALIGNED, bool GREEDY>
__global__ __launch_bounds__(kWave) void fused_verify_kernel(const FusedParams P)
{
    const int lane = threadIdx.x;
    const int gamma = P.gamma, V = P.V, nu = P.nu;
    const float k = P.k;

    if (__builtin_nontemporal_load(P.header + kHdrMagic) != P.magic) {
        // the workspace was not initialised for this shape: report it through the outputs and leave
        if (blockIdx.x == 0)
            for (int b = lane; b < P.B; b += kWave) { P.accept_len[b] = -1; P.next_token[b] = -1; }
        return;
    }

#define SV_STAMP(slot) do { if (P.prof && lane == 0) P.prof[(size_t)u * 8 + (slot)] = wall_clock64(); } while (0)
    int u = blockIdx.x;
    Unit U = decode_unit(P, u);
    Stream<T> S = unit_streams<T>(P, U);
    RawSlice<T, ALIGNED> raw;
    issue_loads<T, ALIGNED>(S, V, raw);
    // lane j < i: log2 r_{j+1} of the earlier rows; lane 0 of a row's first unit: the two logits of
    // draft token X_{i+1}, from which it publishes the row's own ratio
    u64 rt = 1;
    double ya = 0.0, yb = 0.0;
    auto prefetch_scalars = [&](const Unit &W, const Stream<T> &SW, u64 &rt_out, double &ya_out, double &yb_out) {
        rt_out = 1;
        ya_out = yb_out = 0.0;
        if (!W.last_row) {
            if (lane < W.i && P.algo != kToken) rt_out = ld_u64(P.ratio + (size_t)W.b * gamma + lane);
            if (lane == 0 && W.c == 0) {
                const int tok = P.tokens[(size_t)W.b * gamma + W.i];
                ya_out = logit_as_double(SW.rowA + tok);
                yb_out = logit_as_double(SW.rowB + tok);
            }
        }
    };
    prefetch_scalars(U, S, rt, ya, yb);

    for (;;) {
        SV_STAMP(0);
        float xa[kPerThread], xb[kPerThread];
        unpack_slice<T, ALIGNED>(S, V, raw, xa, xb);

        // ---- the next unit's loads go out as soon as the raw registers are free
        const int un = u + P.n_waves;
        const bool has_next = un < P.total_units;
        Unit Un = U;
        Stream<T> Sn = S;
        u64 rt_n = 1;
        double ya_n = 0.0, yb_n = 0.0;
        if (has_next) {
            Un = decode_unit(P, un);
            Sn = unit_streams<T>(P, Un);
            issue_loads<T, ALIGNED>(Sn, V, raw);
            prefetch_scalars(Un, Sn, rt_n, ya_n, yb_n);
        }

        // ---- first sweep: exponentials stay in xa / xb; the unit's two words go out
        float shiftA, mkA, sA, shiftB, mkB, sB;
        exp_sum(xa, k, shiftA, mkA, sA);
        exp_sum(xb, k, shiftB, mkB, sB);
        const size_t trow = (size_t)U.b * (gamma + 1) + U.i, drow = (size_t)U.b * gamma + U.i;
        {
            const u64 stA = wave_stat(mkA, sA), stB = wave_stat(mkB, sB);
            if (lane == 0) {
                st_u64(P.pstat + trow * 2 * P.nuf + (U.last_row ? 2 * U.c : U.c), stA);
                if (U.last_row) st_u64(P.pstat + trow * 2 * P.nuf + 2 * U.c + 1, stB);
                else st_u64(P.qstat + drow * nu + U.c, stB);
            }
        }
        SV_STAMP(1);

        if (!U.last_row) {
            // ---- the words of this row's units give L_p and L_q
            bool gave_up = false;
            float Mp, Mq;
            const double Lp = row_normaliser(P.pstat + trow * 2 * P.nuf, nu, P.spin_limit, gave_up, Mp);
            const double Lq = row_normaliser(P.qstat + drow * nu, nu, P.spin_limit, gave_up, Mq);
            SV_STAMP(2);
            if (lane == 0 && U.c == 0) {
                // log2 r_{i+1} = log2 p_i(X_{i+1}) - log2 q_i(X_{i+1}), published for the later rows.  The sweeps
                // scale logits by the float k; the exact factor is kd = k (1 + k_eps).  To first order that
                // moves a row's log2-normaliser by k_eps * (the scaled logit where the mass sits, taken as the
                // row maximum); only this ratio, whose logs reach hundreds, is sensitive to it.
                const double lp = ya * P.kd - (Lp + P.k_eps * (double)Mp);
                const double lq = yb * P.kd - (Lq + P.k_eps * (double)Mq);
                st_u64(P.ratio + drow, pack_ratio(lp - lq));
            }
            // ---- w_i from the ratios of the earlier rows (Alg. 2: w_i = min(w_{i-1} r_i, 1)); they were
            // fetched a round ago and are polled only if they had not been published by then
            double log2w = 0.0;
            if (P.algo != kToken) {
                if (lane < U.i && rt == 0) rt = wait_word(P.ratio + (size_t)U.b * gamma + lane, P.spin_limit, gave_up);
                for (int j = 0; j < U.i; ++j) {
                    log2w += unpack_ratio(__shfl(rt, j, kWave));
                    if (!GREEDY && log2w > 0.0) log2w = 0.0;
                }
                if (GREEDY) log2w = fmin(log2w, 100.0);         // keeps w p finite in float
            }
            if (gave_up && lane == 0) atomicOr(P.header + kHdrError, 1);
            SV_STAMP(3);

            // ---- second sweep, from registers: w p(x) = xa * cp, q(x) = xb * cq
            const float cp = fast_exp2((float)((double)shiftA - (Lp - log2w)));
            const float cq = fast_exp2((float)((double)shiftB - Lq));
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
                st_f32(P.spart + drow * nu + U.c, acc);
                if constexpr (GREEDY) st_f32(P.rpart + drow * nu + U.c, rej);
            }
            SV_STAMP(4);
        }

        // ---- count this unit as done, after its stores
        if (lane == 0) {
            stores_done();
            __hip_atomic_fetch_add(P.seqcnt + 2 * U.b + (U.last_row ? 1 : 0), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        SV_STAMP(5);
        if (!has_next) break;
        u = un; U = Un; S = Sn; rt = rt_n; ya = ya_n; yb = yb_n;
    }
#undef SV_STAMP

    // ---- no unit left: finish whole sequences.  Waves are dealt sequences from the top index down,
    // because those run out of units first.
    for (int b = P.n_waves - 1 - (int)blockIdx.x; b < P.B; b += P.n_waves) {
        if (P.prof && lane == 0) P.prof[(size_t)P.total_units * 8 + (size_t)b * 8 + 0] = wall_clock64();
        finalize_sequence<T, ALIGNED, GREEDY>(P, b);
        if (P.prof && lane == 0) P.prof[(size_t)P.total_units * 8 + (size_t)b * 8 + 1] = wall_clock64();
    }
}

// Clears the control words of a workspace and marks it initialised.
__global__ void workspace_init_kernel(int *words, size_t n, int magic)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < n) words[idx] = idx == kHdrMagic ? magic : 0;
}

}  // namespace sv
