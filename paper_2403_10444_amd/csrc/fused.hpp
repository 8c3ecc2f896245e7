// Fused path: ONE launch, every logit read from HBM once.
//
// The method needs two sweeps over each (target row i, draft row i) pair: the residual mass
// S_i = sum_x max(w_i p_i(x) - q_i(x), 0) of Alg. 2 depends on the rows' normalisers and on
// w_i, which depends on the normalisers of all earlier rows of the sequence.  Here the second
// sweep never touches memory: the first sweep's exponentials stay in registers until the
// row's normalisers are known.
//
// A *unit* is 64 * LANE contiguous logits (LANE = 32 or 64 per lane: 2048 or 4096) of a (target row i,
// draft row i) pair - the last target row, which has no draft row, counts as a pair without its second
// half - and belongs to one wavefront; a workgroup is four waves (four neighbouring units).  A wave
//   1. loads its 2 x 64 * LANE logits (16-byte loads, 1 KB per load instruction),
//   2. turns them into exp2(y - shift) with a wave-uniform shift per row and KEEPS those 2 x LANE
//      floats per lane in registers; its partial normalisers (shift, sum) meet those of the
//      workgroup's other waves in LDS,
//   3. sleeps at a barrier while the workgroup's first wave publishes the workgroup's two words and
//      looks at log2 w_i, which the previous position's leader published (Alg. 2: w_i = min(w_{i-1} r_i, 1)).
//      The acceptance probability of Alg. 2 / 4 never exceeds w_i, so where the position's uniform is not below
//      w_i its residual mass cannot matter (residual_needed) and the workgroup is done.  Otherwise the first wave
//      waits for the words of the other workgroups of the row, which give L_p and L_q.  The first wave of the
//      row's last workgroup is the row's leader and always stays: it publishes the row's ratio and log2 w_{i+1},
//   4. forms its share of S_i from the registers and publishes it; the row's leader then draws the token that
//      follows if this position becomes tau (draw_from_row) and publishes it.
// Workgroups start position-major inside groups of sequences (all row pairs of position 0, then
// position 1, ..., then the last target rows), so what an earlier position publishes is there
// before a later one asks for it, and a workgroup only ever waits for the workgroups of
// its own row, which start next to it.  The leader of a sequence's last row pair finishes the
// sequence: it collects the ratios and the partial sums, runs the accept tests (finalize_tests), picks up the
// token drawn for position tau (or draws it, if tau is its own position or every token was accepted) and
// zeroes the sequence's words (finalize_cleanup).
//
// Everything that crosses workgroups is a self-announcing word: it is zero between calls and
// non-zero once written (a packed (shift, sum) pair always has a non-zero sum or a -inf shift;
// ratio words and partial sums get their lowest mantissa bit set).  Words are written and read
// with agent-scope atomic accesses, which go through to device memory instead of living in one
// XCD's L2; no agent-scope fence is needed (on this part such a fence writes back /
// invalidates a whole L2 and cost more than the rest of the kernel).
//
// Progress: the hardware starts workgroups in index order (round-robin over the XCDs, in order
// within each).  A unit waits only for units of its own row (at most kMaxUnitsPerRow / 4
// workgroups away; the host refuses rows that do not fit four times into the resident set)
// and of earlier positions of its sequence (earlier workgroups), and publishing never waits:
// the grid always drains.  Every wait is also bounded by a spin limit; running into it sets
// the workspace's error word and goes on instead of hanging.
#pragma once

#include "common.hpp"

namespace sv {

constexpr int kWave = 64;
// LANE, a template parameter of the kernel: logits of one row that a lane holds of a unit, 32 or 64.  A unit is
// kWave * LANE contiguous logits of one row; fatter units mean fewer workgroups per row to wait for and the
// fixed registers of a wave spread over more logits (bf16 rows only: 161 VGPRs, 3 waves per SIMD).
constexpr int kLaneSmall = 32, kLaneLarge = 64;
constexpr int kMaxUnitsPerRow = 512;     // wave chunks per row the fused kernel takes (V <= 1 Mi logits): 8 words per lane

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
    const int32_t *draft_lens;   // NULL, or [B]: sequence b uses its first draft_lens[b] draft positions (1 .. gamma)
    const float *uniforms;
    int B, gamma, V;
    size_t tstride, dstride;     // elements from one target / draft row to the next (>= V)
    float k;              // float(log2(e) / T): the factor the sweeps multiply logits by
    double kd;            // log2(e) / T in double
    double k_eps;         // kd / k - 1: what rounding k to float left out (|k_eps| <= 2^-24)
    int algo;
    int nu;               // units (wave chunks) per row = 4 * workgroups per row
    int group_seqs;       // sequences per group of the row order
    int prune;            // leave out residual masses that cannot matter (residual_needed); off for calls so small that
                          // all positions run at once, where asking for log2 w first only lengthens the chain
    int spin_limit;
    int magic;            // workspace_magic(B, gamma, V)
    int *header;
    u64 *ratio;           // [B, gamma]               log2 r_{i+1} as double bits, lowest bit set
    unsigned *ycand;      // [B, gamma]               token drawn from the row pair's residual by its leader, + 2
    int *gen;             // [B]                      calls this sequence slot has finished (only its parity is used); never zeroed
    u64 *lw;              // [B, gamma]               log2 w_{i+1} (unclamped for greedy) as double bits with bit 0 set and the
                          //                          parity of gen in bit 1 (pack_lw); token verification:
                          //                          0 while every test up to i+1 has passed, kLog2RatioFloor afterwards
    u64 *pstat;           // [B, gamma+1, nu]         packed (shift, sum) per wave chunk of a target row
    u64 *pgrp, *qgrp;     // [B, gamma, nu / 4]       packed (shift, sum) per workgroup chunk of a row pair's target / draft row
    unsigned *spart;      // [B, gamma, nu]           residual partial sums per wave chunk: float bits, lowest bit set
    int32_t *accept_len, *next_token;
    float *debug_out;
    long long *prof;      // NULL, or [workgroups, 16] timestamps (100 MHz ticks) for tuning
};

// ---- agent-scope accessors for words that other waves (on any XCD) write or read
__device__ __forceinline__ int ld_i32(const int *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ unsigned ld_u32(const unsigned *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_u32(unsigned *p, unsigned v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ unsigned pack_partial(float v) { return __float_as_uint(v) | 1u; }
__device__ __forceinline__ float unpack_partial(unsigned w) { return __uint_as_float(w & ~1u); }
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
// The words that carry log2 w from one position to the next are read by workgroups that publish nothing
// afterwards (those whose residual mass is not formed), so nobody could tell when it is safe to zero them.
// They are not zeroed: bit 1 carries the parity of the sequence's call count (`gen`, flipped by the wave that
// finishes the sequence, after everybody who reads these words has read the count), and a word of the other
// parity - the previous call's - counts as not written yet.  Positions that a call does not use are zeroed.
__device__ __forceinline__ u64 pack_lw(double log2w, unsigned par)
{
    return ((u64)__double_as_longlong(log2w) & ~3ull) | 1ull | ((u64)par << 1);
}
__device__ __forceinline__ bool lw_there(u64 v, unsigned par) { return (v & 1ull) != 0 && ((unsigned)(v >> 1) & 1u) == par; }

// The value a given lane holds (lane index uniform over the wave).
__device__ __forceinline__ u64 read_lane_u64(u64 v, int lane)
{
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(v & 0xffffffffull), lane);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(v >> 32), lane);
    return ((u64)hi << 32) | lo;
}

// A word that is zero until its producer has written it: lanes with `need` poll *p until it is
// non-zero (`v` may already hold it).  One loop for the whole wave; gives up after `limit` polls.
__device__ __forceinline__ u64 wait_word(const u64 *p, u64 v, bool need, int limit, bool &gave_up)
{
    int spins = 0;
    while (__any(need && v == 0)) {
        if (++spins > limit) { gave_up = true; break; }
        __builtin_amdgcn_s_sleep(1);
        if (need && v == 0) v = ld_u64(p);
    }
    return v;
}
__device__ __forceinline__ u64 wait_word(const u64 *p, int limit, bool &gave_up)
{
    return wait_word(p, ld_u64(p), true, limit, gave_up);
}

__device__ __forceinline__ u64 wait_lw(const u64 *p, u64 v, unsigned par, bool need, int limit, bool &gave_up)
{
    int spins = 0;
    while (__any(need && !lw_there(v, par))) {
        if (++spins > limit) { gave_up = true; break; }
        __builtin_amdgcn_s_sleep(1);
        if (need && !lw_there(v, par)) v = ld_u64(p);
    }
    return v;
}

__device__ __forceinline__ unsigned wait_word32(const unsigned *p, unsigned v, bool need, int limit, bool &gave_up)
{
    int spins = 0;
    while (__any(need && v == 0)) {
        if (++spins > limit) { gave_up = true; break; }
        __builtin_amdgcn_s_sleep(1);
        if (need && v == 0) v = ld_u32(p);
    }
    return v;
}
__device__ __forceinline__ unsigned wait_word32(const unsigned *p, int limit, bool &gave_up)
{
    return wait_word32(p, ld_u32(p), true, limit, gave_up);
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

// The words of a row's n units as a wave holds them: lane l has entries l, l + 64, ... (NW of them).
template <int NW> struct RowWords { u64 w[NW]; };

// Issues the loads of a row's words (an entry that is still 0 is polled later).
template <int NW>
__device__ __forceinline__ void load_row_words(const u64 *words, int n, RowWords<NW> &r)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int q = 0; q < NW; ++q) {
        const int e = lane + q * kWave;
        r.w[q] = ld_u64(words + (e < n ? e : n - 1));
    }
}

// Log2-normaliser of a row from the words of its n <= 64 NW units: every lane combines its entries
// (in that fixed order), then the wave combines.  Returns L; M_out is the largest shift.
template <int NW>
__device__ __forceinline__ double row_normaliser(const u64 *words, int n, int limit, bool &gave_up, float &M_out, const RowWords<NW> &r)
{
    const int lane = threadIdx.x & 63;
    StatAcc acc;
#pragma unroll
    for (int q = 0; q < NW; ++q) {
        const int e = lane + q * kWave;
        if (q * kWave < n) {
            const u64 w = wait_word(words + (e < n ? e : n - 1), r.w[q], e < n, limit, gave_up);
            if (e < n) acc.add(w);
        }
    }
    const float M = wave_max(acc.m);
    const float z = wave_sum(acc.m > -INFINITY ? acc.z * fast_exp2(acc.m - M) : 0.f);
    M_out = M;
    return (double)M + log2_precise(z);
}

// Largest shift among a row's words, once all of them are there.
__device__ __forceinline__ float row_max_shift(const u64 *words, int n, int limit, bool &gave_up)
{
    const int lane = threadIdx.x & 63;
    float m = -INFINITY;
    for (int e0 = 0; e0 < n; e0 += kWave) {
        const int e = e0 + lane;
        const u64 w = wait_word(words + (e < n ? e : n - 1), 0, e < n, limit, gave_up);
        if (e < n) m = fmaxf(m, stat_shift(w));
    }
    return wave_max(m);
}

// Whether position i's residual mass S_i can matter.  The acceptance probability of block (and greedy block)
// verification never exceeds w_i: h_i = S_i / (S_i + 1 - w_i) with S_i <= w_i.  So a test with eta_i >= w_i fails
// whatever S_i is, the position cannot become tau either (tau is a position whose test passed, or 0), and neither
// its second sweep nor its partial sums are needed.  Decided on log2 w_i as published and the uniform as stored,
// with a margin far above the rounding of h_i; the units of a row and the wave that finishes the sequence evaluate
// this same function on the same values, so they always agree on which partial sums exist.
__device__ __forceinline__ bool can_become_tau(const FusedParams &P, int i, double log2w_i, float eta_i)
{
    if (i == 0) return true;                               // tau = 0: nothing accepted
    // token verification (Alg. 1) stops at the first failure: the word that carries log2 w_i for the other two
    // algorithms carries 0 while every test up to position i has passed and kLog2RatioFloor afterwards; only a
    // position that all earlier tests let through can become tau
    if (P.algo == kToken) return log2w_i > 0.5 * kLog2RatioFloor;
    return (double)__builtin_amdgcn_logf(eta_i) < log2w_i + 1.0e-3;
}
// Whether position i's residual mass is formed: where the position can become tau, and everywhere when the caller
// wants every S_i reported or the call is too small for leaving any out to pay.
__device__ __forceinline__ bool residual_needed(const FusedParams &P, int i, double log2w_i, float eta_i)
{
    return !P.prune || P.debug_out || can_become_tau(P, i, log2w_i, eta_i);
}

struct Unit {
    int b, i, c;          // sequence, position (gamma: the last target row, which has no draft row), wave chunk
    bool last_row;
};

// Workgroup order: groups of `group_seqs` sequences; inside a group the row pairs position-major
// (position, sequence, chunk), then the last target rows (which have no draft row and wait for
// nothing: a light last generation while the sequences are being finished).
// The grid spells this out, (x, y, z) = (chunk / 4, sequence in group, group * (gamma + 1) + slot)
// with slot i for position i and slot gamma for the last target row; x runs fastest in the start order.
// Returns false for the padding of a last, smaller group.
__device__ __forceinline__ bool decode_unit(const FusedParams &P, int wave, Unit &U, int &x)
{
    int grp = 0, slot = blockIdx.z;
    if (P.B > P.group_seqs) { grp = blockIdx.z / (P.gamma + 1); slot = blockIdx.z - grp * (P.gamma + 1); }
    U.b = grp * P.group_seqs + blockIdx.y;
    // which of the row's workgroups takes which chunk rotates from row to row: a row's workgroups go to the
    // XCDs round-robin, and the last chunk (fewest logits, leader's duties) must not always meet the same XCD
    const int wpr = gridDim.x;
    x = (int)((blockIdx.x + blockIdx.y + blockIdx.z) % wpr);
    U.c = x * kWaves + wave;
    U.last_row = slot == P.gamma;
    U.i = slot;
    return U.b < P.B;
}

// The logits a lane holds of one row, as loaded: raw 16-byte vectors on the aligned path.
template <typename T, bool ALIGNED, int LANE> struct RawSlice;
template <typename T, int LANE> struct RawSlice<T, true, LANE> {
    static constexpr int kNV = LANE / ElemTraits<T>::kVec;
    uint4 v[kNV];
};
template <typename T, int LANE> struct RawSlice<T, false, LANE> { };      // the element-wise path loads when it unpacks

// Vector v of a lane starts at element first + v * 64 * kVec of the row, so one load instruction of
// the wave covers 1 KB of contiguous memory.
template <typename T, bool ALIGNED, int LANE>
__device__ __forceinline__ void issue_loads(const T *row, int unit_first, int V, RawSlice<T, ALIGNED, LANE> &raw)
{
    constexpr int kUnitLogits = kWave * LANE;
    if constexpr (ALIGNED) {
        constexpr int kVec = ElemTraits<T>::kVec;
        const char *base = reinterpret_cast<const char *>(row);
        const unsigned lane_off = (unsigned)(unit_first + (int)(threadIdx.x & 63) * kVec) * (unsigned)sizeof(T);
        if (unit_first + kUnitLogits <= V) {                   // wave-uniform: the whole unit lies inside the row
#pragma unroll
            for (int v = 0; v < RawSlice<T, true, LANE>::kNV; ++v)
                raw.v[v] = *reinterpret_cast<const uint4 *>(base + (lane_off + (unsigned)(v * kWave * 16)));
        } else {
#pragma unroll
            for (int v = 0; v < RawSlice<T, true, LANE>::kNV; ++v) {
                const unsigned off = lane_off + (unsigned)(v * kWave * 16);
                // vectors beyond the row are recognised again when the slice is unpacked; load something valid
                raw.v[v] = *reinterpret_cast<const uint4 *>(base + (off < (unsigned)V * (unsigned)sizeof(T) ? off : 0u));
            }
        }
    }
}

template <typename T>
__device__ __forceinline__ void unpack_vec(const uint4 &v, float *out)
{
    if constexpr (ElemTraits<T>::kVec == 4) {
        out[0] = __uint_as_float(v.x); out[1] = __uint_as_float(v.y);
        out[2] = __uint_as_float(v.z); out[3] = __uint_as_float(v.w);
    } else {
        out[0] = bf16_lo(v.x); out[1] = bf16_hi(v.x); out[2] = bf16_lo(v.y); out[3] = bf16_hi(v.y);
        out[4] = bf16_lo(v.z); out[5] = bf16_hi(v.z); out[6] = bf16_lo(v.w); out[7] = bf16_hi(v.w);
    }
}

template <typename T, bool ALIGNED, int LANE>
__device__ __forceinline__ void unpack_slice(const T *row, int unit_first, int V, const RawSlice<T, ALIGNED, LANE> &raw,
                                             float (&x)[LANE])
{
    constexpr int kVec = ElemTraits<T>::kVec;
    constexpr int kNV = LANE / kVec;
    constexpr int kUnitLogits = kWave * LANE;
    const int first = unit_first + (int)(threadIdx.x & 63) * kVec;
    if constexpr (ALIGNED) {
#pragma unroll
        for (int v = 0; v < kNV; ++v) unpack_vec<T>(raw.v[v], x + v * kVec);
        // only a row's last units reach beyond the row (wave-uniform test): blank what lies beyond
        if (unit_first + kUnitLogits > V) {
#pragma unroll
            for (int v = 0; v < kNV; ++v) {
                const bool out = first + v * kWave * kVec >= V;
#pragma unroll
                for (int e = 0; e < kVec; ++e)
                    if (out) x[v * kVec + e] = -INFINITY;
            }
        }
    } else {
#pragma unroll
        for (int v = 0; v < kNV; ++v) load_vec<T, false>(row, V, first + v * kWave * kVec, x + v * kVec);
    }
}

// First sweep over the logits the wave holds of one row: x[j] becomes exp2(x[j] * k - shift) with
// the wave-uniform shift = k * (largest logit of the unit), or 0 when the whole unit lies beyond
// the row.  Returns the unit's word: (k * largest logit, sum of the exponentials); (-inf, 0) beyond.
template <int LANE>
__device__ __forceinline__ u64 first_sweep_row(float (&x)[LANE], float k, float &shift)
{
    float m = x[0];
#pragma unroll
    for (int j = 1; j < LANE; ++j) m = fmaxf(m, x[j]);
    const float Mw = wave_max(m * k);
    shift = Mw > -INFINITY ? Mw : 0.f;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};     // four partial sums: shorter chains, smaller rounding error
#pragma unroll
    for (int j = 0; j < LANE; ++j) {
        x[j] = fast_exp2(__builtin_fmaf(x[j], k, -shift));
        acc[j & 3] += x[j];
    }
    const float sw = wave_sum((acc[0] + acc[1]) + (acc[2] + acc[3]));
    return pack_stat(Mw, sw);
}

// ------------------------------------------------------------------ whole sequences
// Inclusive scans over the 64 lanes through DPP: four shifts inside each row of 16 lanes (lanes
// without a source add 0), then the two row broadcasts.
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ int dpp_shift(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, true);
}
__device__ __forceinline__ float wave_scan(float v)
{
    v += __int_as_float(dpp_shift<0x111>(__float_as_int(v)));          // row_shr:1
    v += __int_as_float(dpp_shift<0x112>(__float_as_int(v)));          // row_shr:2
    v += __int_as_float(dpp_shift<0x114>(__float_as_int(v)));          // row_shr:4
    v += __int_as_float(dpp_shift<0x118>(__float_as_int(v)));          // row_shr:8
    v += __int_as_float(dpp_shift<0x142, 0xa>(__float_as_int(v)));     // row_bcast15 into rows 1 and 3
    v += __int_as_float(dpp_shift<0x143, 0xc>(__float_as_int(v)));     // row_bcast31 into rows 2 and 3
    return v;
}
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ double dpp_shift_double(double v)
{
    const long long bits = __double_as_longlong(v);
    const unsigned lo = (unsigned)dpp_shift<CTRL, ROW_MASK>((int)(unsigned)(bits & 0xffffffffll));
    const unsigned hi = (unsigned)dpp_shift<CTRL, ROW_MASK>((int)(unsigned)((unsigned long long)bits >> 32));
    return __longlong_as_double((long long)(((u64)hi << 32) | lo));
}
__device__ __forceinline__ double wave_scan(double v)
{
    v += dpp_shift_double<0x111>(v);
    v += dpp_shift_double<0x112>(v);
    v += dpp_shift_double<0x114>(v);
    v += dpp_shift_double<0x118>(v);
    v += dpp_shift_double<0x142, 0xa>(v);
    v += dpp_shift_double<0x143, 0xc>(v);
    return v;
}
__device__ __forceinline__ double read_lane_double(double v, int lane)
{
    return __longlong_as_double((long long)read_lane_u64((u64)__double_as_longlong(v), lane));
}

#define FSTAMP(slot) do { if (P.prof && threadIdx.x == 0) P.prof[(((size_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 16 + (slot)] = wall_clock64(); } while (0)

// Inverse-CDF draw of one token from row `row` of sequence b (one wave), in index order, first token whose
// running sum exceeds u * total.  mode 0: from the residual max(w p - q, 0) of row pair `row`, located by the
// partial sums per wave chunk that the pair's units publish (polled here until all are there) and then by
// the weights of that one chunk, formed again from the logits with alpha_p = L_p - log2 w and alpha_q = L_q;
// a residual without any mass falls back to mode 1.  mode 1: from p_row itself, by the target row's
// (shift, sum) words.
template <typename T, bool ALIGNED, int LANE>
__device__ __forceinline__ int draw_from_row(const FusedParams &P, int b, int row, int mode, double alpha_p, double alpha_q,
                                             float u, bool &gave_up)
{
    constexpr int kVec = ElemTraits<T>::kVec;
    constexpr int kNV = LANE / kVec;
    constexpr int kUnitLogits = kWave * LANE;
    const int lane = threadIdx.x & 63;
    const int G = P.gamma, V = P.V, nu = P.nu;
    const float k = P.k;
    const T *target = static_cast<const T *>(P.target);
    const T *draft = static_cast<const T *>(P.draft);
    const size_t base = (size_t)b * (G + 1);
    const size_t drow = (size_t)b * G + (mode == 0 ? row : 0);
    const u64 *st = P.pstat + (base + row) * nu;
    const unsigned *sp = P.spart + drow * nu;

    // ---- first the wave chunk that holds t = u * total ...
    float Mrow = 0.f;
    RowCoef rc = {};
    if (mode == 0) rc = make_row_coef(alpha_p, alpha_q);
    else Mrow = row_max_shift(st, nu, P.spin_limit, gave_up);
    int slot = -1, last_nonzero = 0;
    double t_in = 0.0;
    for (int attempt = 0; attempt < 2 && slot < 0; ++attempt) {
        double total = 0.0, t = 0.0;
        for (int pass_no = 0; pass_no < 2; ++pass_no) {           // pass 0: total; pass 1: locate t = u * total
            double carry = 0.0;
            for (int e0 = 0; e0 < nu; e0 += kWave) {
                const int e = e0 + lane, ee = e < nu ? e : nu - 1;
                double part = 0.0;
                if (mode == 0) {
                    unsigned w = ld_u32(sp + ee);
                    if (pass_no == 0) w = wait_word32(sp + ee, w, e < nu, P.spin_limit, gave_up);
                    if (e < nu) part = (double)unpack_partial(w);
                } else {
                    const u64 v = ld_u64(st + ee);
                    const float sh = stat_shift(v);
                    if (e < nu && sh > -INFINITY) part = (double)(stat_sum(v) * fast_exp2(sh - Mrow));
                }
                const double inc = wave_scan(part) + carry;
                if (pass_no == 1 && slot < 0) {
                    const u64 hit = __ballot(e < nu && inc > t);
                    const u64 nz = __ballot(e < nu && part > 0.0);
                    if (nz) last_nonzero = e0 + 63 - __clzll((long long)nz);
                    if (hit) {
                        const int first = __ffsll((long long)hit) - 1;
                        slot = e0 + first;
                        t_in = t - read_lane_double(inc - part, first);
                    }
                }
                carry = read_lane_double(inc, kWave - 1);
            }
            if (pass_no == 0) { total = carry; t = (double)u * total; }
        }
        if (slot < 0) {
            if (mode == 0 && !(total > 0.0)) {                         // no residual mass: draw from p_row
                mode = 1;
                Mrow = row_max_shift(st, nu, P.spin_limit, gave_up);
                continue;
            }
            slot = last_nonzero; t_in = INFINITY;                      // rounding pushed t past the end
        }
    }
    if (slot < 0) { slot = 0; t_in = INFINITY; }

    // ---- ... then the token inside that chunk: weights recomputed from the logits, walked in
    // vocabulary order (vector, lane, element)
    const T *prow = target + (base + row) * P.tstride;
    const T *qrow = draft + drow * P.dstride;
    const int first = slot * kUnitLogits + lane * kVec;
    float xp[kNV][kVec], xq[kNV][kVec];
#pragma unroll
    for (int v = 0; v < kNV; ++v) {
        load_vec<T, ALIGNED>(prow, V, first + v * kWave * kVec, xp[v]);
        if (mode == 0) load_vec<T, ALIGNED>(qrow, V, first + v * kWave * kVec, xq[v]);
    }
    const u64 sv = wait_word(st + slot, P.spin_limit, gave_up);
    const float shift = stat_shift(sv), scale = fast_exp2(shift - Mrow);
    float t = mode == 0 ? (float)(t_in / (double)rc.cq) : (float)t_in;
    int y = -1, last_positive = -1;
#pragma unroll
    for (int v = 0; v < kNV; ++v) {
        const int idx = first + v * kWave * kVec;
        float wgt[kVec];
        if (mode == 0) {
#pragma unroll
            for (int e = 0; e < kVec; ++e) wgt[e] = fmaxf(residual_term(xp[v][e], xq[v][e], k, rc), 0.f);
        } else {
#pragma unroll
            for (int e = 0; e < kVec; ++e) wgt[e] = fast_exp2(__builtin_fmaf(xp[v][e], k, -shift)) * scale;
        }
        float mine = 0.f;
#pragma unroll
        for (int e = 0; e < kVec; ++e) {
            mine += wgt[e];
            if (wgt[e] > 0.f) last_positive = idx + e;
        }
        const float inc = wave_scan(mine);
        const float total = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(inc), kWave - 1));
        const u64 hit = __ballot(inc > t);
        if (y < 0 && hit) {
            const int first_lane = __ffsll((long long)hit) - 1;
            int cand = -1;
            if (lane == first_lane) {
                float run = inc - mine;
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
            y = __builtin_amdgcn_readlane(cand, first_lane);
        }
        t -= total;
    }
    if (y < 0) {
        // t lies beyond the chunk's recomputed total: the last token of positive weight
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) last_positive = max(last_positive, __shfl_xor(last_positive, off, kWave));
        y = last_positive < 0 ? 0 : last_positive;
    }
    return y;
}

// Accept tests of one sequence (one wave: the leader of the sequence's last row pair).  Returns tau and writes
// it; y_out is the token that the leader of row pair tau has drawn from its residual, or -1 when tau is the
// last row pair or beyond (then the caller draws); lw_own is log2 w of the last row pair.
// `own` (LDS, written by this same wave): log2 r, L_p, L_q and the word for the next position of the
// sequence's last row pair - they need no trip through device memory.
__device__ __forceinline__ int finalize_tests(const FusedParams &P, int b, int gamma, const double *own, unsigned par, int &y_out,
                                              double &lw_own, u64 &last_first, bool &gave_up)
{
    constexpr int kBatch = 8;                           // rows whose words are fetched together (one round trip)
    const int lane = threadIdx.x & 63;
    // `gamma` is this sequence's draft length; G, the call's (largest) draft length, is the stride of every array
    const int G = P.gamma, nu = P.nu;
    const size_t base = (size_t)b * (G + 1);
    const int e_lane = lane < nu ? lane : nu - 1;

    // everything the tests need is asked for at once (one round trip): the rows' ratios, log2 w, the uniforms,
    // the first batch of partial sums and the tokens the rows' leaders have drawn; what is not there yet is
    // polled where it is used.  Lane j holds what belongs to row pair j (gamma <= 64).
    const size_t drow_l = (size_t)b * G + (lane < gamma ? lane : gamma - 1);
    const u64 *lw_word = P.lw + drow_l;
    const float *eta = P.uniforms + (size_t)b * (G + 1);
    u64 w0 = ld_u64(P.ratio + drow_l);
    const u64 lw_first = ld_u64(lw_word);
    unsigned sw_first[kBatch];
#pragma unroll
    for (int jj = 0; jj < kBatch; ++jj) {
        const int j = jj < gamma ? jj : gamma - 1;
        sw_first[jj] = ld_u32(P.spart + ((size_t)b * G + j) * nu + e_lane);
    }
    const unsigned cand_first = ld_u32(P.ycand + drow_l);
    last_first = ld_u64(P.pstat + (base + gamma) * nu + e_lane);    // for the clean-up at the very end
    w0 = wait_word(P.ratio + drow_l, w0, lane < gamma - 1, P.spin_limit, gave_up);
    double my_lr = unpack_ratio(w0);                    // log2 r_{lane+1}
    if (lane == gamma - 1) my_lr = own[0];
    FSTAMP(7);
    // log2 w_j for lane j as the rows' leaders published it (Alg. 2: w_j = min(w_{j-1} r_j, 1); Alg. 4
    // drops the min); lw_last is log2 w_gamma
    double my_lw = 0.0, my_lw_raw = 0.0, lw_last = 0.0;
    {
        double next = unpack_ratio(wait_lw(lw_word, lw_first, par, lane < gamma - 1, P.spin_limit, gave_up));   // log2 w_{lane+1}
        if (lane == gamma - 1) next = own[4];
        const double prev = __shfl_up(next, 1, kWave);
        my_lw_raw = lane ? prev : 0.0;
        if (P.algo != kToken) {                              // token verification: the words only say where the tests stopped
            my_lw = my_lw_raw;
            lw_last = read_lane_double(next, gamma - 1);
            if (P.algo == kGreedy) { my_lw = fmin(my_lw, 100.0); lw_last = fmin(lw_last, 100.0); }
        }
    }
    FSTAMP(8);
    // what the accept tests need of w_j is formed now, before the wait for the partial sums: lane l tests
    // position j = l + 1, whose row values sit in lane j
    const int j = lane + 1;
    const double lw_below = __shfl_down(my_lw, 1, kWave);
    const double lw_j = j < gamma ? lw_below : lw_last;
    const double w_j = exp2(lw_j);
    const double one_minus_w = -expm1(lw_j * 0.69314718055994530942);
    const double h_token = exp2(fmin(my_lr, 0.0));      // min(r_j, 1); lane l holds log2 r_{l+1}
    const float eta_j = eta[j <= gamma ? j - 1 : 0];
    // the positions whose residual mass exists (see residual_needed): bit l stands for position l + 1; position 0
    // always has it.  The rule is evaluated on log2 w as published (before the cap that greedy applies above)
    const double lw_rule = __shfl_down(my_lw_raw, 1, kWave);
    const u64 have = __ballot(j < gamma && residual_needed(P, j, j < gamma ? lw_rule : 0.0, eta_j));
    // the positions that can become tau: their leaders draw the token that would follow (bit l: position l + 1)
    const u64 may = __ballot(j < gamma && can_become_tau(P, j, j < gamma ? lw_rule : 0.0, eta_j));

    // ---- S_j = sum of row j's partial sums, into lane j
    float my_S = 0.f;
    for (int j0 = 0; j0 < gamma; j0 += kBatch) {
        unsigned sw[kBatch];
#pragma unroll
        for (int jj = 0; jj < kBatch; ++jj) {
            const int j = j0 + jj < gamma ? j0 + jj : gamma - 1;
            if (j0 == 0) {                               // asked for at the start
                sw[jj] = sw_first[jj];
            } else {
                sw[jj] = ld_u32(P.spart + ((size_t)b * G + j) * nu + e_lane);
            }
        }
#pragma unroll
        for (int jj = 0; jj < kBatch; ++jj) {
            const int j = j0 + jj;
            if (j >= gamma) continue;
            if (j > 0 && !((have >> (j - 1)) & 1)) continue;      // no partial sums were formed for this row: S stays 0
            const size_t drow = (size_t)b * G + j;
            float acc = 0.f;
            const unsigned w = wait_word32(P.spart + drow * nu + e_lane, sw[jj], lane < nu, P.spin_limit, gave_up);
            if (lane < nu) acc = unpack_partial(w);
            for (int e = lane + kWave; e < nu; e += kWave) {
                acc += unpack_partial(wait_word32(P.spart + drow * nu + e, P.spin_limit, gave_up));
            }
            acc = wave_sum(acc);
            if (lane == j) my_S = acc;
        }
    }

    FSTAMP(9);
    // ---- accept tests eta_j < h_j
    const double S_row = (double)__shfl_down(my_S, 1, kWave);
    bool pass = false;
    if (j <= gamma) {
        const double S = j < gamma ? S_row : w_j;        // q_gamma == 0: S_gamma = w_gamma
        double h;
        if (P.algo == kToken) h = h_token;
        else if (j == gamma) h = fmin(w_j, 1.0);                                           // h_gamma = w_gamma
        // block: S / (S + 1 - w).  Greedy (Alg. 4) divides by the rejected mass sum_x max(q - w p, 0) instead, which
        // is the same number: it equals S - sum_x (w p - q) = S + 1 - w because both rows sum to one (w unclipped;
        // at w >= 1 the ratio is >= 1 and every eta in [0, 1) passes)
        else h = lw_j >= 0.0 ? 1.0 : S / (S + one_minus_w);
        pass = (double)eta_j < h && (j == gamma || ((have & may) >> (j - 1)) & 1);
        if (P.debug_out) {
            float *d = P.debug_out + (base + j) * 3;
            d[0] = (float)w_j; d[1] = (float)S; d[2] = (float)h;
        }
    }
    if (lane == 0 && P.debug_out) {
        float *d = P.debug_out + base * 3;
        d[0] = 1.f; d[1] = my_S; d[2] = 1.f;
    }
    const u64 passed = __ballot(pass);
    int tau;
    if (P.algo == kToken) tau = passed == ~0ull ? 64 : __ffsll((long long)~passed) - 1;    // leading run of passes
    else tau = passed ? 64 - __clzll((long long)passed) : 0;                               // last passing sub-block
    if (lane == 0) P.accept_len[b] = tau;
    FSTAMP(10);

    // ---- the tokens that the leaders of the row pairs before the last one have drawn: all of them are waited
    // for (not only tau's), because their leaders read the partial sums that are zeroed when the sequence is done
    const bool drawn = lane <= gamma - 2 && (lane == 0 || ((may >> (lane - 1)) & 1));
    const unsigned cand = wait_word32(P.ycand + drow_l, cand_first, drawn, P.spin_limit, gave_up);
    y_out = tau <= gamma - 2 ? __builtin_amdgcn_readlane((int)cand, tau) - 2 : -1;
    lw_own = read_lane_double(my_lw, gamma - 1);
    return tau;
}

// The sequence's control words are left zero for the next call (one wave, after Y is known).  Every reader of
// the row-pair words has published something this wave has waited for: the units their partial sums (or, where
// no residual mass is formed, nothing was read but by the leader), the leaders their ratio and their token.
__device__ __forceinline__ void finalize_cleanup(const FusedParams &P, int b, int gamma, u64 last_first, unsigned par, bool &gave_up)
{
    const int lane = threadIdx.x & 63;
    const int G = P.gamma, nu = P.nu;
    const size_t base = (size_t)b * (G + 1);
    const int e_lane = lane < nu ? lane : nu - 1;
    // the last target row's words must all be written before the target rows' words can go (`last_first`: what
    // was there when the tests began)
    const u64 *last = P.pstat + (base + gamma) * nu;
    for (int e = lane; e < G * nu; e += kWave) st_u32(P.spart + (size_t)b * G * nu + e, 0);
    for (int e = lane; e < G * (nu / kWaves); e += kWave) { st_u64(P.pgrp + (size_t)b * G * (nu / kWaves) + e, 0); st_u64(P.qgrp + (size_t)b * G * (nu / kWaves) + e, 0); }
    for (int e = lane; e < G; e += kWave) {
        st_u64(P.ratio + (size_t)b * G + e, 0); st_u32(P.ycand + (size_t)b * G + e, 0);
        if (e >= gamma - 1) st_u64(P.lw + (size_t)b * G + e, 0);     // only where this call had no reader (see pack_lw)
    }
    wait_word(last + e_lane, last_first, lane < nu, P.spin_limit, gave_up);
    for (int e = lane + kWave; e < nu; e += kWave) wait_word(last + e, P.spin_limit, gave_up);
    for (int e = lane; e < (G + 1) * nu; e += kWave) st_u64(P.pstat + base * nu + e, 0);
    // the sequence's next call: every workgroup that reads the count has read it (their words were waited for)
    if (lane == 0) __hip_atomic_store(P.gen + b, (int)(par ^ 1u), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
#undef FSTAMP

// ------------------------------------------------------------------ the kernel
template <typename T, bool ALIGNED, int NW, int LANE>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(LANE == kLaneLarge ? 3 : ElemTraits<T>::kVec == 8 ? 5 : 4)))
void fused_verify_kernel(const FusedParams P)
{
    constexpr int kVec = ElemTraits<T>::kVec;
    constexpr int kUnitLogits = kWave * LANE;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int gamma = P.gamma, V = P.V, nu = P.nu;
    const float k = P.k;

    if (__builtin_nontemporal_load(P.header + kHdrMagic) != P.magic) {
        // the workspace was not initialised for this shape: report it through the outputs and leave
        if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0)
            for (int b = threadIdx.x; b < P.B; b += kThreads) { P.accept_len[b] = -1; P.next_token[b] = -1; }
        return;
    }
#define SV_STAMP(slot) do { if (P.prof && threadIdx.x == 0) P.prof[(((size_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 16 + (slot)] = wall_clock64(); } while (0)
    Unit U;
    int wg_x;
    if (!decode_unit(P, wave, U, wg_x)) return;
    SV_STAMP(0);
    // a sequence with a shorter draft has no row pairs at its unused positions, and its last target row is row gb
    int gb = gamma;
    if (P.draft_lens) { gb = P.draft_lens[U.b]; gb = gb < 1 ? 1 : gb > gamma ? gamma : gb; }   // kept in range whatever the caller wrote
    if (U.last_row) U.i = gb;
    else if (U.i >= gb) return;

    // stream A: the unit's chunk of target row i; stream B: the same chunk of draft row i (none for the last row)
    const size_t trow = (size_t)U.b * (gamma + 1) + U.i, drow = (size_t)U.b * gamma + (U.last_row ? 0 : U.i);
    const T *rowA = static_cast<const T *>(P.target) + trow * P.tstride;
    const T *rowB = static_cast<const T *>(P.draft) + drow * P.dstride;
    const int unit_first = U.c * kUnitLogits;
    RawSlice<T, ALIGNED, LANE> rawA, rawB;
    issue_loads<T, ALIGNED, LANE>(rowA, unit_first, V, rawA);
    if (!U.last_row) issue_loads<T, ALIGNED, LANE>(rowB, unit_first, V, rawB);
    // draft token X_{i+1} and its two logits: the first wave of the row's last workgroup (the one with the
    // fewest logits) publishes the row's ratio from them
    const int nwg = nu / kWaves;
    const bool leader = wave == 0 && wg_x == nwg - 1;
    // log2 w_i (published by the previous position's leader, usually long ago) and the uniform of position i's
    // test: what decides whether this row's residual mass can matter at all
    const bool need_w = U.i > 0 && !U.last_row;
    const u64 *lw_word = P.lw + (size_t)U.b * gamma + (U.i > 0 && !U.last_row ? U.i - 1 : 0);
    // (the sequence's call count rides in the same block of loads as the word itself: a load in a block of its own
    // makes the compiler wait for it, and for every load before it, at the end of that block)
    int gen_count = 0;
#define par ((unsigned)gen_count & 1u)
    u64 wt = 0;
    float eta_i = 0.f, eta_next = 0.f;
    int tok = 0;                                             // the drafted token X_{i+1}, for the leader
    if (wave == 0 && !U.last_row) {
        tok = P.tokens[drow];
        gen_count = P.gen[U.b];                                       // (does not change while the call runs: an ordinary load)
        eta_i = P.uniforms[(size_t)U.b * (gamma + 1) + (U.i > 0 ? U.i - 1 : 0)];
        eta_next = P.uniforms[(size_t)U.b * (gamma + 1) + U.i];      // the uniform of test i + 1, which the leader judges for Alg. 1
        wt = ld_u64(lw_word);
    }

    // ---- first sweep: exponentials stay in xa / xb; the unit's words go out
    __shared__ u64 wave_words[2][kWaves];
    __shared__ double row_values[3];
    __shared__ int row_needed;
    __shared__ double own_values[5];                         // the leader's results for its own use when it finishes the sequence
    float xa[LANE], xb[LANE];
    float shiftA, shiftB;
    unpack_slice<T, ALIGNED, LANE>(rowA, unit_first, V, rawA, xa);
    {
        const u64 stA = first_sweep_row(xa, k, shiftA);
        if (lane == 0) { st_u64(P.pstat + trow * nu + U.c, stA); wave_words[0][wave] = stA; }
    }
    if (U.last_row) return;          // the last target row has no draft row and no residual (whole workgroup)
    // the two logits of the draft token, asked for only now so that the streams above did not queue behind them
    double ya = 0.0, yb = 0.0;
    if (leader) { ya = logit_as_double(rowA + tok); yb = logit_as_double(rowB + tok); }
    unpack_slice<T, ALIGNED, LANE>(rowB, unit_first, V, rawB, xb);
    {
        const u64 stB = first_sweep_row(xb, k, shiftB);
        if (lane == 0) wave_words[1][wave] = stB;
    }
    __syncthreads();

    // ---- L_p, L_q and w_i.  The workgroup's first wave combines the four waves' words into the
    // workgroup's two words, publishes them, collects the words of all workgroups of the row and combines
    // those; the other three waves sleep at the barrier meanwhile.  The row's leader also publishes the
    // row's ratio, normalisers and w_{i+1}.  log2 w_i comes from the leader of the previous position
    // (Alg. 2: w_i = min(w_{i-1} r_i, 1)).
    bool gave_up = false;
    if (wave == 0) {
        SV_STAMP(1);
        StatAcc ga, gb;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) { ga.add(wave_words[0][w]); gb.add(wave_words[1][w]); }
        if (lane == 0) {
            st_u64(P.pgrp + drow * nwg + wg_x, pack_stat(ga.m, ga.z));
            st_u64(P.qgrp + drow * nwg + wg_x, pack_stat(gb.m, gb.z));
        }
        // can this row's residual mass matter?  Needs log2 w_i; a row that is not needed costs its workgroups no wait
        bool needed = true;
        if (need_w && P.prune && !P.debug_out) {
            wt = wait_lw(lw_word, wt, par, true, P.spin_limit, gave_up);
            needed = residual_needed(P, U.i, unpack_ratio(wt), eta_i);
        }
        if (lane == 0) row_needed = needed ? 1 : 0;
    }
    __syncthreads();
    const bool needed = row_needed != 0;
    // the leader of a sequence's last row pair finishes the sequence: what it works out for its row it has at hand
    const bool finisher = leader && U.i == gb - 1;
    // a row whose residual mass cannot matter: only its leader (the next position needs this row's ratio; the
    // last one finishes the sequence) stays; everybody else is done and frees its registers
    if (!needed && !leader) return;

    bool candidate = true;           // whether this position can become tau: then its leader draws the token that would follow
    if (wave == 0 && (needed || leader)) {
        float Mp, Mq;
        double Lp, Lq;
        if (nwg <= kWave / 2) {
            // one poll covers the row: the target row's words in lanes 0.., the draft row's in lanes 32..,
            // log2 w_i beside them; the two halves of the wave are then combined side by side
            const int e = lane & 31;
            const bool need = e < nwg;
            const u64 *word = (lane < 32 ? P.pgrp : P.qgrp) + drow * nwg + (need ? e : nwg - 1);
            u64 v = ld_u64(word);
            if (need_w) wt = ld_u64(lw_word);
            int spins = 0;
            while (__any((need && v == 0) || (need_w && !lw_there(wt, par)))) {
                if (++spins > P.spin_limit) { gave_up = true; break; }
                __builtin_amdgcn_s_sleep(1);
                if (need && v == 0) v = ld_u64(word);
                if (need_w && !lw_there(wt, par)) wt = ld_u64(lw_word);
            }
            StatAcc acc;
            if (need) acc.add(v);
            halves_max(acc.m, Mp, Mq);
            const float Mh = lane < 32 ? Mp : Mq;
            float zp, zq;
            halves_sum(acc.m > -INFINITY ? acc.z * fast_exp2(acc.m - Mh) : 0.f, zp, zq);
            Lp = (double)Mp + log2_precise(zp);
            Lq = (double)Mq + log2_precise(zq);
        } else {
            RowWords<NW> pw, qw;
            load_row_words<NW>(P.pgrp + drow * nwg, nwg, pw);
            load_row_words<NW>(P.qgrp + drow * nwg, nwg, qw);
            if (need_w) wt = ld_u64(lw_word);
            Lp = row_normaliser<NW>(P.pgrp + drow * nwg, nwg, P.spin_limit, gave_up, Mp, pw);
            Lq = row_normaliser<NW>(P.qgrp + drow * nwg, nwg, P.spin_limit, gave_up, Mq, qw);
        }
        double lr = 0.0;
        if (leader) {
            // log2 r_{i+1} = log2 p_i(X_{i+1}) - log2 q_i(X_{i+1}), for whoever finishes the sequence.  The sweeps
            // scale logits by the float k; the exact factor is kd = k (1 + k_eps).  To first order that moves a
            // row's log2-normaliser by k_eps * (the scaled logit where the mass sits, taken as the row
            // maximum); only this ratio, whose logs reach hundreds, is sensitive to it.
            const double lp = ya * P.kd - (Lp + P.k_eps * (double)Mp);
            const double lq = yb * P.kd - (Lq + P.k_eps * (double)Mq);
            lr = fmax(lp - lq, kLog2RatioFloor);    // a drafted token the target masks out: r = 0, kept finite
            if (lane == 0) {
                if (finisher) {                     // nobody else reads the last row pair's words
                    own_values[0] = unpack_ratio(pack_ratio(lr)); own_values[1] = Lp; own_values[2] = Lq;
                } else {
                    st_u64(P.ratio + drow, pack_ratio(lr));
                }
            }
        }
        double log2w = 0.0;
        if (need_w) log2w = unpack_ratio(wait_lw(lw_word, wt, par, true, P.spin_limit, gave_up));
        candidate = can_become_tau(P, U.i, log2w, eta_i);       // (on the word as published, like the finishing wave)
        if (leader) {
            // w_{i+1} for the workgroups of the next position
            double next = log2w + lr;
            if (P.algo == kBlock && next > 0.0) next = 0.0;        // the min{., 1}; greedy block verification omits it
            if (P.algo == kToken) {
                // token verification: 0 while every test so far has passed (test i+1: eta_{i+1} < min(r_{i+1}, 1), the
                // expression the finishing wave evaluates too), kLog2RatioFloor from the first failure on
                const bool pass = log2w > 0.5 * kLog2RatioFloor && (double)eta_next < exp2(fmin(unpack_ratio(pack_ratio(lr)), 0.0));
                next = pass ? 0.0 : kLog2RatioFloor;
            }
            if (lane == 0) {
                if (finisher) own_values[4] = unpack_ratio(pack_ratio(next));
                else st_u64(P.lw + drow, pack_lw(next, par));
            }
        }
        if (P.algo == kToken) log2w = 0.0;                          // the residual of token verification is p - q
        if (lane == 0) { row_values[0] = Lp; row_values[1] = Lq; row_values[2] = log2w; }
        SV_STAMP(2);
    }
    if (gave_up && lane == 0 && ld_i32(P.header + kHdrError) == 0) atomicOr(P.header + kHdrError, 1);
    // a draw that this wave makes: row, mode and the two row constants (see draw_from_row); -1: none
    int draw_row = -1, draw_mode = 0;
    double draw_ap = 0.0, draw_aq = 0.0;
    if (needed) {
    __syncthreads();
    const double Lp = row_values[0], Lq = row_values[1];
    double log2w = row_values[2];
    if (P.algo == kGreedy) log2w = fmin(log2w, 100.0);      // keeps w p finite in float
    SV_STAMP(3);

    // ---- second sweep, from registers: w p(x) = xa * cp, q(x) = xb * cq with wave-uniform cp, cq
    const double log2cp = (double)shiftA - (Lp - log2w), log2cq = (double)shiftB - Lq;
    float acc = 0.f;
    {
        // sum of max(xa cp - xb cq, 0) with the larger factor taken out, so that every term lies in [0, 1]
        // (xa, xb <= 1) and the clamp of the fma is the max: two instructions per pair
        const double log2rho = log2cp - log2cq;
        if (log2rho <= 0.0) {
            const float rho = fast_exp2((float)log2rho);
#pragma unroll
            for (int j = 0; j < LANE; ++j) acc += __builtin_amdgcn_fmed3f(__builtin_fmaf(xa[j], rho, -xb[j]), 0.f, 1.f);
            acc *= fast_exp2((float)log2cq);
        } else {
            const float nrho = -fast_exp2((float)-log2rho);
#pragma unroll
            for (int j = 0; j < LANE; ++j) acc += __builtin_amdgcn_fmed3f(__builtin_fmaf(xb[j], nrho, xa[j]), 0.f, 1.f);
            acc *= fast_exp2((float)log2cp);
        }
    }
    acc = wave_sum(acc);
    if (lane == 0) {
        st_u32(P.spart + drow * nu + U.c, pack_partial(acc));
    }
    SV_STAMP(4);
    // the row's leader draws the token that follows if this position becomes tau, while the later positions are
    // still streaming: whoever finishes the sequence then only picks it up
    if (leader && !finisher && candidate) { draw_row = U.i; draw_ap = Lp - log2w; draw_aq = Lq; }

    }
    if (!leader) return;
    // the leader of a sequence's last row pair finishes the sequence: the earlier positions come before
    // it in the workgroup order, the last target row (needed only if every token is accepted) right after
    int y = -1;
    u64 last_first = 0;
    if (finisher) {
        SV_STAMP(5);
        __builtin_amdgcn_wave_barrier();                     // own_values: written by lane 0 above, read by another lane below
        double lw_own;
        const int tau = finalize_tests(P, U.b, gb, own_values, par, y, lw_own, last_first, gave_up);
        if (y < 0) {
            // tau is the last row pair (its residual: this wave has the row's constants) or every token was
            // accepted (Y comes from the last target row itself)
            draw_row = tau; draw_mode = tau == gb ? 1 : 0;
            draw_ap = own_values[1] - lw_own; draw_aq = own_values[2];
        }
    }
    if (draw_row >= 0) {
        const float u = P.uniforms[(size_t)U.b * (gamma + 1) + gb];
        const int drawn = draw_from_row<T, ALIGNED, LANE>(P, U.b, draw_row, draw_mode, draw_ap, draw_aq, u, gave_up);
        if (finisher) y = drawn;
        else if (lane == 0) st_u32(P.ycand + (size_t)U.b * gamma + draw_row, (unsigned)drawn + 2u);
    }
    if (finisher) {
        if (lane == 0) P.next_token[U.b] = y;
        SV_STAMP(12);
        finalize_cleanup(P, U.b, gb, last_first, par, gave_up);
        SV_STAMP(6);
    }
    if (gave_up && lane == 0 && ld_i32(P.header + kHdrError) == 0) atomicOr(P.header + kHdrError, 1);
#undef SV_STAMP
#undef par
}

// Clears the control words of a workspace and marks it initialised.
__global__ void workspace_init_kernel(int *words, size_t n, int magic)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < n) words[idx] = idx == kHdrMagic ? magic : 0;
}

}  // namespace sv
