// Fused path: ONE launch, every logit read from HBM at most once.
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
//      forms w_i from the ratios log2 r_1 .. log2 r_i that the leaders of the earlier positions have
//      published (Alg. 2: w_i = min(w_{i-1} r_i, 1), evaluated as a scan over the ratios: no position waits
//      for a chain of earlier ones, only for their rows).  The acceptance probability of Alg. 2 / 4 never
//      exceeds w_i, so where the position's uniform is not below w_i its residual mass cannot matter
//      (residual_needed) and the workgroup is done.  Otherwise the first wave waits for the words of the other
//      workgroups of the row, which give L_p and L_q.  The first wave of the row's last workgroup is the
//      row's leader and always stays: it publishes the row's ratio log2 r_{i+1},
//   4. forms its share of S_i from the registers and publishes it; the row's leader then sums the row's
//      shares and judges the position's own accept test (Alg. 2 / 4: eta_i < h_i = S_i / (S_i + 1 - w_i)); where it
//      passes - and at position 0, which is tau when no test passes - it draws the token that follows if this
//      position becomes tau (draw_from_row) and publishes both in one word (lead_row).
// Workgroups start position-major inside groups of sequences (all row pairs of position 0, then
// position 1, ..., then the last target rows), so what an earlier position publishes is there
// before a later one asks for it, and a workgroup only ever waits for the workgroups of
// its own row, which start next to it.  The leader of a sequence's last row pair finishes the
// sequence: it reads one word per earlier position (did its test pass, and the token drawn there), judges the last
// test (eta_gamma < w_gamma) and writes tau and the token drawn for position tau (its own, or one from the last target
// row if every token was accepted).  The last target row is needed only when every token is accepted
// (Y ~ p_gamma): its workgroups wait for the ratios, and where eta_gamma >= w_gamma they load nothing.
//
// Everything that crosses workgroups is a self-announcing word: zero until written, non-zero once written
// (a packed (shift, sum) pair always has a non-zero sum or a -inf shift; ratio words and partial sums
// get their lowest mantissa bit set).  Words are written and read with agent-scope atomic accesses, which
// go through to device memory instead of living in one XCD's L2; no agent-scope fence is needed (on this
// part such a fence writes back / invalidates a whole L2 and cost more than the rest of the kernel).
// The words exist twice.  A sequence's calls use the two copies alternately (the parity of gen[b]), and every row's
// leader clears, in the copy that the call does NOT use, the words of its row - so nobody ever clears a word that
// somebody may still read, and nothing is cleared on the path that ends the kernel.  gen[b] is flipped once every
// workgroup of the sequence has read it: the workgroups of the last target row, which start last, each leave a word
// when they have, and the last of them flips gen[b] as soon as it has those words and one that the sequence's last row
// pair could only publish after every row pair's workgroups had published theirs (and so had read gen[b]).  Nothing
// at the end of a sequence waits for it.
//
// Progress: the hardware starts workgroups in index order (round-robin over the XCDs, in order
// within each).  A unit waits only for units of its own row (at most kMaxUnitsPerRow / 4
// workgroups away; the host refuses rows that do not fit four times into the resident set)
// and of earlier positions of its sequence (earlier workgroups), and publishing never waits:
// the grid always drains.  Every wait is also bounded by a spin limit.  A wave that runs into it sets the
// workspace's error word and from then on publishes only the all-ones word, which every reader passes on;
// the wave that finishes the sequence then writes -1 for tau and Y.  A kernel always exits.
#pragma once

#include "common.hpp"

namespace sv {

constexpr int kWave = 64;
#ifndef SV_WAVES_SMALL
#define SV_WAVES_SMALL 5      // waves per SIMD of the bf16 kernel with the small units
#endif
// LANE, a template parameter of the kernel: logits of one row that a lane holds of a unit, 32 or 64.  A unit is
// kWave * LANE contiguous logits of one row; fatter units mean fewer workgroups per row to wait for and the
// fixed registers of a wave spread over more logits (bf16 rows only: 161 VGPRs, 3 waves per SIMD).
constexpr int kLaneSmall = 32, kLaneLarge = 64;
// Whether the units of a row pair leave out the per-wave word of their target row (see draw_from_target_row): the kernel
// of the smaller units does; the one of the larger units sits at its register limit with the words published, and the
// few instructions of the other way cost it three spilled exponentials in its sweeps.
template <int LANE> constexpr bool kLazyRowWords = LANE == kLaneSmall;
constexpr int kMaxUnitsPerRow = 512;     // wave chunks per row the fused kernel takes (V <= 1 Mi logits): 8 words per lane

// Word 0 of an initialised workspace: a constant mixed with the shape it was initialised for.
__host__ __device__ inline int workspace_magic(int B, int gamma, int V)
{
    return (int)(0x53564b34u ^ ((unsigned)B * 2654435761u + (unsigned)gamma * 40503u + (unsigned)V * 2246822519u));
}

// (kHdrRowWords: non-zero once a kernel that publishes the per-wave words of target rows - the one of the larger units -
// has worked on the workspace: only then do the other kernels' leaders clear those words with the rest of a row's)
enum HeaderWord : int { kHdrMagic = 0, kHdrError = 1, kHdrRowWords = 2, kHdrWords = 64 };

typedef unsigned long long u64;

// The words of one copy (see the head of this file).
struct Words {
    u64 *ratio;           // [B, gamma]               log2 r_{i+1} as double bits, two lowest bits: flags (pack_ratio); by the leader of row pair i
    u64 *lw;              // [B, gamma]               calls larger than one resident set: log2 w_{i+1} as double bits, lowest bit set
                          //                          (Alg. 1: 0 while every test up to i + 1 has passed, kLog2RatioFloor afterwards); by
                          //                          the leader of row pair i
    u64 *rowres;          // [B, gamma]               what position i contributes to tau and Y (pack_rowres): whether its accept test
                          //                          passes (Alg. 2 / 4: eta_i < h_i; Alg. 1: the test of X_{i+1}) and the token drawn from
                          //                          row pair i's residual where tau can still be i; by the leader of row pair i
    u64 *pstat;           // [B, gamma, nu]           (largest scaled logit, sum) per wave chunk of a row pair's target row: filled in
                          //                          only by a wave that has to draw from that row itself (draw_from_target_row)
    u64 *plast;           // [B, nu]                  the same of the sequence's last target row (row draft_lens[b])
    u64 *pgrp, *qgrp;     // [B, gamma, nu / 4, 2]    packed (shift, sum) per workgroup chunk of a row pair's target / draft row, side by
                          //                          side (qgrp = pgrp + 1; entry e of a row's words lies 2 e words on): a workgroup's two
                          //                          words are one write of sixteen bytes
    unsigned *spart;      // [B, gamma, nu]           residual partial sums per wave chunk: float bits, lowest bit set
    u64 *lseen;           // [B, nu / 4]              non-zero once the workgroup of the last target row has read gen[b]
};

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
    unsigned inv_slots, inv_wpr;   // floor(2^32 / d) + 1 for d = gamma + 1 and d = workgroups per row: n / d = mulhi(n, .) for the n that occur
    int prune;            // leave out what cannot matter (residual_needed, the last target row); off for calls so small
                          // that all positions run at once, where asking for the ratios first only lengthens the chain
    int skip_last;        // the last target row is read only where every token can be accepted (its workgroups ask first)
    int spin_limit;
    int magic;            // workspace_magic(B, gamma, V)
    int *header;
    int *gen;             // [B]  calls this sequence slot has finished: its parity selects the copy of the words in use
    Words words;          // copy 0; copy 1 lies copy_bytes further on
    size_t copy_bytes;
    int32_t *accept_len, *next_token;
    float *debug_out;
#ifdef SV_PROFILE
    long long *prof;      // NULL, or [B * (gamma + 1) * workgroups per row, 16] timestamps (100 MHz ticks) for tuning
#endif
};

template <typename X> __device__ __forceinline__ X *shifted(X *p, size_t bytes)
{
    return reinterpret_cast<X *>(reinterpret_cast<char *>(p) + bytes);
}
__device__ __forceinline__ Words words_of(const FusedParams &P, unsigned copy)
{
    const size_t off = copy ? P.copy_bytes : 0;
    Words W;
    W.ratio = shifted(P.words.ratio, off); W.lw = shifted(P.words.lw, off); W.rowres = shifted(P.words.rowres, off); W.pstat = shifted(P.words.pstat, off); W.plast = shifted(P.words.plast, off);
    W.pgrp = shifted(P.words.pgrp, off); W.qgrp = shifted(P.words.qgrp, off); W.spart = shifted(P.words.spart, off); W.lseen = shifted(P.words.lseen, off);
    return W;
}

// The same number, but one the compiler knows nothing about: what is computed from it is computed where it is used and
// not at the top of the kernel (where it would only be spilled until then).
__device__ __forceinline__ unsigned launder(unsigned v) { asm volatile("" : "+s"(v)); return v; }

// A barrier for what the waves of a workgroup hand each other through LDS: it orders LDS accesses only (a load from
// device memory that a wave has under way stays under way across it).
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// A load through the scalar data path for values that do not change while the kernel runs and whose address is the
// same for the whole wave (inputs; the call count of a sequence, which changes only after its last reader).  It
// does not queue behind the wave's sixteen-byte loads.
template <typename X> __device__ __forceinline__ X load_uniform(const X *p)
{
    return *reinterpret_cast<const __attribute__((address_space(4))) X *>(reinterpret_cast<uintptr_t>(p));
}

// ---- agent-scope accessors for words that other waves (on any XCD) write or read
// The words live in device memory.  The accesses say so: a pointer that went through arithmetic on bytes may otherwise
// count as generic, and a generic load is waited for wherever LDS or scalar loads are (and the other way round).
#define SV_GLOBAL(type, p) ((__attribute__((address_space(1))) type *)(p))
__device__ __forceinline__ int ld_i32(const int *p) { return __hip_atomic_load(SV_GLOBAL(const int, p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ unsigned ld_u32(const unsigned *p) { return __hip_atomic_load(SV_GLOBAL(const unsigned, p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_u32(unsigned *p, unsigned v) { __hip_atomic_store(SV_GLOBAL(unsigned, p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ unsigned pack_partial(float v) { return __float_as_uint(v) | 1u; }
__device__ __forceinline__ float unpack_partial(unsigned w) { return __uint_as_float(w & ~1u); }
__device__ __forceinline__ u64 ld_u64(const u64 *p) { return __hip_atomic_load(SV_GLOBAL(const u64, p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_u64(u64 *p, u64 v) { __hip_atomic_store(SV_GLOBAL(u64, p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ u64 pack_stat(float shift, float sum)
{
    return ((u64)__float_as_uint(sum) << 32) | (u64)__float_as_uint(shift);
}
__device__ __forceinline__ float stat_shift(u64 v) { return __uint_as_float((unsigned)(v & 0xffffffffull)); }
__device__ __forceinline__ float stat_sum(u64 v) { return __uint_as_float((unsigned)(v >> 32)); }
// (bit 0: the word is there; bit 1: test i + 1 of Alg. 1 passes, eta_{i+1} < min(r_{i+1}, 1), as its row's leader judged it)
__device__ __forceinline__ u64 pack_ratio(double log2r, bool passes) { return ((u64)__double_as_longlong(log2r) & ~3ull) | 1ull | (passes ? 2ull : 0ull); }
__device__ __forceinline__ double unpack_ratio(u64 v) { return __longlong_as_double((long long)(v & ~3ull)); }
__device__ __forceinline__ bool ratio_passes(u64 v) { return (v & 2ull) != 0; }
// (low half: whether the leader's own accept test passes; high half: the token it drew + 2, 1 if it drew none - so the
// word is never zero)
// (a token of kRowDrawDeferred: the position's residual has no mass; if it becomes tau, Y is drawn from its target row)
constexpr int kRowDrawDeferred = -3;
__device__ __forceinline__ u64 pack_rowres(bool passes, int token) { return ((u64)(unsigned)(token + 2) << 32) | (passes ? 1ull : 0ull); }
__device__ __forceinline__ bool rowres_passes(u64 v) { return (v & 1ull) != 0; }
__device__ __forceinline__ int rowres_token(u64 v) { return (int)(unsigned)(v >> 32) - 2; }
// What a wave publishes instead of a value once one of its waits has run out (or it has read this word itself):
// all ones, which no value packs to (as a float, a double or a pair of floats it would be a NaN).
constexpr u64 kPoison64 = ~0ull;
constexpr unsigned kPoison32 = ~0u;

// The value a given lane holds (lane index uniform over the wave).
__device__ __forceinline__ u64 read_lane_u64(u64 v, int lane)
{
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(v & 0xffffffffull), lane);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(v >> 32), lane);
    return ((u64)hi << 32) | lo;
}

// A word that is zero until its producer has written it: lanes with `need` poll *p until it is
// non-zero (`v` may already hold it).  One loop for the whole wave; gives up after `limit` polls, and counts a
// word of all ones (published by a wave that gave up) as having given up too.
__device__ __forceinline__ u64 wait_word(const u64 *p, u64 v, bool need, int limit, bool &gave_up)
{
    int spins = 0;
    while (__any(need && v == 0)) {
        if (++spins > limit) { gave_up = true; break; }
        __builtin_amdgcn_s_sleep(1);
        if (need && v == 0) v = ld_u64(p);
    }
    if (__any(need && v == kPoison64)) gave_up = true;
    return v;
}
__device__ __forceinline__ u64 wait_word(const u64 *p, int limit, bool &gave_up)
{
    return wait_word(p, ld_u64(p), true, limit, gave_up);
}

__device__ __forceinline__ unsigned wait_word32(const unsigned *p, unsigned v, bool need, int limit, bool &gave_up)
{
    int spins = 0;
    while (__any(need && v == 0)) {
        if (++spins > limit) { gave_up = true; break; }
        __builtin_amdgcn_s_sleep(1);
        if (need && v == 0) v = ld_u32(p);
    }
    if (__any(need && v == kPoison32)) gave_up = true;
    return v;
}
__device__ __forceinline__ unsigned wait_word32(const unsigned *p, int limit, bool &gave_up)
{
    return wait_word32(p, ld_u32(p), true, limit, gave_up);
}

// exp2 of a double of moderate size to a relative error below 1e-12: the integer part goes into the exponent,
// the fraction f in [-0.5, 0.5] through the series of exp(f ln 2) (|f ln 2| <= 0.347: ten terms).
__device__ __forceinline__ double exp2_precise(double x)
{
    const double n = rint(x);
    const double t = (x - n) * 0.69314718055994530942;
    double s = 1.0 / 3628800.0;
    s = s * t + 1.0 / 362880.0;
    s = s * t + 1.0 / 40320.0;
    s = s * t + 1.0 / 5040.0;
    s = s * t + 1.0 / 720.0;
    s = s * t + 1.0 / 120.0;
    s = s * t + 1.0 / 24.0;
    s = s * t + 1.0 / 6.0;
    s = s * t + 0.5;
    s = s * t + 1.0;
    s = s * t + 1.0;
    return ldexp(s, (int)n);
}

// 1 - 2^x for x <= 0 without the cancellation next to x = 0: the series of -expm1(x ln 2) where |x ln 2| < 0.35.
__device__ __forceinline__ double one_minus_exp2(double x)
{
    const double t = x * 0.69314718055994530942;
    if (t > -0.35) {
        double s = 1.0 / 39916800.0;
        s = s * t + 1.0 / 3628800.0;
        s = s * t + 1.0 / 362880.0;
        s = s * t + 1.0 / 40320.0;
        s = s * t + 1.0 / 5040.0;
        s = s * t + 1.0 / 720.0;
        s = s * t + 1.0 / 120.0;
        s = s * t + 1.0 / 24.0;
        s = s * t + 1.0 / 6.0;
        s = s * t + 0.5;
        s = s * t + 1.0;
        return -(s * t);
    }
    return 1.0 - exp2_precise(x);
}

// log2 of a positive double to an absolute error below 1e-12: the hardware's float log2 as a first guess g (off by
// about 1e-7), then log2 z = g + log2(z 2^-g) with z 2^-g - 1 of that size, where two terms of the series are enough.
__device__ __forceinline__ double log2_precise(double z)
{
    int e;
    const double m = frexp(z, &e);            // z = m * 2^e, m in [0.5, 1)
    const double g = (double)__builtin_amdgcn_logf((float)m);
    const double d = m * exp2_precise(-g) - 1.0;
    return (double)e + g + (d - 0.5 * d * d) * 1.4426950408889634074;
}

// A unit's exponentials are taken relative to an INTEGER shift, the smallest one that keeps them at or below 1:
// then sums of different units combine through exact powers of two.  The words carry the unit's largest scaled
// logit itself (the row's maximum is wanted too); this is the shift that belongs to it.
__device__ __forceinline__ float shift_of(float largest) { return largest > -INFINITY ? ceilf(largest) : 0.f; }

// Running combination of (largest scaled logit, sum) words: the sum of exp2 relative to the integer shift of the
// largest so far, in double (the factors between units are exact).
struct StatAcc {
    float m = -INFINITY;      // largest scaled logit so far
    double z = 0.0;
    __device__ __forceinline__ void add(u64 word)
    {
        const float mw = stat_shift(word);
        if (!(mw > -INFINITY)) return;                              // a unit without a finite logit
        const double s = (double)stat_sum(word);
        if (mw > m) {
            z = (m > -INFINITY ? ldexp(z, (int)(shift_of(m) - shift_of(mw))) : 0.0) + s;
            m = mw;
        } else {
            z += ldexp(s, (int)(shift_of(mw) - shift_of(m)));
        }
    }
    // the sum relative to the integer shift of another (larger or equal) maximum
    __device__ __forceinline__ double relative_to(float M) const
    {
        return m > -INFINITY ? ldexp(z, (int)(shift_of(m) - shift_of(M))) : 0.0;
    }
};

// The words of a row's n units as a wave holds them: lane l has entries l, l + 64, ... (NW of them).
template <int NW> struct RowWords { u64 w[NW]; };

// Issues the loads of a row's workgroup words (every second word from `words` on: the other row's lie between them;
// an entry that is still 0 is polled later).
template <int NW>
__device__ __forceinline__ void load_row_words(const u64 *words, int n, RowWords<NW> &r)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int q = 0; q < NW; ++q) {
        const int e = lane + q * kWave;
        r.w[q] = ld_u64(words + 2 * (e < n ? e : n - 1));
    }
}

// Largest scaled logit among a row's words, once all of them are there.
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

// ------------------------------------------------------------------ scans over the 64 lanes
// Inclusive scans through DPP: four shifts inside each row of 16 lanes (lanes without a source get 0), then the
// two row broadcasts.
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
// Lane j gets max(0, v_0, ..., v_j): a lane without a source contributes 0, which the result includes anyway.
__device__ __forceinline__ double wave_scan_max0(double v)
{
    v = fmax(v, 0.0);
    v = fmax(v, dpp_shift_double<0x111>(v));
    v = fmax(v, dpp_shift_double<0x112>(v));
    v = fmax(v, dpp_shift_double<0x114>(v));
    v = fmax(v, dpp_shift_double<0x118>(v));
    v = fmax(v, dpp_shift_double<0x142, 0xa>(v));
    v = fmax(v, dpp_shift_double<0x143, 0xc>(v));
    return v;
}
__device__ __forceinline__ double read_lane_double(double v, int lane)
{
    return __longlong_as_double((long long)read_lane_u64((u64)__double_as_longlong(v), lane));
}
// Sums over each half of the wave (lanes 0..31 and 32..63) at once, in double, through DPP in a fixed order: the
// pairs and quads of lanes, the two mirrors inside a row of 16, then the row broadcast that leaves the halves' sums
// in lanes 31 and 63.
__device__ __forceinline__ void halves_sum_f64(double v, double &first, double &second)
{
    v += dpp_shift_double<0xB1>(v);            // quad_perm:[1,0,3,2]
    v += dpp_shift_double<0x4E>(v);            // quad_perm:[2,3,0,1]
    v += dpp_shift_double<0x141>(v);           // row_half_mirror
    v += dpp_shift_double<0x140>(v);           // row_mirror
    v += dpp_shift_double<0x142, 0xa>(v);      // row_bcast15 into rows 1 and 3
    first = read_lane_double(v, 31);
    second = read_lane_double(v, 63);
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
            const u64 w = wait_word(words + 2 * (e < n ? e : n - 1), r.w[q], e < n, limit, gave_up);
            if (e < n) acc.add(w);
        }
    }
    const float M = wave_max(acc.m);
    double z0, z1;
    halves_sum_f64(acc.relative_to(M), z0, z1);
    const double z = z0 + z1;
    M_out = M;
    return (double)shift_of(M) + log2_precise(z);
}

// ------------------------------------------------------------------ the sequence's weights and what can matter
// log2 w_i for every position from the ratio words of positions 1 .. n (lane j holds the word of log2 r_{j+1} and gets
// log2 w_{j+1}).  Alg. 2: w_i = min(w_{i-1} r_i, 1), w_0 = 1; Alg. 4: without the min.  Alg. 1 has no w: there the value
// is 0 while every test up to the position has passed and kLog2RatioFloor afterwards (what the rule below asks).
__device__ __forceinline__ double weights_from_ratios(int algo, u64 ratio_word, int n)
{
    const int lane = threadIdx.x & 63;
    if (algo == kToken) {
        const u64 passed = __ballot(lane < n && ratio_passes(ratio_word));
        return (~passed & ((2ull << lane) - 1ull)) == 0 ? 0.0 : kLog2RatioFloor;
    }
    // log2 w_i = P_i - max(0, P_1, ..., P_i) with P_i = log2 r_1 + ... + log2 r_i: the recursion's min written out
    // (each time the product would exceed 1 it restarts from 1)
    const double P = wave_scan(lane < n ? unpack_ratio(ratio_word) : 0.0);
    return algo == kBlock ? P - wave_scan_max0(P) : P;
}
// The same one position further, as the leader of row pair i forms it for the workgroups of position i + 1 (calls in
// which the positions follow each other at a distance: one word to read instead of i + 1).
__device__ __forceinline__ double next_weight(int algo, double log2w_i, double log2r, bool passes)
{
    if (algo == kToken) return log2w_i > 0.5 * kLog2RatioFloor && passes ? 0.0 : kLog2RatioFloor;
    const double next = log2w_i + log2r;
    return algo == kBlock && next > 0.0 ? 0.0 : next;
}

// Whether position i (1 <= i <= the draft length) can become tau, given log2 w_i and the position's uniform.  The
// acceptance probability of block (and greedy block) verification never exceeds w_i: h_i = S_i / (S_i + 1 - w_i) with
// S_i <= w_i, and h_gamma = w_gamma.  So a test with eta_i >= w_i fails whatever S_i is, and tau is a position whose
// test passed, or 0.  Decided with a margin far above the rounding of h_i.  Token verification (Alg. 1) stops at the
// first failure: only a position that all tests up to its own let through can become tau.  Position 0 (nothing
// accepted) always can.  Every wave that asks - the waves of the position's workgroups, of the last target row's
// workgroups and the wave that finishes the sequence - evaluates this on the same numbers (the same published word, or
// the same scan over the same published ratios), so they always agree on which sums and which draws exist.
__device__ __forceinline__ bool can_become_tau(int algo, int i, double log2w_i, float eta_i)
{
    if (i == 0) return true;
    if (algo == kToken) return log2w_i > 0.5 * kLog2RatioFloor;
    return (double)__builtin_amdgcn_logf(eta_i) < log2w_i + 1.0e-3;
}
// Whether position i's residual mass is formed: where the position can become tau, and everywhere when the caller
// wants every S_i reported or the call is too small for leaving any out to pay.
__device__ __forceinline__ bool residual_needed(const FusedParams &P, int i, double log2w_i, float eta_i)
{
    return !P.prune || P.debug_out || can_become_tau(P.algo, i, log2w_i, eta_i);
}

// The workgroup's two words from its four waves' words in LDS (one wave: lanes 0..3 take the target row's, lanes 4..7
// the draft row's; each quad combines its four in a fixed order, the sums through exact powers of two).
__device__ __forceinline__ void publish_group_words(const u64 (&wave_words)[2][kWaves], u64 *pgrp_word, u64 *qgrp_word)
{
    const int lane = threadIdx.x & 63;
    const u64 w = wave_words[(lane >> 2) & 1][lane & 3];
    const float m = stat_shift(w);
    float M = fmaxf(m, __int_as_float(dpp_shift<0xB1>(__float_as_int(m))));            // quad_perm:[1,0,3,2]
    M = fmaxf(M, __int_as_float(dpp_shift<0x4E>(__float_as_int(M))));                   // quad_perm:[2,3,0,1]
    double z = m > -INFINITY ? ldexp((double)stat_sum(w), (int)(shift_of(m) - shift_of(M))) : 0.0;
    z += dpp_shift_double<0xB1>(z);
    z += dpp_shift_double<0x4E>(z);
    // (one store instruction for both words: lane 0 holds the target row's, lane 4 the draft row's)
    if (lane == 0 || lane == 4) st_u64(lane == 0 ? pgrp_word : qgrp_word, pack_stat(M, (float)z));
}

struct Unit {
    int b, i, c;          // sequence, position (gamma: the last target row, which has no draft row), wave chunk
    bool last_row;
};

// Workgroup order: groups of `group_seqs` sequences; inside a group the row pairs position-major
// (position, sequence, chunk), then the last target rows.
// The grid spells this out, (x, y, z) = (chunk / 4, sequence in group, group * (gamma + 1) + slot)
// with slot i for position i and slot gamma for the last target row; x runs fastest in the start order.
// Returns false for the padding of a last, smaller group.
__device__ __forceinline__ bool decode_unit(const FusedParams &P, int wave, Unit &U, int &x)
{
    int grp = 0, slot = blockIdx.z;
    if (P.B > P.group_seqs) { grp = (int)__umulhi(blockIdx.z, P.inv_slots); slot = blockIdx.z - grp * (P.gamma + 1); }
    U.b = grp * P.group_seqs + blockIdx.y;
    // which of the row's workgroups takes which chunk rotates from row to row: a row's workgroups go to the
    // XCDs round-robin, and the last chunk (fewest logits, leader's duties) must not always meet the same XCD
    const int wpr = P.nu / kWaves;                        // (= gridDim.x)
    const unsigned turn = blockIdx.x + blockIdx.y + blockIdx.z;
    x = wpr == 1 ? 0 : (int)(turn - __umulhi(turn, P.inv_wpr) * (unsigned)wpr);      // (2^32 / 1 + 1 does not fit the word)
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
                raw.v[v] = load_streamed(base + (lane_off + (unsigned)(v * kWave * 16)));
        } else {
#pragma unroll
            for (int v = 0; v < RawSlice<T, true, LANE>::kNV; ++v) {
                const unsigned off = lane_off + (unsigned)(v * kWave * 16);
                // vectors beyond the row are recognised again when the slice is unpacked; load something valid
                raw.v[v] = load_streamed(base + (off < (unsigned)V * (unsigned)sizeof(T) ? off : 0u));
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
// the wave-uniform integer shift that belongs to the unit's largest scaled logit (shift_of; 0 when the whole unit
// lies beyond the row).  Returns the unit's word: (k * largest logit, sum of the exponentials); (-inf, 0) beyond.
template <int LANE>
__device__ __forceinline__ u64 first_sweep_row(float (&x)[LANE], float k, float &shift)
{
    float m = x[0];
#pragma unroll
    for (int j = 1; j < LANE; ++j) m = fmaxf(m, x[j]);
    const float Mw = wave_max(m * k);
    shift = shift_of(Mw);
    float acc[4] = {0.f, 0.f, 0.f, 0.f};     // four partial sums: shorter chains, smaller rounding error
#pragma unroll
    for (int j = 0; j < LANE; ++j) {
        x[j] = fast_exp2(__builtin_fmaf(x[j], k, -shift));
        acc[j & 3] += x[j];
    }
    const float sw = wave_sum((acc[0] + acc[1]) + (acc[2] + acc[3]));
    return pack_stat(Mw, sw);
}

// Tuning builds (-DSV_PROFILE) store up to sixteen timestamps per workgroup, taken by its first lane, into the
// workgroup's record `stamps`; the default build has none of it.
#ifdef SV_PROFILE
#define SV_STAMP(slot) do { if (stamps && threadIdx.x == 0) stamps[slot] = wall_clock64(); } while (0)
#define SV_NOTE(slot, value) do { if (stamps && threadIdx.x == 0) stamps[slot] = (value); } while (0)
#else
#define SV_STAMP(slot) do { } while (0)
#define SV_NOTE(slot, value) do { } while (0)
#endif

// ------------------------------------------------------------------ the accept test of one position
// Alg. 2 / Alg. 4, position j >= 1 (j < the draft length): eta_j < h_j with h_j = S_j / (S_j + 1 - w_j), 1 where
// w_j >= 1.  Greedy (Alg. 4) divides by the rejected mass sum_x max(q - w p, 0) instead, which is the same number: it
// equals S - sum_x (w p - q) = S + 1 - w because both rows sum to one (w unclipped; at w >= 1 the ratio is >= 1 and
// every eta in [0, 1) passes).  `log2w`: log2 w_j (greedy: capped so that w stays finite).
struct AcceptTest {
    double log2w;
    float eta;
    bool allowed;         // false: the position cannot become tau whatever S_j is (can_become_tau): the test counts as failed
    bool passes;          // out
    double w, h;          // out, for the debug block
    __device__ __forceinline__ void evaluate(double S)
    {
        w = exp2_precise(log2w);
        h = log2w >= 0.0 ? 1.0 : S / (S + one_minus_exp2(fmin(log2w, 0.0)));
        passes = allowed && (double)eta < h;
    }
};

// ------------------------------------------------------------------ the draw of a token
// Row `row` of sequence b (one wave).  First the sum of the weights: mode 0, the residual max(w p - q, 0) of row pair
// `row`, by the partial sums per wave chunk that the pair's units publish (polled here until all are there); mode 1,
// p_row itself, by the target row's words `st` (one per wave chunk).  `total_out` gets that sum (mode 0: S_row).  Then, if
// `want_draw`, the inverse-CDF draw in index order, first token whose running sum exceeds u * total: the wave chunk
// that holds it by a scan over the chunks' sums, then the token by the weights of that one chunk, formed again from
// the logits with alpha_p = L_p - log2 w and alpha_q = L_q.  A residual without any mass is drawn from p_row
// instead.  `test`, if `has_test`: the position's accept test, evaluated on the sum as soon as it is there; nothing is
// drawn where it fails.  Returns the token, or -1 if none was asked for.
template <typename T, bool ALIGNED, int LANE>
__device__ __forceinline__ int draw_from_row(const FusedParams &P, const Words &W, const u64 *st, int b, int row, int mode, bool want_draw,
                                             bool has_test, AcceptTest &test, double alpha_p, double alpha_q, float u, double &total_out, bool &gave_up)
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
    const unsigned *sp = W.spart + drow * nu;

    // ---- first the wave chunk that holds t = u * total ...
    float Mrow = 0.f;
    RowCoef rc = {};
    if (mode == 0) rc = make_row_coef(alpha_p, alpha_q);
    else Mrow = row_max_shift(st, nu, P.spin_limit, gave_up);
    int slot = -1, last_nonzero = 0;
    double t_in = 0.0;
    total_out = 0.0;
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
                    if (e < nu && sh > -INFINITY) part = ldexp((double)stat_sum(v), (int)(shift_of(sh) - shift_of(Mrow)));
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
            if (pass_no == 0) {
                total = carry; t = (double)u * total;
                if (attempt == 0) {
                    total_out = total;
                    if (has_test) { test.evaluate(total); want_draw = want_draw && test.passes; }
                }
                if (!want_draw) return -1;
            }
        }
        if (slot < 0) {
            // no residual mass: Y would be drawn from p_row itself, which takes a sweep over the whole row by this one
            // wave (draw_from_target_row) - left to whoever finishes the sequence, and only if this position is tau
            if (mode == 0 && !(total > 0.0)) {
                if constexpr (kLazyRowWords<LANE>) return kRowDrawDeferred;
                mode = 1;                                               // (larger units: the row's words are there)
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
    // (the sixteen-byte path asks for the whole chunk at once and keeps it as loaded until each vector's turn)
    uint4 rp[ALIGNED ? kNV : 1], rq[ALIGNED ? kNV : 1];
    if constexpr (ALIGNED) {
#pragma unroll
        for (int v = 0; v < kNV; ++v) {
            const int idx = first + v * kWave * kVec;
            rp[v] = *reinterpret_cast<const uint4 *>(prow + (idx < V ? idx : 0));
            if (mode == 0) rq[v] = *reinterpret_cast<const uint4 *>(qrow + (idx < V ? idx : 0));
        }
    }
    float shift = 0.f, scale = 1.f;
    if (mode != 0) {
        const u64 sv = wait_word(st + slot, P.spin_limit, gave_up);
        shift = shift_of(stat_shift(sv)); scale = ldexpf(1.f, (int)(shift - shift_of(Mrow)));
    }
    float t = mode == 0 ? (float)(t_in / (double)rc.cq) : (float)t_in;
    int y = -1, last_positive = -1;
#pragma unroll
    for (int v = 0; v < kNV; ++v) {
        const int idx = first + v * kWave * kVec;
        float wgt[kVec], xpv[kVec], xqv[kVec];
        if constexpr (ALIGNED) {
            unpack_vec<T>(rp[v], xpv);
            if (mode == 0) unpack_vec<T>(rq[v], xqv);
            if (idx >= V) {
#pragma unroll
                for (int e = 0; e < kVec; ++e) { xpv[e] = -INFINITY; xqv[e] = -INFINITY; }
            }
        } else {
            load_vec<T, false>(prow, V, idx, xpv);
            if (mode == 0) load_vec<T, false>(qrow, V, idx, xqv);
        }
        if (mode == 0) {
#pragma unroll
            for (int e = 0; e < kVec; ++e) wgt[e] = fmaxf(residual_term(xpv[e], xqv[e], k, rc), 0.f);
        } else {
#pragma unroll
            for (int e = 0; e < kVec; ++e) wgt[e] = fast_exp2(__builtin_fmaf(xpv[e], k, -shift)) * scale;
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

// Y from p_row for a row pair's target row whose residual has no mass (Alg. 1 / 2 / 4 draw from the residual; where
// rounding leaves none of it, from the row itself: in exact arithmetic such a position cannot become tau).  The units of
// a row pair publish no word of their own per wave chunk - nobody reads them on any other path - so the wave that needs
// them forms them here, chunk by chunk with the units' own arithmetic, into the row's words `pstat` (which only it
// uses), and then draws as from a last target row.  A whole row through one wave: tens of microseconds, on a path that
// consistent inputs do not take.
template <typename T, bool ALIGNED, int LANE>
__device__ __forceinline__ int draw_from_target_row(const FusedParams &P, const Words &W, int b, int row, float u, bool &gave_up)
{
    constexpr int kUnitLogits = kWave * LANE;
    const int lane = threadIdx.x & 63;
    const int nu = P.nu;
    u64 *st = W.pstat + ((size_t)b * P.gamma + row) * nu;
    const T *prow = static_cast<const T *>(P.target) + ((size_t)b * (P.gamma + 1) + row) * P.tstride;
    for (int c = 0; c < nu; ++c) {
        RawSlice<T, ALIGNED, LANE> raw;
        float x[LANE], shift;
        issue_loads<T, ALIGNED, LANE>(prow, c * kUnitLogits, P.V, raw);
        unpack_slice<T, ALIGNED, LANE>(prow, c * kUnitLogits, P.V, raw, x);
        const u64 word = first_sweep_row(x, P.k, shift);
        if (lane == 0) st_u64(st + c, word);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // the words are in memory before they are read back
    AcceptTest none = {};
    double total;
    const int y = draw_from_row<T, ALIGNED, LANE>(P, W, st, b, row, 1, true, false, none, 0.0, 0.0, u, total, gave_up);
    for (int c = lane; c < nu; c += kWave) st_u64(st + c, 0);      // (nobody clears these words for this kernel)
    return y;
}

// ------------------------------------------------------------------ whole sequences
// Whether a row's per-wave words of the target row may hold anything: always for the kernel that publishes them, else
// only if such a kernel has worked on this workspace since it was prepared.
template <int LANE> __device__ __forceinline__ bool row_words_used(const int *header)
{
    if constexpr (!kLazyRowWords<LANE>) return true;
    else return load_uniform(header + kHdrRowWords) != 0;
}

// Clears the words of row slot `slot` of sequence b in one copy (one wave, all lanes, whole rows at a time: full
// cache lines).  Slot gamma holds the words of the sequence's last target row and nothing else.
__device__ __forceinline__ void clear_row_words(const FusedParams &P, const Words &W, int b, int slot, bool row_words)
{
    const int lane = threadIdx.x & 63;
    const int G = P.gamma, nu = P.nu, nwg = nu / kWaves;
    if (slot == G) {
        for (int e = lane; e < nu; e += kWave) st_u64(W.plast + (size_t)b * nu + e, 0);
        for (int e = lane; e < nwg; e += kWave) st_u64(W.lseen + (size_t)b * nwg + e, 0);
        return;
    }
    const size_t drow = (size_t)b * G + slot;
    for (int e = lane; e < nu; e += kWave) { if (row_words) st_u64(W.pstat + drow * nu + e, 0); st_u32(W.spart + drow * nu + e, 0); }
    for (int e = lane; e < 2 * nwg; e += kWave) st_u64(W.pgrp + 2 * drow * nwg + e, 0);
    if (lane == 0) { st_u64(W.ratio + drow, 0); st_u64(W.lw + drow, 0); st_u64(W.rowres + drow, 0); }
}

// A wait of this wave has run out (or it has read a word of a wave that gave up): the workspace's error word says so
// to whoever checks the workspace.
__device__ __forceinline__ void report_gave_up(const FusedParams &P)
{
    if ((threadIdx.x & 63) == 0 && ld_i32(P.header + kHdrError) == 0) atomicOr(P.header + kHdrError, 1);
}

// ------------------------------------------------------------------ the kernel
// The kernel's arguments once more, read from the kernel argument segment where a rarely taken part of the kernel
// begins: what that part needs of them then lives in registers from there on, and not from the top of the kernel
// through its hot part (where it would only be parked in lanes of a vector register and fetched back).
__device__ __forceinline__ FusedParams reread_params()
{
    typedef __attribute__((address_space(4))) const unsigned char ArgByte;
    ArgByte *kp = (ArgByte *)__builtin_amdgcn_kernarg_segment_ptr();      // (FusedParams is the only argument)
    asm volatile("" : "+s"(kp));
    FusedParams Q;
#define SV_ARG(f) Q.f = *reinterpret_cast<__attribute__((address_space(4))) const decltype(Q.f) *>(kp + offsetof(FusedParams, f))
    SV_ARG(target); SV_ARG(draft); SV_ARG(tokens); SV_ARG(draft_lens); SV_ARG(uniforms); SV_ARG(B); SV_ARG(gamma); SV_ARG(V);
    SV_ARG(tstride); SV_ARG(dstride); SV_ARG(k); SV_ARG(kd); SV_ARG(k_eps); SV_ARG(algo); SV_ARG(nu); SV_ARG(group_seqs);
    SV_ARG(inv_slots); SV_ARG(inv_wpr); SV_ARG(prune); SV_ARG(skip_last); SV_ARG(spin_limit);
    SV_ARG(magic); SV_ARG(header); SV_ARG(gen); SV_ARG(copy_bytes); SV_ARG(accept_len); SV_ARG(next_token); SV_ARG(debug_out);
    SV_ARG(words.ratio); SV_ARG(words.lw); SV_ARG(words.rowres); SV_ARG(words.pstat); SV_ARG(words.plast);
    SV_ARG(words.pgrp); SV_ARG(words.qgrp); SV_ARG(words.spart); SV_ARG(words.lseen);
#ifdef SV_PROFILE
    SV_ARG(prof);
#endif
#undef SV_ARG
    return Q;
}

// ------------------------------------------------------------------ the leader of a row pair
// One wave, the first of the last workgroup of row pair i of sequence b, once the row's ratio is out (and, where the
// row's residual mass is formed, the wave's own share of it): what position i contributes to tau and Y.  Alg. 2 / 4:
// the position's own accept test, eta_i < h_i, needs S_i, the sum of the row's partial sums; where it passes (and at
// position 0, which is tau when no test passes) the leader draws the token that follows if this position becomes tau.
// Alg. 1: the test of X_{i+1} was judged with the ratio; the position is tau where every test up to it has passed and
// that one fails.  All of it happens while the later positions are still streaming: the leader of the sequence's last
// row pair (`finisher`; gb is the sequence's draft length) then only picks up one word per position, judges the last
// test, eta_gamma < w_gamma, writes tau and Y and hands the sequence's words over to the next call.
// (A row whose residual mass is not formed has nothing to wait for here: its test fails.)
// `values`: the row's L_p, L_q and log2 w_i as the wave left them in LDS; `res`: the finisher's first look at the
// earlier positions' words (lane l: position l; 0 where the word was not there yet).
template <typename T, bool ALIGNED, int LANE>
__device__ __forceinline__ void lead_row(int b, int i_own, int gb, unsigned par, bool needed, bool candidate, bool finisher, u64 own_word,
                                         double lw_next, u64 res, float eta_i, float eta_next, bool gave_up, const double *values, long long *stamps)
{
    const FusedParams P = reread_params();
    const int lane = threadIdx.x & 63;
    const int nu = P.nu;
    const size_t seq_d = (size_t)b * P.gamma, seq_u = (size_t)b * (P.gamma + 1), drow = seq_d + i_own;
    SV_STAMP(5);
    const Words W = words_of(P, par);
    const double Lp = values[0], Lq = values[1], log2w_row = values[2];
    const float u = load_uniform(P.uniforms + seq_u + gb);
    const bool token_algo = P.algo == kToken;
    const bool next_passes = ratio_passes(own_word);             // Alg. 1: the test of X_{i+1}
    // the finisher's first loads: the earlier positions' words (lane l: position l)
    const u64 *const res_word = W.rowres + seq_d + (lane < gb - 1 ? lane : 0);
    const u64 *const last = W.plast + (size_t)b * nu;
    // the test of the last position, eta_gamma < h_gamma = w_gamma (Alg. 2 / 4), which the finisher judges first: where
    // it passes, tau = gamma and nothing of this row's residual is needed
    double w_last = 1.0;
    bool last_passes = next_passes;                              // Alg. 1: the test of X_gamma
    if (finisher && !token_algo) {
        w_last = exp2_precise(P.algo == kGreedy ? fmin(lw_next, 100.0) : lw_next);
        last_passes = (double)eta_next < fmin(w_last, 1.0);
    }
    AcceptTest test;
    test.log2w = log2w_row; test.eta = eta_i; test.allowed = candidate; test.passes = false; test.w = 1.0; test.h = 1.0;
    const bool has_test = !token_algo && i_own > 0;
    // where the draw is wanted if the position's own test lets it through
    bool want = token_algo ? candidate && !next_passes : true;
    if (finisher && !token_algo && last_passes) want = false;
    double S_own = 0.0;
    int drawn = -1;
    if (needed && (want || has_test || P.debug_out))
        drawn = draw_from_row<T, ALIGNED, LANE>(P, W, W.pstat + drow * nu, b, i_own, 0, want, has_test, test,
                                                Lp - log2w_row, Lq, u, S_own, gave_up);
    const bool own_passes = token_algo ? next_passes : has_test && test.passes;
    if (P.debug_out && lane == 0) {
        // row i of the block: (w_i, S_i, h_i); Alg. 1 has no w, and its h_i = min(r_i, 1) comes from the ratio that
        // the leader of the position before published
        float *d = P.debug_out + (seq_u + i_own) * 3;
        double h_i = test.h;
        if (token_algo && i_own > 0) h_i = exp2_precise(fmin(unpack_ratio(wait_word(W.ratio + drow - 1, P.spin_limit, gave_up)), 0.0));
        d[0] = i_own > 0 && !token_algo ? (float)test.w : 1.f; d[1] = (float)S_own; d[2] = i_own > 0 ? (float)h_i : 1.f;
    }
    if (!finisher) {
        if (gave_up) report_gave_up(P);
        if (lane == 0) st_u64(W.rowres + drow, gave_up ? kPoison64 : pack_rowres(own_passes, drawn));
        SV_STAMP(15);
        return;
    }

    // ---- the leader of a sequence's last row pair finishes the sequence: one word per earlier position
    res = wait_word(res_word, res, lane < gb - 1, P.spin_limit, gave_up);
    const u64 flags = __ballot(lane < gb - 1 && rowres_passes(res));                 // bit l: position l's word says "passes"
    int tau;
    if (token_algo) {
        // bit l: the test of X_{l+1}; tau is the length of the leading run of passes
        const u64 tests = flags | ((u64)(last_passes ? 1 : 0) << (gb - 1));
        tau = __ffsll((long long)~tests) - 1;
        if (tau < 0 || tau > gb) tau = gb;                       // (a draft of 64 tokens, all accepted: no zero bit)
    } else {
        // bit l: the test of position l (none at position 0); tau is the last position whose test passes, else 0
        // (the last position's test apart: with a draft of 64 tokens it has no bit in the word)
        const u64 tests = (flags & ~1ull) | ((u64)(own_passes ? 1 : 0) << (gb - 1));
        tau = last_passes ? gb : tests ? 63 - __clzll((long long)tests) : 0;
    }
    if (lane == 0) P.accept_len[b] = tau;
    if (P.debug_out && lane == 0) {
        float *d = P.debug_out + (seq_u + gb) * 3;       // S_gamma = w_gamma: q_gamma == 0
        d[0] = (float)w_last; d[1] = (float)w_last;
        d[2] = token_algo ? (float)exp2_precise(fmin(unpack_ratio(own_word), 0.0)) : (float)fmin(w_last, 1.0);
    }
    SV_STAMP(10);
    int y;
    if (tau == gb) {
        // every token was accepted: Y comes from the last target row itself
        double total;
        y = draw_from_row<T, ALIGNED, LANE>(P, W, last, b, gb, 1, true, false, test, 0.0, 0.0, u, total, gave_up);
    } else if (tau == gb - 1) {
        y = drawn;
    } else {
        y = rowres_token(read_lane_u64(res, tau));
    }
    if constexpr (kLazyRowWords<LANE>) {
        if (y == kRowDrawDeferred) y = draw_from_target_row<T, ALIGNED, LANE>(P, W, b, tau, u, gave_up);
    }
    SV_STAMP(12);
    if (gave_up) report_gave_up(P);
    if (lane == 0) {
        // a wait that ran out anywhere on the way here leaves nothing to trust
        if (gave_up) { P.accept_len[b] = -1; y = -1; }
        P.next_token[b] = y;
    }
    SV_STAMP(6);
}

template <typename T, bool ALIGNED, int NW, int LANE>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(LANE == kLaneLarge ? 3 : ElemTraits<T>::kVec == 8 ? SV_WAVES_SMALL : 4)))
void fused_verify_kernel(const FusedParams P)
{
    constexpr int kUnitLogits = kWave * LANE;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int gamma = P.gamma, V = P.V, nu = P.nu;
    const float k = P.k;

    // Everything the first loads need comes out of the kernel's arguments in one go (one wait for the scalar loads
    // instead of one per branch below) ...
    const T *const target = static_cast<const T *>(P.target), *const draft = static_cast<const T *>(P.draft);
    const size_t tstride = P.tstride, dstride = P.dstride;
    const int32_t *const draft_lens = P.draft_lens;
    const int *const header = P.header, *const gen = P.gen;
    asm volatile("" :: "s"(target), "s"(draft), "s"(tstride), "s"(dstride), "s"(draft_lens), "s"(header), "s"(gen),
                       "s"(gamma), "s"(V), "s"(nu), "s"(P.B), "s"(P.group_seqs), "s"(P.magic));
    Unit U;
    int wg_x;
    if (!decode_unit(P, wave, U, wg_x)) return;
    const int slot = U.i;
    long long *stamps = nullptr;
#ifdef SV_PROFILE
    // one record per (sequence, slot, workgroup of the row): never beyond B * (gamma + 1) * workgroups per row records
    if (P.prof) stamps = P.prof + (((size_t)U.b * (gamma + 1) + slot) * (nu / kWaves) + blockIdx.x) * 16;
#endif
    SV_STAMP(0);
    // a sequence with a shorter draft has no row pairs at its unused positions, and its last target row is row gb
    int gb = gamma;
    if (draft_lens) { gb = load_uniform(draft_lens + U.b); gb = gb < 1 ? 1 : gb > gamma ? gamma : gb; }   // kept in range whatever the caller wrote
    const bool unused = !U.last_row && U.i >= gb;
    if (U.last_row) U.i = gb;

    // stream A: the unit's chunk of target row i; stream B: the same chunk of draft row i (none for the last row)
    const size_t seq_d = (size_t)U.b * gamma, seq_u = (size_t)U.b * (gamma + 1);
    const size_t trow = seq_u + U.i, drow = seq_d + (U.last_row ? 0 : U.i);
    const T *rowA = target + trow * tstride;
    const T *rowB = draft + drow * dstride;
    const int unit_first = U.c * kUnitLogits;
    const int nwg = nu / kWaves;
    // ... and a row pair's loads go out before anything is asked of the workspace: they depend on the arguments only
    RawSlice<T, ALIGNED, LANE> rawA, rawB;
    if (!U.last_row && !unused) {
        issue_loads<T, ALIGNED, LANE>(rowA, unit_first, V, rawA);
        issue_loads<T, ALIGNED, LANE>(rowB, unit_first, V, rawB);
    }
    asm volatile("" ::: "memory");      // (keeps the two scalar loads below from being waited for in front of them)
    const int magic_word = load_uniform(header + kHdrMagic);
    const unsigned par = (unsigned)load_uniform(gen + U.b) & 1u;
    if (magic_word != P.magic) {
        // the workspace was not initialised for this shape: report it through the outputs and leave
        if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0)
            for (int b = threadIdx.x; b < P.B; b += kThreads) { P.accept_len[b] = -1; P.next_token[b] = -1; }
        return;
    }
    // every row slot's words are cleared, in the copy that this call does not use, by the first wave of the slot's
    // last workgroup (the row's leader, where there is a row)
    const bool clears = wave == 0 && wg_x == nwg - 1;
    if (unused) {
        // the copy in use holds nothing at an unused position; the other may hold an earlier, longer call's words:
        // both are cleared, which needs no look at the call count
        if (clears) { const bool rw = row_words_used<LANE>(header); clear_row_words(P, P.words, U.b, slot, rw); clear_row_words(P, words_of(P, 1), U.b, slot, rw); }
        return;
    }
    // (the copy of the words this call uses for the sequence - see the head of this file - is `par`; the addresses in it
    // are formed block by block where they are used: the kernel is short of scalar registers)
#define SV_WORDS words_of(P, launder(par))

    __shared__ u64 wave_words[2][kWaves];
    __shared__ double row_values[8];
    __shared__ int row_flag;
    __shared__ unsigned wave_shares[kWaves];
    bool gave_up = false;

    // Two ways to w_i.  Calls larger than one resident set ("chain"): the leader of row pair i - 1 publishes log2 w_i
    // itself, one word that the workgroups of position i read at their start - position i starts up to a resident set
    // after position i - 1 (where a position is less than that, the word is often not there yet, and a second look goes
    // out with the workgroup's own words).  Smaller calls, where all positions run at once: the first wave of a
    // workgroup reads the ratios of all earlier positions (lane j: the word of log2 r_{j+1}) and forms w_i from them.
    const int n_prev = U.i;                                   // ratios that w_i is made of
    const bool chain = P.prune != 0;
#define SV_RATIO_WORD (W.ratio + seq_d + (lane < n_prev ? lane : 0))
#define SV_LW_WORD (W.lw + seq_d + (n_prev > 0 ? n_prev - 1 : 0))

    if (U.last_row) {
        // ---- the last target row: needed only if every token is accepted (then Y ~ p_gamma, Alg. 1 / 2 / 4).  In
        // calls large enough for it to pay, its workgroups first look at w_gamma: where eta_gamma >= w_gamma (Alg. 1:
        // where some test fails) the row is not read at all, and nothing is said about it: nobody will ask.
        if (clears) clear_row_words(P, words_of(P, par ^ 1u), U.b, slot, false);       // (slot gamma holds no such words)
        const Words W = SV_WORDS;
        // The row's workgroups are the sequence's last to start.  Each says so once it has read gen[b] (the word hangs on
        // the value read); the last of them hands the sequence's words over to the next call - it flips gen[b] - as soon
        // as it has its siblings' words and proof that every row pair's workgroups have read gen[b] too: a word that the
        // sequence's last row pair publishes only after all of them have published theirs.
        u64 seen = 0;
        if (wave == 0) {
            if (lane == 0 && !clears) st_u64(W.lseen + (size_t)U.b * nwg + wg_x, 1ull + (launder(par) >> 1));
            if (clears) seen = ld_u64(W.lseen + (size_t)U.b * nwg + (lane < nwg - 1 ? lane : 0));
        }
        auto hand_over = [&]() {
            // (first wave of the row's last workgroup)
            wait_word(W.lseen + (size_t)U.b * nwg + (lane < nwg - 1 ? lane : 0), seen, lane < nwg - 1, P.spin_limit, gave_up);
            for (int e = lane + kWave; e < nwg - 1; e += kWave) wait_word(W.lseen + (size_t)U.b * nwg + e, P.spin_limit, gave_up);
            if (lane == 0) __hip_atomic_store(P.gen + U.b, (int)(par ^ 1u), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        };
        if (P.skip_last) {
            if (wave == 0) {
                const float eta_g = load_uniform(P.uniforms + seq_u + gb - 1);
                const u64 wt = wait_word(SV_LW_WORD, P.spin_limit, gave_up);
                if (clears) hand_over();                     // (the word of log2 w_gamma is such a proof)
                const bool wanted = can_become_tau(P.algo, gb, unpack_ratio(wt), eta_g);
                if (lane == 0) row_flag = gave_up ? 2 : wanted ? 0 : 1;
                if (gave_up) report_gave_up(P);
            }
            __syncthreads();
            const int flag = row_flag;
            if (flag != 0) {
                // (nobody asks for the words of a row that cannot be drawn from; a wait that ran out is passed on)
                if (flag == 2 && lane == 0) st_u64(W.plast + (size_t)U.b * nu + U.c, kPoison64);
                SV_STAMP(11);
                return;
            }
        }
        issue_loads<T, ALIGNED, LANE>(rowA, unit_first, V, rawA);
        float xa[LANE], shiftA;
        unpack_slice<T, ALIGNED, LANE>(rowA, unit_first, V, rawA, xa);
        const u64 stA = first_sweep_row(xa, k, shiftA);
        if (lane == 0) st_u64(W.plast + (size_t)U.b * nu + U.c, stA);
        if (!P.skip_last && clears) {
            // (calls whose last target rows ask nobody: the proof is the ratio of every position)
            wait_word(W.ratio + seq_d + (lane < gb ? lane : 0), 0, lane < gb, P.spin_limit, gave_up);
            if (gave_up) report_gave_up(P);
            hand_over();
        }
        return;
    }

    // draft token X_{i+1} and its two logits: the first wave of the row's last workgroup (the one with the
    // fewest logits) publishes the row's ratio from them
    const bool leader = wave == 0 && wg_x == nwg - 1;
    // whether the workgroup finds out right after its first sweep if the row's residual mass can matter at all
    const bool early = chain && !P.debug_out && n_prev > 0;
    u64 wt = 0;                                              // chain: the word of log2 w_i; else, first wave: lane j's ratio word
    float eta_i = 0.f, eta_next = 0.f;                       // the uniforms of test i (this position's) and test i + 1
    int tok = 0;                                             // the drafted token X_{i+1}, for the leader
    if (wave == 0) {
        const Words W = SV_WORDS;
        eta_i = load_uniform(P.uniforms + seq_u + (n_prev > 0 ? n_prev - 1 : 0));
        // (chain: the word of log2 w_i is asked for once the sweeps are done - at a workgroup's start it is there for one
        // workgroup in six only, and a look that finds nothing is one more small read between the streaming ones)
        if (!chain) wt = ld_u64(SV_RATIO_WORD);
    }
    if (wave == 0) {
        tok = load_uniform(P.tokens + drow);
        eta_next = load_uniform(P.uniforms + seq_u + n_prev);
    }
    if (clears) {
        clear_row_words(P, words_of(P, par ^ 1u), U.b, slot, row_words_used<LANE>(header));
        if constexpr (!kLazyRowWords<LANE>) {
            if (lane == 0) __hip_atomic_store(SV_GLOBAL(int, P.header + kHdrRowWords), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }

    // ---- first sweep: exponentials stay in xa / xb; the unit's words go out
    float xa[LANE], xb[LANE];
    float shiftA, shiftB;
    unpack_slice<T, ALIGNED, LANE>(rowA, unit_first, V, rawA, xa);
    const u64 stA = first_sweep_row(xa, k, shiftA);
    // (the draft row's logits are taken out of their load registers before anything else is sent to memory: the
    // hardware counts outstanding loads and stores in one counter, in order, and a wait for these loads placed after
    // a store would be a wait for that store's acknowledgement too)
    unpack_slice<T, ALIGNED, LANE>(rowB, unit_first, V, rawB, xb);
    // (smaller units: the target row's word of this wave, stA, goes to the workgroup's word only - per wave chunk nobody
    // needs it but a draw from the row itself, which forms it again where it happens: 36 864 stores less per call at
    // B = 64, gamma = 8, V = 128256, 52.2 -> 51.1 us)
    if constexpr (!kLazyRowWords<LANE>) {
        if (lane == 0) st_u64(SV_WORDS.pstat + drow * nu + U.c, stA);
    }
    // the two logits of the draft token, asked for only now so that the streams above did not queue behind them, and
    // left as loaded until they are needed: the row's words will have come in by then, and these with them
    uint32_t ya_bits = 0, yb_bits = 0;
    if (leader) { ya_bits = logit_bits(rowA + tok); yb_bits = logit_bits(rowB + tok); }
    const u64 stB = first_sweep_row(xb, k, shiftB);
    // the wave's two words meet the other waves' in LDS; the first wave publishes the workgroup's two words and, in
    // calls larger than one resident set, decides whether this row's residual mass can matter: a row that is not needed
    // costs its workgroups no wait for the row
    if (lane == 0) { wave_words[0][wave] = stA; wave_words[1][wave] = stB; }
    __syncthreads();
    double log2w = 0.0;
    if (wave == 0) {
        SV_STAMP(1);
        const Words W = SV_WORDS;
        // (where the look at the start came too early for the chain's word, the second look goes out in front of the
        // workgroup's own words: one round trip for both, not one after the other)
        if (early) SV_NOTE(14, read_lane_u64(wt, 0) != 0 ? 1 : 2);
        if (early && read_lane_u64(wt, 0) == 0) wt = ld_u64(SV_LW_WORD);
        publish_group_words(wave_words, W.pgrp + 2 * (drow * nwg + wg_x), W.qgrp + 2 * (drow * nwg + wg_x));
        bool wanted = true;
        if (early) {
            wt = wait_word(SV_LW_WORD, wt, true, P.spin_limit, gave_up);
            SV_STAMP(13);
            log2w = unpack_ratio(read_lane_u64(wt, 0));
            wanted = gave_up || can_become_tau(P.algo, U.i, log2w, eta_i);
        }
        if (lane == 0) row_flag = wanted ? 1 : 0;
    }
    __syncthreads();
    const bool needed = row_flag != 0;
    // the leader of a sequence's last row pair finishes the sequence: what it works out for its row it has at hand
    const bool finisher = leader && U.i == gb - 1;
    // a row whose residual mass cannot matter: only its leader (the later positions need this row's ratio; the
    // last one finishes the sequence) stays; everybody else is done and frees its registers
    if (!needed && !leader) return;

    bool candidate = true;           // whether this position can become tau: then its leader draws the token that would follow
    u64 own_word = 0;                // the leader's word of log2 r_{i+1}
    double lw_next = 0.0;            // the leader's log2 w_{i+1}
    u64 res_first = 0;               // the finisher's first look at the earlier positions' words (lane l: position l)
    if (wave == 0) {
        // ---- L_p, L_q: the words of all workgroups of the row
        const Words W = SV_WORDS;
        // (the earlier positions have had a row's lifetime to publish what they contribute: asked for now, their words
        // come in with the row's, and the finisher does not wait for them at the end)
        if (finisher && gb > 1) res_first = ld_u64(W.rowres + seq_d + (lane < gb - 1 ? lane : 0));
        // Alg. 2 / 4 keep the LAST position whose test passes, and test i + 1 passes whatever its uniform is where
        // w_{i+1} >= 1 (h_{i+1} = 1; the last test: eta < min(w, 1)).  Then position i cannot be tau and its residual mass
        // is not needed either.  w_{i+1} = w_i r_{i+1} takes this row's normalisers, which a workgroup that forms S_i waits
        // for anyway: its first wave asks for the drafted token's two logits with them and judges like the leader does,
        // on the same words with the same arithmetic (calls larger than one resident set; not with the debug block).
        const bool may_skip = needed && chain && !P.debug_out && P.algo != kToken;
        if (may_skip && !leader) { ya_bits = logit_bits(rowA + tok); yb_bits = logit_bits(rowB + tok); }
        float Mp, Mq;
        double Lp, Lq;
        const bool need_w = n_prev > 0 && !early;            // w_i still to come: the chain's word, or the ratios
        // (the chain's word is polled beside the row's words; the ratios of the earlier positions only after this row's
        // own ratio is out - it does not depend on them, and the later positions wait for it)
        const bool need_lane = need_w && chain;
        const u64 *const w_word = SV_LW_WORD;
        if (nwg <= kWave / 2) {
            // one poll covers the row: the target row's words in lanes 0.., the draft row's in lanes 32.., what w_i is
            // made of (if still missing) beside them; the two halves of the wave are then combined side by side
            const int e = lane & 31;
            const bool need = e < nwg;
            const u64 *word = (lane < 32 ? W.pgrp : W.qgrp) + 2 * (drow * nwg + (need ? e : nwg - 1));
            u64 v = ld_u64(word);
            int spins = 0;
            while (__any((need && v == 0) || (need_lane && wt == 0))) {
                if (++spins > P.spin_limit) { gave_up = true; break; }
                __builtin_amdgcn_s_sleep(1);
                if (need && v == 0) v = ld_u64(word);
                if (need_lane && wt == 0) wt = ld_u64(w_word);
            }
            if (__any((need && v == kPoison64) || (need_lane && wt == kPoison64))) gave_up = true;
            StatAcc acc;
            if (need) acc.add(v);
            halves_max(acc.m, Mp, Mq);
            // each half relative to its own row's maximum
            double zp, zq;
            halves_sum_f64(acc.relative_to(lane < 32 ? Mp : Mq), zp, zq);
            Lp = (double)shift_of(Mp) + log2_precise(zp);
            Lq = (double)shift_of(Mq) + log2_precise(zq);
        } else {
            RowWords<NW> pw, qw;
            load_row_words<NW>(W.pgrp + 2 * drow * nwg, nwg, pw);
            load_row_words<NW>(W.qgrp + 2 * drow * nwg, nwg, qw);
            Lp = row_normaliser<NW>(W.pgrp + 2 * drow * nwg, nwg, P.spin_limit, gave_up, Mp, pw);
            Lq = row_normaliser<NW>(W.qgrp + 2 * drow * nwg, nwg, P.spin_limit, gave_up, Mq, qw);
            if (need_lane) wt = wait_word(w_word, wt, true, P.spin_limit, gave_up);
        }
        SV_STAMP(7);
        double lr_row = 0.0;                                 // log2 r_{i+1} as its word holds it
        if (leader || may_skip) {
            // log2 r_{i+1} = log2 p_i(X_{i+1}) - log2 q_i(X_{i+1}), for every later position and for whoever finishes
            // the sequence.  The sweeps scale logits by the float k; the exact factor is kd = k (1 + k_eps).  To
            // first order that moves a row's log2-normaliser by k_eps * (the scaled logit where the mass sits, taken
            // as the row maximum); only this ratio, whose logs reach hundreds, is sensitive to it.
            // (the three floats become doubles here and not a moment earlier: registers are scarce until the second sweep)
            asm volatile("" : "+v"(ya_bits), "+v"(yb_bits), "+s"(eta_next));
            const double ya = (double)logit_bits_as_float<T>(ya_bits), yb = (double)logit_bits_as_float<T>(yb_bits);
            const double lp = ya * P.kd - (Lp + P.k_eps * (double)Mp);
            const double lq = yb * P.kd - (Lq + P.k_eps * (double)Mq);
            const double lr = fmax(lp - lq, kLog2RatioFloor);    // a drafted token the target masks out: r = 0, kept finite
            // Alg. 1's test of X_{i+1}, judged here once for everybody: eta_{i+1} < min(r_{i+1}, 1)
            lr_row = unpack_ratio(pack_ratio(lr, false));
            if (leader) {
                const bool passes = P.algo == kToken && (double)eta_next < exp2_precise(fmin(lr, 0.0));
                own_word = pack_ratio(lr, passes);
                if (gave_up) report_gave_up(P);
                if (lane == 0) st_u64(W.ratio + drow, gave_up ? kPoison64 : own_word);
            }
        }
        SV_STAMP(8);
        if (need_w) {
            if (!chain) wt = wait_word(SV_RATIO_WORD, wt, lane < n_prev, P.spin_limit, gave_up);
            log2w = chain ? unpack_ratio(read_lane_u64(wt, 0)) : read_lane_double(weights_from_ratios(P.algo, wt, n_prev), n_prev - 1);
        }
        SV_STAMP(9);
        candidate = can_become_tau(P.algo, U.i, log2w, eta_i);
        if (leader && (chain || finisher)) {
            // (rounded as the word holds it: everybody goes by the same number)
            lw_next = unpack_ratio(pack_ratio(next_weight(P.algo, log2w, unpack_ratio(own_word), ratio_passes(own_word)), false));
            if (gave_up) report_gave_up(P);
            if (chain && lane == 0) st_u64(W.lw + drow, gave_up ? kPoison64 : pack_ratio(lw_next, false));
        }
        // (log2 w_{i+1} rounded as its word holds it, as the next position's leader and the finishing wave will read it)
        const bool sweep = needed && !(may_skip && !gave_up &&
                                       unpack_ratio(pack_ratio(next_weight(P.algo, log2w, lr_row, false), false)) >= 0.0);
        if (P.algo == kToken) log2w = 0.0;                          // the residual of token verification is p - q
        if (P.algo == kGreedy) log2w = fmin(log2w, 100.0);          // keeps w p finite in float
        // the second sweep's row constants: w p(x) = 2^(y_p - A) with A = L_p - log2 w, q(x) = 2^(y_q - L_q).  Their
        // integer parts meet the units' integer shifts in the exponent; the fractions are formed once, here, in double
        // (only where there is a second sweep: the leader of a row without one is on its way to the row's word)
        if (sweep) {
            const double A = Lp - log2w, Ai = rint(A), Qi = rint(Lq);
            const double fq = exp2_precise(Qi - Lq), frho = exp2_precise((Ai - A) - (Qi - Lq));
            if (lane == 0) { row_values[3] = Ai; row_values[4] = Qi; row_values[5] = fq; row_values[6] = frho; row_values[7] = 1.0 / frho; }
        }
        if (lane == 0) {
            row_values[0] = Lp; row_values[1] = Lq; row_values[2] = log2w;
            row_flag = gave_up ? 2 : sweep ? 1 : 3;          // (3: the residual mass was wanted and is not any more)
        }
        if (gave_up) report_gave_up(P);
        SV_STAMP(2);
    }
    bool formed = needed;            // whether the row's residual mass is formed
    if (needed) {
        __syncthreads();
        formed = row_flag != 3;
    }
    if (formed) {
        const bool poisoned = row_flag == 2 || gave_up;
        SV_STAMP(3);

        // ---- second sweep, from registers: w p(x) = xa * cp, q(x) = xb * cq with the wave-uniform cp = 2^(shiftA - A),
        // cq = 2^(shiftB - L_q): powers of two times the row's two fractions
        const int ea = (int)((double)shiftA - row_values[3]), eq = (int)((double)shiftB - row_values[4]);
        const double fq = row_values[5], frho = row_values[6];
        float acc = 0.f;
        {
            // sum of max(xa cp - xb cq, 0) with the larger factor taken out, so that every term lies in [0, 1]
            // (xa, xb <= 1) and the clamp of the fma is the max: two instructions per pair.  The factor rho = cp / cq
            // is rounded once, from double: whatever it is off by multiplies the whole mass of the row's active
            // tokens, which is what is left of S_i where w p and q nearly agree.
            const double rho = ldexp(frho, ea - eq);
            if (rho <= 1.0) {
                const float rho_f = (float)rho;
#pragma unroll
                for (int j = 0; j < LANE; ++j) acc += __builtin_amdgcn_fmed3f(__builtin_fmaf(xa[j], rho_f, -xb[j]), 0.f, 1.f);
                acc *= (float)ldexp(fq, eq);
            } else {
                const float nrho = -(float)ldexp(row_values[7], eq - ea);
#pragma unroll
                for (int j = 0; j < LANE; ++j) acc += __builtin_amdgcn_fmed3f(__builtin_fmaf(xb[j], nrho, xa[j]), 0.f, 1.f);
                acc *= (float)ldexp(fq * frho, ea);
            }
        }
        acc = wave_sum(acc);
        // (the four waves' shares meet in LDS and go out as one write of sixteen bytes: four separate small writes
        // between the streaming reads cost more than the barrier)
        if (lane == 0) wave_shares[wave] = poisoned ? kPoison32 : pack_partial(acc);
        lds_barrier();
        if (wave == 0 && lane < kWaves) st_u32(SV_WORDS.spart + drow * nu + wg_x * kWaves + lane, wave_shares[lane]);
        SV_STAMP(4);
    }
    if (!leader) return;
    lead_row<T, ALIGNED, LANE>(U.b, U.i, gb, par, formed, candidate && formed, finisher, own_word, lw_next, res_first, eta_i, eta_next, gave_up, row_values, stamps);
#undef SV_RATIO_WORD
#undef SV_LW_WORD
#undef SV_WORDS
}

// Clears the control words of a workspace and marks it initialised.
__global__ void workspace_init_kernel(int *words, size_t n, int magic)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < n) words[idx] = idx == kHdrMagic ? magic : 0;
}

}  // namespace sv
