// Calls of few resident sets (all workgroups run at once, or nearly; rows of at most 32 workgroups).
//
// Such a call is as long as its chain of dependent trips through device memory.  The large kernel (fused.hpp) hands a
// row pair's results to ONE wave, the row's leader: it collects the row's partial sums of S_i, judges the position's
// accept test and, for the draw of the token that follows if tau = i, reads the chunk that holds the token a second
// time; the leader of the sequence's last row pair then collects one word per position.  That is the cheapest way for
// a call whose rows follow each other in waves over the device, and two trips too many for a call that is over
// when its one wave of workgroups is.  Here every workgroup of a row pair keeps its exponentials in registers until the
// row's S_i is known, and EVERY workgroup's first wave reads all partial sums of the row: all of them form the same S_i
// from the same words in the same order, judge the same test and find the same place for u * S_i - and the workgroup
// that holds that place draws the token from its registers and publishes the position's word itself.  The last
// target row works the same way (its workgroups know from the ratios alone whether every token is accepted); the first
// wave of its last workgroup writes tau and Y and hands the words over to the next call.  Words, copies, call count:
// the large kernel's (so calls of either may follow each other on one workspace); the arithmetic of the sweeps too.
#pragma once

#include "fused.hpp"

namespace sv {

constexpr int kResidentMaxGroups = 32;        // workgroups per row: one poll of a wave covers the words of both rows
// Up to how many times the workgroups that the device keeps resident the library takes this kernel by itself.  Its
// workgroups hold their registers until the row's S_i is there, which costs nothing while everything runs at once and
// more and more as workgroups queue for the compute units; the large kernel pays a fixed price for its chain of row
// leaders instead.  Measured with gamma = 8, V = 128256 (bf16, 1280 workgroups resident), this kernel / the large one:
// B = 8 (0.9 sets) 15.3 / 16.3 us, B = 9 16.3 / 25.4, B = 16 (1.8 sets) 23.1 / 28.8, B = 24 (2.7 sets) 29.6 / 31.9,
// B = 28 (3.2 sets) 33.6 / 33.8, B = 32 36.7 / 34.8, B = 64 (7.2 sets) 67.7 / 55.3.
constexpr int kResidentSets = 3;

// (largest scaled logit, sum) of four words, one per lane of a quad: every lane of the quad gets the combination
// (fixed order, the sums through exact powers of two).
__device__ __forceinline__ u64 quad_word(u64 w)
{
    const float m = stat_shift(w);
    float M = fmaxf(m, __int_as_float(dpp_shift<0xB1>(__float_as_int(m))));            // quad_perm:[1,0,3,2]
    M = fmaxf(M, __int_as_float(dpp_shift<0x4E>(__float_as_int(M))));                   // quad_perm:[2,3,0,1]
    double z = m > -INFINITY ? ldexp((double)stat_sum(w), (int)(shift_of(m) - shift_of(M))) : 0.0;
    z += dpp_shift_double<0xB1>(z);
    z += dpp_shift_double<0x4E>(z);
    return pack_stat(M, (float)z);
}

// A wave-uniform float as a double, converted where it is used: left to itself the compiler converts the uniforms at
// the top of the kernel and keeps the doubles in vector registers through both sweeps.
__device__ __forceinline__ double late_double(float v)
{
    asm volatile("" : "+s"(v));
    return (double)v;
}

// Where t falls among the entries z of the lanes (inclusive running sums `inc`; lanes beyond the entries hold 0):
// the first entry whose running sum exceeds t, with what is left of t inside it; when rounding leaves none, the last
// entry that has any mass, and all of it.
__device__ __forceinline__ int locate_entry(double z, double inc, double t, double &t_inside)
{
    const u64 hit = __ballot(inc > t), nz = __ballot(z > 0.0);
    if (hit) {
        const int e = __ffsll((long long)hit) - 1;
        t_inside = t - read_lane_double(inc - z, e);
        return e;
    }
    t_inside = INFINITY;
    return nz ? 63 - __clzll((long long)nz) : 0;
}

// The draw inside one wave's unit of 64 * LANE logits (vocabulary order inside the unit: vector, lane, element), in two
// steps.  First, by any wave: `sums` holds the unit's weights summed per (vector, lane), in that order (64 * NV floats
// in LDS); every lane takes NV consecutive ones, one scan over the wave finds the lane and that lane the entry whose
// running sum exceeds t first (else the last entry with any weight).  Returns the entry, `t_e`: what is left of t
// inside it.
template <int NV>
__device__ __forceinline__ int locate_in_sums(const float *sums, double t, double &t_e)
{
    const int lane = threadIdx.x & 63;
    float ent[NV], mine = 0.f;
#pragma unroll
    for (int j = 0; j < NV; ++j) { ent[j] = sums[lane * NV + j]; mine += ent[j]; }
    const double inc = wave_scan((double)mine);
    const u64 hit = __ballot(inc > t), nz = __ballot(mine > 0.f);
    const int hl = hit ? __ffsll((long long)hit) - 1 : nz ? 63 - __clzll((long long)nz) : 0;
    int entry = 0;
    double left = INFINITY;
    if (lane == hl) {
        double r = inc - (double)mine, before = 0.0;
        int last_j = 0, found = -1;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            if (found < 0 && hit && r + (double)ent[j] > t) { found = j; before = r; }
            if (ent[j] > 0.f) last_j = j;
            r += (double)ent[j];
        }
        entry = hl * NV + (found < 0 ? last_j : found);
        if (found >= 0) left = t - before;
    }
    t_e = read_lane_double(left, hl);
    return __builtin_amdgcn_readlane(entry, hl);
}
// Then, by the wave that holds the unit's weights in registers (weight(j), j the register index): the element of that
// entry - KVEC weights of one lane - whose running sum exceeds t_e first, else the last one with any weight.
template <int KVEC, int LANE, typename F>
__device__ __forceinline__ int walk_entry(F weight, int entry, double t_e)
{
    constexpr int kNV = LANE / KVEC;
    const int dv = entry / kWave, dl = entry % kWave;        // the entry's vector and lane
    int cand = 0;
    if ((int)(threadIdx.x & 63) == dl) {
        float wgt[KVEC];
#pragma unroll
        for (int v = 0; v < kNV; ++v)
            if (v == dv) {
#pragma unroll
                for (int e = 0; e < KVEC; ++e) wgt[e] = weight(v * KVEC + e);
            }
        double r = 0.0;
        int last_e = 0, found = -1;
#pragma unroll
        for (int e = 0; e < KVEC; ++e) {
            r += (double)wgt[e];
            if (wgt[e] > 0.f) last_e = e;
            if (found < 0 && r > t_e) found = e;
        }
        cand = found < 0 ? last_e : found;
    }
    return __builtin_amdgcn_readlane(cand, dl);
}
// Both steps by the wave that holds the weights (`sums`: 64 * LANE / KVEC floats that only this wave uses meanwhile).
// Returns the token's offset inside the unit.
template <int KVEC, int LANE, typename F>
__device__ __forceinline__ int draw_in_unit(F weight, double t, float *sums)
{
    constexpr int kNV = LANE / KVEC;
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int v = 0; v < kNV; ++v) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < KVEC; ++e) s += weight(v * KVEC + e);
        sums[v * kWave + lane] = s;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    double t_e;
    const int entry = locate_in_sums<kNV>(sums, t, t_e);
    return entry * KVEC + walk_entry<KVEC, LANE>(weight, entry, t_e);
}

// Grid (x, y, z) = (workgroup of the row, sequence, slot): slot i is row pair i, slot gamma the sequence's last target
// row; x runs fastest in the start order, so a row's workgroups start together and a position's before the next one's.
// (bf16 rows: held to the registers of five waves per SIMD, as the large kernel is - in calls of more than one resident
// set a fifth of the workgroups more run at a time: B = 20 of the shape above 28.3 -> 25.5 us)
template <typename T, bool ALIGNED>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(ElemTraits<T>::kVec == 8 ? SV_WAVES_SMALL : 4)))
void resident_verify_kernel(const FusedParams P)
{
    constexpr int LANE = kLaneSmall, kUnitLogits = kWave * LANE, kVec = ElemTraits<T>::kVec;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int c = blockIdx.x, b = blockIdx.y, slot = blockIdx.z, nwg = gridDim.x;
    const int gamma = P.gamma, V = P.V, nu = P.nu;
    const float k = P.k;
    long long *stamps = nullptr;
#ifdef SV_PROFILE
    if (P.prof) stamps = P.prof + (((size_t)b * (gamma + 1) + slot) * nwg + c) * 16;      // one record per workgroup
#endif
    SV_STAMP(0);
    int gb = gamma;
    if (P.draft_lens) { gb = load_uniform(P.draft_lens + b); gb = gb < 1 ? 1 : gb > gamma ? gamma : gb; }
    const bool last_row = slot == gamma;
    const bool unused = !last_row && slot >= gb;
    const int i = last_row ? gb : slot;
    const size_t seq_d = (size_t)b * gamma, seq_u = (size_t)b * (gamma + 1);
    const size_t drow = seq_d + (last_row ? 0 : i);
    const T *rowA = static_cast<const T *>(P.target) + (seq_u + i) * P.tstride;
    const T *rowB = static_cast<const T *>(P.draft) + drow * P.dstride;
    const int unit_first = (c * kWaves + wave) * kUnitLogits;

    // the rows' loads first: they depend on the arguments only
    RawSlice<T, ALIGNED, LANE> rawA, rawB;
    if (!unused) {
        issue_loads<T, ALIGNED, LANE>(rowA, unit_first, V, rawA);
        if (!last_row) issue_loads<T, ALIGNED, LANE>(rowB, unit_first, V, rawB);
    }
    asm volatile("" ::: "memory");
    const int magic_word = load_uniform(P.header + kHdrMagic);
    const unsigned par = (unsigned)load_uniform(P.gen + b) & 1u;
    if (magic_word != P.magic) {
        if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0)
            for (int s = threadIdx.x; s < P.B; s += kThreads) { P.accept_len[s] = -1; P.next_token[s] = -1; }
        return;
    }
    // every slot's words are cleared, in the copy that this call does not use, by the first wave of the slot's last
    // workgroup (an unused position's in both copies: the other one may hold an earlier, longer call's words)
    const bool leader = wave == 0 && c == nwg - 1;
    if (unused) {
        if (leader) { const bool rw = row_words_used<kLaneSmall>(P.header); clear_row_words(P, P.words, b, slot, rw); clear_row_words(P, words_of(P, 1), b, slot, rw); }
        return;
    }
    if (leader) clear_row_words(P, words_of(P, par ^ 1u), b, slot, slot != P.gamma && row_words_used<kLaneSmall>(P.header));
    const Words W = words_of(P, par);
    const bool token_algo = P.algo == kToken;

    __shared__ u64 wave_words[2][kWaves];
    __shared__ float wave_part[kWaves];
    __shared__ double row_values[8];
    __shared__ int row_flag[4];
    __shared__ float draw_sums[kWaves][kWave * (LANE / kVec)];      // per wave: its unit's weights summed per (vector, lane)
    __shared__ float wave_scale[kWaves];
    // what the first wave keeps across the second sweep lives here meanwhile (its registers are the whole workgroup's):
    // the row's words as its lanes hold them, the words of log2 r_{i+1} and log2 r_i, log2 w_i, the row's largest
    // scaled target logit, whether the position can become tau
    __shared__ u64 kept_grp[kWave], kept_words[4];
    __shared__ float kept_Mp;
    __shared__ int draw_entry;
    bool gave_up = false;

    // =================================================================== the sequence's last target row
    if (last_row) {
        // Y comes from it where every token is accepted, which its workgroups see from the ratios; the leader writes
        // tau and Y (Y from the word of position tau, or from the word that the workgroup holding it publishes)
        u64 *const y_word = W.lw + seq_d + gb - 1;                    // (a word this kernel has no other use for)
        u64 rw = 0, res_first = 0;
        float eta_g = 0.f, u = 0.f;
        if (wave == 0) {
            eta_g = load_uniform(P.uniforms + seq_u + gb - 1);
            u = load_uniform(P.uniforms + seq_u + gb);
            rw = ld_u64(W.ratio + seq_d + (lane < gb ? lane : 0));
            if (leader) res_first = ld_u64(W.rowres + seq_d + (lane < gb ? lane : 0));
        }
        float xa[LANE], shiftA;
        unpack_slice<T, ALIGNED, LANE>(rowA, unit_first, V, rawA, xa);
        const u64 stA = first_sweep_row(xa, k, shiftA);
        if (lane == 0) wave_words[0][wave] = stA;
        __syncthreads();
        bool all_accepted = false;
        double w_last = 1.0;
        u64 pl = 0;                                                   // the row's words (lane e: workgroup e's)
        const u64 *const pl_word = W.plast + (size_t)b * nu + (lane < nwg ? lane : 0);
        if (wave == 0) {
            const u64 own_plast = quad_word(wave_words[0][lane & 3]);
            if (lane == 0) st_u64(W.plast + (size_t)b * nu + c, own_plast);
            rw = wait_word(W.ratio + seq_d + (lane < gb ? lane : 0), rw, lane < gb, P.spin_limit, gave_up);
            // (by now the row's other workgroups have published theirs: a look that the waits below pick up)
            pl = lane == c ? own_plast : ld_u64(pl_word);
            if (token_algo) {
                const u64 failed = __ballot(lane < gb && !ratio_passes(rw));
                all_accepted = failed == 0;
            } else {
                const double lw_g = read_lane_double(weights_from_ratios(P.algo, rw, gb), gb - 1);
                w_last = exp2_precise(P.algo == kGreedy ? fmin(lw_g, 100.0) : lw_g);
                all_accepted = (double)eta_g < fmin(w_last, 1.0);                      // eta_gamma < h_gamma = w_gamma
            }
            int role = 0;
            if (all_accepted && !gave_up) {
                // the row's words, all of them: where u * (the row's sum) falls
                const u64 pw = pl = wait_word(pl_word, pl, lane < nwg, P.spin_limit, gave_up);
                const float m = lane < nwg ? stat_shift(pw) : -INFINITY;
                const float M = wave_max(m);
                const double z = m > -INFINITY ? ldexp((double)stat_sum(pw), (int)(shift_of(m) - shift_of(M))) : 0.0;
                const double inc = wave_scan(z);
                double t_in;
                const int e = locate_entry(z, inc, late_double(u) * read_lane_double(inc, kWave - 1), t_in);
                if (e == c && !gave_up) {
                    // ... and in which of the workgroup's four units
                    const u64 ww = wave_words[0][lane & 3];
                    const float mw = lane < kWaves ? stat_shift(ww) : -INFINITY;
                    const double zw = mw > -INFINITY ? ldexp((double)stat_sum(ww), (int)(shift_of(mw) - shift_of(M))) : 0.0;
                    double t_w;
                    const int wv = locate_entry(zw, wave_scan(zw), t_in, t_w);
                    // (into the units of that wave's exponentials, which are relative to its own shift)
                    const float m_wv = stat_shift(read_lane_u64(ww, wv));
                    if (lane == 0) { row_flag[1] = wv; row_values[0] = ldexp(t_w, (int)(shift_of(M) - shift_of(m_wv))); }
                    role = 1;
                }
            }
            if (gave_up) { report_gave_up(P); if (lane == 0) st_u64(y_word, kPoison64); }
            if (lane == 0) row_flag[0] = role;
        }
        __syncthreads();
        if (row_flag[0] == 1 && wave == row_flag[1]) {
            const int off = draw_in_unit<kVec, LANE>([&](int j) { return xa[j]; }, row_values[0], draw_sums[wave]);
            if (lane == 0) st_u64(y_word, pack_rowres(true, unit_first + off));
        }
        if (!leader) return;

        // ---- the leader: tau and Y
        int tau, y;
        if (all_accepted) {
            tau = gb;
            y = rowres_token(wait_word(y_word, P.spin_limit, gave_up));
        } else if (token_algo) {
            // tau is the length of the leading run of passed tests; its position's word holds the token
            const u64 failed = __ballot(lane < gb && !ratio_passes(rw));
            tau = __ffsll((long long)failed) - 1;
            y = rowres_token(wait_word(W.rowres + seq_d + tau, read_lane_u64(res_first, tau), true, P.spin_limit, gave_up));
        } else {
            // one word per position: bit l, whether the test of position l passes (none at position 0); tau is the
            // last position whose test passes, else 0
            const u64 res = wait_word(W.rowres + seq_d + (lane < gb ? lane : 0), res_first, lane < gb, P.spin_limit, gave_up);
            const u64 tests = __ballot(lane < gb && rowres_passes(res)) & ~1ull;
            tau = tests ? 63 - __clzll((long long)tests) : 0;
            y = rowres_token(read_lane_u64(res, tau));
        }
        if (P.debug_out && lane == 0) {
            float *d = P.debug_out + (seq_u + gb) * 3;       // S_gamma = w_gamma: q_gamma == 0
            d[0] = (float)w_last; d[1] = (float)w_last;
            d[2] = token_algo ? (float)exp2_precise(fmin(unpack_ratio(read_lane_u64(rw, gb - 1)), 0.0)) : (float)fmin(w_last, 1.0);
        }
        // every workgroup of the sequence has read the call count once the last target row's words are there (the row
        // pairs' workgroups published words that the ratios, which this wave has, were made of)
        wait_word(pl_word, pl, lane < nwg, P.spin_limit, gave_up);
        if (gave_up) report_gave_up(P);
        if (lane == 0) {
            P.accept_len[b] = gave_up ? -1 : tau;
            P.next_token[b] = gave_up ? -1 : y;
            __hip_atomic_store(P.gen + b, (int)(par ^ 1u), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        SV_STAMP(6);
        return;
    }

    // =================================================================== a row pair
    const int n_prev = i;                                     // ratios that w_i is made of
    u64 wt = 0;                                               // first wave, lane j: the word of log2 r_{j+1}
    float eta_i = 0.f, eta_next = 0.f, u = 0.f;
    int tok = 0;
    if (wave == 0) {
        eta_i = load_uniform(P.uniforms + seq_u + (n_prev > 0 ? n_prev - 1 : 0));
        eta_next = load_uniform(P.uniforms + seq_u + n_prev);
        u = load_uniform(P.uniforms + seq_u + gb);
        tok = load_uniform(P.tokens + drow);
        wt = ld_u64(W.ratio + seq_d + (lane <= n_prev ? lane : 0));
    }
    // ---- first sweep (as in the large kernel): exponentials stay in xa / xb
    float xa[LANE], xb[LANE];
    float shiftA, shiftB;
    unpack_slice<T, ALIGNED, LANE>(rowA, unit_first, V, rawA, xa);
    const u64 stA = first_sweep_row(xa, k, shiftA);
    unpack_slice<T, ALIGNED, LANE>(rowB, unit_first, V, rawB, xb);
    uint32_t ya_bits = 0, yb_bits = 0;
    if (leader) { ya_bits = logit_bits(rowA + tok); yb_bits = logit_bits(rowB + tok); }
    const u64 stB = first_sweep_row(xb, k, shiftB);
    if (lane == 0) { wave_words[0][wave] = stA; wave_words[1][wave] = stB; }
    __syncthreads();
    SV_STAMP(1);

    if (wave == 0) {
        u64 grp = 0;                // the row's words (lanes 0..: the target row's, lanes 32..: the draft row's)
        float Mp = 0.f;
        double log2w = 0.0;
        u64 own_word = 0, prev_word = 0;
        bool candidate = true;
        publish_group_words(wave_words, W.pgrp + 2 * (drow * nwg + c), W.qgrp + 2 * (drow * nwg + c));
        // ---- L_p, L_q from the words of all workgroups of the row
        const int e = lane & 31;
        const bool need = e < nwg;
        const u64 *word = (lane < 32 ? W.pgrp : W.qgrp) + 2 * (drow * nwg + (need ? e : nwg - 1));
        grp = wait_word(word, ld_u64(word), need, P.spin_limit, gave_up);
        StatAcc acc;
        if (need) acc.add(grp);
        float Mq;
        halves_max(acc.m, Mp, Mq);
        double zp, zq;
        halves_sum_f64(acc.relative_to(lane < 32 ? Mp : Mq), zp, zq);
        const double Lp = (double)shift_of(Mp) + log2_precise(zp), Lq = (double)shift_of(Mq) + log2_precise(zq);
        SV_STAMP(7);
        if (leader) {
            // log2 r_{i+1} = log2 p_i(X_{i+1}) - log2 q_i(X_{i+1}) (see the large kernel for the correction by k_eps)
            const double ya = (double)logit_bits_as_float<T>(ya_bits), yb = (double)logit_bits_as_float<T>(yb_bits);
            const double lp = ya * P.kd - (Lp + P.k_eps * (double)Mp), lq = yb * P.kd - (Lq + P.k_eps * (double)Mq);
            const double lr = fmax(lp - lq, kLog2RatioFloor);
            own_word = pack_ratio(lr, token_algo && (double)eta_next < exp2_precise(fmin(lr, 0.0)));
            if (gave_up) report_gave_up(P);
            if (lane == 0) st_u64(W.ratio + drow, gave_up ? kPoison64 : own_word);
        }
        SV_STAMP(8);
        // ---- the ratios of the earlier positions, and this row's own (the leader has it already)
        wt = wait_word(W.ratio + seq_d + (lane <= n_prev ? lane : 0), wt, lane < n_prev || (lane == n_prev && !leader), P.spin_limit, gave_up);
        if (!leader) own_word = read_lane_u64(wt, n_prev);
        if (n_prev > 0) {
            log2w = read_lane_double(weights_from_ratios(P.algo, wt, n_prev), n_prev - 1);
            prev_word = read_lane_u64(wt, n_prev - 1);
        }
        SV_STAMP(9);
        candidate = can_become_tau(P.algo, i, log2w, eta_i);
        // S_i is formed where the position can become tau (position 0 always can) or the caller wants every S_i
        const bool needed = candidate || P.debug_out != nullptr || gave_up;
        if (token_algo) log2w = 0.0;                                // the residual of token verification is p - q
        if (P.algo == kGreedy) log2w = fmin(log2w, 100.0);          // keeps w p finite in float
        if (needed) {
            // the second sweep's row constants (see the large kernel)
            const double A = Lp - log2w, Ai = rint(A), Qi = rint(Lq);
            const double fq = exp2_precise(Qi - Lq), frho = exp2_precise((Ai - A) - (Qi - Lq));
            if (lane == 0) { row_values[3] = Ai; row_values[4] = Qi; row_values[5] = fq; row_values[6] = frho; row_values[7] = 1.0 / frho; }
        } else if (leader && lane == 0) {
            // nothing more to say about tau than this (Alg. 2 / 4: the test fails; Alg. 1: how the test of X_{i+1} went)
            st_u64(W.rowres + drow, pack_rowres(token_algo && ratio_passes(own_word), -1));
        }
        if (gave_up) report_gave_up(P);
        if (needed) {
            kept_grp[lane] = grp;
            if (lane == 0) {
                kept_words[0] = own_word; kept_words[1] = prev_word; kept_words[2] = (u64)__double_as_longlong(log2w);
                kept_words[3] = candidate ? 1 : 0;
                kept_Mp = Mp;
            }
        }
        if (lane == 0) row_flag[0] = needed ? 1 : 0;
        SV_STAMP(2);
    }
    __syncthreads();
    if (!row_flag[0]) return;

    // ---- second sweep, from registers (as in the large kernel): terms in [0, 1] in units of the larger row factor
    const int ea = (int)((double)shiftA - row_values[3]), eq = (int)((double)shiftB - row_values[4]);
    const double rho = ldexp(row_values[6], ea - eq);
    const bool q_units = rho <= 1.0;
    const float factor = q_units ? (float)rho : -(float)ldexp(row_values[7], eq - ea);
    const float scale = q_units ? (float)ldexp(row_values[5], eq) : (float)ldexp(row_values[5] * row_values[6], ea);
    auto term = [&](int j) {
        return q_units ? __builtin_amdgcn_fmed3f(__builtin_fmaf(xa[j], factor, -xb[j]), 0.f, 1.f)
                       : __builtin_amdgcn_fmed3f(__builtin_fmaf(xb[j], factor, xa[j]), 0.f, 1.f);
    };
    {
        // (the sums per vector stay behind in LDS: the draw, if it falls into this unit, starts from them)
        constexpr int kNV = LANE / kVec;
        float acc = 0.f;
#pragma unroll
        for (int v = 0; v < kNV; ++v) {
            float sv_ = 0.f;
#pragma unroll
            for (int e = 0; e < kVec; ++e) sv_ += term(v * kVec + e);
            draw_sums[wave][v * kWave + lane] = sv_;
            acc += sv_;
        }
        acc = wave_sum(acc * scale);
        if (lane == 0) { wave_part[wave] = acc; wave_scale[wave] = scale; }
    }
    __syncthreads();
    SV_STAMP(4);

    if (wave == 0) {
        // ---- the workgroup's share of S_i goes out; all shares of the row come in
        const float mine = (wave_part[0] + wave_part[1]) + (wave_part[2] + wave_part[3]);
        const unsigned own_part = gave_up ? kPoison32 : pack_partial(mine);
        if (lane == 0) st_u32(W.spart + drow * nu + c, own_part);
        const u64 own_word = kept_words[0], prev_word = kept_words[1];
        const double log2w = __longlong_as_double((long long)kept_words[2]);
        const bool candidate = kept_words[3] != 0;
        // (while the shares travel: what the accept test needs of w_i)
        const bool has_test = !token_algo && i > 0;
        const double one_minus_w = has_test ? one_minus_exp2(fmin(log2w, 0.0)) : 0.0;
        const unsigned sp = wait_word32(W.spart + drow * nu + (lane < nwg ? lane : 0), lane == c ? own_part : 0u, lane < nwg, P.spin_limit, gave_up);
        SV_STAMP(5);
        double z = lane < nwg ? (double)unpack_partial(sp) : 0.0;
        double inc = wave_scan(z);
        const double S_i = read_lane_double(inc, kWave - 1);
        // ---- the position's accept test (Alg. 2 / 4); Alg. 1: the test of X_{i+1} came with the ratio
        // (Alg. 2 / 4, position i >= 1: eta_i < h_i = S_i / (S_i + 1 - w_i), 1 where w_i >= 1 - see AcceptTest; judged
        // without the division)
        const bool test_passes = has_test && candidate && (log2w >= 0.0 || late_double(eta_i) * (S_i + one_minus_w) < S_i);
        const bool next_passes = ratio_passes(own_word);
        const bool own_passes = token_algo ? next_passes : test_passes;
        // the token that follows if this position becomes tau is drawn where it can
        const bool want = !gave_up && (token_algo ? candidate && !next_passes : i == 0 || own_passes);
        if (P.debug_out && leader && lane == 0) {
            float *d = P.debug_out + (seq_u + i) * 3;            // (w_i, S_i, h_i); Alg. 1 has no w, its h_i = min(r_i, 1)
            double h_i = has_test && log2w < 0.0 ? S_i / (S_i + one_minus_w) : 1.0;
            if (token_algo && i > 0) h_i = exp2_precise(fmin(unpack_ratio(prev_word), 0.0));
            d[0] = has_test ? (float)exp2_precise(log2w) : 1.f; d[1] = (float)S_i; d[2] = (float)h_i;
        }
        int role = 0;
        if (want) {
            // where u * S_i falls; a residual without any mass is drawn from p_i instead (weights: the exponentials)
            const bool from_p = !(S_i > 0.0);
            const float Mp = kept_Mp;
            const u64 grp = kept_grp[lane];
            if (from_p) {
                const float m = lane < nwg ? stat_shift(grp) : -INFINITY;
                z = m > -INFINITY ? ldexp((double)stat_sum(grp), (int)(shift_of(m) - shift_of(Mp))) : 0.0;
                inc = wave_scan(z);
            }
            double t_in;
            const int e = locate_entry(z, inc, late_double(u) * read_lane_double(inc, kWave - 1), t_in);
            if (e == c) {
                // ... in which of the workgroup's four units, and what is left of t in that unit's own units
                double t_w;
                int wv;
                if (from_p) {
                    const u64 ww = wave_words[0][lane & 3];
                    const float mw = lane < kWaves ? stat_shift(ww) : -INFINITY;
                    const double zw = mw > -INFINITY ? ldexp((double)stat_sum(ww), (int)(shift_of(mw) - shift_of(Mp))) : 0.0;
                    wv = locate_entry(zw, wave_scan(zw), t_in, t_w);
                    t_w = ldexp(t_w, (int)(shift_of(Mp) - shift_of(stat_shift(read_lane_u64(ww, wv)))));
                } else {
                    double before = 0.0;
                    int last_w = 0;
                    wv = -1; t_w = INFINITY;
#pragma unroll
                    for (int w = 0; w < kWaves; ++w) {
                        const double zw = (double)wave_part[w];
                        if (wv < 0 && before + zw > t_in) { wv = w; t_w = t_in - before; }
                        if (zw > 0.0) last_w = w;
                        before += zw;
                    }
                    if (wv < 0) wv = last_w;
                    // ... and at which (vector, lane) of that unit: its sums per vector are in LDS, in the terms' own
                    // units (the shares were scaled, the terms are not)
                    double t_e;
                    const int entry = locate_in_sums<LANE / kVec>(draw_sums[wv], t_w / (double)wave_scale[wv], t_e);
                    if (lane == 0) draw_entry = entry;
                    t_w = t_e;
                }
                if (lane == 0) { row_flag[1] = wv; row_flag[2] = from_p ? 1 : 0; row_flag[3] = own_passes ? 1 : 0; row_values[0] = t_w; }
                role = 1;
            }
        } else if (leader && lane == 0) {
            st_u64(W.rowres + drow, gave_up ? kPoison64 : pack_rowres(own_passes, -1));
        }
        if (gave_up) report_gave_up(P);
        if (lane == 0) row_flag[0] = role;
        SV_STAMP(10);
    }
    __syncthreads();
    SV_STAMP(11);
    if (row_flag[0] != 1 || wave != row_flag[1]) return;
    // ---- the wave that holds the token draws it from its registers and publishes the position's word
    int off;
    if (row_flag[2]) {
        off = draw_in_unit<kVec, LANE>([&](int j) { return xa[j]; }, row_values[0], draw_sums[wave]);
    } else {
        const int entry = __builtin_amdgcn_readfirstlane(draw_entry);      // (the same for the whole wave, and known to be)
        off = entry * kVec + walk_entry<kVec, LANE>(term, entry, row_values[0]);
    }
    if (lane == 0) st_u64(W.rowres + drow, pack_rowres(row_flag[3] != 0, unit_first + off));
    SV_STAMP(15);
}

}  // namespace sv
