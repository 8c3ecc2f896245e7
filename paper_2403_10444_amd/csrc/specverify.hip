// Draft verification for speculative decoding on gfx950: the C ABI of include/specverify.h.
//
// Host side only: argument checks, workspace layout and kernel launches.  The kernels are in
// fused.hpp (one launch, every logit read from HBM once; the default) and staged.hpp (four
// launches, no limit on the vocabulary size); probs.hpp holds the kernels for inputs that are
// probabilities already.

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>
#include <atomic>
#include <mutex>

#include "../../include/specverify.h"
#include "common.hpp"
#include "fused.hpp"
#include "probs.hpp"
#include "sample.hpp"
#include "staged.hpp"
#include "tiny.hpp"
#include "resident.hpp"

namespace {

using namespace sv;

constexpr int kDefaultSpinLimit = 1 << 20;

std::atomic<int> g_path{0};                       // 0 auto, 1 staged, 2 fused, 5 one workgroup per sequence, 7 the kernel for calls of one resident set (testing hook; 3 / 4: fused with small / large units)
std::atomic<int> g_spin_limit{kDefaultSpinLimit};
std::atomic<int> g_last_kernel{0};                  // the kernels of the last verification call that was launched (SV_KERNEL_*)
std::atomic<int> g_lane{0};                        // 0 auto, 32 or 64: logits per lane of the fused kernel's units (testing hook)
#ifdef SV_PROFILE
std::atomic<long long *> g_prof{nullptr};          // device buffer for per-workgroup timestamps (tuning builds only)
#endif

struct Layout {
    size_t total;
    // fused path
    bool fused_ok;
    int nu;                       // wave chunks per row = 4 * workgroups per row
    size_t fused_grid;            // workgroups of the fused kernel
    size_t control_words;         // header, call counts and both copies of the words that cross waves: in ints, at offset 0
    size_t off_gen, copy_bytes;   // the call counts; bytes from one copy of the words to the other
    size_t off_ratio, off_lw, off_rowres, off_pstat, off_plast, off_pgrp, off_qgrp, off_spart, off_lseen;     // copy 0
    // staged path
    int nchunks;                  // chunks of kChunk logits per row
    size_t rows_total;
    size_t off_stats, off_coef, off_sspart;
};

bool make_layout(int32_t B, int32_t gamma, int32_t V, Layout &L)
{
    if (B < 1 || gamma < 1 || V < 1 || gamma > SV_MAX_GAMMA) return false;
    L.nchunks = (V + kChunk - 1) / kChunk;
    L.rows_total = (size_t)B * (2 * (size_t)gamma + 1);
    if (L.rows_total * (size_t)L.nchunks > 0x7fffffffull) return false;     // 1-D grids of 32-bit size
    const size_t rows_t = (size_t)B * (gamma + 1), rows_d = (size_t)B * gamma;

    // a workgroup is four waves, each with one wave chunk of a row
    L.nu = (V + kWaves * kWave * kLaneSmall - 1) / (kWaves * kWave * kLaneSmall) * kWaves;
    L.fused_grid = rows_t * (size_t)(L.nu / kWaves);
    L.fused_ok = L.nu <= kMaxUnitsPerRow && L.fused_grid <= 0x7fffffffull;
    size_t off = kHdrWords * sizeof(int);
    L.off_gen = off;    off = align_up(off + (size_t)B * sizeof(int), 256);
    const size_t copy0 = off;
    L.off_ratio = off;  off += rows_d * sizeof(u64);
    L.off_lw = off;     off += rows_d * sizeof(u64);
    L.off_rowres = off; off += rows_d * sizeof(u64);
    L.off_pstat = off;  off += rows_d * L.nu * sizeof(u64);
    L.off_plast = off;  off += (size_t)B * L.nu * sizeof(u64);
    off = align_up(off, 16);
    L.off_pgrp = off;   off += rows_d * (L.nu / kWaves) * 2 * sizeof(u64);     // (target word, draft word) pairs
    L.off_qgrp = L.off_pgrp + sizeof(u64);
    L.off_spart = off;  off += rows_d * L.nu * sizeof(unsigned);
    off = align_up(off, 8);
    L.off_lseen = off;  off += (size_t)B * (L.nu / kWaves) * sizeof(u64);
    L.copy_bytes = align_up(off - copy0, 256);
    off = copy0 + 2 * L.copy_bytes;
    L.control_words = off / sizeof(int);
    off = align_up(off, 256);
    // the staged path's scratch follows, so that it never touches the control words
    L.off_stats = off;  off = align_up(off + L.rows_total * L.nchunks * sizeof(float2), 256);
    L.off_coef = off;   off = align_up(off + rows_t * sizeof(SeqCoef), 256);
    L.off_sspart = off; off = align_up(off + rows_d * L.nchunks * sizeof(float), 256);
    L.total = off;
    return true;
}

template <typename T> constexpr int dtype_bytes() { return ElemTraits<T>::kVec == 4 ? 4 : 2; }

// Workgroups of a kernel that the current device keeps resident at once (cached per kernel).
template <typename K>
int resident_workgroups(K kernel, std::atomic<int> &cache)
{
    if (cache.load() > 0) return cache.load();
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kThreads, 0) != hipSuccess) return 0;
    cache.store(cus * per_cu);
    return cus * per_cu;
}

template <typename T, bool ALIGNED>
sv_status_t launch_staged(int algo, const void *target_v, const void *draft_v, const int32_t *tokens, const int32_t *draft_lens,
                          size_t tstride, size_t dstride, const float *uniforms, int B, int gamma, int V, float k, double kd, const Layout &L,
                          char *ws, int32_t *accept_len, int32_t *next_token, float *debug_out,
                          hipStream_t stream)
{
    const T *target = static_cast<const T *>(target_v);
    const T *draft = static_cast<const T *>(draft_v);
    float2 *stats = reinterpret_cast<float2 *>(ws + L.off_stats);
    SeqCoef *coef = reinterpret_cast<SeqCoef *>(ws + L.off_coef);
    float *spart = reinterpret_cast<float *>(ws + L.off_sspart);
    const int n_target_rows = B * (gamma + 1);

    row_stats_kernel<T, ALIGNED><<<(unsigned)(L.rows_total * L.nchunks), kThreads, 0, stream>>>(
        target, draft, tstride, dstride, B, gamma, V, k, L.nchunks, stats);
    const size_t sm2 = 2 * (gamma + 1) * sizeof(double) + 2 * (gamma + 1) * sizeof(float);
    prefix_weights_kernel<T><<<B, 64, sm2, stream>>>(target, draft, tstride, dstride, tokens, gamma, V, k, kd, kd / (double)k - 1.0, L.nchunks,
                                                    n_target_rows, algo, stats, coef, draft_lens, uniforms, debug_out ? 1 : 0);
    const unsigned pair_blocks = (unsigned)((size_t)B * gamma * L.nchunks);
    residual_kernel<T, ALIGNED><<<pair_blocks, kThreads, 0, stream>>>(
        target, draft, tstride, dstride, gamma, V, k, L.nchunks, coef, spart);
    const size_t sm4 = (gamma + 1) * sizeof(double);
    finalize_kernel<T, ALIGNED><<<B, kThreads, sm4, stream>>>(
        target, draft, tstride, dstride, uniforms, gamma, V, k, L.nchunks, algo, stats, coef, spart,
        accept_len, next_token, debug_out, draft_lens);
    return hipGetLastError() == hipSuccess ? SV_OK : SV_ERR_HIP;
}

// Probabilities as inputs: three launches, every element read once.  Scratch: the staged path's areas
// (chunk partial sums where its row statistics go, the weights where its row constants go).
template <typename T, bool ALIGNED>
sv_status_t launch_probs(int algo, const void *target_v, const void *draft_v, const int32_t *tokens, const int32_t *draft_lens,
                         size_t tstride, size_t dstride, const float *uniforms, int B, int gamma, int V, const Layout &L,
                         char *ws, int32_t *accept_len, int32_t *next_token, float *debug_out, hipStream_t stream)
{
    static_assert(sizeof(ProbWeight) <= sizeof(SeqCoef), "the weights reuse the staged path's row-constant area");
    const T *target = static_cast<const T *>(target_v);
    const T *draft = static_cast<const T *>(draft_v);
    float2 *part = reinterpret_cast<float2 *>(ws + L.off_stats);
    ProbWeight *weights = reinterpret_cast<ProbWeight *>(ws + L.off_coef);
    const unsigned blocks = (unsigned)((size_t)B * (gamma + 1) * L.nchunks);
    probs_weights_kernel<T><<<B, 64, 0, stream>>>(target, draft, tstride, dstride, tokens, draft_lens, gamma, algo, weights, uniforms, debug_out ? 1 : 0);
    if (algo == kGreedy)
        probs_residual_kernel<T, ALIGNED, true><<<blocks, kThreads, 0, stream>>>(
            target, draft, tstride, dstride, draft_lens, gamma, V, L.nchunks, part, weights);
    else
        probs_residual_kernel<T, ALIGNED, false><<<blocks, kThreads, 0, stream>>>(
            target, draft, tstride, dstride, draft_lens, gamma, V, L.nchunks, part, weights);
    const size_t kept_floats = (size_t)(gamma + 1) * L.nchunks * (algo == kGreedy ? 2 : 1);      // chunk sums (Alg. 4: and rejected masses)
    const size_t keep = kept_floats <= (size_t)kProbsKeepMax ? kept_floats * sizeof(float) : 0;
    probs_finalize_kernel<T, ALIGNED><<<B, kThreads, 2 * (gamma + 1) * sizeof(double) + keep, stream>>>(
        target, draft, tstride, dstride, uniforms, draft_lens, gamma, V, L.nchunks, algo, part, weights,
        accept_len, next_token, debug_out);
    return hipGetLastError() == hipSuccess ? SV_OK : SV_ERR_HIP;
}

// Whether a sequence's 2 gamma + 1 rows fit the LDS of one workgroup.
bool tiny_ok(int gamma, int V) { return (size_t)(2 * gamma + 1) * (size_t)V <= (size_t)kTinyMaxFloats; }

template <typename T>
sv_status_t launch_tiny(int algo, const void *target, const void *draft, const int32_t *tokens, const int32_t *draft_lens,
                        size_t tstride, size_t dstride, const float *uniforms, int B, int gamma, int V, float k, double kd,
                        char *ws, int32_t *accept_len, int32_t *next_token, float *debug_out, hipStream_t stream)
{
    if (!tiny_ok(gamma, V)) return SV_ERR_UNSUPPORTED;
    FusedParams P = {};
    P.target = target; P.draft = draft; P.tokens = tokens; P.draft_lens = draft_lens; P.uniforms = uniforms;
    P.B = B; P.gamma = gamma; P.V = V; P.tstride = tstride; P.dstride = dstride;
    P.k = k; P.kd = kd; P.k_eps = kd / (double)k - 1.0; P.algo = algo;
    P.magic = workspace_magic(B, gamma, V);
    P.inv_wpr = V > 1 ? (unsigned)(0x100000000ull / (unsigned)V) + 1u : 0u;
    P.header = reinterpret_cast<int *>(ws);
    P.accept_len = accept_len; P.next_token = next_token; P.debug_out = debug_out;
#ifdef SV_PROFILE
    P.prof = g_prof.load();
#endif
    tiny_verify_kernel<T><<<(unsigned)B, kTinyThreads, 0, stream>>>(P);
    return hipGetLastError() == hipSuccess ? SV_OK : SV_ERR_HIP;
}

// The arguments that the kernels working through the control words share: the inputs, the outputs, the words.
FusedParams word_params(int algo, const void *target, const void *draft, const int32_t *tokens, const int32_t *draft_lens,
                        size_t tstride, size_t dstride, const float *uniforms, int B, int gamma, int V, float k, double kd, const Layout &L,
                        char *ws, int32_t *accept_len, int32_t *next_token, float *debug_out)
{
    FusedParams P = {};
    P.target = target; P.draft = draft; P.tokens = tokens; P.draft_lens = draft_lens; P.uniforms = uniforms;
    P.tstride = tstride; P.dstride = dstride;
    P.B = B; P.gamma = gamma; P.V = V; P.k = k; P.kd = kd; P.k_eps = kd / (double)k - 1.0; P.algo = algo;
    P.nu = L.nu;
    P.spin_limit = g_spin_limit.load();
    P.magic = workspace_magic(B, gamma, V);
    P.header = reinterpret_cast<int *>(ws);
    P.gen = reinterpret_cast<int *>(ws + L.off_gen);
    P.words.ratio = reinterpret_cast<u64 *>(ws + L.off_ratio);
    P.words.lw = reinterpret_cast<u64 *>(ws + L.off_lw);
    P.words.rowres = reinterpret_cast<u64 *>(ws + L.off_rowres);
    P.words.pstat = reinterpret_cast<u64 *>(ws + L.off_pstat);
    P.words.plast = reinterpret_cast<u64 *>(ws + L.off_plast);
    P.words.pgrp = reinterpret_cast<u64 *>(ws + L.off_pgrp);
    P.words.qgrp = reinterpret_cast<u64 *>(ws + L.off_qgrp);
    P.words.spart = reinterpret_cast<unsigned *>(ws + L.off_spart);
    P.words.lseen = reinterpret_cast<u64 *>(ws + L.off_lseen);
    P.copy_bytes = L.copy_bytes;
    P.accept_len = accept_len; P.next_token = next_token; P.debug_out = debug_out;
#ifdef SV_PROFILE
    P.prof = g_prof.load();
#endif
    return P;
}

// The kernel for calls of few resident sets; SV_ERR_UNSUPPORTED for the calls it does not take (more workgroups than
// kResidentSets times what the device keeps resident, rows of more than kResidentMaxGroups workgroups).
template <typename T, bool ALIGNED>
sv_status_t launch_resident(int algo, const void *target, const void *draft, const int32_t *tokens, const int32_t *draft_lens,
                            size_t tstride, size_t dstride, const float *uniforms, int B, int gamma, int V, float k, double kd, const Layout &L,
                            char *ws, int32_t *accept_len, int32_t *next_token, float *debug_out, hipStream_t stream)
{
    const int nwg = L.nu / kWaves;
    if (nwg > kResidentMaxGroups || B > 65535) return SV_ERR_UNSUPPORTED;
    static std::atomic<int> cap;
    void (*kernel)(const FusedParams) = resident_verify_kernel<T, ALIGNED>;
    const int capacity = resident_workgroups(kernel, cap);
    if (capacity < 1) return SV_ERR_HIP;
    if ((long long)nwg * B * (gamma + 1) > (long long)kResidentSets * capacity) return SV_ERR_UNSUPPORTED;
    const FusedParams P = word_params(algo, target, draft, tokens, draft_lens, tstride, dstride, uniforms, B, gamma, V, k, kd, L,
                                      ws, accept_len, next_token, debug_out);
    kernel<<<dim3((unsigned)nwg, (unsigned)B, (unsigned)(gamma + 1)), kThreads, 0, stream>>>(P);
    return hipGetLastError() == hipSuccess ? SV_OK : SV_ERR_HIP;
}

template <typename T, bool ALIGNED>
sv_status_t launch_fused(int algo, const void *target, const void *draft, const int32_t *tokens, const int32_t *draft_lens,
                         size_t tstride, size_t dstride, const float *uniforms, int B, int gamma, int V, float k, double kd, const Layout &L,
                         char *ws, int32_t *accept_len, int32_t *next_token, float *debug_out,
                         hipStream_t stream)
{
    // Unit size: 32 logits per lane (5 waves per SIMD).  The kernel also exists with 64 per lane (3 waves per SIMD, half
    // as many workgroups per row to wait for; bf16 rows on the vector path), which used to be the faster one for very wide
    // rows; since the smaller units publish less it is not any more (B = 1024, gamma = 8, V = 256000: 1414 - 1424 us
    // against 1435 - 1439), and only the testing hook asks for it.
    // The workspace is laid out for the smaller units, whose words are a superset.
    constexpr bool kLargeOk = ALIGNED && ElemTraits<T>::kVec == 8;
    const bool large = kLargeOk && g_lane.load() == kLaneLarge;
    const int lane_logits = large ? kLaneLarge : kLaneSmall;
    const int nu = (V + kWaves * kWave * lane_logits - 1) / (kWaves * kWave * lane_logits) * kWaves;
    // the instantiation for this row width (one or two words of a row per lane of the collecting wave) and its
    // resident workgroups
    static std::atomic<int> cap[2][2];
    const int nwg = nu / kWaves;
    const int nw_log = nwg <= kWave ? 0 : 1;
    void (*kernel)(const FusedParams) = nullptr;
#define SV_PICK(LN) (nw_log == 0 ? fused_verify_kernel<T, ALIGNED, 1, LN> : fused_verify_kernel<T, ALIGNED, 2, LN>)
    if constexpr (kLargeOk) {
        if (large) kernel = SV_PICK(kLaneLarge);
    }
    if (!kernel) kernel = SV_PICK(kLaneSmall);
#undef SV_PICK
    const int capacity = resident_workgroups(kernel, cap[nw_log][large ? 1 : 0]);
    const int wpr = nwg;
    // a row's workgroups wait for each other and must fit on the device together, with room to spare
    if (capacity < 4 * wpr) return capacity < 1 ? SV_ERR_HIP : SV_ERR_UNSUPPORTED;
    FusedParams P = word_params(algo, target, draft, tokens, draft_lens, tstride, dstride, uniforms, B, gamma, V, k, kd, L,
                                ws, accept_len, next_token, debug_out);
    P.nu = nu;
    P.inv_slots = (unsigned)(0x100000000ull / (unsigned)(gamma + 1)) + 1u;
    P.inv_wpr = (unsigned)(0x100000000ull / (unsigned)(nu / kWaves)) + 1u;
    // groups of sequences so large that one position of a group fills the device at least once
    const int min_seqs = (capacity + wpr - 1) / wpr;
    const int groups = B / min_seqs > 1 ? B / min_seqs : 1;
    P.group_seqs = (B + groups - 1) / groups;
    const int n_groups = (B + P.group_seqs - 1) / P.group_seqs;
    if ((size_t)n_groups * (gamma + 1) > 65535u || P.group_seqs > 65535) return SV_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)wpr, (unsigned)P.group_seqs, (unsigned)(n_groups * (gamma + 1)));
    // (the testing hook's forced unit sizes also force the pruning, so that small test shapes exercise it)
    P.prune = g_lane.load() != 0 || (size_t)wpr * P.group_seqs * n_groups * (gamma + 1) > (size_t)capacity ? 1 : 0;
    P.skip_last = P.prune;
    kernel<<<grid, kThreads, 0, stream>>>(P);
    return hipGetLastError() == hipSuccess ? SV_OK : SV_ERR_HIP;
}

sv_status_t verify_entry(int algo, bool probs, const void *target, const void *draft, const int32_t *tokens, const int32_t *draft_lens,
                         int64_t target_row_stride, int64_t draft_row_stride,
                         const float *uniforms, int32_t B, int32_t gamma, int32_t V, sv_dtype_t dtype,
                         float temperature, void *workspace, size_t workspace_bytes,
                         int32_t *accept_len, int32_t *next_token, float *debug_out, void *stream_v)
{
    if (!target || !draft || !tokens || !uniforms || !workspace || !accept_len || !next_token)
        return SV_ERR_INVALID_ARG;
    if (B < 1 || gamma < 1 || V < 1) return SV_ERR_INVALID_ARG;
    if (!probs && (!(temperature > 0.f) || !isfinite(temperature))) return SV_ERR_INVALID_ARG;
    if (dtype != SV_DTYPE_F32 && dtype != SV_DTYPE_BF16) return SV_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return SV_ERR_INVALID_ARG;
    Layout L;
    if (!make_layout(B, gamma, V, L)) return SV_ERR_UNSUPPORTED;
    if (workspace_bytes < L.total) return SV_ERR_WORKSPACE_TOO_SMALL;

    const double kd = 1.4426950408889634074 / (double)temperature;
    const float k = (float)kd;
    const size_t esize = dtype == SV_DTYPE_F32 ? 4 : 2;
    // rows are V logits, target_row_stride / draft_row_stride elements apart (0: dense, the stride is V)
    if (target_row_stride < 0 || draft_row_stride < 0) return SV_ERR_INVALID_ARG;
    const size_t tstride = target_row_stride ? (size_t)target_row_stride : (size_t)V;
    const size_t dstride = draft_row_stride ? (size_t)draft_row_stride : (size_t)V;
    if (tstride < (size_t)V || dstride < (size_t)V) return SV_ERR_INVALID_ARG;
    const bool aligned = ((reinterpret_cast<uintptr_t>(target) | reinterpret_cast<uintptr_t>(draft)) & 15u) == 0 &&
                         ((size_t)V * esize) % 16 == 0 && (tstride * esize) % 16 == 0 && (dstride * esize) % 16 == 0;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char *ws = static_cast<char *>(workspace);
    if (probs) {
#define SV_PROBS(TT, AL) launch_probs<TT, AL>(algo, target, draft, tokens, draft_lens, tstride, dstride, uniforms, B, gamma, V, \
                                              L, ws, accept_len, next_token, debug_out, stream)
        g_last_kernel.store(SV_KERNEL_PROBS);
        return dtype == SV_DTYPE_F32 ? (aligned ? SV_PROBS(float, true) : SV_PROBS(float, false))
                                     : (aligned ? SV_PROBS(bf16_t, true) : SV_PROBS(bf16_t, false));
#undef SV_PROBS
    }
    const int path = g_path.load();
    if (path == 2 && !L.fused_ok) return SV_ERR_UNSUPPORTED;
    // sequences small enough for one workgroup each need nothing between workgroups
    if (path == 5 || (path == 0 && tiny_ok(gamma, V))) {
        g_last_kernel.store(SV_KERNEL_TINY);
        return dtype == SV_DTYPE_F32
            ? launch_tiny<float>(algo, target, draft, tokens, draft_lens, tstride, dstride, uniforms, B, gamma, V, k, kd, ws, accept_len, next_token, debug_out, stream)
            : launch_tiny<bf16_t>(algo, target, draft, tokens, draft_lens, tstride, dstride, uniforms, B, gamma, V, k, kd, ws, accept_len, next_token, debug_out, stream);
    }

#define SV_ARGS algo, target, draft, tokens, draft_lens, tstride, dstride, uniforms, B, gamma, V, k, kd, L, ws, \
                accept_len, next_token, debug_out, stream
#define SV_DISPATCH(FN)                                                                   \
    (dtype == SV_DTYPE_F32 ? (aligned ? FN<float, true>(SV_ARGS) : FN<float, false>(SV_ARGS)) \
                           : (aligned ? FN<bf16_t, true>(SV_ARGS) : FN<bf16_t, false>(SV_ARGS)))
    // calls of few resident sets: the kernel without a row leader's second look at the logits
    if ((path == 7 || path == 0) && L.fused_ok) {
        const sv_status_t st = SV_DISPATCH(launch_resident);
        if (st == SV_OK) g_last_kernel.store(SV_KERNEL_RESIDENT);
        if (st != SV_ERR_UNSUPPORTED || path == 7) return st;
    } else if (path == 7) {
        return SV_ERR_UNSUPPORTED;
    }
    // the fused kernel (every logit read once) is the default; the staged kernels (every logit read twice)
    // take the shapes it does not: rows of more than kMaxUnitsPerRow wave chunks, or rows too wide to fit
    // four times into the device's resident set
    if (path != 1 && L.fused_ok) {
        const sv_status_t st = SV_DISPATCH(launch_fused);
        if (st == SV_OK) g_last_kernel.store(SV_KERNEL_FUSED);
        if (st != SV_ERR_UNSUPPORTED || path == 2) return st;
    } else if (path == 2) {
        return SV_ERR_UNSUPPORTED;
    }
    g_last_kernel.store(SV_KERNEL_STAGED);
    return SV_DISPATCH(launch_staged);
#undef SV_DISPATCH
#undef SV_ARGS
}

// ---- the workspace of spec_verify_ex_noalloc: device memory that belongs to the library's code object, one copy per
// GPU that runs it, alive until the process ends.  The name below is only a handle for hipGetSymbolAddress: the
// address that kernels get is looked up once per device and kept.
__device__ __align__(256) unsigned char g_static_scratch[SV_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
struct StaticScratch {
    void *ptr = nullptr;                 // the array's address on this device
    int32_t B = 0, gamma = 0, V = 0;     // the shape its control words were last prepared for (0: never)
};
std::mutex g_static_mutex;
StaticScratch g_static[kMaxDevices];

}  // namespace

extern "C" {

size_t spec_verify_workspace_bytes(int32_t B, int32_t gamma, int32_t V)
{
    Layout L;
    return make_layout(B, gamma, V, L) ? L.total : 0;
}

sv_status_t spec_verify_workspace_init(void *workspace, size_t workspace_bytes,
                                       int32_t B, int32_t gamma, int32_t V, void *stream)
{
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return SV_ERR_INVALID_ARG;
    if (B < 1 || gamma < 1 || V < 1) return SV_ERR_INVALID_ARG;
    Layout L;
    if (!make_layout(B, gamma, V, L)) return SV_ERR_UNSUPPORTED;
    if (workspace_bytes < L.total) return SV_ERR_WORKSPACE_TOO_SMALL;
    const unsigned grid = (unsigned)((L.control_words + 255) / 256);
    workspace_init_kernel<<<grid, 256, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<int *>(workspace), L.control_words, workspace_magic(B, gamma, V));
    return hipGetLastError() == hipSuccess ? SV_OK : SV_ERR_HIP;
}

sv_status_t spec_verify_workspace_check(const void *workspace, int32_t B, int32_t gamma, int32_t V, void *stream)
{
    if (!workspace) return SV_ERR_INVALID_ARG;
    int words[2] = {0, 0};
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(words, workspace, sizeof(words), hipMemcpyDeviceToHost, s) != hipSuccess) return SV_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return SV_ERR_HIP;
    if (words[kHdrMagic] != workspace_magic(B, gamma, V)) return SV_ERR_INVALID_ARG;
    return words[kHdrError] == 0 ? SV_OK : SV_ERR_INTERNAL;
}

int32_t spec_verify_debug_last_kernel(void) { return g_last_kernel.load(); }

void spec_verify_debug_config(int32_t path, int32_t spin_limit)
{
    g_path.store((path >= 0 && path <= 2) || path == 5 || path == 7 ? path : path == 3 || path == 4 ? 2 : 0);
    g_lane.store(path == 3 ? kLaneSmall : path == 4 ? kLaneLarge : 0);
    g_spin_limit.store(spin_limit >= 0 ? spin_limit : kDefaultSpinLimit);
}

// Plain copy, 16 bytes per thread and step: what the HBM traffic counters are calibrated against.
namespace { __global__ __launch_bounds__(256) void copy_probe_kernel(uint4 *dst, const uint4 *src, size_t nvec)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (size_t)gridDim.x * 256) dst[i] = src[i];
} }

sv_status_t spec_verify_debug_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src || bytes == 0 || bytes % 16 != 0) return SV_ERR_INVALID_ARG;
    if (((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15u) != 0) return SV_ERR_INVALID_ARG;
    const size_t nvec = bytes / 16;
    const size_t blocks = (nvec + 255) / 256;
    copy_probe_kernel<<<(unsigned)(blocks < 65536 ? blocks : 65536), 256, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<uint4 *>(dst), static_cast<const uint4 *>(src), nvec);
    return hipGetLastError() == hipSuccess ? SV_OK : SV_ERR_HIP;
}

// What a one-pass kernel of the fused kernel's launch shape can reach: one 256-thread workgroup per 2 x 16 KB (a wave
// reads 4 KB of each of two buffers with eight 16-byte loads per lane, all issued up front), the first sweep's
// arithmetic on bf16 (unpack, maximum, exp2, sum), no traffic between workgroups.  Its registers would let eight waves
// share a SIMD; the launch asks for kProbeLdsBytes of LDS per workgroup so that five workgroups fit a compute unit, as
// with the verifying kernel (five times 32 KiB do not fit beside what the hardware keeps of the 160 KiB for itself:
// 32768 bytes give four workgroups, 32000 give five - found by timing the probe with waits over a range of sizes).
constexpr unsigned kProbeLdsBytes = 32000;
namespace { __global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(5)))
void stream_probe_kernel(const uint4 *a, const uint4 *b, float *out, int short_waits, int long_waits)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint4 *pa = a + (size_t)blockIdx.x * 1024 + wave * 256 + lane;
    const uint4 *pb = b + (size_t)blockIdx.x * 1024 + wave * 256 + lane;
    uint4 va[4], vb[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) va[j] = load_streamed(pa + j * 64);
#pragma unroll
    for (int j = 0; j < 4; ++j) vb[j] = load_streamed(pb + j * 64);
    float res = 0.f;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const uint4 *v = r ? vb : va;
        float x[32];
#pragma unroll
        for (int j = 0; j < 4; ++j) unpack_vec<bf16_t>(v[j], x + j * 8);
        float shift;
        const u64 word = first_sweep_row(x, 1.8f, shift);
        res += stat_sum(word) + shift;
    }
    // the waits of a verifying kernel, modelled: a workgroup keeps its registers for a while after its sweep (the look
    // at log2 w_i; for one in four "rows" of 16 neighbouring workgroups the wait for the row and the second sweep)
    const int waits = ((blockIdx.x >> 4) & 3) == 0 ? long_waits : short_waits;
    if (waits > 0) {
        __syncthreads();
        for (int i = 0; i < waits; ++i) __builtin_amdgcn_s_sleep(8);        // 512 clocks each
        __syncthreads();
    }
    if (lane == 0) out[(size_t)blockIdx.x * 4 + wave] = res;
} }

sv_status_t spec_verify_debug_stream_probe(const void *a, const void *b, size_t bytes_each, float *out,
                                           int32_t short_waits, int32_t long_waits, void *stream)
{
    if (!a || !b || !out || bytes_each == 0 || bytes_each % 16384 != 0) return SV_ERR_INVALID_ARG;
    if (short_waits < 0 || long_waits < 0 || short_waits > 64 || long_waits > 64) return SV_ERR_INVALID_ARG;
    if (((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b)) & 15u) != 0) return SV_ERR_INVALID_ARG;
    const size_t blocks = bytes_each / 16384;
    if (blocks > 0x7fffffffull) return SV_ERR_UNSUPPORTED;
    stream_probe_kernel<<<(unsigned)blocks, 256, kProbeLdsBytes, static_cast<hipStream_t>(stream)>>>(
        static_cast<const uint4 *>(a), static_cast<const uint4 *>(b), out, short_waits, long_waits);
    return hipGetLastError() == hipSuccess ? SV_OK : SV_ERR_HIP;
}

sv_status_t spec_sample_tokens(const void *logits, int64_t rows, int32_t V, sv_dtype_t dtype, float temperature,
                               const float *uniforms, int32_t *tokens, void *stream_v)
{
    if (!logits || !uniforms || !tokens) return SV_ERR_INVALID_ARG;
    if (rows < 1 || V < 1) return SV_ERR_INVALID_ARG;
    if (!(temperature > 0.f) || !isfinite(temperature)) return SV_ERR_INVALID_ARG;
    if (dtype != SV_DTYPE_F32 && dtype != SV_DTYPE_BF16) return SV_ERR_INVALID_ARG;
    if (rows > 0x7fffffffll) return SV_ERR_UNSUPPORTED;
    const float k = (float)(1.4426950408889634074 / (double)temperature);
    const unsigned threads = V > 8192 ? kThreads : kWave;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    if (dtype == SV_DTYPE_F32)
        sample_rows_kernel<float><<<(unsigned)rows, threads, 0, stream>>>(static_cast<const float *>(logits), V, k, uniforms, tokens);
    else
        sample_rows_kernel<bf16_t><<<(unsigned)rows, threads, 0, stream>>>(static_cast<const bf16_t *>(logits), V, k, uniforms, tokens);
    return hipGetLastError() == hipSuccess ? SV_OK : SV_ERR_HIP;
}

#ifdef SV_PROFILE
void spec_verify_debug_profile(void *device_buffer)
{
    g_prof.store(static_cast<long long *>(device_buffer));
}
#endif

sv_status_t spec_verify_block(const void *target_logits, const void *draft_logits,
                              const int32_t *draft_tokens, const float *uniforms,
                              int32_t B, int32_t gamma, int32_t V, sv_dtype_t dtype,
                              float temperature, void *workspace, size_t workspace_bytes,
                              int32_t *accept_len, int32_t *next_token, float *debug_out, void *stream)
{
    return verify_entry(kBlock, false, target_logits, draft_logits, draft_tokens, nullptr, 0, 0, uniforms, B, gamma, V, dtype,
                        temperature, workspace, workspace_bytes, accept_len, next_token, debug_out, stream);
}

sv_status_t spec_verify_token(const void *target_logits, const void *draft_logits,
                              const int32_t *draft_tokens, const float *uniforms,
                              int32_t B, int32_t gamma, int32_t V, sv_dtype_t dtype,
                              float temperature, void *workspace, size_t workspace_bytes,
                              int32_t *accept_len, int32_t *next_token, float *debug_out, void *stream)
{
    return verify_entry(kToken, false, target_logits, draft_logits, draft_tokens, nullptr, 0, 0, uniforms, B, gamma, V, dtype,
                        temperature, workspace, workspace_bytes, accept_len, next_token, debug_out, stream);
}

sv_status_t spec_verify_greedy(const void *target_logits, const void *draft_logits,
                               const int32_t *draft_tokens, const float *uniforms,
                               int32_t B, int32_t gamma, int32_t V, sv_dtype_t dtype,
                               float temperature, void *workspace, size_t workspace_bytes,
                               int32_t *accept_len, int32_t *next_token, float *debug_out, void *stream)
{
    return verify_entry(kGreedy, false, target_logits, draft_logits, draft_tokens, nullptr, 0, 0, uniforms, B, gamma, V, dtype,
                        temperature, workspace, workspace_bytes, accept_len, next_token, debug_out, stream);
}

sv_status_t spec_verify_ex(sv_algo_t algo, const void *target_logits, const void *draft_logits,
                           const int32_t *draft_tokens, const int32_t *draft_lens,
                           int64_t target_row_stride, int64_t draft_row_stride, const float *uniforms,
                           int32_t B, int32_t gamma, int32_t V, sv_dtype_t dtype,
                           float temperature, void *workspace, size_t workspace_bytes,
                           int32_t *accept_len, int32_t *next_token, float *debug_out, void *stream)
{
    if (algo != SV_ALGO_BLOCK && algo != SV_ALGO_TOKEN && algo != SV_ALGO_GREEDY) return SV_ERR_INVALID_ARG;
    const int a = algo == SV_ALGO_BLOCK ? kBlock : algo == SV_ALGO_TOKEN ? kToken : kGreedy;
    return verify_entry(a, false, target_logits, draft_logits, draft_tokens, draft_lens, target_row_stride, draft_row_stride,
                        uniforms, B, gamma, V, dtype, temperature, workspace, workspace_bytes, accept_len, next_token,
                        debug_out, stream);
}

sv_status_t spec_verify_probs(sv_algo_t algo, const void *target_probs, const void *draft_probs,
                              const int32_t *draft_tokens, const int32_t *draft_lens,
                              int64_t target_row_stride, int64_t draft_row_stride, const float *uniforms,
                              int32_t B, int32_t gamma, int32_t V, sv_dtype_t dtype,
                              void *workspace, size_t workspace_bytes,
                              int32_t *accept_len, int32_t *next_token, float *debug_out, void *stream)
{
    if (algo != SV_ALGO_BLOCK && algo != SV_ALGO_TOKEN && algo != SV_ALGO_GREEDY) return SV_ERR_INVALID_ARG;
    const int a = algo == SV_ALGO_BLOCK ? kBlock : algo == SV_ALGO_TOKEN ? kToken : kGreedy;
    return verify_entry(a, true, target_probs, draft_probs, draft_tokens, draft_lens, target_row_stride, draft_row_stride,
                        uniforms, B, gamma, V, dtype, 1.f, workspace, workspace_bytes, accept_len, next_token,
                        debug_out, stream);
}

sv_status_t spec_verify_ex_noalloc(sv_algo_t algo, const void *target_logits, const void *draft_logits,
                                   const int32_t *draft_tokens, const int32_t *draft_lens,
                                   int64_t target_row_stride, int64_t draft_row_stride, const float *uniforms,
                                   int32_t B, int32_t gamma, int32_t V, sv_dtype_t dtype, float temperature,
                                   int32_t *accept_len, int32_t *next_token, float *debug_out, void *stream)
{
    if (algo != SV_ALGO_BLOCK && algo != SV_ALGO_TOKEN && algo != SV_ALGO_GREEDY) return SV_ERR_INVALID_ARG;
    if (B < 1 || gamma < 1 || V < 1) return SV_ERR_INVALID_ARG;
    Layout L;
    if (!make_layout(B, gamma, V, L)) return SV_ERR_UNSUPPORTED;
    if (L.total > (size_t)SV_STATIC_SCRATCH_BYTES) return SV_ERR_STATIC_SCRATCH_TOO_SMALL;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return SV_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return SV_ERR_UNSUPPORTED;
    void *ws = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_static_mutex);
        StaticScratch &st = g_static[dev];
        if (!st.ptr) {
            // once per device, with that device current: every GPU holds its own copy of the array at its own address
            void *p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)) != hipSuccess || !p) return SV_ERR_HIP;
            st.ptr = p;
        }
        ws = st.ptr;
        if (st.B != B || st.gamma != gamma || st.V != V) {
            // the array keeps what the last call left: its control words are prepared again whenever the shape changes
            // (a kernel on the caller's stream, in front of the verification's)
            const sv_status_t rc = spec_verify_workspace_init(ws, SV_STATIC_SCRATCH_BYTES, B, gamma, V, stream);
            if (rc != SV_OK) return rc;
            st.B = B; st.gamma = gamma; st.V = V;
        }
    }
    const int a = algo == SV_ALGO_BLOCK ? kBlock : algo == SV_ALGO_TOKEN ? kToken : kGreedy;
    return verify_entry(a, false, target_logits, draft_logits, draft_tokens, draft_lens, target_row_stride, draft_row_stride,
                        uniforms, B, gamma, V, dtype, temperature, ws, SV_STATIC_SCRATCH_BYTES, accept_len, next_token,
                        debug_out, stream);
}

const char *spec_verify_status_string(sv_status_t status)
{
    switch (status) {
    case SV_OK: return "ok";
    case SV_ERR_INVALID_ARG: return "invalid argument";
    case SV_ERR_UNSUPPORTED: return "unsupported size";
    case SV_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case SV_ERR_HIP: return "HIP call failed";
    case SV_ERR_INTERNAL: return "a bounded wait inside the kernel ran out";
    case SV_ERR_STATIC_SCRATCH_TOO_SMALL: return "the sizes need more than the library's built-in scratch memory";
    }
    return "unknown status";
}

}  // extern "C"
