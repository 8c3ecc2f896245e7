/*
 * specverify -- batched draft verification for speculative decoding on AMD MI355X (gfx950).
 *
 * One call verifies B independent sequences.  For sequence b the caller hands over the
 * target model's logits at gamma+1 positions, the draft model's logits at gamma positions,
 * the gamma drafted tokens and gamma+1 uniforms; the library returns the accept length tau
 * and the extra token Y, so that the text to append is X_1..X_tau, Y ("Return X^tau, Y" in
 * Alg. 1 and Alg. 2 of "Block Verification Accelerates Speculative Decoding").
 *
 * Definitions (row i of a sequence is conditioned on the first i draft tokens):
 *   p_i = softmax(target row i / T), i = 0..gamma;  q_i = softmax(draft row i / T), i < gamma;
 *   r_i = p_{i-1}(X_i) / q_{i-1}(X_i)                 (acceptance ratio, Sec. 1)
 *   block verification (Alg. 2):  w_0 = 1, w_i = min(w_{i-1} r_i, 1);
 *       S_i = sum_x max(w_i p_i(x) - q_i(x), 0),  h_i = S_i / (S_i + 1 - w_i) for i < gamma,
 *       h_gamma = w_gamma (the acceptance-probability box next to Alg. 2);
 *       tau = the LAST i in 1..gamma with eta_i < h_i, or 0;
 *       Y ~ p_gamma if tau = gamma, else Y ~ max(w_tau p_tau - q_tau, 0) normalised.
 *   token verification (Alg. 1):  h_i = min(r_i, 1); tau = number of leading i with
 *       eta_i < h_i; Y ~ p_gamma if tau = gamma, else Y ~ max(p_tau - q_tau, 0) normalised.
 *   greedy block verification (Alg. 4):  w_i = w_{i-1} r_i (no clip);
 *       h_i = S_i / sum_x max(q_i(x) - w_i p_i(x), 0) for i < gamma, h_gamma = w_gamma;
 *       tau and Y as in block verification.
 * Conventions the paper leaves open: uniforms lie in [0,1) and a test passes iff eta < h;
 * h_i = 1 when w_i >= 1; Y is an inverse-CDF draw in vocabulary-index order:
 * Y = min{x : sum_{x' <= x} rho(x') > u * sum rho}, so a token of zero weight is never drawn.
 *
 * All data pointers are DEVICE pointers owned by the caller.  Calls are asynchronous: work
 * is enqueued on `stream` (a hipStream_t passed as void*; NULL is the default stream) and
 * the outputs are valid once the caller has synchronised that stream.  The library never
 * allocates, frees or synchronises, and keeps no reference to any argument after return.
 * Errors are reported by return code only.  Logits are finite (|logit| * log2(e) / T within float
 * range) or -inf (a token masked out by
 * top-k / top-p warping: probability exactly 0), never +inf or NaN; every row keeps at least one
 * finite logit and a drafted token has a finite DRAFT logit (its target logit may be -inf: its
 * ratio is then 0 and it is never accepted).  That, tokens in [0, V) and uniforms in [0, 1) are
 * the caller's contract and are not checked on the device.
 *
 * Calls that share a workspace must not overlap (two calls may run concurrently only with disjoint workspaces); the
 * testing hook spec_verify_debug_config and the one-time look at the device below are the only process-wide state.
 * Graph capture: a call is kernel launches only, but the FIRST call of each kernel variant (logit type, alignment,
 * row width class) asks the runtime once how many of its workgroups the device holds at a time; make one call of the
 * shape outside the capture first.
 * If the verification kernel ever gives up one of its (bounded) waits - which needs a device that does not start
 * workgroups in index order, or another kernel that takes its compute units away for seconds - the sequences concerned
 * get accept_len = next_token = -1 instead of a result, and spec_verify_workspace_check reports SV_ERR_INTERNAL.
 */
#ifndef SPECVERIFY_H
#define SPECVERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SV_OK = 0,
    SV_ERR_INVALID_ARG = 1,          /* NULL pointer, B/gamma/V < 1, bad dtype, T not finite or <= 0 */
    SV_ERR_UNSUPPORTED = 2,          /* gamma above SV_MAX_GAMMA, or sizes that overflow 32-bit grids  */
    SV_ERR_WORKSPACE_TOO_SMALL = 3,
    SV_ERR_HIP = 4,                  /* a launch or copy failed; see hipGetLastError                   */
    SV_ERR_INTERNAL = 5,             /* workspace_check: a bounded wait inside a kernel ran out        */
    SV_ERR_STATIC_SCRATCH_TOO_SMALL = 6  /* spec_verify_ex_noalloc: sizes beyond SV_STATIC_SCRATCH_BYTES  */
} sv_status_t;

typedef enum { SV_DTYPE_F32 = 0, SV_DTYPE_BF16 = 1 } sv_dtype_t;

#define SV_MAX_GAMMA 64

/* Bytes of device workspace a call with these sizes needs (0 if the sizes are invalid).
 * The workspace must be 256-byte aligned.                                                 */
size_t spec_verify_workspace_bytes(int32_t B, int32_t gamma, int32_t V);

/* Prepares a workspace for calls of exactly the shape (B, gamma, V): enqueues one small
 * kernel on `stream` that clears the control words the verification kernel synchronises
 * its workgroups with (they exist twice; a sequence's calls use the two copies alternately and
 * each call clears the copy it does not use).  Required once after allocation (and again before
 * using the same memory for another shape, or after a call that reported -1); every
 * verification call leaves the workspace ready for the next one (its contents between calls
 * are the library's business: do not clear or copy parts of it).  Calls that share a workspace must not overlap; calls on
 * different streams need workspaces of their own.
 * A verification call on a workspace that was not initialised for its shape
 * touches nothing else and writes -1 to every accept_len and next_token.                  */
sv_status_t spec_verify_workspace_init(void *workspace, size_t workspace_bytes,
                                       int32_t B, int32_t gamma, int32_t V, void *stream);

/* Synchronises `stream` and reads the workspace's status words back to the host: SV_OK,
 * SV_ERR_INVALID_ARG if the workspace is not initialised for this shape, SV_ERR_INTERNAL
 * if a workgroup gave up a bounded wait during an earlier call (that call wrote -1 for the
 * sequences concerned; re-initialise the workspace).  Meant for tests and debugging: it is
 * the one entry point that blocks.                                                        */
sv_status_t spec_verify_workspace_check(const void *workspace, int32_t B, int32_t gamma, int32_t V,
                                        void *stream);

/* Testing hook, process-wide: `path` 0 = the library's choice by the shape of the call: sequences whose
 * 2 gamma + 1 rows fit into LDS together, (2 gamma + 1) V <= 14336: the kernel of one workgroup per
 * sequence; else, calls of at most three times the workgroups that the device keeps resident and rows
 * of at most 32 * 8192 logits: the kernel for calls of few resident sets; else the fused kernel where it
 * takes the shape, else the staged kernels.  5 = the one-workgroup-per-sequence kernel, 7 = the
 * kernel for calls of few resident sets (calls beyond their limits are then refused), 1 = the
 * four-launch staged kernels, 2 = the
 * single-launch fused kernel (takes V <= 128 * 8192 and a device that keeps four rows'
 * workgroups resident; other shapes are then refused), 3 / 4 = the fused kernel with its
 * small / large units (32 / 64 logits of a row per lane; large ones exist for bf16 rows on
 * the 16-byte path only, other calls use the small ones; the library by itself takes the small
 * ones; both also switch on, whatever the size of the call, what the library otherwise
 * does only in calls larger than one resident set of workgroups: residual masses that cannot
 * matter are left out, the last target row is read only where every token can be accepted, and
 * w_i travels from position to position as one published word); `spin_limit` bounds every wait
 * inside the kernels that wait for each other's words, in polls (negative: default).        */
void spec_verify_debug_config(int32_t path, int32_t spin_limit);

/* Testing hook: which kernels the last verification call of this process launched (0 before the first).  */
enum {
    SV_KERNEL_STAGED = 1,     /* the four staged kernels                                   */
    SV_KERNEL_FUSED = 2,      /* the single-launch fused kernel                            */
    SV_KERNEL_TINY = 5,       /* one workgroup per sequence                                */
    SV_KERNEL_RESIDENT = 7,   /* the kernel for calls of few resident sets                 */
    SV_KERNEL_PROBS = 8       /* the three kernels that take probabilities                 */
};
int32_t spec_verify_debug_last_kernel(void);

#ifdef SPECVERIFY_PROFILE_BUILD
/* Tuning builds of the library only (compiled with -DSV_PROFILE; the product library exports no such symbol and
 * its kernels hold no such stores).  Process-wide: when `device_buffer` is not NULL the fused kernel stores up to
 * sixteen 64-bit timestamps (100 MHz ticks) per workgroup into it, taken by the workgroup's first wave: 0 start,
 * 1 partial normalisers announced, 2 the row's normalisers and w_i known, 3 second sweep begins, 4 second sweep
 * done; for the workgroup that finishes a sequence also 5 begin, 7..12 its phases, 6 done (the kernel for calls of
 * few resident sets: 0 start, 1 first sweep done, 7 the row's words in, 8 ratio out, 9 w_i known, 2 row constants,
 * 4 second sweep done, 5 the row's shares in, 10 place of the token found, 15 position's word out, 6 tau and Y
 * written).  Record r of the buffer
 * belongs to workgroup x of row slot i (gamma: the last target row) of sequence b, r = (b * (gamma + 1) + i) *
 * ceil(V / 8192) + x: the buffer holds B * (gamma + 1) * ceil(V / 8192) records of 128 bytes and is zeroed by the
 * caller.                                                                                  */
void spec_verify_debug_profile(void *device_buffer);
#endif

/*
 * The drafting step of the outer loop of speculative decoding (Alg. 3: "sample X_1 .. X_gamma from
 * M_s") for a model whose conditional distributions are rows of logits: one token per row from
 * softmax(logits / temperature) by the inverse CDF in vocabulary order, tokens[r] =
 * min{x : C_x > uniforms[r] * C_total} (the convention of the correction token's draw).
 *   logits    [rows, V]  dtype, device, rows dense
 *   uniforms  [rows]     float32 in [0,1), device
 *   tokens    [rows]     int32 out, device
 * Asynchronous on `stream`, allocates nothing.  SV_ERR_INVALID_ARG for null pointers, rows < 1,
 * V < 1, a temperature that is not positive and finite or an unknown dtype; SV_ERR_UNSUPPORTED
 * for more than 2^31 - 1 rows.  Meant for toy and test drafters, not tuned.
 */
sv_status_t spec_sample_tokens(const void *logits, int64_t rows, int32_t V, sv_dtype_t dtype,
                               float temperature, const float *uniforms, int32_t *tokens, void *stream);

/* Measurement hook: copies `bytes` (a multiple of 16, both pointers 16-byte aligned device
 * memory, not overlapping) from `src` to `dst` with a plain copy kernel on `stream`.  It reads
 * and writes exactly `bytes` each, which is what hardware counters of memory traffic are
 * scaled against.  SV_ERR_INVALID_ARG for null, misaligned or ragged arguments.            */
sv_status_t spec_verify_debug_copy(void *dst, const void *src, size_t bytes, void *stream);

/* Measurement hook: the floor of this launch shape.  Reads `bytes_each` bytes (a multiple of 16384) from each of the two
 * 16-byte aligned device buffers `a` and `b` with the access pattern of the verification kernel - one 256-thread
 * workgroup per 2 x 16 KB, eight 16-byte loads per lane issued up front, five workgroups per compute unit (held to
 * that by the LDS the launch asks for: the probe's registers alone would allow eight) - and runs the first
 * sweep's arithmetic on them as bf16 (maximum, exp2, sum), with no traffic between workgroups; one float per wave goes
 * to `out` (bytes_each / 4096 floats).  What this kernel needs for a call's bytes is what no kernel of this shape that
 * also verifies can beat.  `short_waits`, `long_waits` (0 .. 64, units of 512 clocks): how long a workgroup keeps its
 * registers after its sweep before it ends - `long_waits` for one in four groups of 16 neighbouring workgroups,
 * `short_waits` for the others - which models the waits of a kernel that verifies (the look at the weight of the
 * position; the wait for the row and the second sweep) without any of its traffic; 0, 0 is the floor itself.
 * SV_ERR_INVALID_ARG for null, misaligned, ragged or out-of-range arguments.    */
sv_status_t spec_verify_debug_stream_probe(const void *a, const void *b, size_t bytes_each, float *out,
                                           int32_t short_waits, int32_t long_waits, void *stream);

/*
 * Block verification (Alg. 2).
 *   target_logits  [B, gamma+1, V]  dtype, V contiguous, rows dense (stride V)
 *   draft_logits   [B, gamma,   V]  dtype
 *   draft_tokens   [B, gamma]       X_1..X_gamma
 *   uniforms       [B, gamma+1]     eta_1..eta_gamma, then u (draws Y)
 *   temperature    T > 0, applied to both models
 *   accept_len     [B] out: tau in [0, gamma]
 *   next_token     [B] out: Y in [0, V)
 *   debug_out      NULL, or [B, gamma+1, 3] floats out: w_i, S_i, h_i (S_gamma = w_gamma,
 *                  h_0 = 1)
 * 16-byte loads are used when both logit pointers and V*sizeof(dtype) are multiples of 16;
 * any other V or alignment is served by an element-wise path with the same results.
 */
sv_status_t spec_verify_block(const void *target_logits, const void *draft_logits,
                              const int32_t *draft_tokens, const float *uniforms,
                              int32_t B, int32_t gamma, int32_t V, sv_dtype_t dtype,
                              float temperature, void *workspace, size_t workspace_bytes,
                              int32_t *accept_len, int32_t *next_token, float *debug_out,
                              void *stream);

/* Token verification (Alg. 1); same arguments.  debug_out holds w_i = 1,
 * S_i = sum_x max(p_i - q_i, 0) and h_i = min(r_i, 1).                                   */
sv_status_t spec_verify_token(const void *target_logits, const void *draft_logits,
                              const int32_t *draft_tokens, const float *uniforms,
                              int32_t B, int32_t gamma, int32_t V, sv_dtype_t dtype,
                              float temperature, void *workspace, size_t workspace_bytes,
                              int32_t *accept_len, int32_t *next_token, float *debug_out,
                              void *stream);

/* Greedy block verification (Alg. 4); same arguments.  debug_out holds the unclipped
 * w_i, S_i and h_i clipped to [0, 1].  Its output keeps the target distribution only
 * when the caller also applies the paper's distribution modification (Alg. 5) to the
 * following gamma - tau - 1 positions; that step needs the models and is not part of
 * this library.                                                                          */
sv_status_t spec_verify_greedy(const void *target_logits, const void *draft_logits,
                               const int32_t *draft_tokens, const float *uniforms,
                               int32_t B, int32_t gamma, int32_t V, sv_dtype_t dtype,
                               float temperature, void *workspace, size_t workspace_bytes,
                               int32_t *accept_len, int32_t *next_token, float *debug_out,
                               void *stream);

/*
 * The same three algorithms with the input variants a serving stack hands over:
 *
 *  - draft_lens (device, [B] int32, or NULL): sequences carry drafts of different lengths.  Sequence
 *    b uses its first draft_lens[b] draft positions, 1 <= draft_lens[b] <= gamma: target rows
 *    0 .. draft_lens[b], draft rows and tokens 0 .. draft_lens[b] - 1, uniforms[b][0 ..
 *    draft_lens[b] - 1] for the accept tests and uniforms[b][draft_lens[b]] for the draw of Y -
 *    exactly the result of a call with gamma = draft_lens[b] on that sequence's leading rows.
 *    `gamma` remains the row count per sequence in every array; rows beyond a sequence's length
 *    are never read.  Values outside 1 .. gamma are the caller's error and are clamped into that
 *    range on the device.  accept_len[b] lies in 0 .. draft_lens[b].
 *  - target_row_stride, draft_row_stride (in elements, >= V, or 0 for dense rows): the distance
 *    from one row of V logits to the next, e.g. a vocabulary padded for the GEMM that produced
 *    the logits.  Row (b, i) of the target starts (b * (gamma + 1) + i) * target_row_stride
 *    elements after target_logits, row (b, i) of the draft (b * gamma + i) * draft_row_stride
 *    after draft_logits; what lies between rows is never read.  16-byte loads need both strides
 *    in bytes to be multiples of 16 besides the conditions on V and the base pointers.
 *
 * SV_ERR_INVALID_ARG also for an unknown algo, a negative stride or a stride below V.  Everything
 * else as for spec_verify_block.
 */
typedef enum { SV_ALGO_BLOCK = 0, SV_ALGO_TOKEN = 1, SV_ALGO_GREEDY = 2 } sv_algo_t;
sv_status_t spec_verify_ex(sv_algo_t algo, const void *target_logits, const void *draft_logits,
                           const int32_t *draft_tokens, const int32_t *draft_lens,
                           int64_t target_row_stride, int64_t draft_row_stride, const float *uniforms,
                           int32_t B, int32_t gamma, int32_t V, sv_dtype_t dtype,
                           float temperature, void *workspace, size_t workspace_bytes,
                           int32_t *accept_len, int32_t *next_token, float *debug_out, void *stream);

/*
 * spec_verify_ex for callers that cannot allocate device memory or keep a workspace of their own: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspace; the
 * verification's scratch memory is an array of SV_STATIC_SCRATCH_BYTES inside the library's code object instead.  Every
 * GPU that the library runs on holds one copy of it until the process ends.  The call allocates and frees nothing
 * (its first use on a device looks the array's address up).  SV_ERR_STATIC_SCRATCH_TOO_SMALL when
 * spec_verify_workspace_bytes(B, gamma, V) exceeds SV_STATIC_SCRATCH_BYTES (32 MiB: B = 256, gamma = 16, V = 152064 needs
 * 12 MiB and fits; B = 1024, gamma = 8, V = 256000 needs 40 MiB and does not).
 * All calls on one GPU share that one array, which keeps whatever the last call left: when the shape (B, gamma, V)
 * differs from the previous call's on that device, a small kernel that prepares the control words goes onto `stream`
 * in front of the verification (so the first call of a shape launches two kernels); calls that overlap on one GPU -
 * from two streams or two threads - race on the array and give undefined results.  A call whose kernel gave up a wait
 * (accept_len -1) leaves the array unusable until a call with another shape has run.
 */
#define SV_STATIC_SCRATCH_BYTES (32u << 20)
sv_status_t spec_verify_ex_noalloc(sv_algo_t algo, const void *target_logits, const void *draft_logits,
                                   const int32_t *draft_tokens, const int32_t *draft_lens,
                                   int64_t target_row_stride, int64_t draft_row_stride, const float *uniforms,
                                   int32_t B, int32_t gamma, int32_t V, sv_dtype_t dtype, float temperature,
                                   int32_t *accept_len, int32_t *next_token, float *debug_out, void *stream);

/*
 * The three algorithms with the distributions themselves as inputs, the form of the arrays in the
 * paper's App. A: target_probs [B, gamma+1, V] holds p_i(x) = M_b(x | c, X^i), draft_probs
 * [B, gamma, V] holds q_i(x) = M_s(x | c, X^i) (device, dtype, token index contiguous).  The rows are
 * used as given: there is no temperature and no normalisation; the draw of Y divides by the sum of
 * the weights it draws from, whatever that sum is.  Contract (unchecked): values finite and >= 0,
 * every q_{i-1}(X_i) > 0 (the drafter produced X_i), every row with some positive value.  A drafted
 * token with p_{i-1}(X_i) = 0 has ratio 0 and is never accepted.  draft_lens, the row strides and all
 * other arguments as for spec_verify_ex; the workspace is the same one (its initialised state is
 * neither needed nor disturbed).  Every element is read from device memory once, in three launches.
 */
sv_status_t spec_verify_probs(sv_algo_t algo, const void *target_probs, const void *draft_probs,
                              const int32_t *draft_tokens, const int32_t *draft_lens,
                              int64_t target_row_stride, int64_t draft_row_stride, const float *uniforms,
                              int32_t B, int32_t gamma, int32_t V, sv_dtype_t dtype,
                              void *workspace, size_t workspace_bytes,
                              int32_t *accept_len, int32_t *next_token, float *debug_out, void *stream);

const char *spec_verify_status_string(sv_status_t status);

#ifdef __cplusplus
}
#endif
#endif /* SPECVERIFY_H */
