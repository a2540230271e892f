/*
 * ears.h - C ABI of the EARS verification step for AMD MI355X (gfx950).
 *
 * EARS (Efficient Adaptive Rejection Sampling) verifies the K draft tokens of every sequence of a
 * speculative-decoding step against the target model's logits.  For sequence b and draft
 * position i (0-based), with p_t = softmax(target_logits[b,i,:] / T) and
 * p_d = softmax(draft_logits[b,i,:] / T), x = draft_tokens[b,i]:
 *
 *   uncertainty  unc = 1 - max_v p_t(v)                         (paper Section 3.2)
 *   tolerance    Tol = beta * unc                               (Section 3.2, the dynamic tolerance)
 *   ratio        R   = p_t(x) / max(p_d(x), 1e-10)              (Section 3.2 step 2; guard 3.3.2)
 *   threshold    thr = max(U - Tol, 0),  U ~ Uniform[0,1)       (Section 3.2 step 3; clamp 3.3.2)
 *   accept x  iff  R >= thr                                     (Section 3.2 step 5)
 *
 * The first rejected position n ends the accepted prefix (Section 3.1).  At slot n the library
 * emits a replacement token drawn from norm(max(0, p_t - p_d)) of position n (the residual
 * distribution of the standard speculative-sampling scheme the paper builds on, its references
 * [1] and [2]); when all K tokens are accepted (n = K) it emits a bonus token drawn from
 * softmax(target_logits[b,K,:] / T).  Both draws are Gumbel-max with counter-based
 * Philox4x32-10 noise keyed on (seed, sequence id, position, vocabulary index), so a call is a
 * pure function of its arguments.  max_v p_t(v) is obtained in the same single pass over the row
 * that yields p_t(x) (max p = 1/Z with Z the sum of exp((l - max l)/T)); the per-row statistics
 * are kept in the workspace and re-used by the sampling pass: computed once ahead of time and
 * looked up later, as Section 3.3 item 1 asks.
 *
 * Conventions
 *  - Every pointer is a DEVICE pointer on the current HIP device unless marked "host".
 *  - The caller owns every buffer.  Inputs are only read.  Outputs are fully overwritten.
 *  - Calls enqueue work on `stream` (a hipStream_t passed as void*; NULL = the null stream) and
 *    return without synchronising; outputs are valid once the caller has synchronised `stream`.
 *  - Return value: an ears_status.  All argument checks happen on the host before any HIP call.
 *  - Logits: finite values and -inf (a masked vocabulary entry, probability 0) are supported as
 *    long as every row has a finite entry.  A NaN or +inf logit, or a row without a finite entry,
 *    makes the results of its sequence undefined (every emitted token is still an index in
 *    [0, V) or -1, other sequences are not affected) and sets bit 2 of the status word.
 *  - A draft token outside [0, V) is rejected at its position and sets bit 0 of the optional
 *    device status word.
 *  - Two calls that share a workspace (or the library-owned scratch of the simple entry points)
 *    must not overlap in time.
 *  - EARS_ERR_HIP reports a failure of this call's own launches.  HIP keeps one "last error" per
 *    host thread: every call that launches work clears it first, so an error left pending by the
 *    caller's earlier HIP calls is neither reported here nor left for the caller to read.
 *  - Range of the arithmetic: the sampling stage bounds scores in fp32 with fixed margins that
 *    cover |logit| / T up to about 1e3 (e.g. |logit| <= 20 at T >= 0.02); beyond that a replacement
 *    or bonus token may differ from the fp64 definition's.  Accept lengths are not affected.
 */
#ifndef EARS_H
#define EARS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ears_status {
  EARS_OK = 0,
  EARS_ERR_NULL = 1,      /* a required pointer is NULL */
  EARS_ERR_SHAPE = 2,     /* B, K, V or total_draft_rows out of range (also: more than 2^30 draft
                             rows, or more sampling workgroups than a launch can hold) */
  EARS_ERR_PARAM = 3,     /* temperature not finite or <= 0; beta not finite or < 0; bad stages
                             or uncertainty measure */
  EARS_ERR_ALIGN = 4,     /* a pointer is not aligned as documented */
  EARS_ERR_DTYPE = 5,     /* dtype is neither EARS_F32 nor EARS_BF16 */
  EARS_ERR_WORKSPACE = 6, /* workspace NULL or smaller than ears_workspace_bytes() */
  EARS_ERR_HIP = 7        /* a HIP runtime call or kernel launch failed */
} ears_status;

typedef enum ears_dtype {
  EARS_F32 = 0, /* IEEE binary32 logits */
  EARS_BF16 = 1 /* bfloat16 logits (upper half of a binary32) */
} ears_dtype;

/* Stages of one verification call (Section 3.2 steps, Section 3.3 item 1).  A call may run a
 * subset: the statistics stage can run right after the target forward pass and the other two
 * later, against the statistics cached in the same workspace. */
enum {
  EARS_STAGE_STATS = 1,  /* step 1: per row max, sum-exp, logit of the draft token */
  EARS_STAGE_DECIDE = 2, /* steps 2-5 + first-rejection scan: accept lengths, accepted prefix */
  EARS_STAGE_SAMPLE = 4, /* replacement / bonus token at slot n */
  EARS_STAGE_ALL = 7
};

/* Uncertainty measure that scales the tolerance.  MAXPROB is the paper's 1 - max_v p_t(v)
 * (Section 3.2).  The other two are the finer measures that the paper's Section 5 leaves to
 * future work, without formulas: ENTROPY is the normalised Shannon entropy H(p_t) / log V, VARIANCE the
 * total variance sum_v p_t(v) (1 - p_t(v)) = 1 - sum_v p_t(v)^2 of the one-hot outcome drawn from
 * p_t (in [0, 1 - 1/V], never below the MAXPROB measure).  Each comes out of the same single pass
 * over the row. */
typedef enum ears_uncertainty {
  EARS_UNCERTAINTY_MAXPROB = 0,
  EARS_UNCERTAINTY_ENTROPY = 1,
  EARS_UNCERTAINTY_VARIANCE = 2
} ears_uncertainty;

/* Number of doubles per (sequence, position) in `out_stats`:
 *   0 m_t  1 Z_t  2 p_t(x)  3 m_d  4 Z_d  5 p_d(x)  6 unc  7 R  8 U  9 thr
 * (unc is the selected uncertainty measure)                                          */
#define EARS_NSTATS 10

/* Human-readable name of a status code (host pointer to a static string). */
const char* ears_status_string(int status);

/* ---------------------------------------------------------------------------------------------
 * Rectangular batch (the problem statement of Section 3.1: gamma = K draft tokens per sequence).
 *   target_logits  [B, K+1, V] row-major; row K of each sequence is only read for the bonus token
 *   draft_logits   [B, K,   V] row-major
 *   draft_tokens   [B, K] int32
 *   temperature    T > 0 (sampling temperature, Section 4.1); beta >= 0 (base tolerance)
 *   seed           RNG seed; vary it between decoding steps.  Sequence b uses RNG id b.
 *   out_accept_len [B] int32 in [0, K]
 *   out_tokens     [B, K+1] int32: the accepted prefix, then the replacement / bonus token,
 *                  then -1
 * Logit base pointers must be 16-byte aligned, int32 buffers 4-byte aligned.  Any V >= 1 works;
 * rows whose byte length is a multiple of 16 take the vectorised path.
 * These entry points keep their scratch in a library-owned, lazily grown per-device buffer
 * (ears_release() frees it); after the first call of a given size they allocate nothing.
 * ------------------------------------------------------------------------------------------- */
int ears_verify_f32(const float* target_logits, const float* draft_logits,
                    const int32_t* draft_tokens, int B, int K, int V, float temperature,
                    float beta, uint64_t seed, int32_t* out_accept_len, int32_t* out_tokens,
                    void* stream);

int ears_verify_bf16(const void* target_logits, const void* draft_logits,
                     const int32_t* draft_tokens, int B, int K, int V, float temperature,
                     float beta, uint64_t seed, int32_t* out_accept_len, int32_t* out_tokens,
                     void* stream);

/* ---------------------------------------------------------------------------------------------
 * Ragged batch: per-sequence draft length K_b >= 0, temperature and beta (the gathered
 * layout of the sequences still active, Section 3.3 item 3).  A sequence without draft tokens (K_b = 0)
 * has one target row and gets accept length 0 and a token drawn from that row; the batch as a
 * whole needs at least one draft row.
 *   row_offsets      [B+1] int64, device; CSR over the packed DRAFT rows: sequence b owns draft
 *                    rows row_offsets[b] .. row_offsets[b+1); row_offsets[0] = 0
 *   total_draft_rows host value of row_offsets[B] (the caller sized its buffers with it)
 *   target_logits    [total_draft_rows + B, V]: the K_b + 1 target rows of sequence b start at
 *                    packed row row_offsets[b] + b
 *   draft_logits     [total_draft_rows, V]; draft_tokens [total_draft_rows]
 *   temperature,beta [B] float32, device, per sequence (each T > 0, beta >= 0, finite).  They
 *                    cannot be checked on the host: a sequence whose T is not a positive finite
 *                    number is verified with T = 1, one whose beta is negative or not finite with
 *                    beta = 0, and bit 3 of the status word is raised
 *   out_accept_len   [B]; out_tokens [total_draft_rows + B], packed like the target rows
 * ------------------------------------------------------------------------------------------- */
int ears_verify_ragged_f32(const float* target_logits, const float* draft_logits,
                           const int32_t* draft_tokens, const int64_t* row_offsets,
                           int64_t total_draft_rows, int B, int V, const float* temperature,
                           const float* beta, uint64_t seed, int32_t* out_accept_len,
                           int32_t* out_tokens, void* stream);

int ears_verify_ragged_bf16(const void* target_logits, const void* draft_logits,
                            const int32_t* draft_tokens, const int64_t* row_offsets,
                            int64_t total_draft_rows, int B, int V, const float* temperature,
                            const float* beta, uint64_t seed, int32_t* out_accept_len,
                            int32_t* out_tokens, void* stream);

/* Bytes of caller-owned workspace ears_verify_ex needs for a problem with this many packed draft
 * rows (B*K for a rectangular batch), B sequences and vocabulary V.  Returns 0 on invalid sizes.
 * The workspace must be 256-byte aligned. */
size_t ears_workspace_bytes(int64_t total_draft_rows, int B, int V);

/* ---------------------------------------------------------------------------------------------
 * Full-control entry point; the four above are thin wrappers of it.
 *   dtype            ears_dtype of both logit buffers
 *   row_offsets      NULL for a rectangular batch (then K is used and total_draft_rows must be
 *                    B*K); otherwise the CSR offsets of a ragged batch (then K is ignored)
 *   temperature_per_seq, beta_per_seq   device [B] or NULL; when NULL the scalar is used
 *   uncertainty      an ears_uncertainty; the simple entry points use EARS_UNCERTAINTY_MAXPROB.
 *                    The statistics stage caches what the selected measure needs, so STATS and
 *                    DECIDE are called with the same value; a DECIDE stage that asks for a
 *                    measure the cached statistics do not carry decides with MAXPROB instead
 *                    and raises bit 1 of the status word
 *   seq_ids          device [B] int64 or NULL: RNG id of each sequence (low 56 bits used);
 *                    NULL means 0..B-1.  With explicit ids a sequence's result does not depend
 *                    on its slot in the batch.
 *   workspace        device, >= ears_workspace_bytes(total_draft_rows, B, V) bytes, 256-byte
 *                    aligned; holds the cached row statistics between stages.  Its contents need
 *                    no initialisation (the statistics stage and ears_import_stats prepare what
 *                    the later stages count on); calls that run on one workspace at the same
 *                    time race.  A call with all three stages is one or two kernel launches on
 *                    `stream` and nothing else: no allocation, no copy, no synchronisation.
 *                    (One launch for rectangular batches of long rows with at least 512 draft
 *                    positions: its sampling workgroups wait, for a
 *                    bounded time, for the statistics workgroups of their sequence, which the
 *                    same launch started before them; see bit 4 of the status word.)
 *   stages           OR of EARS_STAGE_*; DECIDE needs STATS to have run on the same inputs and
 *                    workspace, SAMPLE needs DECIDE (out_accept_len is read back by SAMPLE)
 *   out_stats        optional device [total_draft_rows, EARS_NSTATS] float64 (written by DECIDE)
 *   out_path         optional device [total_draft_rows] int32, per position independent of the
 *                    prefix: 0 reject, 1 accepted by R >= U, 2 accepted only through the
 *                    tolerance (the three branches of Section 3.2 step 5)
 *   status_word      optional device uint32; bits are OR-ed in, never cleared:
 *                    bit 0 = some draft token was outside [0, V)
 *                    bit 1 = a separate DECIDE stage asked for an uncertainty measure other
 *                            than the one cached by STATS or ears_import_stats
 *                    bit 2 = the STATS stage met a row whose sum of exponentials is not a
 *                            positive finite number (a NaN or +inf logit, or no finite entry at
 *                            all): the results of that sequence are undefined, the others' are
 *                            not affected
 *                    bit 3 = a per-sequence temperature was not a positive finite number (1 was
 *                            used) or a per-sequence beta was negative or not finite (0 was used)
 *                    bit 4 = a sampling workgroup of a single-launch call gave up waiting for
 *                            its sequence's statistics (more than a tenth of a second; not seen
 *                            in any run): that sequence's sampled token has not been written
 * ------------------------------------------------------------------------------------------- */
int ears_verify_ex(int dtype, const void* target_logits, const void* draft_logits,
                   const int32_t* draft_tokens, const int64_t* row_offsets,
                   int64_t total_draft_rows, int B, int K, int V, float temperature, float beta,
                   const float* temperature_per_seq, const float* beta_per_seq, int uncertainty,
                   uint64_t seed, const int64_t* seq_ids, void* workspace, size_t workspace_bytes, int stages,
                   int32_t* out_accept_len, int32_t* out_tokens, double* out_stats,
                   int32_t* out_path, uint32_t* status_word, void* stream);

/* ---------------------------------------------------------------------------------------------
 * ears_verify_ex for callers that must not allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments and results as ears_verify_ex, without
 * the workspace: the scratch is a fixed array of EARS_NOALLOC_SCRATCH_BYTES in device memory that
 * is part of the library's code object (every GPU the library runs on holds its own copy until the
 * process ends).  The call makes no hipMalloc / hipFree and calls no allocating routine.
 *   - Problems whose ears_workspace_bytes(total_draft_rows, B, V) exceeds
 *     EARS_NOALLOC_SCRATCH_BYTES are rejected with EARS_ERR_WORKSPACE (checked on the host, before
 *     any HIP call, like every other argument).  4 MiB covers e.g. B = 1024 ragged sequences with
 *     4608 draft rows, or B = 4096, K = 8.
 *   - The first call on a device looks up the array's address (hipGetSymbolAddress; no
 *     allocation); make that first call outside stream capture.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two threads) race, and a STATS stage's cached statistics last only until the next
 *     call of this entry point on that GPU.  Nothing in the array needs clearing between calls.
 * ------------------------------------------------------------------------------------------- */
#define EARS_NOALLOC_SCRATCH_BYTES (4u << 20)

int ears_verify_noalloc(int dtype, const void* target_logits, const void* draft_logits,
                        const int32_t* draft_tokens, const int64_t* row_offsets,
                        int64_t total_draft_rows, int B, int K, int V, float temperature, float beta,
                        const float* temperature_per_seq, const float* beta_per_seq, int uncertainty,
                        uint64_t seed, const int64_t* seq_ids, int stages, int32_t* out_accept_len,
                        int32_t* out_tokens, double* out_stats, int32_t* out_path,
                        uint32_t* status_word, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Temperature -> 0 (greedy decoding, the deterministic regime of the paper's Section 1).  In that
 * limit p_t and p_d are indicators of their rows' largest logits, R is 1 or 0, the uncertainty
 * and the tolerance vanish: a draft token is accepted iff it is the arg-max of its target row
 * (lowest index among equal maxima), and the token after the accepted prefix is the arg-max of
 * target row n.  No draft logits, no temperature, no random numbers; only target rows are read.
 *   row_offsets   NULL: rectangular, target [B, K+1, V], draft_tokens [B, K], out_tokens [B, K+1];
 *                 else packed as for ears_verify_ragged_* (K ignored)
 *   workspace     device, 256-byte aligned, >= ears_greedy_workspace_bytes() bytes, or NULL to use
 *                 the library-owned scratch of the simple entry points
 * Out-of-range draft tokens never match.  Errors as for ears_verify_ex.
 * ------------------------------------------------------------------------------------------- */
size_t ears_greedy_workspace_bytes(int64_t total_draft_rows, int B);

int ears_verify_greedy(int dtype, const void* target_logits, const int32_t* draft_tokens,
                       const int64_t* row_offsets, int64_t total_draft_rows, int B, int K, int V,
                       void* workspace, size_t workspace_bytes, int32_t* out_accept_len,
                       int32_t* out_tokens, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Producer-side fusion (Section 3.3 item 1 has max P_t computed right behind the target
 * model's forward pass and cached).  The last step of that pass, the vocabulary projection
 *   logits[n, v] = sum_k hidden[n, k] * weight[v, k]      (bf16 inputs, fp32 accumulation, MFMA)
 * is computed here with an epilogue that rounds each logit to bf16 (nearest even), writes it once,
 * and takes the statistics of the ROUNDED row at temperature T while it is still in registers:
 *   out_row_max[n]    = max_v logits[n, v]
 *   out_row_sumexp[n] = sum_v exp((logits[n, v] - max) / T)        (so max_v p(v) = 1 / sumexp)
 * exactly the per-row quantities the statistics stage of ears_verify_ex would otherwise obtain by
 * re-reading the logits.  ears_import_stats() hands them to a verification workspace.
 *   hidden  [N, D] bf16, weight [V, D] bf16 (both row-major, 16-byte aligned); D a multiple of 64
 *   temperature      scalar T > 0, used when row_temperature is NULL
 *   row_temperature  device [N] float or NULL
 *   out_logits       [N, V] bf16;  out_row_max [N] float;  out_row_sumexp [N] double
 *   out_row_entropy  [N] double or NULL: Shannon entropy (nats) of softmax(logits[n,:] / T), for
 *                    the entropy-based uncertainty measure
 *   workspace        device, 256-byte aligned, >= ears_lm_head_workspace_bytes(N, V) bytes
 * D must not exceed 2^20; the matrices themselves may be larger than 4 GiB.
 * ------------------------------------------------------------------------------------------- */
size_t ears_lm_head_workspace_bytes(int N, int V);

int ears_lm_head_bf16(const void* hidden, const void* weight, int N, int D, int V,
                      float temperature, const float* row_temperature, void* out_logits,
                      float* out_row_max, double* out_row_sumexp, double* out_row_entropy,
                      void* workspace, size_t workspace_bytes, void* stream);

/* The same per-row statistics for logits that already exist: one streaming pass over the rows of
 * ONE matrix, [rows, V] row-major (16-byte aligned base), at temperature T (scalar, or per row when
 * row_temperature is not NULL).  A pipeline can run it on the draft logits as soon as the draft
 * model has produced them, and on the target logits after the target pass (the computing ahead of time of
 * Section 3.3 item 1), and hand both to ears_import_stats().
 *   out_row_max [rows] float, out_row_sumexp [rows] double, out_row_entropy [rows] double or NULL
 *   (Shannon entropy in nats, for the entropy-based uncertainty measure) */
int ears_row_stats(int dtype, const void* logits, int64_t rows, int V, float temperature,
                   const float* row_temperature, float* out_row_max, double* out_row_sumexp,
                   double* out_row_entropy, void* stream);

/* Fills the statistics part of a verification workspace from per-row statistics computed by the
 * producers of the logits (ears_lm_head_bf16 for the target and for the draft model), and gathers
 * the draft tokens' logits.  Afterwards ears_verify_ex with stages DECIDE | SAMPLE (same batch,
 * same temperature(s)) completes the step without the statistics pass.
 *   target_row_max / target_row_sumexp   [total_draft_rows + B], packed like the target rows
 *   target_row_entropy                   same shape, or NULL; required before a DECIDE stage
 *                                        with EARS_UNCERTAINTY_ENTROPY (the VARIANCE measure is
 *                                        not carried by imported statistics: it needs the STATS
 *                                        stage of ears_verify_ex; see bit 1 of its status word)
 *   draft_row_max / draft_row_sumexp     [total_draft_rows]
 * Other arguments as for ears_verify_ex. */
int ears_import_stats(int dtype, const void* target_logits, const void* draft_logits,
                      const int32_t* draft_tokens, const int64_t* row_offsets,
                      int64_t total_draft_rows, int B, int K, int V, const float* target_row_max,
                      const double* target_row_sumexp, const double* target_row_entropy,
                      const float* draft_row_max, const double* draft_row_sumexp, void* workspace,
                      size_t workspace_bytes, void* stream);

/* Frees the library-owned scratch of the simple entry points on every device (synchronises). */
void ears_release(void);

/* ---------------------------------------------------------------------------------------------
 * Measurement aids (not part of the method): a read-only streaming kernel and a plain copy, used
 * to report the practical HBM ceiling next to the verification kernels and to calibrate the
 * profiler's byte counters against a transfer of known size.
 *   ears_bench_read: reads `bytes` (multiple of 16, src 16-byte aligned) and writes one 32-bit
 *                    checksum per workgroup to sink (device, >= 4 * ears_bench_read_sink_words()
 *                    bytes)
 *   ears_bench_copy: dst[0..bytes) = src[0..bytes), both 16-byte aligned, bytes multiple of 16
 * ------------------------------------------------------------------------------------------- */
int ears_bench_read_sink_words(void);
/* Test aid for the single-launch form of a whole call (see `workspace` of ears_verify_ex), process-
 * wide, not for production use: `force` != 0 makes every eligible call (rectangular, long rows,
 * all three stages) take the single launch whatever its number of draft positions;
 * `wait_polls` >= 0 replaces the number of polls after which a waiting sampling workgroup gives
 * up and raises bit 4 of the status word (0: after its first look), negative restores the
 * default.  ears_test_single_launch(0, -1) restores normal operation.  With it a test can see the
 * give-up path end normally, every kernel exiting, without anything having gone wrong. */
void ears_test_single_launch(int force, int wait_polls);
int ears_bench_read(const void* src, size_t bytes, uint32_t* sink, void* stream);
int ears_bench_copy(void* dst, const void* src, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* EARS_H */
