/*
 * CPU oracle for the EARS verification step (Efficient Adaptive Rejection Sampling for
 * speculative decoding).  TEST INFRASTRUCTURE ONLY: it exists so that the GPU library can be
 * checked against a slow, plain, fp64 implementation of what the paper defines.  Nothing in the
 * product path may call it; it shares no source, header, table or helper with the GPU code.
 *
 * Every function is sequential fp64 arithmetic written in the order of the paper's Section 3.2
 * (its five steps), with the two guards of Section 3.3 item 2 and the
 * first-rejection rule of Section 3.1.  The replacement token at the rejected slot is drawn from
 * the residual distribution norm(max(0, p_t - p_d)) of the standard speculative sampling scheme
 * that the paper takes as its baseline (its references [1], [2]); the bonus token, when every
 * draft token is accepted, is drawn from the target row after the last draft position.
 *
 * Randomness: the paper only says that U_i is drawn uniformly from (0, 1).  Both the oracle and the GPU
 * library implement, independently, the published counter-based generator Philox4x32-10
 * (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC'11) with the
 * keying documented at ears_oracle_philox_word below.
 *
 * Parity pins (tests/, -m "not gpu"): Philox known-answer vectors; softmax statistics against
 * torch/scipy fp64 routines; beta = 0 against an independently written standard rejection
 * sampler; identical distributions accept everything; closed-form acceptance probability
 * min(1, R + Tol); closed-form output law on tiny vocabularies (chi-square); Gumbel-max against
 * the categorical law; hand-worked examples with exactly representable probabilities.
 */
#ifndef EARS_ORACLE_H
#define EARS_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* logit storage types: 0 = IEEE fp32, 1 = bfloat16 (the upper 16 bits of an fp32) */
#define EARS_ORACLE_F32 0
#define EARS_ORACLE_BF16 1

/* number of fp64 diagnostics stored per (sequence, position):
 *   0 m_t   max target logit                      5 P_d(x)  draft probability of the draft token
 *   1 Z_t   sum_v exp((l_t[v]-m_t)/T)             6 unc     1 - max_v P_t(v)   (Section 3.2)
 *   2 P_t(x) target probability of draft token    7 R       P_t(x) / max(P_d(x), 1e-10)
 *     (or H(P_t)/log V, or sum_v P_t(v)(1 - P_t(v)), when the entropy or the variance measure
 *     is selected)
 *   3 m_d   max draft logit                       8 U       acceptance uniform in [0,1)
 *   4 Z_d   draft sum-exp                         9 thr     max(U - beta*unc, 0)   (Section 3.3)
 */
#define EARS_ORACLE_NDIAG 10

/* number of fp64 diagnostics stored per sequence for the sampled token:
 *   0 best score, 1 second-best score (over distinct vocabulary indices; -inf if none),
 *   2 gap = best - second, 3 mode (0 residual, 1 bonus, 2 residual empty -> target-row fallback),
 *   4 vocabulary index of the second-best score (lowest index among equals; -1 if none)
 */
#define EARS_ORACLE_NSAMP 5

/* uncertainty measure that scales the tolerance: the paper's 1 - max P_t (Section 3.2), the
 * normalised Shannon entropy H(P_t) / log V (the entropy of the distribution, which Section 5 names), or the
 * total variance sum_v P_t(v) (1 - P_t(v)) of the one-hot outcome (the variance that Section 5 names,
 * which the paper does not define further) */
/* Support of the residual distribution norm(max(0, p_t - p_d)): an entry belongs to it when
 * p_t(v) - p_d(v) exceeds this fraction of p_t(v) + p_d(v).  2^-40 is far above the rounding noise
 * of an fp64 softmax (about 2^-50 relative) and far below anything a sampler can resolve (it
 * removes at most 2^-39 of probability mass); without it, entries where the two rows agree exactly
 * in real arithmetic enter or leave the support by the accident of a summation order. */
#define EARS_ORACLE_RESIDUAL_FLOOR 0x1p-40

#define EARS_ORACLE_UNC_MAXPROB 0
#define EARS_ORACLE_UNC_ENTROPY 1
#define EARS_ORACLE_UNC_VARIANCE 2

/* One Philox4x32-10 block: 10 rounds on a 128-bit counter with a 64-bit key. */
void ears_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* The 32-bit word the verification step uses for a given purpose.
 *   key     = (seed & 0xffffffff, seed >> 32)
 *   counter = (blk, pos, seq & 0xffffffff, (domain << 24) | ((seq >> 32) & 0xffffff))
 *   domain 0: acceptance uniform of (seq, pos): blk = 0, word 0
 *   domain 1: coarse Gumbel bits of (seq, pos, v): blk = v >> 4, word (v >> 2) & 3,
 *             byte v & 3 of that word (byte k = bits 8k .. 8k+7)
 *   domain 2: fine Gumbel bits of (seq, pos, v):   blk = v >> 2, word v & 3
 */
uint32_t ears_oracle_philox_word(uint64_t seed, uint64_t seq, uint32_t pos, uint32_t domain,
                                 uint32_t blk, uint32_t word);

/* U = (w >> 8) * 2^-24, in [0, 1), exactly representable in fp32. */
double ears_oracle_accept_uniform(uint64_t seed, uint64_t seq, uint32_t pos);
/* u = (h + (f + 1/2) * 2^-32) * 2^-8 in (0, 1): h the coarse byte, f the fine word; exact in fp64.
 * (The split lets a GPU discard almost every entry from the coarse byte alone.) */
double ears_oracle_gumbel_uniform(uint64_t seed, uint64_t seq, uint32_t pos, uint32_t v);
/* g = -log(-log(u)), standard Gumbel noise. */
double ears_oracle_gumbel(uint64_t seed, uint64_t seq, uint32_t pos, uint32_t v);

/* Three-pass softmax of one logit row at temperature T: p[v] = exp((l[v]-m)/T) / Z.
 * Writes p[0..V), the row maximum m and the sum Z.  Returns the largest probability. */
double ears_oracle_softmax(const void* row, int dtype, int V, double T, double* p, double* m,
                           double* Z);

/* Shannon entropy -sum p log p (nats) of a probability vector. */
double ears_oracle_entropy(const double* p, int V);
/* Total variance sum_v p_v (1 - p_v) of the one-hot outcome drawn from p. */
double ears_oracle_variance(const double* p, int V);

/* Arg-max with lowest-index ties and its runner-up over scores[0..n) (-inf = not a candidate):
 * returns the winner's index (-1 if there is no candidate) and fills samp[0] best score, [1]
 * second-best score, [2] their gap, [4] the runner-up's index; samp[3] is left alone. */
int32_t ears_oracle_top2(const double* scores, int n, double* samp);

/* Verify one sequence.
 *   target_rows [K+1, V], draft_rows [K, V] row-major logits of type dtype
 *   tokens [K] draft tokens (a token outside [0,V) is rejected at its position)
 *   out_tokens [K+1]: accepted prefix, the recovered / bonus token, then -1
 *   diag [K, EARS_ORACLE_NDIAG] (may be NULL), path [K] (may be NULL): per position, evaluated
 *   independently of the prefix: 0 reject, 1 accepted by R >= U, 2 accepted only by the tolerance
 *   samp [EARS_ORACLE_NSAMP] (may be NULL)
 * Returns 0, or 1 if some draft token was out of range. */
int ears_oracle_verify_seq(const void* target_rows, const void* draft_rows, const int32_t* tokens,
                           int dtype, int K, int V, double T, double beta, int unc_mode, uint64_t seed,
                           uint64_t seq_id, int32_t* accept_len, int32_t* out_tokens, double* diag,
                           int32_t* path, double* samp);

/* Rectangular batch: target [B, K+1, V], draft [B, K, V], tokens [B, K]; sequence b uses the RNG
 * id seq_ids[b] (b if seq_ids is NULL).  Sequences are independent; nthreads > 1 runs them on
 * that many OpenMP threads (the arithmetic per sequence is unchanged).
 * Returns the OR of the per-sequence return codes. */
int ears_oracle_verify(const void* target, const void* draft, const int32_t* tokens, int dtype,
                       int B, int K, int V, double T, double beta, int unc_mode, uint64_t seed,
                       const int64_t* seq_ids, int32_t* accept_len, int32_t* out_tokens,
                       double* diag, int32_t* path, double* samp, int nthreads);

/* Ragged batch.  row_offsets [B+1] indexes the packed DRAFT rows: sequence b owns draft rows
 * row_offsets[b] .. row_offsets[b+1), K_b of them; its K_b + 1 target rows start at packed target
 * row row_offsets[b] + b; tokens, diag and path are packed like draft rows, out_tokens like
 * target rows.  T[b] and beta[b] are per sequence. */
int ears_oracle_verify_ragged(const void* target, const void* draft, const int32_t* tokens,
                              const int64_t* row_offsets, int dtype, int B, int V, const float* T,
                              const float* beta, int unc_mode, uint64_t seed, const int64_t* seq_ids,
                              int32_t* accept_len, int32_t* out_tokens, double* diag,
                              int32_t* path, double* samp, int nthreads);

/* Temperature -> 0 (greedy) corner: accept while the draft token equals the arg-max of its
 * target row (lowest index among equal maxima); out_tokens gets the accepted prefix, the target
 * arg-max of row n, then -1.  Rectangular when row_offsets is NULL (target [B, K+1, V], tokens
 * [B, K]), otherwise packed like ears_oracle_verify_ragged.  target_argmax (optional) receives the
 * arg-max of every target row, packed like the target rows. */
void ears_oracle_verify_greedy(const void* target, const int32_t* tokens,
                               const int64_t* row_offsets, int dtype, int B, int K, int V,
                               int32_t* accept_len, int32_t* out_tokens, int32_t* target_argmax);

/* Vocabulary projection that produces the logits: hidden [N, D] and weight [V, D] are bf16 bit
 * patterns; exact[n, v] = sum_k hidden[n,k] * weight[v,k] in fp64 (optional), logits[n, v] its
 * nearest bf16 (optional). */
double ears_oracle_lm_head_dot(const uint16_t* hidden, const uint16_t* weight, int D, int64_t n,
                               int64_t v);
uint16_t ears_oracle_round_bf16(double x);
void ears_oracle_lm_head(const uint16_t* hidden, const uint16_t* weight, int N, int D, int V,
                         double* exact, uint16_t* logits, int nthreads);

#ifdef __cplusplus
}
#endif
#endif
