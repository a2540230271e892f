/*
 * CPU oracle for the EARS verification step.  TEST INFRASTRUCTURE ONLY (see ears_oracle.h).
 * Plain sequential fp64; no blocking, fusion or reordering beyond what the paper states.
 */
#include "ears_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------------------------
 * Philox4x32-10 (Salmon et al., SC'11, Section 3.3 and Table 2 of that paper): each round
 * multiplies counter words 0 and 2 by two fixed odd constants, keeps the low halves, and mixes
 * the high halves with the other two words and the round key; the key is bumped by two Weyl
 * constants between rounds.
 * ------------------------------------------------------------------------------------------ */
void ears_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t prod0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
    uint64_t prod1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
    uint32_t hi0 = (uint32_t)(prod0 >> 32), lo0 = (uint32_t)prod0;
    uint32_t hi1 = (uint32_t)(prod1 >> 32), lo1 = (uint32_t)prod1;
    uint32_t n0 = hi1 ^ c1 ^ k0;
    uint32_t n1 = lo1;
    uint32_t n2 = hi0 ^ c3 ^ k1;
    uint32_t n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

uint32_t ears_oracle_philox_word(uint64_t seed, uint64_t seq, uint32_t pos, uint32_t domain,
                                 uint32_t blk, uint32_t word) {
  uint32_t key[2] = {(uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32)};
  uint32_t ctr[4] = {blk, pos, (uint32_t)(seq & 0xffffffffu),
                     (domain << 24) | (uint32_t)((seq >> 32) & 0xffffffu)};
  uint32_t out[4];
  ears_oracle_philox4x32_10(ctr, key, out);
  return out[word & 3u];
}

/* Acceptance uniform of Section 3.2 step 3: the top 24 bits of one Philox word, in [0, 1). */
double ears_oracle_accept_uniform(uint64_t seed, uint64_t seq, uint32_t pos) {
  uint32_t w = ears_oracle_philox_word(seed, seq, pos, 0u, 0u, 0u);
  return (double)(w >> 8) * 0x1p-24;
}

/* Uniform of vocabulary entry v: 8 leading bits from one byte of a "coarse" block shared by 16
 * consecutive entries, 32 further bits from a "fine" word; a half-step offset keeps it off 0 and
 * 1.  u = (h + (f + 1/2) * 2^-32) * 2^-8, exact in a double. */
double ears_oracle_gumbel_uniform(uint64_t seed, uint64_t seq, uint32_t pos, uint32_t v) {
  uint32_t cw = ears_oracle_philox_word(seed, seq, pos, 1u, v >> 4, (v >> 2) & 3u);
  uint32_t h = (cw >> (8u * (v & 3u))) & 0xffu;
  uint32_t f = ears_oracle_philox_word(seed, seq, pos, 2u, v >> 2, v & 3u);
  return ((double)h + ((double)f + 0.5) * 0x1p-32) * 0x1p-8;
}

double ears_oracle_gumbel(uint64_t seed, uint64_t seq, uint32_t pos, uint32_t v) {
  double u = ears_oracle_gumbel_uniform(seed, seq, pos, v);
  return -log(-log(u));
}

/* ------------------------------------------------------------------------------------------ */

static double logit_at(const void* row, int dtype, int64_t v) {
  if (dtype == EARS_ORACLE_BF16) {
    uint32_t bits = (uint32_t)((const uint16_t*)row)[v] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
  }
  return (double)((const float*)row)[v];
}

static const void* row_ptr(const void* base, int dtype, int64_t row, int V) {
  size_t esz = (dtype == EARS_ORACLE_BF16) ? 2u : 4u;
  return (const char*)base + (size_t)row * (size_t)V * esz;
}

/* The whole distribution over the vocabulary that Section 3.1 works with, at sampling temperature T
 * (Section 4.1 uses T = 0.9): p = softmax(l / T), the textbook three passes. */
double ears_oracle_softmax(const void* row, int dtype, int V, double T, double* p, double* m_out,
                           double* Z_out) {
  double m = -INFINITY;
  for (int v = 0; v < V; ++v) {
    double l = logit_at(row, dtype, v);
    if (l > m) m = l;
  }
  double Z = 0.0;
  for (int v = 0; v < V; ++v) {
    p[v] = exp((logit_at(row, dtype, v) - m) / T);
    Z += p[v];
  }
  double pmax = 0.0;
  for (int v = 0; v < V; ++v) {
    p[v] /= Z;
    if (p[v] > pmax) pmax = p[v];
  }
  *m_out = m;
  *Z_out = Z;
  return pmax;
}

/* argmax over v of score(v), lowest index on ties; also the runner-up (the entry that would win
 * if the winner were taken away: its score and index, again lowest index on ties; index -1 and
 * score -inf while there is none).  Entries are pushed in increasing index order. */
typedef struct {
  double best, second;
  int32_t arg, arg2;
} top2_t;

static void top2_init(top2_t* t) {
  t->best = -INFINITY;
  t->second = -INFINITY;
  t->arg = -1;
  t->arg2 = -1;
}

static void top2_push(top2_t* t, double s, int32_t v) {
  if (t->arg < 0 || s > t->best) {
    t->second = (t->arg < 0) ? -INFINITY : t->best;
    t->arg2 = t->arg;
    t->best = s;
    t->arg = v;
  } else if (t->arg2 < 0 || s > t->second) {
    t->second = s;
    t->arg2 = v;
  }
}

static void top2_report(const top2_t* t, double* samp) {
  samp[0] = t->best;
  samp[1] = t->second;
  samp[2] = t->best - t->second;
  samp[4] = (double)t->arg2;
}

/* The arg-max bookkeeping on its own, over a given score vector (entries equal to -inf are not
 * candidates): returns the winner's index and fills samp[0], [1], [2], [4] as the verification
 * does.  Exposed so that the bookkeeping can be checked on vectors with exact ties, which the
 * noise of the verification itself never produces. */
int32_t ears_oracle_top2(const double* scores, int n, double* samp) {
  top2_t t;
  top2_init(&t);
  for (int v = 0; v < n; ++v)
    if (scores[v] > -INFINITY) top2_push(&t, scores[v], v);
  top2_report(&t, samp);
  return t.arg;
}

/* Shannon entropy of a probability vector in nats, -sum p log p over p > 0. */
double ears_oracle_entropy(const double* p, int V) {
  double H = 0.0;
  for (int v = 0; v < V; ++v)
    if (p[v] > 0.0) H -= p[v] * log(p[v]);
  return H;
}

/* Total variance of the one-hot outcome X ~ p: the trace of its covariance matrix, sum_v of the
 * Bernoulli variances p_v (1 - p_v) (= 1 - sum_v p_v^2, the Gini-Simpson index). */
double ears_oracle_variance(const double* p, int V) {
  double G = 0.0;
  for (int v = 0; v < V; ++v) G += p[v] * (1.0 - p[v]);
  return G;
}

int ears_oracle_verify_seq(const void* target_rows, const void* draft_rows, const int32_t* tokens,
                           int dtype, int K, int V, double T, double beta, int unc_mode, uint64_t seed,
                           uint64_t seq_id, int32_t* accept_len, int32_t* out_tokens, double* diag,
                           int32_t* path, double* samp) {
  int rc = 0;
  double* pt = (double*)malloc((size_t)V * sizeof(double));
  double* pd = (double*)malloc((size_t)V * sizeof(double));
  int n = K; /* number of accepted draft tokens: index of the first rejection (Section 3.1) */
  int first_reject_seen = 0;

  for (int i = 0; i < K; ++i) {
    /* step 1: P_t(x_i), P_d(x_i), max(P_t) */
    double mt, Zt, md, Zd;
    double maxpt = ears_oracle_softmax(row_ptr(target_rows, dtype, i, V), dtype, V, T, pt, &mt, &Zt);
    (void)ears_oracle_softmax(row_ptr(draft_rows, dtype, i, V), dtype, V, T, pd, &md, &Zd);
    int32_t x = tokens[i];
    int valid = (x >= 0 && x < V);
    double Ptx = valid ? pt[x] : 0.0;
    double Pdx = valid ? pd[x] : 0.0;
    /* step 2 with the division guard of Section 3.3 item 2 (epsilon = 1e-10) */
    double Pd_safe = (Pdx > 1e-10) ? Pdx : 1e-10;
    double R = Ptx / Pd_safe;
    /* step 3 */
    double U = ears_oracle_accept_uniform(seed, seq_id, (uint32_t)i);
    /* step 4: uncertainty 1 - max P_t and tolerance beta * uncertainty (Section 3.2); the
     * alternative measure (Section 5 names the entropy of the distribution) is the Shannon entropy of P_t
     * divided by its largest possible value log V; the other one it names, the variance, is taken
     * as the total variance of the one-hot outcome, sum_v P_t(v) (1 - P_t(v)) */
    double unc = 1.0 - maxpt;
    if (unc_mode == EARS_ORACLE_UNC_ENTROPY) unc = (V > 1) ? ears_oracle_entropy(pt, V) / log((double)V) : 0.0;
    if (unc_mode == EARS_ORACLE_UNC_VARIANCE) unc = ears_oracle_variance(pt, V);
    double tol = beta * unc;
    /* threshold clamp of Section 3.3 item 2 */
    double thr = U - tol;
    if (thr < 0.0) thr = 0.0;
    /* step 5: the three-way decision */
    int decision;
    if (!valid) {
      decision = 0;
      rc = 1;
    } else if (R >= U) {
      decision = 1; /* primary path, identical to the traditional rule */
    } else if (R >= thr) {
      decision = 2; /* accepted through the tolerance */
    } else {
      decision = 0;
    }
    if (decision == 0 && !first_reject_seen) {
      first_reject_seen = 1;
      n = i; /* x_i and every later draft token are rejected */
    }
    if (diag) {
      double* d = diag + (size_t)i * EARS_ORACLE_NDIAG;
      d[0] = mt; d[1] = Zt; d[2] = Ptx; d[3] = md; d[4] = Zd; d[5] = Pdx;
      d[6] = unc; d[7] = R; d[8] = U; d[9] = thr;
    }
    if (path) path[i] = decision;
  }

  top2_t top;
  top2_init(&top);
  double mode;
  if (n < K) {
    /* replacement token at the rejected slot: residual distribution norm(max(0, p_t - p_d)),
     * sampled by Gumbel-max: argmax_v log q(v) + g(v) */
    double mt, Zt, md, Zd;
    (void)ears_oracle_softmax(row_ptr(target_rows, dtype, n, V), dtype, V, T, pt, &mt, &Zt);
    (void)ears_oracle_softmax(row_ptr(draft_rows, dtype, n, V), dtype, V, T, pd, &md, &Zd);
    mode = 0.0;
    int any = 0;
    for (int v = 0; v < V; ++v) {
      /* p_t and p_d are fp64 softmax values, each good to a few units in the 16th digit; where
       * they agree to 2^-40 relative their difference is rounding noise, not residual mass, and
       * the entry is outside the residual's support */
      double q = pt[v] - pd[v];
      if (q <= EARS_ORACLE_RESIDUAL_FLOOR * (pt[v] + pd[v])) q = 0.0;
      if (q > 0.0) {
        any = 1;
        top2_push(&top, log(q) + ears_oracle_gumbel(seed, seq_id, (uint32_t)n, (uint32_t)v), v);
      }
    }
    if (!any) {
      /* empty residual (p_t <= p_d everywhere): fall back to the target distribution itself */
      mode = 2.0;
      for (int v = 0; v < V; ++v) {
        if (pt[v] > 0.0)
          top2_push(&top, log(pt[v]) + ears_oracle_gumbel(seed, seq_id, (uint32_t)n, (uint32_t)v),
                    v);
      }
    }
  } else {
    /* every draft token accepted: bonus token from the target row after the last draft
     * position; Gumbel-max on the unnormalised log-probabilities l / T */
    mode = 1.0;
    const void* row = row_ptr(target_rows, dtype, K, V);
    for (int v = 0; v < V; ++v) {
      double l = logit_at(row, dtype, v);
      if (l > -INFINITY)
        top2_push(&top, l / T + ears_oracle_gumbel(seed, seq_id, (uint32_t)K, (uint32_t)v), v);
    }
  }

  *accept_len = n;
  for (int i = 0; i <= K; ++i) out_tokens[i] = -1;
  for (int i = 0; i < n; ++i) out_tokens[i] = tokens[i];
  out_tokens[n] = top.arg;
  if (samp) {
    top2_report(&top, samp);
    samp[3] = mode;
  }
  free(pt);
  free(pd);
  return rc;
}

int ears_oracle_verify(const void* target, const void* draft, const int32_t* tokens, int dtype,
                       int B, int K, int V, double T, double beta, int unc_mode, uint64_t seed,
                       const int64_t* seq_ids, int32_t* accept_len, int32_t* out_tokens,
                       double* diag, int32_t* path, double* samp, int nthreads) {
  int rc = 0;
  if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(dynamic, 1) reduction(| : rc)
  for (int b = 0; b < B; ++b) {
    uint64_t seq = seq_ids ? (uint64_t)seq_ids[b] : (uint64_t)b;
    rc |= ears_oracle_verify_seq(
        row_ptr(target, dtype, (int64_t)b * (K + 1), V), row_ptr(draft, dtype, (int64_t)b * K, V),
        tokens + (size_t)b * K, dtype, K, V, T, beta, unc_mode, seed, seq, accept_len + b,
        out_tokens + (size_t)b * (K + 1), diag ? diag + (size_t)b * K * EARS_ORACLE_NDIAG : NULL,
        path ? path + (size_t)b * K : NULL, samp ? samp + (size_t)b * EARS_ORACLE_NSAMP : NULL);
  }
  return rc;
}

int ears_oracle_verify_ragged(const void* target, const void* draft, const int32_t* tokens,
                              const int64_t* row_offsets, int dtype, int B, int V, const float* T,
                              const float* beta, int unc_mode, uint64_t seed, const int64_t* seq_ids,
                              int32_t* accept_len, int32_t* out_tokens, double* diag,
                              int32_t* path, double* samp, int nthreads) {
  int rc = 0;
  if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(dynamic, 1) reduction(| : rc)
  for (int b = 0; b < B; ++b) {
    int64_t r0 = row_offsets[b];
    int Kb = (int)(row_offsets[b + 1] - r0);
    uint64_t seq = seq_ids ? (uint64_t)seq_ids[b] : (uint64_t)b;
    rc |= ears_oracle_verify_seq(
        row_ptr(target, dtype, r0 + b, V), row_ptr(draft, dtype, r0, V), tokens + r0, dtype, Kb, V,
        (double)T[b], (double)beta[b], unc_mode, seed, seq, accept_len + b, out_tokens + r0 + b,
        diag ? diag + (size_t)r0 * EARS_ORACLE_NDIAG : NULL, path ? path + r0 : NULL,
        samp ? samp + (size_t)b * EARS_ORACLE_NSAMP : NULL);
  }
  return rc;
}

/* ------------------------------------------------------------------------------------------ */
/* The deterministic corner, temperature -> 0 (the paper's introduction: the standard scheme at
 * temperature = 0).  softmax(l / T) tends to the indicator of the row's largest logit, so the
 * ratio of Section 3.2 step 2 tends to 1 when the draft token is the target row's arg-max and to
 * 0 otherwise, the uncertainty 1 - max P_t tends to 0 and with it the tolerance, and the residual
 * and the bonus distribution both tend to the indicator of the target arg-max.  Hence: accept
 * while the draft token equals arg-max of the target row; the token at the first mismatch (or
 * after K matches) is that row's arg-max.  Equal maxima: lowest index.  No random numbers. */
static int32_t argmax_row(const void* row, int dtype, int V) {
  int32_t best = 0;
  double bv = logit_at(row, dtype, 0);
  for (int v = 1; v < V; ++v) {
    double x = logit_at(row, dtype, v);
    if (x > bv) {
      bv = x;
      best = v;
    }
  }
  return best;
}

void ears_oracle_verify_greedy(const void* target, const int32_t* tokens,
                               const int64_t* row_offsets, int dtype, int B, int K, int V,
                               int32_t* accept_len, int32_t* out_tokens, int32_t* target_argmax) {
  for (int b = 0; b < B; ++b) {
    int64_t r0 = row_offsets ? row_offsets[b] : (int64_t)b * K;
    int Kb = row_offsets ? (int)(row_offsets[b + 1] - r0) : K;
    int n = Kb;
    for (int i = 0; i <= Kb; ++i) {
      int32_t a = argmax_row(row_ptr(target, dtype, r0 + b + i, V), dtype, V);
      if (target_argmax) target_argmax[r0 + b + i] = a;
      if (i < Kb && n == Kb && tokens[r0 + i] != a) n = i;
    }
    accept_len[b] = n;
    for (int i = 0; i <= Kb; ++i) {
      int32_t a = argmax_row(row_ptr(target, dtype, r0 + b + i, V), dtype, V);
      out_tokens[r0 + b + i] = i < n ? tokens[r0 + i] : (i == n ? a : -1);
    }
  }
}

/* ------------------------------------------------------------------------------------------ */
/* Producer side (Section 3.3 item 1: the statistics are taken "immediately after the target
 * model's forward pass"): the last step of that pass is the vocabulary projection
 * logits[n, v] = sum_k hidden[n, k] * weight[v, k], stored as bfloat16.  Plain fp64 dot products
 * of the bf16 inputs; round-to-nearest-even to bf16 is a separate, explicit step. */
static double bf16_value(uint16_t bits) {
  uint32_t w = (uint32_t)bits << 16;
  float f;
  memcpy(&f, &w, sizeof f);
  return (double)f;
}

double ears_oracle_lm_head_dot(const uint16_t* hidden, const uint16_t* weight, int D, int64_t n,
                               int64_t v) {
  double acc = 0.0;
  for (int k = 0; k < D; ++k)
    acc += bf16_value(hidden[(size_t)n * D + k]) * bf16_value(weight[(size_t)v * D + k]);
  return acc;
}

/* Nearest bfloat16 (ties to even) of a finite double that is not near the overflow threshold:
 * keep 8 significant bits.  Written with frexp/nearbyint, not with bit tricks, so that it can be
 * read against the definition of the format (1 sign, 8 exponent, 7 fraction bits). */
uint16_t ears_oracle_round_bf16(double x) {
  if (x == 0.0) return signbit(x) ? 0x8000u : 0u;
  int e;
  double m = frexp(fabs(x), &e);          /* |x| = m * 2^e, m in [0.5, 1) */
  if (e - 1 < -126) {                      /* below the normal range: fixed spacing 2^-133 */
    double q = nearbyint(ldexp(fabs(x), 133));
    return (uint16_t)((signbit(x) ? 0x8000u : 0u) | (uint16_t)q);
  }
  double q = nearbyint(ldexp(m, 8));      /* 8 significant bits: q in [128, 256] */
  if (q == 256.0) {
    q = 128.0;
    e += 1;
  }
  unsigned biased = (unsigned)(e - 1 + 127);
  return (uint16_t)((signbit(x) ? 0x8000u : 0u) | (biased << 7) | ((unsigned)q - 128u));
}

void ears_oracle_lm_head(const uint16_t* hidden, const uint16_t* weight, int N, int D, int V,
                         double* exact, uint16_t* logits, int nthreads) {
  if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int v = 0; v < V; ++v) {
      double x = ears_oracle_lm_head_dot(hidden, weight, D, n, v);
      if (exact) exact[(size_t)n * V + v] = x;
      if (logits) logits[(size_t)n * V + v] = ears_oracle_round_bf16(x);
    }
}
