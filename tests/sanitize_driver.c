/*
 * Stand-alone driver for the CPU oracle, built by tests/test_oracle_sanitize.py together with
 * oracle/ears_oracle.c under -fsanitize=address,undefined.  TEST INFRASTRUCTURE ONLY.
 *
 * Reads a file of cases written by the test, runs each through the oracle's C entry points and
 * writes every output to a second file, which the test compares byte for byte with what the
 * ordinary build of the oracle returns for the same cases.  A sanitizer report aborts the run.
 *
 * Case file: int32 ncases, then per case
 *   int32 kind (0 rectangular, 1 ragged, 2 greedy rectangular, 3 projection), dtype, B, K, V, unc,
 *         D (projection only, else 0), pad
 *   double T, beta; uint64 seed
 *   kind 0: target [B,K+1,V], draft [B,K,V], tokens int32 [B,K]
 *   kind 1: int64 row_offsets [B+1], float T [B], float beta [B], target [R+B,V], draft [R,V],
 *           tokens int32 [R]
 *   kind 2: target [B,K+1,V], tokens int32 [B,K]
 *   kind 3: hidden uint16 [B,D], weight uint16 [V,D]      (B plays N)
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "../oracle/ears_oracle.h"

static void* take(FILE* f, size_t bytes) {
  void* p = malloc(bytes ? bytes : 1);
  if (!p || fread(p, 1, bytes, f) != bytes) {
    fprintf(stderr, "short read\n");
    exit(3);
  }
  return p;
}

static void put(FILE* f, const void* p, size_t bytes) {
  if (fwrite(p, 1, bytes, f) != bytes) exit(4);
}

int main(int argc, char** argv) {
  if (argc != 3) return 2;
  FILE* in = fopen(argv[1], "rb");
  FILE* out = fopen(argv[2], "wb");
  if (!in || !out) return 2;
  int32_t ncases;
  if (fread(&ncases, 4, 1, in) != 1) return 3;
  for (int c = 0; c < ncases; ++c) {
    int32_t h[8];
    double par[2];
    uint64_t seed;
    if (fread(h, 4, 8, in) != 8 || fread(par, 8, 2, in) != 2 || fread(&seed, 8, 1, in) != 1) return 3;
    const int kind = h[0], dtype = h[1], B = h[2], K = h[3], V = h[4], unc = h[5], D = h[6];
    const size_t esz = dtype == EARS_ORACLE_BF16 ? 2 : 4;
    if (kind == 0 || kind == 1) {
      int64_t* off = NULL;
      float *Ts = NULL, *betas = NULL;
      int64_t R = (int64_t)B * K;
      if (kind == 1) {
        off = take(in, (size_t)(B + 1) * 8);
        Ts = take(in, (size_t)B * 4);
        betas = take(in, (size_t)B * 4);
        R = off[B];
      }
      void* target = take(in, (size_t)(R + B) * V * esz);
      void* draft = take(in, (size_t)R * V * esz);
      int32_t* tokens = take(in, (size_t)R * 4);
      int32_t* acc = malloc((size_t)B * 4);
      int32_t* tok = malloc((size_t)(R + B) * 4);
      double* diag = malloc((size_t)(R ? R : 1) * EARS_ORACLE_NDIAG * 8);
      int32_t* path = malloc((size_t)(R ? R : 1) * 4);
      double* samp = malloc((size_t)B * EARS_ORACLE_NSAMP * 8);
      int32_t rc;
      if (kind == 0)
        rc = ears_oracle_verify(target, draft, tokens, dtype, B, K, V, par[0], par[1], unc, seed, NULL,
                                acc, tok, diag, path, samp, 2);
      else
        rc = ears_oracle_verify_ragged(target, draft, tokens, off, dtype, B, V, Ts, betas, unc, seed,
                                       NULL, acc, tok, diag, path, samp, 2);
      put(out, &rc, 4);
      put(out, acc, (size_t)B * 4);
      put(out, tok, (size_t)(R + B) * 4);
      put(out, diag, (size_t)R * EARS_ORACLE_NDIAG * 8);
      put(out, path, (size_t)R * 4);
      put(out, samp, (size_t)B * EARS_ORACLE_NSAMP * 8);
      free(off); free(Ts); free(betas); free(target); free(draft); free(tokens);
      free(acc); free(tok); free(diag); free(path); free(samp);
    } else if (kind == 2) {
      void* target = take(in, (size_t)B * (K + 1) * V * esz);
      int32_t* tokens = take(in, (size_t)B * K * 4);
      int32_t* acc = malloc((size_t)B * 4);
      int32_t* tok = malloc((size_t)B * (K + 1) * 4);
      int32_t* amax = malloc((size_t)B * (K + 1) * 4);
      ears_oracle_verify_greedy(target, tokens, NULL, dtype, B, K, V, acc, tok, amax);
      put(out, acc, (size_t)B * 4);
      put(out, tok, (size_t)B * (K + 1) * 4);
      put(out, amax, (size_t)B * (K + 1) * 4);
      free(target); free(tokens); free(acc); free(tok); free(amax);
    } else if (kind == 3) {
      uint16_t* hidden = take(in, (size_t)B * D * 2);
      uint16_t* weight = take(in, (size_t)V * D * 2);
      double* exact = malloc((size_t)B * V * 8);
      uint16_t* logits = malloc((size_t)B * V * 2);
      ears_oracle_lm_head(hidden, weight, B, D, V, exact, logits, 2);
      put(out, exact, (size_t)B * V * 8);
      put(out, logits, (size_t)B * V * 2);
      free(hidden); free(weight); free(exact); free(logits);
    } else {
      return 5;
    }
  }
  /* the generator's published known-answer input and the arg-max bookkeeping on a tie */
  const uint32_t ctr[4] = {0x243f6a88u, 0x85a308d3u, 0x13198a2eu, 0x03707344u};
  const uint32_t key[2] = {0xa4093822u, 0x299f31d0u};
  uint32_t w[4];
  ears_oracle_philox4x32_10(ctr, key, w);
  put(out, w, 16);
  const double scores[4] = {1.0, 5.0, 5.0, -1.0 / 0.0};
  double samp[EARS_ORACLE_NSAMP] = {0, 0, 0, 0, 0};
  int32_t arg = ears_oracle_top2(scores, 4, samp);
  put(out, &arg, 4);
  put(out, samp, sizeof samp);
  fclose(in);
  if (fclose(out) != 0) return 4;
  return 0;
}
