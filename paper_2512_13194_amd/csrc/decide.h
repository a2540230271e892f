// Stage DECIDE of the EARS verification step: ratio, uniform, tolerance, threshold, the three-way
// decision of the paper's Section 3.2 (steps 2-5) with the guards of Section 3.3 item 2, and the
// first-rejection scan of Section 3.1.
#pragma once

#include "ears_device.h"

namespace ears {

// Decision for draft position i of sequence b (packed row r) from the row statistics: row maximum
// m, Z = sum exp((l-m)/T) and the draft token's logit lx, for the target (t) and draft (d) rows,
// and the target row's uncertainty unc (1 - 1/Z_t = 1 - max P_t, or the entropy measure).
// Evaluated in fp64 whenever fp32 could not tell, so the outcome does not depend on fp32 rounding
// of R or the threshold.  Returns 0 reject, 1 accepted by R >= U, 2 accepted only through the
// tolerance (1 for either kind of acceptance when neither statistics nor branch ids are asked
// for).  Writes the optional per-position statistics / branch id and raises the status bit for
// an invalid token.  x is the draft token and U the acceptance uniform of the position (step 3):
// the caller fetches and draws them ahead of time, so that nothing slow is left for the moment the
// statistics arrive.
__device__ __forceinline__ int decide_position(const Problem& p, int b, int64_t r, int32_t x,
                                               double U, double mt, double Zt, double lxt,
                                               double md, double Zd, double lxd, double unc) {
  const double T = (double)seq_temperature(p, b);
  const double beta = (double)seq_beta(p, b);
  const bool valid = x >= 0 && x < p.V;
  if (valid && !p.out_stats && !p.out_path) {
    // Most decisions are far from the threshold: settle those in fp32 with a margin that covers
    // its rounding many times over (1e-4 relative on R, 1e-6 (1 + beta) absolute on the
    // threshold) and leave only the close calls and the guarded division to fp64.
    const float cf = (float)(kLog2e / T);
    const float Ptf = __builtin_amdgcn_exp2f(((float)lxt - (float)mt) * cf) / (float)Zt;
    const float Pdf = __builtin_amdgcn_exp2f(((float)lxd - (float)md) * cf) / (float)Zd;
    if (Pdf > 1e-9f) {
      const float Rf = Ptf / Pdf;
      const float Uf = (float)U;  // 24 bits: exact
      const float thrf = fmaxf(Uf - (float)beta * (float)unc, 0.0f);
      const float slack = 1e-6f * (1.0f + (float)beta);
      if (Rf * (1.0f - 1e-4f) > thrf + slack) return 1;
      if (Rf * (1.0f + 1e-4f) < thrf - slack) return 0;
    }
  }
  const double Ptx = valid ? exp((lxt - mt) / T) / Zt : 0.0;
  const double Pdx = valid ? exp((lxd - md) / T) / Zd : 0.0;
  const double R = Ptx / fmax(Pdx, kEpsilon);                              // step 2, division guard
  const double tol = beta * unc;                          // step 4
  const double thr = fmax(U - tol, 0.0);                  // threshold clamp
  int decision;                                           // step 5
  if (!valid) decision = 0;
  else if (R >= U) decision = 1;
  else if (R >= thr) decision = 2;
  else decision = 0;
  if (p.out_stats) {
    double* d = p.out_stats + r * EARS_NSTATS;
    d[0] = mt; d[1] = Zt; d[2] = Ptx; d[3] = md; d[4] = Zd; d[5] = Pdx;
    d[6] = unc; d[7] = R; d[8] = U; d[9] = thr;
  }
  if (p.out_path) p.out_path[r] = decision;
  if (!valid && p.status_word) atomicOr(p.status_word, 1u);
  return decision;
}

// One wave finds the accept length of one sequence: lane i takes draft position i (positions
// beyond 64 in further rounds) and a ballot of the rejecting lanes gives the first rejection.
// The per-position decisions are read from p.decisions when from_memory is set (the statistics
// kernel left them there), otherwise computed here from the cached row statistics and stored.
// With write_outputs the wave also stores the accept length, the accepted prefix and the -1 tail
// of out_tokens; slot n is left for the sampling stage.  Returns n in every lane.
__device__ __forceinline__ int first_reject_scan(const Problem& p, int b, int lane, bool from_memory,
                                                 bool write_outputs) {
  const int64_t r0 = seq_row_begin(p, b);
  const int Kb = seq_len(p, b);
  int n = Kb;
  for (int base = 0; base < Kb; base += kWave) {
    if (n < Kb && from_memory) break;  // later positions cannot change n
    const int i = base + lane;
    int decision = 1;
    if (i < Kb) {
      const int64_t r = r0 + i;
      if (from_memory) {
        decision = p.decisions[r];
      } else {
        const double Zt = p.Z[2 * r];
        // The cached statistics carry one alternative measure at most; asked for another, the
        // decision falls back to 1 - max P_t = 1 - 1/Z_t and says so in the status word.
        const bool cached = p.unc_mode != 0 && *p.unc_tag == (uint32_t)p.unc_mode;
        if (p.unc_mode != 0 && !cached && i == 0 && p.status_word) atomicOr(p.status_word, 2u);
        if (i == 0 && p.status_word && seq_params_invalid(p, b)) atomicOr(p.status_word, 8u);
        const double unc = cached ? p.unc[r] : 1.0 - 1.0 / Zt;
        const double U = accept_uniform(p.seed, seq_rng_id(p, b), (uint32_t)i);
        decision = decide_position(p, b, r, p.tokens[r], U, (double)p.m[2 * r], Zt,
                                   (double)p.lx[2 * r], (double)p.m[2 * r + 1], p.Z[2 * r + 1],
                                   (double)p.lx[2 * r + 1], unc);
        p.decisions[r] = decision;
      }
    }
    const unsigned long long rejecting = __ballot(decision == 0);
    if (rejecting != 0ull && n == Kb) n = base + (__ffsll((long long)rejecting) - 1);
  }
  if (write_outputs) {
    if (lane == 0) p.accept_len[b] = n;
    int32_t* out = p.out_tokens + r0 + b;
    for (int i = lane; i <= Kb; i += kWave)
      if (i != n) out[i] = i < n ? p.tokens[r0 + i] : -1;
  }
  return n;
}

// The same scan for a workgroup that runs in the SAME launch as the statistics workgroups of its
// sequence (verify_kernel): one wave polls the positions' ready words until every one carries this
// call's tag; the decision comes in the word's two lowest bits.  Coherent loads: the writers may
// sit on another XCD.  The statistics workgroups wait for nobody and are dispatched ahead of
// any workgroup that waits here (lower workgroup ids), so the wait ends; it is bounded all the
// same, and a wave that gives up returns -1.
constexpr int kAwaitPolls = 1 << 17;  // the default of Problem::await_polls; each poll is a trip to
                                      // memory and a short sleep: > 0.1 s
__device__ __forceinline__ int await_first_reject(const Problem& p, int b, int lane,
                                                  bool write_outputs) {
  const int64_t r0 = seq_row_begin(p, b);
  const int Kb = seq_len(p, b);
  int n = Kb;
  for (int base = 0; base < Kb; base += kWave) {
    const int i = base + lane;
    uint32_t word = p.tag | 1u;
    for (int polls = 0;; ++polls) {
      if (i < Kb) word = coherent_load(p.ready + r0 + i);
      if (__ballot((word & ~3u) != p.tag) == 0ull) break;
      if (polls >= p.await_polls) return -1;  // uniform over the wave
      __builtin_amdgcn_s_sleep(16);
    }
    const unsigned long long rejecting = __ballot((word & 3u) == 0u);
    if (rejecting != 0ull && n == Kb) n = base + (__ffsll((long long)rejecting) - 1);
  }
  // what the statistics workgroups stored before their ready words is read after them
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  if (write_outputs) {
    if (lane == 0) p.accept_len[b] = n;
    int32_t* out = p.out_tokens + r0 + b;
    for (int i = lane; i <= Kb; i += kWave)
      if (i != n) out[i] = i < n ? p.tokens[r0 + i] : -1;
  }
  return n;
}

// Stand-alone decision stage: kWavesPerBlock sequences per workgroup, one per wave.  Slot n of out_tokens
// is set to -1 here; the sampling stage overwrites it.
__global__ __launch_bounds__(kBlock) void decide_kernel(Problem p) {
  const int lane = (int)threadIdx.x & (kWave - 1);
  const int b = (int)blockIdx.x * kWavesPerBlock + (int)threadIdx.x / kWave;
  if (b >= p.B) return;
  const int n = first_reject_scan(p, b, lane, false, true);
  if (lane == 0) p.out_tokens[seq_row_begin(p, b) + b + n] = -1;
}

}  // namespace ears
