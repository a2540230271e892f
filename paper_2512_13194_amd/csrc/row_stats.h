// Stage STATS of the EARS verification step: one streaming pass per logit row.
#pragma once

#include "decide.h"
#include "ears_device.h"

namespace ears {

// =================================================================================================
// One workgroup per draft position r: it streams the target row paired with r, then the draft
// row r, and so holds both rows' statistics when it is done.  Its first thread then evaluates the
// acceptance decision for the position on the spot (paper Section 3.2 steps 2-5), so that the
// sampling stage only has to scan K flags per sequence.  (A call that runs the statistics stage
// on its own takes the decision too and leaves it unused: one kernel serves every call.)
//
// Each lane keeps a running maximum m and S = sum exp2(l*c - fl(m*c)), c = log2(e)/T, over the
// elements it has seen.  A chunk of register-resident elements is first reduced to its maximum,
// so the running maximum changes (and S is rescaled) at most once per chunk and the inner loop
// is one FMA, one v_exp_f32 and one add per element.  The lanes are merged with the associative
// rule (m,S) + (m',S') = (M, S*2^(mc-Mc) + S'*2^(m'c-Mc)), M = max(m,m'): a DPP wave reduction of
// the maxima, a per-lane rescale, an fp64 DPP wave sum, and an LDS combine of the workgroup's waves.
// The rounding of fl(M*c) is removed exactly at the end in fp64, so Z = sum exp((l - M)/T) carries
// only the fp32 rounding of the individual terms.  max P = 1/Z needs no second pass
// (Section 3.3 item 1: the maximum is cached, the row is never re-scanned for it).
// =================================================================================================
//
// A second running sum W serves the alternative uncertainty measures (paper Section 5):
//   kMeasureEntropy   W = sum e*y over the same terms, e = exp2(y), y = l*c - fl(m*c) (clamped at
//                     -126 so that a masked entry contributes 0 * finite); it rescales as
//                     W <- f*(W + d*S) when the offset moves by d (f = 2^d); the Shannon entropy of
//                     the row is H = ln Z - ln 2 * W/S: one more FMA and one max per element;
//   kMeasureVariance  W = sum e*e, which rescales as W <- f*f*W; sum_v p_v^2 = W/S^2 and the total
//                     variance of the one-hot outcome is 1 - W/S^2: one more FMA per element.
enum { kMeasureNone = 0, kMeasureEntropy = 1, kMeasureVariance = 2 };

//
// A chunk is summed in fp32; the chunk sums are added to the lane's running sums in fp64 (one
// conversion and one full-rate fp64 add per chunk).  With an fp32 running sum, a lane whose S is
// dominated by one term (a sharply peaked row: S ~ 1, every chunk ~ 1e-8..1e-7) rounds each chunk
// to a multiple of ulp(S) and Z drifts by several 1e-7.
template <int N, int kMeasure>
__device__ __forceinline__ void accumulate(const float (&f)[N], float c, float& m_run, float& mc,
                                           double& S, double& W) {
  float cm = f[0];
#pragma unroll
  for (int j = 1; j < N; ++j) cm = fmaxf(cm, f[j]);
  if (cm > m_run) {
    const float mc_new = cm * c;
    if (m_run == -INFINITY) {
      S = 0.0;
      W = 0.0;
    } else {
      const float d = mc - mc_new;
      const double scale = (double)__builtin_amdgcn_exp2f(d);
      if (kMeasure == kMeasureEntropy) W = scale * ((double)d * S + W);
      if (kMeasure == kMeasureVariance) W = (scale * scale) * W;
      S *= scale;
    }
    m_run = cm;
    mc = mc_new;
  }
  float s[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  float w[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int j = 0; j < N; ++j) {
    float y = fmaf(f[j], c, -mc);
    if (kMeasure == kMeasureEntropy) y = fmaxf(y, -126.0f);
    const float e = __builtin_amdgcn_exp2f(y);
    s[j & 3] += e;
    if (kMeasure == kMeasureEntropy) w[j & 3] = fmaf(e, y, w[j & 3]);
    if (kMeasure == kMeasureVariance) w[j & 3] = fmaf(e, e, w[j & 3]);
  }
  S += (double)((s[0] + s[1]) + (s[2] + s[3]));
  if (kMeasure != kMeasureNone) W += (double)((w[0] + w[1]) + (w[2] + w[3]));
}

// 2^d for |d| below 1e-3 (here: the rounding error of a product fl(M*c), at most half an ulp of
// it), to a relative 1e-16: five terms of the series, where the library routine spends several
// hundred instructions in the one thread every other thread of the workgroup is waiting for.
__device__ __forceinline__ double exp2_tiny(double d) {
  const double x = d * 0.69314718055994530942;
  return 1.0 + x * (1.0 + x * (0.5 + x * (1.0 / 6.0 + x * (1.0 / 24.0))));
}

// Streams one row; on return thread 0 holds the row maximum M, Z = sum exp((l - M)/T) and in
// H_out the Shannon entropy (nats) or the total variance of softmax(l/T), whichever kMeasure names.
// `issued` is called once, after the first round of loads has been requested: the place for
// work whose own loads would otherwise hold up the row's.
struct NoHook { __device__ __forceinline__ void operator()() const {} };
template <typename DT, int kUnroll, int kMeasure, typename Hook = NoHook>
__device__ __forceinline__ void row_pass(const typename DT::storage* base, int V, float c,
                                         float* sh_m, double* sh_s, float& M_out, double& Z_out,
                                         double& H_out, Hook issued = Hook()) {
  const int tid = (int)threadIdx.x;
  float m_run = -INFINITY, mc = 0.0f;
  double S = 0.0, W = 0.0;

  // scalar head up to the first 16-byte boundary and scalar tail after the last whole vector
  // (both empty when rows are 16-byte multiples)
  constexpr int kPer = DT::kPerVec;
  const uintptr_t addr = reinterpret_cast<uintptr_t>(base);
  int head = (int)(((16u - (addr & 15u)) & 15u) / sizeof(typename DT::storage));
  if (head > V) head = V;
  const int nvec = (V - head) / kPer;
  const int tail0 = head + nvec * kPer;
  const int ntail = V - tail0;
  if (tid < head + ntail) {
    float f[1] = {DT::load(base, tid < head ? tid : tail0 + (tid - head))};
    accumulate<1, kMeasure>(f, c, m_run, mc, S, W);
  }

  const uint4* vp = reinterpret_cast<const uint4*>(base + head);
  for (int i0 = tid; i0 < nvec; i0 += kBlock * kUnroll) {
    uint4 raw[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int i = i0 + u * kBlock;
      raw[u] = i < nvec ? load_stream(vp + i) : DT::neg_inf_vec();
    }
    if (i0 == tid) issued();
    float f[kUnroll * kPer];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      float g[kPer];
      DT::unpack(raw[u], g);
#pragma unroll
      for (int j = 0; j < kPer; ++j) f[u * kPer + j] = g[j];
    }
    accumulate<kUnroll * kPer, kMeasure>(f, c, m_run, mc, S, W);
  }

  // merge the lanes of the workgroup
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  const float wm = wave_max(m_run);
  __syncthreads();  // the previous pass has finished with the shared arrays
  if (lane == 0) sh_m[wave] = wm;
  __syncthreads();
  float M = sh_m[0];
#pragma unroll
  for (int w = 1; w < kWavesPerBlock; ++w) M = fmaxf(M, sh_m[w]);
  const float Mc = M * c;
  const float scale = (m_run == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(mc - Mc);
  const double part = wave_sum(S * (double)scale);
  double wpart = 0.0;
  if (kMeasure == kMeasureEntropy)
    wpart = wave_sum((double)scale * (W + (double)(mc - Mc) * S));
  if (kMeasure == kMeasureVariance) wpart = wave_sum(((double)scale * (double)scale) * W);
  if (lane == 0) {
    sh_s[wave] = part;
    if (kMeasure != kMeasureNone) sh_s[kWavesPerBlock + wave] = wpart;
  }
  __syncthreads();
  if (tid == 0) {
    double Zp = 0.0, Wp = 0.0;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) Zp += sh_s[w];
    // the lanes used fl(M*c) as the offset; undo its rounding exactly
    const double delta = (double)Mc - (double)M * (double)c;
    Z_out = Zp * exp2_tiny(delta);
    M_out = M;
    if (kMeasure != kMeasureNone) {
#pragma unroll
      for (int w = 0; w < kWavesPerBlock; ++w) Wp += sh_s[kWavesPerBlock + w];
      // H = ln Z - ln 2 * sum p*y2, and sum p^2 = sum e^2 / (sum e)^2; the offset's rounding shifts
      // or scales both terms equally, so the sums taken with fl(M*c) serve as they are
      if (kMeasure == kMeasureEntropy) H_out = log(Zp) - 0.69314718055994530942 * (Wp / Zp);
      if (kMeasure == kMeasureVariance) H_out = (Zp * Zp - Wp) / (Zp * Zp);
    }
  }
}

// The work of one workgroup on draft position r (see the head of this file).  sh_m holds
// kWavesPerBlock floats and sh_s twice as many doubles.
// kHand: the position's statistics and decision are handed to workgroups of the SAME launch that
// wait for them (verify_kernel): they are written with coherent stores, and once those have been
// acknowledged, ready[r] takes the call's tag.
template <typename DT, int kUnroll, int kMeasure, bool kHand = false>
__device__ __forceinline__ void row_stats_body(const Problem& p, int64_t r, float* sh_m, double* sh_s) {
  using storage = typename DT::storage;
  const int b = seq_of_row(p, r);
  const int V = p.V;
  const float c = (float)(kLog2e / (double)seq_temperature(p, b));
  const storage* trow = static_cast<const storage*>(p.target) + (r + b) * (int64_t)V;
  const storage* drow = static_cast<const storage*>(p.draft) + r * (int64_t)V;

  // The draft token's two logits are fetched while the rows stream, and the position's acceptance
  // uniform is drawn while they do; but only once the first thread's own share of the first row
  // loads has been requested: fetching the token is a trip to memory, the logits' addresses depend
  // on it, and a wave that waits for it before its row loads is late for the whole workgroup.
  float lxt = -INFINITY, lxd = -INFINITY;
  int32_t x = -1;
  double U = 0.0;
  if (threadIdx.x == 0) {
    // the sampling stage counts from zero (a ragged batch may hold more sequences than positions)
    if (kHand) {
      // rectangular batches only: the sequence's first position zeroes its word, ahead of the tag
      // that the sequence's sampling workgroups wait for
      if (r == seq_row_begin(p, b)) coherent_store(p.arrive + b, 0u);
    } else {
      for (int64_t j = r; j < (int64_t)p.B; j += p.R) p.arrive[j] = 0u;
    }
    x = p.tokens[r];
  }
  bool fetched = false;
  auto fetch_token_logits = [&]() {
    fetched = true;
    if (threadIdx.x == 0) {
      if (x >= 0 && x < V) {
        lxt = DT::load(trow, x);
        lxd = DT::load(drow, x);
      }
      U = accept_uniform(p.seed, seq_rng_id(p, b), (uint32_t)(r - seq_row_begin(p, b)));
    }
  };

  float Mt = 0.0f, Md = 0.0f;
  double Zt = 0.0, Zd = 0.0, Ht = 0.0, Hd = 0.0;
  row_pass<DT, kUnroll, kMeasure>(trow, V, c, sh_m, sh_s, Mt, Zt, Ht, fetch_token_logits);
  row_pass<DT, kUnroll, kMeasureNone>(drow, V, c, sh_m, sh_s, Md, Zd, Hd);
  if (!fetched) fetch_token_logits();  // a row shorter than one vector has no first round of loads

  if (threadIdx.x == 0) {
    if (kHand) {
      coherent_store(p.Z + 2 * r, Zt);
      coherent_store(p.Z + 2 * r + 1, Zd);
      coherent_store(p.m + 2 * r, Mt);
      coherent_store(p.m + 2 * r + 1, Md);
    } else {
      p.Z[2 * r] = Zt;
      p.Z[2 * r + 1] = Zd;
      p.m[2 * r] = Mt;
      p.m[2 * r + 1] = Md;
    }
    p.lx[2 * r] = lxt;
    p.lx[2 * r + 1] = lxd;
    // uncertainty of the target distribution: 1 - max P_t = 1 - 1/Z_t, or H / log V, or the
    // total variance 1 - sum P_t^2
    double unc = 1.0 - 1.0 / Zt;
    if (kMeasure == kMeasureEntropy) unc = V > 1 ? fmin(fmax(Ht / log((double)V), 0.0), 1.0) : 0.0;
    if (kMeasure == kMeasureVariance) unc = fmin(fmax(Ht, 0.0), 1.0);
    if (kMeasure != kMeasureNone) p.unc[r] = unc;
    if (r == 0) *p.unc_tag = (uint32_t)kMeasure;
    // a NaN or +inf logit, or a row without any finite entry, leaves Z outside (0, inf)
    if (p.status_word && !(Zt > 0.0 && Zt < INFINITY && Zd > 0.0 && Zd < INFINITY))
      atomicOr(p.status_word, 4u);
    if (p.status_word && seq_params_invalid(p, b)) atomicOr(p.status_word, 8u);
    const int decision = decide_position(p, b, r, x, U, (double)Mt, Zt, (double)lxt, (double)Md,
                                         Zd, (double)lxd, unc);
    p.decisions[r] = decision;
    if (kHand) {
      wait_for_own_stores();
      coherent_store(p.ready + r, p.tag | (uint32_t)decision);
    }
  }
}

template <typename DT, int kUnroll, int kMeasure>
__global__ __launch_bounds__(kBlock) void row_stats_kernel(Problem p) {
  __shared__ float sh_m[kWavesPerBlock];
  __shared__ double sh_s[2 * kWavesPerBlock];
  row_stats_body<DT, kUnroll, kMeasure>(p, (int64_t)blockIdx.x, sh_m, sh_s);
}

// Statistics of the rows of ONE matrix (the target's or the draft's logits on their own): what a
// pipeline runs right after the model that produced them, ahead of the verification step.
struct RowStatsProblem {
  const void* logits;  // [rows, V]
  int64_t rows;
  int V;
  float T;
  const float* row_T;  // [rows] or nullptr
  float* row_m;        // [rows]
  double* row_Z;       // [rows]
  double* row_H;       // [rows] Shannon entropy in nats (only with kEntropy)
};

template <typename DT, int kUnroll, bool kEntropy>
__global__ __launch_bounds__(kBlock) void single_row_stats_kernel(RowStatsProblem p) {
  constexpr int kMeasure = kEntropy ? kMeasureEntropy : kMeasureNone;
  using storage = typename DT::storage;
  __shared__ float sh_m[kWavesPerBlock];
  __shared__ double sh_s[2 * kWavesPerBlock];
  const int64_t row = (int64_t)blockIdx.x;
  const float T = p.row_T ? p.row_T[row] : p.T;
  const float c = (float)(kLog2e / (double)T);
  float M = 0.0f;
  double Z = 0.0, H = 0.0;
  row_pass<DT, kUnroll, kMeasure>(static_cast<const storage*>(p.logits) + row * (int64_t)p.V, p.V,
                                  c, sh_m, sh_s, M, Z, H);
  if (threadIdx.x == 0) {
    p.row_m[row] = M;
    p.row_Z[row] = Z;
    if (kEntropy) p.row_H[row] = H;
  }
}

}  // namespace ears
