// Stage STATS of the EARS verification step: one streaming pass per logit row.
#pragma once

#include "decide.h"
#include "ears_device.h"

namespace ears {

// =================================================================================================
// One workgroup per draft position r: it streams the target row paired with r, then the draft
// row r, and so holds both rows' statistics when it is done.  With kDecide its first thread
// evaluates the acceptance decision for the position on the spot (paper Section 3.2 steps 2-5),
// so that the sampling stage only has to scan K flags per sequence.
//
// Each lane keeps a running maximum m and S = sum exp2(l*c - fl(m*c)), c = log2(e)/T, over the
// elements it has seen.  A chunk of register-resident elements is first reduced to its maximum,
// so the running maximum changes (and S is rescaled) at most once per chunk and the inner loop
// is one FMA, one v_exp_f32 and one add per element.  The lanes are merged with the associative
// rule (m,S) + (m',S') = (M, S*2^(mc-Mc) + S'*2^(m'c-Mc)), M = max(m,m'): a DPP wave reduction of
// the maxima, a per-lane rescale, an fp64 DPP wave sum, and an LDS combine of the four waves.
// The rounding of fl(M*c) is removed exactly at the end in fp64, so Z = sum exp((l - M)/T) carries
// only the fp32 rounding of the individual terms.  max P = 1/Z needs no second pass
// (Section 3.3 item 1: the maximum is cached, the row is never re-scanned for it).
// =================================================================================================
template <int N>
__device__ __forceinline__ void accumulate(const float (&f)[N], float c, float& m_run, float& mc,
                                           float& S) {
  float cm = f[0];
#pragma unroll
  for (int j = 1; j < N; ++j) cm = fmaxf(cm, f[j]);
  if (cm > m_run) {
    const float mc_new = cm * c;
    S = (m_run == -INFINITY) ? 0.0f : S * __builtin_amdgcn_exp2f(mc - mc_new);
    m_run = cm;
    mc = mc_new;
  }
  float s[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int j = 0; j < N; ++j) s[j & 3] += __builtin_amdgcn_exp2f(fmaf(f[j], c, -mc));
  S += (s[0] + s[1]) + (s[2] + s[3]);
}

// Streams one row; on return thread 0 holds the row maximum M and Z = sum exp((l - M)/T).
template <typename DT, int kUnroll>
__device__ __forceinline__ void row_pass(const typename DT::storage* base, int V, float c,
                                         float* sh_m, double* sh_s, float& M_out, double& Z_out) {
  const int tid = (int)threadIdx.x;
  float m_run = -INFINITY, mc = 0.0f, S = 0.0f;

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
    accumulate<1>(f, c, m_run, mc, S);
  }

  const uint4* vp = reinterpret_cast<const uint4*>(base + head);
  for (int i0 = tid; i0 < nvec; i0 += kBlock * kUnroll) {
    uint4 raw[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int i = i0 + u * kBlock;
      raw[u] = i < nvec ? load_stream(vp + i) : DT::neg_inf_vec();
    }
    float f[kUnroll * kPer];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      float g[kPer];
      DT::unpack(raw[u], g);
#pragma unroll
      for (int j = 0; j < kPer; ++j) f[u * kPer + j] = g[j];
    }
    accumulate<kUnroll * kPer>(f, c, m_run, mc, S);
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
  const double part = wave_sum((double)S * (double)scale);
  if (lane == 0) sh_s[wave] = part;
  __syncthreads();
  if (tid == 0) {
    double Zp = 0.0;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) Zp += sh_s[w];
    // the lanes used fl(M*c) as the offset; undo its rounding exactly
    Z_out = Zp * exp2((double)Mc - (double)M * (double)c);
    M_out = M;
  }
}

template <typename DT, int kUnroll, bool kDecide>
__global__ __launch_bounds__(kBlock) void row_stats_kernel(Problem p) {
  using storage = typename DT::storage;
  __shared__ float sh_m[kWavesPerBlock];
  __shared__ double sh_s[kWavesPerBlock];
  const int64_t r = (int64_t)blockIdx.x;
  const int b = seq_of_row(p, r);
  const int V = p.V;
  const float c = (float)(kLog2e / (double)seq_temperature(p, b));
  const storage* trow = static_cast<const storage*>(p.target) + (r + b) * (int64_t)V;
  const storage* drow = static_cast<const storage*>(p.draft) + r * (int64_t)V;

  // the draft token's two logits are fetched first so that they arrive while the rows stream
  float lxt = -INFINITY, lxd = -INFINITY;
  if (threadIdx.x == 0) {
    const int32_t x = p.tokens[r];
    if (x >= 0 && x < V) {
      lxt = DT::load(trow, x);
      lxd = DT::load(drow, x);
    }
  }

  float Mt = 0.0f, Md = 0.0f;
  double Zt = 0.0, Zd = 0.0;
  row_pass<DT, kUnroll>(trow, V, c, sh_m, sh_s, Mt, Zt);
  row_pass<DT, kUnroll>(drow, V, c, sh_m, sh_s, Md, Zd);

  if (threadIdx.x == 0) {
    p.Z[2 * r] = Zt;
    p.Z[2 * r + 1] = Zd;
    p.m[2 * r] = Mt;
    p.m[2 * r + 1] = Md;
    p.lx[2 * r] = lxt;
    p.lx[2 * r + 1] = lxd;
    if (kDecide) {
      const int i = (int)(r - seq_row_begin(p, b));
      p.decisions[r] = decide_position(p, b, i, r, (double)Mt, Zt, (double)lxt, (double)Md, Zd,
                                       (double)lxd);
    }
  }
}

}  // namespace ears
