// Stage STATS of the EARS verification step: one streaming pass per logit row.
#pragma once

#include "ears_device.h"

namespace ears {

// =================================================================================================
// Stage STATS.  One workgroup per logit row; workgroup 2r handles the target row paired with draft
// row r, workgroup 2r+1 the draft row itself.
//
// Each lane keeps a running maximum m and S = sum exp2(l*c - fl(m*c)), c = log2(e)/T, over the
// elements it has seen.  A chunk of register-resident elements is first reduced to its maximum,
// so the running maximum changes (and S is rescaled) at most once per chunk and the inner loop
// is one FMA, one v_exp_f32 and one add per element.  The lanes are merged with the associative
// rule (m,S) + (m',S') = (M, S*2^(mc-Mc) + S'*2^(m'c-Mc)), M = max(m,m'): a DPP wave reduction of
// the maxima, a per-lane rescale, an fp64 DPP wave sum, and an LDS combine of the four waves.
// The rounding of fl(M*c) is removed exactly at the end in fp64, so Z = sum exp((l - M)/T) carries
// only the fp32 rounding of the individual terms.  max P = 1/Z needs no second pass.
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

template <typename DT, int kUnroll>
__global__ __launch_bounds__(kBlock) void row_stats_kernel(Problem p) {
  const int64_t r = (int64_t)(blockIdx.x >> 1);
  const int which = (int)(blockIdx.x & 1u);
  const int b = seq_of_row(p, r);
  const int64_t row = which == 0 ? r + b : r;
  const typename DT::storage* base =
      static_cast<const typename DT::storage*>(which == 0 ? p.target : p.draft) + row * (int64_t)p.V;
  const int V = p.V;
  const int tid = (int)threadIdx.x;
  const float c = (float)(kLog2e / (double)seq_temperature(p, b));

  float m_run = -INFINITY, mc = 0.0f, S = 0.0f;

  // scalar head up to the first 16-byte boundary (empty when rows are 16-byte multiples)
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
      raw[u] = i < nvec ? vp[i] : DT::neg_inf_vec();
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

  // merge the 256 lanes
  __shared__ float sh_m[kWavesPerBlock];
  __shared__ double sh_s[kWavesPerBlock];
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  const float wm = wave_max(m_run);
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
    const double Z = Zp * exp2((double)Mc - (double)M * (double)c);
    const int32_t x = p.tokens[r];
    const int64_t slot = 2 * r + which;
    p.Z[slot] = Z;
    p.m[slot] = M;
    p.lx[slot] = (x >= 0 && x < V) ? DT::load(base, x) : -INFINITY;
    // the sampling stage counts its workgroups per sequence; start that count at zero here
    if (which == 1 && r == seq_row_begin(p, b)) p.arrivals[b] = 0u;
  }
}


}  // namespace ears
