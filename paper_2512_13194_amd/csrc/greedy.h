// Temperature -> 0 corner of the verification step (the deterministic regime the paper's
// introduction sets its method apart from): softmax(l/T) tends to the indicator of the row's largest
// logit, the ratio of Section 3.2 step 2 to 1 or 0, the uncertainty and the tolerance to 0.  A draft
// token is accepted iff it is the arg-max of its target row; the token after the accepted prefix is
// the arg-max of the next target row.  Only the target rows are read, once.
#pragma once

#include "ears_device.h"

namespace ears {

struct GreedyProblem {
  const void* target;          // [R + B, V]: the K_b + 1 rows of sequence b start at row off[b] + b
  const int32_t* tokens;       // [R]
  const int64_t* row_offsets;  // [B + 1] or nullptr (rectangular: K rows per sequence)
  int64_t R;
  int B, K, V;
  int32_t* argmax;             // [R + B] scratch: arg-max of every target row
  int32_t* accept_len;         // [B]
  int32_t* out_tokens;         // [R + B]
};

// (value, index) with the lowest index among equal values; an index of INT32_MAX means "no entry
// seen yet" and loses against everything.
struct ArgMax {
  float val;
  int32_t idx;
};
__device__ __forceinline__ ArgMax argmax_merge(ArgMax a, ArgMax b) {
  const bool take_b = b.val > a.val || (b.val == a.val && b.idx < a.idx);
  return take_b ? b : a;
}

// Arg-max of one row, streamed with the same 16-byte non-temporal loads as the statistics pass.
// A lane visits its entries in increasing index order (scalar head, vectors, scalar tail), so
// keeping the first strict improvement keeps the lowest index.  A chunk is first reduced to its
// maximum; the position is only looked for when that maximum beats the lane's best so far.
template <typename DT, int kUnroll>
__device__ __forceinline__ int32_t row_argmax(const typename DT::storage* base, int V, float* sh_val,
                                              int32_t* sh_idx) {
  const int tid = (int)threadIdx.x;
  ArgMax best = {-INFINITY, INT32_MAX};

  constexpr int kPer = DT::kPerVec;
  const uintptr_t addr = reinterpret_cast<uintptr_t>(base);
  int head = (int)(((16u - (addr & 15u)) & 15u) / sizeof(typename DT::storage));
  if (head > V) head = V;
  const int nvec = (V - head) / kPer;
  const int tail0 = head + nvec * kPer;
  const int ntail = V - tail0;

  if (tid < head) {
    const float x = DT::load(base, tid);
    if (x > best.val) best = {x, tid};
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
    float cm = f[0];
#pragma unroll
    for (int j = 1; j < kUnroll * kPer; ++j) cm = fmaxf(cm, f[j]);
    if (cm > best.val) {
      int pos = 0;  // first entry of the chunk, in index order, that holds the maximum
#pragma unroll
      for (int j = kUnroll * kPer - 1; j >= 0; --j) pos = (f[j] == cm) ? j : pos;
      const int u = pos / kPer, j = pos % kPer;
      best.val = cm;
      best.idx = head + (i0 + u * kBlock) * kPer + j;
    }
  }

  if (tid < ntail) {
    const float x = DT::load(base, tail0 + tid);
    if (x > best.val) best = {x, tail0 + tid};
  }

  // merge the lanes: wave butterfly, then the waves through shared memory
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    ArgMax o;
    o.val = __shfl_xor(best.val, d, 64);
    o.idx = __shfl_xor(best.idx, d, 64);
    best = argmax_merge(best, o);
  }
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  if (lane == 0) {
    sh_val[wave] = best.val;
    sh_idx[wave] = best.idx;
  }
  __syncthreads();
  ArgMax all = {sh_val[0], sh_idx[0]};
#pragma unroll
  for (int w = 1; w < kWavesPerBlock; ++w) all = argmax_merge(all, ArgMax{sh_val[w], sh_idx[w]});
  // a row without any entry above -inf: every entry is an equal maximum, the lowest index is 0
  return all.idx == INT32_MAX ? 0 : all.idx;
}

template <typename DT, int kUnroll>
__global__ __launch_bounds__(kBlock) void row_argmax_kernel(GreedyProblem p) {
  using storage = typename DT::storage;
  __shared__ float sh_val[kWavesPerBlock];
  __shared__ int32_t sh_idx[kWavesPerBlock];
  // one target row per workgroup (grid = R + B): two or more rows per group measured 1-13 % slower
  const int64_t row = (int64_t)blockIdx.x;
  const storage* base = static_cast<const storage*>(p.target) + row * (int64_t)p.V;
  const int32_t a = row_argmax<DT, kUnroll>(base, p.V, sh_val, sh_idx);
  if (threadIdx.x == 0) p.argmax[row] = a;
}

// One wave per sequence: first position whose draft token is not the target arg-max, then the
// outputs (accepted prefix, the arg-max of target row n, -1 after it).
__global__ __launch_bounds__(kBlock) void greedy_scan_kernel(GreedyProblem p) {
  const int lane = (int)threadIdx.x & (kWave - 1);
  const int b = (int)blockIdx.x * kWavesPerBlock + (int)threadIdx.x / kWave;
  if (b >= p.B) return;
  const int64_t r0 = p.row_offsets ? p.row_offsets[b] : (int64_t)b * p.K;
  const int Kb = p.row_offsets ? (int)(p.row_offsets[b + 1] - r0) : p.K;
  const int64_t t0 = r0 + b;
  int n = Kb;
  for (int base = 0; base < Kb && n == Kb; base += kWave) {
    const int i = base + lane;
    const bool mismatch = i < Kb && p.tokens[r0 + i] != p.argmax[t0 + i];
    const unsigned long long mask = __ballot(mismatch);
    if (mask != 0ull) n = base + __builtin_ctzll(mask);
  }
  if (lane == 0) p.accept_len[b] = n;
  for (int i = lane; i <= Kb; i += kWave)
    p.out_tokens[t0 + i] = i < n ? p.tokens[r0 + i] : (i == n ? p.argmax[t0 + i] : -1);
}

}  // namespace ears
