// EARS verification step for MI355X (gfx950): kernels and the C ABI declared in include/ears.h.
//
//   stage STATS  : row_stats_kernel   - one streaming pass per logit row (paper Section 3.2 step 1,
//                                       Section 3.3 item 1: max P_t cached, never re-scanned)
//   stage DECIDE : decide_kernel      - ratio, uniform, tolerance, threshold, three-way decision,
//                                       first-rejection scan (Section 3.2 steps 2-5, Section 3.1)
//   stage SAMPLE : sample_kernel      - residual / bonus token by Gumbel-max at slot n
//
// The path is bound by HBM bandwidth (every needed row is read once, plus one re-read of the row
// pair the sampler needs), so there is no matrix-core work here.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <mutex>

#include "../../include/ears.h"
#include "ears_device.h"

// Products such as fl(m*c) must stay rounded products (their rounding is undone explicitly
// later); fused operations are written as fmaf().
#pragma clang fp contract(off)

namespace ears {

constexpr double kLog2e = 1.4426950408889634074;
constexpr double kEpsilon = 1e-10;  // division guard of Section 3.3 item 2

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
  }
}

// =================================================================================================
// Stage DECIDE.  One thread per sequence, fp64: the B*K decision scalars are cheap, and the
// decision must not depend on fp32 rounding of R or the threshold.
// =================================================================================================
__global__ __launch_bounds__(kBlock) void decide_kernel(Problem p) {
  const int b = (int)(blockIdx.x * blockDim.x + threadIdx.x);
  if (b >= p.B) return;
  const int64_t r0 = seq_row_begin(p, b);
  const int Kb = seq_len(p, b);
  const double T = (double)seq_temperature(p, b);
  const double beta = (double)seq_beta(p, b);
  const uint64_t seq = seq_rng_id(p, b);
  int n = Kb;
  bool bad_token = false;
  for (int i = 0; i < Kb; ++i) {
    const int64_t r = r0 + i;
    const double mt = (double)p.m[2 * r], Zt = p.Z[2 * r], lxt = (double)p.lx[2 * r];
    const double md = (double)p.m[2 * r + 1], Zd = p.Z[2 * r + 1], lxd = (double)p.lx[2 * r + 1];
    const int32_t x = p.tokens[r];
    const bool valid = x >= 0 && x < p.V;
    const double Ptx = valid ? exp((lxt - mt) / T) / Zt : 0.0;
    const double Pdx = valid ? exp((lxd - md) / T) / Zd : 0.0;
    const double R = Ptx / fmax(Pdx, kEpsilon);            // Section 3.2 step 2, guard 3.3 item 2
    const double U = accept_uniform(p.seed, seq, (uint32_t)i);  // step 3
    const double unc = 1.0 - 1.0 / Zt;                     // 1 - max P_t, max P_t = 1/Z_t
    const double tol = beta * unc;                         // step 4
    const double thr = fmax(U - tol, 0.0);                 // threshold clamp, 3.3 item 2
    int decision;                                          // step 5
    if (!valid) { decision = 0; bad_token = true; }
    else if (R >= U) decision = 1;
    else if (R >= thr) decision = 2;
    else decision = 0;
    if (decision == 0 && n == Kb) n = i;                   // first rejection (Section 3.1)
    if (p.out_stats) {
      double* d = p.out_stats + r * EARS_NSTATS;
      d[0] = mt; d[1] = Zt; d[2] = Ptx; d[3] = md; d[4] = Zd; d[5] = Pdx;
      d[6] = unc; d[7] = R; d[8] = U; d[9] = thr;
    }
    if (p.out_path) p.out_path[r] = decision;
  }
  p.accept_len[b] = n;
  int32_t* out = p.out_tokens + r0 + b;
  for (int i = 0; i <= Kb; ++i) out[i] = i < n ? p.tokens[r0 + i] : -1;
  if (bad_token && p.status_word) atomicOr(p.status_word, 1u);
}

// =================================================================================================
// Stage SAMPLE.  One workgroup per sequence; scores in fp64 exactly as defined:
//   residual (n < K): log(max(0, p_t(v) - p_d(v))) + g(v) over rows n, with the cached (m, Z);
//   bonus    (n = K): l_t[K, v] / T + g(v);
//   empty residual  : log p_t(v) + g(v).
// g(v) = -log(-log u(v)), u from Philox keyed (seed, seq, n, v).
// =================================================================================================
__device__ __forceinline__ double gumbel64(uint64_t seed, uint64_t seq, uint32_t pos, uint32_t v) {
  const Philox blk = noise_block(seed, seq, pos, 1u, v >> 2);
  const uint32_t w = (v & 2u) ? ((v & 1u) ? blk.w[3] : blk.w[2]) : ((v & 1u) ? blk.w[1] : blk.w[0]);
  const double u = (double)(w >> 9) * 0x1p-23 + 0x1p-24;
  return -log(-log(u));
}

__device__ Best block_best(Best x) {
  __shared__ double sh_s[kWavesPerBlock];
  __shared__ int32_t sh_v[kWavesPerBlock];
  x = wave_best(x);
  const int lane = (int)threadIdx.x & (kWave - 1), wave = (int)threadIdx.x / kWave;
  __syncthreads();
  if (lane == 0) { sh_s[wave] = x.s; sh_v[wave] = x.v; }
  __syncthreads();
  Best r{sh_s[0], sh_v[0]};
#pragma unroll
  for (int w = 1; w < kWavesPerBlock; ++w)
    if (better(sh_s[w], sh_v[w], r)) r = Best{sh_s[w], sh_v[w]};
  return r;
}

template <typename DT>
__global__ __launch_bounds__(kBlock) void sample_kernel(Problem p) {
  const int b = (int)blockIdx.x;
  const int64_t r0 = seq_row_begin(p, b);
  const int Kb = seq_len(p, b);
  const int n = p.accept_len[b];
  const double T = (double)seq_temperature(p, b);
  const uint64_t seq = seq_rng_id(p, b);
  const int V = p.V;
  const typename DT::storage* trow =
      static_cast<const typename DT::storage*>(p.target) + (r0 + b + n) * (int64_t)V;
  Best best{-INFINITY, -1};
  if (n < Kb) {
    const int64_t r = r0 + n;
    const typename DT::storage* drow =
        static_cast<const typename DT::storage*>(p.draft) + r * (int64_t)V;
    const double mt = (double)p.m[2 * r], Zt = p.Z[2 * r];
    const double md = (double)p.m[2 * r + 1], Zd = p.Z[2 * r + 1];
    for (int v = (int)threadIdx.x; v < V; v += kBlock) {
      const double pt = exp(((double)DT::load(trow, v) - mt) / T) / Zt;
      const double pd = exp(((double)DT::load(drow, v) - md) / T) / Zd;
      const double q = pt - pd;
      if (q > 0.0) {
        const double s = log(q) + gumbel64(p.seed, seq, (uint32_t)n, (uint32_t)v);
        if (better(s, v, best)) best = Best{s, v};
      }
    }
    best = block_best(best);
    if (best.v < 0) {  // empty residual: draw from the target distribution of this position
      for (int v = (int)threadIdx.x; v < V; v += kBlock) {
        const double pt = exp(((double)DT::load(trow, v) - mt) / T) / Zt;
        if (pt > 0.0) {
          const double s = log(pt) + gumbel64(p.seed, seq, (uint32_t)n, (uint32_t)v);
          if (better(s, v, best)) best = Best{s, v};
        }
      }
      best = block_best(best);
    }
  } else {
    for (int v = (int)threadIdx.x; v < V; v += kBlock) {
      const double l = (double)DT::load(trow, v);
      if (l > -INFINITY) {
        const double s = l / T + gumbel64(p.seed, seq, (uint32_t)n, (uint32_t)v);
        if (better(s, v, best)) best = Best{s, v};
      }
    }
    best = block_best(best);
  }
  if (threadIdx.x == 0) p.out_tokens[r0 + b + n] = best.v;
}

// =================================================================================================
// Measurement aids.
// =================================================================================================
constexpr int kBenchBlocks = 4096;

__global__ __launch_bounds__(kBlock) void bench_read_kernel(const uint4* src, size_t nvec,
                                                            uint32_t* sink) {
  uint32_t acc = 0;
  const size_t stride = (size_t)gridDim.x * kBlock;
  size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x;
  for (; i + 3 * stride < nvec; i += 4 * stride) {
    const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < nvec; i += stride) {
    const uint4 a = src[i];
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) acc ^= __shfl_xor(acc, d, 64);
  __shared__ uint32_t sh[kWavesPerBlock];
  if ((threadIdx.x & (kWave - 1)) == 0) sh[threadIdx.x / kWave] = acc;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = sh[0] ^ sh[1] ^ sh[2] ^ sh[3];
}

__global__ __launch_bounds__(kBlock) void bench_copy_kernel(uint4* dst, const uint4* src,
                                                            size_t nvec) {
  const size_t stride = (size_t)gridDim.x * kBlock;
  for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < nvec; i += stride) dst[i] = src[i];
}

// =================================================================================================
// Host side.
// =================================================================================================
struct WorkspaceLayout {
  size_t off_Z, off_m, off_lx, total;
};

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static bool workspace_layout(int64_t R, int B, int V, WorkspaceLayout* w) {
  if (R < 1 || B < 1 || V < 1 || R < B || R > (int64_t)0x3FFFFFFF) return false;
  size_t o = 0;
  w->off_Z = o;  o = align_up(o + (size_t)(2 * R) * sizeof(double), 256);
  w->off_m = o;  o = align_up(o + (size_t)(2 * R) * sizeof(float), 256);
  w->off_lx = o; o = align_up(o + (size_t)(2 * R) * sizeof(float), 256);
  w->total = o;
  return true;
}

static bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

static int validate(int dtype, const void* target, const void* draft, const int32_t* tokens,
                    const int64_t* row_offsets, int64_t R, int B, int K, int V, float T, float beta,
                    const float* T_seq, const float* beta_seq, const int64_t* seq_ids,
                    const void* workspace, size_t workspace_bytes, int stages,
                    const int32_t* out_accept_len, const int32_t* out_tokens,
                    const double* out_stats, const int32_t* out_path, const uint32_t* status_word,
                    WorkspaceLayout* lay) {
  if (dtype != EARS_F32 && dtype != EARS_BF16) return EARS_ERR_DTYPE;
  if (!target || !draft || !tokens || !out_accept_len || !out_tokens) return EARS_ERR_NULL;
  if (B < 1 || V < 1 || R < 1) return EARS_ERR_SHAPE;
  if (row_offsets == nullptr) {
    if (K < 1 || (int64_t)B * (int64_t)K != R) return EARS_ERR_SHAPE;
  }
  if (!workspace_layout(R, B, V, lay)) return EARS_ERR_SHAPE;
  if (stages < 1 || stages > EARS_STAGE_ALL) return EARS_ERR_PARAM;
  if (!T_seq && !(std::isfinite(T) && T > 0.0f)) return EARS_ERR_PARAM;
  if (!beta_seq && !(std::isfinite(beta) && beta >= 0.0f)) return EARS_ERR_PARAM;
  if (!aligned(target, 16) || !aligned(draft, 16) || !aligned(tokens, 4) ||
      !aligned(out_accept_len, 4) || !aligned(out_tokens, 4) || !aligned(row_offsets, 8) ||
      !aligned(T_seq, 4) || !aligned(beta_seq, 4) || !aligned(seq_ids, 8) ||
      !aligned(out_stats, 8) || !aligned(out_path, 4) || !aligned(status_word, 4))
    return EARS_ERR_ALIGN;
  if (!workspace || workspace_bytes < lay->total) return EARS_ERR_WORKSPACE;
  if (!aligned(workspace, 256)) return EARS_ERR_ALIGN;
  return EARS_OK;
}

template <typename DT>
static int launch(const Problem& p, int stages, hipStream_t stream) {
  if (stages & EARS_STAGE_STATS) {
    hipLaunchKernelGGL((row_stats_kernel<DT, 4>), dim3((unsigned)(2 * p.R)), dim3(kBlock), 0, stream, p);
  }
  if (stages & EARS_STAGE_DECIDE) {
    hipLaunchKernelGGL(decide_kernel, dim3((unsigned)((p.B + kBlock - 1) / kBlock)), dim3(kBlock), 0,
                       stream, p);
  }
  if (stages & EARS_STAGE_SAMPLE) {
    hipLaunchKernelGGL((sample_kernel<DT>), dim3((unsigned)p.B), dim3(kBlock), 0, stream, p);
  }
  return hipGetLastError() == hipSuccess ? EARS_OK : EARS_ERR_HIP;
}

// library-owned scratch of the simple entry points, one buffer per device
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch[kMaxDevices] = {};
static size_t g_scratch_bytes[kMaxDevices] = {};

static int scratch_get(size_t bytes, void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return EARS_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_bytes[dev] < bytes) {
    if (g_scratch[dev]) {
      if (hipDeviceSynchronize() != hipSuccess) return EARS_ERR_HIP;
      (void)hipFree(g_scratch[dev]);
      g_scratch[dev] = nullptr;
      g_scratch_bytes[dev] = 0;
    }
    const size_t grow = align_up(bytes + bytes / 4, 1 << 20);
    if (hipMalloc(&g_scratch[dev], grow) != hipSuccess) return EARS_ERR_HIP;
    g_scratch_bytes[dev] = grow;
  }
  *out = g_scratch[dev];
  return EARS_OK;
}

}  // namespace ears

using namespace ears;

extern "C" {

const char* ears_status_string(int status) {
  switch (status) {
    case EARS_OK: return "ok";
    case EARS_ERR_NULL: return "a required pointer is NULL";
    case EARS_ERR_SHAPE: return "B, K, V or total_draft_rows out of range";
    case EARS_ERR_PARAM: return "temperature, beta or stages invalid";
    case EARS_ERR_ALIGN: return "a pointer is not aligned as documented";
    case EARS_ERR_DTYPE: return "unknown dtype";
    case EARS_ERR_WORKSPACE: return "workspace missing or too small";
    case EARS_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

size_t ears_workspace_bytes(int64_t total_draft_rows, int B, int V) {
  WorkspaceLayout lay;
  return workspace_layout(total_draft_rows, B, V, &lay) ? lay.total : 0;
}

int ears_verify_ex(int dtype, const void* target_logits, const void* draft_logits,
                   const int32_t* draft_tokens, const int64_t* row_offsets,
                   int64_t total_draft_rows, int B, int K, int V, float temperature, float beta,
                   const float* temperature_per_seq, const float* beta_per_seq, uint64_t seed,
                   const int64_t* seq_ids, void* workspace, size_t workspace_bytes, int stages,
                   int32_t* out_accept_len, int32_t* out_tokens, double* out_stats,
                   int32_t* out_path, uint32_t* status_word, void* stream) {
  WorkspaceLayout lay;
  const int rc = validate(dtype, target_logits, draft_logits, draft_tokens, row_offsets,
                          total_draft_rows, B, K, V, temperature, beta, temperature_per_seq,
                          beta_per_seq, seq_ids, workspace, workspace_bytes, stages, out_accept_len,
                          out_tokens, out_stats, out_path, status_word, &lay);
  if (rc != EARS_OK) return rc;
  Problem p;
  p.target = target_logits;
  p.draft = draft_logits;
  p.tokens = draft_tokens;
  p.row_offsets = row_offsets;
  p.R = total_draft_rows;
  p.B = B;
  p.K = row_offsets ? 0 : K;
  p.V = V;
  p.T = temperature;
  p.beta = beta;
  p.T_seq = temperature_per_seq;
  p.beta_seq = beta_per_seq;
  p.seed = seed;
  p.seq_ids = seq_ids;
  char* ws = static_cast<char*>(workspace);
  p.Z = reinterpret_cast<double*>(ws + lay.off_Z);
  p.m = reinterpret_cast<float*>(ws + lay.off_m);
  p.lx = reinterpret_cast<float*>(ws + lay.off_lx);
  p.accept_len = out_accept_len;
  p.out_tokens = out_tokens;
  p.out_stats = out_stats;
  p.out_path = out_path;
  p.status_word = status_word;
  hipStream_t s = static_cast<hipStream_t>(stream);
  return dtype == EARS_F32 ? launch<F32>(p, stages, s) : launch<BF16>(p, stages, s);
}

static int verify_simple(int dtype, const void* target, const void* draft, const int32_t* tokens,
                         const int64_t* row_offsets, int64_t R, int B, int K, int V, float T,
                         float beta, const float* T_seq, const float* beta_seq, uint64_t seed,
                         int32_t* out_accept_len, int32_t* out_tokens, void* stream) {
  // validate with a stand-in workspace first so that argument errors never touch the GPU
  WorkspaceLayout lay;
  alignas(256) static char dummy[256];
  int rc = validate(dtype, target, draft, tokens, row_offsets, R, B, K, V, T, beta, T_seq, beta_seq,
                    nullptr, dummy, (size_t)-1, EARS_STAGE_ALL, out_accept_len, out_tokens, nullptr,
                    nullptr, nullptr, &lay);
  if (rc != EARS_OK) return rc;
  void* ws = nullptr;
  rc = scratch_get(lay.total, &ws);
  if (rc != EARS_OK) return rc;
  return ears_verify_ex(dtype, target, draft, tokens, row_offsets, R, B, K, V, T, beta, T_seq,
                        beta_seq, seed, nullptr, ws, lay.total, EARS_STAGE_ALL, out_accept_len,
                        out_tokens, nullptr, nullptr, nullptr, stream);
}

int ears_verify_f32(const float* target_logits, const float* draft_logits,
                    const int32_t* draft_tokens, int B, int K, int V, float temperature,
                    float beta, uint64_t seed, int32_t* out_accept_len, int32_t* out_tokens,
                    void* stream) {
  return verify_simple(EARS_F32, target_logits, draft_logits, draft_tokens, nullptr,
                       (int64_t)B * (int64_t)K, B, K, V, temperature, beta, nullptr, nullptr, seed,
                       out_accept_len, out_tokens, stream);
}

int ears_verify_bf16(const void* target_logits, const void* draft_logits,
                     const int32_t* draft_tokens, int B, int K, int V, float temperature,
                     float beta, uint64_t seed, int32_t* out_accept_len, int32_t* out_tokens,
                     void* stream) {
  return verify_simple(EARS_BF16, target_logits, draft_logits, draft_tokens, nullptr,
                       (int64_t)B * (int64_t)K, B, K, V, temperature, beta, nullptr, nullptr, seed,
                       out_accept_len, out_tokens, stream);
}

int ears_verify_ragged_f32(const float* target_logits, const float* draft_logits,
                           const int32_t* draft_tokens, const int64_t* row_offsets,
                           int64_t total_draft_rows, int B, int V, const float* temperature,
                           const float* beta, uint64_t seed, int32_t* out_accept_len,
                           int32_t* out_tokens, void* stream) {
  if (!row_offsets || !temperature || !beta) return EARS_ERR_NULL;
  return verify_simple(EARS_F32, target_logits, draft_logits, draft_tokens, row_offsets,
                       total_draft_rows, B, 0, V, 1.0f, 0.0f, temperature, beta, seed,
                       out_accept_len, out_tokens, stream);
}

int ears_verify_ragged_bf16(const void* target_logits, const void* draft_logits,
                            const int32_t* draft_tokens, const int64_t* row_offsets,
                            int64_t total_draft_rows, int B, int V, const float* temperature,
                            const float* beta, uint64_t seed, int32_t* out_accept_len,
                            int32_t* out_tokens, void* stream) {
  if (!row_offsets || !temperature || !beta) return EARS_ERR_NULL;
  return verify_simple(EARS_BF16, target_logits, draft_logits, draft_tokens, row_offsets,
                       total_draft_rows, B, 0, V, 1.0f, 0.0f, temperature, beta, seed,
                       out_accept_len, out_tokens, stream);
}

void ears_release(void) {
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  int prev = 0;
  if (hipGetDevice(&prev) != hipSuccess) return;
  for (int d = 0; d < kMaxDevices; ++d) {
    if (!g_scratch[d]) continue;
    if (hipSetDevice(d) == hipSuccess) {
      (void)hipDeviceSynchronize();
      (void)hipFree(g_scratch[d]);
    }
    g_scratch[d] = nullptr;
    g_scratch_bytes[d] = 0;
  }
  (void)hipSetDevice(prev);
}

int ears_bench_read_sink_words(void) { return kBenchBlocks; }

int ears_bench_read(const void* src, size_t bytes, uint32_t* sink, void* stream) {
  if (!src || !sink) return EARS_ERR_NULL;
  if (bytes == 0 || bytes % 16 != 0) return EARS_ERR_SHAPE;
  if (!aligned(src, 16) || !aligned(sink, 4)) return EARS_ERR_ALIGN;
  hipLaunchKernelGGL(bench_read_kernel, dim3(kBenchBlocks), dim3(kBlock), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint4*>(src), bytes / 16,
                     sink);
  return hipGetLastError() == hipSuccess ? EARS_OK : EARS_ERR_HIP;
}

int ears_bench_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!src || !dst) return EARS_ERR_NULL;
  if (bytes == 0 || bytes % 16 != 0) return EARS_ERR_SHAPE;
  if (!aligned(src, 16) || !aligned(dst, 16)) return EARS_ERR_ALIGN;
  hipLaunchKernelGGL(bench_copy_kernel, dim3(kBenchBlocks), dim3(kBlock), 0,
                     static_cast<hipStream_t>(stream), static_cast<uint4*>(dst),
                     static_cast<const uint4*>(src), bytes / 16);
  return hipGetLastError() == hipSuccess ? EARS_OK : EARS_ERR_HIP;
}

}  // extern "C"
