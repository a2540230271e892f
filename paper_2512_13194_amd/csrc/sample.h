// Stage SAMPLE of the EARS verification step: the replacement token at the first rejected slot,
// drawn from norm(max(0, p_t - p_d)), or the bonus token from the target row after the last draft
// position when every draft token is accepted.  Both are Gumbel-max draws:
//
//     token = argmax_v  score(v),   score(v) = log w(v) + g(v),   g(v) = -log(-log u(v)),
//     w(v) = max(0, p_t(v) - p_d(v))  (residual)   or   exp(l_t(v)/T)  (bonus),
//
// with u(v) from Philox keyed (seed, sequence, position, v); ties go to the lowest index.
//
// The winner is the one the fp64 definition gives; fp32 work only discards elements that provably
// cannot win.  Three levels, each sound with respect to the next:
//
//  1. TEST, every element, no transcendental, target row only, one Philox block per 16 elements.
//     u(v) = (h + (f + 1/2) 2^-32) / 256 with h a byte of the "coarse" block; u < (h+1)/256, so
//     with N = 255 - h, w(v) <= p_t(v) and -log u >= 1 - u > N/256, in base-2 logs
//         score2(v) <= a(v) + 8 - log2 N,   a(v) = (l_t(v) - m_t) * log2(e)/T - log2 Z_t
//     (bonus: a(v) = l_t(v) * log2(e)/T), and log2 N >= bits(float(N)) * 2^-23 - 127.  An element
//     whose bound is below the running threshold theta (a lower bound of the best score seen so
//     far) is dropped; the rest (all those with N = 0, one in 256, and a few more) are queued.
//  2. BOUNDS, queued elements, fp32 with explicit margins: s_lo <= score2 <= s_up.  theta rises
//     to the largest s_lo; an element survives while s_up >= theta.
//  3. EXACT (select_kernel, one workgroup per sequence): a lone survivor wins as it stands; several
//     are scored in fp64 by the definition above as written, argmax with lowest-index ties.
//
// Rows the bounds cannot separate (nearly identical target and draft rows, an empty residual,
// a survivor list that overflows) fall back to an fp64 scan, so the result is always the
// definition's.  The accept / first-reject scan runs in the filter kernel's prologue (one wave),
// so a whole verification is three back-to-back launches: row statistics, filter, select; two when
// a row is split into at most two chunks (sample_select_kernel: filter and select in one).
#pragma once

#include "decide.h"
#include "ears_device.h"

namespace ears {

constexpr int kSurvivorCap = kWave;            // survivors kept per wave while it filters
constexpr float kExpMargin = 0x1p-12f;         // on a(v): covers fp32 rounding of (l-m)*c - log2 Z
constexpr float kScoreMargin = 0x1p-12f;       // on the fp32 score: v_log_f32 / adds
constexpr float kBonusMargin = 0x1p-10f;       // bonus scores carry l*c itself (|l|/T up to ~1e3)
constexpr float kTestMargin = 0x1p-10f;        // slack of the level-1 test
constexpr float kDegenerate = -100.0f;         // residual rows whose best lower bound is below
                                               // 2^-100 are scanned in fp64 instead
// "no bound yet".  Finite, and still finite after scaling by 2^23, so that the level-1 bound of a
// masked or out-of-range element (-inf) never reaches it.
constexpr float kNoThreshold = -1.0e30f;

enum { kModeResidual = 0, kModeBonus = 1, kModeTargetFallback = 2 };

struct SampleCtx {
  const void* trow;
  const void* drow;
  double mt, Zt, md, Zd, T;
  uint64_t seed, seq;
  uint32_t pos;
  int V;
  bool exact;  // Zt and Zd are fp64 sums (not the statistics pass's fp32-lane sums)
};

// word v & 3 of a block, by value selects (no indexed access to the block)
__device__ __forceinline__ uint32_t philox_pick(const Philox blk, uint32_t v) {
  const uint32_t w0 = blk.w0, w1 = blk.w1, w2 = blk.w2, w3 = blk.w3;
  const uint32_t lo = (v & 1u) ? w1 : w0;
  const uint32_t hi = (v & 1u) ? w3 : w2;
  return (v & 2u) ? hi : lo;
}

// The statistics pass sums exponentials in fp32 lanes: its Z is within this relative distance of
// the fp64 sum (measured: 4.3e-7 at most).  p_t(v) - p_d(v) inherits an absolute uncertainty of
// kZRelError * (p_t + p_d), which matters where the two nearly cancel.
constexpr double kZRelError = 1.0e-6;
// Support of the residual: p_t(v) - p_d(v) must exceed this fraction of p_t(v) + p_d(v); below it the
// difference of two fp64 softmax values is rounding noise (same constant on the checking side).
constexpr double kResidualFloor = 0x1p-40;

// Level 3: the score exactly as defined, fp64.  -inf means "not a candidate".  With `lo` / `hi` the
// score's range under the uncertainty of the cached Z is returned as well (residual mode; the
// other modes have lo = hi = score).
template <typename DT>
__device__ double exact_score(const SampleCtx& c, int v, int mode, double* lo = nullptr,
                              double* hi = nullptr) {
  const double lt = (double)DT::load(c.trow, v);
  double logw, logw_lo, logw_hi;
  if (lo) *lo = -INFINITY;
  if (hi) *hi = -INFINITY;
  if (mode == kModeBonus) {
    if (!(lt > -INFINITY)) return -INFINITY;
    logw = logw_lo = logw_hi = lt / c.T;
  } else {
    const double pt = exp((lt - c.mt) / c.T) / c.Zt;
    if (mode == kModeResidual) {
      const double pd = exp(((double)DT::load(c.drow, v) - c.md) / c.T) / c.Zd;
      const double q = pt - pd;
      const double floor_q = kResidualFloor * (pt + pd);
      // with the cached Z the difference is only known to within dq; with fp64 sums it is exact
      const double dq = c.exact ? 0.0 : kZRelError * (pt + pd);
      if (!(q + dq > floor_q)) return -INFINITY;
      logw_hi = log(q + dq);
      logw_lo = (q - dq > floor_q) ? log(q - dq) : -INFINITY;
      logw = (q > floor_q) ? log(q) : -INFINITY;
    } else {
      if (!(pt > 0.0)) return -INFINITY;
      logw = logw_lo = logw_hi = log(pt);
    }
  }
  const uint32_t cw = philox_pick(noise_block(c.seed, c.seq, c.pos, kDomainCoarse, (uint32_t)v >> 4),
                                  (uint32_t)v >> 2);
  const uint32_t h = (cw >> (8u * ((uint32_t)v & 3u))) & 0xFFu;
  const uint32_t f = philox_pick(noise_block(c.seed, c.seq, c.pos, kDomainFine, (uint32_t)v >> 2),
                                 (uint32_t)v);
  const double u = ((double)h + ((double)f + 0.5) * 0x1p-32) * 0x1p-8;
  const double g = -log(-log(u));
  if (lo) *lo = logw_lo + g;
  if (hi) *hi = logw_hi + g;
  return logw + g;
}

// Z = sum_v exp((l_v - m) / T) of one row, fp64 throughout, by the whole workgroup (slow: only for
// rows whose winner the cached Z cannot settle).
template <typename DT>
__device__ double block_sumexp64(const void* row, int V, double m, double T) {
  __shared__ double sh_part[kWavesPerBlock];
  double acc = 0.0;
  for (int v = (int)threadIdx.x; v < V; v += kBlock) {
    const double l = (double)DT::load(row, v);
    if (l > -INFINITY) acc += exp((l - m) / T);
  }
  acc = wave_sum(acc);
  __syncthreads();
  if (((int)threadIdx.x & (kWave - 1)) == 0) sh_part[(int)threadIdx.x / kWave] = acc;
  __syncthreads();
  double Z = 0.0;
#pragma unroll
  for (int w = 0; w < kWavesPerBlock; ++w) Z += sh_part[w];
  return Z;
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
__device__ Best exact_scan(const SampleCtx& c, int v0, int v1, int mode, Best best) {
  for (int v = v0 + (int)threadIdx.x; v < v1; v += kBlock) {
    const double s = exact_score<DT>(c, v, mode);
    if (s > -INFINITY && better(s, v, best)) best = Best{s, v};
  }
  return best;
}

__device__ __forceinline__ int lanes_below(unsigned long long mask) {
  return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                        __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// The filter of chunk s = blockIdx.x * G + g of sequence blockIdx.y, by sub-block g (512 threads)
// of a workgroup of G * 512 threads.  With G > 1 a workgroup filters G chunks of one row side by
// side; the sub-blocks share nothing but the accept length and the barriers.
// kLate: the decisions are taken here, from the cached statistics (a DECIDE | SAMPLE call); kept
// out of the other instantiations because the fp64 decision raises the register count.
template <typename DT, int G, bool kLate>
__device__ __forceinline__ void sample_body(const Problem& p) {
  constexpr int kPer = DT::kPerVec;
  constexpr int kVecs = kSampleLaneElems / kPer;  // 16-byte loads per lane and tile
  constexpr int kTile = kSampleTileElems;
  constexpr int kQueueCap = 2 * kWave;  // drained as soon as it holds a full batch
  using storage = typename DT::storage;

  constexpr int kWaves = G * kWavesPerBlock;               // waves of the whole workgroup
  __shared__ int sh_queue[kWaves][kQueueCap];              // queued vocabulary indices ...
  __shared__ int sh_queue_h[kWaves][kQueueCap];            // ... and their coarse noise bytes
  __shared__ int sh_surv_v[kWaves][kSurvivorCap];
  __shared__ float sh_surv_s[kWaves][kSurvivorCap];
  __shared__ float sh_theta[kWaves];
  __shared__ int sh_n, sh_count_g[G], sh_overflow_g[G];

  const int g = (int)threadIdx.x / kBlock;                 // sub-block, uniform over a wave
  const int tid = (int)threadIdx.x - g * kBlock, lane = tid & (kWave - 1);
  const int wave = (int)threadIdx.x / kWave;               // index into the per-wave arrays
  const int wave_g = tid / kWave;                          // wave within the sub-block
  const int s = (int)blockIdx.x * G + g, b = (int)blockIdx.y;
  const int V = p.V;

  // ---- accept length of this sequence ---------------------------------------------------------
  const int Kb = seq_len(p, b);
  if (tid == 0) { sh_count_g[g] = 0; sh_overflow_g[g] = 0; }
  if (p.decide_fused) {
    // one decision per position, left by the statistics kernel or taken here from the cached
    // statistics; the first rejection is the accept length
    if (wave == 0) {
      const int nn = first_reject_scan(p, b, lane, !kLate, s == 0);
      if (lane == 0) sh_n = nn;
    }
  } else if (threadIdx.x == 0) {
    const int nn = p.accept_len[b];
    sh_n = nn < 0 ? 0 : (nn > Kb ? Kb : nn);
  }
  __syncthreads();
  const int n = sh_n;

  const int64_t r0 = seq_row_begin(p, b);
  const bool residual = n < Kb;
  const int64_t r = r0 + (residual ? n : Kb - 1);  // draft row of the rejected slot (if any)
  const storage* trow = static_cast<const storage*>(p.target) + (r0 + b + n) * (int64_t)V;
  const storage* drow = static_cast<const storage*>(p.draft) + r * (int64_t)V;
  const float Tf = seq_temperature(p, b);
  const uint64_t seed = p.seed, seq = seq_rng_id(p, b);
  const uint32_t pos = (uint32_t)n;

  // fp32 constants of levels 1 and 2
  const float c = (float)(kLog2e / (double)Tf);
  float mt = 0.0f, kt = 0.0f, md = 0.0f, kd = 0.0f;
  if (residual) {
    mt = p.m[2 * r];
    md = p.m[2 * r + 1];
    kt = -__builtin_amdgcn_logf((float)p.Z[2 * r]);
    kd = -__builtin_amdgcn_logf((float)p.Z[2 * r + 1]);
  }
  // level-1 bound, scaled by 2^23: l*cs + ks - bits(float(N)) >= theta * 2^23
  const float cs = c * 0x1p23f;
  const float ks = (float)(((double)kt + 135.0 + (double)kTestMargin - (double)mt * (double)c) * 0x1p23);

  float theta = kNoThreshold;  // wave-uniform: best proven lower bound of the maximum score (log2)
  int qcount = 0;            // wave-uniform: queued candidates
  int scount = 0;            // wave-uniform: survivors of this wave
  bool overflow = false;

  // Level 2 for up to 64 queued elements, one per lane.  h_known is the element's coarse noise
  // byte when the caller has it (queued elements), -1 when it has to be generated here.
  auto evaluate = [&](int v, int h_known, bool active, float& s_up, float& s_lo) {
    s_up = -INFINITY;
    s_lo = -INFINITY;
    const int vv = active ? v : 0;
    const float lt = DT::load(trow, vv);
    // u = (h + (f + 1/2) 2^-32) / 256 and 1 - u, each to fp32 relative accuracy
    uint32_t h = (uint32_t)h_known;
    if (h_known < 0) {
      const uint32_t cw = philox_pick(noise_block(seed, seq, pos, kDomainCoarse, (uint32_t)vv >> 4),
                                      (uint32_t)vv >> 2);
      h = (cw >> (8u * ((uint32_t)vv & 3u))) & 0xFFu;
    }
    const uint32_t f = philox_pick(noise_block(seed, seq, pos, kDomainFine, (uint32_t)vv >> 2),
                                   (uint32_t)vv);
    const float u = ((float)h + fmaf((float)f, 0x1p-32f, 0x1p-33f)) * 0x1p-8f;
    const float om = ((float)(255u - h) + fmaf((float)(~f), 0x1p-32f, 0x1p-33f)) * 0x1p-8f;
    // E = -ln u bracketed by [e_lo, e_hi]; close to u = 1 from the series of -ln(1 - x)
    float e_lo, e_hi;
    if (om < 0x1p-6f) {
      const float t = fmaf(0.5f, om, 1.0f);
      e_lo = om * t;                          // x + x^2/2
      e_hi = om * fmaf(0.5f * om, om, t);     // x + x^2/2 + x^3/2, an upper bound for x <= 1/4
    } else {
      e_lo = e_hi = -__builtin_amdgcn_logf(u) * 0.6931471805599453f;
    }
    const float g_hi = -__builtin_amdgcn_logf(e_lo);   // -log2(-ln u), from above
    const float g_lo = -__builtin_amdgcn_logf(e_hi);   //               and from below
    float up = -INFINITY, lo = -INFINITY;
    if (residual) {
      // with p_d = 0 the score could be at most a(v) + g: only lanes that can still reach theta
      // that way fetch the draft logit (a scattered access) and evaluate the residual
      const float at = fmaf(lt - mt, c, kt);
      if (active && at + kExpMargin + g_hi + kScoreMargin >= theta) {
        const float ld = DT::load(drow, vv);
        const float ad = fmaf(ld - md, c, kd);
        const float q_up = __builtin_amdgcn_exp2f(at + kExpMargin) - __builtin_amdgcn_exp2f(ad - kExpMargin);
        const float q_lo = __builtin_amdgcn_exp2f(at - kExpMargin) - __builtin_amdgcn_exp2f(ad + kExpMargin);
        up = q_up > 0.0f ? __builtin_amdgcn_logf(q_up) + g_hi + kScoreMargin : -INFINITY;
        lo = q_lo > 0.0f ? __builtin_amdgcn_logf(q_lo) + g_lo - kScoreMargin : -INFINITY;
      }
    } else {
      up = fmaf(lt, c, g_hi) + kBonusMargin;
      lo = fmaf(lt, c, g_lo) - kBonusMargin;
    }
    if (active && up > -INFINITY) { s_up = up; s_lo = lo; }
  };

  auto compact_survivors = [&]() {
    // drop survivors that the risen threshold has overtaken (one entry per lane)
    const bool have = lane < scount;
    const int v = have ? sh_surv_v[wave][lane] : 0;
    const float su = have ? sh_surv_s[wave][lane] : -INFINITY;
    const bool keep = have && su >= theta;
    const unsigned long long km = __ballot(keep);
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    if (keep) {
      const int slot = lanes_below(km);
      sh_surv_v[wave][slot] = v;
      sh_surv_s[wave][slot] = su;
    }
    scount = __popcll(km);
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
  };

  auto evaluate_batch = [&](int cnt) {
    const bool active = lane < cnt;
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    const int v = active ? sh_queue[wave][qcount - cnt + lane] : 0;
    const int h = active ? sh_queue_h[wave][qcount - cnt + lane] : 0;
    qcount -= cnt;
    float s_up, s_lo;
    evaluate(v, h, active, s_up, s_lo);
    theta = fmaxf(theta, wave_max(s_lo));
    const bool surv = active && s_up > -INFINITY && s_up >= theta;
    const unsigned long long sm = __ballot(surv);
    const int add = __popcll(sm);
    if (add == 0) return;
    if (scount + add > kSurvivorCap) compact_survivors();
    if (scount + add > kSurvivorCap) { overflow = true; return; }
    if (surv) {
      const int slot = scount + lanes_below(sm);
      sh_surv_v[wave][slot] = v;
      sh_surv_s[wave][slot] = s_up;
    }
    scount += add;
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
  };

  const int v_begin = s * p.chunk;
  const int v_end = (V - v_begin) < p.chunk ? V : v_begin + p.chunk;
  const bool vector_ok = (reinterpret_cast<uintptr_t>(trow) & 15u) == 0;

  // One 16-byte load; rows that are not 16-byte aligned (or the ragged last vector) are assembled
  // from element loads into the same packed form, padded with -inf.  Ordinary cached loads: a
  // lane's loads of one tile are adjacent 16-byte pieces of the same cache lines, which
  // non-temporal loads would fetch from memory once per piece (1.6x the row's bytes, measured).
  auto load_raw = [&](int vb) -> uint4 {
    if (vb >= v_end) return DT::neg_inf_vec();
    if (vector_ok && vb + kPer <= v_end) return *reinterpret_cast<const uint4*>(trow + vb);
    uint32_t wds[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      if (sizeof(storage) == 2) {
        const uint32_t lo = (vb + 2 * d < v_end) ? (uint32_t)reinterpret_cast<const uint16_t*>(trow)[vb + 2 * d] : 0xFF80u;
        const uint32_t hi = (vb + 2 * d + 1 < v_end) ? (uint32_t)reinterpret_cast<const uint16_t*>(trow)[vb + 2 * d + 1] : 0xFF80u;
        wds[d] = lo | (hi << 16);
      } else {
        wds[d] = (vb + d < v_end) ? reinterpret_cast<const uint32_t*>(trow)[vb + d] : 0xFF800000u;
      }
    }
    return make_uint4(wds[0], wds[1], wds[2], wds[3]);
  };

  // a lane owns kSampleLaneElems consecutive entries of each tile: kVecs 16-byte loads and
  // exactly one coarse Philox block
  uint4 raw[kVecs];
#pragma unroll
  for (int k = 0; k < kVecs; ++k) raw[k] = load_raw(v_begin + tid * kSampleLaneElems + k * kPer);

  // warm start: a first threshold from 64 elements of this wave's part of the chunk (their loads
  // travel together with the first tile's)
  {
    const int v = v_begin + wave_g * kWave + lane;
    float s_up, s_lo;
    evaluate(v, -1, v < v_end, s_up, s_lo);
    theta = fmaxf(theta, wave_max(s_lo));
  }

  for (int tile0 = v_begin; tile0 < v_end; tile0 += kTile) {
    const int vbase = tile0 + tid * kSampleLaneElems;
    float l[kSampleLaneElems];
#pragma unroll
    for (int k = 0; k < kVecs; ++k) {
      float g[kPer];
      DT::unpack(raw[k], g);
#pragma unroll
      for (int j = 0; j < kPer; ++j) l[k * kPer + j] = g[j];
      raw[k] = load_raw(vbase + kTile + k * kPer);  // next tile, in flight while this one is tested
    }
    // level 1
    const float Theta = theta * 0x1p23f;
    const Philox coarse = noise_block(seed, seq, pos, kDomainCoarse, (uint32_t)vbase >> 4);
    float bound[kSampleLaneElems];
    uint32_t nw[4];
    float bmax = -INFINITY;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      nw[k] = ~coarse.word(k);  // bytes N = 255 - h
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int j = 4 * k + t;
        const float Nf = (float)((nw[k] >> (8 * t)) & 0xFFu);
        // the bit pattern of float(N), read as an integer, is (log2 N + 127) * 2^23 from below
        bound[j] = fmaf(l[j], cs, ks) - (float)__float_as_int(Nf);
        bmax = fmaxf(bmax, bound[j]);
      }
    }
    if (__ballot(bmax >= Theta) != 0ull) {
#pragma unroll
      for (int j = 0; j < kSampleLaneElems; ++j) {
        const bool pj = bound[j] >= Theta;
        const unsigned long long bal = __ballot(pj);
        if (bal != 0ull) {
          if (pj) {
            const int slot = qcount + lanes_below(bal);
            sh_queue[wave][slot] = vbase + j;
            sh_queue_h[wave][slot] = (int)(255u - ((nw[j >> 2] >> (8 * (j & 3))) & 0xFFu));
          }
          qcount += __popcll(bal);
          if (qcount >= kWave) evaluate_batch(kWave);
        }
      }
    }
  }
  if (qcount > 0) evaluate_batch(qcount);
  compact_survivors();

  // ---- merge the four waves into this chunk's record -------------------------------------------
  if (lane == 0) sh_theta[wave] = theta;
  __syncthreads();
  float theta_wg = sh_theta[g * kWavesPerBlock];
#pragma unroll
  for (int w = 1; w < kWavesPerBlock; ++w) theta_wg = fmaxf(theta_wg, sh_theta[g * kWavesPerBlock + w]);
  uint32_t* rec = p.records + ((size_t)b * p.S + s) * kRecordWords;
  {
    const bool have = lane < scount;
    const int v = have ? sh_surv_v[wave][lane] : 0;
    const float su = have ? sh_surv_s[wave][lane] : -INFINITY;
    const bool keep = have && su >= theta_wg;
    const unsigned long long km = __ballot(keep);
    int base = 0;
    if (lane == 0 && km != 0ull) base = atomicAdd(&sh_count_g[g], __popcll(km));
    base = __shfl(base, 0, 64);
    if (keep) {
      const int slot = base + lanes_below(km);
      if (slot < kRecordCap) {
        rec[2 + 2 * slot] = (uint32_t)v;
        rec[3 + 2 * slot] = __float_as_uint(su);
      }
    }
    if (overflow && lane == 0) sh_overflow_g[g] = 1;
  }
  __syncthreads();
  if (tid == 0) {
    rec[0] = __float_as_uint(theta_wg);
    rec[1] = (sh_overflow_g[g] || sh_count_g[g] > kRecordCap) ? (uint32_t)kRecordOverflow
                                                            : (uint32_t)sh_count_g[g];
  }
}

template <typename DT, bool kLate>
__global__ __launch_bounds__(kBlock) void sample_kernel(Problem p) {
  sample_body<DT, 1, kLate>(p);
}

// Level 3.  One workgroup per sequence reads the chunk records of the filter kernel.  A single
// survivor is the winner as it stands; several are scored in fp64 by the definition; rows the
// bounds could not separate are scanned in fp64.  In the common case everything this kernel needs
// (accept length, chunk headers, survivor entries) is requested in one round of loads.
template <typename DT>
__device__ __forceinline__ void select_body(const Problem& p, int b) {
  using storage = typename DT::storage;
  __shared__ float sh_theta[kWavesPerBlock];
  __shared__ int sh_any_overflow, sh_total, sh_only;
  const int tid = (int)threadIdx.x;
  const int V = p.V;
  const uint32_t* recs = p.records + (size_t)b * p.S * kRecordWords;
  const int total = p.S * kRecordCap;

  // ---- one round of loads ---------------------------------------------------------------------
  const int n_raw = p.accept_len[b];
  const int64_t r0 = seq_row_begin(p, b);
  const int Kb = seq_len(p, b);
  float th = kNoThreshold;
  bool ovf = false;
  for (int i = tid; i < p.S; i += kBlock) {
    th = fmaxf(th, __uint_as_float(recs[(size_t)i * kRecordWords]));
    ovf = ovf || (int)recs[(size_t)i * kRecordWords + 1] == kRecordOverflow;
  }
  // this thread's survivor entry (further entries, for rows split into many chunks, come later)
  int e_cnt = 0, e_j = 0, e_v = -1;
  float e_s = -INFINITY;
  if (tid < total) {
    const int i = tid / kRecordCap;
    e_j = tid - i * kRecordCap;
    const uint32_t* rc = recs + (size_t)i * kRecordWords;
    e_cnt = (int)rc[1];
    e_v = (int)rc[2 + 2 * e_j];
    e_s = __uint_as_float(rc[3 + 2 * e_j]);
  }
  if (tid == 0) { sh_any_overflow = 0; sh_total = 0; sh_only = -1; }

  // ---- best lower bound over the chunks of this row ----------------------------------------------
  th = wave_max(th);
  __syncthreads();
  if ((tid & (kWave - 1)) == 0) sh_theta[tid / kWave] = th;
  if (ovf) sh_any_overflow = 1;
  __syncthreads();
  float theta_g = sh_theta[0];
#pragma unroll
  for (int w = 1; w < kWavesPerBlock; ++w) theta_g = fmaxf(theta_g, sh_theta[w]);
  const bool any_overflow = sh_any_overflow != 0;

  const int n = n_raw < 0 ? 0 : (n_raw > Kb ? Kb : n_raw);
  const bool residual = n < Kb;
  const bool separable = theta_g > (residual ? kDegenerate : kNoThreshold);

  // ---- survivors of the whole row: entries whose upper bound reaches the best lower bound --------
  auto is_survivor = [&](int cnt, int j, float su) {
    return cnt != kRecordOverflow && j < cnt && su >= theta_g;
  };
  int mine = 0, my_v = -1;
  if (separable) {
    if (is_survivor(e_cnt, e_j, e_s)) { mine = 1; my_v = e_v; }
    for (int idx = tid + kBlock; idx < total; idx += kBlock) {
      const int i = idx / kRecordCap, j = idx - i * kRecordCap;
      const uint32_t* rc = recs + (size_t)i * kRecordWords;
      if (is_survivor((int)rc[1], j, __uint_as_float(rc[3 + 2 * j]))) { ++mine; my_v = (int)rc[2 + 2 * j]; }
    }
    if (mine > 0) { atomicAdd(&sh_total, mine); sh_only = my_v; }
  }
  __syncthreads();
  if (separable && !any_overflow && sh_total == 1) {
    if (tid == 0) p.out_tokens[r0 + b + n] = sh_only;  // nothing to compare it with
    return;
  }

  // ---- several survivors, or a row the bounds could not separate: fp64 ---------------------------
  const int64_t r = r0 + (residual ? n : Kb - 1);
  SampleCtx ctx;
  ctx.trow = static_cast<const storage*>(p.target) + (r0 + b + n) * (int64_t)V;
  ctx.drow = static_cast<const storage*>(p.draft) + r * (int64_t)V;
  ctx.mt = residual ? (double)p.m[2 * r] : 0.0;
  ctx.Zt = residual ? p.Z[2 * r] : 1.0;
  ctx.md = residual ? (double)p.m[2 * r + 1] : 0.0;
  ctx.Zd = residual ? p.Z[2 * r + 1] : 1.0;
  ctx.T = (double)seq_temperature(p, b);
  ctx.seed = p.seed;
  ctx.seq = seq_rng_id(p, b);
  ctx.pos = (uint32_t)n;
  ctx.V = V;
  ctx.exact = false;
  const int mode = residual ? kModeResidual : kModeBonus;
  __shared__ double sh_lo_best;
  // replaces the cached Z of both rows by fp64 sums: after it the scores are the definition's
  auto make_exact = [&]() {
    if (ctx.exact) return;  // uniform
    ctx.Zt = block_sumexp64<DT>(ctx.trow, V, ctx.mt, ctx.T);
    ctx.Zd = block_sumexp64<DT>(ctx.drow, V, ctx.md, ctx.T);
    ctx.exact = true;
  };
  // Scores of the surviving entries; a thread keeps what it computed for its first entry, so the
  // second pass (ranges) costs nothing more in the usual case of at most one entry per thread.
  int c_v = -1;
  double c_s = -INFINITY, c_lo = -INFINITY, c_hi = -INFINITY;
  auto score_survivors = [&](bool with_range, int skip_v, Best& out, double& lo_of_skip) {
    // out: arg-max of the score (with_range false) or of the upper ends over v != skip_v (true)
    for (int idx = tid; idx < total; idx += kBlock) {
      const int i = idx / kRecordCap, j = idx - i * kRecordCap;
      const uint32_t* rc = recs + (size_t)i * kRecordWords;
      if (is_survivor((int)rc[1], j, __uint_as_float(rc[3 + 2 * j]))) {
        const int v = (int)rc[2 + 2 * j];
        double sc, lo, hi;
        if (idx == tid && c_v == v) {
          sc = c_s; lo = c_lo; hi = c_hi;
        } else {
          sc = exact_score<DT>(ctx, v, mode, &lo, &hi);
          if (idx == tid) { c_v = v; c_s = sc; c_lo = lo; c_hi = hi; }
        }
        if (!with_range) {
          if (sc > -INFINITY && better(sc, v, out)) out = Best{sc, v};
        } else if (v == skip_v) {
          lo_of_skip = lo;
        } else if (hi > -INFINITY && better(hi, v, out)) {
          out = Best{hi, v};
        }
      }
    }
  };
  Best best{-INFINITY, -1};
  double unused = 0.0;
  if (separable && !any_overflow) {
    score_survivors(false, -1, best, unused);
    best = block_best(best);
    if (residual) {
      // Is the winner beyond the reach of the cached Z's uncertainty?  Its lowest possible score
      // must exceed the highest possible score of every other survivor.
      Best rival{-INFINITY, -1};
      double lo_best = -INFINITY;
      if (tid == 0) sh_lo_best = -INFINITY;
      __syncthreads();
      score_survivors(true, best.v, rival, lo_best);
      if (lo_best > -INFINITY) sh_lo_best = lo_best;  // one thread owns the winner's entry
      rival = block_best(rival);
      __syncthreads();
      const bool settled = best.v >= 0 && (rival.v < 0 || sh_lo_best > rival.s);
      if (!settled) {
        make_exact();
        c_v = -1;  // cached scores used the cached Z
        best = Best{-INFINITY, -1};
        score_survivors(false, -1, best, unused);
        best = block_best(best);
      }
    }
  } else {
    if (residual) make_exact();
    if (separable) {
      score_survivors(false, -1, best, unused);
      for (int i = 0; i < p.S; ++i) {
        if ((int)recs[(size_t)i * kRecordWords + 1] == kRecordOverflow) {
          const int c0 = i * p.chunk;
          const int c1 = (V - c0) < p.chunk ? V : c0 + p.chunk;
          best = exact_scan<DT>(ctx, c0, c1, mode, best);
        }
      }
      best = block_best(best);
    }
  }
  if (best.v < 0) {
    // the bounds could not separate this row, or no survivor has a positive residual: evaluate the
    // definition over the whole row (with fp64 sums for Z: make_exact is idempotent)
    if (residual) make_exact();
    best = block_best(exact_scan<DT>(ctx, 0, V, mode, Best{-INFINITY, -1}));
    if (best.v < 0 && residual)  // empty residual: draw from the target distribution itself
      best = block_best(exact_scan<DT>(ctx, 0, V, kModeTargetFallback, Best{-INFINITY, -1}));
  }
  if (tid == 0) p.out_tokens[r0 + b + n] = best.v;
}

template <typename DT>
__global__ __launch_bounds__(kBlock) void select_kernel(Problem p) {
  select_body<DT>(p, (int)blockIdx.x);
}

// Filter and exact choice in one launch, for rows that are split into G <= 2 chunks: a workgroup of
// G * 512 threads filters all chunks of its row, then its first 512 threads read the records it
// has just written (visible within the workgroup after the barrier) and choose.  Saves a launch
// and the dependent start of a second kernel.  Registers: the single-chunk bf16 variant is held to
// 80 (three 512-thread groups per CU, as the filter alone); the others run one or two groups per
// CU whatever they use.
template <typename DT, int G, bool kLate>
__global__ __launch_bounds__(kBlock* G, (G == 1 && !kLate && sizeof(typename DT::storage) == 2) ? 6 : 4)
void sample_select_kernel(Problem p) {
  sample_body<DT, G, kLate>(p);
  __syncthreads();
  if ((int)threadIdx.x >= kBlock) return;  // whole waves
  select_body<DT>(p, (int)blockIdx.y);
}

}  // namespace ears
