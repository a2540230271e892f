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
//  3. EXACT (select_body, one workgroup per sequence): a lone survivor wins as it stands; several
//     are scored in fp64 by the definition above as written, argmax with lowest-index ties.
//
// Rows the bounds cannot separate (nearly identical target and draft rows, an empty residual,
// a survivor list that overflows) fall back to an fp64 scan, so the result is always the
// definition's.  The accept / first-reject scan runs in the filter's prologue (one wave) and the
// exact choice in its epilogue, so a whole verification is two back-to-back launches: row
// statistics, then filter and choice; or one launch in which the workgroups that run this code
// follow those of the statistics (verify.h).
#pragma once

#include <type_traits>

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

// A load whose address is the same in every lane, from memory that no kernel writes while this one
// runs: through the constant address space it is a scalar load.
template <typename T>
__device__ __forceinline__ T uniform_load(const T* ptr) {
  typedef const T __attribute__((address_space(4))) * const_ptr;
  return *(const_ptr)(uintptr_t)ptr;
}

// Integers ordered like the floats they stand for (finite values), and back.
__device__ __forceinline__ int ordered_int(float x) {
  const int b = __float_as_int(x);
  return b ^ ((b >> 31) & 0x7FFFFFFF);
}
__device__ __forceinline__ float ordered_float(int k) {
  return __int_as_float(k ^ ((k >> 31) & 0x7FFFFFFF));
}

__device__ __forceinline__ int lanes_below(unsigned long long mask) {
  return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                        __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// The filter of chunk s = blockIdx.x * G + g of sequence blockIdx.y, by sub-block g (512 threads)
// of a workgroup of G * 512 threads.  With G > 1 a workgroup filters G chunks of one row side by
// side; the sub-blocks share the accept length, the thresholds their waves publish, and the
// barriers.  Returns true when the workgroup has settled the row's token by itself (kFused: the
// chunks of this workgroup are the whole row, exactly one entry survived and it has been written).
// kLate: the decisions are taken here, from the cached statistics (a DECIDE | SAMPLE call); kept
// out of the other instantiations because the fp64 decision raises the register count.
//
// Per tile a lane owns kSampleLaneElems consecutive entries and one coarse Philox block.  The
// common path never looks at an entry on its own:
//   - entries whose coarse byte is 255 (N = 0: the level-1 bound is vacuous) are found with three
//     bit operations per noise word and queued for level 2;
//   - all other entries have N >= 1, so none of the lane's entries can pass level 1 unless the
//     lane's largest logit passes it with N = 1; a lane for which it does is queued as a whole
//     ("group") and its 16 entries are tested one by one later, 64 groups at a time, against the
//     threshold of that later moment.
// Waves publish their thresholds in LDS and pick up the largest at every tile: a lower bound of
// the best score of any part of the row is one of the whole row's best score.
// n_out receives the sequence's accept length.
// kHand: the statistics and decisions of the sequence come from workgroups of the same launch
// (verify_kernel): the first wave waits for them, and they are read with coherent loads; n_out is
// -1, and nothing has been done, if the wait was given up.  `bid` is the workgroup's number among
// those of the sampling stage.
template <typename DT, int G, bool kLate, bool kFused, bool kHand = false>
__device__ __forceinline__ bool sample_body(const Problem& p, int& n_out, unsigned bid) {
  constexpr int kPer = DT::kPerVec;
  constexpr int kVecs = kSampleLaneElems / kPer;  // 16-byte loads per lane and tile
  constexpr int kTile = kSampleTileElems;
  constexpr int kQueueCap = 2 * kWave;  // drained as soon as it holds a full batch
  using storage = typename DT::storage;

  constexpr int kWaves = G * kWavesPerBlock;               // waves of the whole workgroup
  // Entries queued for level 2 (vocabulary index and coarse noise byte) and groups queued for the
  // entry-by-entry level 1 (index of their first entry): kQueueCap slots per wave, then a pool that
  // all waves of the workgroup fill and empty together (each contributes fewer than 64).
  constexpr int kPool = kWaves * kQueueCap, kPoolCap = kWaves * kWave;
  __shared__ int sh_ent_v[kPool + kPoolCap];
  __shared__ int sh_ent_h[kPool + kPoolCap];
  __shared__ int sh_grp[kPool + kPoolCap];
  __shared__ int sh_pool_n[3];                             // warm-up entries, last groups, last entries
  __shared__ int sh_surv_v[kWaves][kSurvivorCap];
  __shared__ float sh_surv_s[kWaves][kSurvivorCap];
  __shared__ int sh_theta_row;                             // the row's threshold, as an ordered integer
  __shared__ int sh_n, sh_count_g[G], sh_overflow_g[G], sh_only;

  // wave-uniform quantities are kept in scalar registers: the branches on them are scalar branches
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x / kWave);  // within the workgroup
  const int g = wave / kWavesPerBlock;                     // sub-block
  const int wave_g = wave - g * kWavesPerBlock;            // wave within the sub-block
  const int tid = (int)threadIdx.x - g * kBlock, lane = (int)threadIdx.x & (kWave - 1);
  // workgroups are numbered along x: all those of a row one after the other
  const int groups_per_row = kFused ? 1 : p.S;
  const int b = (int)(bid / (unsigned)groups_per_row);
  const int s = ((int)bid - b * groups_per_row) * G + g;
  const int V = p.V;

  // ---- accept length of this sequence ---------------------------------------------------------
  const int Kb = seq_len(p, b);
  if (tid == 0) { sh_count_g[g] = 0; sh_overflow_g[g] = 0; }
  if (threadIdx.x == 0) sh_only = -1;
  if (threadIdx.x == 0) sh_theta_row = ordered_int(kNoThreshold);
  if (threadIdx.x < 3) sh_pool_n[threadIdx.x] = 0;
  int n;
  if (kHand) {
    if (wave == 0) {
      const int nn = await_first_reject(p, b, lane, s == 0);
      if (lane == 0) sh_n = nn;
    }
    lds_barrier();
    n = sh_n;
    if (n < 0) {  // uniform over the workgroup
      n_out = -1;
      return false;
    }
  } else if (!kLate && p.decide_fused) {
    // one decision per position, left by the statistics kernel: every wave scans them for itself
    // (the same few words for all of them), the first wave of the row's first chunk stores the
    // accept length and the accepted prefix
    n = first_reject_scan(p, b, lane, true, s == 0 && wave_g == 0);
    lds_barrier();  // thresholds initialised before any wave reads another's
  } else {
    if (kLate) {
      // the decisions are taken here from the cached statistics, by one wave
      if (wave == 0) {
        const int nn = first_reject_scan(p, b, lane, false, s == 0);
        if (lane == 0) sh_n = nn;
      }
    } else if (threadIdx.x == 0) {
      const int nn = p.accept_len[b];
      sh_n = nn < 0 ? 0 : (nn > Kb ? Kb : nn);
    }
    lds_barrier();
    n = sh_n;
  }
  n = __builtin_amdgcn_readfirstlane(n);
  n_out = n;

  const int64_t r0 = seq_row_begin(p, b);
  const bool residual = n < Kb;
  const int64_t r = r0 + (residual ? n : Kb - 1);  // draft row of the rejected slot (if any)
  const storage* trow = static_cast<const storage*>(p.target) + (r0 + b + n) * (int64_t)V;
  const storage* drow = static_cast<const storage*>(p.draft) + r * (int64_t)V;
  const float Tf = seq_temperature(p, b);
  const uint64_t seed = p.seed, seq = seq_rng_id(p, b);
  const uint32_t pos = (uint32_t)n;

  const int v_begin = s * p.chunk;
  const int v_end = (V - v_begin) < p.chunk ? V : v_begin + p.chunk;
  const bool vector_ok = (reinterpret_cast<uintptr_t>(trow) & 15u) == 0;

  // One 16-byte load; rows that are not 16-byte aligned (or the ragged last vector) are assembled
  // from element loads into the same packed form, padded with -inf.  Ordinary cached loads: a
  // lane's loads of one tile are adjacent 16-byte pieces of the same cache lines, which
  // non-temporal loads would fetch from memory once per piece (1.6x the row's bytes, measured).
  auto load_raw = [&](int vb, int v_end) -> uint4 {
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

  const int lane_off = tid * kSampleLaneElems;

  // fp32 constants of levels 1 and 2.  The cached statistics are the same words for every lane:
  // read through the constant address space they are scalar loads, which leave the vector-memory
  // counter to the tile loads that follow.
  // (kHand: they come from workgroups of the running launch and are vector loads of device scope;
  // they are requested here and first looked at, in take_statistics, once the first tile's loads
  // have been requested behind them, so that the two trips to memory are one.)
  const float c = (float)(kLog2e / (double)Tf);
  float mt = 0.0f, kt = 0.0f, md = 0.0f, kd = 0.0f;
  float hand_mt = 0.0f, hand_md = 0.0f;
  double hand_Zt = 1.0, hand_Zd = 1.0;
  if (residual) {
    if (kHand) {
      hand_mt = coherent_load(p.m + 2 * r);
      hand_md = coherent_load(p.m + 2 * r + 1);
      hand_Zt = coherent_load(p.Z + 2 * r);
      hand_Zd = coherent_load(p.Z + 2 * r + 1);
    } else {
      mt = uniform_load(p.m + 2 * r);
      md = uniform_load(p.m + 2 * r + 1);
      kt = -__builtin_amdgcn_logf((float)uniform_load(p.Z + 2 * r));
      kd = -__builtin_amdgcn_logf((float)uniform_load(p.Z + 2 * r + 1));
    }
  }
  // level-1 bound, scaled by 2^23: l*cs + ks - bits(float(N)) >= theta * 2^23
  const float cs = c * 0x1p23f;
  float ks = (float)(((double)kt + 135.0 + (double)kTestMargin - (double)mt * (double)c) * 0x1p23);
  auto take_statistics = [&]() {
    if (kHand && residual) {
      // keeps the compiler from looking at the loaded values (and waiting for them) any earlier
      __builtin_amdgcn_sched_barrier(0);
      asm volatile("" : "+v"(hand_mt), "+v"(hand_md), "+v"(hand_Zt), "+v"(hand_Zd));
      mt = hand_mt;
      md = hand_md;
      kt = -__builtin_amdgcn_logf((float)hand_Zt);
      kd = -__builtin_amdgcn_logf((float)hand_Zd);
      ks = (float)(((double)kt + 135.0 + (double)kTestMargin - (double)mt * (double)c) * 0x1p23);
    }
  };

  float theta = kNoThreshold;  // wave-uniform: best proven lower bound of the maximum score (log2)
  int qcount = 0;            // wave-uniform: queued candidates
  int gcount = 0;            // wave-uniform: queued groups
  int scount = 0;            // wave-uniform: survivors of this wave
  bool overflow = false;

  // Level 2 for up to 64 queued elements, one per lane; h is the element's coarse noise byte.
  auto evaluate = [&](int v, uint32_t h, bool active, float& s_up, float& s_lo) {
    s_up = -INFINITY;
    s_lo = -INFINITY;
    const int vv = active ? v : 0;
    const float lt = DT::load(trow, vv);
    // u = (h + (f + 1/2) 2^-32) / 256 and 1 - u, each to fp32 relative accuracy
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

  // The row's threshold: every wave of the workgroup filters the same row, so a lower bound of the
  // best score of one wave's entries is one of the whole row's.  Kept in LDS as an integer whose
  // order is the floats' (atomic maximum); a wave adopts it at every tile.
  auto publish_threshold = [&]() {
    if (lane == 0) atomicMax(&sh_theta_row, ordered_int(theta));
  };
  auto adopt_threshold = [&]() {
    theta = fmaxf(theta, ordered_float(__hip_atomic_load(&sh_theta_row, __ATOMIC_RELAXED,
                                                         __HIP_MEMORY_SCOPE_WORKGROUP)));
  };

  // level 2 for the cnt (at most 64) entries that start at slot `base` of the entry arrays
  auto evaluate_batch = [&](int base, int cnt) {
    const bool active = lane < cnt;
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    const int v = active ? sh_ent_v[base + lane] : 0;
    const int h = active ? sh_ent_h[base + lane] : 0;
    float s_up, s_lo;
    evaluate(v, (uint32_t)h, active, s_up, s_lo);
    const float best_lo = wave_max(s_lo);
    if (best_lo > theta) {
      theta = best_lo;
      publish_threshold();
    }
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
  const int q0 = wave * kQueueCap;  // this wave's slots of the entry and group arrays

  // Entries waiting to be queued for level 2: bit 8 t + k of pend_pm stands for entry 4 k + t of the
  // group that starts at pend_vb, whose coarse byte is byte t of noise word pend_w[k].
  uint32_t pend_pm = 0u, pend_w0 = 0u, pend_w1 = 0u, pend_w2 = 0u, pend_w3 = 0u;
  int pend_vb = 0;

  // One round: every lane with a waiting entry queues one (as a rule one round empties them all).
  auto queue_round = [&]() {
    const bool has = pend_pm != 0u;
    const int q = has ? __builtin_ctz(pend_pm) : 0;
    pend_pm &= pend_pm - 1u;
    const int k = q & 7, t = q >> 3;
    const int v = pend_vb + 4 * k + t;
    const bool ok = has && v < V;  // beyond the row's end: padding of the last tile
    const unsigned long long bal = __ballot(ok);
    if (ok) {
      // noise word k by bitwise selection (an indexed table of the four words would live in memory)
      const uint32_t k0 = 0u - (uint32_t)(k & 1), k1 = 0u - (uint32_t)((k >> 1) & 1);
      const uint32_t w_lo = (pend_w1 & k0) | (pend_w0 & ~k0), w_hi = (pend_w3 & k0) | (pend_w2 & ~k0);
      const uint32_t wk = (w_hi & k1) | (w_lo & ~k1);
      const int slot = q0 + qcount + lanes_below(bal);
      sh_ent_v[slot] = v;
      sh_ent_h[slot] = (int)((wk >> (8 * t)) & 0xFFu);
    }
    qcount += __popcll(bal);
  };

  // Level 1 entry by entry for the cnt (at most 64) groups that start at slot `base` of the group
  // array, one group per lane: its entries and its coarse block are fetched again (the lines are
  // still in the caches), and every entry with N >= 1 whose bound reaches the threshold of this
  // moment is left waiting for the level-2 queue.
  auto inspect_groups = [&](int base, int cnt) {
    const bool active = lane < cnt;
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    // (a pooled group may belong to another chunk of the row than this wave's: the row's end bounds it)
    const int vb = active ? sh_grp[base + lane] : V;
    const float Theta = theta * 0x1p23f;
    float l[kSampleLaneElems];
#pragma unroll
    for (int k = 0; k < kVecs; ++k) {
      float e[kPer];
      DT::unpack(load_raw(vb + k * kPer, V), e);
#pragma unroll
      for (int j = 0; j < kPer; ++j) l[k * kPer + j] = e[j];
    }
    const Philox coarse = noise_block(seed, seq, pos, kDomainCoarse, (uint32_t)(active ? vb : 0) >> 4);
    uint32_t pm = 0u;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint32_t nw = ~coarse.word(k);  // bytes N = 255 - h
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const float Nf = (float)((nw >> (8 * t)) & 0xFFu);
        // the bit pattern of float(N), read as an integer, is (log2 N + 127) * 2^23 from below
        const float bound = fmaf(l[4 * k + t], cs, ks) - (float)__float_as_int(Nf);
        // entries with N = 0 went to level 2 when their tile was filtered
        if (bound >= Theta && Nf > 0.0f) pm |= 1u << (8 * t + k);
      }
    }
    pend_pm = active ? pm : 0u;
    pend_vb = vb;
    pend_w0 = coarse.w0; pend_w1 = coarse.w1; pend_w2 = coarse.w2; pend_w3 = coarse.w3;
  };

  // Second half: the lane's entries other than those just left waiting have N >= 1, so none of them
  // passes level 1 unless the largest logit does with N = 1 (bits(1.0f) = 127 * 2^23); a lane for
  // which it does is queued as a group.
  auto tile_groups = [&](float lmax, int tile0) {
    const bool whole_group = fmaf(lmax, cs, ks) - 1065353216.0f >= theta * 0x1p23f;
    const unsigned long long gb = __ballot(whole_group);
    if (gb != 0ull) {
      if (whole_group) sh_grp[q0 + gcount + lanes_below(gb)] = tile0 + lane_off;
      gcount += __popcll(gb);
    }
  };

  // Empties what a step left waiting: rounds of queueing; level 2 whenever a full batch is queued;
  // level 1 entry by entry whenever 64 groups are queued.  Leaves fewer than 64 entries and at most
  // 64 groups.
  auto settle = [&]() {
    for (;;) {
      const bool waiting = __ballot(pend_pm != 0u) != 0ull;
      if (waiting) queue_round();
      if (qcount >= kWave) {
        qcount -= kWave;
        evaluate_batch(q0 + qcount, kWave);
      }
      if (waiting) continue;
      if (gcount < kWave) break;
      adopt_threshold();
      // without any threshold every entry would pass: wait for one (another wave's, as a rule) as
      // long as the next tile's groups still fit
      if (theta <= kNoThreshold && gcount <= kQueueCap - kWave) break;
      gcount -= kWave;
      inspect_groups(q0 + gcount, kWave);
    }
  };

  // All waves of the workgroup move what they have queued (fewer than 64 entries each) to the pool
  // and share the level-2 work, 64 entries at a time, lanes fully used.  `which` names the pool's
  // counter (each is used once).  Ends with the threshold of all of it adopted.
  auto pool_evaluate = [&](int which) {
    int base = 0;
    if (lane == 0 && qcount > 0) base = atomicAdd(&sh_pool_n[which], qcount);
    base = __builtin_amdgcn_readfirstlane(base);
    if (lane < qcount) {
      sh_ent_v[kPool + base + lane] = sh_ent_v[q0 + lane];
      sh_ent_h[kPool + base + lane] = sh_ent_h[q0 + lane];
    }
    qcount = 0;
    lds_barrier();
    const int total = sh_pool_n[which];
    adopt_threshold();
    for (int b0 = wave * kWave; b0 < total; b0 += kWaves * kWave)
      evaluate_batch(kPool + b0, total - b0 < kWave ? total - b0 : kWave);
    lds_barrier();
    adopt_threshold();
  };

  // ---- the tiles of this chunk --------------------------------------------------------------------
  // kFast: rows that start on a 16-byte boundary and hold whole 16-byte vectors.  Their tile loads
  // are unconditional vector loads (addresses clamped to the chunk, what lies beyond its end is
  // masked after the load), so that the loads of the tiles ahead stay in flight while a tile is
  // worked on: the count of outstanding loads is then known at every point of the loop.  Other rows
  // are assembled from element loads.
  auto stream = [&](auto fast_tag) {
    constexpr bool kFast = decltype(fast_tag)::value;
    const int last_vec = v_end - kPer;
    auto load_tile = [&](uint4 (&raw)[kVecs], int tile_begin) {
#pragma unroll
      for (int k = 0; k < kVecs; ++k) {
        const int vb = tile_begin + lane_off + k * kPer;
        if (kFast) raw[k] = *reinterpret_cast<const uint4*>(trow + (vb < last_vec ? vb : last_vec));
        else raw[k] = load_raw(vb, v_end);
      }
    };
    // kDepth tiles are in flight per lane (eight 16-byte loads), requested before anything else
    // that depends on n.  The buffers are named apart and taken in turn: a copy from one to the
    // next would wait for the load it copies.
    constexpr int kDepth = 8 / kVecs;
    static_assert(kDepth == 4 || kDepth == 2, "tile buffers");
    uint4 raw0[kVecs], raw1[kVecs], raw2[kVecs], raw3[kVecs];
    load_tile(raw0, v_begin);
    // kHand: the workgroup starts on a chip that is running empty, not beside every other
    // workgroup of its kind: nothing is gained by holding the next tiles back until the first has
    // arrived, and their trip to memory is saved
    if (kHand) {
      load_tile(raw1, v_begin + kTile);
      if (kDepth == 4) {
        load_tile(raw2, v_begin + 2 * kTile);
        load_tile(raw3, v_begin + 3 * kTile);
      }
    }
    take_statistics();

    // One tile, first half: `raw` holds this lane's entries of the tile that starts at tile0 and is
    // refilled with those of the tile kDepth further on.  Leaves the entries with coarse byte 255
    // waiting for the level-2 queue and returns the lane's largest logit.
    auto tile_noise = [&](uint4 (&raw)[kVecs], int tile0, bool first) -> float {
      const int vbase = tile0 + lane_off;
      const Philox coarse = noise_block(seed, seq, pos, kDomainCoarse, (uint32_t)vbase >> 4);
      float l[kSampleLaneElems];
#pragma unroll
      for (int k = 0; k < kVecs; ++k) {
        float e[kPer];
        DT::unpack(raw[k], e);
#pragma unroll
        for (int j = 0; j < kPer; ++j) l[k * kPer + j] = e[j];
      }
      if (!first) load_tile(raw, tile0 + kDepth * kTile);
      if (kFast && tile0 > v_end - kTile) {  // uniform: the chunk's last, partial tile
#pragma unroll
        for (int j = 0; j < kSampleLaneElems; ++j) l[j] = vbase + j < v_end ? l[j] : -INFINITY;
      }
      // bit 7 of a byte of fl is set iff that byte of the noise word is 255
      uint32_t pm = 0u;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint32_t w = coarse.word(k);
        const uint32_t fl = ((w & 0x7F7F7F7Fu) + 0x01010101u) & w & 0x80808080u;
        pm |= fl >> (7 - k);
      }
      pend_pm = pm;
      pend_vb = vbase;
      pend_w0 = coarse.w0; pend_w1 = coarse.w1; pend_w2 = coarse.w2; pend_w3 = coarse.w3;
      float lmax = l[0];
#pragma unroll
      for (int j = 1; j < kSampleLaneElems; ++j) lmax = fmaxf(lmax, l[j]);
      return lmax;
    };

    // First tiles: a threshold before anything is tested against one.  Every wave draws the noise
    // of its first kDepth tiles as their data arrive and queues their entries with coarse byte 255;
    // those of all waves then go through level 2 together (a few hundred entries: a threshold
    // within a few units of the final one), and only then are the lanes' other entries of these
    // tiles tested.  That keeps the vector units busy while the first half of the row is on its way.
    // Memory serves a compute unit's requests in order, so the later tiles are only requested when
    // every wave's first tile has long been requested.
    {
      float lmax0, lmax1 = -INFINITY, lmax2 = -INFINITY, lmax3 = -INFINITY;
      lmax0 = tile_noise(raw0, v_begin, true);
      settle();
      __builtin_amdgcn_sched_barrier(0);
      if (!kHand) {
        load_tile(raw1, v_begin + kTile);
        if (kDepth == 4) {
          load_tile(raw2, v_begin + 2 * kTile);
          load_tile(raw3, v_begin + 3 * kTile);
        }
      }
      load_tile(raw0, v_begin + kDepth * kTile);
      __builtin_amdgcn_sched_barrier(0);
      if (v_begin + kTile < v_end) {
        lmax1 = tile_noise(raw1, v_begin + kTile, false);
        settle();
      }
      if (kDepth == 4 && v_begin + 2 * kTile < v_end) {
        lmax2 = tile_noise(raw2, v_begin + 2 * kTile, false);
        settle();
      }
      if (kDepth == 4 && v_begin + 3 * kTile < v_end) {
        lmax3 = tile_noise(raw3, v_begin + 3 * kTile, false);
        settle();
      }
      pool_evaluate(0);
      tile_groups(lmax0, v_begin);
      settle();
      tile_groups(lmax1, v_begin + kTile);
      settle();
      if (kDepth == 4) {
        tile_groups(lmax2, v_begin + 2 * kTile);
        settle();
        tile_groups(lmax3, v_begin + 3 * kTile);
        settle();
      }
    }
    // The other tiles, kDepth at a time, each from its own buffer.  Both queues hold at most 63 / 64
    // entries when a step that appends (at most 64) starts.
    for (int tile0 = v_begin + kDepth * kTile; tile0 < v_end; tile0 += kDepth * kTile) {
#pragma unroll
      for (int u = 0; u < kDepth; ++u) {
        const int t0 = tile0 + u * kTile;
        if (t0 < v_end) {  // uniform
          adopt_threshold();
          const float lmax = tile_noise(u == 0 ? raw0 : (u == 1 ? raw1 : (u == 2 ? raw2 : raw3)), t0, false);
          tile_groups(lmax, t0);
          settle();
        }
      }
    }
  };
  if (vector_ok && V % kPer == 0 && v_end - v_begin >= kPer) stream(std::true_type{});
  else stream(std::false_type{});

  // ---- no tiles left: this wave's queued groups, then the queued entries of all waves together -----
  while (gcount > 0) {
    adopt_threshold();
    const int cnt = gcount < kWave ? gcount : kWave;
    gcount -= cnt;
    inspect_groups(q0 + gcount, cnt);
    settle();
  }
  pool_evaluate(2);
  compact_survivors();
  publish_threshold();

  // ---- merge the waves' survivors into the workgroup's records -------------------------------------
  // The waves share their level-2 work, so a wave's survivors come from anywhere in the
  // workgroup's range: they fill the workgroup's G records one after the other, and what neither a
  // wave nor the records could hold makes every one of them say "overflow" (the exact choice then
  // scans the whole range).
  lds_barrier();
  // every wave of the workgroup has published its last threshold: this is the workgroup's
  const float theta_wg = ordered_float(sh_theta_row);
  uint32_t* rec0 = p.records + ((size_t)b * p.S + (s - g)) * kRecordWords;  // the first of the G records
  // records that another workgroup will read (the one that finishes the row last) are written
  // with coherent stores; those of a workgroup that chooses by itself with ordinary ones
  auto put = [](uint32_t* ptr, uint32_t v) {
    if (kFused) *ptr = v;
    else coherent_store(ptr, v);
  };
  {
    const bool have = lane < scount;
    const int v = have ? sh_surv_v[wave][lane] : 0;
    const float su = have ? sh_surv_s[wave][lane] : -INFINITY;
    const bool keep = have && su >= theta_wg;
    const unsigned long long km = __ballot(keep);
    int base = 0;
    if (lane == 0 && km != 0ull) base = atomicAdd(&sh_count_g[0], __popcll(km));
    base = __shfl(base, 0, 64);
    if (keep) {
      const int slot = base + lanes_below(km);
      if (slot < G * kRecordCap) {
        uint32_t* rec = rec0 + (slot / kRecordCap) * kRecordWords;
        put(rec + 2 + 2 * (slot % kRecordCap), (uint32_t)v);
        put(rec + 3 + 2 * (slot % kRecordCap), __float_as_uint(su));
      }
      if (kFused) sh_only = v;
    }
    if (overflow && lane == 0) sh_overflow_g[0] = 1;
  }
  lds_barrier();
  const int total = sh_count_g[0];
  const bool any_overflow = sh_overflow_g[0] != 0 || total > G * kRecordCap;
  if (tid == 0) {
    uint32_t* rec = rec0 + g * kRecordWords;
    const int mine = total - g * kRecordCap;
    put(rec, __float_as_uint(theta_wg));
    put(rec + 1, any_overflow ? (uint32_t)kRecordOverflow
                              : (uint32_t)(mine < 0 ? 0 : (mine > kRecordCap ? kRecordCap : mine)));
  }
  if (kFused) {
    // exactly one entry of the whole row survived: it is the winner, nothing to compare it with
    const bool separable = theta_wg > (residual ? kDegenerate : kNoThreshold);
    if (separable && !any_overflow && total == 1) {
      if (threadIdx.x == 0) p.out_tokens[r0 + b + n] = sh_only;
      return true;
    }
  }
  return false;
}

// Level 3.  One workgroup per sequence reads the chunk records of the filter kernel.  A single
// survivor is the winner as it stands; several are scored in fp64 by the definition; rows the
// bounds could not separate are scanned in fp64.  In the common case everything this kernel needs
// (accept length, chunk headers, survivor entries) is requested in one round of loads.
// n is the sequence's accept length.  kCoherent: the records come from other workgroups of the
// running kernel, which have counted in since (arrive_is_last).  kHand: so do the statistics.
template <typename DT, bool kCoherent, bool kHand = false>
__device__ __forceinline__ void select_body(const Problem& p, int b, int n) {
  using storage = typename DT::storage;
  __shared__ float sh_theta[kWavesPerBlock];
  __shared__ int sh_any_overflow, sh_total, sh_only;
  const int tid = (int)threadIdx.x;
  const int V = p.V;
  const uint32_t* recs = p.records + (size_t)b * p.S * kRecordWords;
  const int total = p.S * kRecordCap;
  auto rd = [](const uint32_t* ptr) -> uint32_t { return kCoherent ? coherent_load(ptr) : *ptr; };

  // ---- one round of loads ---------------------------------------------------------------------
  const int64_t r0 = seq_row_begin(p, b);
  const int Kb = seq_len(p, b);
  float th = kNoThreshold;
  bool ovf = false;
  for (int i = tid; i < p.S; i += kBlock) {
    th = fmaxf(th, __uint_as_float(rd(recs + (size_t)i * kRecordWords)));
    ovf = ovf || (int)rd(recs + (size_t)i * kRecordWords + 1) == kRecordOverflow;
  }
  // this thread's survivor entry (further entries, for rows split into many chunks, come later)
  int e_cnt = 0, e_j = 0, e_v = -1;
  float e_s = -INFINITY;
  if (tid < total) {
    const int i = tid / kRecordCap;
    e_j = tid - i * kRecordCap;
    const uint32_t* rc = recs + (size_t)i * kRecordWords;
    e_cnt = (int)rd(rc + 1);
    e_v = (int)rd(rc + 2 + 2 * e_j);
    e_s = __uint_as_float(rd(rc + 3 + 2 * e_j));
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
      if (is_survivor((int)rd(rc + 1), j, __uint_as_float(rd(rc + 3 + 2 * j)))) { ++mine; my_v = (int)rd(rc + 2 + 2 * j); }
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
  if (kHand) {
    ctx.mt = residual ? (double)coherent_load(p.m + 2 * r) : 0.0;
    ctx.Zt = residual ? coherent_load(p.Z + 2 * r) : 1.0;
    ctx.md = residual ? (double)coherent_load(p.m + 2 * r + 1) : 0.0;
    ctx.Zd = residual ? coherent_load(p.Z + 2 * r + 1) : 1.0;
  } else {
    ctx.mt = residual ? (double)p.m[2 * r] : 0.0;
    ctx.Zt = residual ? p.Z[2 * r] : 1.0;
    ctx.md = residual ? (double)p.m[2 * r + 1] : 0.0;
    ctx.Zd = residual ? p.Z[2 * r + 1] : 1.0;
  }
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
      if (is_survivor((int)rd(rc + 1), j, __uint_as_float(rd(rc + 3 + 2 * j)))) {
        const int v = (int)rd(rc + 2 + 2 * j);
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
        if ((int)rd(recs + (size_t)i * kRecordWords + 1) == kRecordOverflow) {
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

// Rows split into more than two chunks: one workgroup per chunk, and the workgroup that finishes a
// row's last chunk goes on to the exact choice among the records of all of them.
template <typename DT, bool kLate>
__global__ __launch_bounds__(kBlock) void sample_kernel(Problem p) {
  __shared__ int sh_last;
  int n;
  (void)sample_body<DT, 1, kLate, false>(p, n, blockIdx.x);
  const int b = (int)(blockIdx.x / (unsigned)p.S);
  if (!arrive_is_last(p.arrive + b, (uint32_t)p.S, &sh_last)) return;
  select_body<DT, true>(p, b, n);
}

// Filter and exact choice in one launch, for rows that are split into G <= 2 chunks: a workgroup of
// G * 512 threads filters all chunks of its row, then its first 512 threads read the records it
// has just written (visible within the workgroup after the barrier) and choose.  Saves a launch
// and the dependent start of a second kernel.  Registers: the single-chunk bf16 variant is held to
// 80 (three 512-thread groups per CU, as the filter alone); the others run one or two groups per
// CU whatever they use.
template <typename DT, int G, bool kLate>
__global__ __launch_bounds__(kBlock* G, 4)
void sample_select_kernel(Problem p) {
  int n;
  if (sample_body<DT, G, kLate, true>(p, n, blockIdx.x)) return;  // uniform over the workgroup
  __syncthreads();
  if ((int)threadIdx.x >= kBlock) return;  // whole waves
  select_body<DT, false>(p, (int)blockIdx.x, n);
}

}  // namespace ears
