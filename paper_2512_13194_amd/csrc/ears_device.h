// Device-side building blocks of the EARS verification kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ears {

constexpr int kWave = 64;
constexpr int kBlock = 512;             // threads per workgroup: 8 waves
constexpr int kWavesPerBlock = kBlock / kWave;

constexpr double kLog2e = 1.4426950408889634074;
constexpr double kEpsilon = 1e-10;      // division guard of the paper's Section 3.3 item 2

// Sampling stage: each workgroup filters one chunk of a row and leaves a record of
// kRecordWords 32-bit words: [0] threshold (float bits), [1] survivor count or kRecordOverflow,
// then kRecordCap pairs (vocabulary index, upper score bound as float bits).
constexpr int kRecordCap = 48;
constexpr int kRecordWords = 2 + 2 * kRecordCap + 2;
constexpr int kRecordOverflow = -1;
// The filter hands each lane 16 consecutive vocabulary entries per tile (one coarse Philox block).
constexpr int kSampleLaneElems = 16;
constexpr int kSampleTileElems = kBlock * kSampleLaneElems;

// Everything a kernel needs to locate its rows.  Rectangular batches have row_offsets == nullptr:
// sequence b then owns draft rows b*K .. b*K+K-1.  In both layouts draft row r of sequence b
// pairs with target row r + b (every earlier sequence has one extra, "bonus", target row).
struct Problem {
  const void* target;
  const void* draft;
  const int32_t* tokens;
  const int64_t* row_offsets;
  int64_t R;  // packed draft rows
  int B;
  int K;
  int V;
  float T;
  float beta;
  const float* T_seq;
  const float* beta_seq;
  uint64_t seed;
  const int64_t* seq_ids;
  // cached row statistics, index 2*r + which (0 target, 1 draft)
  double* Z;
  float* m;
  float* lx;
  double* unc;          // [R] uncertainty of the alternative measures (when unc_mode != 0)
  uint32_t* unc_tag;    // [1] which measure unc[] holds: written by whoever fills the statistics
  int unc_mode;         // 0: 1 - max p_t, 1: normalised entropy, 2: total variance
  int32_t* decisions;   // [R] per position: 0 reject, 1 primary accept, 2 accepted by tolerance
  // sampling stage scratch: per-chunk records
  uint32_t* records;    // [B, S, kRecordWords]
  int S;                // chunks per row
  int chunk;            // vocabulary entries per chunk (a multiple of the tile size)
  int decide_fused;     // where the filter kernel finds the accept length: 0 in accept_len (an earlier
                        // DECIDE stage left it), 1 by scanning the decisions the statistics kernel
                        // left, 2 by deciding each position itself from the cached statistics
  uint32_t* arrive;     // [B] "last one out" words (see arrive_is_last), zero between calls
  uint32_t* ready;      // [R] single-launch calls: ready[r] == tag | decision once position r's
                        // statistics are in memory (see verify_kernel); zero between calls
  uint32_t tag;         // this call's value for ready[]: never zero, its two lowest bits clear
  int await_polls;      // how often a sampling workgroup of a single-launch call polls before it gives up
  // outputs
  int32_t* accept_len;
  int32_t* out_tokens;
  double* out_stats;
  int32_t* out_path;
  uint32_t* status_word;
};

__device__ __forceinline__ int seq_of_row(const Problem& p, int64_t r) {
  if (p.row_offsets == nullptr) return (int)(r / p.K);
  int lo = 0, hi = p.B;  // invariant: off[lo] <= r < off[hi]
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (p.row_offsets[mid] <= r) lo = mid; else hi = mid;
  }
  return lo;
}

__device__ __forceinline__ int64_t seq_row_begin(const Problem& p, int b) {
  return p.row_offsets ? p.row_offsets[b] : (int64_t)b * p.K;
}
__device__ __forceinline__ int seq_len(const Problem& p, int b) {
  return p.row_offsets ? (int)(p.row_offsets[b + 1] - p.row_offsets[b]) : p.K;
}
// Per-sequence parameters come from device memory and cannot be checked on the host: a
// temperature that is not a positive finite number is replaced by 1, a beta that is negative or
// not finite by 0 (so that the sequence's arithmetic stays finite), and the statistics / decision
// stage raises status bit 3.
__device__ __forceinline__ float seq_temperature(const Problem& p, int b) {
  const float T = p.T_seq ? p.T_seq[b] : p.T;
  return (T > 0.0f && T < INFINITY) ? T : 1.0f;
}
__device__ __forceinline__ float seq_beta(const Problem& p, int b) {
  const float beta = p.beta_seq ? p.beta_seq[b] : p.beta;
  return (beta >= 0.0f && beta < INFINITY) ? beta : 0.0f;
}
__device__ __forceinline__ bool seq_params_invalid(const Problem& p, int b) {
  const float T = p.T_seq ? p.T_seq[b] : p.T;
  const float beta = p.beta_seq ? p.beta_seq[b] : p.beta;
  return !(T > 0.0f && T < INFINITY) || !(beta >= 0.0f && beta < INFINITY);
}
__device__ __forceinline__ uint64_t seq_rng_id(const Problem& p, int b) {
  return p.seq_ids ? (uint64_t)p.seq_ids[b] : (uint64_t)b;
}

// ---- logits --------------------------------------------------------------------------------
// 16-byte load of data that is read once: the non-temporal hint keeps the stream from displacing
// other lines in the caches, which on this part is worth more than a tenth of the read bandwidth.
__device__ __forceinline__ uint4 load_stream(const uint4* ptr) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(ptr));
  return make_uint4(v.x, v.y, v.z, v.w);
}

struct F32 {
  using storage = float;
  static constexpr int kPerVec = 4;  // elements in one 16-byte load
  static __device__ __forceinline__ float load(const void* base, int64_t i) {
    return static_cast<const float*>(base)[i];
  }
  static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[4]) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
  static __device__ __forceinline__ uint4 neg_inf_vec() {
    return make_uint4(0xFF800000u, 0xFF800000u, 0xFF800000u, 0xFF800000u);
  }
};

struct BF16 {
  using storage = uint16_t;
  static constexpr int kPerVec = 8;
  static __device__ __forceinline__ float load(const void* base, int64_t i) {
    return __uint_as_float((uint32_t)static_cast<const uint16_t*>(base)[i] << 16);
  }
  // a dword holds two bf16: the low half is the element with the lower index
  static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[8]) {
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xFFFF0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xFFFF0000u);
  }
  static __device__ __forceinline__ uint4 neg_inf_vec() {
    return make_uint4(0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u);
  }
};

// ---- Philox4x32-10 (Salmon et al., SC'11) ----------------------------------------------------
// Ten rounds; each multiplies counter words 0 and 2 by fixed odd constants and mixes the high
// halves with the other words and the round key, which advances by two Weyl constants.
struct Philox {
  uint32_t w0, w1, w2, w3;
  __device__ __forceinline__ uint32_t word(int i) const {  // i is a compile-time constant at every use
    return i == 0 ? w0 : (i == 1 ? w1 : (i == 2 ? w2 : w3));
  }
};

__device__ __forceinline__ Philox philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int i = 0; i < 10; ++i) {
    const uint64_t a = (uint64_t)0xD2511F53u * c0;
    const uint64_t b = (uint64_t)0xCD9E8D57u * c2;
    // three-way exclusive or in one instruction (truth table 0x96)
    const uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(b >> 32), c1, k0, 0x96);
    const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(a >> 32), c3, k1, 0x96);
    c1 = (uint32_t)b;
    c3 = (uint32_t)a;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return Philox{c0, c1, c2, c3};
}

// counter = (block, position, seq low 32, domain << 24 | seq bits 32..55); key = seed halves.
// domain 0: acceptance uniform (block 0, word 0);
// domain 1: coarse Gumbel bits, block = v >> 4, one byte per vocabulary entry (word (v >> 2) & 3,
//           byte v & 3, byte k = bits 8k..8k+7);
// domain 2: fine Gumbel bits, block = v >> 2, word = v & 3.
// The Gumbel uniform of entry v is u = (h + (f + 1/2) * 2^-32) * 2^-8, h the coarse byte and f the
// fine word: the byte alone bounds -log(-log u) from above, which is all the filter needs for
// almost every entry.
__device__ __forceinline__ Philox noise_block(uint64_t seed, uint64_t seq, uint32_t pos,
                                              uint32_t domain, uint32_t blk) {
  return philox4x32_10(blk, pos, (uint32_t)seq, (domain << 24) | ((uint32_t)(seq >> 32) & 0xFFFFFFu),
                       (uint32_t)seed, (uint32_t)(seed >> 32));
}

// Acceptance uniform U in [0,1) on a 2^-24 grid (exact in fp32).
__device__ __forceinline__ double accept_uniform(uint64_t seed, uint64_t seq, uint32_t pos) {
  return (double)(noise_block(seed, seq, pos, 0u, 0u).w0 >> 8) * 0x1p-24;
}
constexpr uint32_t kDomainAccept = 0u, kDomainCoarse = 1u, kDomainFine = 2u;

// Workgroup barrier that orders LDS accesses only.  __syncthreads() also waits for every global
// load the wave has in flight, which stalls a wave that keeps loads of later data outstanding.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---- last one out ----------------------------------------------------------------------------
// Workgroups that each finish one part of a piece of work (the chunks of a row) count in on a word
// in device memory, and the one that completes the count goes on with what needs all the parts.
// Nobody waits for anybody: every workgroup either leaves or carries on.  The word is zero when
// the first part arrives: whatever fills a workspace with statistics (the statistics kernel, the
// import of a producer's statistics) zeroes the words first, and the last to arrive puts the zero
// back for the next call.
//
// What the parts hand over is a few words, and those are written with coherent_store and read
// with coherent_load (device-scope atomic accesses: they go to the memory side of the caches).
// A device-scope release fence would order ordinary stores as well, but it writes back the whole
// L2 of the workgroup's XCD, once per workgroup: measured, that cost more than the launch it was
// to save.  Here every wave waits until its own coherent stores have been acknowledged
// (wait_for_own_stores), the workgroup meets at a barrier, and only then its first thread counts
// in; the last one reads after its count has returned.
__device__ __forceinline__ void wait_for_own_stores() {
  // vmcnt(0): every vector-memory access this wave has issued, stores included, has been
  // acknowledged.  (A workgroup barrier alone does not wait for them on this target: the waves of
  // a workgroup share their CU's cache, so the compiler leaves the wait out of the barrier's
  // workgroup-scope fence.)
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0x0F70);
}

// Called by every thread of the workgroup; returns true in all of them or in none.
__device__ __forceinline__ bool arrive_is_last(uint32_t* word, uint32_t parts, int* sh_flag) {
  wait_for_own_stores();
  __syncthreads();  // every wave's stores have completed
  if (threadIdx.x == 0) {
    const uint32_t before = __hip_atomic_fetch_add(word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const bool last = before + 1u >= parts;
    if (last) __hip_atomic_store(word, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *sh_flag = last ? 1 : 0;
  }
  __syncthreads();
  return *sh_flag != 0;
}

__device__ __forceinline__ uint32_t coherent_load(const uint32_t* ptr) {
  return __hip_atomic_load(ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void coherent_store(uint32_t* ptr, uint32_t v) {
  __hip_atomic_store(ptr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float coherent_load(const float* ptr) {
  return __hip_atomic_load(ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double coherent_load(const double* ptr) {
  return __hip_atomic_load(ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int32_t coherent_load(const int32_t* ptr) {
  return __hip_atomic_load(ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void coherent_store(float* ptr, float v) {
  __hip_atomic_store(ptr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void coherent_store(double* ptr, double v) {
  __hip_atomic_store(ptr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void coherent_store(int32_t* ptr, int32_t v) {
  __hip_atomic_store(ptr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- wave64 all-reduce through DPP / swizzle / permlane ---------------------------------------
// After the call every lane of the wave holds the reduction.  Steps: xor 1 and xor 2 inside a
// quad (quad_perm), then mirror inside 8 and 16 lanes (row_half_mirror, row_mirror; valid because
// the earlier steps made each quad / half-row uniform), then swap 16-lane rows inside each half
// (ds_swizzle) and finally the two halves (a cross-lane shuffle).
template <int kCtrl>
__device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), kCtrl, 0xF, 0xF, false));
}
__device__ __forceinline__ float swap_rows16_f32(float v) {
  // ds_swizzle bit-mask mode: and_mask 0x1F, or_mask 0, xor_mask 0x10 -> lane ^ 16 within 32 lanes
  return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(v), 0x401F));
}
__device__ __forceinline__ float swap_halves_f32(float v) {
  return __shfl_xor(v, 32, 64);
}

constexpr int kDppQuadXor1 = 0xB1;       // quad_perm [1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;       // quad_perm [2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowMirror = 0x140;

__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_f32<kDppQuadXor1>(v));
  v = fmaxf(v, dpp_f32<kDppQuadXor2>(v));
  v = fmaxf(v, dpp_f32<kDppRowHalfMirror>(v));
  v = fmaxf(v, dpp_f32<kDppRowMirror>(v));
  v = fmaxf(v, swap_rows16_f32(v));
  v = fmaxf(v, swap_halves_f32(v));
  return v;
}

template <int kCtrl>
__device__ __forceinline__ double dpp_f64(double v) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __builtin_amdgcn_update_dpp(0, lo, kCtrl, 0xF, 0xF, false);
  hi = __builtin_amdgcn_update_dpp(0, hi, kCtrl, 0xF, 0xF, false);
  return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double swap_rows16_f64(double v) {
  int lo = __builtin_amdgcn_ds_swizzle(__double2loint(v), 0x401F);
  int hi = __builtin_amdgcn_ds_swizzle(__double2hiint(v), 0x401F);
  return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double wave_sum(double v) {
  v += dpp_f64<kDppQuadXor1>(v);
  v += dpp_f64<kDppQuadXor2>(v);
  v += dpp_f64<kDppRowHalfMirror>(v);
  v += dpp_f64<kDppRowMirror>(v);
  v += swap_rows16_f64(v);
  v += __shfl_xor(v, 32, 64);
  return v;
}

// (score, index) argmax: larger score wins, equal scores go to the lower index.
struct Best {
  double s;
  int32_t v;
};
__device__ __forceinline__ bool better(double s, int32_t v, const Best& o) {
  return o.v < 0 || (v >= 0 && (s > o.s || (s == o.s && v < o.v)));
}
__device__ __forceinline__ Best wave_best(Best x) {
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    Best o;
    o.s = __shfl_xor(x.s, d, 64);
    o.v = __shfl_xor(x.v, d, 64);
    if (better(o.s, o.v, x)) x = o;
  }
  return x;
}

}  // namespace ears
