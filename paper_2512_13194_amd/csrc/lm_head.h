// Producer-side fusion (paper Section 3.3 item 1 has the statistics computed right behind the target
// model's forward pass): the vocabulary projection logits[n, v] = sum_k hidden[n, k] *
// weight[v, k] on the matrix cores, whose epilogue rounds the logits to bf16, takes the softmax
// statistics (row maximum, sum of exponentials) of the rounded values while they are still in
// registers, and writes the logits once.  The verification step then starts from cached statistics
// and never re-reads the logits for them.
//
// One workgroup (8 waves, two per SIMD) computes a 256 (vocabulary) x 256 (tokens) tile; each wave
// owns 128 x 64 as 4 x 2 blocks of v_mfma_f32_32x32x16_bf16 (128 accumulator registers, so that two
// waves fit a SIMD's register file) with the vocabulary on the MFMA's row index: a lane's 16
// accumulator registers of a block are 16 vocabulary entries of ONE token and the statistics start
// as in-lane reductions.
#pragma once

#include "ears_device.h"

namespace ears {

constexpr int kLmTile = 256;          // tile edge, vocabulary and tokens
constexpr int kLmBK = 64;             // depth of one staged slab (bf16 elements): 128 bytes per row
constexpr int kLmThreads = 512;       // 8 waves as 2 (vocabulary) x 4 (tokens)
constexpr int kLmWaveV = 128;         // wave tile along the vocabulary: 4 MFMA blocks
constexpr int kLmWaveN = 64;          // wave tile along the tokens: 2 MFMA blocks
constexpr int kLmStageRow = kLmTile * 2 + 8;                 // epilogue staging: 520-byte token rows
// Four shared arrays: operand A and B of the two slab buffers (32 KiB of each are slab data).  The
// epilogue reuses them to stage 64 token rows each, hence the 520-byte rows' worth of size.
constexpr int kLmArrayBytes = 64 * kLmStageRow;              // 33 280 B
constexpr int kLmWeightPolicy = 2;    // weights stream through once per XCD: non-temporal
constexpr int kLmHiddenPolicy = 0;    // hidden states are re-read by every vocabulary tile
constexpr int kLmPartsPerTile = 2;                           // one partial per wave row of a tile

struct LmHeadProblem {
  const uint16_t* hidden;   // [N, D] bf16
  const uint16_t* weight;   // [V, D] bf16
  const float* row_T;       // [N] per-row temperature or nullptr
  float T;
  int N, D, V;
  int n_vtiles, n_ttiles;   // tiles along the vocabulary and along the tokens
  uint16_t* logits;         // [N, V] bf16
  float* part_m;            // [N, nparts] maximum of the rounded logits of one 128-entry slice
  float* part_S;            // [N, nparts] sum of e = exp2(y), y = l*c - fl(m*c), over the slice
  float* part_W;            // [N, nparts] sum of e*y over the slice (for the entropy)
  int nparts;               // 2 * n_vtiles
  float* row_m;             // [N]
  double* row_Z;            // [N]
  double* row_H;            // [N] Shannon entropy (nats) of softmax(row / T), or nullptr
};

typedef __bf16 lm_bf16x8 __attribute__((ext_vector_type(8)));
typedef float lm_f32x16 __attribute__((ext_vector_type(16)));

// 16-byte chunk c (0..7) of slab row `row` lives at chunk position c ^ swizzle(row): 8 or 16
// consecutive rows then spread over all banks for both the 16-byte fragment reads and the writes.
__device__ __forceinline__ int lm_swizzle(int row) { return (row & 7) ^ ((row >> 3) & 1); }

__device__ __forceinline__ uint16_t lm_round_bf16(float x) {
  return __builtin_bit_cast(uint16_t, (__bf16)x);  // round to nearest even
}

// Slab loads go straight from global memory to LDS (16 bytes per lane, lane i of a wave lands at
// base + 16 i): one instruction fills 8 slab rows.  Wave w, instruction j fills rows 64 j + 8 w ..
// + 8; lane i supplies the chunk that belongs at position (i & 7) of row (i >> 3) under the swizzle.
// Buffer addressing: the operand is a raw buffer (base and byte size in a scalar descriptor), a lane
// adds its own 32-bit byte offset and the instruction a scalar one (slab and row block), so the
// loop needs no address arithmetic; rows past the end of the matrix fall outside the buffer and
// read as zero.  kAux is the cache-policy operand of the load: 0 default, 2 non-temporal.
template <int kAux>
__device__ __forceinline__ void lm_issue_slab(unsigned char* dst, __amdgpu_buffer_rsrc_t rsrc,
                                              uint32_t lane_off, uint32_t slab_off,
                                              uint32_t block_stride, int wave) {
#pragma unroll
  for (int j = 0; j < 4; ++j)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, dst + (64 * j + 8 * wave) * (kLmBK * 2), 16,
                                             lane_off, slab_off + (uint32_t)j * block_stride, 0, kAux);
}

// Fragments of one k-step: 4 blocks of vocabulary rows (A) and 2 blocks of token rows (B).
struct LmFrags {
  lm_bf16x8 a[4], b[2];
};
__device__ __forceinline__ void lm_read_frags(LmFrags& f, const unsigned char* sA,
                                              const unsigned char* sB, int off) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
    f.a[i] = *reinterpret_cast<const lm_bf16x8*>(sA + off + i * 32 * (kLmBK * 2));
#pragma unroll
  for (int j = 0; j < 2; ++j)
    f.b[j] = *reinterpret_cast<const lm_bf16x8*>(sB + off + j * 32 * (kLmBK * 2));
}

// One slab: 4 k-steps of 16.  `f0` already holds the fragments of step 0; the fragments of the next
// step are read while the current step's 8 MFMAs issue.
__device__ __forceinline__ void lm_compute_slab(LmFrags& f0, const unsigned char* sA,
                                                const unsigned char* sB, const int (&fr_off)[4],
                                                lm_f32x16 (&acc)[4][2]) {
  LmFrags f1;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    LmFrags& cur = (s & 1) ? f1 : f0;
    LmFrags& nxt = (s & 1) ? f0 : f1;
    if (s + 1 < 4) lm_read_frags(nxt, sA, sB, fr_off[s + 1]);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur.a[i], cur.b[j], acc[i][j], 0, 0, 0);
  }
}

// all of this wave's direct-to-LDS loads have landed; then every wave's
__device__ __forceinline__ void lm_slab_ready() {
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), other counters untouched
  __syncthreads();
}

__global__ __launch_bounds__(kLmThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void lm_head_kernel(LmHeadProblem p) {
  __shared__ __attribute__((aligned(16))) unsigned char s_a0[kLmArrayBytes];
  __shared__ __attribute__((aligned(16))) unsigned char s_b0[kLmArrayBytes];
  __shared__ __attribute__((aligned(16))) unsigned char s_a1[kLmArrayBytes];
  __shared__ __attribute__((aligned(16))) unsigned char s_b1[kLmArrayBytes];

  // Workgroup ids go round-robin over the 8 XCDs.  The token tiles that share a vocabulary tile
  // (hence the same weight rows) get consecutive ids on ONE XCD, so the weights reach each L2 once.
  const int id = (int)blockIdx.x;
  const int xcd = id & 7, local = id >> 3;
  const int vt = (local / p.n_ttiles) * 8 + xcd;
  const int tt = local % p.n_ttiles;
  if (vt >= p.n_vtiles) return;  // uniform over the workgroup
  const int v0 = vt * kLmTile, n0 = tt * kLmTile;

  const int tid = (int)threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform, and known to be
  const int wv = wave >> 2, wn = wave & 3;  // wave's 128-slice of the vocabulary / 64-slice of the tokens

  // ---- global -> LDS: this lane's chunk of rows ld_row + 64 j of both operands ----
  const int ld_row = 8 * wave + (lane >> 3);
  const uint32_t ld_chunk_off = (uint32_t)(((lane & 7) ^ lm_swizzle(ld_row)) * 16);
  const uint32_t row_bytes = (uint32_t)(p.D * 2);
  const uint32_t block_stride = 64u * row_bytes;
  const uint32_t offA = (uint32_t)ld_row * row_bytes + ld_chunk_off;
  const uint32_t offB = offA;
  // Raw buffer descriptors (stride 0, 32-bit data format) over this tile's rows only: the base is
  // the tile's first row (64-bit), the extent its rows that exist, so the 32-bit offsets never see
  // the size of the whole matrix and rows past its end read as zero.
  const int rows_a = p.V - v0 < kLmTile ? p.V - v0 : kLmTile;
  const int rows_b = p.N - n0 < kLmTile ? p.N - n0 : kLmTile;
  const __amdgpu_buffer_rsrc_t rA = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(p.weight) + (size_t)v0 * (size_t)p.D, 0, (int)((uint32_t)rows_a * row_bytes),
      0x00020000);
  const __amdgpu_buffer_rsrc_t rB = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(p.hidden) + (size_t)n0 * (size_t)p.D, 0, (int)((uint32_t)rows_b * row_bytes),
      0x00020000);

  // ---- fragment reads: lane supplies row (lane & 31), k-offset 8 * (lane >> 5) of each block ----
  const int fr_swz = lm_swizzle(lane & 31);
  int fr_off[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) fr_off[s] = (lane & 31) * (kLmBK * 2) + (((2 * s + (lane >> 5)) ^ fr_swz) << 4);
  const int fr_A = wv * kLmWaveV * (kLmBK * 2);
  const int fr_B = wn * kLmWaveN * (kLmBK * 2);

  lm_f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // Two slab buffers in separate arrays: the loads of slab s + 1 are in flight while slab s is
  // multiplied; the barrier that ends slab s also says that everyone is done reading it.
  const int n_slabs = p.D / kLmBK;
  const uint32_t slab_bytes = kLmBK * 2;
  lm_issue_slab<kLmWeightPolicy>(s_a0, rA, offA, 0u, block_stride, wave);
  lm_issue_slab<kLmHiddenPolicy>(s_b0, rB, offB, 0u, block_stride, wave);
  lm_slab_ready();
  LmFrags f0;
  for (int slab = 0; slab < n_slabs; slab += 2) {
    // the first fragments of the slab are asked for before the next slab's loads are issued
    lm_read_frags(f0, s_a0 + fr_A, s_b0 + fr_B, fr_off[0]);
    if (slab + 1 < n_slabs) {  // uniform
      lm_issue_slab<kLmWeightPolicy>(s_a1, rA, offA, (uint32_t)(slab + 1) * slab_bytes, block_stride, wave);
      lm_issue_slab<kLmHiddenPolicy>(s_b1, rB, offB, (uint32_t)(slab + 1) * slab_bytes, block_stride, wave);
    }
    lm_compute_slab(f0, s_a0 + fr_A, s_b0 + fr_B, fr_off, acc);
    lm_slab_ready();
    if (slab + 1 < n_slabs) {
      lm_read_frags(f0, s_a1 + fr_A, s_b1 + fr_B, fr_off[0]);
      if (slab + 2 < n_slabs) {
        lm_issue_slab<kLmWeightPolicy>(s_a0, rA, offA, (uint32_t)(slab + 2) * slab_bytes, block_stride, wave);
        lm_issue_slab<kLmHiddenPolicy>(s_b0, rB, offB, (uint32_t)(slab + 2) * slab_bytes, block_stride, wave);
      }
      lm_compute_slab(f0, s_a1 + fr_A, s_b1 + fr_B, fr_off, acc);
      lm_slab_ready();
    }
  }

  // ---- epilogue ------------------------------------------------------------------------------
  // acc[i][j][r] is vocabulary entry v0 + wv*128 + i*32 + 8*(r/4) + 4*(lane/32) + r%4 of token
  // n0 + wn*64 + j*32 + lane%32.  Round, take the statistics of the rounded values, stage the
  // tile as [token][vocabulary] rows and write them out whole.
  const int half = lane >> 5;
  // 64 token rows per shared array: the wave's tokens are rows 0..63 of array wn
  unsigned char* stage_array = wn == 0 ? s_a0 : wn == 1 ? s_b0 : wn == 2 ? s_a1 : s_b1;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int tok_local = wn * kLmWaveN + j * 32 + (lane & 31);
    const int tok = n0 + tok_local;
    unsigned char* stage = stage_array + (j * 32 + (lane & 31)) * kLmStageRow;
    const float T = p.row_T ? p.row_T[tok < p.N ? tok : p.N - 1] : p.T;
    const float c = (float)(kLog2e / (double)T);
    float xr[4][16];
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int v_local = wv * kLmWaveV + i * 32 + 8 * g + 4 * half;
        uint16_t b[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          b[q] = lm_round_bf16(acc[i][j][4 * g + q]);
          const float x = __uint_as_float((uint32_t)b[q] << 16);
          const bool valid = v0 + v_local + q < p.V;
          xr[i][4 * g + q] = valid ? x : -INFINITY;
          m = fmaxf(m, xr[i][4 * g + q]);
        }
        uint2 packed;
        packed.x = (uint32_t)b[0] | ((uint32_t)b[1] << 16);
        packed.y = (uint32_t)b[2] | ((uint32_t)b[3] << 16);
        *reinterpret_cast<uint2*>(stage + v_local * 2) = packed;
      }
    }
    // the other half-wave holds the other 64 entries of the same token's 128-slice
    m = fmaxf(m, __shfl_xor(m, 32, 64));
    // 16 short fp32 sums of 4 terms each, combined in fp64: the slice that holds a row's dominant
    // entry (one term of 1 beside terms near 1e-8) then loses at most three small terms to ulp(1)
    double S = 0.0, W = 0.0;
    if (m != -INFINITY) {
      const float mc = m * c;
      float s16[16], w16[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) s16[r] = w16[r] = 0.0f;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float y = fmaxf(fmaf(xr[i][r], c, -mc), -126.0f);  // a masked entry adds 0 * finite
          const float e = __builtin_amdgcn_exp2f(y);
          s16[r] += e;
          w16[r] = fmaf(e, y, w16[r]);
        }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        S += (double)s16[r];
        W += (double)w16[r];
      }
    }
    S += __shfl_xor(S, 32, 64);
    W += __shfl_xor(W, 32, 64);
    if (half == 0 && tok < p.N) {
      const size_t slot = (size_t)tok * p.nparts + vt * kLmPartsPerTile + wv;
      p.part_m[slot] = m;
      p.part_S[slot] = (float)S;
      p.part_W[slot] = (float)W;
    }
  }
  __syncthreads();
  // whole rows out: a wave writes one 512-byte token row per instruction (8 bytes per lane)
  const int v_lane = v0 + lane * 4;
  for (int row = wave; row < kLmTile; row += kLmThreads / 64) {
    const int tok = n0 + row;
    if (tok >= p.N) break;  // uniform over the wave
    const unsigned char* stage_array = (row >> 6) == 0 ? s_a0 : (row >> 6) == 1 ? s_b0
                                       : (row >> 6) == 2 ? s_a1 : s_b1;
    const uint2 val = *reinterpret_cast<const uint2*>(stage_array + (row & 63) * kLmStageRow + lane * 8);
    uint16_t* dst = p.logits + (size_t)tok * p.V + v_lane;
    if (v_lane + 3 < p.V && ((reinterpret_cast<uintptr_t>(dst) & 7u) == 0)) {
      *reinterpret_cast<uint2*>(dst) = val;
    } else {
      const uint16_t e[4] = {(uint16_t)(val.x & 0xFFFFu), (uint16_t)(val.x >> 16),
                             (uint16_t)(val.y & 0xFFFFu), (uint16_t)(val.y >> 16)};
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (v_lane + q < p.V) dst[q] = e[q];
    }
  }
}

// Merges the per-slice partials of one token row with the associative rule of the statistics pass:
// M = max m, Z = sum S * 2^d, W = sum 2^d (W_p + d S_p) with d = fl(m c) - fl(M c), in fp64; then
// the rounding of fl(M c) is undone for Z, and H = ln Z - ln 2 * W / Z (the offset's rounding shifts
// both terms of H equally).
__global__ __launch_bounds__(kBlock) void lm_head_merge_kernel(LmHeadProblem p) {
  const int lane = (int)threadIdx.x & (kWave - 1);
  const int row = (int)blockIdx.x * kWavesPerBlock + (int)threadIdx.x / kWave;
  if (row >= p.N) return;  // uniform over the wave
  const float T = p.row_T ? p.row_T[row] : p.T;
  const float c = (float)(kLog2e / (double)T);
  const float* pm = p.part_m + (size_t)row * p.nparts;
  const float* pS = p.part_S + (size_t)row * p.nparts;
  const float* pW = p.part_W + (size_t)row * p.nparts;
  float M = -INFINITY;
  for (int i = lane; i < p.nparts; i += kWave) M = fmaxf(M, pm[i]);
  M = wave_max(M);
  const float Mc = M * c;
  double Z = 0.0, W = 0.0;
  for (int i = lane; i < p.nparts; i += kWave) {
    const float m = pm[i];
    if (m != -INFINITY) {
      // as in the lanes of the statistics pass: the rescaling factor in fp32, the sums in fp64
      const float d = m * c - Mc;
      const double scale = (double)__builtin_amdgcn_exp2f(d);
      Z += (double)pS[i] * scale;
      W += scale * ((double)pW[i] + (double)d * (double)pS[i]);
    }
  }
  Z = wave_sum(Z);
  W = wave_sum(W);
  if (lane == 0) {
    p.row_m[row] = M;
    p.row_Z[row] = Z * exp2((double)Mc - (double)M * (double)c);
    if (p.row_H) p.row_H[row] = log(Z) - 0.69314718055994530942 * (W / Z);
  }
}

// Hands producer-side statistics to the verification workspace: draft position r of sequence b
// pairs target row r + b with draft row r (the layout the statistics pass writes).
template <typename DT>
__global__ __launch_bounds__(kBlock) void import_stats_kernel(Problem p, const float* t_max,
                                                               const double* t_sum,
                                                               const double* t_entropy,
                                                               const float* d_max,
                                                               const double* d_sum) {
  const int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (r >= p.R) return;
  for (int64_t j = r; j < (int64_t)p.B; j += p.R) p.arrive[j] = 0u;  // as the statistics pass does
  const int b = seq_of_row(p, r);
  const int32_t x = p.tokens[r];
  float lxt = -INFINITY, lxd = -INFINITY;
  if (x >= 0 && x < p.V) {
    lxt = DT::load(p.target, (r + b) * (int64_t)p.V + x);
    lxd = DT::load(p.draft, r * (int64_t)p.V + x);
  }
  p.Z[2 * r] = t_sum[r + b];
  p.Z[2 * r + 1] = d_sum[r];
  p.m[2 * r] = t_max[r + b];
  p.m[2 * r + 1] = d_max[r];
  p.lx[2 * r] = lxt;
  p.lx[2 * r + 1] = lxd;
  // entropy-based uncertainty H / log V of the target row (Section 5), when the producer has it
  if (t_entropy)
    p.unc[r] = p.V > 1 ? fmin(fmax(t_entropy[r + b] / log((double)p.V), 0.0), 1.0) : 0.0;
  if (r == 0) *p.unc_tag = t_entropy ? 1u : 0u;  // as the statistics pass tags its measure
}

}  // namespace ears
