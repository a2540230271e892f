// EARS verification step for MI355X (gfx950): kernels and the C ABI declared in include/ears.h.
//
//   stage STATS  : row_stats_kernel   - one streaming pass per logit row (paper Section 3.2 step 1,
//                                       Section 3.3 item 1: max P_t cached, never re-scanned)
//   stage DECIDE : decide_kernel      - ratio, uniform, tolerance, threshold, three-way decision,
//                                       first-rejection scan (Section 3.2 steps 2-5, Section 3.1)
//   stage SAMPLE : sample_select_kernel - residual / bonus token by Gumbel-max at slot n: a filter
//                  sample_kernel          that leaves a few survivors per row, then the exact choice,
//                                         in one launch (rows split into more than two chunks: one
//                                         workgroup per chunk, the last to finish a row chooses);
//                                         when DECIDE and SAMPLE run in one call the scan runs in
//                                         the filter's prologue
//   all three    : verify_kernel      - rectangular batches of long rows: the statistics code and
//                                       the sampling code as the workgroups of ONE launch (verify.h)
//
// The path is bound by HBM bandwidth (every needed row is read once, plus one re-read of the row
// pair the sampler needs): no matrix-core work in it.
//
// Beside it: greedy.h (temperature -> 0: arg-max of the target rows and a prefix scan), lm_head.h
// (the vocabulary projection on the matrix cores with a statistics epilogue, and the import of
// producer-side statistics into a verification workspace), and single_row_stats_kernel in
// row_stats.h (the statistics pass over one matrix on its own).
#include <hip/hip_runtime.h>

#include <cmath>
#include <atomic>
#include <cstdio>
#include <mutex>

#include "../../include/ears.h"
#include "bench_aids.h"
#include "decide.h"
#include "ears_device.h"
#include "row_stats.h"
#include "greedy.h"
#include "lm_head.h"
#include "sample.h"
#include "verify.h"

// Products such as fl(m*c) must stay rounded products (their rounding is undone explicitly
// later); fused operations are written as fmaf().
#pragma clang fp contract(off)

namespace ears {

// =================================================================================================
// Host side.
// =================================================================================================
struct WorkspaceLayout {
  size_t off_Z, off_m, off_lx, off_unc, off_unc_tag, off_decisions, off_records, off_arrive, off_ready, total;
  int S, chunk;  // how the sampling stage splits a row
};

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// The sampling stage touches only B rows, so each row is split into S chunks of whole tiles
// (one tile = 16 vocabulary entries per thread of a workgroup) until about kSampleTargetGroups
// workgroups exist.  A workgroup's time is the arrival of its part of the row plus a fixed start
// and tail, so more, shorter workgroups only add their fixed cost.  Filter + select at B = 256,
// V = 128256 on 256 CUs: 31.6 us with 256 groups, 28.6 with 512, 29.5 with 768, 32.6 with 1024,
// 39 with 2048.
constexpr int kSampleTargetGroups = 512;
// rows of at least this many bytes take the statistics kernel with eight loads in flight per lane
constexpr size_t kDeepRowBytes = 128000;
// A rectangular call with all three stages on long rows runs as ONE launch (verify_kernel) once
// its statistics workgroups alone fill the chip (two of them per CU at that kernel's register
// count): the sampling workgroups then take over the CUs as the statistics workgroups run out,
// instead of starting from an empty chip after a launch gap.  B = 256, K = 8, V = 128256 bf16:
// 182.6 us against 186.6 us; B = 96: 79 against 89; B = 512, K = 4, V = 151936: 222 against 225.
// Below, all workgroups are resident from the start and the hand-over through memory costs what
// the launch gap did (B = 32, K = 8: 41.2 us against 40.9 us); short rows want more than two
// statistics workgroups per CU, which the sampling code's registers do not allow in a common
// kernel (B = 256, K = 8, V = 32000: 67.5 us against 61.3 us).  With the entropy and variance
// measures the same headline batch takes 181 and 177 us against 185 and 183 us.
constexpr int64_t kSingleLaunchMinRows = 512;
// test aid (ears_test_single_launch): take the single launch below that size too, and the number
// of polls after which a waiting workgroup gives up
static std::atomic<int> g_force_single_launch{0};
static std::atomic<int> g_await_polls{kAwaitPolls};

static void sample_split(int B, int V, int elems_per_tile, int* S, int* chunk) {
  const int ntiles = (V + elems_per_tile - 1) / elems_per_tile;
  int want = (kSampleTargetGroups + B - 1) / B;
  if (want < 1) want = 1;
  if (want > ntiles) want = ntiles;
  const int tiles_per_chunk = (ntiles + want - 1) / want;
  *chunk = tiles_per_chunk * elems_per_tile;
  *S = (V + *chunk - 1) / *chunk;
}

static bool workspace_layout(int64_t R, int B, int V, WorkspaceLayout* w) {
  if (R < 1 || B < 1 || V < 1 || R > (int64_t)0x3FFFFFFF) return false;
  int S4, chunk;
  sample_split(B, V, kSampleTileElems, &S4, &chunk);
  size_t o = 0;
  w->off_Z = o;        o = align_up(o + (size_t)(2 * R) * sizeof(double), 256);
  w->off_m = o;        o = align_up(o + (size_t)(2 * R) * sizeof(float), 256);
  w->off_lx = o;       o = align_up(o + (size_t)(2 * R) * sizeof(float), 256);
  w->off_unc = o;      o = align_up(o + (size_t)R * sizeof(double), 256);
  w->off_unc_tag = o;  o = align_up(o + sizeof(uint32_t), 256);
  w->off_decisions = o; o = align_up(o + (size_t)R * sizeof(int32_t), 256);
  w->off_records = o;  o = align_up(o + (size_t)B * S4 * kRecordWords * sizeof(uint32_t), 256);
  w->off_arrive = o;   o = align_up(o + (size_t)B * sizeof(uint32_t), 256);
  w->off_ready = o;    o = align_up(o + (size_t)R * sizeof(uint32_t), 256);
  w->total = o;
  w->S = S4;
  w->chunk = chunk;
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
  // every launch is one-dimensional; the largest is rows (bounded above) or workgroups of the
  // sampling stage, B times the chunks of a row
  if ((int64_t)B * (int64_t)lay->S > (int64_t)0x7FFFFFFF) return EARS_ERR_SHAPE;
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

// The sampling stage, one launch: filter and exact choice by the same workgroup when a row is
// split into one or two chunks; otherwise a workgroup per chunk, and the one that finishes a row
// last chooses.
template <typename DT, bool kLate>
static void launch_sample(const Problem& p, hipStream_t stream) {
  if (p.S == 1) {
    hipLaunchKernelGGL((sample_select_kernel<DT, 1, kLate>), dim3((unsigned)p.B), dim3(kBlock), 0,
                       stream, p);
  } else if (p.S == 2) {
    hipLaunchKernelGGL((sample_select_kernel<DT, 2, kLate>), dim3((unsigned)p.B), dim3(2 * kBlock),
                       0, stream, p);
  } else {
    // (S * B fits a grid: checked with the other shapes)
    hipLaunchKernelGGL((sample_kernel<DT, kLate>), dim3((unsigned)p.S * (unsigned)p.B), dim3(kBlock), 0,
                       stream, p);
  }
}

template <typename DT>
static int launch(Problem p, int stages, hipStream_t stream) {
  (void)hipGetLastError();  // a stale error of the caller's own HIP calls is not this call's
  sample_split(p.B, p.V, kSampleTileElems, &p.S, &p.chunk);
  const bool stats = (stages & EARS_STAGE_STATS) != 0;
  const bool decide = (stages & EARS_STAGE_DECIDE) != 0;
  const bool sample = (stages & EARS_STAGE_SAMPLE) != 0;
  // All three stages in one call: the statistics kernel decides each position as it finishes it
  // and the filter kernel's prologue scans the decisions for the first rejection.  DECIDE and
  // SAMPLE on cached statistics: the filter kernel's prologue takes the decisions itself.  DECIDE
  // on its own: a small kernel decides and scans.
  const bool fused = stats && decide && sample;
  // DECIDE and SAMPLE on statistics cached earlier: the filter kernel's prologue decides
  const bool late = !stats && decide && sample;
  p.decide_fused = fused ? 1 : (late ? 2 : 0);
  // Long rows run with eight 16-byte loads in flight per lane, short ones with four.  Eight
  // cost registers (two workgroups fewer per CU) and pay where a launch ends with few groups per
  // CU left: -2 us of 155 at B = 256, K = 8, V = 128256, +3 % on large batches of 64 KB rows.
  // The variants with a second running sum have more to compute per element and are better off
  // with four (entropy: 171 us against 178 us).
  const bool deep = (size_t)p.V * sizeof(typename DT::storage) >= kDeepRowBytes;
  if (fused && p.row_offsets == nullptr && deep &&
      (p.R >= kSingleLaunchMinRows || g_force_single_launch.load() != 0) &&
      p.R + (int64_t)p.B * (int64_t)p.S <= (int64_t)0x7FFFFFFF) {
    // One launch: statistics workgroups first, the sampling workgroups behind them (verify.h).
    // The tag of a call: never zero, its two lowest bits clear, different from call to call.
    static std::atomic<uint32_t> calls{0};
    p.tag = ((calls.fetch_add(1u) + 1u) * 2654435761u) & ~3u;
    if (p.tag == 0u) p.tag = 4u;
    p.await_polls = g_await_polls.load();
    const dim3 grid((unsigned)(p.R + (int64_t)p.B * (int64_t)p.S)), block(kBlock);
    // (eight loads in flight for every measure: the kernel runs two workgroups per CU whatever the
    // statistics code needs, and with two, four loads in flight are no better for the entropy)
    if (p.unc_mode == EARS_UNCERTAINTY_ENTROPY)
      hipLaunchKernelGGL((verify_kernel<DT, 8, kMeasureEntropy>), grid, block, 0, stream, p);
    else if (p.unc_mode == EARS_UNCERTAINTY_VARIANCE)
      hipLaunchKernelGGL((verify_kernel<DT, 8, kMeasureVariance>), grid, block, 0, stream, p);
    else
      hipLaunchKernelGGL((verify_kernel<DT, 8, kMeasureNone>), grid, block, 0, stream, p);
    return hipGetLastError() == hipSuccess ? EARS_OK : EARS_ERR_HIP;
  }
  if (stats) {
    const dim3 grid((unsigned)p.R), block(kBlock);
    // The kernel always takes each position's decision as it finishes it.  Only a call that runs
    // all three stages uses it (the sampling stage scans the decisions); otherwise it is left in
    // the workspace unused and reports nothing: the decision stage takes its own from the
    // statistics, with the parameters of its own call.
    Problem ps = p;
    if (!fused) {
      ps.out_stats = nullptr;
      ps.out_path = nullptr;
    }
    if (p.unc_mode == EARS_UNCERTAINTY_ENTROPY)
      hipLaunchKernelGGL((row_stats_kernel<DT, 4, kMeasureEntropy>), grid, block, 0, stream, ps);
    else if (p.unc_mode == EARS_UNCERTAINTY_VARIANCE)
      hipLaunchKernelGGL((row_stats_kernel<DT, 4, kMeasureVariance>), grid, block, 0, stream, ps);
    else if (deep)
      hipLaunchKernelGGL((row_stats_kernel<DT, 8, kMeasureNone>), grid, block, 0, stream, ps);
    else
      hipLaunchKernelGGL((row_stats_kernel<DT, 4, kMeasureNone>), grid, block, 0, stream, ps);
  }
  if (decide && !fused && !late) {
    hipLaunchKernelGGL(decide_kernel, dim3((unsigned)((p.B + kWavesPerBlock - 1) / kWavesPerBlock)),
                       dim3(kBlock), 0, stream, p);
  }
  if (sample) {
    if (late) launch_sample<DT, true>(p, stream);
    else launch_sample<DT, false>(p, stream);
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

// Scratch of ears_verify_noalloc: a fixed array in device memory that comes with the code object,
// one copy per device the library runs on, each at its own address.  In host code the array's
// name is only a handle for hipGetSymbolAddress; kernels get the resolved address as an argument.
static __device__ __align__(256) unsigned char scratch[EARS_NOALLOC_SCRATCH_BYTES];
static std::mutex g_static_mutex;
static void* g_static_ptr[kMaxDevices] = {};

static int static_scratch_get(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return EARS_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (!g_static_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr)
      return EARS_ERR_HIP;
    g_static_ptr[dev] = ptr;
  }
  *out = g_static_ptr[dev];
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
    case EARS_ERR_PARAM: return "temperature, beta, stages or uncertainty measure invalid";
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
                   const float* temperature_per_seq, const float* beta_per_seq, int uncertainty,
                   uint64_t seed, const int64_t* seq_ids, void* workspace, size_t workspace_bytes,
                   int stages,
                   int32_t* out_accept_len, int32_t* out_tokens, double* out_stats,
                   int32_t* out_path, uint32_t* status_word, void* stream) {
  WorkspaceLayout lay;
  const int rc = validate(dtype, target_logits, draft_logits, draft_tokens, row_offsets,
                          total_draft_rows, B, K, V, temperature, beta, temperature_per_seq,
                          beta_per_seq, seq_ids, workspace, workspace_bytes, stages, out_accept_len,
                          out_tokens, out_stats, out_path, status_word, &lay);
  if (rc != EARS_OK) return rc;
  if (uncertainty != EARS_UNCERTAINTY_MAXPROB && uncertainty != EARS_UNCERTAINTY_ENTROPY &&
      uncertainty != EARS_UNCERTAINTY_VARIANCE)
    return EARS_ERR_PARAM;
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
  p.unc = reinterpret_cast<double*>(ws + lay.off_unc);
  p.unc_tag = reinterpret_cast<uint32_t*>(ws + lay.off_unc_tag);
  p.unc_mode = uncertainty;
  p.decisions = reinterpret_cast<int32_t*>(ws + lay.off_decisions);
  p.records = reinterpret_cast<uint32_t*>(ws + lay.off_records);
  p.arrive = reinterpret_cast<uint32_t*>(ws + lay.off_arrive);
  p.ready = reinterpret_cast<uint32_t*>(ws + lay.off_ready);
  p.tag = 0u;
  p.await_polls = kAwaitPolls;
  p.S = 0;
  p.chunk = 0;
  p.decide_fused = 0;
  p.accept_len = out_accept_len;
  p.out_tokens = out_tokens;
  p.out_stats = out_stats;
  p.out_path = out_path;
  p.status_word = status_word;
  hipStream_t s = static_cast<hipStream_t>(stream);
  return dtype == EARS_F32 ? launch<F32>(p, stages, s) : launch<BF16>(p, stages, s);
}

int ears_verify_noalloc(int dtype, const void* target_logits, const void* draft_logits,
                        const int32_t* draft_tokens, const int64_t* row_offsets,
                        int64_t total_draft_rows, int B, int K, int V, float temperature, float beta,
                        const float* temperature_per_seq, const float* beta_per_seq, int uncertainty,
                        uint64_t seed, const int64_t* seq_ids, int stages, int32_t* out_accept_len,
                        int32_t* out_tokens, double* out_stats, int32_t* out_path,
                        uint32_t* status_word, void* stream) {
  // every argument check, and the size limit, before the first HIP call
  WorkspaceLayout lay;
  alignas(256) static char dummy[256];
  int rc = validate(dtype, target_logits, draft_logits, draft_tokens, row_offsets, total_draft_rows,
                    B, K, V, temperature, beta, temperature_per_seq, beta_per_seq, seq_ids, dummy,
                    (size_t)-1, stages, out_accept_len, out_tokens, out_stats, out_path, status_word,
                    &lay);
  if (rc != EARS_OK) return rc;
  if (uncertainty != EARS_UNCERTAINTY_MAXPROB && uncertainty != EARS_UNCERTAINTY_ENTROPY &&
      uncertainty != EARS_UNCERTAINTY_VARIANCE)
    return EARS_ERR_PARAM;
  if (lay.total > (size_t)EARS_NOALLOC_SCRATCH_BYTES) return EARS_ERR_WORKSPACE;
  void* ws = nullptr;
  rc = static_scratch_get(&ws);
  if (rc != EARS_OK) return rc;
  // Nothing in the scratch has to start at zero: every word a stage reads was written earlier in
  // the same call (or by the stage that cached the statistics), so the last call's contents are
  // simply overwritten.
  return ears_verify_ex(dtype, target_logits, draft_logits, draft_tokens, row_offsets,
                        total_draft_rows, B, K, V, temperature, beta, temperature_per_seq,
                        beta_per_seq, uncertainty, seed, seq_ids, ws, EARS_NOALLOC_SCRATCH_BYTES,
                        stages, out_accept_len, out_tokens, out_stats, out_path, status_word, stream);
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
                        beta_seq, EARS_UNCERTAINTY_MAXPROB, seed, nullptr, ws, lay.total,
                        EARS_STAGE_ALL, out_accept_len,
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

size_t ears_greedy_workspace_bytes(int64_t total_draft_rows, int B) {
  if (total_draft_rows < 1 || B < 1 || total_draft_rows > (int64_t)0x3FFFFFFF)
    return 0;
  return align_up((size_t)(total_draft_rows + B) * sizeof(int32_t), 256);
}

int ears_verify_greedy(int dtype, const void* target_logits, const int32_t* draft_tokens,
                       const int64_t* row_offsets, int64_t total_draft_rows, int B, int K, int V,
                       void* workspace, size_t workspace_bytes, int32_t* out_accept_len,
                       int32_t* out_tokens, void* stream) {
  if (dtype != EARS_F32 && dtype != EARS_BF16) return EARS_ERR_DTYPE;
  if (!target_logits || !draft_tokens || !out_accept_len || !out_tokens) return EARS_ERR_NULL;
  if (B < 1 || V < 1 || total_draft_rows < 1) return EARS_ERR_SHAPE;
  if (row_offsets == nullptr && (K < 1 || (int64_t)B * (int64_t)K != total_draft_rows))
    return EARS_ERR_SHAPE;
  const size_t need = ears_greedy_workspace_bytes(total_draft_rows, B);
  if (need == 0) return EARS_ERR_SHAPE;
  if (!aligned(target_logits, 16) || !aligned(draft_tokens, 4) || !aligned(out_accept_len, 4) ||
      !aligned(out_tokens, 4) || !aligned(row_offsets, 8))
    return EARS_ERR_ALIGN;
  if (workspace) {
    if (workspace_bytes < need) return EARS_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return EARS_ERR_ALIGN;
  } else {
    const int rc = scratch_get(need, &workspace);
    if (rc != EARS_OK) return rc;
  }
  (void)hipGetLastError();  // a stale error of the caller's own HIP calls is not this call's
  GreedyProblem p;
  p.target = target_logits;
  p.tokens = draft_tokens;
  p.row_offsets = row_offsets;
  p.R = total_draft_rows;
  p.B = B;
  p.K = K;
  p.V = V;
  p.argmax = static_cast<int32_t*>(workspace);
  p.accept_len = out_accept_len;
  p.out_tokens = out_tokens;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int64_t nrows = total_draft_rows + B;
  const dim3 rows_grid((unsigned)nrows);
  if (dtype == EARS_F32)
    hipLaunchKernelGGL((row_argmax_kernel<F32, 4>), rows_grid, dim3(kBlock), 0, s, p);
  else
    hipLaunchKernelGGL((row_argmax_kernel<BF16, 4>), rows_grid, dim3(kBlock), 0, s, p);
  hipLaunchKernelGGL(greedy_scan_kernel, dim3((unsigned)((B + kWavesPerBlock - 1) / kWavesPerBlock)),
                     dim3(kBlock), 0, s, p);
  return hipGetLastError() == hipSuccess ? EARS_OK : EARS_ERR_HIP;
}

size_t ears_lm_head_workspace_bytes(int N, int V) {
  if (N < 1 || V < 1) return 0;
  const size_t nparts = (size_t)kLmPartsPerTile * (size_t)((V + kLmTile - 1) / kLmTile);
  return 3 * align_up((size_t)N * nparts * sizeof(float), 256);
}

int ears_lm_head_bf16(const void* hidden, const void* weight, int N, int D, int V,
                      float temperature, const float* row_temperature, void* out_logits,
                      float* out_row_max, double* out_row_sumexp, double* out_row_entropy,
                      void* workspace, size_t workspace_bytes, void* stream) {
  if (!hidden || !weight || !out_logits || !out_row_max || !out_row_sumexp) return EARS_ERR_NULL;
  if (N < 1 || V < 1 || D < kLmBK || D % kLmBK != 0) return EARS_ERR_SHAPE;
  // the kernel addresses the 256 rows of a tile with 32-bit byte offsets
  if (D > (1 << 20)) return EARS_ERR_SHAPE;
  if (!row_temperature && !(std::isfinite(temperature) && temperature > 0.0f)) return EARS_ERR_PARAM;
  if (!aligned(hidden, 16) || !aligned(weight, 16) || !aligned(out_logits, 2) ||
      !aligned(out_row_max, 4) || !aligned(out_row_sumexp, 8) || !aligned(out_row_entropy, 8) ||
      !aligned(row_temperature, 4))
    return EARS_ERR_ALIGN;
  const size_t need = ears_lm_head_workspace_bytes(N, V);
  if (!workspace || workspace_bytes < need) return EARS_ERR_WORKSPACE;
  if (!aligned(workspace, 256)) return EARS_ERR_ALIGN;
  (void)hipGetLastError();  // a stale error of the caller's own HIP calls is not this call's
  LmHeadProblem p;
  p.hidden = static_cast<const uint16_t*>(hidden);
  p.weight = static_cast<const uint16_t*>(weight);
  p.row_T = row_temperature;
  p.T = temperature;
  p.N = N;
  p.D = D;
  p.V = V;
  p.n_vtiles = (V + kLmTile - 1) / kLmTile;
  p.n_ttiles = (N + kLmTile - 1) / kLmTile;
  p.logits = static_cast<uint16_t*>(out_logits);
  p.nparts = kLmPartsPerTile * p.n_vtiles;
  p.part_m = static_cast<float*>(workspace);
  p.part_S = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + need / 3);
  p.part_W = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + 2 * (need / 3));
  p.row_m = out_row_max;
  p.row_Z = out_row_sumexp;
  p.row_H = out_row_entropy;
  const int64_t groups = (int64_t)8 * ((p.n_vtiles + 7) / 8) * p.n_ttiles;
  if (groups > (int64_t)0x7FFFFFFF) return EARS_ERR_SHAPE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(lm_head_kernel, dim3((unsigned)groups), dim3(kLmThreads), 0, s, p);
  hipLaunchKernelGGL(lm_head_merge_kernel, dim3((unsigned)((N + kWavesPerBlock - 1) / kWavesPerBlock)),
                     dim3(kBlock), 0, s, p);
  return hipGetLastError() == hipSuccess ? EARS_OK : EARS_ERR_HIP;
}

int ears_row_stats(int dtype, const void* logits, int64_t rows, int V, float temperature,
                   const float* row_temperature, float* out_row_max, double* out_row_sumexp,
                   double* out_row_entropy, void* stream) {
  if (dtype != EARS_F32 && dtype != EARS_BF16) return EARS_ERR_DTYPE;
  if (!logits || !out_row_max || !out_row_sumexp) return EARS_ERR_NULL;
  if (rows < 1 || rows > (int64_t)0x7FFFFFFF || V < 1) return EARS_ERR_SHAPE;
  if (!row_temperature && !(std::isfinite(temperature) && temperature > 0.0f)) return EARS_ERR_PARAM;
  if (!aligned(logits, 16) || !aligned(out_row_max, 4) || !aligned(out_row_sumexp, 8) ||
      !aligned(out_row_entropy, 8) || !aligned(row_temperature, 4))
    return EARS_ERR_ALIGN;
  (void)hipGetLastError();  // a stale error of the caller's own HIP calls is not this call's
  RowStatsProblem p;
  p.logits = logits;
  p.rows = rows;
  p.V = V;
  p.T = temperature;
  p.row_T = row_temperature;
  p.row_m = out_row_max;
  p.row_Z = out_row_sumexp;
  p.row_H = out_row_entropy;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const dim3 grid((unsigned)rows), block(kBlock);
  if (dtype == EARS_F32 && out_row_entropy)
    hipLaunchKernelGGL((single_row_stats_kernel<F32, 4, true>), grid, block, 0, s, p);
  else if (dtype == EARS_F32)
    hipLaunchKernelGGL((single_row_stats_kernel<F32, 4, false>), grid, block, 0, s, p);
  else if (out_row_entropy)
    hipLaunchKernelGGL((single_row_stats_kernel<BF16, 4, true>), grid, block, 0, s, p);
  else
    hipLaunchKernelGGL((single_row_stats_kernel<BF16, 4, false>), grid, block, 0, s, p);
  return hipGetLastError() == hipSuccess ? EARS_OK : EARS_ERR_HIP;
}

int ears_import_stats(int dtype, const void* target_logits, const void* draft_logits,
                      const int32_t* draft_tokens, const int64_t* row_offsets,
                      int64_t total_draft_rows, int B, int K, int V, const float* target_row_max,
                      const double* target_row_sumexp, const double* target_row_entropy,
                      const float* draft_row_max, const double* draft_row_sumexp, void* workspace,
                      size_t workspace_bytes, void* stream) {
  if (!target_row_max || !target_row_sumexp || !draft_row_max || !draft_row_sumexp)
    return EARS_ERR_NULL;
  WorkspaceLayout lay;
  // the output pointers of a verification call are not involved: stand-ins pass its null checks
  const int32_t* stand_in = draft_tokens;
  const int rc = validate(dtype, target_logits, draft_logits, draft_tokens, row_offsets,
                          total_draft_rows, B, K, V, 1.0f, 0.0f, nullptr, nullptr, nullptr, workspace,
                          workspace_bytes, EARS_STAGE_STATS, stand_in, stand_in, nullptr, nullptr,
                          nullptr, &lay);
  if (rc != EARS_OK) return rc;
  if (!aligned(target_row_max, 4) || !aligned(draft_row_max, 4) || !aligned(target_row_sumexp, 8) ||
      !aligned(draft_row_sumexp, 8) || !aligned(target_row_entropy, 8))
    return EARS_ERR_ALIGN;
  (void)hipGetLastError();  // a stale error of the caller's own HIP calls is not this call's
  Problem p = {};
  p.target = target_logits;
  p.draft = draft_logits;
  p.tokens = draft_tokens;
  p.row_offsets = row_offsets;
  p.R = total_draft_rows;
  p.B = B;
  p.K = K;
  p.V = V;
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  p.Z = reinterpret_cast<double*>(ws + lay.off_Z);
  p.m = reinterpret_cast<float*>(ws + lay.off_m);
  p.lx = reinterpret_cast<float*>(ws + lay.off_lx);
  p.unc = reinterpret_cast<double*>(ws + lay.off_unc);
  p.unc_tag = reinterpret_cast<uint32_t*>(ws + lay.off_unc_tag);
  p.arrive = reinterpret_cast<uint32_t*>(ws + lay.off_arrive);
  p.ready = reinterpret_cast<uint32_t*>(ws + lay.off_ready);
  p.tag = 0u;
  p.await_polls = kAwaitPolls;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const dim3 grid((unsigned)((total_draft_rows + kBlock - 1) / kBlock));
  if (dtype == EARS_F32)
    hipLaunchKernelGGL(import_stats_kernel<F32>, grid, dim3(kBlock), 0, s, p, target_row_max,
                       target_row_sumexp, target_row_entropy, draft_row_max, draft_row_sumexp);
  else
    hipLaunchKernelGGL(import_stats_kernel<BF16>, grid, dim3(kBlock), 0, s, p, target_row_max,
                       target_row_sumexp, target_row_entropy, draft_row_max, draft_row_sumexp);
  return hipGetLastError() == hipSuccess ? EARS_OK : EARS_ERR_HIP;
}

void ears_test_single_launch(int force, int wait_polls) {
  g_force_single_launch.store(force != 0 ? 1 : 0);
  g_await_polls.store(wait_polls >= 0 ? wait_polls : kAwaitPolls);
}

int ears_bench_read_sink_words(void) { return kBenchBlocks; }

int ears_bench_read(const void* src, size_t bytes, uint32_t* sink, void* stream) {
  if (!src || !sink) return EARS_ERR_NULL;
  if (bytes == 0 || bytes % 16 != 0) return EARS_ERR_SHAPE;
  if (!aligned(src, 16) || !aligned(sink, 4)) return EARS_ERR_ALIGN;
  (void)hipGetLastError();
  // slabs of about 256 KiB, their number a multiple of 1024 (four workgroups of kBlock threads on each
  // of 256 CUs) so that the last round of workgroups is a full one
  const size_t nvec = bytes / 16;
  size_t rounds = (nvec + 1024 * kBenchSlabVecs / 2) / (1024 * kBenchSlabVecs);
  if (rounds < 1) rounds = 1;
  const size_t slab_vecs = (nvec + 1024 * rounds - 1) / (1024 * rounds);
  // two slabs per workgroup, half a buffer apart, like the target and draft rows of one position
  size_t blocks = 1024 * ((rounds + 1) / 2);
  if (blocks > (size_t)kBenchBlocks) blocks = kBenchBlocks;
  hipLaunchKernelGGL(bench_read_kernel, dim3((unsigned)blocks), dim3(kBlock), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint4*>(src), nvec,
                     slab_vecs, sink);
  return hipGetLastError() == hipSuccess ? EARS_OK : EARS_ERR_HIP;
}

int ears_bench_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!src || !dst) return EARS_ERR_NULL;
  if (bytes == 0 || bytes % 16 != 0) return EARS_ERR_SHAPE;
  if (!aligned(src, 16) || !aligned(dst, 16)) return EARS_ERR_ALIGN;
  (void)hipGetLastError();
  hipLaunchKernelGGL(bench_copy_kernel, dim3(kBenchBlocks), dim3(kBlock), 0,
                     static_cast<hipStream_t>(stream), static_cast<uint4*>(dst),
                     static_cast<const uint4*>(src), bytes / 16);
  return hipGetLastError() == hipSuccess ? EARS_OK : EARS_ERR_HIP;
}

}  // extern "C"
