// The whole verification step in ONE launch (rectangular batches, all three stages in one call).
#pragma once

#include "row_stats.h"
#include "sample.h"

namespace ears {

// =================================================================================================
// Workgroups 0 .. R-1 are the statistics workgroups of the draft positions (row_stats_body), the
// B * S after them the sampling workgroups, one per chunk of a sequence's row (sample_body, and
// select_body in the one that finishes a row last).  A sampling workgroup needs the decisions of
// all positions of its sequence and the statistics of one.  A statistics workgroup hands them
// over through device memory: m and Z with coherent stores, and once those have been
// acknowledged, ready[r] = tag | decision.  The first wave of a sampling workgroup waits until
// the ready words of its sequence carry the call's tag.
//
// Why the wait ends: workgroups are dispatched in the order of their ids, so every statistics
// workgroup has been dispatched before any sampling workgroup is, and statistics workgroups wait
// for nobody.  (With several XCDs each one dispatches its own share of the ids in order, and its
// CUs are only ever held by its own earlier workgroups: the argument holds per XCD.)  The wait is
// bounded nonetheless; a workgroup that gives up raises status bit 4 and leaves its row's slot of
// out_tokens as it found it.
//
// What it saves over two launches: the gap between them and an empty chip at the start of the
// second.  The sampling workgroups take over the CUs one by one as the statistics workgroups run
// out; those of sequences that finished long ago never wait, only those of the last sequences
// do, briefly.  (Placing the sampling workgroups of a sequence earlier among the ids, a fixed
// number of sequences behind its statistics workgroups, so that they run beside the stream rather
// than at its end, lost all of the gain: 185.7 us against 182.2 us at B = 256, K = 8, V = 128256.
// Splitting the rows of the last sequences, whose sampling workgroups run as the chip empties,
// into more and shorter chunks than the others gained nothing either: 181-182 us whether those 64
// rows were cut in two or in four, 185-186 us in eight.)
//
// The ready words are zero between calls: the workgroup that finishes a row last clears those of
// its sequence (every waiter of the sequence has counted in by then).  The tag differs from call
// to call, so that a workspace with arbitrary contents is as good as a zeroed one (a stale word
// would have to equal the tag in its 30 upper bits), and the clearing covers the one case where
// it does not differ: a captured graph replays the call with the tag it was captured with.
// =================================================================================================
template <typename DT, int kUnroll, int kMeasure>
__global__ __launch_bounds__(kBlock) void verify_kernel(Problem p) {
  __shared__ float sh_m[kWavesPerBlock];
  __shared__ double sh_s[2 * kWavesPerBlock];
  __shared__ int sh_last;
  if ((int64_t)blockIdx.x < p.R) {  // uniform over the workgroup
    row_stats_body<DT, kUnroll, kMeasure, true>(p, (int64_t)blockIdx.x, sh_m, sh_s);
    return;
  }
  const unsigned bid = blockIdx.x - (unsigned)p.R;
  int n;
  (void)sample_body<DT, 1, false, false, true>(p, n, bid);
  if (n < 0) {  // uniform: the wait was given up
    if (threadIdx.x == 0 && p.status_word) atomicOr(p.status_word, 16u);
    return;
  }
  const int b = (int)(bid / (unsigned)p.S);
  if (!arrive_is_last(p.arrive + b, (uint32_t)p.S, &sh_last)) return;
  for (int i = (int)threadIdx.x; i < p.K; i += kBlock) coherent_store(p.ready + (int64_t)b * p.K + i, 0u);
  select_body<DT, true, true>(p, b, n);
}

}  // namespace ears
