// First-digit histogram of the radix selection (Eq. 2), shared by the selection kernels and by the
// score kernels that build it while the scores are still on chip.
#pragma once
#include "esa_common.h"

namespace esa {

constexpr int kRadixBins = 2048;        // 11-bit digits (the last pass uses 10 bits of them)
// Copies of each global histogram; workgroup w adds into copy w % kHistReplicas and a reader sums the copies.
// Adds to one address are served one after the other (about 30 ns each, measured), and where most scores share
// a digit every workgroup adds to the same few bins: 250 workgroups on one copy cost 5 us, on four copies 0.4 us.
constexpr int kHistReplicas = 4;
constexpr int kHistWords = 3 * kHistReplicas * kRadixBins;   // the three passes' histograms of one batch row

// Workspace of one batch row of the selection, in uint32 words.
struct TopkLayout {
  static constexpr int hist = 0;                              // [3][kHistReplicas][kRadixBins]
  static constexpr int pick = kHistWords;                     // [2][2]: (bin, remaining rank) chosen in the first / second histogram
  static constexpr int blk = kHistWords + 4;                  // [2][nblk]: per block, scores above the 22-bit prefix / sharing it
  // then [nblk][cap] uint16: last digits of the scores sharing the prefix, cap = scores per block
};

// One LDS-histogram increment per lane, with the lanes of a wave that hit the leader's bin
// folded into a single atomic (scores of one row share their exponent, so in the first pass
// almost every lane hits the same bin).  Every lane of the wave must call it.
__device__ __forceinline__ void hist_add(uint32_t* h, bool active, uint32_t bin) {
  const uint64_t act = __ballot(active);
  if (act == 0ull) return;
  const int leader = __ffsll((long long)act) - 1;
  const uint32_t lead_bin = (uint32_t)__builtin_amdgcn_readlane((int)bin, leader);     // leader is the same in every lane
  const uint64_t same = __ballot(active && bin == lead_bin);
  if ((int)(__builtin_amdgcn_workitem_id_x() & 63) == leader) atomicAdd(&h[lead_bin], (uint32_t)__popcll(same));
  if (active && bin != lead_bin) atomicAdd(&h[bin], 1u);
}

// A workgroup's finished LDS histogram h, added to its copy of one pass's global histogram gh ([kHistReplicas][kRadixBins]).
__device__ __forceinline__ void hist_flush(uint32_t* __restrict__ gh, const uint32_t* h, int wg, int tid, int n_threads) {
  uint32_t* g = gh + (wg % kHistReplicas) * kRadixBins;
  for (int i = tid; i < kRadixBins; i += n_threads)
    if (h[i]) atomicAdd(&g[i], h[i]);
}

// Words of one batch row's selection workspace and the stride between rows (host side).
int64_t topk_row_stride_words(int64_t n, int batch);

}  // namespace esa
