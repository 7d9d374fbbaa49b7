// Token-level top-k over the middle-token scores (Eq. 2): exact radix select on
// order-preserving 32-bit keys, then an ordered compaction.
//
// Three histogram passes (11 + 11 + 10 bits, most significant first) pin down the key T of the
// k-th largest score and how many scores equal to T are still needed; a counting pass and a
// writing pass then emit the positions of every score above T plus the first `need` scores
// equal to T, in ascending position order (equal scores: the lower position wins).
// All cross-block traffic is integer atomics, so the result is deterministic.  The block that
// finishes a pass last (ticket counter) does that pass's serial step; no block ever waits for
// another, so no co-residency is assumed.
#include "esa_common.h"

namespace esa {
namespace {

constexpr int kThreads = 256;
constexpr int kItems = 8;                       // consecutive scores per thread
constexpr int kTile = kThreads * kItems;        // scores per block
constexpr int kBins = 2048;

// Workspace of one batch row, in uint32 words.
struct TopkLayout {
  static constexpr int hist = 0;                         // [3][kBins]
  static constexpr int prefix = 3 * kBins;               // key bits fixed so far
  static constexpr int k_rem = prefix + 1;               // scores still to take at/below the prefix
  static constexpr int done = prefix + 2;                // [4] ticket counters: three histogram passes, count
  static constexpr int blk = prefix + 8;                 // [2][nblk]: above-T and equal-T counts / offsets
};

__host__ __device__ inline int64_t topk_row_words(int64_t nblk) { return TopkLayout::blk + 2 * nblk; }

__device__ __forceinline__ uint32_t coherent_load(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Exclusive prefix sum of one value per thread over the block; *total gets the block sum.
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* total, uint32_t* wave_sums) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  uint32_t incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    uint32_t t = __shfl_up(incl, off, 64);
    if (lane >= off) incl += t;
  }
  __syncthreads();                       // wave_sums may still be read from a previous call
  if (lane == 63) wave_sums[w] = incl;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < kThreads / 64; ++i) {
    uint32_t s = wave_sums[i];
    if (i < w) base += s;
    tot += s;
  }
  *total = tot;
  return base + incl - v;
}

__device__ __forceinline__ void load_keys(const float* row, int64_t n, int64_t first, uint32_t (&key)[kItems],
                                          bool (&ok)[kItems]) {
#pragma unroll
  for (int e = 0; e < kItems; ++e) {
    int64_t i = first + e;
    ok[e] = i < n;
    key[e] = ok[e] ? ordered_key(row[i]) : 0u;
  }
}

__global__ void topk_init(uint32_t* ws, int64_t row_words, int k_eff) {
  uint32_t* w = ws + (int64_t)blockIdx.x * row_words;
  for (int i = threadIdx.x; i < TopkLayout::blk; i += blockDim.x) w[i] = 0u;
  __syncthreads();
  if (threadIdx.x == 0) w[TopkLayout::k_rem] = (uint32_t)k_eff;
}

// PASS 0: bits 31..21, PASS 1: bits 20..10, PASS 2: bits 9..0.
template <int PASS>
__global__ __launch_bounds__(kThreads) void topk_hist(const float* __restrict__ score, int64_t n, int64_t score_bs,
                                                      uint32_t* __restrict__ ws, int64_t row_words, int nblk) {
  __shared__ uint32_t h[kBins];
  __shared__ uint32_t wave_sums[kThreads / 64];
  __shared__ int is_last;
  const float* row = score + (int64_t)blockIdx.y * score_bs;
  uint32_t* w = ws + (int64_t)blockIdx.y * row_words;
  for (int i = threadIdx.x; i < kBins; i += kThreads) h[i] = 0u;
  const uint32_t prefix = (PASS == 0) ? 0u : w[TopkLayout::prefix];
  __syncthreads();

  uint32_t key[kItems];
  bool ok[kItems];
  load_keys(row, n, (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems, key, ok);
#pragma unroll
  for (int e = 0; e < kItems; ++e) {
    if (!ok[e]) continue;
    if (PASS == 0) {
      atomicAdd(&h[key[e] >> 21], 1u);
    } else if (PASS == 1) {
      if ((key[e] >> 21) == (prefix >> 21)) atomicAdd(&h[(key[e] >> 10) & 2047u], 1u);
    } else {
      if ((key[e] >> 10) == (prefix >> 10)) atomicAdd(&h[key[e] & 1023u], 1u);
    }
  }
  __syncthreads();
  uint32_t* gh = w + TopkLayout::hist + PASS * kBins;
  for (int i = threadIdx.x; i < kBins; i += kThreads)
    if (h[i]) atomicAdd(&gh[i], h[i]);
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) is_last = (atomicAdd(&w[TopkLayout::done + PASS], 1u) == (uint32_t)(nblk - 1));
  __syncthreads();
  if (!is_last) return;
  __threadfence();

  // Serial step: walk the finished histogram from the top bin down to the bin holding rank k_rem.
  for (int i = threadIdx.x; i < kBins; i += kThreads) h[i] = coherent_load(&gh[i]);
  const uint32_t k_rem = coherent_load(&w[TopkLayout::k_rem]);
  __syncthreads();
  constexpr int per = kBins / kThreads;                  // bins per thread, thread 0 owns the highest
  const int top = kBins - 1 - threadIdx.x * per;
  uint32_t mine = 0;
#pragma unroll
  for (int e = 0; e < per; ++e) mine += h[top - e];
  uint32_t total;
  const uint32_t above = block_excl_scan(mine, &total, wave_sums);
  if (above < k_rem && k_rem <= above + mine) {          // exactly one thread
    uint32_t cum = above;
    for (int e = 0; e < per; ++e) {
      const uint32_t c = h[top - e];
      if (cum + c >= k_rem) {
        const uint32_t bin = (uint32_t)(top - e);
        const uint32_t shift = (PASS == 0) ? 21u : (PASS == 1) ? 10u : 0u;
        w[TopkLayout::prefix] = prefix | (bin << shift);
        w[TopkLayout::k_rem] = k_rem - cum;
        break;
      }
      cum += c;
    }
  }
}

// Per block: how many scores lie above T and how many equal T; the last block turns both
// arrays into exclusive offsets.
__global__ __launch_bounds__(kThreads) void topk_count(const float* __restrict__ score, int64_t n, int64_t score_bs,
                                                       uint32_t* __restrict__ ws, int64_t row_words, int nblk) {
  __shared__ uint32_t wave_sums[kThreads / 64];
  __shared__ int is_last;
  const float* row = score + (int64_t)blockIdx.y * score_bs;
  uint32_t* w = ws + (int64_t)blockIdx.y * row_words;
  const uint32_t T = w[TopkLayout::prefix];
  uint32_t key[kItems];
  bool ok[kItems];
  load_keys(row, n, (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems, key, ok);
  uint32_t gt = 0, eq = 0;
#pragma unroll
  for (int e = 0; e < kItems; ++e) {
    gt += (ok[e] && key[e] > T) ? 1u : 0u;
    eq += (ok[e] && key[e] == T) ? 1u : 0u;
  }
  uint32_t tot_gt, tot_eq;
  block_excl_scan(gt, &tot_gt, wave_sums);
  block_excl_scan(eq, &tot_eq, wave_sums);
  uint32_t* bg = w + TopkLayout::blk;
  uint32_t* be = bg + nblk;
  if (threadIdx.x == 0) {
    __hip_atomic_store(&bg[blockIdx.x], tot_gt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&be[blockIdx.x], tot_eq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __threadfence();
    is_last = (atomicAdd(&w[TopkLayout::done + 3], 1u) == (uint32_t)(nblk - 1));
  }
  __syncthreads();
  if (!is_last) return;
  __threadfence();
  uint32_t carry_gt = 0, carry_eq = 0;
  for (int base = 0; base < nblk; base += kThreads) {
    const int i = base + threadIdx.x;
    const uint32_t g = (i < nblk) ? coherent_load(&bg[i]) : 0u;
    const uint32_t q = (i < nblk) ? coherent_load(&be[i]) : 0u;
    uint32_t tg, tq;
    const uint32_t xg = block_excl_scan(g, &tg, wave_sums);
    const uint32_t xq = block_excl_scan(q, &tq, wave_sums);
    if (i < nblk) {
      bg[i] = carry_gt + xg;
      be[i] = carry_eq + xq;
    }
    carry_gt += tg;
    carry_eq += tq;
  }
}

__global__ __launch_bounds__(kThreads) void topk_write(const float* __restrict__ score, int64_t n, int64_t score_bs,
                                                       const uint32_t* __restrict__ ws, int64_t row_words, int nblk,
                                                       int64_t base, int32_t* __restrict__ idx, int64_t idx_bs,
                                                       int k_eff) {
  __shared__ uint32_t wave_sums[kThreads / 64];
  const float* row = score + (int64_t)blockIdx.y * score_bs;
  const uint32_t* w = ws + (int64_t)blockIdx.y * row_words;
  int32_t* out = idx + (int64_t)blockIdx.y * idx_bs;
  const uint32_t T = w[TopkLayout::prefix];
  const uint32_t need = w[TopkLayout::k_rem];            // equal-to-T scores to take, lowest positions first
  const uint32_t off_gt = w[TopkLayout::blk + blockIdx.x];
  const uint32_t off_eq = w[TopkLayout::blk + nblk + blockIdx.x];
  const int64_t first = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems;
  uint32_t key[kItems];
  bool ok[kItems];
  load_keys(row, n, first, key, ok);
  uint32_t gt = 0, eq = 0;
#pragma unroll
  for (int e = 0; e < kItems; ++e) {
    gt += (ok[e] && key[e] > T) ? 1u : 0u;
    eq += (ok[e] && key[e] == T) ? 1u : 0u;
  }
  uint32_t tot;
  uint32_t g_before = off_gt + block_excl_scan(gt, &tot, wave_sums);
  uint32_t e_before = off_eq + block_excl_scan(eq, &tot, wave_sums);
#pragma unroll
  for (int e = 0; e < kItems; ++e) {
    if (!ok[e]) continue;
    const bool is_gt = key[e] > T, is_eq = key[e] == T;
    if (is_gt || (is_eq && e_before < need)) {
      const uint32_t slot = g_before + (e_before < need ? e_before : need);
      if (slot < (uint32_t)k_eff) out[slot] = (int32_t)(base + first + e);
    }
    g_before += is_gt ? 1u : 0u;
    e_before += is_eq ? 1u : 0u;
  }
}

// k >= n: every middle token is selected.
__global__ void topk_all(int64_t n, int64_t base, int32_t* idx, int64_t idx_bs) {
  int32_t* out = idx + (int64_t)blockIdx.y * idx_bs;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    out[i] = (int32_t)(base + i);
}

}  // namespace

size_t topk_workspace_bytes(int64_t n, int k, int batch) {
  if (n <= 0 || k <= 0 || batch <= 0 || k >= n) return 256;
  const int64_t nblk = (n + kTile - 1) / kTile;
  return align_up((size_t)topk_row_words(nblk) * sizeof(uint32_t), 256) * (size_t)batch;
}

int launch_topk(const float* score, int64_t n, int k, int64_t base, int32_t* idx, int batch, int64_t score_bs,
                int64_t idx_bs, void* ws, size_t ws_bytes, hipStream_t st) {
  if (k >= n) {
    const int blocks = (int)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
    topk_all<<<dim3(blocks, batch), 256, 0, st>>>(n, base, idx, idx_bs);
    ESA_LAUNCH_CHECK("topk_all");
    return ESA_OK;
  }
  const int64_t nblk64 = (n + kTile - 1) / kTile;
  const int nblk = (int)nblk64;
  const int64_t row_words = (int64_t)(align_up((size_t)topk_row_words(nblk) * sizeof(uint32_t), 256) / sizeof(uint32_t));
  uint32_t* w = (uint32_t*)ws;
  const dim3 grid(nblk, batch);
  topk_init<<<batch, 256, 0, st>>>(w, row_words, k);
  topk_hist<0><<<grid, kThreads, 0, st>>>(score, n, score_bs, w, row_words, nblk);
  topk_hist<1><<<grid, kThreads, 0, st>>>(score, n, score_bs, w, row_words, nblk);
  topk_hist<2><<<grid, kThreads, 0, st>>>(score, n, score_bs, w, row_words, nblk);
  topk_count<<<grid, kThreads, 0, st>>>(score, n, score_bs, w, row_words, nblk);
  topk_write<<<grid, kThreads, 0, st>>>(score, n, score_bs, w, row_words, nblk, base, idx, idx_bs, k);
  ESA_LAUNCH_CHECK("topk");
  return ESA_OK;
}

}  // namespace esa
