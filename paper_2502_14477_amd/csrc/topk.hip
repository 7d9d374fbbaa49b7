// Token-level top-k over the middle-token scores (Eq. 2): exact radix select on
// order-preserving 32-bit keys, then an ordered compaction.
//
// Three histogram passes (11 + 11 + 10 bits, most significant first) pin down the key T of the
// k-th largest score and how many scores equal to T are still needed; a writing pass then emits
// the positions of every score above T plus the first `need` scores equal to T, in ascending
// position order (equal scores: the lower position wins).  For its output offsets a workgroup of
// the writing pass needs the number of selected scores in the workgroups before it; the third
// histogram pass leaves that per workgroup in two pieces: the count of scores above the 22-bit
// prefix fixed so far (selected whatever the last digit of T turns out to be), and the list of the
// last digits of the scores that share the prefix (usually a handful), which the writing pass
// compares with T's last digit once it knows it.
// All cross-block traffic is integer atomics and plain stores, so the result is deterministic.
// No workgroup ever waits for another: what one pass leaves in global memory (a 2048-bin
// histogram, or the per-block counts) is re-read and scanned by EVERY workgroup of the next
// launch, redundantly, instead of being finished by a last-arriving workgroup — a launch is then
// one round trip to memory plus a little LDS work, which is what bounds this latency-bound call.
#include <atomic>

#include "esa_common.h"
#include "radix_hist.h"

namespace esa {
namespace {

constexpr int kThreads = 512;
constexpr int kItems = 2;                       // consecutive scores per thread
constexpr int kTile = kThreads * kItems;        // scores per block
constexpr int kBins = kRadixBins;

struct TopkPlan {
  int64_t sub;      // tiles of kTile scores per workgroup
  int64_t nblk;     // workgroups per row
};
// One tile of kTile scores per workgroup while that keeps the chip busy (a call is latency-bound
// then); with many rows a workgroup takes several tiles, so that the fixed work per workgroup
// (prefix resolution, histogram flush) is paid by fewer of them.
__host__ inline TopkPlan topk_plan(int64_t n, int batch) {
  const int64_t tiles = (n + kTile - 1) / kTile;
  int64_t sub = (tiles * batch + 767) / 768;
  sub = sub < 1 ? 1 : (sub > 8 ? 8 : sub);
  TopkPlan p;
  p.sub = sub;
  p.nblk = (tiles + sub - 1) / sub;
  return p;
}
__host__ inline int64_t topk_row_words(const TopkPlan& p) {
  const int64_t cand_words = (p.nblk * p.sub * kTile + 1) / 2;
  return TopkLayout::blk + 2 * p.nblk + cand_words;
}

// Inclusive prefix sum over the 64 lanes of a wave in the vector unit: shifts inside the 16-lane rows, then the
// last lane of row 0 / 2 is added into row 1 / 3 and lane 31 into the upper half (every lane of the wave must be
// active).  The LDS-routed shuffles this replaces cost a crossbar round trip per step.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, false);   // row_shr:1 (lanes without a source add 0)
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, false);   // row_shr:2
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, false);   // row_shr:4
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, false);   // row_shr:8
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);   // row_bcast:15 into rows 1 and 3
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);   // row_bcast:31 into rows 2 and 3
  return v;
}

// Exclusive prefix sums of two values per thread over the block (one pair of barriers for both); *total_a and
// *total_b get the block sums.  wave_sums: 2 * kThreads / 64 words.
__device__ __forceinline__ void block_excl_scan2(uint32_t a, uint32_t b, uint32_t* before_a, uint32_t* before_b,
                                                 uint32_t* total_a, uint32_t* total_b, uint32_t* wave_sums) {
  constexpr int kWavesPerBlock = kThreads / 64;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const uint32_t ia = wave_incl_scan(a), ib = wave_incl_scan(b);
  __syncthreads();                       // wave_sums may still be read from a previous call
  if (lane == 63) {
    wave_sums[w] = ia;
    wave_sums[kWavesPerBlock + w] = ib;
  }
  __syncthreads();
  uint32_t base_a = 0, tot_a = 0, base_b = 0, tot_b = 0;
#pragma unroll
  for (int i = 0; i < kWavesPerBlock; ++i) {
    const uint32_t sa = wave_sums[i], sb = wave_sums[kWavesPerBlock + i];
    if (i < w) {
      base_a += sa;
      base_b += sb;
    }
    tot_a += sa;
    tot_b += sb;
  }
  *total_a = tot_a;
  *total_b = tot_b;
  *before_a = base_a + ia - a;
  *before_b = base_b + ib - b;
}

// Exclusive prefix sum of one value per thread over the block; *total gets the block sum.
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* total, uint32_t* wave_sums) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const uint32_t incl = wave_incl_scan(v);
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
  // unconditional loads (a position past the end reads score 0 instead): both are in flight together, and with
  // the histogram loads that follow, rather than one round trip each behind a branch
  float v[kItems];
#pragma unroll
  for (int e = 0; e < kItems; ++e) {
    const int64_t i = first + e;
    ok[e] = i < n;
    v[e] = row[ok[e] ? i : 0];
  }
#pragma unroll
  for (int e = 0; e < kItems; ++e) key[e] = ok[e] ? ordered_key(v[e]) : 0u;
}

// One thread's share of a finished 2048-bin histogram; thread 0 owns the highest bins.
constexpr int kBinsPerThread = kBins / kThreads;
struct BinSlice {
  uint32_t c[kBinsPerThread];
};
__device__ __forceinline__ BinSlice load_slice(const uint32_t* __restrict__ gh) {   // gh: [kHistReplicas][kBins]
  static_assert(kBinsPerThread == 4, "one 16-byte load per copy");
  BinSlice s;
  const uint4* lowest = (const uint4*)gh + (kThreads - 1 - threadIdx.x);      // bins top-3 .. top of this thread
  uint4 c[kHistReplicas];
#pragma unroll
  for (int r = 0; r < kHistReplicas; ++r) c[r] = lowest[r * (kBins / 4)];
  uint4 t = c[0];
#pragma unroll
  for (int r = 1; r < kHistReplicas; ++r) {
    t.x += c[r].x; t.y += c[r].y; t.z += c[r].z; t.w += c[r].w;
  }
  s.c[0] = t.w; s.c[1] = t.z; s.c[2] = t.y; s.c[3] = t.x;
  return s;
}

// Where rank k_rem falls in a histogram, walking from the top bin down: the bin, and the rank
// inside that bin.  Every thread of the block gets the result.
struct BinPick {
  uint32_t bin, k_rem;
};
__device__ __forceinline__ BinPick pick_bin(const BinSlice& sl, uint32_t k_rem, uint32_t* wave_sums,
                                            uint32_t* result) {
  const int top = kBins - 1 - threadIdx.x * kBinsPerThread;
  uint32_t mine = 0;
#pragma unroll
  for (int e = 0; e < kBinsPerThread; ++e) mine += sl.c[e];
  uint32_t total;
  const uint32_t above = block_excl_scan(mine, &total, wave_sums);
  if (above < k_rem && k_rem <= above + mine) {          // exactly one thread
    uint32_t cum = above;
    bool done = false;
#pragma unroll
    for (int e = 0; e < kBinsPerThread; ++e) {
      if (!done && cum + sl.c[e] >= k_rem) {
        result[0] = (uint32_t)(top - e);
        result[1] = k_rem - cum;
        done = true;
      }
      cum += sl.c[e];
    }
  }
  __syncthreads();
  BinPick r;
  r.bin = result[0];
  r.k_rem = result[1];
  __syncthreads();                       // result[] is free for the next pick
  return r;
}

// Key bits fixed by the passes before PASS, and the rank still to find below them.  All
// histogram loads are issued before the first scan, so they cost one round trip together.
// A pass picks one histogram itself (the one the pass before it filled) and reads what the earlier passes
// picked from the workspace, where the pass that made the pick left it (every workgroup writes the same
// two words).
template <int PASS>
__device__ __forceinline__ void resolve_prefix(uint32_t* __restrict__ w, uint32_t k, uint32_t* wave_sums,
                                               uint32_t* result, uint32_t* prefix, uint32_t* k_rem) {
  uint32_t p = 0, kr = k;
  if (PASS == 0) {
    *prefix = 0;
    *k_rem = k;
    return;
  }
  const BinSlice sl = load_slice(w + TopkLayout::hist + (PASS - 1) * kHistReplicas * kBins);
  uint32_t b0 = 0, k0 = 0, b1 = 0, k1 = 0;
  if (PASS >= 2) {
    b0 = w[TopkLayout::pick + 0];
    k0 = w[TopkLayout::pick + 1];
  }
  if (PASS >= 3) {
    b1 = w[TopkLayout::pick + 2];
    k1 = w[TopkLayout::pick + 3];
  }
  if (PASS == 1) {
    const BinPick b = pick_bin(sl, k, wave_sums, result);
    if (threadIdx.x == 0) {
      w[TopkLayout::pick + 0] = b.bin;
      w[TopkLayout::pick + 1] = b.k_rem;
    }
    p = b.bin << 21;
    kr = b.k_rem;
  } else if (PASS == 2) {
    const BinPick b = pick_bin(sl, k0, wave_sums, result);
    if (threadIdx.x == 0) {
      w[TopkLayout::pick + 2] = b.bin;
      w[TopkLayout::pick + 3] = b.k_rem;
    }
    p = (b0 << 21) | (b.bin << 10);
    kr = b.k_rem;
  } else {
    const BinPick b = pick_bin(sl, k1, wave_sums, result);
    p = (b0 << 21) | (b1 << 10) | b.bin;
    kr = b.k_rem;
  }
  *prefix = p;
  *k_rem = kr;
}

__global__ void topk_init(uint32_t* ws, int64_t row_words) {
  uint32_t* w = ws + (int64_t)blockIdx.y * row_words;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < kHistWords; i += gridDim.x * blockDim.x) w[i] = 0u;
}

// PASS 0: bits 31..21, PASS 1: bits 20..10, PASS 2: bits 9..0.
template <int PASS>
__global__ __launch_bounds__(kThreads) void topk_hist(const float* __restrict__ score, int64_t n, int64_t score_bs,
                                                      uint32_t* __restrict__ ws, int64_t row_words, int nblk,
                                                      uint32_t k, int sub) {
  __shared__ uint32_t h[kBins];
  __shared__ uint32_t wave_sums[kThreads / 64];
  __shared__ uint32_t result[2];
  __shared__ uint32_t n_above, n_cand;             // PASS 2: this workgroup's scores above / sharing the prefix
  const float* row = score + (int64_t)blockIdx.y * score_bs;
  uint32_t* w = ws + (int64_t)blockIdx.y * row_words;
  const int64_t first = (int64_t)blockIdx.x * kTile * sub + (int64_t)threadIdx.x * kItems;
  uint32_t key[kItems];
  bool ok[kItems];
  load_keys(row, n, first, key, ok);
  for (int i = threadIdx.x; i < kBins; i += kThreads) h[i] = 0u;
  if (threadIdx.x == 0) {
    n_above = 0u;
    n_cand = 0u;
  }
  uint32_t prefix, k_rem;
  resolve_prefix<PASS>(w, k, wave_sums, result, &prefix, &k_rem);
  __syncthreads();
  uint16_t* cand = (uint16_t*)(w + TopkLayout::blk + 2 * nblk) + (int64_t)blockIdx.x * kTile * sub;
  uint32_t above = 0;
  for (int st = 0; st < sub; ++st) {               // `sub` tiles of kTile scores, one histogram
    if (st > 0) load_keys(row, n, first + (int64_t)st * kTile, key, ok);
#pragma unroll
    for (int e = 0; e < kItems; ++e) {
      if (PASS == 0) {
        hist_add(h, ok[e], key[e] >> 21);
      } else if (PASS == 1) {
        hist_add(h, ok[e] && (key[e] >> 21) == (prefix >> 21), (key[e] >> 10) & 2047u);
      } else {
        const bool shares = ok[e] && (key[e] >> 10) == (prefix >> 10);
        hist_add(h, shares, key[e] & 1023u);
        above += (ok[e] && (key[e] >> 10) > (prefix >> 10)) ? 1u : 0u;
        if (shares) cand[atomicAdd(&n_cand, 1u)] = (uint16_t)(key[e] & 1023u);   // order does not matter: they are counted
      }
    }
  }
  if (PASS == 2) {
    above = wave_incl_scan(above);                 // lane 63 holds the wave's total
    if ((threadIdx.x & 63) == 63) atomicAdd(&n_above, above);
  }
  __syncthreads();
  hist_flush(w + TopkLayout::hist + PASS * kHistReplicas * kBins, h, blockIdx.x, threadIdx.x, kThreads);
  if (PASS == 2 && threadIdx.x == 0) {
    w[TopkLayout::blk + blockIdx.x] = n_above;
    w[TopkLayout::blk + nblk + blockIdx.x] = n_cand;
  }
}

__global__ __launch_bounds__(kThreads) void topk_write(const float* __restrict__ score, int64_t n, int64_t score_bs,
                                                       uint32_t* __restrict__ ws, int64_t row_words, int nblk,
                                                       int64_t base, int32_t* __restrict__ idx, int64_t idx_bs,
                                                       uint32_t k, int sub) {
  __shared__ uint32_t wave_sums[2 * kThreads / 64];
  __shared__ uint32_t result[2];
  const float* row = score + (int64_t)blockIdx.y * score_bs;
  uint32_t* w = ws + (int64_t)blockIdx.y * row_words;
  int32_t* out = idx + (int64_t)blockIdx.y * idx_bs;
  const int64_t first0 = (int64_t)blockIdx.x * kTile * sub + (int64_t)threadIdx.x * kItems;
  uint32_t key[kItems];
  bool ok[kItems];
  load_keys(row, n, first0, key, ok);
  // What the third histogram pass left about the first workgroup this thread looks at: requested
  // before T is resolved, so that the two round trips overlap.
  constexpr int kPeek = 4;
  const uint16_t* cand_all = (const uint16_t*)(w + TopkLayout::blk + 2 * nblk);
  const int64_t cap = (int64_t)kTile * sub;
  uint32_t c0 = 0, above0 = 0, peek[kPeek];
#pragma unroll
  for (int j = 0; j < kPeek; ++j) peek[j] = 0u;
  if ((int)threadIdx.x < (int)blockIdx.x) {
    above0 = w[TopkLayout::blk + threadIdx.x];
    c0 = w[TopkLayout::blk + nblk + threadIdx.x];
    // read whether or not that workgroup left so many (its slots exist either way; the count decides below what
    // is used): asking for the count first would put a second round trip in front of them
    static_assert(kPeek <= kTile, "a workgroup's candidate slots");
#pragma unroll
    for (int j = 0; j < kPeek; ++j) peek[j] = cand_all[threadIdx.x * cap + j];
  }
  uint32_t T, need;                                      // need: equal-to-T scores to take, lowest positions first
  resolve_prefix<3>(w, k, wave_sums, result, &T, &need);
  // scores above / equal to T in the workgroups before this one: those above the 22-bit prefix, plus
  // those sharing it whose last digit is above / equal to T's
  const uint32_t t_digit = T & 1023u;
  uint32_t my_gt = 0, my_eq = 0;
  for (int i = threadIdx.x; i < (int)blockIdx.x; i += kThreads) {
    const bool head = i == (int)threadIdx.x;
    uint32_t c = head ? c0 : w[TopkLayout::blk + nblk + i];
    c = c < (uint32_t)cap ? c : (uint32_t)cap;           // a workgroup cannot have left more than its scores: the reads below stay inside its slots
    my_gt += head ? above0 : w[TopkLayout::blk + i];
    uint32_t j0 = 0;
    if (head) {
#pragma unroll
      for (int j = 0; j < kPeek; ++j) {
        my_gt += ((uint32_t)j < c && peek[j] > t_digit) ? 1u : 0u;
        my_eq += ((uint32_t)j < c && peek[j] == t_digit) ? 1u : 0u;
      }
      j0 = kPeek;
    }
    for (uint32_t j = j0; j < c; ++j) {
      const uint32_t dgt = cand_all[i * cap + j];
      my_gt += dgt > t_digit ? 1u : 0u;
      my_eq += dgt == t_digit ? 1u : 0u;
    }
  }
  uint32_t off_gt, off_eq, unused_a, unused_b;
  block_excl_scan2(my_gt, my_eq, &unused_a, &unused_b, &off_gt, &off_eq, wave_sums);
  for (int st = 0; st < sub; ++st) {                     // tiles in position order; the offsets run on
    const int64_t first = first0 + (int64_t)st * kTile;
    if (st > 0) load_keys(row, n, first, key, ok);
    uint32_t gt = 0, eq = 0;
#pragma unroll
    for (int e = 0; e < kItems; ++e) {
      gt += (ok[e] && key[e] > T) ? 1u : 0u;
      eq += (ok[e] && key[e] == T) ? 1u : 0u;
    }
    uint32_t tot_g, tot_e, g_before, e_before;
    block_excl_scan2(gt, eq, &g_before, &e_before, &tot_g, &tot_e, wave_sums);
    g_before += off_gt;
    e_before += off_eq;
#pragma unroll
    for (int e = 0; e < kItems; ++e) {
      if (!ok[e]) continue;
      const bool is_gt = key[e] > T, is_eq = key[e] == T;
      if (is_gt || (is_eq && e_before < need)) {
        const uint32_t slot = g_before + (e_before < need ? e_before : need);
        if (slot < k) out[slot] = (int32_t)(base + first + e);
      }
      g_before += is_gt ? 1u : 0u;
      e_before += is_eq ? 1u : 0u;
    }
    off_gt += tot_g;
    off_eq += tot_e;
  }
}

// k >= n: every middle token is selected.
__global__ void topk_all(int64_t n, int64_t base, int32_t* idx, int64_t idx_bs) {
  int32_t* out = idx + (int64_t)blockIdx.y * idx_bs;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    out[i] = (int32_t)(base + i);
}

}  // namespace

// ---------------------------------------------------------------- library-owned scratch (no caller workspace)
// For callers that cannot allocate.  One array per GPU, held until the process ends; every call on
// a GPU shares it, so calls that overlap in time on one GPU race.  In host code the array's name is
// only a handle: its device address is looked up once per device and that address is what the
// kernels are given.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_addr[kMaxDevices];

// Device address of `scratch` on the current device (looked up on first use).
static int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_failed(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) ESA_FAIL(ESA_EUNSUPPORTED, "device ordinal %d beyond %d", dev, kMaxDevices - 1);
  void* p = g_scratch_addr[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return hip_failed(e, "hipGetSymbolAddress(scratch)");
    g_scratch_addr[dev].store(p, std::memory_order_release);     // every thread finds the same address
  }
  *out = p;
  return ESA_OK;
}

size_t topk_static_capacity() { return kStaticScratchBytes; }

int topk_static_prepare() {
  void* p;
  return static_scratch(&p);
}

int launch_topk_static(const float* score, int64_t n, int k, int64_t base, int32_t* idx, int batch, int64_t score_bs,
                       int64_t idx_bs, hipStream_t st) {
  const size_t need = topk_workspace_bytes(n, k, batch);
  if (need > kStaticScratchBytes)
    ESA_FAIL(ESA_EWORKSPACE, "esa_select_topk_static: %lld scores x %d rows need %zu bytes of scratch, the library holds %zu",
             (long long)n, batch, need, kStaticScratchBytes);
  void* ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc != ESA_OK) return rc;
  return launch_topk(score, n, k, base, idx, batch, score_bs, idx_bs, ws, kStaticScratchBytes, st, false);
}

size_t topk_workspace_bytes(int64_t n, int k, int batch) {
  if (n <= 0 || k <= 0 || batch <= 0 || k >= n) return 256;
  return align_up((size_t)topk_row_words(topk_plan(n, batch)) * sizeof(uint32_t), 256) * (size_t)batch;
}

int64_t topk_row_stride_words(int64_t n, int batch) {
  return (int64_t)(align_up((size_t)topk_row_words(topk_plan(n, batch)) * sizeof(uint32_t), 256) / sizeof(uint32_t));
}

int launch_topk(const float* score, int64_t n, int k, int64_t base, int32_t* idx, int batch, int64_t score_bs,
                int64_t idx_bs, void* ws, size_t ws_bytes, hipStream_t st, bool first_hist_ready) {
  if (k >= n) {
    const int blocks = (int)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
    topk_all<<<dim3(blocks, batch), 256, 0, st>>>(n, base, idx, idx_bs);
    ESA_LAUNCH_CHECK("topk_all");
    return ESA_OK;
  }
  const TopkPlan plan = topk_plan(n, batch);
  const int sub = (int)plan.sub, nblk = (int)plan.nblk;
  const int64_t row_words = topk_row_stride_words(n, batch);
  uint32_t* w = (uint32_t*)ws;
  const dim3 grid(nblk, batch);
  if (!first_hist_ready) {     // otherwise the score call has zeroed the histograms and filled the first one
    topk_init<<<dim3(3 * kHistReplicas, batch), 1024, 0, st>>>(w, row_words);
    topk_hist<0><<<grid, kThreads, 0, st>>>(score, n, score_bs, w, row_words, nblk, (uint32_t)k, sub);
  }
  topk_hist<1><<<grid, kThreads, 0, st>>>(score, n, score_bs, w, row_words, nblk, (uint32_t)k, sub);
  topk_hist<2><<<grid, kThreads, 0, st>>>(score, n, score_bs, w, row_words, nblk, (uint32_t)k, sub);
  topk_write<<<grid, kThreads, 0, st>>>(score, n, score_bs, w, row_words, nblk, base, idx, idx_bs, (uint32_t)k, sub);
  ESA_LAUNCH_CHECK("topk");
  return ESA_OK;
}

}  // namespace esa
