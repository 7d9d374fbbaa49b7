// Selected attention (Eq. 1) on the matrix cores: bf16 storage, head size 128.
//
// Work decomposition.  The query heads of one KV group share keys and values, so a workgroup
// owns 256 "rows" = (heads of one KV group) x (256/G consecutive current tokens) and one slice of
// the virtual key sequence [I | M_k | L | C]; slices of one row tile are merged afterwards with
// the log-sum-exp rule of Algorithm 1 (esa_attend_merge).  Eight waves of 32 rows each, two waves
// per SIMD, so that one wave's softmax arithmetic overlaps the other's matrix instructions; the
// kernel stays under 256 registers per lane for that.  Workgroups are numbered so that all
// workgroups of one (batch element, KV head) land on the same XCD and share its L2.
//
// Matrix-core formulation (v_mfma_f32_32x32x16_bf16, D[32x32] += A[32x16] B[16x32]; lane l feeds
// A row l%32 / B column l%32 with eight consecutive reduction elements chosen by l/32, and owns
// D[8*(v/4) + 4*(l/32) + v%4][l%32] in accumulator register v).  Both products are computed
// transposed so that a lane always stands for one query:
//     S^T [keys x queries] = K_tile [keys x d] . Q^T [d x queries]        A = K (LDS), B = Q (registers)
//     O^T [d x queries]   += V_tile^T [d x keys] . P^T [keys x queries]   A = V^T (LDS), B = P (registers)
// so the softmax over keys is an in-lane reduction over accumulator registers plus one exchange
// between the two half-waves, and S^T's accumulator layout is directly P^T's B-operand layout once
// the reduction slots of the second product are assigned to keys accordingly (the V^T tile is
// stored in LDS in that key order).  V is transposed on its way from global memory to LDS in
// registers (4x4 blocks of bf16), K is copied as is.  Tiles of 64 keys are double buffered in LDS:
// one barrier per tile, the next tile's global loads in flight during the current tile's math.
#include "attend_mfma.h"
#include "keyspace.h"

namespace esa {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kD = 128;             // head size
constexpr int kKT = 64;             // virtual keys per tile
constexpr int kRows = 256;          // query rows per workgroup
constexpr int kWaves = 8;
constexpr int kThreads = 64 * kWaves;
constexpr int kKLd = kD + 8;        // LDS row stride of the K tile in elements (272 B: conflict-free 16-byte reads)
constexpr int kVLd = kKT + 8;       // LDS row stride of the V^T tile in elements (144 B)
constexpr int kKElems = kKT * kKLd;
constexpr int kVElems = kD * kVLd;
constexpr int kStageElems = kKElems + kVElems;
constexpr int kLdsBytes = 2 * kStageElems * 2;
constexpr int kMaxSplits = 8;
constexpr int kMaxSlots = 2 * kMaxSplits;   // two-call form: local slices, then selected slices
constexpr int kMinLc = 16;          // shorter chunks go to the plain kernel
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLazy = 8.f;        // the softmax reference lags the running maximum by at most 2^8
constexpr float kLn2 = 0.6931471805599453f;

struct AttendArgs {
  const bf16_t* q;
  bf16_t* out;
  float* lse;
  uint16_t* part_o;   // [batch][n_slot][l_c][h][128] fp16 partial outputs, each normalised by its own sum
  float* part_ml;     // [batch][n_slot][l_c][h][2]   running maximum (log2 domain) and sum
  const char* k_cache;
  const char* v_cache;
  const char* k_sel;
  const char* v_sel;
  uint32_t tok_bytes, sel_bytes;    // row strides of the cache / the gathered buffers
  uint32_t i_end, n_sel, l_start;
  int l_c, h, h_kv, group, qpt, n_qt, n_split, batch;
  int xcd_mapping;                  // 1: (batch, KV head) pairs are a multiple of 8
  uint32_t n_fixed;
  int with_chunk;     // 1: the virtual sequence ends with the current chunk (causal); 0: every key is visible to every row
  int slot0, n_slot;  // partial results go to slots [slot0, slot0 + n_split) of n_slot
  int to_slots;       // 1: write partial results even when n_split == 1
  float c2;           // scale * log2(e)
  int64_t q_bs, out_bs, cache_bs_bytes, sel_bs_bytes;
};

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 f = {lo, hi};
  bf16x2 b = __builtin_convertvector(f, bf16x2);
  return *(uint32_t*)&b;
}

__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
  f16x2 h = {(_Float16)lo, (_Float16)hi};
  return *(uint32_t*)&h;
}

// Row of virtual key j: which buffer, and the byte offset inside it (branch-free).
struct RowRef {
  bool in_sel;
  uint64_t off;
};
__device__ __forceinline__ RowRef row_ref(const AttendArgs& a, uint32_t j) {
  const bool in_i = j < a.i_end;
  const bool in_s = !in_i && (j < a.i_end + a.n_sel);
  const uint32_t row = in_i ? j : (in_s ? j - a.i_end : j - a.i_end - a.n_sel + a.l_start);
  RowRef r;
  r.in_sel = in_s;
  r.off = (uint64_t)row * (in_s ? a.sel_bytes : a.tok_bytes);
  return r;
}

__global__ __launch_bounds__(kThreads) void attend_mfma_bf16(AttendArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  bf16_t* lds = (bf16_t*)lds_raw;     // [2 stages][K tile | V^T tile]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 31, hi = lane >> 5;

  // ---- which (batch element, KV head, row tile, key slice) is this workgroup
  const int per_pair = a.n_qt * a.n_split;
  int pair, inner;
  if (a.xcd_mapping) {                 // consecutive workgroup ids go to consecutive XCDs
    const int xcd = blockIdx.x & 7, k = blockIdx.x >> 3;
    pair = xcd + 8 * (k / per_pair);
    inner = k % per_pair;
  } else {
    pair = blockIdx.x / per_pair;
    inner = blockIdx.x % per_pair;
  }
  const int b = pair / a.h_kv, g = pair % a.h_kv;
  const int qt = inner % a.n_qt, split = inner / a.n_qt;

  const char* kc = a.k_cache + (int64_t)b * a.cache_bs_bytes + (int64_t)g * kD * 2;
  const char* vc = a.v_cache + (int64_t)b * a.cache_bs_bytes + (int64_t)g * kD * 2;
  const char* ksl = a.k_sel + (a.n_sel ? (int64_t)b * a.sel_bs_bytes + (int64_t)g * kD * 2 : 0);
  const char* vsl = a.v_sel + (a.n_sel ? (int64_t)b * a.sel_bs_bytes + (int64_t)g * kD * 2 : 0);

  // ---- this workgroup's rows and key slice
  const int q0 = qt * a.qpt;
  const int c_last = (q0 + a.qpt < a.l_c ? q0 + a.qpt : a.l_c) - 1;
  const uint32_t n_vis = a.n_fixed + (a.with_chunk ? c_last + 1 : 0);   // keys the tile's last token sees
  const uint32_t n_tiles = (n_vis + kKT - 1) / kKT;
  const uint32_t tile_begin = (uint32_t)((uint64_t)n_tiles * split / a.n_split);
  const uint32_t tile_end = (uint32_t)((uint64_t)n_tiles * (split + 1) / a.n_split);
  const uint32_t k_end = tile_end * kKT < n_vis ? tile_end * kKT : n_vis;

  // ---- this wave's 32 rows: one head, 32 consecutive current tokens, one per lane (both half-waves)
  const int tph = a.qpt / 32;                                      // 32-row tiles per head
  const int head = g * a.group + wave / tph;
  const int c = q0 + (wave % tph) * 32 + r;
  const bool c_ok = c < a.l_c;
  const int cc = c_ok ? c : a.l_c - 1;                             // rows past the chunk repeat its last token
  const uint32_t vis = a.n_fixed + (a.with_chunk ? cc + 1 : 0);
  const uint32_t lim = vis < k_end ? vis : k_end;                  // first virtual key this lane's query may NOT see
  const uint32_t lim_lo = __shfl(lim, 0, 64);                      // smallest limit in the wave (r = 0)
  bf16x8 qf[kD / 16];                                              // loaded below, behind the first tile's loads

  f32x16 o[4];
#pragma unroll
  for (int md = 0; md < 4; ++md)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[md][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  // ---- staging of one tile: global -> registers -> LDS.  K: two 16-byte pieces per thread
  // (key = piece / 16, 16 pieces per 256-byte row).  V: one 4-key x 4-dim block per thread.
  uint4 k0, k1;
  uint2 v0, v1, v2, v3;
  const int kp0 = tid, kp1 = tid + kThreads;
  const int vb = (lane >> 3) + 8 * (wave & 3);                     // which 4 head-dims (0..31)
  const int ap = (lane & 7) + 8 * (wave >> 2);                     // 4-key group as stored in LDS (0..15)
  const int sw = ap & 3;
  const int ag = (ap & ~3) | (sw == 1 ? 2 : sw == 2 ? 1 : sw);     // 4-key group in key order
  // Per-thread row numbers inside a tile.  A tile whose 64 keys lie inside one segment of the
  // virtual sequence (the usual case) is addressed as uniform base + row * stride + column, the base
  // and stride chosen on the scalar unit; tiles that straddle a segment boundary or the end of
  // the slice take the general per-row path.
  const uint32_t kr0 = kp0 >> 4, kr1 = kp1 >> 4, kcol0 = (kp0 & 15) * 16, kcol1 = (kp1 & 15) * 16;
  const uint32_t vr = 4 * ag, vcol = vb * 8;
  auto k_src = [&](uint32_t j0, int piece) -> const uint4* {
    uint32_t j = j0 + (piece >> 4);
    j = j < k_end ? j : k_end - 1;                                 // the tail repeats a key; masked below
    const RowRef rr = row_ref(a, j);
    return (const uint4*)((rr.in_sel ? ksl : kc) + rr.off + (piece & 15) * 16);
  };
  auto v_src = [&](uint32_t j0, int kk) -> const uint2* {
    uint32_t j = j0 + 4 * ag + kk;
    j = j < k_end ? j : k_end - 1;
    const RowRef rr = row_ref(a, j);
    return (const uint2*)((rr.in_sel ? vsl : vc) + rr.off + vb * 8);
  };
  auto tile_load = [&](uint32_t j0) {
    const uint32_t sel_end = a.i_end + a.n_sel;
    int seg = -1;                                                  // 0: cache rows, 1: gathered rows
    uint32_t row0 = 0;
    if (j0 + kKT <= a.i_end) {
      seg = 0;
      row0 = j0;
    } else if (j0 >= a.i_end && j0 + kKT <= sel_end) {
      seg = 1;
      row0 = j0 - a.i_end;
    } else if (j0 >= sel_end && j0 + kKT <= k_end) {
      seg = 0;
      row0 = j0 - sel_end + a.l_start;
    }
    if (seg >= 0) {
      const uint32_t stride = seg ? a.sel_bytes : a.tok_bytes;
      const char* kb = (seg ? ksl : kc) + (uint64_t)row0 * stride;
      const char* vbase = (seg ? vsl : vc) + (uint64_t)row0 * stride;
      k0 = *(const uint4*)(kb + (kr0 * stride + kcol0));
      k1 = *(const uint4*)(kb + (kr1 * stride + kcol1));
      v0 = *(const uint2*)(vbase + (vr * stride + vcol));
      v1 = *(const uint2*)(vbase + ((vr + 1) * stride + vcol));
      v2 = *(const uint2*)(vbase + ((vr + 2) * stride + vcol));
      v3 = *(const uint2*)(vbase + ((vr + 3) * stride + vcol));
    } else {
      k0 = *k_src(j0, kp0);
      k1 = *k_src(j0, kp1);
      v0 = *v_src(j0, 0);
      v1 = *v_src(j0, 1);
      v2 = *v_src(j0, 2);
      v3 = *v_src(j0, 3);
    }
  };
#define ESA_TILE_LOAD(j0) tile_load(j0)
  auto tile_store = [&](int stage) {
    bf16_t* kt = lds + stage * kStageElems;
    bf16_t* vt = kt + kKElems;
    *(uint4*)&kt[(kp0 >> 4) * kKLd + (kp0 & 15) * 8] = k0;
    *(uint4*)&kt[(kp1 >> 4) * kKLd + (kp1 & 15) * 8] = k1;
    // 4 keys x 4 dims -> 4 dims x 4 keys
    uint2 d0, d1, d2, d3;
    d0.x = (v0.x & 0xFFFFu) | (v1.x << 16);
    d0.y = (v2.x & 0xFFFFu) | (v3.x << 16);
    d1.x = (v0.x >> 16) | (v1.x & 0xFFFF0000u);
    d1.y = (v2.x >> 16) | (v3.x & 0xFFFF0000u);
    d2.x = (v0.y & 0xFFFFu) | (v1.y << 16);
    d2.y = (v2.y & 0xFFFFu) | (v3.y << 16);
    d3.x = (v0.y >> 16) | (v1.y & 0xFFFF0000u);
    d3.y = (v2.y >> 16) | (v3.y & 0xFFFF0000u);
    bf16_t* dst = &vt[(4 * vb) * kVLd + 4 * ap];
    *(uint2*)(dst) = d0;
    *(uint2*)(dst + kVLd) = d1;
    *(uint2*)(dst + 2 * kVLd) = d2;
    *(uint2*)(dst + 3 * kVLd) = d3;
  };

  // The first tile's loads go out before the query fragments' so that the two round trips overlap.
  if (tile_begin < tile_end) ESA_TILE_LOAD(tile_begin * kKT);
  {
    const bf16_t* qp = a.q + (int64_t)b * a.q_bs + ((int64_t)cc * a.h + head) * kD + hi * 8;
#pragma unroll
    for (int ks16 = 0; ks16 < kD / 16; ++ks16) qf[ks16] = *(const bf16x8*)(qp + ks16 * 16);
    // Pin the fragments as arrived values here: otherwise every use inside the tile loop carries a
    // wait on the vector-memory counter, which would also wait for the tile loads just issued.
#pragma unroll
    for (int ks16 = 0; ks16 < kD / 16; ++ks16) asm volatile("" : "+v"(qf[ks16]));
  }
  if (tile_begin < tile_end) tile_store(0);
  for (uint32_t t = tile_begin; t < tile_end; ++t) {
    const uint32_t j0 = t * kKT;
    const int stage = (int)((t - tile_begin) & 1);
    __syncthreads();                     // tile t is in LDS; every wave is done with tile t-1
    if (t + 1 < tile_end) ESA_TILE_LOAD(j0 + kKT);
    const bf16_t* kt = lds + stage * kStageElems;
    const bf16_t* vt = kt + kKElems;

    // ---- S^T = K Q^T
    f32x16 s[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int v = 0; v < 16; ++v) s[mt][v] = 0.f;
#pragma unroll
    for (int ks16 = 0; ks16 < kD / 16; ++ks16)
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        const bf16x8 ka = *(const bf16x8*)&kt[(32 * mt + r) * kKLd + 16 * ks16 + 8 * hi];
        s[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[ks16], s[mt], 0, 0, 0);
      }

    // ---- mask keys beyond each query's limit (causal diagonal, end of the slice)
    if (j0 + kKT > lim_lo) {
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const uint32_t j = j0 + 32 * mt + 8 * (v / 4) + 4 * hi + (v % 4);
          if (j >= lim) s[mt][v] = -INFINITY;
        }
    }

    // ---- online softmax, one query per lane
    float mx = s[0][0];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[mt][v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    // The reference m_run of the exponentials follows the running maximum lazily: it moves only when
    // a tile's maximum exceeds it by more than 2^kLazy, so probabilities stay below 2^kLazy (harmless
    // in bf16 and fp32) and the accumulators are rescaled once or twice per row instead of per tile.
    const float cand = mx * a.c2;
    const float m_new = cand > m_run + kLazy ? cand : m_run;
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float corr = __builtin_amdgcn_exp2f(m_run - m_use);
    m_run = m_new;
    float psum = 0.f;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[mt][v], a.c2, -m_use));
        s[mt][v] = p;
        psum += p;
      }
    l_run = l_run * corr + psum;
    if (__ballot(corr != 1.f) != 0ull) {
#pragma unroll
      for (int md = 0; md < 4; ++md)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[md][v] *= corr;
    }
    bf16x8 pf[4];
#pragma unroll
    for (int kp = 0; kp < 4; ++kp) {
      const int mt = kp >> 1, e0 = (kp & 1) * 8;
      uint4 w;
      w.x = pack_bf16x2(s[mt][e0 + 0], s[mt][e0 + 1]);
      w.y = pack_bf16x2(s[mt][e0 + 2], s[mt][e0 + 3]);
      w.z = pack_bf16x2(s[mt][e0 + 4], s[mt][e0 + 5]);
      w.w = pack_bf16x2(s[mt][e0 + 6], s[mt][e0 + 7]);
      pf[kp] = *(bf16x8*)&w;
    }

    // ---- O^T += V^T P^T
#pragma unroll
    for (int kp = 0; kp < 4; ++kp)
#pragma unroll
      for (int md = 0; md < 4; ++md) {
        const bf16x8 va = *(const bf16x8*)&vt[(32 * md + r) * kVLd + 16 * kp + 8 * hi];
        o[md] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pf[kp], o[md], 0, 0, 0);
      }

    if (t + 1 < tile_end) tile_store(stage ^ 1);
  }
#undef ESA_TILE_LOAD

  // ---- results.  Accumulator register v of tile md is head-dim 32*md + 8*(v/4) + 4*hi + v%4 of this
  // lane's query, so a lane holds its whole output row in 8-byte pieces.  The rows are normalised,
  // narrowed to 16 bits and turned into whole 256-byte rows in LDS (free by now), from where each wave
  // writes its own 32 rows with fully coalesced 16-byte stores.  Final outputs are bf16; partial
  // results of a key slice are fp16 (normalised values are bounded by max |v|, and fp16's 11-bit
  // significand keeps their rounding well below that of the bf16 output) next to fp32 (maximum, sum).
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const bool final_out = a.n_split == 1 && !a.to_slots;
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  __syncthreads();                       // every wave is done with the last tile
  {
    uint16_t* ot = (uint16_t*)lds + (wave * 32 + r) * kKLd;
#pragma unroll
    for (int md = 0; md < 4; ++md)
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        uint2 w;
        if (final_out) {
          w.x = pack_bf16x2(o[md][4 * vg + 0] * inv, o[md][4 * vg + 1] * inv);
          w.y = pack_bf16x2(o[md][4 * vg + 2] * inv, o[md][4 * vg + 3] * inv);
        } else {
          w.x = pack_f16x2(o[md][4 * vg + 0] * inv, o[md][4 * vg + 1] * inv);
          w.y = pack_f16x2(o[md][4 * vg + 2] * inv, o[md][4 * vg + 3] * inv);
        }
        *(uint2*)(ot + 32 * md + 8 * vg + 4 * hi) = w;
      }
  }
  __syncthreads();
  const int c_wave = q0 + (wave % tph) * 32;                        // first current token of this wave's rows
  uint16_t* dst;
  if (final_out) {
    dst = (uint16_t*)a.out + (int64_t)b * a.out_bs + ((int64_t)c_wave * a.h + head) * kD;
  } else {
    const int64_t prow0 = ((int64_t)(b * a.n_slot + a.slot0 + split) * a.l_c) * a.h;
    dst = a.part_o + (prow0 + (int64_t)c_wave * a.h + head) * kD;
    if (hi == 0 && c_ok) {
      float2 ml = {m_run, l_tot};
      *(float2*)(a.part_ml + (prow0 + (int64_t)c * a.h + head) * 2) = ml;
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int rw = 4 * i + (lane >> 4), piece = lane & 15;
    if (c_wave + rw < a.l_c) {
      const uint4 w = *(const uint4*)((const uint16_t*)lds + (wave * 32 + rw) * kKLd + piece * 8);
      *(uint4*)(dst + (int64_t)rw * a.h * kD + piece * 8) = w;
    }
  }
  if (final_out && a.lse && hi == 0 && c_ok)
    a.lse[(int64_t)b * a.l_c * a.h + (int64_t)c * a.h + head] = (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2;
}

// Algorithm 1's merge over partial results: weights 2^(m_s - M) with the maximum subtracted first.
// The slots in use are [0, ns_a) and [slot_b, slot_b + ns_b) of n_slot.  32 lanes per row (four
// head-dims each), eight rows per workgroup.
__global__ __launch_bounds__(256) void esa_attend_merge(const uint16_t* __restrict__ part_o,
                                                        const float* __restrict__ part_ml, int n_slot, int ns_a,
                                                        int slot_b, int ns_b, int64_t rows, bf16_t* __restrict__ out,
                                                        float* __restrict__ lse, int64_t out_bs, int64_t lse_bs) {
  const int64_t row = (int64_t)blockIdx.x * 8 + (threadIdx.x >> 5);
  const int d4 = (threadIdx.x & 31) * 4;
  const int b = blockIdx.y;
  if (row >= rows) return;
  // Every load of the row goes out before the first use (one round trip): the slices' (maximum, sum)
  // pairs and their outputs.  A slice that saw no key of this row stored zeros and sum 0.
  float m[kMaxSlots], l[kMaxSlots];
  uint2 po[kMaxSlots];
#pragma unroll
  for (int s = 0; s < kMaxSlots; ++s) {
    m[s] = -INFINITY;
    l[s] = 0.f;
    po[s] = make_uint2(0u, 0u);
    if (s < ns_a || (s >= slot_b && s < slot_b + ns_b)) {
      const int64_t prow = ((int64_t)b * n_slot + s) * rows + row;
      const float2 ml = *(const float2*)(part_ml + prow * 2);
      m[s] = ml.x;
      l[s] = ml.y;
      po[s] = *(const uint2*)(part_o + prow * kD + d4);
    }
  }
  float M = -INFINITY;
#pragma unroll
  for (int s = 0; s < kMaxSlots; ++s) M = fmaxf(M, m[s]);
  float L = 0.f;
  float4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < kMaxSlots; ++s) {
    const float w = m[s] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m[s] - M) * l[s];   // outputs are normalised by the slice's sum
    const f16x2 p01 = *(const f16x2*)&po[s].x, p23 = *(const f16x2*)&po[s].y;
    L += w;
    acc.x += w * (float)p01[0];
    acc.y += w * (float)p01[1];
    acc.z += w * (float)p23[0];
    acc.w += w * (float)p23[1];
  }
  const float inv = 1.f / L;
  uint2 w2;
  w2.x = pack_bf16x2(acc.x * inv, acc.y * inv);
  w2.y = pack_bf16x2(acc.z * inv, acc.w * inv);
  *(uint2*)(out + (int64_t)b * out_bs + row * kD + d4) = w2;
  if (lse && d4 == 0) lse[(int64_t)b * lse_bs + row] = (M + __builtin_amdgcn_logf(L)) * kLn2;
}

int choose_splits(int l_c, int group, int h_kv, int batch) {
  const int qpt = kRows / group;
  const int64_t row_tiles = (int64_t)((l_c + qpt - 1) / qpt) * h_kv * batch;
  int64_t ns = (256 + row_tiles - 1) / row_tiles;
  return (int)(ns < 1 ? 1 : (ns > kMaxSplits ? kMaxSplits : ns));
}

}  // namespace

bool attend_mfma_supported(int l_c, int h, int h_kv, int d, int dtype) {
  if (dtype != ESA_BF16 || d != kD || l_c < kMinLc || h % h_kv != 0) return false;
  const int group = h / h_kv;
  return group == 1 || group == 2 || group == 4 || group == 8;
}

bool attend_mfma_aligned(const void* q, const void* k_cache, const void* v_cache, const void* k_sel,
                         const void* v_sel, const void* out, int64_t tok_stride, int64_t q_bs, int64_t cache_bs,
                         int64_t sel_bs, int64_t out_bs) {
  const uintptr_t p = (uintptr_t)q | (uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)k_sel | (uintptr_t)v_sel |
                      (uintptr_t)out;
  const int64_t s = tok_stride | q_bs | cache_bs | sel_bs | out_bs;
  return (p % 16 == 0) && (s % 8 == 0);
}

namespace {

// Planned slice counts.  One call: `all` slices of the whole virtual sequence.  Two calls: the local
// part [ I | L | C ] runs beside other work, so it gets fewer, longer slices than the selected part,
// which is on the critical path and should cover the chip by itself.
struct SplitPlan {
  int all, local, sel;
};
SplitPlan plan_splits(int l_c, int group, int h_kv, int batch) {
  SplitPlan p;
  p.all = choose_splits(l_c, group, h_kv, batch);
  p.sel = p.all;
  p.local = p.all > 1 ? p.all / 2 : 1;
  return p;
}

size_t slots_bytes(int n_slot, int l_c, int h, int batch) {
  const size_t rows = (size_t)batch * n_slot * l_c * h;
  return align_up(rows * kD * sizeof(uint16_t), 256) + align_up(rows * 2 * sizeof(float), 256);
}

}  // namespace

size_t attend_mfma_workspace_bytes(int l_c, int h, int h_kv, int d, int batch) {
  const SplitPlan p = plan_splits(l_c, h / h_kv, h_kv, batch);
  const int n_slot = p.local + p.sel > p.all ? p.local + p.sel : p.all;
  return slots_bytes(n_slot, l_c, h, batch);
}

int launch_attend_mfma(int part, int split, const void* q, int l_c, int h, int h_kv, int d, const void* k_cache,
                       const void* v_cache, int64_t tok_stride, int64_t t0, int64_t i_end, int64_t l_start,
                       const void* k_sel, const void* v_sel, int n_sel, float scale, void* out, float* lse, int batch,
                       int64_t q_bs, int64_t cache_bs, int64_t sel_bs, int64_t out_bs, void* ws, size_t ws_bytes,
                       hipStream_t st) {
  if (!(scale > 0.f)) ESA_FAIL(ESA_EINVAL, "esa_attend: scale must be positive");
  if (t0 + l_c >= ((int64_t)1 << 31) || tok_stride * 2 >= ((int64_t)1 << 32))
    ESA_FAIL(ESA_EUNSUPPORTED, "esa_attend: positions beyond 2^31 are not supported by the matrix-core kernel");
  AttendArgs a;
  a.q = (const bf16_t*)q;
  a.out = (bf16_t*)out;
  a.lse = lse;
  a.k_cache = (const char*)k_cache;
  a.v_cache = (const char*)v_cache;
  a.k_sel = (const char*)k_sel;
  a.v_sel = (const char*)v_sel;
  a.tok_bytes = (uint32_t)(tok_stride * 2);
  a.sel_bytes = (uint32_t)((int64_t)h_kv * d * 2);
  a.l_c = l_c;
  a.h = h;
  a.h_kv = h_kv;
  a.group = h / h_kv;
  a.qpt = kRows / a.group;
  a.n_qt = (l_c + a.qpt - 1) / a.qpt;
  a.batch = batch;
  a.c2 = scale * kLog2e;
  a.q_bs = q_bs;
  a.out_bs = out_bs;
  a.cache_bs_bytes = cache_bs * 2;
  a.sel_bs_bytes = sel_bs * 2;
  a.xcd_mapping = ((batch * h_kv) % 8 == 0) ? 1 : 0;

  const SplitPlan plan = plan_splits(l_c, a.group, h_kv, batch);
  const int first_rows = l_c < a.qpt ? l_c : a.qpt;
  auto clamp = [](int ns, int64_t keys_of_first_tile) {
    const int64_t tiles = (keys_of_first_tile + kKT - 1) / kKT;
    return (int)(ns > tiles ? (tiles > 0 ? tiles : 1) : ns);
  };
  // slices in use: one call -> `all`; two calls -> local in slots [0, ns_local), selected in [plan.local, +ns_sel)
  const int ns_all = clamp(plan.all, i_end + n_sel + (t0 - l_start) + first_rows);
  // split == ESA_SPLIT_ALGORITHM1 moves the initial tokens from the early part to the late one
  const int64_t i_early = split == ESA_SPLIT_ALGORITHM1 ? 0 : i_end, i_late = i_end - i_early;
  const int ns_local = clamp(plan.local, i_early + (t0 - l_start) + first_rows);
  const int ns_sel = i_late + n_sel > 0 ? clamp(plan.sel, i_late + n_sel) : 0;
  const int n_slot = part == kAttendAll ? ns_all : plan.local + plan.sel;

  a.part_o = nullptr;
  a.part_ml = nullptr;
  if (part != kAttendAll || ns_all > 1) {
    const size_t need = slots_bytes(n_slot, l_c, h, batch);
    if (!ws || ws_bytes < need) ESA_FAIL(ESA_EWORKSPACE, "esa_attend: workspace needs %zu bytes", need);
    const size_t rows = (size_t)batch * n_slot * l_c * h;
    a.part_o = (uint16_t*)ws;
    a.part_ml = (float*)((char*)ws + align_up(rows * kD * sizeof(uint16_t), 256));
  }
  a.n_slot = n_slot;
  static bool lds_limit_raised = false;          // idempotent; a race only repeats the call
  if (!lds_limit_raised) {
    hipError_t e = hipFuncSetAttribute((const void*)attend_mfma_bf16, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       kLdsBytes);
    if (e != hipSuccess) return hip_failed(e, "hipFuncSetAttribute(attend_mfma_bf16)");
    lds_limit_raised = true;
  }
  auto launch = [&](int64_t n_wg) { attend_mfma_bf16<<<dim3((unsigned)n_wg), kThreads, kLdsBytes, st>>>(a); };
  const int64_t rows = (int64_t)l_c * h;
  const dim3 merge_grid((unsigned)((rows + 7) / 8), batch);
  if (part == kAttendAll) {
    a.i_end = (uint32_t)i_end;
    a.n_sel = (uint32_t)n_sel;
    a.l_start = (uint32_t)l_start;
    a.n_fixed = (uint32_t)(i_end + n_sel + (t0 - l_start));
    a.with_chunk = 1;
    a.n_split = ns_all;
    a.slot0 = 0;
    a.to_slots = 0;
    launch((int64_t)batch * h_kv * a.n_qt * ns_all);
    if (ns_all > 1)
      esa_attend_merge<<<merge_grid, 256, 0, st>>>(a.part_o, a.part_ml, n_slot, ns_all, 0, 0, rows, (bf16_t*)out, lse,
                                                   out_bs, rows);
  } else if (part == kAttendLocal) {
    a.i_end = (uint32_t)i_early;
    a.n_sel = 0;
    a.l_start = (uint32_t)l_start;
    a.n_fixed = (uint32_t)(i_early + (t0 - l_start));
    a.with_chunk = 1;
    a.n_split = ns_local;
    a.slot0 = 0;
    a.to_slots = 1;
    launch((int64_t)batch * h_kv * a.n_qt * ns_local);
  } else {
    if (ns_sel > 0) {
      a.i_end = (uint32_t)i_late;
      a.n_sel = (uint32_t)n_sel;
      a.l_start = 0;
      a.n_fixed = (uint32_t)(i_late + n_sel);
      a.with_chunk = 0;
      a.n_split = ns_sel;
      a.slot0 = plan.local;
      a.to_slots = 1;
      launch((int64_t)batch * h_kv * a.n_qt * ns_sel);
    }
    esa_attend_merge<<<merge_grid, 256, 0, st>>>(a.part_o, a.part_ml, n_slot, ns_local, plan.local, ns_sel, rows,
                                                 (bf16_t*)out, lse, out_bs, rows);
  }
  ESA_LAUNCH_CHECK("attend_mfma");
  return ESA_OK;
}

}  // namespace esa
