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
// the reduction slots of the second product are assigned to keys accordingly.
//
// Tiles of 64 keys are double buffered in LDS and arrive there without passing through registers:
// global_load_lds_dwordx4 deposits 16 bytes per lane at consecutive LDS addresses, so one wave
// instruction brings four 256-byte rows, and which 16 bytes of its row a lane fetches is chosen
// such that the rows land XOR-swizzled (K: 16-byte pieces by row % 16, V: 64-byte chunks by
// row % 4), which makes the fragment reads below free of bank conflicts without padding.  K
// fragments are plain 16-byte reads.  V stays row-major [key][dim]; its transposed fragments (eight
// keys of one head dimension per lane) come from ds_read_b64_tr_b16, which hands lane i of a 16-lane
// group element i%4 of the 8 bytes addressed by lanes 4e + i/4 (e = 0..3): sixteen lanes that point
// at a 4-key x 16-dim block receive one dimension each, four consecutive keys of it.
// One barrier per tile; the next tile's loads are in flight during the current tile's math.
#include "attend_mfma.h"
#include "keyspace.h"

namespace esa {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef short i16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) i16x4 lds_i16x4;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void global_void;

constexpr int kD = 128;             // head size
constexpr int kKT = 64;             // virtual keys per tile
constexpr int kRows = 256;          // query rows per workgroup
constexpr int kWaves = 8;
constexpr int kThreads = 64 * kWaves;
constexpr int kTileElems = kKT * kD;    // one K or V tile in LDS: 64 rows of 256 bytes, unpadded, swizzled
constexpr int kMaxSplits = 8;
constexpr int kMaxSlots = 2 * kMaxSplits;   // two-call form: local slices, then selected slices
constexpr int kMinLc = 16;          // shorter chunks go to the plain kernel
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLazy = 8.f;        // the softmax reference lags the running maximum by at most 2^8
constexpr float kLn2 = 0.6931471805599453f;

// What one slice of a launch attends to: a query tensor and a virtual key sequence
// [ cache rows [0, i_end) | n_sel gathered rows | cache rows [l_start, ..) ].  A launch carries two views;
// the usual one uses view 0 only, the re-encoded attention of Section 3.2 gives the local keys (their own
// encoding of queries and keys, causal) to view 0 and the initial and selected keys (queries at the fixed
// position, every key visible) to view 1, so that both parts run in one launch.
struct KeyView {
  const bf16_t* q;
  const char* k_cache;
  const char* v_cache;
  int64_t q_bs, cache_bs_bytes;
  uint32_t tok_bytes;               // row stride of the cache
  uint32_t i_end, n_sel, l_start;
  uint32_t n_fixed;                 // keys every row sees
  const int32_t* sel_idx;           // not null: the n_sel selected rows are cache rows sel_idx[0..n_sel), not a gathered buffer
  int64_t idx_bs;                   // batch stride of the index list
  uint32_t idx_limit;               // indices are clamped into [0, idx_limit)
  int with_chunk;     // 1: the virtual sequence ends with the current chunk (causal); 0: every key is visible to every row
  int n_split;        // slices of this view (view 0's slices come first)
  int slot0;          // partial results of slice s go to slot slot0 + s
};

struct AttendArgs {
  KeyView view[2];
  bf16_t* out;
  float* lse;
  uint16_t* part_o;   // [batch][n_slot][l_c][h][128] fp16 partial outputs, un-normalised, scaled by 2^-E per row
  float* part_ml;     // [batch][n_slot][l_c][h][2]   softmax reference (log2 domain) + E, and sum * 2^-E
  const char* k_sel;
  const char* v_sel;
  uint32_t sel_bytes;               // row stride of the gathered buffers
  int l_c, h, h_kv, group, qpt, n_qt, batch;
  int xcd_mapping;                  // 1: (batch, KV head) pairs are a multiple of 8
  int n_slot;         // slots per row in the partial-result arrays
  int to_slots;       // 1: write partial results even when the launch has a single slice
  float c2;           // scale * log2(e)
  int64_t out_bs, sel_bs_bytes;
};

// Maximum / sum of a value over the two lanes 32 places apart: a lane swap in the vector unit.  (A general
// shuffle goes through the LDS crossbar, and the wait for it is a wait for every LDS read in flight.)
__device__ __forceinline__ float halves_max(float v) {
  const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));     // lower half's value, upper half's value
}
__device__ __forceinline__ float halves_sum(float v) {
  const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
}

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
__device__ __forceinline__ uint32_t clamped_index(const KeyView& V, const int32_t* sidx, uint32_t pos) {
  const int32_t v = sidx[pos];      // a middle token's position; clamped so that a bad index cannot leave the cache
  return v < 0 ? 0u : ((uint32_t)v < V.idx_limit ? (uint32_t)v : V.idx_limit - 1);
}
// sidx: this batch element's index list, or null when the selected rows come from the gathered buffer
__device__ __forceinline__ RowRef row_ref(const KeyView& V, const int32_t* sidx, uint32_t sel_bytes, uint32_t j) {
  const bool in_i = j < V.i_end;
  const bool in_s = !in_i && (j < V.i_end + V.n_sel);
  uint32_t row = in_i ? j : (in_s ? j - V.i_end : j - V.i_end - V.n_sel + V.l_start);
  RowRef r;
  r.in_sel = in_s && !sidx;
  if (in_s && sidx) row = clamped_index(V, sidx, row);
  r.off = (uint64_t)row * (r.in_sel ? sel_bytes : V.tok_bytes);
  return r;
}

__global__ __launch_bounds__(kThreads) void attend_mfma_bf16(AttendArgs a) {
  // Two stages of a K tile and a V tile.  Separate arrays, so that the compiler can tell a load into one
  // stage from a fragment read of the other and does not wait for the load first.
  __shared__ __attribute__((aligned(1024))) bf16_t k_st0[kTileElems];
  __shared__ __attribute__((aligned(1024))) bf16_t k_st1[kTileElems];
  __shared__ __attribute__((aligned(1024))) bf16_t v_st0[kTileElems];
  __shared__ __attribute__((aligned(1024))) bf16_t v_st1[kTileElems];

  const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, hi = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);        // uniform: scalar address arithmetic


  // ---- which (batch element, KV head, row tile, key slice) is this workgroup
  const int n_slices = a.view[0].n_split + a.view[1].n_split;
  const int per_pair = a.n_qt * n_slices;
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
  const int qt = inner % a.n_qt, slice = inner / a.n_qt;
  const int vw = slice >= a.view[0].n_split ? 1 : 0;             // which view this slice belongs to
  // field-wise select (not an indexed load): every kernel argument is then fetched in the first round trip
  KeyView V;
  {
    const KeyView &v0 = a.view[0], &v1 = a.view[1];
    V.q = vw ? v1.q : v0.q;
    V.k_cache = vw ? v1.k_cache : v0.k_cache;
    V.v_cache = vw ? v1.v_cache : v0.v_cache;
    V.q_bs = vw ? v1.q_bs : v0.q_bs;
    V.cache_bs_bytes = vw ? v1.cache_bs_bytes : v0.cache_bs_bytes;
    V.tok_bytes = vw ? v1.tok_bytes : v0.tok_bytes;
    V.i_end = vw ? v1.i_end : v0.i_end;
    V.n_sel = vw ? v1.n_sel : v0.n_sel;
    V.l_start = vw ? v1.l_start : v0.l_start;
    V.n_fixed = vw ? v1.n_fixed : v0.n_fixed;
    V.sel_idx = vw ? v1.sel_idx : v0.sel_idx;
    V.idx_bs = vw ? v1.idx_bs : v0.idx_bs;
    V.idx_limit = vw ? v1.idx_limit : v0.idx_limit;
    V.with_chunk = vw ? v1.with_chunk : v0.with_chunk;
    V.n_split = vw ? v1.n_split : v0.n_split;
    V.slot0 = vw ? v1.slot0 : v0.slot0;
  }
  const int split = slice - (vw ? a.view[0].n_split : 0);        // slice number inside the view

  const char* kc = V.k_cache + (int64_t)b * V.cache_bs_bytes + (int64_t)g * kD * 2;
  const char* vc = V.v_cache + (int64_t)b * V.cache_bs_bytes + (int64_t)g * kD * 2;
  const char* ksl = a.k_sel + (V.n_sel ? (int64_t)b * a.sel_bs_bytes + (int64_t)g * kD * 2 : 0);
  const char* vsl = a.v_sel + (V.n_sel ? (int64_t)b * a.sel_bs_bytes + (int64_t)g * kD * 2 : 0);

  // ---- this workgroup's rows and key slice
  const int q0 = qt * a.qpt;
  const int c_last = (q0 + a.qpt < a.l_c ? q0 + a.qpt : a.l_c) - 1;
  const uint32_t n_vis = V.n_fixed + (V.with_chunk ? c_last + 1 : 0);   // keys the tile's last token sees
  const uint32_t n_tiles = (n_vis + kKT - 1) / kKT;
  const uint32_t tile_begin = (uint32_t)((uint64_t)n_tiles * split / V.n_split);
  const uint32_t tile_end = (uint32_t)((uint64_t)n_tiles * (split + 1) / V.n_split);
  const uint32_t k_end = tile_end * kKT < n_vis ? tile_end * kKT : n_vis;

  // ---- this wave's 32 rows: one head, 32 consecutive current tokens, one per lane (both half-waves)
  const int tph = a.qpt / 32;                                      // 32-row tiles per head
  const int head = g * a.group + wave / tph;
  const int c = q0 + (wave % tph) * 32 + r;
  const bool c_ok = c < a.l_c;
  const int cc = c_ok ? c : a.l_c - 1;                             // rows past the chunk repeat its last token
  const uint32_t vis = V.n_fixed + (V.with_chunk ? cc + 1 : 0);
  const uint32_t lim = vis < k_end ? vis : k_end;                  // first virtual key this lane's query may NOT see
  const uint32_t lim_lo = __shfl(lim, 0, 64);                      // smallest limit in the wave (r = 0)
  bf16x8 qf[kD / 16];                                              // loaded below, behind the first tile's loads

  f32x16 o[4];
#pragma unroll
  for (int md = 0; md < 4; ++md)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[md][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  // ---- staging of one tile: global -> LDS directly, 16 bytes per lane.  A wave instruction fills 1 KB =
  // four rows; wave w brings row groups w and w + 8 of K and of V.  Lane l fills 16-byte slot l%16 of row
  // l/16 of its group; the piece of the global row it fetches for that slot undoes the swizzle:
  // K slot s of row R holds piece s ^ (R%16); V slot s of row R holds piece s%4 of chunk (s/4) ^ (R%4).
  const uint32_t st_row = 4 * wave + (lane >> 4);                  // first of this lane's two rows (second: + 32)
  const uint32_t st_slot = lane & 15;
  const uint32_t kcol = (st_slot ^ (st_row & 15)) * 16;            // byte column of the piece fetched for K
  const uint32_t vcol = ((((st_slot >> 2) ^ (st_row & 3)) << 2) | (st_slot & 3)) * 16;   // ... for V
  auto dma16 = [&](const char* src, bf16_t* dst_wave_uniform) {
    __builtin_amdgcn_global_load_lds((global_void*)src, (lds_void*)dst_wave_uniform, 16, 0, 0);
  };
  // Index-driven selected rows (the gather folded into this kernel): the two cache rows this lane fetches
  // for a tile that lies inside the selected segment are looked up one tile ahead of the tile's loads,
  // so that the look-up is not a dependent round trip in front of them.
  const int32_t* sidx = V.sel_idx ? V.sel_idx + (int64_t)b * V.idx_bs : nullptr;
  // The entries are kept as loaded and clamped where tile_load uses them, a whole tile later: clamping here
  // would be a use, and the wait in front of it would also wait for the tile loads issued just before, which
  // are meant to land during the tile's arithmetic.
  int32_t idx_a = 0, idx_b = 0;
  auto idx_prefetch = [&](uint32_t t) {
    const uint32_t j0 = t * kKT;
    if (sidx && t < tile_end && j0 >= V.i_end && j0 + kKT <= V.i_end + V.n_sel) {
      idx_a = sidx[j0 - V.i_end + st_row];
      idx_b = sidx[j0 - V.i_end + st_row + 32];
    }
  };
  // a middle token's position, clamped so that a bad index cannot leave the cache
  auto cache_row = [&](int32_t v) -> uint32_t { return v < 0 ? 0u : ((uint32_t)v < V.idx_limit ? (uint32_t)v : V.idx_limit - 1); };
  auto tile_load = [&](uint32_t j0, bf16_t* kt, bf16_t* vt) {
    const uint32_t sel_end = V.i_end + V.n_sel;
    int seg = -1;                                                  // 0: cache rows, 1: gathered rows
    uint32_t row0 = 0;
    // A tile whose 64 keys lie inside one segment of the virtual sequence (the usual case) is addressed
    // as uniform base + row * stride + column; tiles that straddle a segment boundary or the end of the
    // slice take the general per-row path.
    if (j0 + kKT <= V.i_end) {
      seg = 0;
      row0 = j0;
    } else if (j0 >= V.i_end && j0 + kKT <= sel_end) {
      seg = 1;
      row0 = j0 - V.i_end;
    } else if (j0 >= sel_end && j0 + kKT <= k_end) {
      seg = 0;
      row0 = j0 - sel_end + V.l_start;
    }
    bf16_t* kd0 = kt + wave * 512;                                 // 1 KB per row group
    bf16_t* kd1 = kt + (wave + 8) * 512;
    bf16_t* vd0 = vt + wave * 512;
    bf16_t* vd1 = vt + (wave + 8) * 512;
    if (seg == 1 && sidx) {             // rows idx_a / idx_b of the cache, looked up by idx_prefetch for this tile
      const uint32_t row_a = cache_row(idx_a), row_b = cache_row(idx_b);
      dma16(kc + ((uint64_t)row_a * V.tok_bytes + kcol), kd0);
      dma16(kc + ((uint64_t)row_b * V.tok_bytes + kcol), kd1);
      dma16(vc + ((uint64_t)row_a * V.tok_bytes + vcol), vd0);
      dma16(vc + ((uint64_t)row_b * V.tok_bytes + vcol), vd1);
    } else if (seg >= 0) {
      const uint32_t stride = seg ? a.sel_bytes : V.tok_bytes;
      const char* kb = (seg ? ksl : kc) + (uint64_t)row0 * stride;
      const char* vbase = (seg ? vsl : vc) + (uint64_t)row0 * stride;
      dma16(kb + (st_row * stride + kcol), kd0);
      dma16(kb + ((st_row + 32) * stride + kcol), kd1);
      dma16(vbase + (st_row * stride + vcol), vd0);
      dma16(vbase + ((st_row + 32) * stride + vcol), vd1);
    } else {
      uint32_t ja = j0 + st_row, jb = j0 + st_row + 32;
      ja = ja < k_end ? ja : k_end - 1;                            // the tail repeats a key; masked below
      jb = jb < k_end ? jb : k_end - 1;
      const RowRef ra = row_ref(V, sidx, a.sel_bytes, ja), rb = row_ref(V, sidx, a.sel_bytes, jb);
      dma16((ra.in_sel ? ksl : kc) + ra.off + kcol, kd0);
      dma16((rb.in_sel ? ksl : kc) + rb.off + kcol, kd1);
      dma16((ra.in_sel ? vsl : vc) + ra.off + vcol, vd0);
      dma16((rb.in_sel ? vsl : vc) + rb.off + vcol, vd1);
    }
  };
  // Every load of this wave has landed in LDS (vmcnt = 0; the other counters are left alone).
  auto loads_landed = [&]() { __builtin_amdgcn_s_waitcnt(0x0F70); };

  // Lane constants of the transposed V reads: inside its 16-lane group lane i points at key i/4 of a
  // four-key block and at four consecutive dims 4*(i%4).. of the group's sixteen.
  const int tr_key = (lane & 15) >> 2;
  const int tr_dim = ((lane >> 4) & 1) * 16 + 4 * (lane & 3);

  // ---- one tile: S^T = K Q^T, online softmax, O^T += V^T P^T
  auto tile_math = [&](uint32_t t, const bf16_t* kt, const bf16_t* vt) {
    const uint32_t j0 = t * kKT;
    f32x16 s[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int v = 0; v < 16; ++v) s[mt][v] = 0.f;
    // The sixteen K fragments of the tile are requested eight ahead of the matrix instructions that use
    // them (the order is pinned below): LDS latency is paid once per tile, not once per reduction step.
    bf16x8 kf[kD / 16][2];
#pragma unroll
    for (int ks16 = 0; ks16 < kD / 16; ++ks16)
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
        kf[ks16][mt] = *(const bf16x8*)&kt[(32 * mt + r) * kD + (((2 * ks16 + hi) ^ (r & 15)) << 3)];
#pragma unroll
    for (int ks16 = 0; ks16 < kD / 16; ++ks16)
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
        s[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks16][mt], qf[ks16], s[mt], 0, 0, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);

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
    mx = halves_max(mx);
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
    // Accumulator register v = 8*(e/4) + e%4 (+ 4*hi in the key number): fragment kp of P^T is S^T's
    // registers 8*(kp%2) .. + 7 of key tile kp/2, i.e. keys 16*kp + 4*hi + {0..3} and 16*kp + 8 + 4*hi + {0..3}.
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

    // ---- O^T += V^T P^T.  Row key of the V tile holds chunk c (dims 32c .. 32c+31) at chunk slot c ^ (key%4).
#pragma unroll
    for (int kp = 0; kp < 4; ++kp)
#pragma unroll
      for (int md = 0; md < 4; ++md) {
        const bf16_t* vp = vt + (16 * kp + 4 * hi + tr_key) * kD + ((md ^ tr_key) << 5) + tr_dim;
        const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)vp);             // keys 16kp + 4hi + 0..3
        const i16x4 up = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(vp + 8 * kD));  // keys 16kp + 8 + 4hi + 0..3
        const i16x8 both = __builtin_shufflevector(lo, up, 0, 1, 2, 3, 4, 5, 6, 7);
        o[md] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pf[kp], o[md], 0, 0, 0);
      }
    // the V fragments of sixteen keys (eight reads) are requested ahead of the four matrix instructions that use them
    __builtin_amdgcn_sched_group_barrier(0x100, 16, 0);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
  };

  // The first tile's loads go out before the query fragments' so that the two round trips overlap.
  idx_prefetch(tile_begin);
  if (tile_begin < tile_end) tile_load(tile_begin * kKT, k_st0, v_st0);
  idx_prefetch(tile_begin + 1);
  {
    const bf16_t* qp = V.q + (int64_t)b * V.q_bs + ((int64_t)cc * a.h + head) * kD + hi * 8;
#pragma unroll
    for (int ks16 = 0; ks16 < kD / 16; ++ks16) qf[ks16] = *(const bf16x8*)(qp + ks16 * 16);
    // Pin the fragments as arrived values here: otherwise every use inside the tile loop carries a
    // wait on the vector-memory counter.
#pragma unroll
    for (int ks16 = 0; ks16 < kD / 16; ++ks16) asm volatile("" : "+v"(qf[ks16]));
  }
  // Two tiles per trip so that every stage is named statically.  At each barrier tile t is in LDS and
  // every wave is done with tile t-1, whose stage the loads issued right after the barrier overwrite.
  for (uint32_t t = tile_begin; t < tile_end; t += 2) {
    loads_landed();
    __syncthreads();
    if (t + 1 < tile_end) tile_load((t + 1) * kKT, k_st1, v_st1);
    idx_prefetch(t + 2);
    tile_math(t, k_st0, v_st0);
    if (t + 1 < tile_end) {
      loads_landed();
      __syncthreads();
      if (t + 2 < tile_end) tile_load((t + 2) * kKT, k_st0, v_st0);
      idx_prefetch(t + 3);
      tile_math(t + 1, k_st1, v_st1);
    }
  }

  // ---- results.  Accumulator register v of tile md is head-dim 32*md + 8*(v/4) + 4*hi + v%4 of this
  // lane's query, so a lane holds its whole output row in 8-byte pieces.  The rows are narrowed to 16
  // bits and turned into whole 256-byte rows in LDS (free by now), from where each wave writes its own
  // 32 rows with fully coalesced 16-byte stores.  Final outputs are normalised and rounded to bf16.
  // Partial results of a key slice stay un-normalised and are stored as fp16 with a per-row power-of-two
  // scale 2^-E that brings the row's largest magnitude to about 2^13 (fp16's 11-bit significand keeps the
  // rounding well below that of the bf16 output, and any magnitude bf16 inputs can produce fits); beside
  // them go m + E and l * 2^-E, so that the merge's sums of 2^(m+E-M) * (O 2^-E) and 2^(m+E-M) * (l 2^-E)
  // are the plain log-sum-exp combination of Algorithm 1 with no trace of E.
  const float l_tot = halves_sum(l_run);
  const bool final_out = n_slices == 1 && !a.to_slots;
  float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  float m_store = m_run, l_store = l_tot;
  if (!final_out) {
    float amax = 0.f;
#pragma unroll
    for (int md = 0; md < 4; ++md)
#pragma unroll
      for (int v = 0; v < 16; ++v) amax = fmaxf(amax, __builtin_fabsf(o[md][v]));
    amax = halves_max(amax);
    int s_exp = 267 - (int)((__float_as_uint(amax) >> 23) & 0xFFu);      // biased exponent of 2^-E
    s_exp = s_exp < 17 ? 17 : (s_exp > 167 ? 167 : s_exp);              // 2^-110 .. 2^40
    inv = __uint_as_float((uint32_t)s_exp << 23);
    m_store = m_run - (float)(s_exp - 127);
    l_store = l_tot * inv;
  }
  __syncthreads();                       // every wave is done with the last tile
  {
    // wave w's 32 rows of 256 bytes go to half (w%2) of stage array w/2, 16-byte slots swizzled by row % 16
    uint16_t* ot = (uint16_t*)(wave < 2 ? k_st0 : wave < 4 ? k_st1 : wave < 6 ? v_st0 : v_st1) + ((wave & 1) * 32 + r) * kD;
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
        *(uint2*)(ot + (((4 * md + vg) ^ (r & 15)) << 3) + 4 * hi) = w;
      }
  }
  __syncthreads();
  const int c_wave = q0 + (wave % tph) * 32;                        // first current token of this wave's rows
  uint16_t* dst;
  if (final_out) {
    dst = (uint16_t*)a.out + (int64_t)b * a.out_bs + ((int64_t)c_wave * a.h + head) * kD;
  } else {
    const int64_t prow0 = ((int64_t)(b * a.n_slot + V.slot0 + split) * a.l_c) * a.h;
    dst = a.part_o + (prow0 + (int64_t)c_wave * a.h + head) * kD;
    if (hi == 0 && c_ok) {
      float2 ml = {m_store, l_store};
      *(float2*)(a.part_ml + (prow0 + (int64_t)c * a.h + head) * 2) = ml;
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int rw = 4 * i + (lane >> 4), piece = lane & 15;
    if (c_wave + rw < a.l_c) {
      const uint16_t* ob = (const uint16_t*)(wave < 2 ? k_st0 : wave < 4 ? k_st1 : wave < 6 ? v_st0 : v_st1);
      const uint4 w = *(const uint4*)(ob + ((wave & 1) * 32 + rw) * kD + ((piece ^ (rw & 15)) << 3));
      *(uint4*)(dst + (int64_t)rw * a.h * kD + piece * 8) = w;
    }
  }
  if (final_out && a.lse && hi == 0 && c_ok)
    a.lse[(int64_t)b * a.l_c * a.h + (int64_t)c * a.h + head] = (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2;
}

// Algorithm 1's merge over partial results (un-normalised outputs and sums, both relative to the slice's
// reference m_s): weights 2^(m_s - M) with the maximum subtracted first.
// The slots in use are [0, ns_a) and [slot_b, slot_b + ns_b) of n_slot.  16 lanes per row (eight
// head-dims, 16 bytes of fp16 partials, each), sixteen rows per workgroup.
__global__ __launch_bounds__(256) void esa_attend_merge(const uint16_t* __restrict__ part_o,
                                                        const float* __restrict__ part_ml, int n_slot, int ns_a,
                                                        int slot_b, int ns_b, int64_t rows, bf16_t* __restrict__ out,
                                                        float* __restrict__ lse, int64_t out_bs, int64_t lse_bs) {
  const int64_t row = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
  const int d8 = (threadIdx.x & 15) * 8;
  const int b = blockIdx.y;
  if (row >= rows) return;
  // Every load of the row goes out before the first use (one round trip): the slices' (maximum, sum)
  // pairs and their outputs.  A slice that saw no key of this row stored zeros and sum 0.
  float m[kMaxSlots], l[kMaxSlots];
  uint4 po[kMaxSlots];
#pragma unroll
  for (int s = 0; s < kMaxSlots; ++s) {
    m[s] = -INFINITY;
    l[s] = 0.f;
    po[s] = make_uint4(0u, 0u, 0u, 0u);
    if (s < ns_a || (s >= slot_b && s < slot_b + ns_b)) {
      const int64_t prow = ((int64_t)b * n_slot + s) * rows + row;
      const float2 ml = *(const float2*)(part_ml + prow * 2);
      m[s] = ml.x;
      l[s] = ml.y;
      po[s] = *(const uint4*)(part_o + prow * kD + d8);
    }
  }
  float M = -INFINITY;
#pragma unroll
  for (int s = 0; s < kMaxSlots; ++s) M = fmaxf(M, m[s]);
  float L = 0.f;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
#pragma unroll
  for (int s = 0; s < kMaxSlots; ++s) {
    const float w = m[s] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m[s] - M);
    const uint32_t u[4] = {po[s].x, po[s].y, po[s].z, po[s].w};
    L += w * l[s];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const f16x2 p = *(const f16x2*)&u[i];
      acc[2 * i] += w * (float)p[0];
      acc[2 * i + 1] += w * (float)p[1];
    }
  }
  const float inv = 1.f / L;
  uint4 w4;
  w4.x = pack_bf16x2(acc[0] * inv, acc[1] * inv);
  w4.y = pack_bf16x2(acc[2] * inv, acc[3] * inv);
  w4.z = pack_bf16x2(acc[4] * inv, acc[5] * inv);
  w4.w = pack_bf16x2(acc[6] * inv, acc[7] * inv);
  *(uint4*)(out + (int64_t)b * out_bs + row * kD + d8) = w4;
  if (lse && d8 == 0) lse[(int64_t)b * lse_bs + row] = (M + __builtin_amdgcn_logf(L)) * kLn2;
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

namespace {

KeyView make_view(const void* q, int64_t q_bs, const void* k_cache, const void* v_cache, int64_t tok_stride,
                  int64_t cache_bs, int64_t i_end, int n_sel, int64_t l_start, int64_t n_fixed, int with_chunk,
                  int n_split, int slot0, const int32_t* sel_idx = nullptr, int64_t idx_bs = 0, int64_t idx_limit = 1) {
  KeyView v;
  v.sel_idx = n_sel > 0 ? sel_idx : nullptr;
  v.idx_bs = idx_bs;
  v.idx_limit = (uint32_t)(idx_limit > 0 ? idx_limit : 1);
  v.q = (const bf16_t*)q;
  v.k_cache = (const char*)k_cache;
  v.v_cache = (const char*)v_cache;
  v.q_bs = q_bs;
  v.cache_bs_bytes = cache_bs * 2;
  v.tok_bytes = (uint32_t)(tok_stride * 2);
  v.i_end = (uint32_t)i_end;
  v.n_sel = (uint32_t)n_sel;
  v.l_start = (uint32_t)l_start;
  v.n_fixed = (uint32_t)n_fixed;
  v.with_chunk = with_chunk;
  v.n_split = n_split;
  v.slot0 = slot0;
  return v;
}

int clamp_splits(int ns, int64_t keys_of_first_tile) {
  const int64_t tiles = (keys_of_first_tile + kKT - 1) / kKT;
  return (int)(ns > tiles ? (tiles > 0 ? tiles : 1) : ns);
}

}  // namespace

int launch_attend_mfma(int part, int split, const void* q, int l_c, int h, int h_kv, int d, const void* k_cache,
                       const void* v_cache, int64_t tok_stride, int64_t t0, int64_t i_end, int64_t l_start,
                       const void* k_sel, const void* v_sel, int n_sel, const int32_t* sel_idx, int64_t idx_bs,
                       float scale, void* out, float* lse, int batch, int64_t q_bs, int64_t cache_bs, int64_t sel_bs,
                       int64_t out_bs, void* ws, size_t ws_bytes, hipStream_t st) {
  if (!(scale > 0.f)) ESA_FAIL(ESA_EINVAL, "esa_attend: scale must be positive");
  if (t0 + l_c >= ((int64_t)1 << 31) || tok_stride * 2 >= ((int64_t)1 << 32))
    ESA_FAIL(ESA_EUNSUPPORTED, "esa_attend: positions beyond 2^31 are not supported by the matrix-core kernel");
  AttendArgs a;
  a.out = (bf16_t*)out;
  a.lse = lse;
  a.k_sel = (const char*)k_sel;
  a.v_sel = (const char*)v_sel;
  a.sel_bytes = (uint32_t)((int64_t)h_kv * d * 2);
  a.l_c = l_c;
  a.h = h;
  a.h_kv = h_kv;
  a.group = h / h_kv;
  a.qpt = kRows / a.group;
  a.n_qt = (l_c + a.qpt - 1) / a.qpt;
  a.batch = batch;
  a.c2 = scale * kLog2e;
  a.out_bs = out_bs;
  a.sel_bs_bytes = sel_bs * 2;
  a.xcd_mapping = ((batch * h_kv) % 8 == 0) ? 1 : 0;

  const SplitPlan plan = plan_splits(l_c, a.group, h_kv, batch);
  const int first_rows = l_c < a.qpt ? l_c : a.qpt;
  // slices in use: one call -> `all`; two calls -> local in slots [0, ns_local), selected in [plan.local, +ns_sel)
  const int ns_all = clamp_splits(plan.all, i_end + n_sel + (t0 - l_start) + first_rows);
  // split == ESA_SPLIT_ALGORITHM1 moves the initial tokens from the early part to the late one
  const int64_t i_early = split == ESA_SPLIT_ALGORITHM1 ? 0 : i_end, i_late = i_end - i_early;
  const int ns_local = clamp_splits(plan.local, i_early + (t0 - l_start) + first_rows);
  const int ns_sel = i_late + n_sel > 0 ? clamp_splits(plan.sel, i_late + n_sel) : 0;
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
  a.view[1] = make_view(q, q_bs, k_cache, v_cache, tok_stride, cache_bs, 0, 0, 0, 0, 0, 0, 0);   // unused
  auto launch = [&](int64_t n_wg) { attend_mfma_bf16<<<dim3((unsigned)n_wg), kThreads, 0, st>>>(a); };
  const int64_t rows = (int64_t)l_c * h;
  const dim3 merge_grid((unsigned)((rows + 15) / 16), batch);
  if (part == kAttendAll) {
    a.view[0] = make_view(q, q_bs, k_cache, v_cache, tok_stride, cache_bs, i_end, n_sel, l_start,
                          i_end + n_sel + (t0 - l_start), 1, ns_all, 0, sel_idx, idx_bs, l_start);
    a.to_slots = 0;
    launch((int64_t)batch * h_kv * a.n_qt * ns_all);
    if (ns_all > 1)
      esa_attend_merge<<<merge_grid, 256, 0, st>>>(a.part_o, a.part_ml, n_slot, ns_all, 0, 0, rows, (bf16_t*)out, lse,
                                                   out_bs, rows);
  } else if (part == kAttendLocal) {
    a.view[0] = make_view(q, q_bs, k_cache, v_cache, tok_stride, cache_bs, i_early, 0, l_start,
                          i_early + (t0 - l_start), 1, ns_local, 0);
    a.to_slots = 1;
    launch((int64_t)batch * h_kv * a.n_qt * ns_local);
  } else {
    if (ns_sel > 0) {
      a.view[0] = make_view(q, q_bs, k_cache, v_cache, tok_stride, cache_bs, i_late, n_sel, 0, i_late + n_sel, 0, ns_sel,
                            plan.local, sel_idx, idx_bs, l_start);
      a.to_slots = 1;
      launch((int64_t)batch * h_kv * a.n_qt * ns_sel);
    }
    esa_attend_merge<<<merge_grid, 256, 0, st>>>(a.part_o, a.part_ml, n_slot, ns_local, plan.local, ns_sel, rows,
                                                 (bf16_t*)out, lse, out_bs, rows);
  }
  ESA_LAUNCH_CHECK("attend_mfma");
  return ESA_OK;
}

// Section 3.2 in one launch: the local keys (dense re-encoded copy, rows [0, n_loc + l_c), causal) with the
// queries q_loc, and the initial and selected keys (caller's un-encoded cache and gathered rows, every key
// visible) with the queries q_glob; the slices of both share the launch and the merge.
int launch_attend_mfma_two_views(const void* q_loc, const void* q_glob, int64_t qw_bs, int l_c, int h, int h_kv, int d,
                                 const void* k_loc, const void* v_loc, int64_t n_loc, int64_t loc_bs,
                                 const void* k_cache, const void* v_cache, int64_t tok_stride, int64_t cache_bs,
                                 int64_t i_end, const void* k_sel, const void* v_sel, int n_sel, int64_t sel_bs,
                                 float scale, void* out, float* lse, int batch, int64_t out_bs, void* ws, size_t ws_bytes,
                                 hipStream_t st) {
  if (!(scale > 0.f)) ESA_FAIL(ESA_EINVAL, "esa_attend: scale must be positive");
  if (n_loc + l_c >= ((int64_t)1 << 31) || tok_stride * 2 >= ((int64_t)1 << 32))
    ESA_FAIL(ESA_EUNSUPPORTED, "esa_attend: positions beyond 2^31 are not supported by the matrix-core kernel");
  AttendArgs a;
  a.out = (bf16_t*)out;
  a.lse = lse;
  a.k_sel = (const char*)k_sel;
  a.v_sel = (const char*)v_sel;
  a.sel_bytes = (uint32_t)((int64_t)h_kv * d * 2);
  a.l_c = l_c;
  a.h = h;
  a.h_kv = h_kv;
  a.group = h / h_kv;
  a.qpt = kRows / a.group;
  a.n_qt = (l_c + a.qpt - 1) / a.qpt;
  a.batch = batch;
  a.c2 = scale * kLog2e;
  a.out_bs = out_bs;
  a.sel_bs_bytes = sel_bs * 2;
  a.xcd_mapping = ((batch * h_kv) % 8 == 0) ? 1 : 0;
  // the planned number of slices is shared out in proportion to the two parts' lengths, at least one each
  const SplitPlan plan = plan_splits(l_c, a.group, h_kv, batch);
  const int first_rows = l_c < a.qpt ? l_c : a.qpt;
  const int64_t keys_a = n_loc + (l_c + 1) / 2, keys_b = i_end + n_sel;
  int ns_b = keys_b > 0 ? (int)((plan.all * keys_b + (keys_a + keys_b) / 2) / (keys_a + keys_b)) : 0;
  if (keys_b > 0 && ns_b < 1) ns_b = 1;
  int ns_a = plan.all - ns_b < 1 ? 1 : plan.all - ns_b;
  ns_a = clamp_splits(ns_a, n_loc + first_rows);
  if (ns_b > 0) ns_b = clamp_splits(ns_b, keys_b);
  const int n_slot = ns_a + ns_b;
  const size_t need = slots_bytes(n_slot, l_c, h, batch);
  a.part_o = nullptr;
  a.part_ml = nullptr;
  if (n_slot > 1) {
    if (!ws || ws_bytes < need) ESA_FAIL(ESA_EWORKSPACE, "esa_attend: workspace needs %zu bytes", need);
    const size_t rows = (size_t)batch * n_slot * l_c * h;
    a.part_o = (uint16_t*)ws;
    a.part_ml = (float*)((char*)ws + align_up(rows * kD * sizeof(uint16_t), 256));
  }
  a.n_slot = n_slot;
  a.to_slots = 0;
  a.view[0] = make_view(q_loc, qw_bs, k_loc, v_loc, (int64_t)h_kv * d, loc_bs, 0, 0, 0, n_loc, 1, ns_a, 0);
  a.view[1] = make_view(q_glob, qw_bs, k_cache, v_cache, tok_stride, cache_bs, i_end, n_sel, 0, keys_b, 0, ns_b, ns_a);
  attend_mfma_bf16<<<dim3((unsigned)((int64_t)batch * h_kv * a.n_qt * n_slot)), kThreads, 0, st>>>(a);
  const int64_t rows = (int64_t)l_c * h;
  if (n_slot > 1) {
    const dim3 merge_grid((unsigned)((rows + 15) / 16), batch);
    esa_attend_merge<<<merge_grid, 256, 0, st>>>(a.part_o, a.part_ml, n_slot, n_slot, 0, 0, rows, (bf16_t*)out, lse, out_bs,
                                                 rows);
  }
  ESA_LAUNCH_CHECK("attend_mfma (two views)");
  return ESA_OK;
}

}  // namespace esa
