// Importance of every middle token (Eq. 6 inside Eq. 4):
//   S[c,m] = q'_c . k'_m,  mu[c] = max_m S[c,m],  F[m] = max_c (S[c,m] - mu[c]),
// optionally followed by the proximity max-pool of Eq. 8.
//
// F needs every row maximum before any column maximum, so K' is swept twice and S is
// recomputed instead of being stored (S would be l_C x N fp32; K' is only N x d_c storage
// elements).  Both sweeps compute S[c,m] with the same instruction sequence, so the second one
// reproduces the first bit for bit: the row arg-max token gets F = 0 exactly and F <= 0 everywhere.
// Row maxima are combined across workgroups with integer atomicMax on order-preserving keys
// (exact and order-independent).
//
// This file is compiled with the IEEE mode bit off and NaNs declared absent (see build.py): with the bit
// on, every fmaxf() on a matrix-core result costs three instructions, because the compiler first
// "canonicalises" each operand it cannot prove free of signalling NaNs (a max of the value with
// itself).  No NaN occurs here (inputs are finite by contract; -inf is only ever compared).
#include "esa_common.h"
#include <type_traits>
#include "radix_hist.h"

namespace esa {
namespace {

// Work-item and workgroup numbers are taken from the hardware builtins in this file: with the IEEE mode bit
// off (see build.py) the device library's accessors behind threadIdx / blockIdx / gridDim are not inlined (their
// floating-point mode attributes differ from the kernels'), and every use would be a function call.

// Workspace: [batch][l_c] row maxima (uint32 keys or fp32), [batch][blocks][l_c] fp32 partial row maxima of the
// matrix-core kernel, then (eps > 0) [batch][n] fp32 unpooled scores.
__host__ __device__ inline size_t mu_bytes(int l_c, int batch) {      // rows padded to whole groups of 64
  return align_up((size_t)((l_c + 63) / 64 * 64) * batch * 4, 256);
}

__global__ void fill_u32(uint32_t* p, int64_t n, uint32_t v) {
  const int64_t i = (int64_t)__builtin_amdgcn_workgroup_id_x() * 256 + __builtin_amdgcn_workitem_id_x();   // one thread per word
  if (i < n) p[i] = v;
}

// ------------------------------------------------------------------------------------------ generic
constexpr int kGTok = 64;      // middle tokens per block (one per lane)

// One fixed-order fp32 dot product, shared by both sweeps.
template <typename T>
__device__ __forceinline__ float dot_fixed(const T* __restrict__ q, const float* __restrict__ krow, int d_c) {
  float s = 0.f;
  for (int i = 0; i < d_c; ++i) s = __fmaf_rn(load_f32(q + i), krow[i], s);
  return s;
}

// SWEEP 0: row maxima into mu_keys.  SWEEP 1: F into score.
template <typename T, int SWEEP>
__global__ __launch_bounds__(256) void score_fma(const T* __restrict__ qc, int l_c, const T* __restrict__ kc,
                                                 int64_t m_lo, int64_t n, int d_c, uint32_t* __restrict__ mu_keys,
                                                 float* __restrict__ score, int64_t q_bs, int64_t kc_bs,
                                                 int64_t score_bs) {
  extern __shared__ float smem[];                 // kt[kGTok][d_c+1], then red[4][kGTok]
  const int ldk = d_c + 1;
  float* kt = smem;
  float* red = smem + kGTok * ldk;
  const int b = __builtin_amdgcn_workgroup_id_y();
  const T* q = qc + (int64_t)b * q_bs;
  const T* k = kc + (int64_t)b * kc_bs + m_lo * (int64_t)d_c;
  uint32_t* mu = mu_keys + (int64_t)b * l_c;
  const int64_t m0 = (int64_t)__builtin_amdgcn_workgroup_id_x() * kGTok;
  for (int e = __builtin_amdgcn_workitem_id_x(); e < kGTok * d_c; e += 256) {
    const int t = e / d_c, i = e % d_c;
    kt[t * ldk + i] = (m0 + t < n) ? load_f32(k + (m0 + t) * (int64_t)d_c + i) : 0.f;
  }
  __syncthreads();
  const int lane = __builtin_amdgcn_workitem_id_x() & 63, wave = __builtin_amdgcn_workitem_id_x() >> 6;
  const bool valid = (m0 + lane) < n;
  float best = -INFINITY;
  for (int c = wave; c < l_c; c += 4) {
    float s = dot_fixed(q + (int64_t)c * d_c, kt + lane * ldk, d_c);
    if (!valid) s = -INFINITY;
    if (SWEEP == 0) {
      const float mx = wave_max(s);
      if (lane == 0) atomicMax(&mu[c], ordered_key(mx));
    } else {
      best = fmaxf(best, s - ordered_key_to_f32(mu[c]));
    }
  }
  if (SWEEP == 1) {
    red[wave * kGTok + lane] = best;
    __syncthreads();
    if (wave == 0 && valid) {
      const float f = fmaxf(fmaxf(red[lane], red[kGTok + lane]), fmaxf(red[2 * kGTok + lane], red[3 * kGTok + lane]));
      score[(int64_t)b * score_bs + m0 + lane] = f;
    }
  }
}


// ------------------------------------------------------------------------------------------ MFMA (bf16, d_c = 128)
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// v_mfma_f32_32x32x16_bf16 computes D[32x32] += A[32x16] B[16x32].  Lane l supplies eight
// consecutive reduction elements of A row l%32 and of B column l%32 (which eight depends only on
// l/32, identically for A and B), and owns D[8*(v/4) + 4*(l/32) + v%4][l%32] in register v.
//
// Here A rows are current tokens (queries), B columns are middle tokens.  A workgroup of eight
// waves (two per SIMD) owns up to 512 consecutive middle tokens.  Its whole share of K' (at most
// 128 KB) goes from memory straight into LDS, without passing through registers: sixteen
// global_load_lds_dwordx4 per thread, issued back to back at the start of the kernel, each wave
// instruction bringing four 256-byte rows.  Which 16 bytes of its row a lane fetches is chosen such
// that the rows land XOR-swizzled (piece p of row R in slot p ^ R%16), which makes the fragment
// reads free of bank conflicts without padding.  Loads complete in order, so tile t (32 tokens,
// instruction t of every wave) is usable once every wave has waited for its own instruction t and
// a barrier has passed; the tiles are consumed as they land, two per barrier.  Queries are the
// register-resident operand (64 per wave as A fragments for the whole d_c = 128; chunks longer than
// 512 loop over query blocks against the same LDS tile), so K' is read from memory once per sweep.
//
// Inside a wave the tiles are software-pipelined: right after the matrix instructions of reduction
// step ks of tile t have issued, fragment ks of tile t+1 is read from LDS into the registers they
// have just released, and the maximum / subtract work on tile t-1's accumulators (a second
// accumulator set) sits between the matrix instructions, so that one wave alone keeps the matrix
// pipe fed.  With a token per lane, the column maximum of Eq. 4 is an in-lane reduction over the
// accumulator registers plus one exchange between the two half-waves, folded across waves with an
// LDS integer maximum on order-preserving keys; the row maximum is kept per register across all
// tiles and reduced across lanes once, then written as this workgroup's partial row maxima (no
// atomics across workgroups) for score_rowmax_reduce.
//
// While the share is landing, every LDS access of the tile loop is written as an instruction of its
// own with its own counter waits: an LDS access the compiler generates is preceded by a wait for ALL
// outstanding loads into LDS (it cannot tell which rows they fill), which would turn the stream into
// one round trip followed by the arithmetic.  LDS operations complete in order, which the waits
// below rely on: "at most 7 outstanding" before the use of fragment ks means that fragment has
// arrived, because exactly seven fragment reads were issued after it (the rest of this tile's and the
// first ks of the next tile's).  Operations the compiler adds on the same counter are newer still
// and only make these waits stricter.
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(3))) unsigned char lds_byte;
typedef __attribute__((address_space(1))) const void global_void;
constexpr int kDc = 128;
constexpr int kKSteps = kDc / 16;        // MFMA reduction steps per tile
constexpr int kWaves = 8;
constexpr int kThreads = 64 * kWaves;
constexpr int kMT = 2;                   // 32-query tiles per wave
constexpr int kQPerWave = 32 * kMT;
constexpr int kQPerBlock = kWaves * kQPerWave;
constexpr int kMaxTilesPerBlock = 16;    // 512 tokens: 128 KB of LDS; one load instruction per thread and tile
constexpr int kTileBytes = 32 * kDc * 2; // one tile of K' in LDS

__host__ __device__ inline int64_t mfma_tiles_per_block(int64_t n) {
  const int64_t n_tiles = (n + 31) / 32;
  const int64_t per = ((n_tiles + 255) / 256 + 1) / 2 * 2;   // about one workgroup per compute unit; even
  return per < 2 ? 2 : (per > kMaxTilesPerBlock ? kMaxTilesPerBlock : per);
}
__host__ __device__ inline int64_t mfma_blocks(int64_t n) {
  const int64_t per = mfma_tiles_per_block(n);
  return ((n + 31) / 32 + per - 1) / per;
}
// K' share, column maxima, digit histogram
__host__ __device__ inline size_t mfma_lds_bytes(int64_t per) {
  return (size_t)per * kTileBytes + (size_t)(per + 1) * 32 * sizeof(uint32_t) + (size_t)kRadixBins * sizeof(uint32_t);
}
// Row maxima of the matrix-core path: one row of mfma_mu_stride(l_c) floats per batch entry, so that groups
// of four are 16-byte aligned and in bounds for every query tile that holds a query.
__host__ __device__ inline int mfma_mu_stride(int l_c) { return (l_c + 63) / 64 * 64; }

// Wait until at most `left` (14, 12, 8 or 0) vector-memory loads of this wave are outstanding, then the
// workgroup barrier.  Only the first one (14) also waits for the LDS operations issued before it, the
// initialising writes; in the tile loop the fragment reads in flight stay in flight across the barrier.
__device__ __forceinline__ void wait_loads_then_barrier(int left) {
  switch (left) {
    case 0: asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory"); break;
    case 8: asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory"); break;
    case 12: asm volatile("s_waitcnt vmcnt(12)\n\ts_barrier" ::: "memory"); break;
    default: asm volatile("s_waitcnt vmcnt(14) lgkmcnt(0)\n\ts_barrier" ::: "memory"); break;
  }
}

// PASS 0: partial row maxima into part_max[l_c][blocks].  PASS 1: F into score, using mu; with
// first_hist given, also the histogram of the scores' leading 11 key bits (the first digit of the radix
// selection that follows: the scores are in LDS here, so the selection need not read them for it).
template <int PASS>
__global__ __launch_bounds__(kThreads) void score_mfma_bf16(const bf16_t* __restrict__ qc, int l_c,
                                                            const bf16_t* __restrict__ kc, int64_t m_lo, int64_t n,
                                                            float* __restrict__ part_max,
                                                            const float* __restrict__ mu_all,
                                                            float* __restrict__ score, int64_t q_bs, int64_t kc_bs,
                                                            int64_t score_bs, int tiles_per_block,
                                                            uint32_t* __restrict__ first_hist, int64_t first_hist_bs,
                                                            bf16_t* __restrict__ qfrag, int64_t qfrag_bs, int n_wg) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];   // n_wg: workgroups per batch entry
  const int tpb = tiles_per_block;
  const int span = tpb * 32;                                           // tokens of this workgroup
  uint32_t* colmax = (uint32_t*)(lds_raw + (size_t)tpb * kTileBytes);  // PASS 1: [32 spare + span] keys
  uint32_t* digit_hist = colmax + 32 + span;                           // PASS 1: [kRadixBins]
  const int b = __builtin_amdgcn_workgroup_id_y();
  const bf16_t* q = qc + (int64_t)b * q_bs;
  const int mu_stride = mfma_mu_stride(l_c);
  const float* mu = mu_all + (int64_t)b * mu_stride;
  const int tid = __builtin_amdgcn_workitem_id_x(), lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // uniform: lives in a scalar register
  const int r = lane & 31, hi = lane >> 5;
  const int64_t tok_base = (int64_t)__builtin_amdgcn_workgroup_id_x() * span;
  const char* kshare = (const char*)(kc + (int64_t)b * kc_bs + (m_lo + tok_base) * (int64_t)kDc);
  const uint32_t last_row = (uint32_t)(n - tok_base - 1 < span - 1 ? n - tok_base - 1 : span - 1);
  const uint32_t lds_tiles = (uint32_t)(uintptr_t)(lds_byte*)lds_raw;  // LDS byte address of the share
  const uint32_t lds_colmax = lds_tiles + (uint32_t)tpb * kTileBytes;

  bf16x8 a[kMT][kKSteps];
  float aux[kMT][16];                    // PASS 0: running row maxima.  PASS 1: mu of the lane's rows.
  // Rows past the chunk repeat its last query: a repeated row changes no maximum, and its own results
  // are never written (PASS 0) or are pushed to -inf by mu = +inf (PASS 1).  Register v of tile mt
  // belongs to row 8*(v/4) + 4*hi + v%4 of the tile.
  //
  // The requests for the fragments and (PASS 1) the row maxima are instructions written out here, and so
  // is the wait that ends them (queries_arrived): had the compiler generated the loads, its own wait for them
  // would be a wait for everything once loads into LDS are outstanding behind them (it does not count on
  // those completing in order with ordinary loads), which would put a round trip in front of the share's
  // requests.  Between request and wait the registers are only named by that wait.
  f32x4 mu4[kMT][4];
  int qb_now = 0;
  auto wave_has_queries = [&](int qb) { return qb * kQPerBlock + wave * kQPerWave < l_c; };
  // Fragment-ordered copy of Q' in the workspace, [block][wave][tile][step][lane] x 16 bytes: written by the
  // first workgroups of sweep 0 from their registers (every workgroup holds the same fragments), read by
  // every workgroup of sweep 1.
  auto qfrag_of = [&](int qb, int mt) -> bf16_t* {
    return qfrag + (int64_t)b * qfrag_bs + ((((int64_t)qb * kWaves + wave) * kMT + mt) * kKSteps * 64 + lane) * 8;
  };
  auto request_query_block = [&](int qb) {
    const int q0 = qb * kQPerBlock + wave * kQPerWave;
    if (!wave_has_queries(qb)) {          // a wave without queries only takes part in the loads and barriers
#pragma unroll
      for (int mt = 0; mt < kMT; ++mt) {
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) a[mt][ks] = (bf16x8){0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) mu4[mt][g4] = (f32x4){0.f, 0.f, 0.f, 0.f};
      }
      return;
    }
#pragma unroll
    for (int mt = 0; mt < kMT; ++mt) {
      if (PASS == 1) {
        // the copy of the fragments in register order that sweep 0 left: a wave instruction reads 1 KB in one
        // piece (eight cache lines) instead of 16 bytes of 32 rows (32 lines), a quarter of the address work
        const bf16_t* p = qfrag_of(qb, mt);
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) {
          if (ks < 4) asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(a[mt][ks]) : "v"(p), "n"(ks * 1024));
          else asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(a[mt][ks]) : "v"(p + 2048), "n"((ks - 4) * 1024));
        }
      } else {
        int row = q0 + 32 * mt + r;
        row = row < l_c ? row : l_c - 1;
        const bf16_t* p = q + (int64_t)row * kDc + hi * 8;
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks)
          asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(a[mt][ks]) : "v"(p), "n"(ks * 32));
      }
      if (PASS == 1) {
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int qrow = q0 + 32 * mt + 8 * g4 + 4 * hi;
          const float* mp = mu + (qrow < mu_stride - 4 ? qrow : mu_stride - 4);
          asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(mu4[mt][g4]) : "v"(mp));
        }
      }
    }
  };
#define ESA_QUERY_REGS(mt)                                                                                     \
  "+v"(a[mt][0]), "+v"(a[mt][1]), "+v"(a[mt][2]), "+v"(a[mt][3]), "+v"(a[mt][4]), "+v"(a[mt][5]), "+v"(a[mt][6]), \
      "+v"(a[mt][7])
#define ESA_MU_REGS(mt) "+v"(mu4[mt][0]), "+v"(mu4[mt][1]), "+v"(mu4[mt][2]), "+v"(mu4[mt][3])
  // Everything requested before the share has arrived once at most fourteen of the share's sixteen requests
  // are outstanding (first block; tiles 0 and 1 are in LDS then as well), or nothing at all (later blocks).
  auto queries_arrived = [&](bool first) {
    if (PASS == 0) {
      if (first) asm volatile("s_waitcnt vmcnt(14)" : ESA_QUERY_REGS(0), ESA_QUERY_REGS(1));
      else asm volatile("s_waitcnt vmcnt(0)" : ESA_QUERY_REGS(0), ESA_QUERY_REGS(1));
    } else {
      if (first) asm volatile("s_waitcnt vmcnt(14)" : ESA_QUERY_REGS(0), ESA_QUERY_REGS(1), ESA_MU_REGS(0), ESA_MU_REGS(1));
      else asm volatile("s_waitcnt vmcnt(0)" : ESA_QUERY_REGS(0), ESA_QUERY_REGS(1), ESA_MU_REGS(0), ESA_MU_REGS(1));
    }
#pragma unroll
    for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        if (PASS == 0) {
#pragma unroll
          for (int e = 0; e < 4; ++e) aux[mt][4 * g4 + e] = -INFINITY;
        } else {
          const int qrow = (qb_now * kQPerBlock + wave * kQPerWave) + 32 * mt + 8 * g4 + 4 * hi;
          const f32x4 m4 = mu4[mt][g4];
          aux[mt][4 * g4 + 0] = qrow + 0 < l_c ? m4.x : INFINITY;
          aux[mt][4 * g4 + 1] = qrow + 1 < l_c ? m4.y : INFINITY;
          aux[mt][4 * g4 + 2] = qrow + 2 < l_c ? m4.z : INFINITY;
          aux[mt][4 * g4 + 3] = qrow + 3 < l_c ? m4.w : INFINITY;
        }
      }
  };
#undef ESA_QUERY_REGS
#undef ESA_MU_REGS

  // ---- the pipeline over this workgroup's tiles
  bf16x8 bfr[kKSteps];
  f32x16 acc0[kMT], acc1[kMT];
  // LDS byte address of this lane's fragment ks of tile nt: row r, slot (2 ks + hi) ^ (r % 16).  The share
  // starts at a multiple of 256 bytes, so the slot's ks bits can be XORed into the address of fragment 0.
  const uint32_t frag0_at = lds_tiles + (uint32_t)r * (kDc * 2) + (uint32_t)((hi ^ (r & 15)) * 16);
  auto read_fragment = [&](int nt, int ks) {
    asm volatile("ds_read_b128 %0, %1" : "=v"(bfr[ks]) : "v"((frag0_at ^ (uint32_t)(ks * 32)) + (uint32_t)nt * kTileBytes));
  };
  float best = -INFINITY;
  // One eighth of the maximum / subtract work on a finished tile's accumulators.
  auto epilogue_part = [&](f32x16 (&P)[kMT], int part) {
#pragma unroll
    for (int e = 4 * part; e < 4 * part + 4; ++e) {
      const int mt = e / 16, v = e % 16;
      if (PASS == 0) aux[mt][v] = fmaxf(aux[mt][v], P[mt][v]);
      else best = fmaxf(best, P[mt][v] - aux[mt][v]);
    }
  };
  auto epilogue_end = [&](int nt) {
    if (PASS == 1) {
      // The other half-wave's maximum for the same token: a lane swap in the vector unit (an LDS-routed
      // shuffle would put a wait for every outstanding fragment read into each tile).  Both halves then hold
      // the column maximum and both fold it into LDS: an integer maximum, exact and order-free.
      const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(best), __float_as_uint(best), false, false);
      best = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
      asm volatile("ds_max_u32 %0, %1" ::"v"(lds_colmax + (uint32_t)(32 * (nt + 1) + r) * 4), "v"(ordered_key(best)) : "memory");
      best = -INFINITY;
    }
  };
  // Tile nt into C; meanwhile the fragments of tile nt+1 are fetched and the epilogue of tile nt-1, held in
  // P, is done.  The first tile's "previous tile" is a set of -inf (its column maxima go to the spare slots in
  // front of colmax); behind the last tile the fetch reads what follows the share in LDS and nothing uses it:
  // every step is the same code.
  auto step = [&](int nt, f32x16 (&C)[kMT], f32x16 (&P)[kMT]) {
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < kKSteps; ++ks) {
      asm volatile("s_waitcnt lgkmcnt(7)" : "+v"(bfr[ks]));
#pragma unroll
      for (int mt = 0; mt < kMT; ++mt)
        C[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mt][ks], bfr[ks], ks == 0 ? zero : C[mt], 0, 0, 0);
      read_fragment(nt + 1, ks);
      epilogue_part(P, ks);
    }
    epilogue_end(nt - 1);
    __builtin_amdgcn_sched_barrier(0);                       // a tile's work stays inside its step
  };
  // streaming: the share is still landing.  Tiles become usable in growing groups: 0-1 behind the barrier in
  // front of the loop, then 2-3, 4-7 and 8-15, each behind a barrier in front of the odd step that fetches
  // the group's first fragments.  Early on this follows the arrival of the data; later, when the data is
  // ahead of the arithmetic, the waves run free of each other (a barrier per pair of tiles costs more than
  // it hides: of the two waves of a SIMD one gets ahead, waits, and the other cannot fill the matrix pipe
  // alone).  The number of tiles is even.
  auto run_tiles = [&](bool streaming, bool active) {
    if (!active) {
      if (streaming)
        for (int nt = 0; nt + 2 < tpb && nt <= 6; nt += nt + 2)       // nt = 0, 2, 6: the barriers below
          wait_loads_then_barrier(nt == 0 ? 12 : (nt == 2 ? 8 : 0));
      return;
    }
#pragma unroll
    for (int ks = 0; ks < kKSteps; ++ks) read_fragment(0, ks);
#pragma unroll
    for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc1[mt][v] = -INFINITY;
    __builtin_amdgcn_s_waitcnt(0xC07F);                      // lgkmcnt(0), where the compiler sees it: not inside the loop
    for (int nt = 0; nt < tpb; nt += 2) {
      step(nt, acc0, acc1);
      if (streaming && nt + 2 < tpb && (nt == 0 || nt == 2 || nt == 6))
        wait_loads_then_barrier(nt == 0 ? 12 : (nt == 2 ? 8 : 0));
      step(nt + 1, acc1, acc0);
    }
#pragma unroll
    for (int ks = 0; ks < kKSteps; ++ks) epilogue_part(acc1, ks);
    epilogue_end(tpb - 1);
  };

  // PASS 0: 32 running maxima per lane, each to be reduced over the 32 lanes of a half-wave: a butterfly
  // that halves the number of values per step (31 exchanges instead of 160).  Every exchange is a vector-unit
  // move: the two 16-lane rows of the half-wave swap (v_permlane16_swap hands both directions over at once),
  // then inside a row lane i pairs with i ^ 8 (row rotation by 8), with 7 - i inside its group of eight
  // (half-row mirror), with i ^ 1 and with i ^ 2 (quad permutations).  The side a lane keeps is decided by its
  // bits 4, 3, 2, 0, 1 in that order, so lane r ends up with value (r & 28) | (r & 1) << 1 | (r >> 1) & 1.
  auto flush_row_maxima = [&](int q0) {
    float red[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) red[i] = aux[i / 16][i % 16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {     // rows: an even row keeps values 0..15, the odd row 16..31
      const auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(red[i]), __float_as_uint(red[i + 16]), false, false);
      red[i] = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    }
#define ESA_EXCHANGE_STEP(cnt, bit, ctrl)                                                                          \
    {                                                                                                              \
      const bool upper = (r & (bit)) != 0;                                                                         \
      _Pragma("unroll") for (int i = 0; i < (cnt) / 2; ++i) {                                                      \
        const float lo_v = red[i], hi_v = red[i + (cnt) / 2];                                                      \
        const float keep = upper ? hi_v : lo_v, send = upper ? lo_v : hi_v;                                        \
        red[i] = fmaxf(keep, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(send), (ctrl), 0xF, 0xF, true))); \
      }                                                                                                            \
    }
    ESA_EXCHANGE_STEP(16, 8, 0x128)    // row_ror:8
    ESA_EXCHANGE_STEP(8, 4, 0x141)     // row_half_mirror
    ESA_EXCHANGE_STEP(4, 1, 0xB1)      // quad_perm [1,0,3,2]
    ESA_EXCHANGE_STEP(2, 2, 0x4E)      // quad_perm [2,3,0,1]
#undef ESA_EXCHANGE_STEP
    const int held = (r & 28) | ((r & 1) << 1) | ((r >> 1) & 1);
    const int mt = held / 16, v = held % 16;
    const int qrow = q0 + 32 * mt + 8 * (v / 4) + 4 * hi + (v % 4);
    // 32-bit index (batch x l_c x workgroups stays far below 2^32): scalar base + lane offset, no 64-bit address
    // to carry through the tile loop
    if (qrow < l_c) part_max[((uint32_t)b * (uint32_t)l_c + (uint32_t)qrow) * (uint32_t)n_wg + __builtin_amdgcn_workgroup_id_x()] = red[0];
  };

  // ---- requests, in the order their results are needed (loads complete in order): query fragments and row
  // maxima, then the K' share.  Instruction i of wave w fills row group 8*i + w (four rows, 1 KB of
  // LDS); lane l fetches, for slot l%16 of row l/16 of the group, the piece that undoes the swizzle.
  // Rows past the end of the middle segment repeat its last token (no maximum changes, nothing of theirs
  // is stored); shares shorter than sixteen tiles repeat their last instruction, identical data to an
  // identical place, so that the count of outstanding loads means the same in every workgroup.
  if (PASS == 1) {
    for (int i = tid; i < span + 32; i += kThreads) colmax[i] = kOrderedKeyOfMinusInf;
    if (first_hist)
      for (int i = tid; i < kRadixBins; i += kThreads) digit_hist[i] = 0u;
  }
  request_query_block(0);
  __builtin_amdgcn_sched_barrier(0);
  {
    const uint32_t row_in_tile = 4 * wave + (lane >> 4);
    const uint32_t piece = (lane & 15) ^ (row_in_tile & 15);
#pragma unroll
    for (int i = 0; i < kMaxTilesPerBlock; ++i) {
      const int t = i < tpb ? i : tpb - 1;
      uint32_t row = 32 * t + row_in_tile;
      row = row < last_row ? row : last_row;
      __builtin_amdgcn_global_load_lds((global_void*)(kshare + (size_t)row * (kDc * sizeof(bf16_t)) + piece * 16),
                                       (lds_void*)(lds_raw + (size_t)(8 * t + wave) * 1024), 16, 0, 0);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  queries_arrived(true);
  wait_loads_then_barrier(14);                               // tiles 0 and 1 (and this wave's LDS writes above)

  // ---- query blocks (chunks longer than 512 tokens take several); from the second on, the share is in LDS
  for (int qb = 0; qb * kQPerBlock < l_c; ++qb) {
    if (qb > 0) {
      qb_now = qb;
      request_query_block(qb);
      queries_arrived(false);
    }
    run_tiles(qb == 0, wave_has_queries(qb));
    if (PASS == 0 && wave_has_queries(qb)) {      // the sixteen fragments are shared out over the first workgroups
      // The lane number is taken afresh here: an address computed at the top of the kernel would be one more
      // value to keep (or spill) through the tile loop, whose registers are all spoken for.
      // fragment i goes out from workgroup i (from workgroup 0 on a tiny grid)
      uint32_t lane_now;
      asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane_now));
#pragma unroll
      for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks)
          if (mt * kKSteps + ks == (int)__builtin_amdgcn_workgroup_id_x() || (__builtin_amdgcn_workgroup_id_x() == 0 && mt * kKSteps + ks >= n_wg))
            *(bf16x8*)(qfrag + (int64_t)b * qfrag_bs + ((((int64_t)qb * kWaves + wave) * kMT + mt) * kKSteps + ks) * 512 +
                       lane_now * 8) = a[mt][ks];
    }
    if (PASS == 0 && wave_has_queries(qb)) flush_row_maxima(qb * kQPerBlock + wave * kQPerWave);
    if (qb == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // repeated instructions of a short share
  }

  if (PASS == 1) {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // this wave's column maxima are in LDS
    __syncthreads();
    for (int i0 = 0; i0 < span; i0 += kThreads) {          // whole waves stay in step for hist_add
      const int i = i0 + tid;
      const int64_t m = tok_base + i;
      const bool ok = i < span && m < n;
      const uint32_t key = ok ? colmax[32 + i] : 0u;
      if (ok) score[(int64_t)b * score_bs + m] = ordered_key_to_f32(key);
      if (first_hist) hist_add(digit_hist, ok, key >> 21);
    }
    if (first_hist) {
      __syncthreads();
      uint32_t* gh = first_hist + (int64_t)b * first_hist_bs;
      hist_flush(gh, digit_hist, __builtin_amdgcn_workgroup_id_x(), tid, kThreads);
    }
  }
}

// mu[c] = max over workgroups of their partial row maxima ([l_c][blocks] layout): one wave per query.
// Running between the two sweeps, it also zeroes the selection's three digit histograms when given them.
__global__ __launch_bounds__(256) void score_rowmax_reduce(const float* __restrict__ part_max, int nblk, int l_c,
                                                           float* __restrict__ mu, int mu_stride,
                                                           uint32_t* __restrict__ hists, int64_t hists_bs) {
  const int lane = __builtin_amdgcn_workitem_id_x() & 63;
  const int c = __builtin_amdgcn_workgroup_id_x() * 4 + (__builtin_amdgcn_workitem_id_x() >> 6);
  const int b = __builtin_amdgcn_workgroup_id_y();
  if (hists)
    for (int i = __builtin_amdgcn_workgroup_id_x() * 256 + __builtin_amdgcn_workitem_id_x(); i < kHistWords; i += (l_c + 3) / 4 * 256)
      hists[(int64_t)b * hists_bs + i] = 0u;                 // (l_c + 3) / 4 workgroups of 256 threads
  if (c >= l_c) return;
  const float* p = part_max + ((int64_t)b * l_c + c) * nblk;
  float m = -INFINITY;
  for (int i0 = lane; i0 < nblk; i0 += 4 * 64) {      // four loads in flight per lane (256 workgroups per trip)
    float v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + 64 * u;
      v[u] = p[i < nblk ? i : lane];
      if (i >= nblk) v[u] = -INFINITY;
    }
    m = fmaxf(fmaxf(m, v[0]), fmaxf(fmaxf(v[1], v[2]), v[3]));
  }
  m = wave_max(m);
  if (lane == 0) mu[(int64_t)b * mu_stride + c] = m;
}

// ------------------------------------------------------------------------------------------ decode (l_c = 1)
// One current token: S is a matrix-vector product over the whole compressed-key cache, pure HBM
// streaming.  LPR lanes share a K' row (16 bytes each), so a wave reads 64*16 contiguous bytes per
// step; a workgroup covers 256 rows with all its steps' loads in flight.  Writes S and the workgroup's maximum of it (no atomics: thousands of
// workgroups folding into one word serialise in L2); score_sub_mu then reduces those maxima to mu,
// every workgroup for itself, and forms F = S - mu.
constexpr int kGemvRows = 256;           // rows per workgroup
// grids of the passes over the scores (host and device agree on them; the kernels do not ask the dispatch packet)
__host__ __device__ inline int sub_mu_blocks(int64_t n) { return (int)((n + 1023) / 1024 < 2048 ? (n + 1023) / 1024 : 2048); }
__host__ __device__ inline int maxpool_blocks(int64_t n) { return (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096); }

// Sum over groups of LPR consecutive lanes (LPR = 8, 16, 32) with DPP moves; every lane gets the total.
template <int LPR>
__device__ __forceinline__ float lanes_sum(float v) {
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));    // quad_perm [1,0,3,2]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));    // quad_perm [2,3,0,1]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true));   // row_half_mirror
  if (LPR >= 16) v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true));   // row_mirror
  if (LPR >= 32) v += __shfl_xor(v, 16, 64);
  return v;
}

template <int LPR>
__global__ __launch_bounds__(256) void score_gemv_bf16(const bf16_t* __restrict__ qc, const bf16_t* __restrict__ kc,
                                                       int64_t m_lo, int64_t n, float* __restrict__ part,
                                                       float* __restrict__ raw, int64_t q_bs, int64_t kc_bs,
                                                       int64_t raw_bs, uint32_t* __restrict__ hists, int64_t hists_bs) {
  constexpr int kDcv = LPR * 8;
  constexpr int kRowsPerStep = 256 / LPR;
  constexpr int kGemvSteps = kGemvRows / kRowsPerStep;
  const int n_wg = (int)((n + kGemvRows - 1) / kGemvRows);           // workgroups per batch entry (the launch's grid)
  __shared__ float red[4];
  const int b = __builtin_amdgcn_workgroup_id_y();
  if (hists)       // the selection's digit histograms, zeroed here for the pass that follows
    for (int i = __builtin_amdgcn_workgroup_id_x() * 256 + __builtin_amdgcn_workitem_id_x(); i < kHistWords; i += n_wg * 256)
      hists[(int64_t)b * hists_bs + i] = 0u;
  const bf16_t* kmid = kc + (int64_t)b * kc_bs + m_lo * (int64_t)kDcv;
  const int sub = __builtin_amdgcn_workitem_id_x() % LPR, grp = __builtin_amdgcn_workitem_id_x() / LPR;
  float qv[8];
  {
    const uint4 u = *(const uint4*)(qc + (int64_t)b * q_bs + sub * 8);
    qv[0] = __uint_as_float(u.x << 16); qv[1] = __uint_as_float(u.x & 0xFFFF0000u);
    qv[2] = __uint_as_float(u.y << 16); qv[3] = __uint_as_float(u.y & 0xFFFF0000u);
    qv[4] = __uint_as_float(u.z << 16); qv[5] = __uint_as_float(u.z & 0xFFFF0000u);
    qv[6] = __uint_as_float(u.w << 16); qv[7] = __uint_as_float(u.w & 0xFFFF0000u);
  }
  float best = -INFINITY;
  const int64_t row0 = (int64_t)__builtin_amdgcn_workgroup_id_x() * kGemvRows;
#pragma unroll
  for (int it = 0; it < kGemvSteps; ++it) {
    const int64_t row = row0 + it * kRowsPerStep + grp;
    uint4 u = make_uint4(0u, 0u, 0u, 0u);
    if (row < n) u = *(const uint4*)(kmid + row * kDcv + sub * 8);
    float s = qv[0] * __uint_as_float(u.x << 16);
    s = __fmaf_rn(qv[1], __uint_as_float(u.x & 0xFFFF0000u), s);
    s = __fmaf_rn(qv[2], __uint_as_float(u.y << 16), s);
    s = __fmaf_rn(qv[3], __uint_as_float(u.y & 0xFFFF0000u), s);
    s = __fmaf_rn(qv[4], __uint_as_float(u.z << 16), s);
    s = __fmaf_rn(qv[5], __uint_as_float(u.z & 0xFFFF0000u), s);
    s = __fmaf_rn(qv[6], __uint_as_float(u.w << 16), s);
    s = __fmaf_rn(qv[7], __uint_as_float(u.w & 0xFFFF0000u), s);
    s = lanes_sum<LPR>(s);
    if (row < n) {
      if (sub == 0) raw[(int64_t)b * raw_bs + row] = s;
      best = fmaxf(best, s);
    }
  }
  best = wave_max(best);
  if ((__builtin_amdgcn_workitem_id_x() & 63) == 0) red[__builtin_amdgcn_workitem_id_x() >> 6] = best;
  __syncthreads();
  if (__builtin_amdgcn_workitem_id_x() == 0)
    part[(int64_t)b * n_wg + __builtin_amdgcn_workgroup_id_x()] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

__global__ __launch_bounds__(256) void score_sub_mu(float* __restrict__ raw, int64_t n, const float* __restrict__ part,
                                                    int n_part, int64_t raw_bs, uint32_t* __restrict__ first_hist,
                                                    int64_t first_hist_bs) {
  __shared__ float red[4];
  __shared__ uint32_t digit_hist[kRadixBins];
  const int n_wg = sub_mu_blocks(n);                          // workgroups per batch entry (the launch's grid)
  if (first_hist)
    for (int i = __builtin_amdgcn_workitem_id_x(); i < kRadixBins; i += 256) digit_hist[i] = 0u;
  float* p = raw + (int64_t)__builtin_amdgcn_workgroup_id_y() * raw_bs;
  // A workgroup owns chunks of 1024 consecutive scores (the first one is the chunk the selection's workgroup of
  // the same number reads next: written and read on the same XCD), a thread four scores 256 apart.
  const int64_t first = (int64_t)__builtin_amdgcn_workgroup_id_x() * 1024 + __builtin_amdgcn_workitem_id_x(), stride = 256;
  const int64_t chunk_stride = (int64_t)n_wg * 1024;
  // this thread's first four scores are requested together with the partial maxima: one round trip
  float x[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int64_t i = first + u * stride;
    x[u] = i < n ? p[i] : 0.f;
  }
  float mu = -INFINITY;
  for (int i0 = __builtin_amdgcn_workitem_id_x(); i0 < n_part; i0 += 4 * 256) {
    float v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + 256 * u;
      v[u] = part[(int64_t)__builtin_amdgcn_workgroup_id_y() * n_part + (i < n_part ? i : 0)];
      if (i >= n_part) v[u] = -INFINITY;
    }
    mu = fmaxf(fmaxf(mu, v[0]), fmaxf(fmaxf(v[1], v[2]), v[3]));
  }
  mu = wave_max(mu);
  if ((__builtin_amdgcn_workitem_id_x() & 63) == 0) red[__builtin_amdgcn_workitem_id_x() >> 6] = mu;
  __syncthreads();
  mu = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int64_t i = first + u * stride;
    const float f = x[u] - mu;
    if (i < n) p[i] = f;
    if (first_hist) hist_add(digit_hist, i < n, ordered_key(f) >> 21);
  }
  // whole waves stay in the loop together (hist_add is a wave-wide operation); four scores in flight per lane
  for (int64_t c0 = (int64_t)__builtin_amdgcn_workgroup_id_x() * 1024 + chunk_stride; c0 < n; c0 += chunk_stride) {
    float y[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t i = c0 + u * stride + __builtin_amdgcn_workitem_id_x();
      y[u] = i < n ? p[i] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t i = c0 + u * stride + __builtin_amdgcn_workitem_id_x();
      const float f = y[u] - mu;
      if (i < n) p[i] = f;
      if (first_hist) hist_add(digit_hist, i < n, ordered_key(f) >> 21);
    }
  }
  if (first_hist) {
    __syncthreads();
    uint32_t* gh = first_hist + (int64_t)__builtin_amdgcn_workgroup_id_y() * first_hist_bs;
    hist_flush(gh, digit_hist, __builtin_amdgcn_workgroup_id_x(), __builtin_amdgcn_workitem_id_x(), 256);
  }
}

// Eq. 8: out[j] = max(in[max(j-eps,0) .. min(j+eps,n-1)]).  With first_hist given, also the histogram of the
// pooled scores' leading 11 key bits (this is the kernel that writes the scores the selection reads).
__global__ __launch_bounds__(256) void proximity_maxpool(const float* __restrict__ in, float* __restrict__ out, int64_t n,
                                                         int eps, int64_t in_bs, int64_t out_bs,
                                                         uint32_t* __restrict__ first_hist, int64_t first_hist_bs) {
  __shared__ uint32_t digit_hist[kRadixBins];
  const int n_wg = maxpool_blocks(n);                         // workgroups per batch entry (the launch's grid)
  if (first_hist)
    for (int i = __builtin_amdgcn_workitem_id_x(); i < kRadixBins; i += 256) digit_hist[i] = 0u;
  __syncthreads();
  const float* src = in + (int64_t)__builtin_amdgcn_workgroup_id_y() * in_bs;
  float* dst = out + (int64_t)__builtin_amdgcn_workgroup_id_y() * out_bs;
  // whole waves stay in the loop together (hist_add is a wave-wide operation)
  for (int64_t j0 = (int64_t)__builtin_amdgcn_workgroup_id_x() * 256 + (__builtin_amdgcn_workitem_id_x() & ~63); j0 < n; j0 += (int64_t)n_wg * 256) {
    const int64_t j = j0 + (__builtin_amdgcn_workitem_id_x() & 63);
    float m = 0.f;
    if (j < n) {
      const int64_t lo = j - eps > 0 ? j - eps : 0, hi = j + eps < n - 1 ? j + eps : n - 1;
      m = src[lo];
      for (int64_t w = lo + 1; w <= hi; ++w) m = fmaxf(m, src[w]);
      dst[j] = m;
    }
    if (first_hist) hist_add(digit_hist, j < n, ordered_key(m) >> 21);
  }
  if (first_hist) {
    __syncthreads();
    uint32_t* gh = first_hist + (int64_t)__builtin_amdgcn_workgroup_id_y() * first_hist_bs;
    hist_flush(gh, digit_hist, __builtin_amdgcn_workgroup_id_x(), __builtin_amdgcn_workitem_id_x(), 256);
  }
}

}  // namespace

__host__ inline size_t part_bytes(int l_c, int64_t n_mid, int batch) {
  size_t blocks = (size_t)mfma_blocks(n_mid) * l_c;
  if (l_c == 1) {   // the one-token kernel: a partial maximum per workgroup of at least 256 rows
    const size_t gemv_blocks = (size_t)((n_mid + 255) / 256);
    blocks = gemv_blocks > blocks ? gemv_blocks : blocks;
  }
  return align_up(blocks * batch * 4, 256);
}

// fragment-ordered copy of Q' (matrix-core path): whole blocks of 512 queries, 256 bytes each
__host__ inline size_t qfrag_bytes_per_batch(int l_c) {
  return l_c > 1 ? (size_t)((l_c + kQPerBlock - 1) / kQPerBlock) * kQPerBlock * kDc * sizeof(bf16_t) : 0;
}

size_t score_workspace_bytes(int l_c, int64_t n_mid, int eps, int batch) {
  if (l_c <= 0 || batch <= 0 || n_mid < 0) return 256;
  size_t b = mu_bytes(l_c, batch) + part_bytes(l_c, n_mid, batch);
  if (eps > 0) b += align_up((size_t)n_mid * 4, 256) * (size_t)batch;
  b += qfrag_bytes_per_batch(l_c) * (size_t)batch;
  return b;
}

int launch_score(const void* qc, int l_c, const void* kc_cache, int64_t m_lo, int64_t m_hi, int d_c, int eps,
                 float* score, int dtype, int batch, int64_t q_bs, int64_t kc_bs, int64_t score_bs, void* ws,
                 size_t ws_bytes, hipStream_t st, uint32_t* first_hist, int64_t first_hist_bs, bool* first_hist_done) {
  const int64_t n = m_hi - m_lo;
  // With pooling the kernel that writes the final scores is the pooling pass: the kernels before it only zero
  // the histograms (pool_hist), it fills the first one.
  uint32_t* pool_hist = eps > 0 ? first_hist : nullptr;
  bool zeroed = false;
  if (first_hist_done) *first_hist_done = false;
  uint32_t* mu = (uint32_t*)ws;
  float* raw = score;
  int64_t raw_bs = score_bs;
  if (eps > 0) {
    raw = (float*)((char*)ws + mu_bytes(l_c, batch) + part_bytes(l_c, n, batch));
    raw_bs = (int64_t)(align_up((size_t)n * 4, 256) / 4);
  }
  const bool vec_ok = dtype == ESA_BF16 && (((uintptr_t)qc | (uintptr_t)kc_cache) % 16 == 0) && q_bs % 8 == 0 &&
                      kc_bs % 8 == 0;
  if (vec_ok && l_c == 1 && (d_c == 64 || d_c == 128 || d_c == 256)) {
    const int lpr = d_c / 8;
    const int nblk = (int)((n + kGemvRows - 1) / kGemvRows);
    const dim3 grid((unsigned)nblk, batch);
    const bf16_t* q = (const bf16_t*)qc;
    const bf16_t* k = (const bf16_t*)kc_cache;
    float* part = (float*)((char*)ws + mu_bytes(l_c, batch));
    uint32_t* fh = first_hist;
    const int64_t fbs = first_hist_bs;
    zeroed = fh != nullptr;
    if (lpr == 8) score_gemv_bf16<8><<<grid, 256, 0, st>>>(q, k, m_lo, n, part, raw, q_bs, kc_bs, raw_bs, fh, fbs);
    else if (lpr == 16) score_gemv_bf16<16><<<grid, 256, 0, st>>>(q, k, m_lo, n, part, raw, q_bs, kc_bs, raw_bs, fh, fbs);
    else score_gemv_bf16<32><<<grid, 256, 0, st>>>(q, k, m_lo, n, part, raw, q_bs, kc_bs, raw_bs, fh, fbs);
    const int blocks = sub_mu_blocks(n);
    score_sub_mu<<<dim3(blocks, batch), 256, 0, st>>>(raw, n, part, nblk, raw_bs, pool_hist ? nullptr : fh, fbs);
    if (fh && !pool_hist && first_hist_done) *first_hist_done = true;
  } else if (vec_ok && d_c == kDc) {
    const int per = (int)mfma_tiles_per_block(n);
    const int nblk = (int)mfma_blocks(n);
    const dim3 grid(nblk, batch);
    float* part = (float*)((char*)ws + mu_bytes(l_c, batch));
    float* muf = (float*)ws;
    const size_t lds0 = mfma_lds_bytes(per), lds1 = lds0;
    static bool lds_limit_raised = false;      // idempotent; a race only repeats the call
    if (!lds_limit_raised) {
      const int most = (int)mfma_lds_bytes(kMaxTilesPerBlock);
      hipError_t e = hipFuncSetAttribute((const void*)score_mfma_bf16<0>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         most);
      if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)score_mfma_bf16<1>, hipFuncAttributeMaxDynamicSharedMemorySize, most);
      if (e != hipSuccess) return hip_failed(e, "hipFuncSetAttribute(score_mfma_bf16)");
      lds_limit_raised = true;
    }
    size_t qfrag_at = mu_bytes(l_c, batch) + part_bytes(l_c, n, batch);
    if (eps > 0) qfrag_at += align_up((size_t)n * 4, 256) * (size_t)batch;
    bf16_t* qfrag = (bf16_t*)((char*)ws + qfrag_at);
    const int64_t qfrag_bs = (int64_t)(qfrag_bytes_per_batch(l_c) / sizeof(bf16_t));
    score_mfma_bf16<0><<<grid, kThreads, lds0, st>>>((const bf16_t*)qc, l_c, (const bf16_t*)kc_cache, m_lo, n, part, muf,
                                                raw, q_bs, kc_bs, raw_bs, per, nullptr, 0, qfrag, qfrag_bs, nblk);
    score_rowmax_reduce<<<dim3((l_c + 3) / 4, batch), 256, 0, st>>>(part, nblk, l_c, muf, mfma_mu_stride(l_c), first_hist,
                                                                  first_hist_bs);
    score_mfma_bf16<1><<<grid, kThreads, lds1, st>>>((const bf16_t*)qc, l_c, (const bf16_t*)kc_cache, m_lo, n, part, muf,
                                                raw, q_bs, kc_bs, raw_bs, per, pool_hist ? nullptr : first_hist,
                                                first_hist_bs, qfrag, qfrag_bs, nblk);
    zeroed = first_hist != nullptr;
    if (first_hist && !pool_hist && first_hist_done) *first_hist_done = true;
  } else {
    fill_u32<<<(l_c * batch + 255) / 256, 256, 0, st>>>(mu, (int64_t)l_c * batch, kOrderedKeyOfMinusInf);
    const dim3 grid((unsigned)((n + kGTok - 1) / kGTok), batch);
    const size_t smem = (size_t)(kGTok * (d_c + 1) + 4 * kGTok) * sizeof(float);
    if (smem > 65536) {   // d_c > 240: raise the dynamic LDS limit of the four instantiations
      const void* fns[] = {(const void*)score_fma<bf16_t, 0>, (const void*)score_fma<bf16_t, 1>,
                           (const void*)score_fma<float, 0>, (const void*)score_fma<float, 1>};
      for (const void* f : fns) {
        hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return hip_failed(e, "hipFuncSetAttribute(score_fma)");
      }
    }
    if (dtype == ESA_BF16) {
      score_fma<bf16_t, 0><<<grid, 256, smem, st>>>((const bf16_t*)qc, l_c, (const bf16_t*)kc_cache, m_lo, n, d_c, mu,
                                                    raw, q_bs, kc_bs, raw_bs);
      score_fma<bf16_t, 1><<<grid, 256, smem, st>>>((const bf16_t*)qc, l_c, (const bf16_t*)kc_cache, m_lo, n, d_c, mu,
                                                    raw, q_bs, kc_bs, raw_bs);
    } else {
      score_fma<float, 0><<<grid, 256, smem, st>>>((const float*)qc, l_c, (const float*)kc_cache, m_lo, n, d_c, mu,
                                                   raw, q_bs, kc_bs, raw_bs);
      score_fma<float, 1><<<grid, 256, smem, st>>>((const float*)qc, l_c, (const float*)kc_cache, m_lo, n, d_c, mu,
                                                   raw, q_bs, kc_bs, raw_bs);
    }
  }
  if (eps > 0) {
    const int blocks = maxpool_blocks(n);
    uint32_t* ph = zeroed ? pool_hist : nullptr;       // only behind kernels that have zeroed the histograms
    proximity_maxpool<<<dim3(blocks, batch), 256, 0, st>>>(raw, score, n, eps, raw_bs, score_bs, ph, first_hist_bs);
    if (ph && first_hist_done) *first_hist_done = true;
  }
  ESA_LAUNCH_CHECK("score");
  return ESA_OK;
}

}  // namespace esa
