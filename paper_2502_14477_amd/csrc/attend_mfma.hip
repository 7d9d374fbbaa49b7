// Selected attention (Eq. 1) on the matrix cores: bf16 storage, head size 128.
//
// Work decomposition.  The query heads of one KV group share keys and values, so a workgroup
// owns 256 "rows" = (heads of one KV group) x (256/G consecutive current tokens) and one slice of
// the virtual key sequence [I | M_k | L | C]; slices of one row tile are merged afterwards with
// the log-sum-exp rule of Algorithm 1 (esa_attend_merge).  Four waves, 64 rows each.
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
// registers (4x4 blocks of bf16), K is copied as is.
#include "attend_mfma.h"
#include "keyspace.h"

namespace esa {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kD = 128;             // head size
constexpr int kKT = 64;             // virtual keys per tile
constexpr int kRows = 256;          // query rows per workgroup
constexpr int kKLd = kD + 8;        // LDS row stride of the K tile in elements (272 B: conflict-free 16-byte reads)
constexpr int kVLd = kKT + 8;       // LDS row stride of the V^T tile in elements (144 B)
constexpr int kMaxSplits = 8;
constexpr int kMinLc = 16;          // shorter chunks go to the plain kernel
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct AttendArgs {
  const bf16_t* q;
  bf16_t* out;
  float* lse;
  float* part_o;      // [batch][n_split][l_c][h][128] unnormalised partial outputs
  float* part_ml;     // [batch][n_split][l_c][h][2]   running maximum (log2 domain) and sum
  KeySpace ks;
  int l_c, h, h_kv, group, qpt, n_qt, n_split;
  int64_t n_fixed;
  float c2;           // scale * log2(e)
  int64_t q_bs, out_bs, cache_bs_bytes, sel_bs_bytes;
};

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 f = {lo, hi};
  bf16x2 b = __builtin_convertvector(f, bf16x2);
  return *(uint32_t*)&b;
}

__global__ __launch_bounds__(256) void attend_mfma_bf16(AttendArgs a) {
  __shared__ __attribute__((aligned(16))) bf16_t k_lds[kKT * kKLd];
  __shared__ __attribute__((aligned(16))) bf16_t vt_lds[kD * kVLd];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 31, hi = lane >> 5;
  const int qt = blockIdx.x % a.n_qt, split = blockIdx.x / a.n_qt, g = blockIdx.y, b = blockIdx.z;
  KeySpace ks = a.ks;
  ks.k_cache += (int64_t)b * a.cache_bs_bytes + (int64_t)g * kD * 2;
  ks.v_cache += (int64_t)b * a.cache_bs_bytes + (int64_t)g * kD * 2;
  if (ks.n_sel > 0) {
    ks.k_sel += (int64_t)b * a.sel_bs_bytes + (int64_t)g * kD * 2;
    ks.v_sel += (int64_t)b * a.sel_bs_bytes + (int64_t)g * kD * 2;
  }

  // ---- this workgroup's rows and key slice
  const int q0 = qt * a.qpt;
  const int c_last = (q0 + a.qpt < a.l_c ? q0 + a.qpt : a.l_c) - 1;
  const int64_t n_vis = a.n_fixed + c_last + 1;                    // keys the tile's last token sees
  const int64_t n_tiles = (n_vis + kKT - 1) / kKT;
  const int64_t tile_begin = n_tiles * split / a.n_split, tile_end = n_tiles * (split + 1) / a.n_split;
  const int64_t k_end = tile_end * kKT < n_vis ? tile_end * kKT : n_vis;

  const int tph = a.qpt / 32;                                      // 32-row tiles per head
  int head[2], c[2];
  bool c_ok[2];
  int64_t lim[2];                                                  // first virtual key this lane's query may NOT see
  bf16x8 qf[2][kD / 16];
#pragma unroll
  for (int nq = 0; nq < 2; ++nq) {
    const int nt = 2 * wave + nq;
    head[nq] = g * a.group + nt / tph;
    c[nq] = q0 + (nt % tph) * 32 + r;
    c_ok[nq] = c[nq] < a.l_c;
    const int cc = c_ok[nq] ? c[nq] : a.l_c - 1;                   // rows past the chunk repeat its last token
    const int64_t vis = a.n_fixed + cc + 1;
    lim[nq] = vis < k_end ? vis : k_end;
    const bf16_t* qp = a.q + (int64_t)b * a.q_bs + ((int64_t)cc * a.h + head[nq]) * kD + hi * 8;
#pragma unroll
    for (int ks16 = 0; ks16 < kD / 16; ++ks16) qf[nq][ks16] = *(const bf16x8*)(qp + ks16 * 16);
  }
  const int64_t lim_lo0 = __shfl(lim[0], 0, 64), lim_lo1 = __shfl(lim[1], 0, 64);
  const int64_t lim_lo = lim_lo0 < lim_lo1 ? lim_lo0 : lim_lo1;    // smallest limit in the wave (r = 0)

  f32x16 o[2][4];
#pragma unroll
  for (int nq = 0; nq < 2; ++nq)
#pragma unroll
    for (int md = 0; md < 4; ++md)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[nq][md][v] = 0.f;
  float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};

  // ---- staging of one tile: global -> registers -> LDS
  uint4 kreg[4];
  uint2 vreg[2][4];
  const int vb = (lane >> 3) + 8 * wave;                           // which 4 head-dims (0..31)
  auto load_tile = [&](int64_t j0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + 256 * i;
      int64_t j = j0 + (id >> 4);
      j = j < k_end ? j : k_end - 1;                               // the tail repeats a key; masked below
      kreg[i] = *(const uint4*)(key_row(ks, j, false) + (id & 15) * 16);
    }
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int ap = (lane & 7) + 8 * p;                           // 4-key group as stored in LDS
      const int sw = ap & 3;
      const int ag = (ap & ~3) | (sw == 1 ? 2 : sw == 2 ? 1 : sw); // 4-key group in key order
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        int64_t j = j0 + 4 * ag + kk;
        j = j < k_end ? j : k_end - 1;
        vreg[p][kk] = *(const uint2*)(key_row(ks, j, true) + vb * 8);
      }
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + 256 * i;
      *(uint4*)&k_lds[(id >> 4) * kKLd + (id & 15) * 8] = kreg[i];
    }
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int ap = (lane & 7) + 8 * p;
      // 4 keys x 4 dims -> 4 dims x 4 keys
      const uint32_t r0l = vreg[p][0].x, r0h = vreg[p][0].y, r1l = vreg[p][1].x, r1h = vreg[p][1].y;
      const uint32_t r2l = vreg[p][2].x, r2h = vreg[p][2].y, r3l = vreg[p][3].x, r3h = vreg[p][3].y;
      uint2 d0, d1, d2, d3;
      d0.x = (r0l & 0xFFFFu) | (r1l << 16);
      d0.y = (r2l & 0xFFFFu) | (r3l << 16);
      d1.x = (r0l >> 16) | (r1l & 0xFFFF0000u);
      d1.y = (r2l >> 16) | (r3l & 0xFFFF0000u);
      d2.x = (r0h & 0xFFFFu) | (r1h << 16);
      d2.y = (r2h & 0xFFFFu) | (r3h << 16);
      d3.x = (r0h >> 16) | (r1h & 0xFFFF0000u);
      d3.y = (r2h >> 16) | (r3h & 0xFFFF0000u);
      bf16_t* dst = &vt_lds[(4 * vb) * kVLd + 4 * ap];
      *(uint2*)(dst) = d0;
      *(uint2*)(dst + kVLd) = d1;
      *(uint2*)(dst + 2 * kVLd) = d2;
      *(uint2*)(dst + 3 * kVLd) = d3;
    }
  };

  if (tile_begin < tile_end) load_tile(tile_begin * kKT);
  for (int64_t t = tile_begin; t < tile_end; ++t) {
    const int64_t j0 = t * kKT;
    __syncthreads();                     // every wave is done reading the previous tile
    store_tile();
    __syncthreads();
    if (t + 1 < tile_end) load_tile(j0 + kKT);

    // ---- S^T = K Q^T
    f32x16 s[2][2];
#pragma unroll
    for (int nq = 0; nq < 2; ++nq)
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) s[nq][mt][v] = 0.f;
#pragma unroll
    for (int ks16 = 0; ks16 < kD / 16; ++ks16)
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        const bf16x8 ka = *(const bf16x8*)&k_lds[(32 * mt + r) * kKLd + 16 * ks16 + 8 * hi];
#pragma unroll
        for (int nq = 0; nq < 2; ++nq)
          s[nq][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[nq][ks16], s[nq][mt], 0, 0, 0);
      }

    // ---- mask keys beyond each query's limit (causal diagonal, end of the slice)
    if (j0 + kKT > lim_lo) {
#pragma unroll
      for (int nq = 0; nq < 2; ++nq)
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int64_t j = j0 + 32 * mt + 8 * (v / 4) + 4 * hi + (v % 4);
            if (j >= lim[nq]) s[nq][mt][v] = -INFINITY;
          }
    }

    // ---- online softmax, one query per lane
    bf16x8 pf[2][4];
#pragma unroll
    for (int nq = 0; nq < 2; ++nq) {
      float mx = s[nq][0][0];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[nq][mt][v]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run[nq], mx * a.c2);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float corr = __builtin_amdgcn_exp2f(m_run[nq] - m_use);
      m_run[nq] = m_new;
      float psum = 0.f;
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[nq][mt][v], a.c2, -m_use));
          s[nq][mt][v] = p;
          psum += p;
        }
      l_run[nq] = l_run[nq] * corr + psum;
      if (__ballot(corr != 1.f) != 0ull) {
#pragma unroll
        for (int md = 0; md < 4; ++md)
#pragma unroll
          for (int v = 0; v < 16; ++v) o[nq][md][v] *= corr;
      }
#pragma unroll
      for (int kp = 0; kp < 4; ++kp) {
        const int mt = kp >> 1, v0 = (kp & 1) * 8;
        uint4 w;
        w.x = pack_bf16x2(s[nq][mt][v0 + 0], s[nq][mt][v0 + 1]);
        w.y = pack_bf16x2(s[nq][mt][v0 + 2], s[nq][mt][v0 + 3]);
        w.z = pack_bf16x2(s[nq][mt][v0 + 4], s[nq][mt][v0 + 5]);
        w.w = pack_bf16x2(s[nq][mt][v0 + 6], s[nq][mt][v0 + 7]);
        pf[nq][kp] = *(bf16x8*)&w;
      }
    }

    // ---- O^T += V^T P^T
#pragma unroll
    for (int kp = 0; kp < 4; ++kp)
#pragma unroll
      for (int md = 0; md < 4; ++md) {
        const bf16x8 va = *(const bf16x8*)&vt_lds[(32 * md + r) * kVLd + 16 * kp + 8 * hi];
#pragma unroll
        for (int nq = 0; nq < 2; ++nq)
          o[nq][md] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pf[nq][kp], o[nq][md], 0, 0, 0);
      }
  }

  // ---- results: accumulator register v of tile md is head-dim 32*md + 8*(v/4) + 4*hi + v%4 of this lane's query
#pragma unroll
  for (int nq = 0; nq < 2; ++nq) {
    const float l_tot = l_run[nq] + __shfl_xor(l_run[nq], 32, 64);
    if (!c_ok[nq]) continue;
    const int64_t row = (int64_t)c[nq] * a.h + head[nq];
    if (a.n_split == 1) {
      const float inv = 1.f / l_tot;
      bf16_t* op = a.out + (int64_t)b * a.out_bs + row * kD;
#pragma unroll
      for (int md = 0; md < 4; ++md)
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
          uint2 w;
          w.x = pack_bf16x2(o[nq][md][4 * vg + 0] * inv, o[nq][md][4 * vg + 1] * inv);
          w.y = pack_bf16x2(o[nq][md][4 * vg + 2] * inv, o[nq][md][4 * vg + 3] * inv);
          *(uint2*)(op + 32 * md + 8 * vg + 4 * hi) = w;
        }
      if (a.lse && hi == 0) a.lse[(int64_t)b * a.l_c * a.h + row] = (m_run[nq] + __builtin_amdgcn_logf(l_tot)) * kLn2;
    } else {
      const int64_t prow = ((int64_t)(b * a.n_split + split) * a.l_c) * a.h + row;
      float* pp = a.part_o + prow * kD;
#pragma unroll
      for (int md = 0; md < 4; ++md)
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
          float4 w = {o[nq][md][4 * vg + 0], o[nq][md][4 * vg + 1], o[nq][md][4 * vg + 2], o[nq][md][4 * vg + 3]};
          *(float4*)(pp + 32 * md + 8 * vg + 4 * hi) = w;
        }
      if (hi == 0) {
        float2 ml = {m_run[nq], l_tot};
        *(float2*)(a.part_ml + prow * 2) = ml;
      }
    }
  }
}

// Algorithm 1's merge over the key slices: weights 2^(m_s - M) with the maximum subtracted first.
__global__ __launch_bounds__(128) void esa_attend_merge(const float* __restrict__ part_o,
                                                        const float* __restrict__ part_ml, int n_split, int64_t rows,
                                                        bf16_t* __restrict__ out, float* __restrict__ lse,
                                                        int64_t out_bs, int64_t lse_bs) {
  const int64_t row = blockIdx.x;
  const int b = blockIdx.y;
  float m[kMaxSplits], l[kMaxSplits];
  float M = -INFINITY;
  for (int s = 0; s < n_split; ++s) {
    const float2 ml = *(const float2*)(part_ml + (((int64_t)b * n_split + s) * rows + row) * 2);
    m[s] = ml.x;
    l[s] = ml.y;
    M = fmaxf(M, ml.x);
  }
  float L = 0.f, acc = 0.f;
  for (int s = 0; s < n_split; ++s) {
    if (m[s] == -INFINITY) continue;              // a slice this query saw nothing of
    const float w = __builtin_amdgcn_exp2f(m[s] - M);
    L += w * l[s];
    acc += w * part_o[(((int64_t)b * n_split + s) * rows + row) * kD + threadIdx.x];
  }
  out[(int64_t)b * out_bs + row * kD + threadIdx.x] = f32_to_bf16(acc / L);
  if (lse && threadIdx.x == 0) lse[(int64_t)b * lse_bs + row] = (M + __builtin_amdgcn_logf(L)) * kLn2;
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

size_t attend_mfma_workspace_bytes(int l_c, int h, int h_kv, int d, int batch) {
  const int ns = choose_splits(l_c, h / h_kv, h_kv, batch);
  if (ns == 1) return 256;
  const size_t rows = (size_t)batch * ns * l_c * h;
  return align_up(rows * kD * sizeof(float), 256) + align_up(rows * 2 * sizeof(float), 256);
}

int launch_attend_mfma(const void* q, int l_c, int h, int h_kv, int d, const void* k_cache, const void* v_cache,
                       int64_t tok_stride, int64_t t0, int64_t i_end, int64_t l_start, const void* k_sel,
                       const void* v_sel, int n_sel, float scale, void* out, float* lse, int batch, int64_t q_bs,
                       int64_t cache_bs, int64_t sel_bs, int64_t out_bs, void* ws, size_t ws_bytes, hipStream_t st) {
  if (!(scale > 0.f)) ESA_FAIL(ESA_EINVAL, "esa_attend: scale must be positive");
  AttendArgs a;
  a.q = (const bf16_t*)q;
  a.out = (bf16_t*)out;
  a.lse = lse;
  a.ks.k_cache = (const char*)k_cache;
  a.ks.v_cache = (const char*)v_cache;
  a.ks.k_sel = (const char*)k_sel;
  a.ks.v_sel = (const char*)v_sel;
  a.ks.tok_bytes = tok_stride * 2;
  a.ks.sel_bytes = (int64_t)h_kv * d * 2;
  a.ks.i_end = i_end;
  a.ks.n_sel = n_sel;
  a.ks.l_start = l_start;
  a.l_c = l_c;
  a.h = h;
  a.h_kv = h_kv;
  a.group = h / h_kv;
  a.qpt = kRows / a.group;
  a.n_qt = (l_c + a.qpt - 1) / a.qpt;
  a.n_fixed = i_end + n_sel + (t0 - l_start);
  a.c2 = scale * kLog2e;
  a.q_bs = q_bs;
  a.out_bs = out_bs;
  a.cache_bs_bytes = cache_bs * 2;
  a.sel_bs_bytes = sel_bs * 2;
  int ns = choose_splits(l_c, a.group, h_kv, batch);
  const int64_t min_tiles = (a.n_fixed + (l_c < a.qpt ? l_c : a.qpt) + kKT - 1) / kKT;   // tiles of the first row tile
  if (ns > min_tiles) ns = (int)min_tiles;
  a.n_split = ns;
  a.part_o = nullptr;
  a.part_ml = nullptr;
  if (ns > 1) {
    const size_t rows = (size_t)batch * ns * l_c * h;
    const size_t need = align_up(rows * kD * sizeof(float), 256) + align_up(rows * 2 * sizeof(float), 256);
    if (!ws || ws_bytes < need) ESA_FAIL(ESA_EWORKSPACE, "esa_attend: workspace needs %zu bytes", need);
    a.part_o = (float*)ws;
    a.part_ml = (float*)((char*)ws + align_up(rows * kD * sizeof(float), 256));
  }
  attend_mfma_bf16<<<dim3(a.n_qt * ns, h_kv, batch), 256, 0, st>>>(a);
  if (ns > 1)
    esa_attend_merge<<<dim3((unsigned)((int64_t)l_c * h), batch), 128, 0, st>>>(a.part_o, a.part_ml, ns,
                                                                                (int64_t)l_c * h, (bf16_t*)out, lse,
                                                                                out_bs, (int64_t)l_c * h);
  ESA_LAUNCH_CHECK("attend_mfma");
  return ESA_OK;
}

}  // namespace esa
