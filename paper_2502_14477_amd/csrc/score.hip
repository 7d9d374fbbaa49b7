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
#include "esa_common.h"

namespace esa {
namespace {

// Workspace: [batch][l_c] row maxima (uint32 keys or fp32), [batch][blocks][l_c] fp32 partial row maxima of the
// matrix-core kernel, then (eps > 0) [batch][n] fp32 unpooled scores.
__host__ __device__ inline size_t mu_bytes(int l_c, int batch) { return align_up((size_t)l_c * batch * 4, 256); }

__global__ void fill_u32(uint32_t* p, int64_t n, uint32_t v) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
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
  const int b = blockIdx.y;
  const T* q = qc + (int64_t)b * q_bs;
  const T* k = kc + (int64_t)b * kc_bs + m_lo * (int64_t)d_c;
  uint32_t* mu = mu_keys + (int64_t)b * l_c;
  const int64_t m0 = (int64_t)blockIdx.x * kGTok;
  for (int e = threadIdx.x; e < kGTok * d_c; e += 256) {
    const int t = e / d_c, i = e % d_c;
    kt[t * ldk + i] = (m0 + t < n) ? load_f32(k + (m0 + t) * (int64_t)d_c + i) : 0.f;
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
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

// v_mfma_f32_32x32x16_bf16 computes D[32x32] += A[32x16] B[16x32].  Lane l supplies eight
// consecutive reduction elements of A row l%32 and of B column l%32 (which eight depends only on
// l/32, identically for A and B), and owns D[8*(v/4) + 4*(l/32) + v%4][l%32] in register v.
//
// Here A rows are current tokens (queries), B columns are middle tokens.  A workgroup of eight
// waves (two per SIMD, so one wave's maximum/subtract work overlaps the other's matrix
// instructions) keeps up to 512 compressed queries in registers (64 per wave, as A fragments for
// the whole d_c = 128) and streams its contiguous share of K' past them: 128-token stages are
// copied global -> registers -> LDS with full 256-byte rows per 16 lanes (double buffered, one
// barrier per stage), and every wave reads its B fragments from LDS.  K' is thus read from memory
// once per sweep and Q' once per workgroup.  With a token per lane, the column maximum of Eq. 4 is
// an in-lane reduction over the accumulator registers plus one exchange between the two
// half-waves; the row maximum is kept per register across all tiles and reduced across lanes
// once, then written as this workgroup's partial row maxima (no atomics) for score_rowmax_reduce.
constexpr int kDc = 128;
constexpr int kKSteps = kDc / 16;        // MFMA reduction steps per tile
constexpr int kWaves = 8;
constexpr int kThreads = 64 * kWaves;
constexpr int kMT = 2;                   // 32-query tiles per wave
constexpr int kQPerWave = 32 * kMT;
constexpr int kQPerBlock = kWaves * kQPerWave;
constexpr int kStageTok = 128;           // tokens per LDS stage
constexpr int kStageLd = kDc + 8;        // LDS row stride in elements (272 B: conflict-free 16-byte reads)
constexpr int kStageElems = kStageTok * kStageLd;
constexpr int kMaxTilesPerBlock = 32;    // 1024 tokens: bounds the LDS column-maximum buffer

__host__ __device__ inline int64_t mfma_tiles_per_block(int64_t n) {
  const int64_t n_tiles = (n + 31) / 32;
  int64_t per = (n_tiles + 255) / 256;   // about one workgroup per compute unit
  per = (per + 3) / 4 * 4;               // whole stages
  return per < 4 ? 4 : (per > kMaxTilesPerBlock ? kMaxTilesPerBlock : per);
}
__host__ __device__ inline int64_t mfma_blocks(int64_t n) {
  const int64_t per = mfma_tiles_per_block(n);
  return ((n + 31) / 32 + per - 1) / per;
}

// PASS 0: partial row maxima into part_max[block][l_c].  PASS 1: F into score, using mu[l_c].
template <int PASS>
__global__ __launch_bounds__(kThreads) void score_mfma_bf16(const bf16_t* __restrict__ qc, int l_c,
                                                            const bf16_t* __restrict__ kc, int64_t m_lo, int64_t n,
                                                            float* __restrict__ part_max,
                                                            const float* __restrict__ mu_all,
                                                            float* __restrict__ score, int64_t q_bs, int64_t kc_bs,
                                                            int64_t score_bs, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  bf16_t* stage = (bf16_t*)lds_raw;                                   // [2][kStageTok][kStageLd]
  float* fpart = (float*)(lds_raw + 2 * kStageElems * sizeof(bf16_t)); // PASS 1: [kWaves][span] column maxima
  const int b = blockIdx.y;
  const bf16_t* q = qc + (int64_t)b * q_bs;
  const bf16_t* kmid = kc + (int64_t)b * kc_bs + m_lo * (int64_t)kDc;
  const float* mu = mu_all + (int64_t)b * l_c;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, hi = lane >> 5;
  const int64_t n_tiles = (n + 31) / 32;
  const int64_t tile0 = (int64_t)blockIdx.x * tiles_per_block;
  const int64_t tile1 = (tile0 + tiles_per_block) < n_tiles ? (tile0 + tiles_per_block) : n_tiles;
  const int span = tiles_per_block * 32;
  const int n_stages = (int)((tile1 - tile0 + 3) / 4);
  const int64_t tok_base = tile0 * 32;

  // One stage in flight between global memory and LDS: four 16-byte pieces per thread, kept in
  // named registers.
  uint4 s0, s1, s2, s3;
  auto piece_src = [&](int s, int i) -> const uint4* {
    const int id = tid + kThreads * i;
    int64_t tok = tok_base + (int64_t)s * kStageTok + (id >> 4);
    tok = tok < n ? tok : n - 1;           // a repeated token changes no maximum and is never stored
    return (const uint4*)(kmid + tok * kDc + (id & 15) * 8);
  };
  auto piece_dst = [&](int s, int i) -> uint4* {
    const int id = tid + kThreads * i;
    return (uint4*)&stage[(s & 1) * kStageElems + (id >> 4) * kStageLd + (id & 15) * 8];
  };
#define ESA_STAGE_LOAD(s)                                                                       \
  do {                                                                                          \
    s0 = *piece_src(s, 0); s1 = *piece_src(s, 1); s2 = *piece_src(s, 2); s3 = *piece_src(s, 3); \
  } while (0)
#define ESA_STAGE_STORE(s)                                                                      \
  do {                                                                                          \
    *piece_dst(s, 0) = s0; *piece_dst(s, 1) = s1; *piece_dst(s, 2) = s2; *piece_dst(s, 3) = s3; \
  } while (0)

  for (int qb = 0; qb * kQPerBlock < l_c; ++qb) {
    const int q0 = qb * kQPerBlock + wave * kQPerWave;
    int n_mt = (l_c - q0 + 31) / 32;     // 32-query tiles of this wave that hold at least one query
    n_mt = n_mt < 0 ? 0 : (n_mt > kMT ? kMT : n_mt);

    bf16x8 a[kMT][kKSteps];
    float aux[kMT][16];                  // PASS 0: running row maxima.  PASS 1: mu of the lane's rows.
#pragma unroll
    for (int mt = 0; mt < kMT; ++mt) {
      const int row = q0 + 32 * mt + r;
      const bool ok = row < l_c;
      const bf16_t* p = q + (int64_t)(ok ? row : 0) * kDc + hi * 8;
#pragma unroll
      for (int ks = 0; ks < kKSteps; ++ks) {
        bf16x8 v = *(const bf16x8*)(p + ks * 16);
        if (!ok) v = (bf16x8){0, 0, 0, 0, 0, 0, 0, 0};
        a[mt][ks] = v;
      }
      // Pin the fragments as arrived values: otherwise every use inside the stage loop carries a wait on
      // the vector-memory counter, which would also wait for the stage loads just issued.
#pragma unroll
      for (int ks = 0; ks < kKSteps; ++ks) asm volatile("" : "+v"(a[mt][ks]));
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        if (PASS == 0) {
          aux[mt][v] = -INFINITY;
        } else {
          const int qrow = q0 + 32 * mt + 8 * (v / 4) + 4 * hi + (v % 4);
          aux[mt][v] = (qrow < l_c) ? mu[qrow] : INFINITY;
        }
      }
      if (PASS == 1) {
#pragma unroll
        for (int v = 0; v < 16; ++v) asm volatile("" : "+v"(aux[mt][v]));
      }
    }

    __syncthreads();                     // the previous query block is done with both stage buffers
    if (n_stages > 0) {
      ESA_STAGE_LOAD(0);
      ESA_STAGE_STORE(0);
    }
    for (int s = 0; s < n_stages; ++s) {
      __syncthreads();
      if (s + 1 < n_stages) ESA_STAGE_LOAD(s + 1);
      const bf16_t* buf = stage + (s & 1) * kStageElems;
      int nt_lim = (int)(tile1 - tile0) - 4 * s;
      nt_lim = nt_lim > 4 ? 4 : nt_lim;
      if (n_mt > 0) {
        for (int nt = 0; nt < nt_lim; ++nt) {
          bf16x8 bfr[kKSteps];
#pragma unroll
          for (int ks = 0; ks < kKSteps; ++ks)
            bfr[ks] = *(const bf16x8*)&buf[(32 * nt + r) * kStageLd + 16 * ks + 8 * hi];
          f32x16 acc[kMT];
#pragma unroll
          for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mt][v] = 0.f;
#pragma unroll
          for (int ks = 0; ks < kKSteps; ++ks)
#pragma unroll
            for (int mt = 0; mt < kMT; ++mt)
              acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mt][ks], bfr[ks], acc[mt], 0, 0, 0);
          if (PASS == 0) {
#pragma unroll
            for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
              for (int v = 0; v < 16; ++v) aux[mt][v] = fmaxf(aux[mt][v], acc[mt][v]);
          } else {
            float best = -INFINITY;
#pragma unroll
            for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
              for (int v = 0; v < 16; ++v) best = fmaxf(best, acc[mt][v] - aux[mt][v]);
            best = fmaxf(best, __shfl_xor(best, 32, 64));
            if (hi == 0) {
              float* slot = &fpart[wave * span + (4 * s + nt) * 32 + r];
              *slot = (qb == 0) ? best : fmaxf(*slot, best);
            }
          }
        }
      } else if (PASS == 1 && qb == 0) {
        // a wave without queries still owns a column-maximum row: neutral element
        for (int nt = 0; nt < nt_lim; ++nt)
          if (hi == 0) fpart[wave * span + (4 * s + nt) * 32 + r] = -INFINITY;
      }
      if (s + 1 < n_stages) ESA_STAGE_STORE(s + 1);
    }

    if (PASS == 0) {
#pragma unroll
      for (int mt = 0; mt < kMT; ++mt)
        if (mt < n_mt) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            float m = aux[mt][v];
#pragma unroll
            for (int off = 16; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
            const int qrow = q0 + 32 * mt + 8 * (v / 4) + 4 * hi + (v % 4);
            if (r == 0 && qrow < l_c)
              part_max[((int64_t)b * gridDim.x + blockIdx.x) * l_c + qrow] = m;
          }
        }
    }
  }

  if (PASS == 1) {
    __syncthreads();
    for (int i = tid; i < span; i += kThreads) {
      const int64_t m = tile0 * 32 + i;
      if (m < n && m < tile1 * 32) {
        float f = fpart[i];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) f = fmaxf(f, fpart[w * span + i]);
        score[(int64_t)b * score_bs + m] = f;
      }
    }
  }
}

#undef ESA_STAGE_LOAD
#undef ESA_STAGE_STORE

// mu[c] = max over workgroups of their partial row maxima.  16 queries per block, 16 slices of the
// workgroup list per query, combined through LDS.
__global__ __launch_bounds__(256) void score_rowmax_reduce(const float* __restrict__ part_max, int nblk, int l_c,
                                                           float* __restrict__ mu) {
  __shared__ float red[16][17];
  const int cl = threadIdx.x & 15, slice = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + cl;
  const int b = blockIdx.y;
  float m = -INFINITY;
  if (c < l_c)
    for (int i = slice; i < nblk; i += 16) m = fmaxf(m, part_max[((int64_t)b * nblk + i) * l_c + c]);
  red[slice][cl] = m;
  __syncthreads();
  if (threadIdx.x < 16 && c < l_c) {
    float t = red[0][cl];
#pragma unroll
    for (int i = 1; i < 16; ++i) t = fmaxf(t, red[i][cl]);
    mu[(int64_t)b * l_c + c] = t;
  }
}

// ------------------------------------------------------------------------------------------ decode (l_c = 1)
// One current token: S is a matrix-vector product over the whole compressed-key cache, pure HBM
// streaming.  LPR lanes share a K' row (16 bytes each), so a wave reads 64*16 contiguous bytes per
// step.  Writes S and folds its maximum into mu; score_sub_mu then forms F = S - mu.
template <int LPR>
__global__ __launch_bounds__(256) void score_gemv_bf16(const bf16_t* __restrict__ qc, const bf16_t* __restrict__ kc,
                                                       int64_t m_lo, int64_t n, uint32_t* __restrict__ mu_keys,
                                                       float* __restrict__ raw, int64_t q_bs, int64_t kc_bs,
                                                       int64_t raw_bs) {
  constexpr int kDcv = LPR * 8;
  constexpr int kRowsPerStep = 256 / LPR;
  constexpr int kSteps = 16;
  __shared__ float red[4];
  const int b = blockIdx.y;
  const bf16_t* kmid = kc + (int64_t)b * kc_bs + m_lo * (int64_t)kDcv;
  const int sub = threadIdx.x % LPR, grp = threadIdx.x / LPR;
  float qv[8];
  {
    const uint4 u = *(const uint4*)(qc + (int64_t)b * q_bs + sub * 8);
    const bf16_t* pq = (const bf16_t*)&u;
#pragma unroll
    for (int i = 0; i < 8; ++i) qv[i] = bf16_to_f32(pq[i]);
  }
  float best = -INFINITY;
  const int64_t row0 = (int64_t)blockIdx.x * (kRowsPerStep * kSteps);
#pragma unroll 4
  for (int it = 0; it < kSteps; ++it) {
    const int64_t row = row0 + it * kRowsPerStep + grp;
    float s = 0.f;
    if (row < n) {
      const uint4 u = *(const uint4*)(kmid + row * kDcv + sub * 8);
      const bf16_t* pk = (const bf16_t*)&u;
#pragma unroll
      for (int i = 0; i < 8; ++i) s = __fmaf_rn(qv[i], bf16_to_f32(pk[i]), s);
    }
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (row < n) {
      if (sub == 0) raw[(int64_t)b * raw_bs + row] = s;
      best = fmaxf(best, s);
    }
  }
  best = wave_max(best);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = best;
  __syncthreads();
  if (threadIdx.x == 0)
    atomicMax(&mu_keys[b], ordered_key(fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]))));
}

__global__ void score_sub_mu(float* __restrict__ raw, int64_t n, const uint32_t* __restrict__ mu_keys, int64_t raw_bs) {
  const float mu = ordered_key_to_f32(mu_keys[blockIdx.y]);
  float* p = raw + (int64_t)blockIdx.y * raw_bs;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    p[i] = p[i] - mu;
}

// Eq. 8: out[j] = max(in[max(j-eps,0) .. min(j+eps,n-1)]).
__global__ void proximity_maxpool(const float* __restrict__ in, float* __restrict__ out, int64_t n, int eps,
                                  int64_t in_bs, int64_t out_bs) {
  const float* src = in + (int64_t)blockIdx.y * in_bs;
  float* dst = out + (int64_t)blockIdx.y * out_bs;
  for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < n; j += (int64_t)gridDim.x * blockDim.x) {
    const int64_t lo = j - eps > 0 ? j - eps : 0, hi = j + eps < n - 1 ? j + eps : n - 1;
    float m = src[lo];
    for (int64_t w = lo + 1; w <= hi; ++w) m = fmaxf(m, src[w]);
    dst[j] = m;
  }
}

}  // namespace

__host__ inline size_t part_bytes(int l_c, int64_t n_mid, int batch) {
  return align_up((size_t)mfma_blocks(n_mid) * l_c * batch * 4, 256);
}

size_t score_workspace_bytes(int l_c, int64_t n_mid, int eps, int batch) {
  if (l_c <= 0 || batch <= 0 || n_mid < 0) return 256;
  size_t b = mu_bytes(l_c, batch) + part_bytes(l_c, n_mid, batch);
  if (eps > 0) b += align_up((size_t)n_mid * 4, 256) * (size_t)batch;
  return b;
}

int launch_score(const void* qc, int l_c, const void* kc_cache, int64_t m_lo, int64_t m_hi, int d_c, int eps,
                 float* score, int dtype, int batch, int64_t q_bs, int64_t kc_bs, int64_t score_bs, void* ws,
                 size_t ws_bytes, hipStream_t st) {
  const int64_t n = m_hi - m_lo;
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
    fill_u32<<<(batch + 255) / 256, 256, 0, st>>>(mu, (int64_t)batch, kOrderedKeyOfMinusInf);
    const int lpr = d_c / 8;
    const int rows_per_block = (256 / lpr) * 16;
    const dim3 grid((unsigned)((n + rows_per_block - 1) / rows_per_block), batch);
    const bf16_t* q = (const bf16_t*)qc;
    const bf16_t* k = (const bf16_t*)kc_cache;
    if (lpr == 8) score_gemv_bf16<8><<<grid, 256, 0, st>>>(q, k, m_lo, n, mu, raw, q_bs, kc_bs, raw_bs);
    else if (lpr == 16) score_gemv_bf16<16><<<grid, 256, 0, st>>>(q, k, m_lo, n, mu, raw, q_bs, kc_bs, raw_bs);
    else score_gemv_bf16<32><<<grid, 256, 0, st>>>(q, k, m_lo, n, mu, raw, q_bs, kc_bs, raw_bs);
    const int blocks = (int)((n + 1023) / 1024 < 2048 ? (n + 1023) / 1024 : 2048);
    score_sub_mu<<<dim3(blocks, batch), 256, 0, st>>>(raw, n, mu, raw_bs);
  } else if (vec_ok && d_c == kDc) {
    const int per = (int)mfma_tiles_per_block(n);
    const int nblk = (int)mfma_blocks(n);
    const dim3 grid(nblk, batch);
    float* part = (float*)((char*)ws + mu_bytes(l_c, batch));
    float* muf = (float*)ws;
    const size_t lds0 = (size_t)2 * kStageElems * sizeof(bf16_t);
    const size_t lds1 = lds0 + (size_t)kWaves * per * 32 * sizeof(float);
    static bool lds_limit_raised = false;      // idempotent; a race only repeats the call
    if (!lds_limit_raised) {
      hipError_t e = hipFuncSetAttribute((const void*)score_mfma_bf16<0>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)lds0);
      if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)score_mfma_bf16<1>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)(lds0 + (size_t)kWaves * kMaxTilesPerBlock * 32 * sizeof(float)));
      if (e != hipSuccess) return hip_failed(e, "hipFuncSetAttribute(score_mfma_bf16)");
      lds_limit_raised = true;
    }
    score_mfma_bf16<0><<<grid, kThreads, lds0, st>>>((const bf16_t*)qc, l_c, (const bf16_t*)kc_cache, m_lo, n, part, muf,
                                                raw, q_bs, kc_bs, raw_bs, per);
    score_rowmax_reduce<<<dim3((l_c + 15) / 16, batch), 256, 0, st>>>(part, nblk, l_c, muf);
    score_mfma_bf16<1><<<grid, kThreads, lds1, st>>>((const bf16_t*)qc, l_c, (const bf16_t*)kc_cache, m_lo, n, part, muf,
                                                raw, q_bs, kc_bs, raw_bs, per);
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
    const int blocks = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
    proximity_maxpool<<<dim3(blocks, batch), 256, 0, st>>>(raw, score, n, eps, raw_bs, score_bs);
  }
  ESA_LAUNCH_CHECK("score");
  return ESA_OK;
}

}  // namespace esa
