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

// Workspace: [batch][l_c] uint32 row-maximum keys, then (eps > 0) [batch][n] fp32 unpooled scores.
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

size_t score_workspace_bytes(int l_c, int64_t n_mid, int eps, int batch) {
  if (l_c <= 0 || batch <= 0 || n_mid < 0) return 256;
  size_t b = mu_bytes(l_c, batch);
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
    raw = (float*)((char*)ws + mu_bytes(l_c, batch));
    raw_bs = (int64_t)(align_up((size_t)n * 4, 256) / 4);
  }
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
  if (eps > 0) {
    const int blocks = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
    proximity_maxpool<<<dim3(blocks, batch), 256, 0, st>>>(raw, score, n, eps, raw_bs, score_bs);
  }
  ESA_LAUNCH_CHECK("score");
  return ESA_OK;
}

}  // namespace esa
