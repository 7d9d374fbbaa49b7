// Query/key compression (Eq. 5): out[n, :] = x[n, :] . W (+ bias), one linear layer on the
// head-concatenated vector, fp32 accumulation, result rounded to the storage type.
//
// Two kernels:
//   * compress_mfma_bf16 — bf16 storage, matrix cores.  A workgroup owns 16 tokens x 64 outputs and
//     walks the whole reduction dimension, so every output is accumulated in one fixed order
//     (deterministic; no atomics, no split-K).
//   * compress_fma — any storage type and shape, plain fp32 FMAs in ascending reduction order.
#include "esa_common.h"

namespace esa {
namespace {

// ------------------------------------------------------------------------------------------ generic
constexpr int kTok = 16;       // tokens per block
constexpr int kChunk = 64;     // reduction elements staged per step
constexpr int kMaxColsPerLane = 4;

template <typename T>
__global__ __launch_bounds__(256) void compress_fma(const T* __restrict__ x, int64_t n_tok, int64_t d_in, int64_t ldx,
                                                    const T* __restrict__ W, const T* __restrict__ bias, int d_c,
                                                    T* __restrict__ out, int64_t ldo, int64_t x_bs, int64_t out_bs) {
  __shared__ float xs[kTok][kChunk + 1];
  const T* xb = x + (int64_t)blockIdx.y * x_bs;
  T* ob = out + (int64_t)blockIdx.y * out_bs;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t tok0 = (int64_t)blockIdx.x * kTok;
  float acc[4][kMaxColsPerLane];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int c = 0; c < kMaxColsPerLane; ++c) acc[t][c] = 0.f;

  for (int64_t i0 = 0; i0 < d_in; i0 += kChunk) {
    __syncthreads();
    for (int e = threadIdx.x; e < kTok * kChunk; e += 256) {
      const int t = e / kChunk, c = e % kChunk;
      const int64_t tok = tok0 + t, i = i0 + c;
      xs[t][c] = (tok < n_tok && i < d_in) ? load_f32(xb + tok * ldx + i) : 0.f;
    }
    __syncthreads();
    const int lim = (d_in - i0) < kChunk ? (int)(d_in - i0) : kChunk;
    for (int ii = 0; ii < lim; ++ii) {
      float wv[kMaxColsPerLane];
#pragma unroll
      for (int c = 0; c < kMaxColsPerLane; ++c) {
        const int j = lane + 64 * c;
        wv[c] = (j < d_c) ? load_f32(W + (i0 + ii) * (int64_t)d_c + j) : 0.f;
      }
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const float xv = xs[wave * 4 + t][ii];
#pragma unroll
        for (int c = 0; c < kMaxColsPerLane; ++c) acc[t][c] = __fmaf_rn(xv, wv[c], acc[t][c]);
      }
    }
  }
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int64_t tok = tok0 + wave * 4 + t;
    if (tok >= n_tok) continue;
#pragma unroll
    for (int c = 0; c < kMaxColsPerLane; ++c) {
      const int j = lane + 64 * c;
      if (j < d_c) {
        float v = acc[t][c];
        if (bias) v += load_f32(bias + j);
        store_f32(ob + tok * ldo + j, v);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------ MFMA
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// Tile: 16 tokens x 64 outputs per workgroup (4 waves, one 16x16 output tile each), the whole
// reduction dimension walked in steps of 128.  v_mfma_f32_16x16x32_bf16: lane l supplies
// A[l%16][8*(l/16) .. +7] and B[8*(l/16) .. +7][l%16], and owns C[4*(l/16) .. +3][l%16].
// x rows are read straight from global memory (16 bytes per lane); W is staged transposed in LDS
// so that a lane's eight reduction elements of one output column are contiguous.
constexpr int kMTok = 16;
constexpr int kMCols = 64;
constexpr int kMStep = 128;

__global__ __launch_bounds__(256) void compress_mfma_bf16(const bf16_t* __restrict__ x, int64_t n_tok, int64_t d_in,
                                                          int64_t ldx, const bf16_t* __restrict__ W,
                                                          const bf16_t* __restrict__ bias, int d_c,
                                                          bf16_t* __restrict__ out, int64_t ldo, int64_t x_bs,
                                                          int64_t out_bs) {
  // wt[col][k]: 64 columns x 128 reduction elements, row padded by 8 elements (16 bytes).
  __shared__ __attribute__((aligned(16))) bf16_t wt[kMCols][kMStep + 8];
  const bf16_t* xb = x + (int64_t)blockIdx.z * x_bs;
  bf16_t* ob = out + (int64_t)blockIdx.z * out_bs;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t tok0 = (int64_t)blockIdx.x * kMTok;
  const int col0 = blockIdx.y * kMCols;
  const int r = lane & 15, q = lane >> 4;
  int64_t tok = tok0 + r;
  const bool tok_ok = tok < n_tok;
  if (!tok_ok) tok = n_tok - 1;                      // keep the address valid; result discarded
  const bf16_t* xrow = xb + tok * ldx;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};

  for (int64_t i0 = 0; i0 < d_in; i0 += kMStep) {
    __syncthreads();
    // Stage W[i0 .. i0+128, col0 .. col0+64) transposed: thread handles 2 rows x 16 columns... simple 2-byte scatter.
    for (int e = threadIdx.x; e < kMStep * (kMCols / 8); e += 256) {
      const int kk = e / (kMCols / 8), c8 = (e % (kMCols / 8)) * 8;
      const uint4 v = *(const uint4*)(W + (i0 + kk) * (int64_t)d_c + col0 + c8);
      const bf16_t* pv = (const bf16_t*)&v;
#pragma unroll
      for (int j = 0; j < 8; ++j) wt[c8 + j][kk] = pv[j];
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < kMStep / 32; ++ks) {
      const bf16x8 a = *(const bf16x8*)(xrow + i0 + ks * 32 + q * 8);
      const bf16x8 b = *(const bf16x8*)(&wt[wave * 16 + r][ks * 32 + q * 8]);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0);
    }
  }
  // C[4q+v][r]: token tok0+4q+v, column col0 + wave*16 + r.
  const int col = col0 + wave * 16 + r;
  const float bv = bias ? bf16_to_f32(bias[col]) : 0.f;
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int64_t t = tok0 + q * 4 + v;
    if (t < n_tok) ob[t * ldo + col] = f32_to_bf16(acc[v] + bv);
  }
}

}  // namespace

int launch_compress(const void* x, int64_t n_tok, int64_t d_in, int64_t ldx, const void* W, const void* bias,
                    int d_c, void* out, int64_t ldo, int dtype, int batch, int64_t x_bs, int64_t out_bs,
                    hipStream_t st) {
  const int64_t nblk = (n_tok + kTok - 1) / kTok;
  if (dtype == ESA_BF16) {
    const bool mfma_ok = (d_c % kMCols == 0) && (d_in % kMStep == 0) && (ldx % 8 == 0) && (x_bs % 8 == 0) &&
                         (((uintptr_t)x | (uintptr_t)W) % 16 == 0);
    if (mfma_ok) {
      compress_mfma_bf16<<<dim3((unsigned)nblk, d_c / kMCols, batch), 256, 0, st>>>(
          (const bf16_t*)x, n_tok, d_in, ldx, (const bf16_t*)W, (const bf16_t*)bias, d_c, (bf16_t*)out, ldo, x_bs,
          out_bs);
    } else {
      compress_fma<bf16_t><<<dim3((unsigned)nblk, batch), 256, 0, st>>>((const bf16_t*)x, n_tok, d_in, ldx,
                                                                       (const bf16_t*)W, (const bf16_t*)bias, d_c,
                                                                       (bf16_t*)out, ldo, x_bs, out_bs);
    }
  } else {
    compress_fma<float><<<dim3((unsigned)nblk, batch), 256, 0, st>>>((const float*)x, n_tok, d_in, ldx,
                                                                    (const float*)W, (const float*)bias, d_c,
                                                                    (float*)out, ldo, x_bs, out_bs);
  }
  ESA_LAUNCH_CHECK("compress");
  return ESA_OK;
}

}  // namespace esa
