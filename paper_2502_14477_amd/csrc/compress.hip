// Query/key compression (Eq. 5): out[n, :] = x[n, :] . W (+ bias), one linear layer on the
// head-concatenated vector, fp32 accumulation, result rounded to the storage type.
//
// Kernels:
//   * compress_mfma_packed_bf16 — bf16 storage, weights in the packed (output-major) layout written by
//     esa_pack_weights.  Both MFMA operands then have their reduction elements contiguous in memory
//     and are loaded straight from global memory, 16 bytes per lane, with no LDS staging.  A
//     workgroup owns a 16-token x 16-output tile; its four (many tokens) or sixteen (few tokens:
//     latency-bound) waves each reduce an equal share of d_in and the partial tiles are added in a
//     fixed order (deterministic, no atomics).
//   * compress_few_packed_bf16 — the same inputs for one to four tokens (a decode step): one workgroup per
//     output, a dot product per token.
//   * compress_mfma_bf16 — bf16 storage, weights as given ([d_in, d_c]); W is transposed through LDS.
//   * compress_fma — any storage type, shape and weight layout, plain fp32 FMAs in ascending
//     reduction order.
//   * pack_weights — the one-time transposition [d_in, d_c] -> [d_c, d_in].
#include "esa_common.h"

namespace esa {
namespace {

// ------------------------------------------------------------------------------------------ generic
constexpr int kTok = 16;       // tokens per block
constexpr int kChunk = 64;     // reduction elements staged per step
constexpr int kMaxColsPerLane = 4;

template <typename T, bool PACKED>
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
        wv[c] = (j < d_c) ? load_f32(PACKED ? W + (int64_t)j * d_in + (i0 + ii) : W + (i0 + ii) * (int64_t)d_c + j) : 0.f;
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


// ------------------------------------------------------------------------------------------ MFMA, packed weights
// v_mfma_f32_16x16x32_bf16: lane l supplies A[l%16][8*(l/16) .. +7] and B[8*(l/16) .. +7][l%16] and owns
// C[4*(l/16) .. +3][l%16].  A rows are tokens, B columns are outputs, so a lane reads eight consecutive
// reduction elements of one token row of x and of one output row of the packed weights.
// One launch serves up to two inputs ("jobs") that share the token count, d_c and the batch: the chunk's
// queries and keys are compressed side by side (Eq. 5 has both).  The job is the slow index of the grid
// (blockIdx.y = job * col_tiles + column tile), so that all workgroups of job 0 are dispatched before
// those of job 1 and a compute unit gets one of each rather than two of the long ones.
struct CompressJob {
  const bf16_t* x;
  const bf16_t* Wt;
  const bf16_t* bias;
  bf16_t* out;
  int64_t d_in, ldx, ldo, x_bs, out_bs;
};

template <int NW>
__global__ __launch_bounds__(64 * NW) void compress_mfma_packed_bf16(CompressJob j0, CompressJob j1, int64_t n_tok,
                                                                 int col_tiles) {
  __shared__ float red[NW][256];
  const bool second = (int)blockIdx.y >= col_tiles;
  // field-wise select: every kernel argument is fetched in the first round trip
  const bf16_t* x = second ? j1.x : j0.x;
  const bf16_t* Wt = second ? j1.Wt : j0.Wt;
  const bf16_t* bias = second ? j1.bias : j0.bias;
  bf16_t* out = second ? j1.out : j0.out;
  const int64_t d_in = second ? j1.d_in : j0.d_in, ldx = second ? j1.ldx : j0.ldx, ldo = second ? j1.ldo : j0.ldo;
  const int64_t x_bs = second ? j1.x_bs : j0.x_bs, out_bs = second ? j1.out_bs : j0.out_bs;
  const bf16_t* xb = x + (int64_t)blockIdx.z * x_bs;
  bf16_t* ob = out + (int64_t)blockIdx.z * out_bs;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, q = lane >> 4;
  const int64_t tok0 = (int64_t)blockIdx.x * 16;
  const int col0 = ((int)blockIdx.y - (second ? col_tiles : 0)) * 16;
  int64_t tok = tok0 + r;
  tok = tok < n_tok ? tok : n_tok - 1;               // keep the address valid; the row is discarded
  const int64_t kq = d_in / NW;                      // this wave's share of the reduction (multiple of 32)
  const bf16_t* xp = xb + tok * ldx + wave * kq + q * 8;
  const bf16_t* wp = Wt + (int64_t)(col0 + r) * d_in + wave * kq + q * 8;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  // One pair of loads in flight per wave is enough here: sixteen waves per workgroup and two workgroups
  // per compute unit hide the latency.  Putting eight steps' loads in flight at once changed nothing
  // (11.8 us for the chunk's queries and keys either way), and was slower when the short job had to issue
  // surplus loads to fit the same unrolled loop (17.5 us).
  for (int64_t ks = 0; ks < kq; ks += 32) {
    const bf16x8 a = *(const bf16x8*)(xp + ks);
    const bf16x8 b = *(const bf16x8*)(wp + ks);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0);
  }
#pragma unroll
  for (int v = 0; v < 4; ++v) red[wave][(4 * q + v) * 16 + r] = acc[v];
  __syncthreads();
  const int t = threadIdx.x;
  if (t >= 256) return;
  const int64_t row = tok0 + (t >> 4);
  const int col = col0 + (t & 15);
  if (row < n_tok) {
    float v = red[0][t];
#pragma unroll
    for (int w = 1; w < NW; ++w) v += red[w][t];     // fixed order: deterministic
    if (bias) v += bf16_to_f32(bias[col]);
    ob[row * ldo + col] = f32_to_bf16(v);
  }
}

// Up to four tokens (a decode step): the matrix-core kernel above would occupy d_c / 16 workgroups per input and
// leave the chip idle while sixteen compute units pull the weights through; here every output is a workgroup of
// its own (d_c per input, two inputs per launch), which streams its weight row once, 16 bytes per lane and step,
// against the one to four token rows, and adds up in a fixed order (in-lane, wave butterfly, four waves through
// LDS): deterministic, no atomics.  blockIdx.x = output, blockIdx.y = input (job), blockIdx.z = batch entry.
constexpr int kFewTok = 4;
constexpr int kFewBatch = 4;     // larger batches re-read the weights once per entry here: the matrix-core kernel wins
__global__ __launch_bounds__(256) void compress_few_packed_bf16(CompressJob j0, CompressJob j1, int n_tok) {
  __shared__ float red[4][kFewTok];
  const bool second = blockIdx.y != 0;
  const bf16_t* x = second ? j1.x : j0.x;
  const bf16_t* Wt = second ? j1.Wt : j0.Wt;
  const bf16_t* bias = second ? j1.bias : j0.bias;
  bf16_t* out = second ? j1.out : j0.out;
  const int64_t d_in = second ? j1.d_in : j0.d_in, ldx = second ? j1.ldx : j0.ldx, ldo = second ? j1.ldo : j0.ldo;
  const int64_t x_bs = second ? j1.x_bs : j0.x_bs, out_bs = second ? j1.out_bs : j0.out_bs;
  const bf16_t* xb = x + (int64_t)blockIdx.z * x_bs;
  const int col = blockIdx.x;
  const bf16_t* wrow = Wt + (int64_t)col * d_in;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float acc[kFewTok] = {0.f, 0.f, 0.f, 0.f};
  // Two steps of the reduction per trip, every load of the trip requested before the first is used and none of
  // them behind a branch (a step past the end re-reads the trip's first, a token past the last re-reads token 0;
  // neither is added): the kernel is a handful of round trips long, and loads that wait for each other are
  // most of them.
  constexpr int kAhead = 2;
  for (int64_t i0 = (int64_t)tid * 8; i0 < d_in; i0 += 256 * 8 * kAhead) {
    bf16x8 w[kAhead], v[kAhead][kFewTok];
#pragma unroll
    for (int a = 0; a < kAhead; ++a) {
      const int64_t i = i0 + a * 256 * 8, ic = i < d_in ? i : i0;
      w[a] = *(const bf16x8*)(wrow + ic);
#pragma unroll
      for (int t = 0; t < kFewTok; ++t) v[a][t] = *(const bf16x8*)(xb + (int64_t)(t < n_tok ? t : 0) * ldx + ic);
    }
#pragma unroll
    for (int a = 0; a < kAhead; ++a) {
      if (i0 + a * 256 * 8 < d_in) {
#pragma unroll
        for (int t = 0; t < kFewTok; ++t) {
          if (t < n_tok) {
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[t] = __fmaf_rn((float)v[a][t][e], (float)w[a][e], acc[t]);
          }
        }
      }
    }
  }
#pragma unroll
  for (int t = 0; t < kFewTok; ++t) {
    if (t >= n_tok) break;
    acc[t] = wave_sum(acc[t]);
    if (lane == 0) red[wave][t] = acc[t];
  }
  __syncthreads();
  if (tid < n_tok) {
    float v = ((red[0][tid] + red[1][tid]) + red[2][tid]) + red[3][tid];
    if (bias) v += bf16_to_f32(bias[col]);
    out[(int64_t)blockIdx.z * out_bs + (int64_t)tid * ldo + col] = f32_to_bf16(v);
  }
}

// W [d_in, d_c] -> Wt [d_c, d_in], through a padded LDS tile so both sides are coalesced.
template <typename T>
__global__ __launch_bounds__(256) void pack_weights(const T* __restrict__ W, int64_t d_in, int d_c, T* __restrict__ Wt) {
  __shared__ T tile[32][33];
  const int64_t i0 = (int64_t)blockIdx.x * 32;
  const int j0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
  for (int yy = ty; yy < 32; yy += 8)
    if (i0 + yy < d_in && j0 + tx < d_c) tile[yy][tx] = W[(i0 + yy) * d_c + j0 + tx];
  __syncthreads();
  for (int yy = ty; yy < 32; yy += 8)
    if (j0 + yy < d_c && i0 + tx < d_in) Wt[(int64_t)(j0 + yy) * d_in + i0 + tx] = tile[tx][yy];
}

}  // namespace

int launch_pack_weights(const void* W, int64_t d_in, int d_c, int dtype, void* Wt, hipStream_t st) {
  const dim3 grid((unsigned)((d_in + 31) / 32), (unsigned)((d_c + 31) / 32));
  if (dtype == ESA_BF16) pack_weights<bf16_t><<<grid, 256, 0, st>>>((const bf16_t*)W, d_in, d_c, (bf16_t*)Wt);
  else pack_weights<float><<<grid, 256, 0, st>>>((const float*)W, d_in, d_c, (float*)Wt);
  ESA_LAUNCH_CHECK("pack_weights");
  return ESA_OK;
}

int launch_compress(const void* x, int64_t n_tok, int64_t d_in, int64_t ldx, const void* W, int w_layout,
                    const void* bias, int d_c, void* out, int64_t ldo, int dtype, int batch, int64_t x_bs,
                    int64_t out_bs, hipStream_t st) {
  const int64_t nblk = (n_tok + kTok - 1) / kTok;
  const bool packed = (w_layout == ESA_W_PACKED);
  if (dtype == ESA_BF16) {
    const bool vec_ok = (ldx % 8 == 0) && (x_bs % 8 == 0) && (((uintptr_t)x | (uintptr_t)W) % 16 == 0);
    if (packed && vec_ok && d_c % 16 == 0 && d_in % 128 == 0) {
      // few tokens: the reduction is cut sixteen ways so that every lane's loads are all in flight at once
      const int tiles = (int)((n_tok + 15) / 16);
      const dim3 grid((unsigned)tiles, d_c / 16, batch);
      const CompressJob job{(const bf16_t*)x, (const bf16_t*)W, (const bf16_t*)bias, (bf16_t*)out, d_in, ldx, ldo, x_bs, out_bs};
      if (n_tok <= kFewTok && batch <= kFewBatch)
        compress_few_packed_bf16<<<dim3(d_c, 1, batch), 256, 0, st>>>(job, job, (int)n_tok);
      else if (d_in % 512 == 0 && n_tok <= 4096)
        compress_mfma_packed_bf16<16><<<grid, 1024, 0, st>>>(job, job, n_tok, d_c / 16);
      else
        compress_mfma_packed_bf16<4><<<grid, 256, 0, st>>>(job, job, n_tok, d_c / 16);
    } else if (!packed && vec_ok && (d_c % kMCols == 0) && (d_in % kMStep == 0)) {
      compress_mfma_bf16<<<dim3((unsigned)nblk, d_c / kMCols, batch), 256, 0, st>>>(
          (const bf16_t*)x, n_tok, d_in, ldx, (const bf16_t*)W, (const bf16_t*)bias, d_c, (bf16_t*)out, ldo, x_bs,
          out_bs);
    } else if (packed) {
      compress_fma<bf16_t, true><<<dim3((unsigned)nblk, batch), 256, 0, st>>>(
          (const bf16_t*)x, n_tok, d_in, ldx, (const bf16_t*)W, (const bf16_t*)bias, d_c, (bf16_t*)out, ldo, x_bs,
          out_bs);
    } else {
      compress_fma<bf16_t, false><<<dim3((unsigned)nblk, batch), 256, 0, st>>>(
          (const bf16_t*)x, n_tok, d_in, ldx, (const bf16_t*)W, (const bf16_t*)bias, d_c, (bf16_t*)out, ldo, x_bs,
          out_bs);
    }
  } else if (packed) {
    compress_fma<float, true><<<dim3((unsigned)nblk, batch), 256, 0, st>>>(
        (const float*)x, n_tok, d_in, ldx, (const float*)W, (const float*)bias, d_c, (float*)out, ldo, x_bs, out_bs);
  } else {
    compress_fma<float, false><<<dim3((unsigned)nblk, batch), 256, 0, st>>>(
        (const float*)x, n_tok, d_in, ldx, (const float*)W, (const float*)bias, d_c, (float*)out, ldo, x_bs, out_bs);
  }
  ESA_LAUNCH_CHECK("compress");
  return ESA_OK;
}

// Two inputs in one launch when both take the short-reduction matrix-core kernel; otherwise one launch each.
int launch_compress_pair(const void* x0, int64_t d_in0, int64_t ldx0, const void* W0, const void* bias0, void* out0,
                         int64_t ldo0, int64_t x0_bs, int64_t out0_bs, const void* x1, int64_t d_in1, int64_t ldx1,
                         const void* W1, const void* bias1, void* out1, int64_t ldo1, int64_t x1_bs, int64_t out1_bs,
                         int64_t n_tok, int d_c, int w_layout, int dtype, int batch, hipStream_t st) {
  auto fast = [&](const void* x, int64_t d_in, int64_t ldx, const void* W, int64_t x_bs) {
    return (ldx % 8 == 0) && (x_bs % 8 == 0) && (((uintptr_t)x | (uintptr_t)W) % 16 == 0) && d_in % 512 == 0;
  };
  if (dtype == ESA_BF16 && w_layout == ESA_W_PACKED && d_c % 16 == 0 && n_tok <= 4096 && n_tok > 0 &&
      fast(x0, d_in0, ldx0, W0, x0_bs) && fast(x1, d_in1, ldx1, W1, x1_bs)) {
    const int tiles = (int)((n_tok + 15) / 16);
    const CompressJob j0{(const bf16_t*)x0, (const bf16_t*)W0, (const bf16_t*)bias0, (bf16_t*)out0, d_in0, ldx0, ldo0, x0_bs, out0_bs};
    const CompressJob j1{(const bf16_t*)x1, (const bf16_t*)W1, (const bf16_t*)bias1, (bf16_t*)out1, d_in1, ldx1, ldo1, x1_bs, out1_bs};
    if (n_tok <= kFewTok && batch <= kFewBatch)
      compress_few_packed_bf16<<<dim3(d_c, 2, batch), 256, 0, st>>>(j0, j1, (int)n_tok);
    else
      compress_mfma_packed_bf16<16><<<dim3(tiles, 2 * (d_c / 16), batch), 1024, 0, st>>>(j0, j1, n_tok, d_c / 16);
    ESA_LAUNCH_CHECK("compress (pair)");
    return ESA_OK;
  }
  const int rc = launch_compress(x0, n_tok, d_in0, ldx0, W0, w_layout, bias0, d_c, out0, ldo0, dtype, batch, x0_bs, out0_bs, st);
  if (rc != ESA_OK) return rc;
  return launch_compress(x1, n_tok, d_in1, ldx1, W1, w_layout, bias1, d_c, out1, ldo1, dtype, batch, x1_bs, out1_bs, st);
}

}  // namespace esa
