// Selected attention (Eq. 1): softmax attention of the current tokens over the virtual key
// sequence  [ I | M_k | L | C ]  =  cache rows [0,i_end) ++ gathered rows [0,n_sel) ++ cache rows
// [l_start, t0+l_c).  Current token c sees virtual keys [0, n_fixed + c], n_fixed = i_end + n_sel +
// (t0 - l_start): everything before the chunk plus the chunk up to itself (Algorithm 1).
#include "esa_common.h"
#include "attend_mfma.h"
#include "attend_decode.h"
#include "keyspace.h"

namespace esa {
namespace {

__device__ __forceinline__ float block_max(float v, float* red) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

// One workgroup per (current token, query head, batch element); fp32 arithmetic with full-precision
// expf/logf.  Serves fp32 storage and every shape the matrix-core kernel does not cover.
template <typename T>
__global__ __launch_bounds__(256) void attend_fma(const T* __restrict__ q, int l_c, int h, int h_kv, int d, KeySpace ks,
                                                  int64_t n_fixed, int with_chunk, float scale, T* __restrict__ out,
                                                  float* __restrict__ out32, float* __restrict__ lse, int64_t q_bs,
                                                  int64_t cache_bs_bytes, int64_t sel_bs_bytes, int64_t idx_bs,
                                                  int64_t out_bs) {
  __shared__ float qs[256];
  __shared__ float p[256];
  __shared__ float red[4];
  __shared__ float accs[256];
  const int c = blockIdx.x, hh = blockIdx.y, b = blockIdx.z;
  const int g = hh / (h / h_kv);
  ks.k_cache += (int64_t)b * cache_bs_bytes;
  ks.v_cache += (int64_t)b * cache_bs_bytes;
  if (ks.sel_idx) {
    ks.sel_idx += (int64_t)b * idx_bs;
  } else if (ks.n_sel > 0) {
    ks.k_sel += (int64_t)b * sel_bs_bytes;
    ks.v_sel += (int64_t)b * sel_bs_bytes;
  }
  const T* qrow = q + (int64_t)b * q_bs + ((int64_t)c * h + hh) * d;
  if ((int)threadIdx.x < d) qs[threadIdx.x] = load_f32(qrow + threadIdx.x);
  __syncthreads();
  const int64_t n_keys = n_fixed + (with_chunk ? c + 1 : 0);   // without the chunk every key is visible to every token
  const int nsub = 256 / d, dim = threadIdx.x % d, sub = threadIdx.x / d;
  float m_run = -INFINITY, l_run = 0.f, acc = 0.f;
  for (int64_t j0 = 0; j0 < n_keys; j0 += 256) {
    const int64_t j = j0 + threadIdx.x;
    float logit = -INFINITY;
    if (j < n_keys) {
      const T* kr = (const T*)key_row(ks, j, false) + (int64_t)g * d;
      float s = 0.f;
      for (int i = 0; i < d; ++i) s = __fmaf_rn(qs[i], load_f32(kr + i), s);
      logit = s * scale;
    }
    const float m_new = fmaxf(m_run, block_max(logit, red));
    const float pj = (j < n_keys) ? expf(logit - m_new) : 0.f;
    const float s_tile = block_sum(pj, red);
    const float corr = (m_run == -INFINITY) ? 0.f : expf(m_run - m_new);
    l_run = l_run * corr + s_tile;
    acc *= corr;
    p[threadIdx.x] = pj;
    __syncthreads();
    const int lim = (n_keys - j0) < 256 ? (int)(n_keys - j0) : 256;
    for (int jj = sub; jj < lim; jj += nsub) {
      const T* vr = (const T*)key_row(ks, j0 + jj, true) + (int64_t)g * d;
      acc = __fmaf_rn(p[jj], load_f32(vr + dim), acc);
    }
    m_run = m_new;
    __syncthreads();
  }
  accs[threadIdx.x] = acc;
  __syncthreads();
  if ((int)threadIdx.x < d) {
    float o = 0.f;
    for (int s = 0; s < nsub; ++s) o += accs[s * d + threadIdx.x];
    if (out32) out32[(((int64_t)b * l_c + c) * h + hh) * d + threadIdx.x] = o / l_run;   // one part of a two-call attention
    else store_f32(out + (int64_t)b * out_bs + ((int64_t)c * h + hh) * d + threadIdx.x, o / l_run);
  }
  if (lse && threadIdx.x == 0) lse[((int64_t)b * l_c + c) * h + hh] = m_run + logf(l_run);
}

// Algorithm 1's merge of two attentions over disjoint key sets (normalised outputs and natural-log
// normalisers): weights exp(lse_i - max).  A part without keys is passed as nullptr.
template <typename T>
__global__ void attend_merge_two(const float* __restrict__ o_a, const float* __restrict__ lse_a,
                                 const float* __restrict__ o_b, const float* __restrict__ lse_b, int64_t rows_per_batch,
                                 int d, T* __restrict__ out, int64_t out_bs, float* __restrict__ lse) {
  const int64_t row = blockIdx.x, b = blockIdx.y, r = b * rows_per_batch + row;
  const float la = lse_a[r], lb = lse_b ? lse_b[r] : -INFINITY;
  const float m = fmaxf(la, lb);
  const float wa = expf(la - m), wb = lse_b ? expf(lb - m) : 0.f;
  const float inv = 1.f / (wa + wb);
  for (int i = threadIdx.x; i < d; i += blockDim.x) {
    const float v = (wa * o_a[r * d + i] + (o_b ? wb * o_b[r * d + i] : 0.f)) * inv;
    store_f32(out + b * out_bs + row * d + i, v);
  }
  if (lse && threadIdx.x == 0) lse[r] = m + logf(wa + wb);
}

size_t generic_parts_bytes(int l_c, int h, int d, int batch) {
  const size_t rows = (size_t)batch * l_c * h;
  return 2 * (align_up(rows * d * sizeof(float), 256) + align_up(rows * sizeof(float), 256));
}

}  // namespace

size_t attend_indexed_workspace_bytes(int l_c, int h, int h_kv, int d, int dtype, int batch, int n_sel) {
  (void)n_sel;      // every kernel follows the indices itself: no room for gathered rows is needed
  return attend_workspace_bytes(l_c, h, h_kv, d, dtype, batch);
}

size_t attend_workspace_bytes(int l_c, int h, int h_kv, int d, int dtype, int batch) {
  if (l_c <= 0 || h <= 0 || h_kv <= 0 || d <= 0 || batch <= 0) return 256;
  if (attend_mfma_supported(l_c, h, h_kv, d, dtype)) return attend_mfma_workspace_bytes(l_c, h, h_kv, d, batch);
  // shapes outside the matrix-core kernel: room for the two parts of a two-call attention
  const size_t parts = generic_parts_bytes(l_c, h, d, batch);
  if (attend_decode_supported(l_c, h, h_kv, d, dtype)) {
    const size_t dec = attend_decode_workspace_bytes(l_c, h, batch);
    return dec > parts ? dec : parts;
  }
  return parts;
}

int launch_attend(int part, int split, const void* q, int l_c, int h, int h_kv, int d, const void* k_cache, const void* v_cache,
                  int64_t tok_stride, int64_t t0, int64_t l_i, int64_t l_l, const void* k_sel, const void* v_sel,
                  int n_sel, const int32_t* sel_idx, int64_t idx_bs, float scale, void* out, float* lse, int dtype,
                  int batch, int64_t q_bs, int64_t cache_bs, int64_t sel_bs, int64_t out_bs, void* ws, size_t ws_bytes,
                  hipStream_t st) {
  const Segments sg = segments(t0, l_i, l_l);
  if (n_sel == 0) sel_idx = nullptr;
  const int64_t n_fixed = sg.i_end + n_sel + (t0 - sg.l_start);
  const bool mfma_shape = attend_mfma_supported(l_c, h, h_kv, d, dtype);
  const bool mfma_aligned =
      attend_mfma_aligned(q, k_cache, v_cache, k_sel, v_sel, out, tok_stride, q_bs, cache_bs, sel_bs, out_bs);
  // The two calls of a separately encoded attention must take the same kernel: no fallback between them.
  if (mfma_shape && !mfma_aligned && part != kAttendAll && split == ESA_SPLIT_ALGORITHM1)
    ESA_FAIL(ESA_EINVAL, "esa_attend (two calls, Algorithm 1 grouping): pointers and strides must be 16-byte aligned");
  if (mfma_shape && mfma_aligned) {
    // an index list is followed by the kernel itself (index-driven tile loads): no gathered copy
    return launch_attend_mfma(part, split, q, l_c, h, h_kv, d, k_cache, v_cache, tok_stride, t0, sg.i_end, sg.l_start, k_sel,
                              v_sel, n_sel, sel_idx, idx_bs, scale, out, lse, batch, q_bs, cache_bs, sel_bs, out_bs, ws,
                              ws_bytes, st);
  }
  // Every other shape.  With the initial tokens in the early part the finishing (or the only) call
  // computes everything; Algorithm 1's grouping (separately encoded parts) runs the plain kernel once
  // per part and merges.
  const bool two_parts = part != kAttendAll && split == ESA_SPLIT_ALGORITHM1;
  if (part == kAttendLocal && !two_parts) return ESA_OK;
  if (two_parts && attend_decode_supported(l_c, h, h_kv, d, dtype) && (int64_t)batch * l_c <= 65535 &&
      attend_decode_covers_parts(t0 - sg.l_start + l_c, l_c, h_kv, batch)) {
    // decode-sized chunk in Algorithm 1's two parts: both calls must agree on this kernel, so nothing
    // that only one of them knows (the number of selected tokens, its pointers' alignment) may veto it
    if (!attend_mfma_aligned(q, k_cache, v_cache, k_sel, v_sel, out, tok_stride, q_bs, cache_bs, sel_bs, out_bs))
      ESA_FAIL(ESA_EINVAL, "esa_attend (two calls, Algorithm 1 grouping): pointers and strides must be 16-byte aligned");
    return launch_attend_decode(part == kAttendLocal ? 1 : 2, q, l_c, h, h_kv, k_cache, v_cache, tok_stride, t0, sg.i_end,
                                sg.l_start, k_sel, v_sel, n_sel, sel_idx, idx_bs, scale, out, lse, batch, q_bs, cache_bs,
                                sel_bs, out_bs, ws, ws_bytes, st);
  }
  if (!two_parts && attend_decode_supported(l_c, h, h_kv, d, dtype) && (int64_t)batch * l_c <= 65535 &&
      attend_decode_covers(n_fixed + l_c, l_c, h_kv, batch) &&
      attend_mfma_aligned(q, k_cache, v_cache, k_sel, v_sel, out, tok_stride, q_bs, cache_bs, sel_bs, out_bs)) {
    return launch_attend_decode(0, q, l_c, h, h_kv, k_cache, v_cache, tok_stride, t0, sg.i_end, sg.l_start, k_sel, v_sel,
                                n_sel, sel_idx, idx_bs, scale, out, lse, batch, q_bs, cache_bs, sel_bs, out_bs, ws, ws_bytes, st);
  }
  const int64_t esz = (dtype == ESA_F32) ? 4 : 2;
  KeySpace ks;
  ks.k_cache = (const char*)k_cache;
  ks.v_cache = (const char*)v_cache;
  ks.k_sel = (const char*)k_sel;
  ks.v_sel = (const char*)v_sel;
  ks.sel_idx = sel_idx;
  ks.tok_bytes = tok_stride * esz;
  ks.sel_bytes = (int64_t)h_kv * d * esz;
  ks.i_end = sg.i_end;
  ks.n_sel = n_sel;
  ks.l_start = sg.l_start;
  int64_t fixed = n_fixed;
  int with_chunk = 1;
  float* o32 = nullptr;
  float* lse_part = lse;
  const size_t rows = (size_t)batch * l_c * h;
  const size_t o_bytes = align_up(rows * d * sizeof(float), 256), l_bytes = align_up(rows * sizeof(float), 256);
  float* o_a = (float*)ws;
  float* lse_a = (float*)((char*)ws + o_bytes);
  float* o_b = (float*)((char*)ws + o_bytes + l_bytes);
  float* lse_b = (float*)((char*)ws + 2 * o_bytes + l_bytes);
  if (two_parts) {
    if (!ws || ws_bytes < generic_parts_bytes(l_c, h, d, batch)) ESA_FAIL(ESA_EWORKSPACE, "esa_attend: workspace too small");
    if (part == kAttendLocal) {          // [ L | C ]
      ks.i_end = 0;
      ks.n_sel = 0;
      fixed = t0 - sg.l_start;
      o32 = o_a;
      lse_part = lse_a;
    } else {                             // [ I | M_k ], every key visible
      fixed = sg.i_end + n_sel;
      with_chunk = 0;
      o32 = o_b;
      lse_part = lse_b;
    }
  }
  const dim3 grid(l_c, h, batch);
  if (!two_parts || part == kAttendLocal || fixed > 0) {
    if (dtype == ESA_BF16) {
      attend_fma<bf16_t><<<grid, 256, 0, st>>>((const bf16_t*)q, l_c, h, h_kv, d, ks, fixed, with_chunk, scale,
                                               (bf16_t*)out, o32, lse_part, q_bs, cache_bs * esz, sel_bs * esz, idx_bs, out_bs);
    } else {
      attend_fma<float><<<grid, 256, 0, st>>>((const float*)q, l_c, h, h_kv, d, ks, fixed, with_chunk, scale, (float*)out,
                                              o32, lse_part, q_bs, cache_bs * esz, sel_bs * esz, idx_bs, out_bs);
    }
  }
  if (two_parts && part == kAttendFinish) {
    const bool have_b = fixed > 0;
    const dim3 mgrid((unsigned)(l_c * h), batch);
    if (dtype == ESA_BF16)
      attend_merge_two<bf16_t><<<mgrid, 64, 0, st>>>(o_a, lse_a, have_b ? o_b : nullptr, have_b ? lse_b : nullptr,
                                                     (int64_t)l_c * h, d, (bf16_t*)out, out_bs, lse);
    else
      attend_merge_two<float><<<mgrid, 64, 0, st>>>(o_a, lse_a, have_b ? o_b : nullptr, have_b ? lse_b : nullptr,
                                                    (int64_t)l_c * h, d, (float*)out, out_bs, lse);
  }
  ESA_LAUNCH_CHECK("attend_fma");
  return ESA_OK;
}

size_t attend_reencoded_workspace_bytes(int l_c, int h, int h_kv, int d, int dtype, int batch, int64_t l_l) {
  if (l_c <= 0 || h <= 0 || h_kv <= 0 || d <= 0 || batch <= 0 || l_l < 0) return 256;
  const size_t esz = (dtype == ESA_F32) ? 4 : 2;
  const size_t q_bytes = align_up((size_t)batch * l_c * h * d * esz, 256);
  const size_t kv_bytes = align_up((size_t)batch * (size_t)(l_l + l_c) * h_kv * d * esz, 256);
  return align_up(attend_workspace_bytes(l_c, h, h_kv, d, dtype, batch), 256) + 2 * q_bytes + 2 * kv_bytes;
}

// Section 3.2 on un-encoded queries and keys.  The workspace holds, behind the attention workspace
// proper, the chunk's queries in their two encodings and a dense re-encoded copy of the local rows
// [l_start, t0 + l_c) of the key cache with the matching value rows; the local part then runs on
// that copy as a sequence of its own (no initial tokens, window = all of it), the global part on
// the caller's un-encoded caches (position 0 is the identity), merged by Algorithm 1's rule.
int launch_attend_reencoded(const void* q, int l_c, int h, int h_kv, int d, const void* k_cache, const void* v_cache,
                            int64_t tok_stride, int64_t t0, int64_t l_i, int64_t l_l, const void* k_sel,
                            const void* v_sel, int n_sel, float scale, double w, double base, void* out, float* lse,
                            int dtype, int batch, int64_t q_bs, int64_t cache_bs, int64_t sel_bs, int64_t out_bs,
                            void* ws, size_t ws_bytes, hipStream_t st) {
  const Segments sg = segments(t0, l_i, l_l);
  const int64_t n_loc = t0 - sg.l_start, rows = n_loc + l_c;
  const size_t esz = (dtype == ESA_F32) ? 4 : 2;
  const size_t own = align_up(attend_workspace_bytes(l_c, h, h_kv, d, dtype, batch), 256);
  const size_t q_bytes = align_up((size_t)batch * l_c * h * d * esz, 256);
  const size_t kv_bytes = align_up((size_t)batch * (size_t)rows * h_kv * d * esz, 256);
  if (!ws || ws_bytes < own + 2 * q_bytes + 2 * kv_bytes)
    ESA_FAIL(ESA_EWORKSPACE, "esa_attend_reencoded: workspace needs %zu bytes", own + 2 * q_bytes + 2 * kv_bytes);
  char* q_loc = (char*)ws + own;
  char* q_glob = q_loc + q_bytes;
  char* k_loc = q_glob + q_bytes;
  char* v_loc = k_loc + kv_bytes;
  const int64_t q_row = (int64_t)h * d, kv_row = (int64_t)h_kv * d;
  const int64_t qw_bs = (int64_t)l_c * q_row, kvw_bs = rows * kv_row;
  if (attend_mfma_supported(l_c, h, h_kv, d, dtype) &&
      !attend_mfma_aligned(q_loc, k_cache, v_cache, k_sel, v_sel, out, tok_stride, qw_bs, cache_bs, sel_bs, out_bs))
    ESA_FAIL(ESA_EINVAL, "esa_attend_reencoded: pointers and strides must be 16-byte aligned for this shape");
  // decode-sized chunks on the split-key kernel: the global part must fit its half of the slices too
  // (checked here so that nothing is enqueued when it does not)
  if (attend_decode_supported(l_c, h, h_kv, d, dtype) && (int64_t)batch * l_c <= 65535 &&
      attend_decode_covers_parts(n_loc + l_c, l_c, h_kv, batch) && sg.i_end + n_sel > 0 &&
      !attend_decode_covers_parts(sg.i_end + n_sel, l_c, h_kv, batch))
    ESA_FAIL(ESA_EUNSUPPORTED, "esa_attend_reencoded: %lld initial and selected keys exceed the decode kernel's range",
             (long long)(sg.i_end + n_sel));

  RopeJob jobs[4];
  jobs[0] = RopeJob{q, q_loc, l_c, q_row, q_row, q_bs, qw_bs, (double)n_loc, 1.0, h, 1};     // local queries, in order
  jobs[1] = RopeJob{q, q_glob, l_c, q_row, q_row, q_bs, qw_bs, w, 0.0, h, 1};                // global queries, all at w
  const char* k_rows = (const char*)k_cache + (size_t)sg.l_start * tok_stride * esz;
  const char* v_rows = (const char*)v_cache + (size_t)sg.l_start * tok_stride * esz;
  jobs[2] = RopeJob{k_rows, k_loc, rows, tok_stride, kv_row, cache_bs, kvw_bs, 0.0, 1.0, h_kv, 1};   // local keys from 0
  jobs[3] = RopeJob{v_rows, v_loc, rows, tok_stride, kv_row, cache_bs, kvw_bs, 0.0, 0.0, h_kv, 0};   // their values
  int rc = launch_rope_jobs(jobs, 4, d, base, dtype, batch, st);
  if (rc != ESA_OK) return rc;
  if (attend_mfma_supported(l_c, h, h_kv, d, dtype))     // both parts in one launch of the matrix-core kernel
    return launch_attend_mfma_two_views(q_loc, q_glob, qw_bs, l_c, h, h_kv, d, k_loc, v_loc, n_loc, kvw_bs, k_cache, v_cache,
                                        tok_stride, cache_bs, sg.i_end, k_sel, v_sel, n_sel, sel_bs, scale, out, lse, batch,
                                        out_bs, ws, own, st);
  rc = launch_attend(kAttendLocal, ESA_SPLIT_ALGORITHM1, q_loc, l_c, h, h_kv, d, k_loc, v_loc, kv_row, n_loc, 0, n_loc,
                     nullptr, nullptr, 0, nullptr, 0, scale, nullptr, nullptr, dtype, batch, qw_bs, kvw_bs, 0, 0, ws, own, st);
  if (rc != ESA_OK) return rc;
  return launch_attend(kAttendFinish, ESA_SPLIT_ALGORITHM1, q_glob, l_c, h, h_kv, d, k_cache, v_cache, tok_stride, t0, l_i,
                       l_l, k_sel, v_sel, n_sel, nullptr, 0, scale, out, lse, dtype, batch, qw_bs, cache_bs, sel_bs, out_bs,
                       ws, own, st);
}

}  // namespace esa
