// The C ABI of libesa: argument validation and dispatch.  No kernel code here.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include "esa_common.h"
#include "attend_mfma.h"
#include "radix_hist.h"

namespace esa {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int hip_failed(hipError_t e, const char* what) {
  set_error("%s: %s", what, hipGetErrorString(e));
  return ESA_EHIP;
}

static bool dtype_ok(int dtype) { return dtype == ESA_F32 || dtype == ESA_BF16; }
static size_t elem_size(int dtype) { return dtype == ESA_F32 ? 4 : 2; }
static bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }
constexpr int kMaxBatch = 65535;

}  // namespace esa

using namespace esa;

extern "C" {

int esa_version(void) { return 100; }

const char* esa_last_error(void) { return g_err; }

int esa_segments(int64_t t0, int64_t l_i, int64_t l_l, int64_t* i_end, int64_t* l_start) {
  if (!i_end || !l_start) ESA_FAIL(ESA_EINVAL, "esa_segments: null output pointer");
  if (t0 < 0 || l_i < 0 || l_l < 0) ESA_FAIL(ESA_EINVAL, "esa_segments: negative argument");
  const Segments s = segments(t0, l_i, l_l);
  *i_end = s.i_end;
  *l_start = s.l_start;
  return ESA_OK;
}

int esa_pack_weights(const void* W, int64_t d_in, int d_c, int dtype, void* W_packed, void* stream) {
  if (!dtype_ok(dtype)) ESA_FAIL(ESA_EUNSUPPORTED, "esa_pack_weights: dtype %d", dtype);
  if (d_in <= 0 || d_c <= 0) ESA_FAIL(ESA_EINVAL, "esa_pack_weights: bad size (d_in=%lld d_c=%d)", (long long)d_in, d_c);
  if (!W || !W_packed || W == W_packed) ESA_FAIL(ESA_EINVAL, "esa_pack_weights: null or aliased pointer");
  if (!aligned(W, elem_size(dtype)) || !aligned(W_packed, elem_size(dtype)))
    ESA_FAIL(ESA_EINVAL, "esa_pack_weights: misaligned pointer");
  return launch_pack_weights(W, d_in, d_c, dtype, W_packed, (hipStream_t)stream);
}

int esa_compress(const void* x, int64_t n_tok, int64_t d_in, int64_t ldx, const void* W, int w_layout,
                 const void* bias, int d_c, void* out, int64_t ldo, int dtype, int batch, int64_t x_bs,
                 int64_t out_bs, void* stream) {
  if (!dtype_ok(dtype)) ESA_FAIL(ESA_EUNSUPPORTED, "esa_compress: dtype %d", dtype);
  if (w_layout != ESA_W_ROWMAJOR && w_layout != ESA_W_PACKED)
    ESA_FAIL(ESA_EINVAL, "esa_compress: weight layout %d", w_layout);
  if (n_tok < 0 || d_in <= 0 || d_c <= 0 || batch <= 0 || batch > kMaxBatch)
    ESA_FAIL(ESA_EINVAL, "esa_compress: bad size (n_tok=%lld d_in=%lld d_c=%d batch=%d)", (long long)n_tok,
             (long long)d_in, d_c, batch);
  if (d_c % 16 != 0 || d_c > 256) ESA_FAIL(ESA_EUNSUPPORTED, "esa_compress: d_c=%d (multiple of 16, <= 256)", d_c);
  if (ldx < d_in || ldo < d_c) ESA_FAIL(ESA_EINVAL, "esa_compress: row stride smaller than the row");
  if (n_tok >= (int64_t)1 << 31) ESA_FAIL(ESA_EINVAL, "esa_compress: n_tok too large");
  if (n_tok == 0) return ESA_OK;
  if (!x || !W || !out) ESA_FAIL(ESA_EINVAL, "esa_compress: null pointer");
  const size_t es = elem_size(dtype);
  if (!aligned(x, es) || !aligned(W, es) || !aligned(out, es) || !aligned(bias, es))
    ESA_FAIL(ESA_EINVAL, "esa_compress: misaligned pointer");
  return launch_compress(x, n_tok, d_in, ldx, W, w_layout, bias, d_c, out, ldo, dtype, batch, x_bs, out_bs,
                         (hipStream_t)stream);
}

int esa_compress_qk(const void* xq, int64_t d_in_q, int64_t ldxq, const void* Wq, const void* bias_q, void* out_q,
                    int64_t ldoq, int64_t xq_bs, int64_t outq_bs, const void* xk, int64_t d_in_k, int64_t ldxk,
                    const void* Wk, const void* bias_k, void* out_k, int64_t ldok, int64_t xk_bs, int64_t outk_bs,
                    int64_t n_tok, int d_c, int w_layout, int dtype, int batch, void* stream) {
  if (!dtype_ok(dtype)) ESA_FAIL(ESA_EUNSUPPORTED, "esa_compress_qk: dtype %d", dtype);
  if (w_layout != ESA_W_ROWMAJOR && w_layout != ESA_W_PACKED)
    ESA_FAIL(ESA_EINVAL, "esa_compress_qk: weight layout %d", w_layout);
  if (n_tok < 0 || d_in_q <= 0 || d_in_k <= 0 || d_c <= 0 || batch <= 0 || batch > kMaxBatch || n_tok >= (int64_t)1 << 31)
    ESA_FAIL(ESA_EINVAL, "esa_compress_qk: bad size (n_tok=%lld d_in=%lld/%lld d_c=%d batch=%d)", (long long)n_tok,
             (long long)d_in_q, (long long)d_in_k, d_c, batch);
  if (d_c % 16 != 0 || d_c > 256) ESA_FAIL(ESA_EUNSUPPORTED, "esa_compress_qk: d_c=%d (multiple of 16, <= 256)", d_c);
  if (ldxq < d_in_q || ldxk < d_in_k || ldoq < d_c || ldok < d_c)
    ESA_FAIL(ESA_EINVAL, "esa_compress_qk: row stride smaller than the row");
  if (n_tok == 0) return ESA_OK;
  if (!xq || !Wq || !out_q || !xk || !Wk || !out_k) ESA_FAIL(ESA_EINVAL, "esa_compress_qk: null pointer");
  const size_t es = elem_size(dtype);
  if (!aligned(xq, es) || !aligned(Wq, es) || !aligned(out_q, es) || !aligned(bias_q, es) || !aligned(xk, es) ||
      !aligned(Wk, es) || !aligned(out_k, es) || !aligned(bias_k, es))
    ESA_FAIL(ESA_EINVAL, "esa_compress_qk: misaligned pointer");
  return launch_compress_pair(xq, d_in_q, ldxq, Wq, bias_q, out_q, ldoq, xq_bs, outq_bs, xk, d_in_k, ldxk, Wk, bias_k, out_k,
                              ldok, xk_bs, outk_bs, n_tok, d_c, w_layout, dtype, batch, (hipStream_t)stream);
}

size_t esa_score_workspace_bytes(int l_c, int64_t n_mid, int eps, int batch) {
  return score_workspace_bytes(l_c, n_mid, eps, batch);
}

int esa_score(const void* qc, int l_c, const void* kc_cache, int64_t m_lo, int64_t m_hi, int d_c, int eps,
              float* score, int dtype, int batch, int64_t q_bs, int64_t kc_bs, int64_t score_bs, void* workspace,
              size_t ws_bytes, void* stream) {
  if (!dtype_ok(dtype)) ESA_FAIL(ESA_EUNSUPPORTED, "esa_score: dtype %d", dtype);
  if (l_c <= 0 || d_c <= 0 || batch <= 0 || batch > kMaxBatch || eps < 0 || m_lo < 0 || m_hi < m_lo)
    ESA_FAIL(ESA_EINVAL, "esa_score: bad size (l_c=%d d_c=%d batch=%d eps=%d m=[%lld,%lld))", l_c, d_c, batch, eps,
             (long long)m_lo, (long long)m_hi);
  if (d_c % 16 != 0 || d_c > 256) ESA_FAIL(ESA_EUNSUPPORTED, "esa_score: d_c=%d (multiple of 16, <= 256)", d_c);
  if (m_hi - m_lo >= (int64_t)1 << 31) ESA_FAIL(ESA_EINVAL, "esa_score: more than 2^31-1 middle tokens");
  if (m_hi == m_lo) return ESA_OK;
  if (!qc || !kc_cache || !score) ESA_FAIL(ESA_EINVAL, "esa_score: null pointer");
  const size_t es = elem_size(dtype);
  if (!aligned(qc, es) || !aligned(kc_cache, es) || !aligned(score, 4))
    ESA_FAIL(ESA_EINVAL, "esa_score: misaligned pointer");
  if (!workspace || !aligned(workspace, 256) || ws_bytes < score_workspace_bytes(l_c, m_hi - m_lo, eps, batch))
    ESA_FAIL(ESA_EWORKSPACE, "esa_score: workspace needs %zu bytes, 256-byte aligned",
             score_workspace_bytes(l_c, m_hi - m_lo, eps, batch));
  return launch_score(qc, l_c, kc_cache, m_lo, m_hi, d_c, eps, score, dtype, batch, q_bs, kc_bs, score_bs, workspace,
                      ws_bytes, (hipStream_t)stream);
}

size_t esa_select_topk_workspace_bytes(int64_t n, int k, int batch) { return topk_workspace_bytes(n, k, batch); }

int esa_select_topk(const float* score, int64_t n, int k, int64_t base, int32_t* idx, int batch, int64_t score_bs,
                    int64_t idx_bs, void* workspace, size_t ws_bytes, void* stream) {
  if (n < 0 || k < 0 || batch <= 0 || batch > kMaxBatch)
    ESA_FAIL(ESA_EINVAL, "esa_select_topk: bad size (n=%lld k=%d batch=%d)", (long long)n, k, batch);
  if (base < 0 || base + n > (int64_t)INT32_MAX) ESA_FAIL(ESA_EINVAL, "esa_select_topk: positions exceed int32");
  if (n == 0 || k == 0) return ESA_OK;
  if (!score || !idx) ESA_FAIL(ESA_EINVAL, "esa_select_topk: null pointer");
  if (!aligned(score, 4) || !aligned(idx, 4)) ESA_FAIL(ESA_EINVAL, "esa_select_topk: misaligned pointer");
  if (!workspace || !aligned(workspace, 256) || ws_bytes < topk_workspace_bytes(n, k, batch))
    ESA_FAIL(ESA_EWORKSPACE, "esa_select_topk: workspace needs %zu bytes, 256-byte aligned",
             topk_workspace_bytes(n, k, batch));
  return launch_topk(score, n, k, base, idx, batch, score_bs, idx_bs, workspace, ws_bytes, (hipStream_t)stream);
}

size_t esa_score_select_gather_workspace_bytes(int l_c, int64_t n_mid, int eps, int k, int batch) {
  return align_up(score_workspace_bytes(l_c, n_mid, eps, batch), 256) + topk_workspace_bytes(n_mid, k, batch);
}

int esa_score_select_gather(const void* qc, int l_c, const void* kc_cache, int64_t m_lo, int64_t m_hi, int d_c, int eps,
                            int k, float* score, int32_t* idx, const void* k_cache, const void* v_cache, int64_t tok_stride,
                            int h_kv, int d, void* k_sel, void* v_sel, int dtype, int batch, int64_t q_bs,
                            int64_t kc_bs, int64_t score_bs, int64_t idx_bs, int64_t cache_bs, int64_t sel_bs,
                            void* workspace, size_t ws_bytes, void* stream) {
  if (!dtype_ok(dtype)) ESA_FAIL(ESA_EUNSUPPORTED, "esa_score_select_gather: dtype %d", dtype);
  if (l_c <= 0 || d_c <= 0 || batch <= 0 || batch > kMaxBatch || k < 0 || eps < 0 || m_lo < 0 || m_hi < m_lo)
    ESA_FAIL(ESA_EINVAL, "esa_score_select_gather: bad size (l_c=%d d_c=%d batch=%d k=%d eps=%d m=[%lld,%lld))", l_c, d_c, batch,
             k, eps, (long long)m_lo, (long long)m_hi);
  if (d_c % 16 != 0 || d_c > 256) ESA_FAIL(ESA_EUNSUPPORTED, "esa_score_select_gather: d_c=%d (multiple of 16, <= 256)", d_c);
  if (m_hi > (int64_t)INT32_MAX) ESA_FAIL(ESA_EINVAL, "esa_score_select_gather: positions exceed int32");
  const int64_t n = m_hi - m_lo;
  if (n == 0 || k == 0) return ESA_OK;
  const bool gathers = k_cache || v_cache || k_sel || v_sel;
  if (!qc || !kc_cache || !idx || (k < n && !score)) ESA_FAIL(ESA_EINVAL, "esa_score_select_gather: null pointer");
  const size_t es = elem_size(dtype);
  if (!aligned(qc, es) || !aligned(kc_cache, es) || !aligned(score, 4) || !aligned(idx, 4))
    ESA_FAIL(ESA_EINVAL, "esa_score_select_gather: misaligned pointer");
  if (gathers) {
    if (!k_cache || !v_cache || !k_sel || !v_sel) ESA_FAIL(ESA_EINVAL, "esa_score_select_gather: the gather needs all four buffers");
    if (h_kv <= 0 || d <= 0 || tok_stride < (int64_t)h_kv * d)
      ESA_FAIL(ESA_EINVAL, "esa_score_select_gather: bad size (h_kv=%d d=%d tok_stride=%lld)", h_kv, d, (long long)tok_stride);
    if (!aligned(k_cache, es) || !aligned(v_cache, es) || !aligned(k_sel, es) || !aligned(v_sel, es))
      ESA_FAIL(ESA_EINVAL, "esa_score_select_gather: misaligned pointer");
  }
  const size_t need = esa_score_select_gather_workspace_bytes(l_c, n, eps, k, batch);
  if (!workspace || !aligned(workspace, 256) || ws_bytes < need)
    ESA_FAIL(ESA_EWORKSPACE, "esa_score_select_gather: workspace needs %zu bytes, 256-byte aligned", need);
  hipStream_t st = (hipStream_t)stream;
  const int k_eff = (int)(k < n ? k : n);
  const size_t score_ws = align_up(score_workspace_bytes(l_c, n, eps, batch), 256);
  char* topk_ws = (char*)workspace + score_ws;
  bool hist_done = false;
  int rc = ESA_OK;
  if (k < n) {     // otherwise every middle token is taken and no score is needed
    uint32_t* hists = (uint32_t*)topk_ws + TopkLayout::hist;
    rc = launch_score(qc, l_c, kc_cache, m_lo, m_hi, d_c, eps, score, dtype, batch, q_bs, kc_bs, score_bs, workspace, score_ws,
                      st, hists, topk_row_stride_words(n, batch), &hist_done);
    if (rc != ESA_OK) return rc;
  }
  rc = launch_topk(score, n, k, m_lo, idx, batch, score_bs, idx_bs, topk_ws, ws_bytes - score_ws, st, hist_done);
  if (rc != ESA_OK) return rc;
  if (gathers)
    rc = launch_gather(k_cache, v_cache, tok_stride, idx, k_eff, h_kv, d, k_sel, v_sel, dtype, batch, cache_bs, idx_bs, sel_bs, st);
  return rc;
}

size_t esa_select_topk_static_capacity(void) { return topk_static_capacity(); }

int esa_select_topk_static_prepare(void) { return topk_static_prepare(); }

int esa_select_topk_static(const float* score, int64_t n, int k, int64_t base, int32_t* idx, int batch,
                           int64_t score_bs, int64_t idx_bs, void* stream) {
  if (n < 0 || k < 0 || batch <= 0 || batch > kMaxBatch)
    ESA_FAIL(ESA_EINVAL, "esa_select_topk_static: bad size (n=%lld k=%d batch=%d)", (long long)n, k, batch);
  if (base < 0 || base + n > (int64_t)INT32_MAX) ESA_FAIL(ESA_EINVAL, "esa_select_topk_static: positions exceed int32");
  if (n == 0 || k == 0) return ESA_OK;
  if (!score || !idx) ESA_FAIL(ESA_EINVAL, "esa_select_topk_static: null pointer");
  if (!aligned(score, 4) || !aligned(idx, 4)) ESA_FAIL(ESA_EINVAL, "esa_select_topk_static: misaligned pointer");
  return launch_topk_static(score, n, k, base, idx, batch, score_bs, idx_bs, (hipStream_t)stream);
}

int esa_gather_kv(const void* k_cache, const void* v_cache, int64_t tok_stride, const int32_t* idx, int n_sel,
                  int h_kv, int d, void* k_sel, void* v_sel, int dtype, int batch, int64_t cache_bs, int64_t idx_bs,
                  int64_t sel_bs, void* stream) {
  if (!dtype_ok(dtype)) ESA_FAIL(ESA_EUNSUPPORTED, "esa_gather_kv: dtype %d", dtype);
  if (n_sel < 0 || h_kv <= 0 || d <= 0 || batch <= 0 || batch > kMaxBatch || tok_stride < (int64_t)h_kv * d)
    ESA_FAIL(ESA_EINVAL, "esa_gather_kv: bad size (n_sel=%d h_kv=%d d=%d batch=%d tok_stride=%lld)", n_sel, h_kv, d,
             batch, (long long)tok_stride);
  if (n_sel == 0) return ESA_OK;
  if (!k_cache || !v_cache || !idx || !k_sel || !v_sel) ESA_FAIL(ESA_EINVAL, "esa_gather_kv: null pointer");
  const size_t es = elem_size(dtype);
  if (!aligned(k_cache, es) || !aligned(v_cache, es) || !aligned(k_sel, es) || !aligned(v_sel, es) || !aligned(idx, 4))
    ESA_FAIL(ESA_EINVAL, "esa_gather_kv: misaligned pointer");
  return launch_gather(k_cache, v_cache, tok_stride, idx, n_sel, h_kv, d, k_sel, v_sel, dtype, batch, cache_bs, idx_bs,
                       sel_bs, (hipStream_t)stream);
}

size_t esa_attend_workspace_bytes(int l_c, int h, int h_kv, int d, int dtype, int batch) {
  return attend_workspace_bytes(l_c, h, h_kv, d, dtype, batch);
}

// Argument checks shared by every form of the attention call (everything but the workspace size).
static int attend_args_ok(int part, int split, const void* q, int l_c, int h, int h_kv, int d, const void* k_cache,
                          const void* v_cache, int64_t tok_stride, int64_t t0, int64_t l_i, int64_t l_l,
                          const void* k_sel, const void* v_sel, int n_sel, const int32_t* sel_idx, float scale,
                          const void* out, const float* lse, int dtype, int batch) {
  if (!dtype_ok(dtype)) ESA_FAIL(ESA_EUNSUPPORTED, "esa_attend: dtype %d", dtype);
  if (!(scale > 0.f) || !(scale < 3.0e38f)) ESA_FAIL(ESA_EINVAL, "esa_attend: scale must be positive and finite");
  if (t0 + l_c >= ((int64_t)1 << 31) || tok_stride >= ((int64_t)1 << 31))
    ESA_FAIL(ESA_EUNSUPPORTED, "esa_attend: positions or token strides beyond 2^31 are not supported");
  if (split != ESA_SPLIT_I_EARLY && split != ESA_SPLIT_ALGORITHM1) ESA_FAIL(ESA_EINVAL, "esa_attend: split %d", split);
  if (l_c <= 0 || h <= 0 || h_kv <= 0 || d <= 0 || batch <= 0 || batch > kMaxBatch || n_sel < 0 || t0 < 0 ||
      l_i < 0 || l_l < 0 || l_c > 65535 || h > 65535)
    ESA_FAIL(ESA_EINVAL, "esa_attend: bad size (l_c=%d h=%d h_kv=%d d=%d batch=%d n_sel=%d t0=%lld)", l_c, h, h_kv, d,
             batch, n_sel, (long long)t0);
  if (h % h_kv != 0) ESA_FAIL(ESA_EINVAL, "esa_attend: h=%d is not a multiple of h_kv=%d", h, h_kv);
  if (d > 256 || 256 % d != 0) ESA_FAIL(ESA_EUNSUPPORTED, "esa_attend: head size %d (32, 64, 128 or 256)", d);
  if (tok_stride < (int64_t)h_kv * d) ESA_FAIL(ESA_EINVAL, "esa_attend: tok_stride smaller than a token");
  if (!q || !k_cache || !v_cache || (part != kAttendLocal && !out)) ESA_FAIL(ESA_EINVAL, "esa_attend: null pointer");
  if (n_sel > 0 && !sel_idx && (!k_sel || !v_sel))
    ESA_FAIL(ESA_EINVAL, "esa_attend: null gathered buffer with n_sel > 0");
  if (sel_idx && !aligned(sel_idx, 4)) ESA_FAIL(ESA_EINVAL, "esa_attend_indexed: misaligned index list");
  {
    const Segments sg = segments(t0, l_i, l_l);
    if (n_sel > sg.l_start - sg.i_end)
      ESA_FAIL(ESA_EINVAL, "esa_attend: n_sel=%d exceeds the %lld middle tokens", n_sel,
               (long long)(sg.l_start - sg.i_end));
  }
  const size_t es = elem_size(dtype);
  if (!aligned(q, es) || !aligned(k_cache, es) || !aligned(v_cache, es) || !aligned(k_sel, es) || !aligned(v_sel, es) ||
      !aligned(out, es) || !aligned(lse, 4))
    ESA_FAIL(ESA_EINVAL, "esa_attend: misaligned pointer");
  return ESA_OK;
}

static int attend_checked(int part, int split, const void* q, int l_c, int h, int h_kv, int d, const void* k_cache,
                          const void* v_cache, int64_t tok_stride, int64_t t0, int64_t l_i, int64_t l_l,
                          const void* k_sel, const void* v_sel, int n_sel, const int32_t* sel_idx, int64_t idx_bs,
                          float scale, void* out, float* lse, int dtype, int batch, int64_t q_bs, int64_t cache_bs,
                          int64_t sel_bs, int64_t out_bs, void* workspace, size_t ws_bytes, void* stream) {
  const int rc = attend_args_ok(part, split, q, l_c, h, h_kv, d, k_cache, v_cache, tok_stride, t0, l_i, l_l, k_sel, v_sel,
                                n_sel, sel_idx, scale, out, lse, dtype, batch);
  if (rc != ESA_OK) return rc;
  const size_t need = sel_idx ? attend_indexed_workspace_bytes(l_c, h, h_kv, d, dtype, batch, n_sel)
                              : attend_workspace_bytes(l_c, h, h_kv, d, dtype, batch);
  if (need > 256 && (!workspace || !aligned(workspace, 256) || ws_bytes < need))
    ESA_FAIL(ESA_EWORKSPACE, "esa_attend: workspace needs %zu bytes, 256-byte aligned", need);
  return launch_attend(part, split, q, l_c, h, h_kv, d, k_cache, v_cache, tok_stride, t0, l_i, l_l, k_sel, v_sel, n_sel,
                       n_sel > 0 ? sel_idx : nullptr, idx_bs, scale, out, lse, dtype, batch, q_bs, cache_bs, sel_bs, out_bs, workspace, ws_bytes, (hipStream_t)stream);
}

int esa_attend(const void* q, int l_c, int h, int h_kv, int d, const void* k_cache, const void* v_cache,
               int64_t tok_stride, int64_t t0, int64_t l_i, int64_t l_l, const void* k_sel, const void* v_sel,
               int n_sel, float scale, void* out, float* lse, int dtype, int batch, int64_t q_bs, int64_t cache_bs,
               int64_t sel_bs, int64_t out_bs, void* workspace, size_t ws_bytes, void* stream) {
  return attend_checked(kAttendAll, ESA_SPLIT_I_EARLY, q, l_c, h, h_kv, d, k_cache, v_cache, tok_stride, t0, l_i, l_l, k_sel, v_sel, n_sel,
                        nullptr, 0, scale, out, lse, dtype, batch, q_bs, cache_bs, sel_bs, out_bs, workspace, ws_bytes, stream);
}

int esa_attend_local(const void* q, int l_c, int h, int h_kv, int d, const void* k_cache, const void* v_cache,
                     int64_t tok_stride, int64_t t0, int64_t l_i, int64_t l_l, float scale, int split, int dtype,
                     int batch, int64_t q_bs, int64_t cache_bs, void* workspace, size_t ws_bytes, void* stream) {
  return attend_checked(kAttendLocal, split, q, l_c, h, h_kv, d, k_cache, v_cache, tok_stride, t0, l_i, l_l, nullptr, nullptr,
                        0, nullptr, 0, scale, nullptr, nullptr, dtype, batch, q_bs, cache_bs, 0, 0, workspace, ws_bytes, stream);
}

int esa_attend_finish(const void* q, int l_c, int h, int h_kv, int d, const void* k_cache, const void* v_cache,
                      int64_t tok_stride, int64_t t0, int64_t l_i, int64_t l_l, const void* k_sel, const void* v_sel,
                      int n_sel, float scale, int split, void* out, float* lse, int dtype, int batch, int64_t q_bs,
                      int64_t cache_bs, int64_t sel_bs, int64_t out_bs, void* workspace, size_t ws_bytes,
                      void* stream) {
  return attend_checked(kAttendFinish, split, q, l_c, h, h_kv, d, k_cache, v_cache, tok_stride, t0, l_i, l_l, k_sel, v_sel,
                        n_sel, nullptr, 0, scale, out, lse, dtype, batch, q_bs, cache_bs, sel_bs, out_bs, workspace, ws_bytes,
                        stream);
}

size_t esa_attend_indexed_workspace_bytes(int l_c, int h, int h_kv, int d, int dtype, int batch, int n_sel) {
  return attend_indexed_workspace_bytes(l_c, h, h_kv, d, dtype, batch, n_sel);
}

int esa_attend_indexed(const void* q, int l_c, int h, int h_kv, int d, const void* k_cache, const void* v_cache,
                       int64_t tok_stride, int64_t t0, int64_t l_i, int64_t l_l, const int32_t* idx, int n_sel,
                       int64_t idx_bs, float scale, void* out, float* lse, int dtype, int batch, int64_t q_bs,
                       int64_t cache_bs, int64_t out_bs, void* workspace, size_t ws_bytes, void* stream) {
  if (n_sel > 0 && !idx) ESA_FAIL(ESA_EINVAL, "esa_attend_indexed: null index list with n_sel > 0");
  return attend_checked(kAttendAll, ESA_SPLIT_I_EARLY, q, l_c, h, h_kv, d, k_cache, v_cache, tok_stride, t0, l_i, l_l,
                        nullptr, nullptr, n_sel, idx, idx_bs, scale, out, lse, dtype, batch, q_bs, cache_bs, 0, out_bs,
                        workspace, ws_bytes, stream);
}

int esa_rope(const void* x, int64_t n_tok, int heads, int d, int64_t ldx, double pos0, double pos_step, double base,
             void* out, int64_t ldo, int dtype, int batch, int64_t x_bs, int64_t out_bs, void* stream) {
  if (!dtype_ok(dtype)) ESA_FAIL(ESA_EUNSUPPORTED, "esa_rope: dtype %d", dtype);
  if (n_tok < 0 || heads <= 0 || d <= 0 || batch <= 0 || batch > kMaxBatch || n_tok >= (int64_t)1 << 31)
    ESA_FAIL(ESA_EINVAL, "esa_rope: bad size (n_tok=%lld heads=%d d=%d batch=%d)", (long long)n_tok, heads, d, batch);
  if (!rope_head_size_ok(d)) ESA_FAIL(ESA_EUNSUPPORTED, "esa_rope: head size %d (a power of two from 2 to 256)", d);
  if (ldx < (int64_t)heads * d || ldo < (int64_t)heads * d) ESA_FAIL(ESA_EINVAL, "esa_rope: row stride smaller than the row");
  if (!(base > 0.0)) ESA_FAIL(ESA_EINVAL, "esa_rope: base must be positive");
  if (n_tok == 0) return ESA_OK;
  if (!x || !out) ESA_FAIL(ESA_EINVAL, "esa_rope: null pointer");
  if (!aligned(x, elem_size(dtype)) || !aligned(out, elem_size(dtype))) ESA_FAIL(ESA_EINVAL, "esa_rope: misaligned pointer");
  if (x == out && (ldx != ldo || x_bs != out_bs)) ESA_FAIL(ESA_EINVAL, "esa_rope: in place needs equal strides");
  const RopeJob job{x, out, n_tok, ldx, ldo, x_bs, out_bs, pos0, pos_step, heads, 1};
  return launch_rope_jobs(&job, 1, d, base, dtype, batch, (hipStream_t)stream);
}

size_t esa_attend_reencoded_workspace_bytes(int l_c, int h, int h_kv, int d, int dtype, int batch, int64_t l_l) {
  return attend_reencoded_workspace_bytes(l_c, h, h_kv, d, dtype, batch, l_l);
}

int esa_attend_reencoded(const void* q, int l_c, int h, int h_kv, int d, const void* k_cache, const void* v_cache,
                         int64_t tok_stride, int64_t t0, int64_t l_i, int64_t l_l, const void* k_sel, const void* v_sel,
                         int n_sel, float scale, double w, double rope_base, void* out, float* lse, int dtype, int batch,
                         int64_t q_bs, int64_t cache_bs, int64_t sel_bs, int64_t out_bs, void* workspace, size_t ws_bytes,
                         void* stream) {
  const int rc = attend_args_ok(kAttendAll, ESA_SPLIT_ALGORITHM1, q, l_c, h, h_kv, d, k_cache, v_cache, tok_stride, t0, l_i,
                                l_l, k_sel, v_sel, n_sel, nullptr, scale, out, lse, dtype, batch);
  if (rc != ESA_OK) return rc;
  if (!rope_head_size_ok(d)) ESA_FAIL(ESA_EUNSUPPORTED, "esa_attend_reencoded: head size %d", d);
  if (!(rope_base > 0.0) || !(w >= 0.0)) ESA_FAIL(ESA_EINVAL, "esa_attend_reencoded: base must be positive and w non-negative");
  const Segments sg = segments(t0, l_i, l_l);
  const size_t need = attend_reencoded_workspace_bytes(l_c, h, h_kv, d, dtype, batch, t0 - sg.l_start);
  if (!workspace || !aligned(workspace, 256) || ws_bytes < need)
    ESA_FAIL(ESA_EWORKSPACE, "esa_attend_reencoded: workspace needs %zu bytes, 256-byte aligned", need);
  return launch_attend_reencoded(q, l_c, h, h_kv, d, k_cache, v_cache, tok_stride, t0, l_i, l_l, k_sel, v_sel, n_sel, scale, w,
                                 rope_base, out, lse, dtype, batch, q_bs, cache_bs, sel_bs, out_bs, workspace, ws_bytes,
                                 (hipStream_t)stream);
}

}  // extern "C"
