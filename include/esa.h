/*
 * libesa — the per-step hot path of Efficient Selective Attention (ESA, arXiv 2502.14477)
 * for AMD MI355X (gfx950).  C ABI; every tensor argument is a DEVICE pointer owned by the
 * caller.  The library never allocates, frees or keeps a pointer; every call only enqueues
 * kernels on `stream` (a hipStream_t passed as void*, NULL = the default stream) and
 * returns without synchronising.
 *
 * One ESA step for the current tokens C at positions [t0, t0+l_c) (Section 3.1):
 *   preceding tokens split into  I = [0, i_end)   i_end   = min(l_i, t0)
 *                                M = [i_end, l_start)
 *                                L = [l_start, t0)  l_start = max(t0 - l_l, i_end)
 *   1. esa_compress     q'_c = f_theta_q(q_c), k'_m = f_theta_k(k_m)            (Eq. 5)
 *   2. esa_score        F_s(m;C) = max_c ( q'_c.k'_m - max_m' q'_c.k'_m' )      (Eq. 6 in Eq. 4)
 *   3. esa_select_topk  M_k = the k middle tokens with the highest F_s           (Eq. 2)
 *   4. esa_gather_kv    full-size keys/values of M_k                             (Section 1, App. B)
 *   5. esa_attend       O = Attn(Q_C, K_[I,M_k,L,C], V_[I,M_k,L,C])              (Eq. 1)
 *
 * Layout conventions: row-major, innermost dimension contiguous, strides in ELEMENTS.
 * `dtype` is the storage type of Q, K, V, W, bias, K', Q' and O; scores and lse are always
 * fp32, indices int32.  Arithmetic accumulates in fp32.  `batch` independent sequences are
 * processed by one call; `*_bs` arguments are the element strides between them.
 *
 * Return value: ESA_OK or a negative error code.  Nothing is enqueued when an error is
 * returned.  esa_last_error() gives a text for the calling thread's last error.
 * The library never throws, aborts or prints.
 */
#ifndef ESA_H
#define ESA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Exported symbols (the library is built with hidden default visibility). */
#define ESA_API __attribute__((visibility("default")))

#define ESA_F32 0
#define ESA_BF16 1

#define ESA_OK 0
#define ESA_EINVAL (-1)       /* null pointer, non-positive size, bad range, misaligned pointer, H % H_kv != 0 */
#define ESA_EUNSUPPORTED (-2) /* dtype / head size / compressed size not built */
#define ESA_EWORKSPACE (-3)   /* workspace missing or smaller than esa_*_workspace_bytes says */
#define ESA_EHIP (-4)         /* a HIP call failed; see esa_last_error() */

/* Library version: major*10000 + minor*100 + patch. */
ESA_API int esa_version(void);

/* Text of the calling thread's most recent error ("" if none).  Host pointer, owned by the library. */
ESA_API const char* esa_last_error(void);

/* Host-side segment arithmetic of Section 3.1 (no GPU work): writes i_end and l_start. */
ESA_API int esa_segments(int64_t t0, int64_t l_i, int64_t l_l, int64_t* i_end, int64_t* l_start);

/* Layout of the compression weights handed to esa_compress. */
#define ESA_W_ROWMAJOR 0      /* W [d_in, d_c], as a linear layer y = x W stores it */
#define ESA_W_PACKED 1        /* W^T [d_c, d_in], written by esa_pack_weights: the fast path */

/*
 * One-time re-layout of a compression weight matrix (per layer, at load time; not part of a
 * step): W [d_in, d_c] contiguous -> W_packed [d_c, d_in] contiguous, same dtype.  With packed
 * weights both matrix-core operands of Eq. 5 are read with their reduction elements contiguous.
 */
ESA_API int esa_pack_weights(const void* W, int64_t d_in, int d_c, int dtype, void* W_packed, void* stream);

/*
 * Eq. 5 — compression by one linear layer on the head-concatenated vector.
 *   x    [batch][n_tok, d_in]  row stride ldx, batch stride x_bs.  A [n_tok, heads, d] tensor is
 *        its own head-major concatenation (Section 3.1), so d_in = heads*d and ldx = heads*d.
 *   W    [d_in, d_c] contiguous (w_layout = ESA_W_ROWMAJOR) or its packed form [d_c, d_in]
 *        (ESA_W_PACKED), shared by the batch;  bias [d_c] or NULL.
 *   out  [batch][n_tok, d_c]   row stride ldo, batch stride out_bs; rounded to `dtype`
 *        (nearest-even).  Writing K' rows of the current tokens straight into the compressed-key
 *        cache is done by pointing `out` at cache row t0.
 * n_tok == 0 is a no-op.  d_c must be a multiple of 16 and at most 256.
 */
ESA_API int esa_compress(const void* x, int64_t n_tok, int64_t d_in, int64_t ldx,
                 const void* W, int w_layout, const void* bias, int d_c,
                 void* out, int64_t ldo,
                 int dtype, int batch, int64_t x_bs, int64_t out_bs, void* stream);

/*
 * Eq. 5 for the chunk's queries and keys in one call: exactly what two esa_compress calls compute
 * (queries: xq, Wq, bias_q -> out_q; keys: xk, Wk, bias_k -> out_k, e.g. rows t0.. of the compressed-key
 * cache), over the same n_tok tokens, d_c, weight layout, dtype and batch.  With packed weights and bf16
 * the two products share one launch.  Arguments as esa_compress, per tensor.
 */
ESA_API int esa_compress_qk(const void* xq, int64_t d_in_q, int64_t ldxq, const void* Wq, const void* bias_q,
                 void* out_q, int64_t ldoq, int64_t xq_bs, int64_t outq_bs,
                 const void* xk, int64_t d_in_k, int64_t ldxk, const void* Wk, const void* bias_k,
                 void* out_k, int64_t ldok, int64_t xk_bs, int64_t outk_bs,
                 int64_t n_tok, int d_c, int w_layout, int dtype, int batch, void* stream);

/*
 * Eq. 6 inside Eq. 4 — importance of every middle token m in [m_lo, m_hi):
 *   S[c,m] = qc[c] . kc_cache[m];  mu[c] = max_m S[c,m];  score[m-m_lo] = max_c (S[c,m] - mu[c]).
 * Consequently score <= 0, its maximum is exactly 0, and every current token's best middle
 * token scores exactly 0.  With eps > 0 the result is then replaced by its running maximum over
 * [m-eps, m+eps] clamped to the middle segment (Eq. 8).
 *   qc        [batch][l_c, d_c]  contiguous rows, batch stride q_bs
 *   kc_cache  [batch][>= m_hi, d_c] contiguous rows, batch stride kc_bs
 *   score     [batch][m_hi-m_lo] fp32, batch stride score_bs
 *   workspace esa_score_workspace_bytes(l_c, m_hi-m_lo, eps, batch) bytes, 256-byte aligned
 * m_hi == m_lo is a no-op.
 */
ESA_API size_t esa_score_workspace_bytes(int l_c, int64_t n_mid, int eps, int batch);
ESA_API int esa_score(const void* qc, int l_c,
              const void* kc_cache, int64_t m_lo, int64_t m_hi, int d_c,
              int eps, float* score, int dtype,
              int batch, int64_t q_bs, int64_t kc_bs, int64_t score_bs,
              void* workspace, size_t ws_bytes, void* stream);

/*
 * Eq. 2 — indices of the k_eff = min(k, n) largest scores, written as ASCENDING absolute
 * positions (array index + base).  Equal scores: the lower position wins.  Scores are compared
 * as IEEE fp32 totally ordered by value (-0 < +0; NaN must not occur).
 *   score [batch][n] fp32;  idx [batch][k_eff] int32, batch stride idx_bs
 *   workspace esa_select_topk_workspace_bytes(n, k, batch) bytes, 256-byte aligned
 * n == 0 or k == 0 is a no-op.
 */
ESA_API size_t esa_select_topk_workspace_bytes(int64_t n, int k, int batch);
ESA_API int esa_select_topk(const float* score, int64_t n, int k, int64_t base,
                    int32_t* idx,
                    int batch, int64_t score_bs, int64_t idx_bs,
                    void* workspace, size_t ws_bytes, void* stream);

/*
 * esa_score, esa_select_topk (base = m_lo) and, if wanted, esa_gather_kv in one call, with two
 * kernels fewer than the three calls: the kernel that writes the scores (Eq. 4, or Eq. 8's pooling
 * pass when eps > 0) also leaves the first digit histogram of the radix selection (Eq. 2) while the
 * scores are still on chip, and the zero-fill of the histograms rides on an earlier kernel of the
 * score call.
 * Results are those of the separate calls, bit for bit.
 *   score    [batch][m_hi-m_lo] fp32, written as by esa_score; if k >= m_hi-m_lo every middle token is
 *            selected, nothing is scored and `score` is left untouched (it may then be NULL)
 *   idx      [batch][min(k, m_hi-m_lo)] int32, ascending absolute positions
 *   k_cache, v_cache, k_sel, v_sel, tok_stride, h_kv, d, cache_bs, sel_bs as in esa_gather_kv; pass all
 *            four pointers as NULL to skip the gather
 *   workspace esa_score_select_gather_workspace_bytes(l_c, m_hi-m_lo, eps, k, batch) bytes, 256-byte aligned
 * Shapes outside the fused kernels (fp32, d_c other than 64/128/256) run the kernels of the three
 * calls in sequence.  m_hi == m_lo or k == 0 is a no-op.
 */
ESA_API size_t esa_score_select_gather_workspace_bytes(int l_c, int64_t n_mid, int eps, int k, int batch);
ESA_API int esa_score_select_gather(const void* qc, int l_c,
                    const void* kc_cache, int64_t m_lo, int64_t m_hi, int d_c, int eps, int k,
                    float* score, int32_t* idx,
                    const void* k_cache, const void* v_cache, int64_t tok_stride, int h_kv, int d,
                    void* k_sel, void* v_sel,
                    int dtype, int batch, int64_t q_bs, int64_t kc_bs, int64_t score_bs, int64_t idx_bs,
                    int64_t cache_bs, int64_t sel_bs,
                    void* workspace, size_t ws_bytes, void* stream);

/*
 * esa_select_topk for callers that cannot allocate device memory or pass a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation): the same kernels, with
 * their scratch in an array that the library itself holds on every GPU it runs on, from load until
 * the process ends.  No allocation of any kind happens in these calls.
 *   esa_select_topk_static_capacity  bytes of scratch held per GPU; a call is accepted when
 *                                    esa_select_topk_workspace_bytes(n, k, batch) does not exceed it
 *                                    (e.g. 16 rows of 262144 scores), ESA_EWORKSPACE otherwise
 *   esa_select_topk_static_prepare   optional: looks the array's device address up for the current
 *                                    device now (otherwise the first call on a device does it); a
 *                                    host-side query, nothing is enqueued
 *   esa_select_topk_static           arguments and results exactly as esa_select_topk
 * All calls on one GPU share the one array, which keeps the previous call's contents (what must start
 * at zero is cleared by the call itself): calls that overlap in time on the same GPU, from any
 * stream or thread, race.  Calls on different GPUs are independent.
 */
ESA_API size_t esa_select_topk_static_capacity(void);
ESA_API int esa_select_topk_static_prepare(void);
ESA_API int esa_select_topk_static(const float* score, int64_t n, int k, int64_t base,
                    int32_t* idx,
                    int batch, int64_t score_bs, int64_t idx_bs, void* stream);

/*
 * Fetch the full-size keys and values of the selected tokens into dense buffers.
 *   k_cache, v_cache [batch][S, h_kv, d]  token stride tok_stride (>= h_kv*d), batch stride cache_bs
 *   idx              [batch][n_sel] token positions (each in [0, S); not checked on the device)
 *   k_sel, v_sel     [batch][n_sel, h_kv, d] contiguous, batch stride sel_bs
 * n_sel == 0 is a no-op.  The caches only have to be addressable by the GPU: with the KV cache
 * offloaded to pinned, device-mapped host memory (Appendix B) the selected rows are fetched over
 * the host link by the same call.
 */
ESA_API int esa_gather_kv(const void* k_cache, const void* v_cache, int64_t tok_stride,
                  const int32_t* idx, int n_sel, int h_kv, int d,
                  void* k_sel, void* v_sel,
                  int dtype, int batch, int64_t cache_bs, int64_t idx_bs, int64_t sel_bs, void* stream);

/*
 * Eq. 1 — softmax attention of the current tokens over [I, M_k, L, C]:
 *   out[c,h] = sum_j softmax_j( scale * q[c,h].k[j,g] ) v[j,g],   g = h / (h / h_kv),
 *   j over cache rows [0, i_end), the n_sel gathered rows, cache rows [l_start, t0),
 *   and cache rows [t0, t0+c] (a current token sees itself and earlier current tokens;
 *   Algorithm 1: causal local part, non-causal global part, one normalisation).
 * The caller has already stored the current tokens' keys/values in cache rows [t0, t0+l_c).
 *   q    [batch][l_c, h, d] contiguous, batch stride q_bs
 *   k_cache, v_cache as in esa_gather_kv;  k_sel, v_sel [batch][n_sel, h_kv, d] (may be NULL if n_sel == 0)
 *   out  [batch][l_c, h, d] contiguous, batch stride out_bs
 *   lse  [batch][l_c, h] fp32 natural-log normaliser, batch stride l_c*h; NULL to skip
 *   workspace esa_attend_workspace_bytes(...) bytes, 256-byte aligned
 * Values may use the whole finite range of the storage type as long as the products and sums of Eq. 1
 * stay finite in fp32; intermediate results that pass through the workspace carry their own scale.
 */
ESA_API size_t esa_attend_workspace_bytes(int l_c, int h, int h_kv, int d, int dtype, int batch);
ESA_API int esa_attend(const void* q, int l_c, int h, int h_kv, int d,
               const void* k_cache, const void* v_cache, int64_t tok_stride,
               int64_t t0, int64_t l_i, int64_t l_l,
               const void* k_sel, const void* v_sel, int n_sel,
               float scale, void* out, float* lse,
               int dtype, int batch, int64_t q_bs, int64_t cache_bs, int64_t sel_bs, int64_t out_bs,
               void* workspace, size_t ws_bytes, void* stream);

/*
 * Eq. 1 in two calls, cut where Algorithm 1 cuts it: the keys that do not depend on the selection
 * and the keys that do, each part a softmax of its own (running maximum and sum kept), the two merged
 * by their log-sum-exp weights.  esa_attend_local can be enqueued on another stream at the start of
 * the step and run beside compress / score / select / gather; esa_attend_finish needs the gathered
 * rows and must be ordered after esa_attend_local (event or same stream).
 *   split = ESA_SPLIT_I_EARLY    early part [ I | L | C ], late part M_k: the initial tokens are known
 *                                before the selection, so they go with the early part.  Both calls
 *                                are given the same q and caches; the pair computes what esa_attend
 *                                computes, to rounding (the slices' boundaries differ).
 *   split = ESA_SPLIT_ALGORITHM1 early part [ L | C ] (causal), late part [ I | M_k ] (every key
 *                                visible): Algorithm 1's grouping, for the position encoding of
 *                                Section 3.2, where the two parts see differently encoded queries
 *                                and keys.  esa_attend_local is given the queries and the key cache
 *                                encoded with in-order positions; esa_attend_finish the queries
 *                                encoded at the fixed position w, the key cache (rows [0, i_end) are
 *                                read) and the gathered keys encoded at position 0.  Values are the
 *                                same in both.  One softmax over the union, as in Eq. 1.
 *   esa_attend_local   arguments as esa_attend, without the gathered rows and the outputs; leaves
 *                      partial results in `workspace`
 *   esa_attend_finish  arguments exactly as esa_attend, same `workspace`; writes out / lse
 * Both calls must be given identical sizes, strides, split and workspace.  With ESA_SPLIT_I_EARLY,
 * shapes outside the matrix-core kernel (fp32, head sizes other than 128, chunks shorter than 16
 * tokens) are served whole by esa_attend_finish and esa_attend_local enqueues nothing; with
 * ESA_SPLIT_ALGORITHM1 they run the plain kernel once per part.
 */
#define ESA_SPLIT_I_EARLY 0
#define ESA_SPLIT_ALGORITHM1 1
ESA_API int esa_attend_local(const void* q, int l_c, int h, int h_kv, int d,
               const void* k_cache, const void* v_cache, int64_t tok_stride,
               int64_t t0, int64_t l_i, int64_t l_l, float scale, int split,
               int dtype, int batch, int64_t q_bs, int64_t cache_bs,
               void* workspace, size_t ws_bytes, void* stream);
ESA_API int esa_attend_finish(const void* q, int l_c, int h, int h_kv, int d,
               const void* k_cache, const void* v_cache, int64_t tok_stride,
               int64_t t0, int64_t l_i, int64_t l_l,
               const void* k_sel, const void* v_sel, int n_sel,
               float scale, int split, void* out, float* lse,
               int dtype, int batch, int64_t q_bs, int64_t cache_bs, int64_t sel_bs, int64_t out_bs,
               void* workspace, size_t ws_bytes, void* stream);

/*
 * esa_gather_kv and esa_attend in one call: the selected tokens' keys and values are read from the
 * caches through the index list (ascending absolute positions, as esa_select_topk writes them), so
 * no gathered copy is written and read back: only the selected rows are read, once (Appendix B's
 * per-step loading of the selected keys and values).  Computes exactly what esa_gather_kv followed by esa_attend computes.  Every
 * kernel follows the indices itself; the matrix-core prefill kernel looks the rows of a tile up one
 * tile ahead of the tile's loads.
 *   idx  [batch][n_sel] int32, batch stride idx_bs; entries are positions of middle tokens (an entry
 *        outside [0, l_start) is clamped into it rather than followed)
 *   workspace esa_attend_indexed_workspace_bytes(...) bytes, 256-byte aligned
 * Other arguments as esa_attend.
 */
ESA_API size_t esa_attend_indexed_workspace_bytes(int l_c, int h, int h_kv, int d, int dtype, int batch, int n_sel);
ESA_API int esa_attend_indexed(const void* q, int l_c, int h, int h_kv, int d,
               const void* k_cache, const void* v_cache, int64_t tok_stride,
               int64_t t0, int64_t l_i, int64_t l_l,
               const int32_t* idx, int n_sel, int64_t idx_bs,
               float scale, void* out, float* lse,
               int dtype, int batch, int64_t q_bs, int64_t cache_bs, int64_t out_bs,
               void* workspace, size_t ws_bytes, void* stream);

/*
 * Rotary position encoding of rows (Section 3.2 assumes a model that uses it): row i of
 * x [n_tok][heads][d] is turned to position pos0 + i*pos_step, i.e. element j of a head's first half
 * and element j of its second half rotate by the angle pos * base^(-2j/d) (rotate-half pairing).
 * Position 0 leaves a row unchanged.  pos_step = 0 puts every row at pos0 (Section 3.2's fixed
 * distance w of the global queries), pos_step = 1 numbers them in order (its local window).
 * Computed in fp64 and rounded once into the storage type.
 *   x, out  device pointers, row strides ldx / ldo and batch strides x_bs / out_bs in elements;
 *           out may equal x when the strides are equal (in place), otherwise they must not overlap
 *   d       a power of two from 2 to 256
 * Errors: ESA_EINVAL (sizes, null or misaligned pointer, base <= 0), ESA_EUNSUPPORTED (dtype, d).
 */
ESA_API int esa_rope(const void* x, int64_t n_tok, int heads, int d, int64_t ldx,
               double pos0, double pos_step, double base,
               void* out, int64_t ldo, int dtype, int batch, int64_t x_bs, int64_t out_bs, void* stream);

/*
 * Eq. 1 with the position re-encoding of Section 3.2, on queries and key caches that carry NO
 * position encoding yet: the local keys (the rows of L and C present) are encoded at positions
 * 0, 1, ... in order and the chunk's queries at the positions that follow the local window; for
 * the global part every query sits at the fixed position w and the initial and selected keys at
 * position 0; the two groups of logits share one softmax (Algorithm 1's merge of the two partial
 * attentions).  The library encodes the chunk's queries twice and the local rows of the key cache
 * once into its workspace (esa_rope's arithmetic), then runs the local and the global part.
 *   q, k_cache, k_sel   un-encoded; v_cache, v_sel, out, lse, sizes and strides as esa_attend
 *   w, rope_base        the global queries' position and the encoding's base
 *   workspace           esa_attend_reencoded_workspace_bytes(..., l_l) bytes, 256-byte aligned
 * For bf16 storage with head size 128 and chunks of 16 tokens or more, pointers and strides must
 * be 16-byte aligned (ESA_EINVAL otherwise).  Other errors as esa_attend.
 */
ESA_API size_t esa_attend_reencoded_workspace_bytes(int l_c, int h, int h_kv, int d, int dtype, int batch, int64_t l_l);
ESA_API int esa_attend_reencoded(const void* q, int l_c, int h, int h_kv, int d,
               const void* k_cache, const void* v_cache, int64_t tok_stride,
               int64_t t0, int64_t l_i, int64_t l_l,
               const void* k_sel, const void* v_sel, int n_sel,
               float scale, double w, double rope_base, void* out, float* lse,
               int dtype, int batch, int64_t q_bs, int64_t cache_bs, int64_t sel_bs, int64_t out_bs,
               void* workspace, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ESA_H */
