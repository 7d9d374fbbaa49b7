// Shared declarations of libesa's translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "esa.h"

namespace esa {

// ---------------------------------------------------------------- errors (host)
void set_error(const char* fmt, ...);
int hip_failed(hipError_t e, const char* what);   // records the text, returns ESA_EHIP

#define ESA_FAIL(code, ...)          \
  do {                               \
    ::esa::set_error(__VA_ARGS__);   \
    return (code);                   \
  } while (0)

#define ESA_LAUNCH_CHECK(what)                                   \
  do {                                                           \
    hipError_t e__ = hipGetLastError();                          \
    if (e__ != hipSuccess) return ::esa::hip_failed(e__, what);  \
  } while (0)

// ---------------------------------------------------------------- storage types
typedef uint16_t bf16_t;   // raw bfloat16 bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// Round to nearest, ties to even.  Inputs are finite in every use inside the library.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T> __device__ __forceinline__ float load_f32(const T* p);
template <> __device__ __forceinline__ float load_f32<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_f32<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }

template <typename T> __device__ __forceinline__ void store_f32(T* p, float v);
template <> __device__ __forceinline__ void store_f32<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_f32<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// ---------------------------------------------------------------- order-preserving keys
// fp32 -> uint32 such that a < b (as floats, -0 < +0) <=> key(a) < key(b) (as unsigned).
__device__ __forceinline__ uint32_t ordered_key(float f) {
  uint32_t u = __float_as_uint(f);
  return u ^ ((u & 0x80000000u) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float ordered_key_to_f32(uint32_t k) {
  uint32_t u = k ^ ((k & 0x80000000u) ? 0x80000000u : 0xFFFFFFFFu);
  return __uint_as_float(u);
}
constexpr uint32_t kOrderedKeyOfMinusInf = 0x007FFFFFu;   // ordered_key(-inf)

// ---------------------------------------------------------------- wave helpers (64 lanes)
// Maximum / sum over the 64 lanes of a wave, every lane gets the result.  In the vector unit throughout: DPP moves
// inside the 16-lane rows, row swaps across them (v_permlane16_swap, v_permlane32_swap).  A general shuffle goes
// through the LDS crossbar and costs a round trip per step.  Every lane of the wave must be active.
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true)));    // quad_perm [1,0,3,2]
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true)));    // quad_perm [2,3,0,1]
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true)));   // row_half_mirror
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true)));   // row_mirror
  auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
  sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true));
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true));
  auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
  sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
}

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---------------------------------------------------------------- segment arithmetic (Section 3.1)
struct Segments {
  int64_t i_end, l_start;
};
static inline Segments segments(int64_t t0, int64_t l_i, int64_t l_l) {
  Segments s;
  s.i_end = l_i < t0 ? l_i : t0;
  s.l_start = (t0 - l_l) > s.i_end ? (t0 - l_l) : s.i_end;
  return s;
}

// ---------------------------------------------------------------- launchers (one per .hip file)
int launch_pack_weights(const void* W, int64_t d_in, int d_c, int dtype, void* Wt, hipStream_t st);
int launch_compress(const void* x, int64_t n_tok, int64_t d_in, int64_t ldx, const void* W, int w_layout,
                    const void* bias, int d_c, void* out, int64_t ldo, int dtype, int batch, int64_t x_bs,
                    int64_t out_bs, hipStream_t st);

int launch_compress_pair(const void* x0, int64_t d_in0, int64_t ldx0, const void* W0, const void* bias0, void* out0,
                         int64_t ldo0, int64_t x0_bs, int64_t out0_bs, const void* x1, int64_t d_in1, int64_t ldx1,
                         const void* W1, const void* bias1, void* out1, int64_t ldo1, int64_t x1_bs, int64_t out1_bs,
                         int64_t n_tok, int d_c, int w_layout, int dtype, int batch, hipStream_t st);

size_t score_workspace_bytes(int l_c, int64_t n_mid, int eps, int batch);
// first_hist: null, or [batch] rows (stride first_hist_bs words) holding the three digit histograms of the
// selection that follows; when the kernels in use can, they zero all three and fill the first with the
// leading digits of the scores they write, and *first_hist_done is set.
int launch_score(const void* qc, int l_c, const void* kc_cache, int64_t m_lo, int64_t m_hi, int d_c, int eps,
                 float* score, int dtype, int batch, int64_t q_bs, int64_t kc_bs, int64_t score_bs,
                 void* ws, size_t ws_bytes, hipStream_t st, uint32_t* first_hist = nullptr, int64_t first_hist_bs = 0,
                 bool* first_hist_done = nullptr);

size_t topk_workspace_bytes(int64_t n, int k, int batch);
// first_hist_ready: the workspace's histograms are zeroed and the first one already holds the scores'
// leading digits (left there by launch_score).
int launch_topk(const float* score, int64_t n, int k, int64_t base, int32_t* idx, int batch, int64_t score_bs,
                int64_t idx_bs, void* ws, size_t ws_bytes, hipStream_t st, bool first_hist_ready = false);

size_t topk_static_capacity();
int topk_static_prepare();
int launch_topk_static(const float* score, int64_t n, int k, int64_t base, int32_t* idx, int batch, int64_t score_bs,
                       int64_t idx_bs, hipStream_t st);

int launch_gather(const void* k_cache, const void* v_cache, int64_t tok_stride, const int32_t* idx, int n_sel,
                  int h_kv, int d, void* k_sel, void* v_sel, int dtype, int batch, int64_t cache_bs,
                  int64_t idx_bs, int64_t sel_bs, hipStream_t st);

size_t attend_workspace_bytes(int l_c, int h, int h_kv, int d, int dtype, int batch);
size_t attend_indexed_workspace_bytes(int l_c, int h, int h_kv, int d, int dtype, int batch, int n_sel);
int launch_attend(int part, int split, const void* q, int l_c, int h, int h_kv, int d, const void* k_cache, const void* v_cache,
                  int64_t tok_stride, int64_t t0, int64_t l_i, int64_t l_l, const void* k_sel, const void* v_sel,
                  int n_sel, const int32_t* sel_idx, int64_t idx_bs, float scale, void* out, float* lse, int dtype,
                  int batch, int64_t q_bs, int64_t cache_bs, int64_t sel_bs, int64_t out_bs, void* ws, size_t ws_bytes,
                  hipStream_t st);

// Section 3.2: rotary re-encoding.  One launch serves up to four row sets ("jobs"); row i of a job
// is rotated to position pos0 + i * pos_step, or copied unchanged when rotate == 0.
constexpr int kMaxRopeJobs = 4;
struct RopeJob {
  const void* x;
  void* out;
  int64_t n_tok, ldx, ldo, x_bs, out_bs;   // rows; row strides and batch strides in elements
  double pos0, pos_step;
  int heads, rotate;
};
bool rope_head_size_ok(int d);
int launch_rope_jobs(const RopeJob* jobs, int n_jobs, int d, double base, int dtype, int batch, hipStream_t st);

size_t attend_reencoded_workspace_bytes(int l_c, int h, int h_kv, int d, int dtype, int batch, int64_t l_l);
int launch_attend_reencoded(const void* q, int l_c, int h, int h_kv, int d, const void* k_cache, const void* v_cache,
                            int64_t tok_stride, int64_t t0, int64_t l_i, int64_t l_l, const void* k_sel,
                            const void* v_sel, int n_sel, float scale, double w, double base, void* out, float* lse,
                            int dtype, int batch, int64_t q_bs, int64_t cache_bs, int64_t sel_bs, int64_t out_bs,
                            void* ws, size_t ws_bytes, hipStream_t st);

}  // namespace esa
