// Rotary position encoding of query / key rows (Section 3.2 re-encodes positions per step: local
// keys and queries in order, global queries at one fixed position, initial and selected keys at
// position 0, which is the identity).  Rotate-half pairing: element i of a head's first half and
// element i of its second half turn by the angle pos * base^(-2i/d).
//
// The arithmetic is fp64 end to end and rounds once into the storage type, so a row encoded here
// equals the fp64 definition rounded to storage.  The volume is small (the chunk's queries and the
// local window's keys, a few MB per step); one workgroup per row, one frequency per thread.
#include "esa_common.h"

namespace esa {
namespace {

struct RopeJobs {
  RopeJob j[kMaxRopeJobs];
};

// fp64 -> bf16, round to nearest even in one step (through fp32 first would round twice).
__device__ __forceinline__ bf16_t f64_to_bf16(double v) {
  const float f = (float)v;
  const float a = fabsf(f);
  if (!(a >= 1.1754944e-38f && a < 3.0e38f)) return f32_to_bf16(f);   // zero, subnormal, huge, NaN: via fp32
  uint64_t u = (uint64_t)__double_as_longlong(v);
  u += ((1ull << 44) - 1) + ((u >> 45) & 1ull);      // 52 - 7 = 45 fraction bits go
  u &= ~((1ull << 45) - 1);
  return (bf16_t)(__float_as_uint((float)__longlong_as_double((long long)u)) >> 16);   // exact conversions
}

template <typename T> __device__ __forceinline__ double load_f64(const T* p);
template <> __device__ __forceinline__ double load_f64<float>(const float* p) { return (double)*p; }
template <> __device__ __forceinline__ double load_f64<bf16_t>(const bf16_t* p) { return (double)bf16_to_f32(*p); }
template <typename T> __device__ __forceinline__ void store_f64(T* p, double v);
template <> __device__ __forceinline__ void store_f64<float>(float* p, double v) { *p = (float)v; }
template <> __device__ __forceinline__ void store_f64<bf16_t>(bf16_t* p, double v) { *p = f64_to_bf16(v); }

// grid (rows, jobs, batch); 256 threads; 256 % (d/2) == 0.
template <typename T>
__global__ __launch_bounds__(256) void rope_rows(RopeJobs jobs, int d, double base) {
  const RopeJob jb = jobs.j[blockIdx.y];
  const int64_t row = blockIdx.x;
  if (row >= jb.n_tok) return;
  const int half = d >> 1;
  const int i = threadIdx.x % half, h0 = threadIdx.x / half, h_step = 256 / half;
  const T* x = (const T*)jb.x + (int64_t)blockIdx.z * jb.x_bs + row * jb.ldx;
  T* o = (T*)jb.out + (int64_t)blockIdx.z * jb.out_bs + row * jb.ldo;
  if (!jb.rotate) {                       // plain copy of the row
    for (int e = threadIdx.x; e < jb.heads * d; e += 256) o[e] = x[e];
    return;
  }
  const double pos = jb.pos0 + (double)row * jb.pos_step;
  double c = 1.0, s = 0.0;
  if (pos != 0.0) {
    const double ang = pos * pow(base, -2.0 * (double)i / (double)d);
    s = sin(ang);
    c = cos(ang);
  }
  for (int h = h0; h < jb.heads; h += h_step) {
    const double x1 = load_f64<T>(x + h * d + i), x2 = load_f64<T>(x + h * d + half + i);
    store_f64<T>(o + h * d + i, x1 * c - x2 * s);
    store_f64<T>(o + h * d + half + i, x2 * c + x1 * s);
  }
}

}  // namespace

bool rope_head_size_ok(int d) { return d >= 2 && d <= 256 && (d & (d - 1)) == 0; }

int launch_rope_jobs(const RopeJob* jobs, int n_jobs, int d, double base, int dtype, int batch, hipStream_t st) {
  RopeJobs js;
  int64_t rows = 0;
  for (int k = 0; k < kMaxRopeJobs; ++k) {
    js.j[k] = jobs[k < n_jobs ? k : 0];
    if (k >= n_jobs) js.j[k].n_tok = 0;
    if (js.j[k].n_tok > rows) rows = js.j[k].n_tok;
  }
  if (rows == 0) return ESA_OK;
  const dim3 grid((unsigned)rows, n_jobs, batch);
  if (dtype == ESA_BF16)
    rope_rows<bf16_t><<<grid, 256, 0, st>>>(js, d, base);
  else
    rope_rows<float><<<grid, 256, 0, st>>>(js, d, base);
  ESA_LAUNCH_CHECK("rope_rows");
  return ESA_OK;
}

}  // namespace esa
