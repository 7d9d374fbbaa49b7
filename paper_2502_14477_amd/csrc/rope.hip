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

// grid (rows, jobs, batch); 256 threads.  The row's d/2 angles are computed once (fp64) and shared
// through LDS; every thread then turns VEC consecutive pairs per step (VEC elements = 16 bytes per
// access when VEC > 1; VEC == 1 serves unaligned rows).
template <typename T, int VEC>
__global__ __launch_bounds__(256) void rope_rows(RopeJobs jobs, int d, double base) {
  __shared__ double cs[2][128];
  const RopeJob jb = jobs.j[blockIdx.y];
  const int64_t row = blockIdx.x;
  if (row >= jb.n_tok) return;
  const int half = d >> 1;
  const T* x = (const T*)jb.x + (int64_t)blockIdx.z * jb.x_bs + row * jb.ldx;
  T* o = (T*)jb.out + (int64_t)blockIdx.z * jb.out_bs + row * jb.ldo;
  typedef T vec_t __attribute__((ext_vector_type(VEC)));
  if (!jb.rotate) {                       // plain copy of the row
    const int n = jb.heads * d;
    for (int e = threadIdx.x * VEC; e < n; e += 256 * VEC) *(vec_t*)(o + e) = *(const vec_t*)(x + e);
    return;
  }
  const double pos = jb.pos0 + (double)row * jb.pos_step;
  if ((int)threadIdx.x < half) {
    double c = 1.0, s = 0.0;
    if (pos != 0.0) {
      const double ang = pos * pow(base, -2.0 * (double)threadIdx.x / (double)d);
      s = sin(ang);
      c = cos(ang);
    }
    cs[0][threadIdx.x] = c;
    cs[1][threadIdx.x] = s;
  }
  __syncthreads();
  const int n_pairs = jb.heads * half;    // half is a multiple of VEC
  for (int p = threadIdx.x * VEC; p < n_pairs; p += 256 * VEC) {
    const int h = p / half, i = p % half;
    const vec_t a = *(const vec_t*)(x + h * d + i), b = *(const vec_t*)(x + h * d + half + i);
    vec_t ra, rb;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      T ae = a[e], be = b[e];
      const double x1 = load_f64<T>(&ae), x2 = load_f64<T>(&be);
      const double c = cs[0][i + e], sn = cs[1][i + e];
      T r1, r2;
      store_f64<T>(&r1, x1 * c - x2 * sn);
      store_f64<T>(&r2, x2 * c + x1 * sn);
      ra[e] = r1;
      rb[e] = r2;
    }
    *(vec_t*)(o + h * d + i) = ra;
    *(vec_t*)(o + h * d + half + i) = rb;
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
  // 16-byte accesses when every row of every job starts on a 16-byte boundary
  const int vec = dtype == ESA_BF16 ? 8 : 4;
  bool wide = (d / 2) % vec == 0;
  for (int k = 0; k < n_jobs; ++k) {
    const RopeJob& j = jobs[k];
    wide = wide && ((uintptr_t)j.x % 16 == 0) && ((uintptr_t)j.out % 16 == 0) && j.ldx % vec == 0 && j.ldo % vec == 0 &&
           j.x_bs % vec == 0 && j.out_bs % vec == 0;
  }
  if (dtype == ESA_BF16) {
    if (wide)
      rope_rows<bf16_t, 8><<<grid, 256, 0, st>>>(js, d, base);
    else
      rope_rows<bf16_t, 1><<<grid, 256, 0, st>>>(js, d, base);
  } else {
    if (wide)
      rope_rows<float, 4><<<grid, 256, 0, st>>>(js, d, base);
    else
      rope_rows<float, 1><<<grid, 256, 0, st>>>(js, d, base);
  }
  ESA_LAUNCH_CHECK("rope_rows");
  return ESA_OK;
}

}  // namespace esa
