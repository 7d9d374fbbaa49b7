// Index-driven fetch of the selected tokens' full-size keys and values (Section 1, Appendix B).
//
// A token's keys (all KV heads) are one contiguous row of h_kv*d elements (2 KB for 8 heads of
// 128 bf16), likewise its values.  One workgroup moves a few rows: every lane copies 16 bytes
// of K and 16 bytes of V per step, so a wave reads and writes whole 1 KB runs and the writes
// to the dense destination are fully coalesced.  Pure byte movement: HBM-bound.
#include "esa_common.h"

namespace esa {
namespace {

constexpr int kRowsPerBlock = 4;

template <typename Vec>
__global__ __launch_bounds__(256) void gather_rows(const char* __restrict__ k_cache, const char* __restrict__ v_cache,
                                                   int64_t tok_bytes, const int32_t* __restrict__ idx, int n_sel,
                                                   int row_vecs, char* __restrict__ k_sel, char* __restrict__ v_sel,
                                                   int64_t cache_bs_bytes, int64_t idx_bs, int64_t sel_bs_bytes) {
  const int b = blockIdx.y;
  const int32_t* ix = idx + (int64_t)b * idx_bs;
  const char* kc = k_cache + (int64_t)b * cache_bs_bytes;
  const char* vc = v_cache + (int64_t)b * cache_bs_bytes;
  char* ks = k_sel + (int64_t)b * sel_bs_bytes;
  char* vs = v_sel + (int64_t)b * sel_bs_bytes;
  const int64_t row_bytes = (int64_t)row_vecs * (int64_t)sizeof(Vec);
  const int lanes_per_row = blockDim.x / kRowsPerBlock;
  const int r = blockIdx.x * kRowsPerBlock + threadIdx.x / lanes_per_row;
  if (r >= n_sel) return;
  const int lane = threadIdx.x % lanes_per_row;
  const int64_t tok = ix[r];
  const Vec* ksrc = (const Vec*)(kc + tok * tok_bytes);
  const Vec* vsrc = (const Vec*)(vc + tok * tok_bytes);
  Vec* kdst = (Vec*)(ks + (int64_t)r * row_bytes);
  Vec* vdst = (Vec*)(vs + (int64_t)r * row_bytes);
  for (int i = lane; i < row_vecs; i += lanes_per_row) {
    const Vec a = ksrc[i];
    const Vec c = vsrc[i];
    kdst[i] = a;
    vdst[i] = c;
  }
}

}  // namespace

int launch_gather(const void* k_cache, const void* v_cache, int64_t tok_stride, const int32_t* idx, int n_sel,
                  int h_kv, int d, void* k_sel, void* v_sel, int dtype, int batch, int64_t cache_bs,
                  int64_t idx_bs, int64_t sel_bs, hipStream_t st) {
  const int64_t esz = (dtype == ESA_F32) ? 4 : 2;
  const int64_t row_bytes = (int64_t)h_kv * d * esz;
  const int64_t tok_bytes = tok_stride * esz;
  const dim3 grid((n_sel + kRowsPerBlock - 1) / kRowsPerBlock, batch);
  const uintptr_t all = (uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)k_sel | (uintptr_t)v_sel |
                        (uintptr_t)row_bytes | (uintptr_t)tok_bytes | (uintptr_t)(cache_bs * esz) |
                        (uintptr_t)(sel_bs * esz);
  if ((all & 15) == 0) {
    gather_rows<uint4><<<grid, 256, 0, st>>>((const char*)k_cache, (const char*)v_cache, tok_bytes, idx, n_sel,
                                             (int)(row_bytes / 16), (char*)k_sel, (char*)v_sel, cache_bs * esz,
                                             idx_bs, sel_bs * esz);
  } else if ((all & 3) == 0) {
    gather_rows<uint32_t><<<grid, 256, 0, st>>>((const char*)k_cache, (const char*)v_cache, tok_bytes, idx, n_sel,
                                                (int)(row_bytes / 4), (char*)k_sel, (char*)v_sel, cache_bs * esz,
                                                idx_bs, sel_bs * esz);
  } else {
    gather_rows<uint16_t><<<grid, 256, 0, st>>>((const char*)k_cache, (const char*)v_cache, tok_bytes, idx, n_sel,
                                                (int)(row_bytes / 2), (char*)k_sel, (char*)v_sel, cache_bs * esz,
                                                idx_bs, sel_bs * esz);
  }
  ESA_LAUNCH_CHECK("gather_rows");
  return ESA_OK;
}

}  // namespace esa
