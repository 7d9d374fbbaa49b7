// The virtual key sequence one ESA step attends over (Eq. 1):
//   [ I | M_k | L | C ]  =  cache rows [0, i_end) ++ gathered rows [0, n_sel) ++ cache rows [l_start, t0 + l_c).
// M_k is read either from the gathered buffers or, through an index list, from the caches themselves.
// Current token c sees virtual keys [0, n_fixed + c], n_fixed = i_end + n_sel + (t0 - l_start).
#pragma once
#include "esa_common.h"

namespace esa {

struct KeySpace {
  const char* k_cache;
  const char* v_cache;
  const char* k_sel;
  const char* v_sel;
  const int32_t* sel_idx; // non-null: selected row j is cache row sel_idx[j] (no gathered buffers)
  int64_t tok_bytes;      // cache token stride in bytes
  int64_t sel_bytes;      // gathered-row stride in bytes
  int64_t i_end, n_sel, l_start;
};

// Address of virtual key j's row (all KV heads) in the key or value storage.
__device__ __forceinline__ const char* key_row(const KeySpace& ks, int64_t j, bool values) {
  if (j < ks.i_end) return (values ? ks.v_cache : ks.k_cache) + j * ks.tok_bytes;
  j -= ks.i_end;
  if (j < ks.n_sel) {
    if (ks.sel_idx) {
      int64_t row = ks.sel_idx[j];                       // a middle token: clamped so that a bad index cannot leave the cache
      row = row < 0 ? 0 : (row < ks.l_start ? row : ks.l_start - 1);
      return (values ? ks.v_cache : ks.k_cache) + row * ks.tok_bytes;
    }
    return (values ? ks.v_sel : ks.k_sel) + j * ks.sel_bytes;
  }
  j -= ks.n_sel;
  return (values ? ks.v_cache : ks.k_cache) + (ks.l_start + j) * ks.tok_bytes;
}

}  // namespace esa
