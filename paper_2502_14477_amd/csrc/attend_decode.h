// Split-key attention kernel for decode-sized chunks, bf16 storage, head size 128 (defined in attend_decode.hip).
#pragma once
#include "esa_common.h"

namespace esa {

bool attend_decode_supported(int l_c, int h, int h_kv, int d, int dtype);
// false when the virtual key sequence is longer than the kernel's slices cover
bool attend_decode_covers(int64_t n_keys_max, int l_c, int h_kv, int batch);
size_t attend_decode_workspace_bytes(int l_c, int h, int batch);
// two-part form: false when the local part alone needs more than half of the kernel's slices
bool attend_decode_covers_parts(int64_t n_local_max, int l_c, int h_kv, int batch);
// part: 0 everything; 1 the local keys [ L | C ] (partial results only); 2 the global keys [ I | M_k ] and the merge
int launch_attend_decode(int part, const void* q, int l_c, int h, int h_kv, const void* k_cache, const void* v_cache,
                         int64_t tok_stride, int64_t t0, int64_t i_end, int64_t l_start, const void* k_sel,
                         const void* v_sel, int n_sel, const int32_t* sel_idx, int64_t idx_bs, float scale, void* out,
                         float* lse, int batch, int64_t q_bs, int64_t cache_bs, int64_t sel_bs, int64_t out_bs, void* ws,
                         size_t ws_bytes, hipStream_t st);

}  // namespace esa
