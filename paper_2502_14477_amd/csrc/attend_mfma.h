// Matrix-core attention kernel for bf16 storage, head size 128 (declared here, defined in attend_mfma.hip).
#pragma once
#include "esa_common.h"

namespace esa {

bool attend_mfma_supported(int l_c, int h, int h_kv, int d, int dtype);
bool attend_mfma_aligned(const void* q, const void* k_cache, const void* v_cache, const void* k_sel,
                         const void* v_sel, const void* out, int64_t tok_stride, int64_t q_bs, int64_t cache_bs,
                         int64_t sel_bs, int64_t out_bs);
// Which part of Eq. 1's key set a launch covers: everything (one call), or Algorithm 1's split into the part
// that does not depend on the selection ([ I | L | C ], partial results only) and the selected part plus merge.
enum { kAttendAll = 0, kAttendLocal = 1, kAttendFinish = 2 };
size_t attend_mfma_workspace_bytes(int l_c, int h, int h_kv, int d, int batch);
int launch_attend_mfma(int part, int split, const void* q, int l_c, int h, int h_kv, int d, const void* k_cache, const void* v_cache,
                       int64_t tok_stride, int64_t t0, int64_t i_end, int64_t l_start, const void* k_sel,
                       const void* v_sel, int n_sel, const int32_t* sel_idx, int64_t idx_bs, float scale, void* out,
                       float* lse, int batch, int64_t q_bs, int64_t cache_bs, int64_t sel_bs, int64_t out_bs, void* ws,
                       size_t ws_bytes, hipStream_t st);

// Section 3.2's two differently encoded parts in one launch (see attend_mfma.hip).
int launch_attend_mfma_two_views(const void* q_loc, const void* q_glob, int64_t qw_bs, int l_c, int h, int h_kv, int d,
                                 const void* k_loc, const void* v_loc, int64_t n_loc, int64_t loc_bs,
                                 const void* k_cache, const void* v_cache, int64_t tok_stride, int64_t cache_bs,
                                 int64_t i_end, const void* k_sel, const void* v_sel, int n_sel, int64_t sel_bs,
                                 float scale, void* out, float* lse, int batch, int64_t out_bs, void* ws, size_t ws_bytes,
                                 hipStream_t st);

}  // namespace esa
