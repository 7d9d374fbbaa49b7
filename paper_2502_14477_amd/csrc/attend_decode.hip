// Selected attention (Eq. 1) for decode-sized chunks (fewer than 16 current tokens), bf16 storage,
// head size 128.  A decode step reads every attended key and value once (17 MB per sequence at the
// Llama shape) for a few hundred FLOPs per byte less than the matrix cores need, so the kernel is
// built around memory parallelism: the virtual key sequence [ I | M_k | L | C ] is cut into slices,
// one workgroup per (slice, KV head, current token, batch element), and the G query heads that share
// the KV head are served by the same loads.  Slices are merged with the log-sum-exp rule of
// Algorithm 1 by a second small kernel.
#include "esa_common.h"
#include "attend_decode.h"
#include "keyspace.h"

namespace esa {
namespace {

constexpr int kD = 128;            // head size
constexpr int kLanesPerKey = 16;   // 16 lanes x 16 bytes = one 256-byte key row of one KV head
constexpr int kGroups = 16;        // key rows in flight per workgroup and load instruction (256 threads)
constexpr int kUnroll = 4;         // independent loads per lane before the first use
constexpr int kMaxSlice = 1024;    // keys per workgroup (logits are kept in LDS)
constexpr int kMaxSplits = 128;   // the merge kernel holds two slices per lane
constexpr int kTargetWorkgroups = 1024;

// Sum over the 16 lanes of a DPP row; every lane receives the total.
__device__ __forceinline__ float row16_sum(float v) {
  int x;
  x = __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true);    // quad_perm [1,0,3,2]
  v += __int_as_float(x);
  x = __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
  v += __int_as_float(x);
  x = __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true);   // row_half_mirror
  v += __int_as_float(x);
  x = __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true);   // row_mirror
  v += __int_as_float(x);
  return v;
}

// The same value summed / maximised over the lanes 16 and 32 apart, in the vector unit (row swaps), where a
// general shuffle goes through the LDS crossbar and waits for it.
__device__ __forceinline__ float across_rows_sum(float v) {
  auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
  sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
}
__device__ __forceinline__ float across_rows_max(float v) {
  auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
  sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}
// Maximum over the 16 lanes of a DPP row; every lane receives it.
__device__ __forceinline__ float row16_max(float v) {
  int x;
  x = __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true);
  v = fmaxf(v, __int_as_float(x));
  x = __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true);
  v = fmaxf(v, __int_as_float(x));
  x = __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true);
  v = fmaxf(v, __int_as_float(x));
  x = __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true);
  v = fmaxf(v, __int_as_float(x));
  return v;
}

__device__ __forceinline__ void unpack8(const uint4& r, float* f) {
  f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xFFFF0000u);
  f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xFFFF0000u);
  f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xFFFF0000u);
  f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xFFFF0000u);
}

struct DecodeArgs {
  const bf16_t* q;
  KeySpace ks;
  int64_t n_fixed;
  float scale_log2e;
  int l_c, h_kv, splits, slice;   // splits: slots per output row (the row stride of the partial results)
  int slot0;         // this launch fills slots slot0 + blockIdx.x
  int with_chunk;    // 1: the virtual sequence ends with the current tokens (causal); 0: every key is visible
  float* part_o;     // [rows][splits][128]
  float* part_ml;    // [rows][splits][2]  (max of the base-2 logits, sum of 2^(logit - max))
  int64_t q_bs, cache_bs_bytes, sel_bs_bytes, idx_bs;
};

template <int G>
__global__ __launch_bounds__(256) void attend_decode_bf16(DecodeArgs a) {
  __shared__ float logit[G][kMaxSlice];
  __shared__ int32_t src_row[kMaxSlice];     // where key jj of the slice lives: cache row r as r, gathered row r as ~r
  __shared__ float red[4][G * kD];
  __shared__ float head_m[G], head_l[G];

  const int tid = threadIdx.x, sub = tid % kLanesPerKey, group = tid / kLanesPerKey;
  const int split = a.slot0 + blockIdx.x, g = blockIdx.y, c = blockIdx.z % a.l_c, b = blockIdx.z / a.l_c;
  const int h = a.h_kv * G;
  KeySpace ks = a.ks;
  ks.k_cache += (int64_t)b * a.cache_bs_bytes;
  ks.v_cache += (int64_t)b * a.cache_bs_bytes;
  if (ks.sel_idx) {
    ks.sel_idx += (int64_t)b * a.idx_bs;
  } else if (ks.n_sel > 0) {
    ks.k_sel += (int64_t)b * a.sel_bs_bytes;
    ks.v_sel += (int64_t)b * a.sel_bs_bytes;
  }
  const int64_t n_keys = a.n_fixed + (a.with_chunk ? c + 1 : 0);
  const int64_t j_lo = (int64_t)blockIdx.x * a.slice;
  const int cnt = (int)(n_keys - j_lo < a.slice ? (n_keys - j_lo > 0 ? n_keys - j_lo : 0) : a.slice);
  const int64_t row0 = ((int64_t)b * a.l_c + c) * h + (int64_t)g * G;   // first of this workgroup's G output rows
  const int64_t head_off = (int64_t)g * kD * 2 + sub * 16;              // byte offset inside a token row

  if (cnt == 0) {   // slice past this token's causal limit
    if (tid < G) {
      float* ml = a.part_ml + ((row0 + tid) * a.splits + split) * 2;
      ml[0] = -INFINITY;
      ml[1] = 0.f;
    }
    return;
  }

  // this lane's 8 elements of each of the G queries (scaled below so that logits are base-2 exponents)
  uint4 q_raw[G];
#pragma unroll
  for (int hh = 0; hh < G; ++hh)
    q_raw[hh] = *(const uint4*)(a.q + (int64_t)b * a.q_bs + ((int64_t)c * h + g * G + hh) * kD + sub * 8);

  // ---- where every key of the slice lives.  Resolved for the whole slice up front, with the index list's
  // entries requested together: done key by key in front of each row load, every look-up is a round trip of
  // its own that the row loads behind it wait for.
  {
    constexpr int kPerThread = kMaxSlice / 256;
    int32_t picked[kPerThread];
#pragma unroll
    for (int u = 0; u < kPerThread; ++u) picked[u] = 0;
    if (ks.sel_idx && ks.n_sel > 0) {      // unconditional loads (entry 0 where there is nothing to look up): all in flight together
#pragma unroll
      for (int u = 0; u < kPerThread; ++u) {
        const int jj = tid + 256 * u;
        const int64_t js = j_lo + jj - ks.i_end;
        picked[u] = ks.sel_idx[(jj < cnt && js >= 0 && js < ks.n_sel) ? js : 0];
      }
    }
#pragma unroll
    for (int u = 0; u < kPerThread; ++u) {
      const int jj = tid + 256 * u;
      if (jj < cnt) {
        const int64_t j = j_lo + jj, js = j - ks.i_end;
        int64_t row;
        bool gathered = false;
        if (js < 0) {
          row = j;
        } else if (js < ks.n_sel) {
          if (ks.sel_idx) {     // a middle token: clamped so that a bad index cannot leave the cache
            row = picked[u];
            row = row < ks.l_start ? row : ks.l_start - 1;
            row = row < 0 ? 0 : row;
          } else {
            row = js;
            gathered = true;
          }
        } else {
          row = ks.l_start + (js - ks.n_sel);
        }
        src_row[jj] = gathered ? ~(int32_t)row : (int32_t)row;
      }
    }
  }
  float qf[G][8];
#pragma unroll
  for (int hh = 0; hh < G; ++hh) {
    unpack8(q_raw[hh], qf[hh]);
#pragma unroll
    for (int i = 0; i < 8; ++i) qf[hh][i] *= a.scale_log2e;
  }
  __syncthreads();

  // byte offset of key jj's row and whether it is a gathered row (a key past the slice's end stands for key 0:
  // its row is loaded and not used)
  auto locate = [&](int jj, bool* gathered) -> int64_t {
    const int32_t code = src_row[jj < cnt ? jj : 0];
    *gathered = code < 0;
    return code < 0 ? (int64_t)(~code) * ks.sel_bytes : (int64_t)code * ks.tok_bytes;
  };

  // values of the first round of keys: requested now, used after the softmax
  uint4 v_first[kUnroll];
  {
    uint4 r[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      bool gathered;
      const int64_t off = locate(u * kGroups + group, &gathered) + head_off;
      v_first[u] = *(const uint4*)((gathered ? ks.v_sel : ks.v_cache) + off);
      r[u] = *(const uint4*)((gathered ? ks.k_sel : ks.k_cache) + off);
    }
    // ---- logits of the slice: 16 lanes per key, kUnroll keys per lane group in flight
    for (int j0 = 0; j0 < cnt; j0 += kGroups * kUnroll) {
      if (j0 > 0) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
          bool gathered;
          const int64_t off = locate(j0 + u * kGroups + group, &gathered) + head_off;
          r[u] = *(const uint4*)((gathered ? ks.k_sel : ks.k_cache) + off);
        }
      }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int jj = j0 + u * kGroups + group;
        float kf[8];
        unpack8(r[u], kf);
        float mine = 0.f;
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
          float s = 0.f;
#pragma unroll
          for (int i = 0; i < 8; ++i) s = __fmaf_rn(qf[hh][i], kf[i], s);
          s = row16_sum(s);
          if (sub == hh) mine = s;
        }
        if (sub < G && jj < cnt) logit[sub][jj] = mine;
      }
    }
  }
  __syncthreads();

  // ---- per head: maximum, probabilities (unnormalised) and their sum
  for (int hh = tid >> 6; hh < G; hh += 4) {
    const int lane = tid & 63;
    float m = -INFINITY;
    for (int jj = lane; jj < cnt; jj += 64) m = fmaxf(m, logit[hh][jj]);
    m = across_rows_max(row16_max(m));
    float l = 0.f;
    for (int jj = lane; jj < cnt; jj += 64) {
      const float p = __builtin_amdgcn_exp2f(logit[hh][jj] - m);      // arguments <= 0: no range handling needed
      logit[hh][jj] = p;
      l += p;
    }
    l = across_rows_sum(row16_sum(l));
    if (lane == 0) {
      head_m[hh] = m;
      head_l[hh] = l;
    }
  }
  __syncthreads();

  // ---- weighted sum of the values: lane keeps 8 output dims of each head for its key subset
  float acc[G][8];
#pragma unroll
  for (int hh = 0; hh < G; ++hh)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[hh][i] = 0.f;
  for (int j0 = 0; j0 < cnt; j0 += kGroups * kUnroll) {
    uint4 r[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int jj = j0 + u * kGroups + group;
      r[u] = v_first[u];
      if (j0 > 0) {
        bool gathered;
        const int64_t off = locate(jj, &gathered) + head_off;
        r[u] = *(const uint4*)((gathered ? ks.v_sel : ks.v_cache) + off);
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int jj = j0 + u * kGroups + group;
      if (jj < cnt) {
        float vf[8];
        unpack8(r[u], vf);
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
          const float p = logit[hh][jj];
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[hh][i] = __fmaf_rn(p, vf[i], acc[hh][i]);
        }
      }
    }
  }
  // the four lane groups of a wave, then the four waves
#pragma unroll
  for (int hh = 0; hh < G; ++hh)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      acc[hh][i] = across_rows_sum(acc[hh][i]);
    }
  if ((tid & 63) < kLanesPerKey) {
#pragma unroll
    for (int hh = 0; hh < G; ++hh)
#pragma unroll
      for (int i = 0; i < 8; ++i) red[tid >> 6][hh * kD + sub * 8 + i] = acc[hh][i];
  }
  __syncthreads();
  for (int e = tid; e < G * kD; e += 256) {
    const float o = (red[0][e] + red[1][e]) + (red[2][e] + red[3][e]);
    const int hh = e / kD, dim = e % kD;
    a.part_o[((row0 + hh) * a.splits + split) * kD + dim] = o;
  }
  if (tid < G) {
    float* ml = a.part_ml + ((row0 + tid) * a.splits + split) * 2;
    ml[0] = head_m[tid];
    ml[1] = head_l[tid];
  }
}

// One workgroup per output row (batch element, current token, query head): slices combined by their
// maxima and sums.  The call is two dependent round trips at most if nothing is done about it (the weights come
// from the (max, sum) pairs, the sum needs the weights), and round trips are all it costs: so every lane requests
// the pairs of up to two slices and, without waiting for them, the partial outputs of all the slices of its wave
// (wave w takes slices w, w + 8, ...: eight or sixteen independent loads, two output dims per lane).  The eight
// waves' shares meet in LDS and are added in a fixed order.
constexpr int kMergeWaves = 8;
__global__ __launch_bounds__(kMergeWaves * 64) void attend_decode_merge(const float* __restrict__ part_o,
                                                                        const float* __restrict__ part_ml, int splits,
                                                                        int stride, int l_c, int h,
                                                                        bf16_t* __restrict__ out, int64_t out_bs,
                                                                        float* __restrict__ lse) {
  static_assert(kMaxSplits <= 128 && kMaxSplits <= 16 * kMergeWaves, "two pairs per lane, sixteen slices per wave");
  __shared__ float red[kMergeWaves][kD];
  const int64_t row = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float2* ml = (const float2*)(part_ml + row * stride * 2);   // slots [0, splits) of `stride` are in use
  float2 a0 = make_float2(-INFINITY, 0.f), a1 = make_float2(-INFINITY, 0.f);
  if (lane < splits) a0 = ml[lane];
  if (lane + 64 < splits) a1 = ml[lane + 64];
  const float* po = part_o + row * stride * kD + lane * 2;
  float2 o[16];
  // a slice past the end re-reads slice 0 and gets weight 0
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const int s = wave + kMergeWaves * u;
    o[u] = *(const float2*)(po + (int64_t)(s < splits ? s : 0) * kD);
  }
  if (splits > 8 * kMergeWaves) {
#pragma unroll
    for (int u = 8; u < 16; ++u) {
      const int s = wave + kMergeWaves * u;
      o[u] = *(const float2*)(po + (int64_t)(s < splits ? s : 0) * kD);
    }
  } else {
#pragma unroll
    for (int u = 8; u < 16; ++u) o[u] = make_float2(0.f, 0.f);
  }
  const float m = wave_max(fmaxf(a0.x, a1.x));
  const float w0 = a0.y > 0.f ? exp2f(a0.x - m) : 0.f;
  const float w1 = a1.y > 0.f ? exp2f(a1.x - m) : 0.f;
  const float l = wave_sum(__fmaf_rn(w0, a0.y, w1 * a1.y));
  float o0 = 0.f, o1 = 0.f;
#pragma unroll
  for (int u = 0; u < 16; ++u) {
    const int s = wave + kMergeWaves * u;              // below 64 for u < 8, from 64 on otherwise
    const float ws = u < 8 ? __shfl(w0, s, 64) : __shfl(w1, s - 64, 64);
    const float w = s < splits ? ws : 0.f;
    o0 += w != 0.f ? w * o[u].x : 0.f;                 // slices past the causal limit hold no output
    o1 += w != 0.f ? w * o[u].y : 0.f;
  }
  red[wave][lane * 2] = o0;
  red[wave][lane * 2 + 1] = o1;
  __syncthreads();
  if (wave == 0) {
    o0 = ((red[0][lane * 2] + red[1][lane * 2]) + (red[2][lane * 2] + red[3][lane * 2])) +
         ((red[4][lane * 2] + red[5][lane * 2]) + (red[6][lane * 2] + red[7][lane * 2]));
    o1 = ((red[0][lane * 2 + 1] + red[1][lane * 2 + 1]) + (red[2][lane * 2 + 1] + red[3][lane * 2 + 1])) +
         ((red[4][lane * 2 + 1] + red[5][lane * 2 + 1]) + (red[6][lane * 2 + 1] + red[7][lane * 2 + 1]));
    const int64_t b = row / ((int64_t)l_c * h), r = row % ((int64_t)l_c * h);
    const float inv = 1.f / l;
    const uint32_t packed = (uint32_t)f32_to_bf16(o0 * inv) | ((uint32_t)f32_to_bf16(o1 * inv) << 16);
    *(uint32_t*)(out + b * out_bs + r * kD + lane * 2) = packed;
    if (lse && lane == 0) lse[row] = (m + log2f(l)) * 0.6931471805599453f;
  }
}

struct Plan {
  int splits, slice;
};

// Slices of at most kMaxSlice keys (a multiple of the 64 keys one workgroup has in flight), enough of
// them to put about kTargetWorkgroups on the chip.  splits == 0: more keys than the kernel covers.
Plan plan_for(int64_t n_keys_max, int l_c, int h_kv, int batch) {
  const int64_t per_slice_wgs = (int64_t)l_c * h_kv * batch;
  int64_t want = (kTargetWorkgroups + per_slice_wgs - 1) / per_slice_wgs;
  if (want > kMaxSplits) want = kMaxSplits;
  if (want < 1) want = 1;
  int64_t slice = (n_keys_max + want - 1) / want;
  slice = (slice + 63) / 64 * 64;
  if (slice > kMaxSlice) slice = kMaxSlice;
  const int64_t splits = (n_keys_max + slice - 1) / slice;
  Plan p;
  p.slice = (int)slice;
  p.splits = splits > kMaxSplits ? 0 : (int)splits;
  return p;
}

}  // namespace

bool attend_decode_supported(int l_c, int h, int h_kv, int d, int dtype) {
  if (dtype != ESA_BF16 || d != kD || l_c >= 16 || h % h_kv != 0) return false;
  const int group = h / h_kv;
  return group == 1 || group == 2 || group == 4 || group == 8;
}

bool attend_decode_covers(int64_t n_keys_max, int l_c, int h_kv, int batch) {
  return plan_for(n_keys_max, l_c, h_kv, batch).splits > 0;
}

size_t attend_decode_workspace_bytes(int l_c, int h, int batch) {
  const size_t rows = (size_t)batch * l_c * h;
  return align_up(rows * kMaxSplits * kD * sizeof(float), 256) + align_up(rows * kMaxSplits * 2 * sizeof(float), 256);
}

bool attend_decode_covers_parts(int64_t n_local_max, int l_c, int h_kv, int batch) {
  const Plan p = plan_for(n_local_max, l_c, h_kv, batch);
  return p.splits > 0 && p.splits <= kMaxSplits / 2;
}

// part: 0 whole key sequence and merge; 1 the local keys [ L | C ] into the first slots; 2 the global
// keys [ I | M_k ] (every key visible) into the slots behind them, then the merge over both.  The two-part
// form gives each part at most half of the slots and addresses rows with the full stride, so that the
// first call needs to know nothing about the second.
int launch_attend_decode(int part, const void* q, int l_c, int h, int h_kv, const void* k_cache, const void* v_cache,
                         int64_t tok_stride, int64_t t0, int64_t i_end, int64_t l_start, const void* k_sel,
                         const void* v_sel, int n_sel, const int32_t* sel_idx, int64_t idx_bs, float scale, void* out,
                         float* lse, int batch, int64_t q_bs, int64_t cache_bs, int64_t sel_bs, int64_t out_bs, void* ws,
                         size_t ws_bytes, hipStream_t st) {
  const int64_t n_local = t0 - l_start, n_global = i_end + n_sel;
  const int64_t n_fixed = part == 0 ? n_global + n_local : part == 1 ? n_local : n_global;
  const int with_chunk = part != 2;
  const int64_t n_part = n_fixed + (with_chunk ? l_c : 0);
  Plan p;
  p.splits = 0;
  p.slice = 64;
  if (n_part > 0) p = plan_for(n_part, l_c, h_kv, batch);
  int slot0 = 0, used = p.splits, stride = p.splits;
  if (part != 0) {
    const Plan pl = plan_for(n_local + l_c, l_c, h_kv, batch);
    if (pl.splits <= 0 || pl.splits > kMaxSplits / 2 || (part == 2 && n_part > 0 && (p.splits <= 0 || p.splits > kMaxSplits / 2)))
      ESA_FAIL(ESA_EUNSUPPORTED, "attend_decode (two parts): a part of %lld keys exceeds the kernel's range",
               (long long)(part == 1 ? n_local + l_c : n_fixed));
    stride = kMaxSplits;
    slot0 = part == 1 ? 0 : pl.splits;
    used = part == 1 ? pl.splits : pl.splits + p.splits;
  } else if (p.splits <= 0) {
    ESA_FAIL(ESA_EUNSUPPORTED, "attend_decode: %lld keys exceed the kernel's range", (long long)(n_fixed + l_c));
  }
  if (ws_bytes < attend_decode_workspace_bytes(l_c, h, batch)) ESA_FAIL(ESA_EWORKSPACE, "attend_decode: workspace too small");
  if (t0 + l_c > (int64_t)INT32_MAX || n_sel < 0)     // the kernel keeps row numbers as 32-bit integers
    ESA_FAIL(ESA_EUNSUPPORTED, "attend_decode: %lld cache rows exceed the kernel's range", (long long)(t0 + l_c));
  const size_t rows = (size_t)batch * l_c * h;
  DecodeArgs a;
  a.q = (const bf16_t*)q;
  a.ks.k_cache = (const char*)k_cache;
  a.ks.v_cache = (const char*)v_cache;
  a.ks.k_sel = (const char*)k_sel;
  a.ks.v_sel = (const char*)v_sel;
  a.ks.sel_idx = sel_idx;
  a.idx_bs = idx_bs;
  a.ks.tok_bytes = tok_stride * 2;
  a.ks.sel_bytes = (int64_t)h_kv * kD * 2;
  a.ks.i_end = part == 1 ? 0 : i_end;
  a.ks.n_sel = part == 1 ? 0 : n_sel;
  a.ks.l_start = l_start;
  a.n_fixed = n_fixed;
  a.with_chunk = with_chunk;
  a.slot0 = slot0;
  a.scale_log2e = scale * 1.4426950408889634f;
  a.l_c = l_c;
  a.h_kv = h_kv;
  a.splits = stride;
  a.slice = p.slice;
  a.part_o = (float*)ws;
  a.part_ml = (float*)((char*)ws + align_up(rows * kMaxSplits * kD * sizeof(float), 256));
  a.q_bs = q_bs;
  a.cache_bs_bytes = cache_bs * 2;
  a.sel_bs_bytes = sel_bs * 2;
  if (p.splits > 0) {
    const dim3 grid(p.splits, h_kv, batch * l_c);
    switch (h / h_kv) {
      case 1: attend_decode_bf16<1><<<grid, 256, 0, st>>>(a); break;
      case 2: attend_decode_bf16<2><<<grid, 256, 0, st>>>(a); break;
      case 4: attend_decode_bf16<4><<<grid, 256, 0, st>>>(a); break;
      default: attend_decode_bf16<8><<<grid, 256, 0, st>>>(a); break;
    }
    ESA_LAUNCH_CHECK("attend_decode_bf16");
  }
  if (part != 1) {
    attend_decode_merge<<<(unsigned)rows, kMergeWaves * 64, 0, st>>>(a.part_o, a.part_ml, used, stride, l_c, h, (bf16_t*)out, out_bs, lse);
    ESA_LAUNCH_CHECK("attend_decode_merge");
  }
  return ESA_OK;
}

}  // namespace esa
