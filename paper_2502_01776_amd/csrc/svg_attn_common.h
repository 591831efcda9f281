// Types, kernel arguments and small device helpers shared by the attention kernels.
#pragma once
#include "svg_internal.h"

namespace svg {
namespace attn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

enum Mode { kDense = 0, kSparse = 1, kProfile = 2, kSparseExact = 3 };

constexpr int kCodeDrop = 0x7fffffff;   // key beyond N: never kept
constexpr int kCodeKeep = 0x7ffffffe;   // text key / sink key: kept by every query
constexpr float kNegBig = -1.0e30f;     // finite stand-in for -inf as the initial row maximum
constexpr float kLazySum = 8192.0f;      // a lane's per-tile sum of exponentials above this forces a new reference maximum

struct AttnArgs {
  const __bf16* q;
  const __bf16* k;
  const __bf16* v;
  const __bf16* k_t;          // sparse: P-outer copies of k and v read by temporal heads instead of k, v; may be null
  const __bf16* v_t;
  void* o;                    // bf16 [B,H,N,D] (dense, sparse) or fp32 [3][BH][t][D] (profile)
  const uint8_t* labels;      // sparse: per-head pattern, may be null
  const int32_t* row_ptr[2];
  const int32_t* col_idx[2];
  const int32_t* rows;        // profile: sampled rows
  const int32_t* order_t;     // profile: indices into rows[], grouped by in-frame position (temporal variant)
  int t;                      // profile: number of sampled rows
  int nsplit;                 // profile: key ranges the unmasked pass is cut into
  int rows_per_group;         // profile: sampled rows per workgroup (the groups are balanced)
  float2* stats;              // profile: (reference maximum, row sum) per (key range, head, row)
  int N, nk, BH;
  int nqt;                    // workgroups per head: query tiles (dense, sparse) or ceil(t / rows per workgroup) (profile)
  int reverse_q;              // process query tiles last-to-first (heavy text-suffix tiles first)
  int total;                  // logical workgroups
  int qo_token_order;         // sparse: q is read and o written in token order also for temporal heads
  float scale_log2;           // softmax scale * log2(e)
  int off, video_end, F, P, w_s, w_t, sink;
};

// Lanes l and l^32 own the two halves of one query's keys.  v_permlane32_swap with
// both operands equal returns {x[l % 32], x[32 + l % 32]} in every lane, so the
// combined maximum / sum needs no LDS traffic.
__device__ __forceinline__ float both_halves_max(float x) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float both_halves_sum(float x) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

}  // namespace attn

}  // namespace svg
