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
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) i16x4 lds_i16x4;   // operand type of the transposing LDS read

enum Mode { kDense = 0, kSparse = 1, kProfile = 2, kSparseExact = 3, kSparseGather = 4 };

constexpr int kCodeDrop = 0x7fffffff;   // key beyond N: never kept
constexpr int kCodeKeep = 0x7ffffffe;   // text key / sink key: kept by every query
constexpr float kNegBig = -1.0e30f;     // finite stand-in for -inf as the initial row maximum
constexpr float kLazySum = 8192.0f;      // a lane's per-tile sum of exponentials above this forces a new reference maximum

// --------------------------------------------------------------------------------------------
// Dispatch order of the block-sparse passes.
//
// Workgroups are dealt round-robin to the 8 XCDs (blockIdx.x % 8) and start in the order of
// blockIdx.x / 8, so what a workgroup works on decides both which L2 serves it and when it
// starts.  Two things make query tiles unequal: a tile that holds a text row keeps every key
// tile (its list is many times longer than the others'), and the lists of the two patterns
// differ in length while the labels, known on the device only, say which heads have which.
//  * Heavy tiles (those with a text row) start first on every XCD, a head's heavy tiles on
//    one XCD (they stream the same K and V), heads dealt to the XCDs in turn.  Started last
//    they would run on alone after every other workgroup of their XCD has finished.
//  * The other tiles of all heads with the same label form one sequence (head after head,
//    ascending query tiles); every XCD takes one contiguous eighth of the spatial sequence
//    and one of the temporal sequence, the one with the longer lists first.  Each XCD so gets
//    the same share of both kinds of work whatever the labels are, and consecutive workgroups
//    of an XCD still are nearby query tiles of one head (overlapping key windows).
//  * Inside the part of a head that an XCD takes, the query tiles are dispatched with a stride:
//    0, r, 2r, ..., then 1, r+1, ...  A workgroup walks its list one key tile per tile time, the
//    window of query tile g + 1 lies BM / BN = 2 key tiles above that of g, and in steady state
//    a place on the XCD frees up every T / slots tile times (T: tiles per list, slots: resident
//    workgroups).  With r = T / (2 slots) the next workgroup starts exactly as much later as
//    its window lies higher, so all workgroups of the XCD read the same key tile at the same
//    time and L2 serves all but one of them.  r is rounded, at least 1, per label (the lists of
//    the two patterns differ in length).
// With more than 256 heads the labels are not looked at: one sequence in head order.
// --------------------------------------------------------------------------------------------
constexpr int kWideLabelWords = 4;     // label classes are formed for up to 64 * kWideLabelWords heads

struct SparseOrder {
  int g_lo;    // a head's query tiles without a text row are [g_lo, g_lo + nl)
  int nl;
  int nh;      // tiles with a text row per head (the others, ascending)
  int hmax;    // workgroups per XCD reserved for them
  int slots;   // workgroups resident on one XCD (sets the stride, see above)
};

inline SparseOrder sparse_order(int BH, int nqt, int BM, int off, int video_end, int N, int slots) {
  SparseOrder so;
  const int lo = off > 0 ? (off + BM - 1) / BM : 0;
  int hi = video_end < N ? video_end / BM : nqt;
  so.g_lo = lo < nqt ? lo : nqt;
  if (hi < so.g_lo) hi = so.g_lo;
  so.nl = hi - so.g_lo;
  so.nh = nqt - so.nl;
  so.hmax = so.nh * ((BH + 7) / 8);
  so.slots = slots;
  return so;
}

// grid size: an XCD's two eighths together hold at most floor(BH nl / 8) + 2 tiles
inline unsigned sparse_grid(const SparseOrder& so, int BH) {
  return 8u * (unsigned)(so.hmax + (long long)BH * so.nl / 8 + 2);
}

// Which (head, query tile, pattern) does this workgroup take?  false: none.  For a tile without
// text rows, cl is its index in its label's sequence and head_cl0 the index of its head's first
// tile there (cl = -1 for a heavy tile).  Every value returned is the same in all lanes.
// (LW: 64-head words of label bits; the kernels are built for 1 and for kWideLabelWords, and the
// launcher takes the wide form only when there are more than 64 heads)
template <int LW>
__device__ __forceinline__ bool sparse_slot(const SparseOrder so, const int BH, const uint8_t* labels,
                                            const int32_t* rp_s, const int32_t* rp_t, int& bh, int& grp,
                                            int& pat, int& cl, int& head_cl0) {
  const int xcd = blockIdx.x & 7, loc = blockIdx.x >> 3;
  const int lane = threadIdx.x & 63;
  // the labels as bit masks, 64 heads per word (bit = temporal)
  const bool classed = labels != nullptr && BH <= 64 * LW;
  unsigned long long m[LW];
  int nT = 0;
#pragma unroll
  for (int w = 0; w < LW; ++w) {
    const int h = 64 * w + lane;
    m[w] = classed && 64 * w < BH ? __builtin_amdgcn_ballot_w64(h < BH && labels[h < BH ? h : 0] != 0) : 0ull;
    nT += __builtin_popcountll(m[w]);
  }
  auto label_bit = [&](int h) -> int {
    unsigned long long word = m[0];
#pragma unroll
    for (int w = 1; w < LW; ++w) word = (h >> 6) == w ? m[w] : word;
    return (int)((word >> (h & 63)) & 1);
  };
  cl = -1;
  head_cl0 = 0;
  if (loc < so.hmax) {
    const int hh = loc / so.nh, j = loc - hh * so.nh;
    bh = xcd + 8 * hh;
    if (bh >= BH) return false;
    grp = j < so.g_lo ? j : j + so.nl;
    pat = classed ? label_bit(bh) : (labels ? labels[bh] != 0 : 0);
    return true;
  }
  if (so.nl == 0) return false;
  int l = loc - so.hmax;
  const int nS = BH - nT;
  int first = nS == 0;            // the label whose sequence comes first
  const int nnz_s = nS > 0 ? rp_s[so.g_lo + so.nl] - rp_s[so.g_lo] : 0;      // list tiles of a head's light query tiles
  const int nnz_t = nT > 0 ? rp_t[so.g_lo + so.nl] - rp_t[so.g_lo] : 0;
  if (nT > 0 && nS > 0) first = nnz_t > nnz_s;
  const int nA = first ? nT : nS;
  const long long NA = (long long)nA * so.nl, NB = (long long)(BH - nA) * so.nl;
  const int a0 = (int)((xcd * NA) >> 3), a1 = (int)(((xcd + 1) * NA) >> 3);
  const int b0 = (int)((xcd * NB) >> 3), b1 = (int)(((xcd + 1) * NB) >> 3);
  int c = first;
  if (l < a1 - a0) {
    cl = a0 + l;
  } else {
    l -= a1 - a0;
    if (l >= b1 - b0) return false;
    cl = b0 + l;
    c = !first;
  }
  const int kth = cl / so.nl;
  head_cl0 = kth * so.nl;
  {
    // strided order inside the part [s0, s1) of this head that lies in the XCD's chunk
    const int c0 = c == first ? a0 : b0, c1 = c == first ? a1 : b1;
    const int s0 = max(c0, head_cl0), s1 = min(c1, head_cl0 + so.nl);
    const int len = s1 - s0;
    const int tiles_per_list = (c ? nnz_t : nnz_s) / so.nl;
    const int r = min(16, (tiles_per_list + so.slots) / (2 * so.slots));      // round(T / (2 slots))
    int idx = cl - s0;
    if (r > 1 && len > r) {
      int p = 0;
      for (; p < r; ++p) {        // which pass (p, p + r, p + 2r, ...) the idx-th workgroup belongs to
        const int in_pass = (len - p + r - 1) / r;
        if (idx < in_pass) break;
        idx -= in_pass;
      }
      idx = p + idx * r;
    }
    cl = s0 + idx;
  }
  grp = so.g_lo + (cl - head_cl0);
  if (classed) {
    // the kth head (from 0) with label c: find its word, then its bit
    bh = 0;
    int before = 0;
    bool found = false;
#pragma unroll
    for (int w = 0; w < LW; ++w) {
      const int left = BH - 64 * w;
      const unsigned long long valid = left >= 64 ? ~0ull : left > 0 ? (1ull << left) - 1 : 0ull;
      const unsigned long long cm = c ? m[w] : ~m[w] & valid;
      const int cnt = __builtin_popcountll(cm);
      if (!found && kth < before + cnt) {
        const int rank = __builtin_popcountll(cm & ((1ull << lane) - 1));
        const unsigned long long hit = __builtin_amdgcn_ballot_w64(((cm >> lane) & 1) != 0 && rank == kth - before);
        bh = 64 * w + __builtin_ctzll(hit);
        found = true;
      }
      before += cnt;
    }
    pat = c;
  } else {
    bh = kth;
    pat = labels ? labels[bh] != 0 : 0;
  }
  return true;
}

struct AttnArgs {
  const __bf16* q;
  const __bf16* k;
  const __bf16* v;
  const __bf16* k_t;          // sparse: P-outer copies of k and v read by temporal heads instead of k, v; may be null
  const __bf16* v_t;
  void* o;                    // bf16 [B,H,N,D] (dense, sparse) or fp32 [3][BH][t][D] (profile)
  const uint8_t* labels;      // sparse: per-head pattern, may be null
  const int32_t* row_table;   // gathering sparse form: token row of every P-outer row, nk * BN entries
  const int32_t* row_ptr[2];
  const int32_t* col_idx[2];
  const int32_t* rows;        // profile: sampled rows
  const int32_t* order_t;     // profile: indices into rows[], grouped by in-frame position (temporal variant)
  int t;                      // profile: number of sampled rows
  ProfilePlan plan;           // profile: parts of the unmasked pass and of the masked passes
  int rows_per_group;         // profile: sampled rows per workgroup (the groups are balanced)
  float2* stats;              // profile: (reference maximum, row sum) per (output slot, head, row)
  int N, nk, BH;
  int nqt;                    // workgroups per head: query tiles (dense, sparse) or ceil(t / rows per workgroup) (profile)
  SparseOrder so;             // sparse: which workgroup takes which (head, query tile)
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
