// FlashAttention-style forward kernels for gfx950 (MI355X): dense attention, the
// block-sparse pass over a kept-tile list (Sec. 4.3), and the three masked passes
// of online profiling over sampled query rows (Alg. 1, Sec. 4.1).
//
// One workgroup owns one query tile of one head; each of its NW wavefronts owns 32
// query rows and all BN keys of the current key tile.  Both matrix products are
// computed TRANSPOSED with v_mfma_f32_32x32x16_bf16:
//     S^T = K Q^T      (A = K tile from LDS,  B = Q^T held in registers)
//     O^T += V^T P^T   (A = V^T from LDS,     B = P^T taken from S^T's registers)
// In the 32x32 accumulator layout a lane holds ONE query column (lane % 32) and 16
// key rows, so the online-softmax row maximum and row sum are per-lane register
// reductions plus one exchange between lane l and lane l+32, the rescale factor is
// one scalar per lane, and the exponentiated S^T registers are, after bf16
// packing, exactly the B operand of the second product: register pair (2kk, 2kk+1)
// of a 32-key block holds keys {16kk+4g+j} and {16kk+8+4g+j}, j<4, g = lane/32,
// and the V^T operand is fetched for the same keys, so no cross-lane shuffle and no
// LDS round trip is needed for P.
//
// K and V tiles are staged global -> registers -> LDS, double buffered, with the
// loads of tile j+1 in flight while tile j is computed (one barrier per tile).
// K is stored row-major with an XOR swizzle of its 16-byte pieces (conflict-free
// ds_read_b128 of the A operand).  V is transposed in registers on the way in
// (v_perm_b32) to a [key/4][d][4 keys] layout, so the V^T operand of 8 keys at one
// d is two ds_read_b64.
//
// Softmax runs in fp32 with base-2 exponentials (scale * log2 e folded into one
// FMA per element); P is rounded to bf16 for the second product; accumulation is
// fp32; the running sum uses the unrounded P.
#include "svg_internal.h"

namespace svg {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

enum Mode { kDense = 0, kSparse = 1, kProfile = 2 };

constexpr int kCodeDrop = 0x7fffffff;   // key beyond N: never kept
constexpr int kCodeKeep = 0x7ffffffe;   // text key / sink key: kept by every query
constexpr float kNegBig = -1.0e30f;     // finite stand-in for -inf as the initial row maximum
constexpr float kLazyLog2 = 8.0f;       // exponentials may reach 2^8 before the maximum is raised

struct AttnArgs {
  const __bf16* q;
  const __bf16* k;
  const __bf16* v;
  void* o;                    // bf16 [B,H,N,D] (dense, sparse) or fp32 [3][BH][t][D] (profile)
  const uint8_t* labels;      // sparse: per-head pattern, may be null
  const int32_t* row_ptr[2];
  const int32_t* col_idx[2];
  const int32_t* rows;        // profile: sampled rows
  int t;                      // profile: number of sampled rows
  int N, nk, BH;
  int nqt;                    // query tiles per head (profile: ceil(t/BM))
  int reverse_q;              // process query tiles last-to-first (heavy text-suffix tiles first)
  int total;                  // logical workgroups
  float scale_log2;           // softmax scale * log2(e)
  float lazy_tau;             // raw-logit margin below which the running maximum is not raised
  int off, video_end, F, P, w_s, w_t, sink;
};

template <int D>
__device__ __forceinline__ int k_swizzle(int key) {
  // XOR applied to the 16-byte piece index of a K row so that the 16 lanes served
  // together by a ds_read_b128 hit 16 different 4-bank groups.
  return D == 128 ? (key & 15) : ((key >> 1) & 7);
}

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

template <int D, int NW, int BN, int MODE>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void attn_kernel(AttnArgs a) {
  constexpr int BM = 32 * NW;
  constexpr int THREADS = 64 * NW;
  constexpr int CPR = D / 8;             // 16-byte pieces per row
  constexpr int KB = BN / 32;            // 32-key blocks per tile
  constexpr int DS = D / 16;             // k-steps of the first product
  constexpr int DB = D / 32;             // 32-row blocks of O^T
  constexpr int K_PIECES = BN * CPR;
  constexpr int K_PER_THREAD = K_PIECES / THREADS;
  constexpr int V_UNITS = (BN / 4) * CPR;   // a unit = 4 keys x 8 channels
  constexpr int V_PER_THREAD = (V_UNITS + THREADS - 1) / THREADS;
  constexpr int K_BYTES = BN * D * 2;
  // V^T staging: [key/4][d][4 keys] with each key-group row padded by 128 bytes, so
  // that the two half-waves of a ds_read_b64 (key groups kg and kg+1) fall on
  // different banks.
  constexpr int V_ROW = D * 8 + 128;
  constexpr int V_BYTES = (BN / 4) * V_ROW;
  constexpr int STAGE_BYTES = K_BYTES + V_BYTES;
  static_assert(K_PIECES % THREADS == 0, "K tile must split evenly over the workgroup");

  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * STAGE_BYTES];
  __shared__ __attribute__((aligned(16))) int key_code[MODE == kProfile ? 2 * BN : 4];

  // ---- which (head, query tile) is this workgroup?  Consecutive logical ids are
  // placed on the same XCD (workgroups are dealt round-robin over the 8 XCDs), so
  // the query tiles that stream the same K/V share one L2.
  const int per_xcd = (a.total + 7) >> 3;
  const int lid = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (lid >= a.total) return;
  int bh, qt, variant = 0;
  if (MODE == kProfile) {
    bh = lid / (3 * a.nqt);
    const int rem = lid - bh * 3 * a.nqt;
    variant = rem / a.nqt;
    qt = rem - variant * a.nqt;
  } else {
    bh = lid / a.nqt;
    qt = lid - bh * a.nqt;
    if (a.reverse_q) qt = a.nqt - 1 - qt;
  }

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int g = lane >> 5;       // which half of the wavefront
  const int r = lane & 31;       // query column within the wave / row of the A operand

  const size_t head = (size_t)bh * a.N;
  const __bf16* kh = a.k + head * D;
  const __bf16* vh = a.v + head * D;

  // ---- tile range
  int j0 = 0, j1 = a.nk;
  const int32_t* cols = nullptr;
  if (MODE == kSparse) {
    const int pat = a.labels ? (a.labels[bh] != 0) : 0;
    const int32_t* rp = a.row_ptr[pat];
    cols = a.col_idx[pat];
    j0 = rp[qt];
    j1 = rp[qt + 1];
  }

  // ---- this lane's query row
  const int qslot = qt * BM + wave * 32 + r;        // row of the tile (profile: index into rows[])
  int qrow;
  if (MODE == kProfile) qrow = a.rows[min(qslot, a.t - 1)];
  else qrow = min(qslot, a.N - 1);

  // profile: window test  (unsigned)(code - lo) <= span  ||  code == kCodeKeep
  int win_lo = 0;
  unsigned win_span = 0x7ffffffeu;
  if (MODE == kProfile && variant != 0) {
    const bool text_q = qrow < a.off || qrow >= a.video_end;
    if (!text_q) {
      const int vq = qrow - a.off;
      const int fq = vq / a.P;
      const int c = variant == 1 ? fq : vq - fq * a.P;
      const int w = variant == 1 ? a.w_s : a.w_t;
      win_lo = c - w;
      win_span = 2u * (unsigned)w;
    }
  }

  // ---- Q^T as the B operand: lane (g, r) holds Q[qrow][16 s + 8 g .. +8]
  bf16x8 qreg[DS];
  {
    const __bf16* qp = a.q + (head + qrow) * D + g * 8;
#pragma unroll
    for (int s = 0; s < DS; ++s) qreg[s] = *reinterpret_cast<const bf16x8*>(qp + s * 16);
  }

  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[db][e] = 0.f;
  float m_run = kNegBig;   // running row maximum (raw logits, before scaling)
  float l_run = 0.f;       // this lane's share of the running row sum

  u32x4 kst[K_PER_THREAD];
  u32x4 vst[V_PER_THREAD][4];

  auto load_tile = [&](int col) {
    const int key0 = col * BN;
#pragma unroll
    for (int i = 0; i < K_PER_THREAD; ++i) {
      const int u = tid + i * THREADS;
      const int key = u / CPR, c = u % CPR;
      const int krow = min(key0 + key, a.N - 1);
      kst[i] = *reinterpret_cast<const u32x4*>(kh + (size_t)krow * D + c * 8);
    }
#pragma unroll
    for (int i = 0; i < V_PER_THREAD; ++i) {
      const int u = tid + i * THREADS;
      if (V_UNITS % THREADS == 0 || u < V_UNITS) {
        const int kg = u / CPR, c = u % CPR;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          const int vrow = min(key0 + kg * 4 + rr, a.N - 1);
          vst[i][rr] = *reinterpret_cast<const u32x4*>(vh + (size_t)vrow * D + c * 8);
        }
      }
    }
  };

  auto store_tile = [&](int buf, int col) {
    unsigned char* kb = lds + buf * STAGE_BYTES;
    unsigned char* vb = kb + K_BYTES;
#pragma unroll
    for (int i = 0; i < K_PER_THREAD; ++i) {
      const int u = tid + i * THREADS;
      const int key = u / CPR, c = u % CPR;
      *reinterpret_cast<u32x4*>(kb + key * (D * 2) + ((c ^ k_swizzle<D>(key)) << 4)) = kst[i];
    }
#pragma unroll
    for (int i = 0; i < V_PER_THREAD; ++i) {
      const int u = tid + i * THREADS;
      if (V_UNITS % THREADS == 0 || u < V_UNITS) {
        const int kg = u / CPR, c = u % CPR;
        // 4 keys x 8 channels -> 8 channels x 4 keys: piece w holds channels 2w, 2w+1
        u32x4 outv[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          outv[w][0] = __builtin_amdgcn_perm(vst[i][1][w], vst[i][0][w], 0x05040100u);  // d=2w  : keys 0,1
          outv[w][1] = __builtin_amdgcn_perm(vst[i][3][w], vst[i][2][w], 0x05040100u);  // d=2w  : keys 2,3
          outv[w][2] = __builtin_amdgcn_perm(vst[i][1][w], vst[i][0][w], 0x07060302u);  // d=2w+1: keys 0,1
          outv[w][3] = __builtin_amdgcn_perm(vst[i][3][w], vst[i][2][w], 0x07060302u);  // d=2w+1: keys 2,3
        }
        // the four 16-byte pieces of this thread's 64-byte segment go to slots
        // w ^ ((c >> 1) & 3): 8 consecutive lanes then cover all banks once
        unsigned char* dst = vb + kg * V_ROW + c * 64;
        const int sw = (c >> 1) & 3;
#pragma unroll
        for (int w = 0; w < 4; ++w) *reinterpret_cast<u32x4*>(dst + ((w ^ sw) << 4)) = outv[w];
      }
    }
    if (MODE == kProfile && tid < BN) {
      const int key = col * BN + tid;
      int code;
      if (key >= a.N) {
        code = kCodeDrop;
      } else if (variant == 0 || key < a.off || key >= a.video_end) {
        code = kCodeKeep;
      } else {
        const int vk = key - a.off;
        const int fk = vk / a.P;
        code = variant == 1 ? fk : vk - fk * a.P;
        if (a.sink && fk == 0) code = kCodeKeep;
      }
      key_code[buf * BN + tid] = code;
    }
  };

  if (j0 < j1) {
    load_tile(MODE == kSparse ? cols[j0] : j0);
    store_tile(0, MODE == kSparse ? cols[j0] : j0);
  }
  __syncthreads();

  int buf = 0;
  const int swz = k_swizzle<D>(r);   // tile rows kb*32 + r: swizzle depends on r only
  // byte offset of channel d = 32 db + r inside a V^T key-group row (see store_tile)
  int v_off[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) {
    const int d = db * 32 + r;
    const int c = d >> 3, w = (d >> 1) & 3;
    v_off[db] = c * 64 + ((w ^ ((c >> 1) & 3)) << 4) + (d & 1) * 8;
  }
  for (int j = j0; j < j1; ++j) {
    const int col = MODE == kSparse ? cols[j] : j;
    const bool has_next = j + 1 < j1;
    int next_col = 0;
    if (has_next) {
      next_col = MODE == kSparse ? cols[j + 1] : j + 1;
      load_tile(next_col);
    }

    const unsigned char* kbuf = lds + buf * STAGE_BYTES;
    const unsigned char* vbuf = kbuf + K_BYTES;

    // ---- S^T = K Q^T
    f32x16 sacc[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[kb][e] = 0.f;
      const unsigned char* krow = kbuf + (kb * 32 + r) * (D * 2);
#pragma unroll
      for (int s = 0; s < DS; ++s) {
        const bf16x8 ka = *reinterpret_cast<const bf16x8*>(krow + (((2 * s + g) ^ swz) << 4));
        sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[s], sacc[kb], 0, 0, 0);
      }
    }

    // ---- masking.  sacc[kb][4 i + jj] belongs to key  col*BN + 32 kb + 8 i + 4 g + jj.
    if (MODE == kProfile) {
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const i32x4 cc = *reinterpret_cast<const i32x4*>(&key_code[buf * BN + kb * 32 + 8 * i + 4 * g]);
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            const bool keep = ((unsigned)(cc[jj] - win_lo) <= win_span) || cc[jj] == kCodeKeep;
            if (!keep) sacc[kb][4 * i + jj] = -INFINITY;
          }
        }
    } else if ((col + 1) * BN > a.N) {
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int jj = 0; jj < 4; ++jj)
            if (col * BN + kb * 32 + 8 * i + 4 * g + jj >= a.N) sacc[kb][4 * i + jj] = -INFINITY;
    }

    // ---- online softmax: one query per lane
    float m_loc = sacc[0][0];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) m_loc = fmaxf(m_loc, sacc[kb][e]);
    m_loc = both_halves_max(m_loc);
    // The running maximum is only raised when some row's tile maximum exceeds it by
    // more than 2^kLazyLog2 after scaling; until then the exponentials are taken
    // against the older (smaller) reference and may reach 2^kLazyLog2, which fp32
    // sums and bf16 weights hold without loss.  The result is mathematically the
    // same softmax; the O^T and row-sum rescale is skipped on most tiles.
    if (__builtin_amdgcn_ballot_w64(m_loc > m_run + a.lazy_tau) != 0) {
      const float m_new = fmaxf(m_run, m_loc);
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * a.scale_log2);
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[db][e] *= alpha;
    }
    const float mc = m_run * a.scale_log2;
    float l_loc = 0.f;
    bf16x8 pb[KB][2];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        f32x8 p;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][8 * kk + e], a.scale_log2, -mc));
          l_loc += p[e];
        }
        pb[kb][kk] = __builtin_convertvector(p, bf16x8);
      }
    l_run += l_loc;

    // ---- O^T += V^T P^T
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        const int kg = kb * 8 + kk * 4 + g;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const unsigned char* vp = vbuf + kg * V_ROW + v_off[db];
          const bf16x4 lo = *reinterpret_cast<const bf16x4*>(vp);
          const bf16x4 hi = *reinterpret_cast<const bf16x4*>(vp + 2 * V_ROW);
          const bf16x8 va = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[kb][kk], oacc[db], 0, 0, 0);
        }
      }

    if (has_next) store_tile(buf ^ 1, next_col);
    __syncthreads();
    buf ^= 1;
  }

  // ---- epilogue: normalise and store.  oacc[db][4 i + jj] = O[query r][32 db + 8 i + 4 g + jj]
  const float l_tot = both_halves_sum(l_run);
  const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
  if (MODE == kProfile) {
    if (qslot < a.t) {
      float* op = static_cast<float*>(a.o) + (((size_t)variant * a.BH + bh) * a.t + qslot) * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          f32x4 x;
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) x[jj] = oacc[db][4 * i + jj] * inv;
          *reinterpret_cast<f32x4*>(op + db * 32 + 8 * i + 4 * g) = x;
        }
    }
  } else {
    if (qslot < a.N) {
      __bf16* op = static_cast<__bf16*>(a.o) + (head + qslot) * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          f32x4 x;
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) x[jj] = oacc[db][4 * i + jj] * inv;
          *reinterpret_cast<bf16x4*>(op + db * 32 + 8 * i + 4 * g) = __builtin_convertvector(x, bf16x4);
        }
    }
  }
}

// MSE_s, MSE_t and the label of one head from the three profiled outputs
// (Alg. 1, last block).  One workgroup per head, fixed-order tree reduction.
__global__ __launch_bounds__(256) void profile_finalize_kernel(const float* ws, int BH, int t, int D,
                                                               uint8_t* labels, float* mse) {
  const int bh = blockIdx.x;
  const size_t per = (size_t)t * D;
  const float* of = ws + ((size_t)0 * BH + bh) * per;
  const float* os = ws + ((size_t)1 * BH + bh) * per;
  const float* ot = ws + ((size_t)2 * BH + bh) * per;
  float acc_s = 0.f, acc_t = 0.f;
  for (size_t e = threadIdx.x; e < per; e += 256) {
    const float f = of[e];
    const float ds = f - os[e], dt = f - ot[e];
    acc_s = __builtin_fmaf(ds, ds, acc_s);
    acc_t = __builtin_fmaf(dt, dt, acc_t);
  }
  __shared__ float red_s[256], red_t[256];
  red_s[threadIdx.x] = acc_s;
  red_t[threadIdx.x] = acc_t;
  __syncthreads();
  for (int step = 128; step > 0; step >>= 1) {
    if (threadIdx.x < step) {
      red_s[threadIdx.x] += red_s[threadIdx.x + step];
      red_t[threadIdx.x] += red_t[threadIdx.x + step];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const float ms = red_s[0] / (float)per, mt = red_t[0] / (float)per;
    if (mse) {
      mse[2 * bh + 0] = ms;
      mse[2 * bh + 1] = mt;
    }
    labels[bh] = ms < mt ? SVG_HEAD_SPATIAL : SVG_HEAD_TEMPORAL;
  }
}

template <int D, int NW, int BN, int MODE>
int launch_one(const AttnArgs& a, hipStream_t stream) {
  const unsigned grid = (unsigned)(((a.total + 7) / 8) * 8);
  (void)hipGetLastError();   // drop any stale error left by earlier runtime calls of the process
  hipLaunchKernelGGL((attn_kernel<D, NW, BN, MODE>), dim3(grid), dim3(64 * NW), 0, stream, a);
  return hip_status(hipGetLastError());
}

template <int MODE>
int dispatch(const Geo& g, const AttnArgs& a, hipStream_t stream) {
  if (g.bm == 128) {
    return g.D == 128 ? launch_one<128, 4, 64, MODE>(a, stream) : launch_one<64, 4, 64, MODE>(a, stream);
  }
  return g.D == 128 ? launch_one<128, 1, 32, MODE>(a, stream) : launch_one<64, 1, 32, MODE>(a, stream);
}

AttnArgs base_args(const Geo& g, const void* q, const void* k, const void* v, void* o) {
  AttnArgs a = {};
  a.q = static_cast<const __bf16*>(q);
  a.k = static_cast<const __bf16*>(k);
  a.v = static_cast<const __bf16*>(v);
  a.o = o;
  a.N = g.N; a.nk = g.nk; a.BH = g.B * g.H;
  a.scale_log2 = g.scale * 1.4426950408889634f;
  a.lazy_tau = kLazyLog2 / a.scale_log2;
  a.off = g.off; a.video_end = g.video_end; a.F = g.F; a.P = g.P;
  a.w_s = g.w_s; a.w_t = g.w_t; a.sink = g.sink;
  return a;
}

}  // namespace

int launch_attention(const Geo& g, const void* q, const void* k, const void* v, void* o,
                     const uint8_t* labels, const int32_t* row_ptr_s, const int32_t* col_idx_s,
                     const int32_t* row_ptr_t, const int32_t* col_idx_t, bool sparse,
                     hipStream_t stream) {
  AttnArgs a = base_args(g, q, k, v, o);
  a.labels = labels;
  a.row_ptr[0] = row_ptr_s; a.col_idx[0] = col_idx_s;
  a.row_ptr[1] = row_ptr_t; a.col_idx[1] = col_idx_t;
  a.nqt = g.nq;
  a.total = a.BH * a.nqt;
  // query tiles holding text rows keep every key tile: start them first
  a.reverse_q = (sparse && g.T > 0 && !g.text_first) ? 1 : 0;
  return sparse ? dispatch<kSparse>(g, a, stream) : dispatch<kDense>(g, a, stream);
}

int launch_profile(const Geo& g, const void* q, const void* k, const void* v, const int32_t* rows,
                   int t, uint8_t* labels, float* mse, float* workspace, hipStream_t stream) {
  AttnArgs a = base_args(g, q, k, v, workspace);
  a.rows = rows;
  a.t = t;
  a.nqt = (t + g.bm - 1) / g.bm;
  a.total = 3 * a.BH * a.nqt;
  int rc = dispatch<kProfile>(g, a, stream);
  if (rc != SVG_OK) return rc;
  (void)hipGetLastError();   // drop any stale error left by earlier runtime calls of the process
  hipLaunchKernelGGL(profile_finalize_kernel, dim3(a.BH), dim3(256), 0, stream, workspace, a.BH, t,
                     g.D, labels, mse);
  return hip_status(hipGetLastError());
}

}  // namespace svg
