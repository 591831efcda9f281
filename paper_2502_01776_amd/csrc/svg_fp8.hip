// FP8 variant of the block-sparse attention pass (Sec. 4.3 "Quantization", Sec. 5.2) for
// gfx950 (MI355X): q, k, v quantised to 8-bit floating point (OCP E4M3, one scale per head
// and tensor, scale = max|x| / 448), both matrix products on the FP8 matrix instruction
// v_mfma_f32_32x32x64_f8f6f4 (twice the bf16 rate, half the operand bytes), fp32
// accumulation and softmax, bf16 output.  Head dimension 128 and 128 x 64 tiles only (the
// paper applies FP8 only there: with head dimension 64 it gains nothing, Sec. 5.2).
//
// Two steps:
//   svg_fp8_quantize         one pass for the per-head maxima, one pass that converts and, for
//                            temporal heads, applies the layout transformation of Sec. 4.2 to
//                            k and v on the way (so the bf16 layout passes are not needed);
//                            v is written as ready-made LDS images of its 64-key tiles.
//   svg_sparse_attn_fp8_fwd  the attention kernel.  Same decomposition as the bf16 kernel
//                            (one workgroup per query tile, 32 query rows per wavefront, both
//                            products transposed so that a lane owns one query), but a whole
//                            64-key tile is ONE k-step of the second product, the attention
//                            weights are packed four to a register (E4M3 after scaling by 2^8,
//                            which puts weights down to 2^-17 of the row maximum inside the
//                            format's range), and the row sums come out of the matrix unit too:
//                            a ninth product per tile multiplies the weights with a block of
//                            ones, so the denominator is the sum of the ROUNDED weights, the
//                            result is an exact weighted mean of v rows, and 32 additions per
//                            lane and tile leave the VALU, which is the busiest unit here.
#include "svg_attn_common.h"

namespace svg {

namespace {

using namespace attn;

typedef int i32x8 __attribute__((ext_vector_type(8)));

constexpr int kD = 128;                    // head dimension = bytes of a quantised row
constexpr int kBM = 128, kBN = 64;
constexpr int kNoTile = 0x7fffffff;
constexpr int kCohort = 64;
constexpr unsigned kRsrcFlags = 0x00020000u;
constexpr float kE4M3Max = 448.0f;
constexpr float kWeightShift = 8.0f;       // attention weights are stored as 2^8 * exp(s - max) <= 256 < 448

// LDS image of a key tile.  K: 64 rows of 128 bytes, padded by 16 so that the 16 lanes a
// ds_read_b128 serves together (consecutive keys, same channel piece) fall on different banks.
constexpr int kKRow = kD + 16;
constexpr int kKBytes = kBN * kKRow;
// V^T: [half-wave g][channel d][32 key slots]; slot i = 4 j + c of half-wave g is key
// 32 (j / 4) + 8 (j % 4) + 4 g + c, the key whose weight sits in byte c of register j of
// the packed weights.  The two 16-byte halves of a channel's 32 bytes are swapped for
// channels with bit 3 set, which makes the operand reads conflict-free.
constexpr int kVBytes = 2 * kD * 32;
constexpr int kStageBytes = kKBytes + kVBytes;
constexpr int kTileBytes = kBN * kD;       // bytes of one tile in k8 and in v8t (8192 each)

__host__ __device__ constexpr int v_slot_key(int g, int i) {
  return 32 * ((i >> 2) >> 2) + 8 * ((i >> 2) & 3) + 4 * g + (i & 3);
}

// --------------------------------------------------------------------------------------------
// Quantisation
// --------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fp8_zero_kernel(unsigned* p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0u;
}

constexpr int kAmaxPieces = 16;            // 16-byte pieces per thread

// Largest magnitude of each (tensor, head): bf16 magnitudes compare like their bit patterns.
__global__ __launch_bounds__(256) void fp8_amax_kernel(const u32x4* q, const u32x4* k, const u32x4* v,
                                                       unsigned long long pieces_per_head, unsigned* amax,
                                                       int BH) {
  const int bh = blockIdx.y, tensor = blockIdx.z;
  const u32x4* src = (tensor == 0 ? q : tensor == 1 ? k : v) + (size_t)bh * pieces_per_head;
  const unsigned long long base = (unsigned long long)blockIdx.x * (256 * kAmaxPieces) + threadIdx.x;
  unsigned m = 0;
#pragma unroll 4
  for (int i = 0; i < kAmaxPieces; ++i) {
    const unsigned long long u = base + (unsigned long long)i * 256;
    if (u < pieces_per_head) {
      const u32x4 x = __builtin_nontemporal_load(&src[u]);
#pragma unroll
      for (int w = 0; w < 4; ++w) m = max(m, max(x[w] & 0x7fffu, (x[w] >> 16) & 0x7fffu));
    }
  }
  __shared__ unsigned red[256];
  red[threadIdx.x] = m;
  __syncthreads();
  for (unsigned step = 128; step > 0; step >>= 1) {
    if (threadIdx.x < step) red[threadIdx.x] = max(red[threadIdx.x], red[threadIdx.x + step]);
    __syncthreads();
  }
  if (threadIdx.x == 0) atomicMax(&amax[tensor * BH + bh], red[0] << 16);    // as fp32 bits
}

struct QuantArgs {
  const u32x4* in[3];          // q, k, v: bf16 [B,H,N,128] in token order
  unsigned char* q8;           // [B,H,N,128]
  unsigned char* k8;           // [B,H,nk*64,128], rows beyond N zero
  unsigned char* v8t;          // [B,H,nk][8192]: LDS images
  float* scales;               // [3][BH]
  const unsigned* amax;        // [3][BH] fp32 bits
  const uint8_t* labels;
  int N, BH, off, video_end, F, P, sink;
};

// One workgroup converts one 64-row tile of one head of one tensor.
__global__ __launch_bounds__(256) void fp8_quantize_kernel(QuantArgs a) {
  const int tile = blockIdx.x, bh = blockIdx.y, tensor = blockIdx.z;
  const int tid = threadIdx.x;
  const float amax = __uint_as_float(a.amax[tensor * a.BH + bh]);
  const float scale = amax > 0.f ? amax / kE4M3Max : 1.0f;
  if (tile == 0 && tid == 0) a.scales[tensor * a.BH + bh] = scale;
  const float inv_scale = 1.0f / scale;      // codes = nearest even of x * (1 / scale), both in fp32
  // k and v of temporal heads are written in P-outer order: row m holds token off + f P + p
  // with m = off + p F + f (Sec. 4.2); q stays in token order (the attention kernel gathers it)
  const bool permute = tensor != 0 && a.labels != nullptr && a.labels[bh] == SVG_HEAD_TEMPORAL;
  const u32x4* src = a.in[tensor] + (size_t)bh * a.N * (kD / 8);

  __shared__ __attribute__((aligned(16))) unsigned char tile_bytes[kBN * (kD + 4)];   // v only: [key][d], rows padded
  uint2 packed[4];
  int row_of[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int u = tid + 256 * i;                 // piece: row u / 16, channels 8 (u % 16) ..
    const int rr = u >> 4, c = u & 15;
    const int m = tile * kBN + rr;
    row_of[i] = m;
    u32x4 x = {0u, 0u, 0u, 0u};
    if (m < a.N) {
      int s = m;
      if (permute && m >= a.off && m < a.video_end) {
        s = a.off + (int)transformed_to_token((unsigned)(m - a.off), (unsigned)a.F, (unsigned)a.P, a.sink);
      }
      x = __builtin_nontemporal_load(&src[(size_t)s * (kD / 8) + c]);
    }
    unsigned out[2];
#pragma unroll
    for (int w = 0; w < 2; ++w) {
      float y[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const unsigned word = x[2 * w + (e >> 1)];
        const float val = __uint_as_float((e & 1) ? (word & 0xffff0000u) : (word << 16));
        y[e] = fminf(fmaxf(val * inv_scale, -kE4M3Max), kE4M3Max);
      }
      int pk = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], 0, false);
      pk = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], pk, true);
      out[w] = (unsigned)pk;
    }
    packed[i] = make_uint2(out[0], out[1]);
  }
  if (tensor != 2) {
    unsigned char* dst = tensor == 0 ? a.q8 + (size_t)bh * a.N * kD
                                     : a.k8 + ((size_t)bh * gridDim.x) * kTileBytes;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int u = tid + 256 * i;
      if (tensor == 1 || row_of[i] < a.N)
        *reinterpret_cast<uint2*>(dst + (size_t)row_of[i] * kD + (u & 15) * 8) = packed[i];
    }
    return;
  }
  // v: transpose through LDS into the tile's image
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int u = tid + 256 * i;
    unsigned char* p = tile_bytes + (u >> 4) * (kD + 4) + (u & 15) * 8;
    *reinterpret_cast<unsigned*>(p) = packed[i].x;
    *reinterpret_cast<unsigned*>(p + 4) = packed[i].y;
  }
  __syncthreads();
  const int g = tid >> 7, d = tid & 127;
  unsigned img[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    unsigned w = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) w |= (unsigned)tile_bytes[v_slot_key(g, 4 * j + c) * (kD + 4) + d] << (8 * c);
    img[j] = w;
  }
  unsigned char* dst = a.v8t + ((size_t)bh * gridDim.x + tile) * kTileBytes + g * (kD * 32) + d * 32;
  const int sw = (d >> 3) & 1;
  *reinterpret_cast<u32x4*>(dst + 16 * sw) = u32x4{img[0], img[1], img[2], img[3]};
  *reinterpret_cast<u32x4*>(dst + 16 * (1 - sw)) = u32x4{img[4], img[5], img[6], img[7]};
}

// --------------------------------------------------------------------------------------------
// Attention
// --------------------------------------------------------------------------------------------
struct Fp8Args {
  const unsigned char* q8;
  const unsigned char* k8;
  const unsigned char* v8t;
  const float* scales;         // [3][BH]: q, k, v
  __bf16* o;                   // [B,H,N,128] bf16, token order
  const uint8_t* labels;
  const int32_t* row_ptr[2];
  const int32_t* col_idx[2];
  int N, nk, BH, nqt;
  SparseOrder so;              // which workgroup takes which (head, query tile)
  float scale_log2;            // softmax scale * log2(e), before the quantisation scales
  int off, video_end, F, P, sink, w_s, w_t;
};

template <int LW>
__global__ __launch_bounds__(256, 2) void attn_fp8_kernel(Fp8Args a) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * kStageBytes];

  // heavy query tiles first, then an eighth of each label's sequence of tiles (the same
  // dispatch order as the bf16 kernel)
  int bh = 0, grp = 0, pat = 0, cl = -1, head_cl0 = 0;
  if (!sparse_slot<LW>(a.so, a.BH, a.labels, a.row_ptr[0], a.row_ptr[1], bh, grp, pat, cl, head_cl0)) return;
  bh = __builtin_amdgcn_readfirstlane(bh);
  grp = __builtin_amdgcn_readfirstlane(grp);
  pat = __builtin_amdgcn_readfirstlane(pat);
  cl = __builtin_amdgcn_readfirstlane(cl);
  head_cl0 = __builtin_amdgcn_readfirstlane(head_cl0);

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, r = lane & 31;

  const size_t tiles_head = (size_t)bh * a.nk;
  const unsigned char* kh = a.k8 + tiles_head * kTileBytes;
  const unsigned char* vh = a.v8t + tiles_head * kTileBytes;

  // this lane's query: position qslot in the order the tile list refers to; for a temporal
  // head that is token off + f P + p with qslot = off + p F + f (q and o stay in token order)
  const int qslot = grp * kBM + wave * 32 + r;
  const int qrow = min(qslot, a.N - 1);
  int io_row = qrow;
  if (pat && qrow >= a.off && qrow < a.video_end)
    io_row = a.off + (int)transformed_to_token((unsigned)(qrow - a.off), (unsigned)a.F, (unsigned)a.P, a.sink);
  i32x8 qreg[2];       // lane (g, r) holds channels 64 s + 32 g .. + 32 of its query
  {
    const unsigned char* qp = a.q8 + ((size_t)bh * a.N + io_row) * kD + g * 32;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const i32x4 lo = *reinterpret_cast<const i32x4*>(qp + s * 64);
      const i32x4 hi = *reinterpret_cast<const i32x4*>(qp + s * 64 + 16);
      qreg[s] = i32x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    }
  }
  // logits in units of log2: s_raw * c with the two quantisation scales folded in
  const float c_log2 = a.scale_log2 * a.scales[bh] * a.scales[a.BH + bh];
  const float v_scale = a.scales[2 * a.BH + bh];

  // ---- tile cursor: the query tile's list row, walked cyclically from the cohort's common
  // starting tile (same scheme as the bf16 kernel)
  const int32_t* rp = a.row_ptr[pat];
  const int32_t* cols = a.col_idx[pat];
  const int lbeg = __builtin_amdgcn_readfirstlane(rp[grp]);
  const int lend = __builtin_amdgcn_readfirstlane(rp[grp + 1]);
  int lj = lbeg, lleft = lend - lbeg;
  // cohort size by geometry: the largest power of two for which the anchor lies inside every
  // member's key window; short windows start at their own first tile
  const int win_tiles = (int)min((pat ? (2LL * a.w_t + 1) * a.F : (2LL * a.w_s + 1) * a.P) / kBN, 1LL << 20);
  int cs = kCohort;
  while (cs > 1 && (cs - 1) * (kBM / kBN) >= win_tiles) cs >>= 1;
  if (lleft > 1 && cl >= 0 && cs >= 8) {
    const int first_video_tile = (a.off + kBN - 1) / kBN;
    const int top = a.so.g_lo + min(cl | (cs - 1), head_cl0 + a.so.nl - 1) - head_cl0;
    const int c_first = cols[lbeg], c_last = cols[lend - 1];
    int anchor = -1;
    for (int j = rp[top], e = min(rp[top + 1], rp[top] + 8); j < e; ++j)
      if (cols[j] >= first_video_tile) { anchor = cols[j]; break; }
    if (anchor >= c_first && anchor <= c_last) {
      int lo = 0, hi = lleft;
      const int from_front = anchor - c_first;
      if (from_front < lleft && cols[lbeg + from_front] == anchor) {
        lo = from_front;
      } else {
        while (lo < hi) {
          const int mid = (lo + hi) >> 1;
          if (cols[lbeg + mid] < anchor) lo = mid + 1; else hi = mid;
        }
      }
      if (lo < lleft && cols[lbeg + lo] == anchor) lj = lbeg + lo;
    }
    lj = __builtin_amdgcn_readfirstlane(lj);
  }
  int lane_zero = 0;
  asm volatile("" : "+v"(lane_zero));
  int pend = kNoTile;
  auto fetch_begin = [&]() { pend = lleft > 0 ? cols[lj + lane_zero] : kNoTile; };
  auto fetch_end = [&]() -> int {
    if (lleft <= 0) return kNoTile;
    const int c = __builtin_amdgcn_readfirstlane(pend);
    --lleft;
    if (++lj >= lend) lj = lbeg;
    return c;
  };
  auto next_tile = [&]() -> int {
    fetch_begin();
    return fetch_end();
  };

  // ---- staging: both tile images are 8 KB = two 16-byte pieces per thread each
  u32x4 kst[2], vst[2];
  auto load_tile = [&](int col_any) {
    const int tile = __builtin_amdgcn_readfirstlane(col_any);
    const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned char*>(kh + (size_t)tile * kTileBytes), 0, kTileBytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned char*>(vh + (size_t)tile * kTileBytes), 0, kTileBytes, kRsrcFlags);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      kst[i] = __builtin_amdgcn_raw_buffer_load_b128(rk, (tid + 256 * i) * 16, 0, 0);
      vst[i] = __builtin_amdgcn_raw_buffer_load_b128(rv, (tid + 256 * i) * 16, 0, 0);
    }
  };
  auto store_tile = [&](int buf) {
    unsigned char* kb = lds + buf * kStageBytes;
    unsigned char* vb = kb + kKBytes;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int u = tid + 256 * i;
      *reinterpret_cast<u32x4*>(kb + (u >> 3) * kKRow + ((u & 7) << 4)) = kst[i];
      *reinterpret_cast<u32x4*>(vb + (u << 4)) = vst[i];
    }
  };

  // ---- per-lane operand addresses
  const int k_rd = r * kKRow + 32 * g;
  const int sw = (r >> 3) & 1;
  const int v_rd_lo = g * (kD * 32) + r * 32 + 16 * sw;
  const int v_rd_hi = g * (kD * 32) + r * 32 + 16 * (1 - sw);
  auto read32 = [](const unsigned char* lo, const unsigned char* hi) -> i32x8 {
    const i32x4 x = *reinterpret_cast<const i32x4*>(lo);
    const i32x4 y = *reinterpret_cast<const i32x4*>(hi);
    return i32x8{x[0], x[1], x[2], x[3], y[0], y[1], y[2], y[3]};
  };

  f32x16 oacc[4], lacc;
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    lacc[e] = 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db) oacc[db][e] = 0.f;
  }
  i32x8 ones;          // 32 x E4M3 1.0
#pragma unroll
  for (int j = 0; j < 8; ++j) ones[j] = 0x38383838;
  asm volatile("" : "+v"(ones));
  float m_run = kNegBig;     // running row maximum, raw logits

  int col = next_tile(), col1 = next_tile(), col2 = next_tile(), col3 = next_tile();
  if (col != kNoTile) {
    load_tile(col);
    store_tile(0);
  }
  __syncthreads();
  asm volatile("" ::"v"(qreg[0]), "v"(qreg[1]));

  int buf = 0;
  const bool ragged = (a.N % kBN) != 0;

  while (col != kNoTile) {
    const int next_col = col1;
    col1 = col2;
    col2 = col3;
    fetch_begin();
    if (next_col != kNoTile) load_tile(next_col);

    const unsigned char* kbuf = lds + buf * kStageBytes;
    const unsigned char* vbuf = kbuf + kKBytes;

    // ---- S^T = K Q^T: two 32-key blocks x two 64-channel steps
    i32x8 opnd[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const unsigned char* p = kbuf + (i >> 1) * 32 * kKRow + (i & 1) * 64 + k_rd;
      opnd[i] = read32(p, p + 16);
    }
    f32x16 sacc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[kb][e] = 0.f;
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      __builtin_amdgcn_sched_barrier(0);
      sacc[i >> 1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(opnd[i], qreg[i & 1], sacc[i >> 1], 0, 0, 0, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_setprio(0);
    // V^T operands of the second product: requested before the softmax
#pragma unroll
    for (int db = 0; db < 4; ++db) opnd[db] = read32(vbuf + db * 1024 + v_rd_lo, vbuf + db * 1024 + v_rd_hi);

    // ---- softmax
    if (ragged && col == a.nk - 1) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (col * kBN + 32 * kb + 8 * (e >> 2) + 4 * g + (e & 3) >= a.N) sacc[kb][e] = -INFINITY;
    }
    float tmax = sacc[0][0];
#pragma unroll
    for (int e = 1; e < 16; ++e) tmax = fmaxf(tmax, sacc[0][e]);
#pragma unroll
    for (int e = 0; e < 16; ++e) tmax = fmaxf(tmax, sacc[1][e]);
    tmax = both_halves_max(tmax);
    if (__builtin_amdgcn_ballot_w64(tmax > m_run) != 0) {      // some row of the wavefront has a new maximum
      const float m_new = fmaxf(m_run, tmax);
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c_log2);
      m_run = m_new;
      lacc[0] *= alpha;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[db][e] *= alpha;
    }
    const float mc = m_run * c_log2 - kWeightShift;
    i32x8 pb;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float p[4];
#pragma unroll
      for (int c = 0; c < 4; ++c)
        p[c] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[j >> 2][4 * (j & 3) + c], c_log2, -mc));
      // (the first conversion writes the low half of its destination and keeps the rest: giving it
      // a value that dies here as the "rest" saves a register clear; the second one fills the high half)
      int w = __builtin_amdgcn_cvt_pk_fp8_f32(p[0], p[1], (int)__float_as_uint(p[0]), false);
      pb[j] = __builtin_amdgcn_cvt_pk_fp8_f32(p[2], p[3], w, true);
    }

    // ---- O^T += V^T P^T (one 64-key step per 32-channel block), row sums += 1 P^T
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      __builtin_amdgcn_sched_barrier(0);
      oacc[db] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(opnd[db], pb, oacc[db], 0, 0, 0, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    lacc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ones, pb, lacc, 0, 0, 0, 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(0);

    if (next_col != kNoTile) store_tile(buf ^ 1);
    col3 = fetch_end();
    __syncthreads();
    buf ^= 1;
    col = next_col;
  }

  // ---- epilogue: oacc[db][4 i + jj] = O[query r][32 db + 8 i + 4 g + jj]; lacc[0] = row sum
  const float l_tot = lacc[0];
  const float inv = l_tot > 0.f ? v_scale / l_tot : 0.f;
  if (qslot < a.N) {
    __bf16* op = a.o + ((size_t)bh * a.N + io_row) * kD;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        f32x4 x;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) x[jj] = oacc[db][4 * i + jj] * inv;
        *reinterpret_cast<bf16x4*>(op + db * 32 + 8 * i + 4 * g) = __builtin_convertvector(x, bf16x4);
      }
  }
}

}  // namespace

int launch_fp8_quantize(const Geo& g, const void* q, const void* k, const void* v, const uint8_t* labels,
                        void* q8, void* k8, void* v8t, float* scales, hipStream_t stream) {
  const int BH = g.B * g.H;
  if (BH > 65535) return SVG_ERR_UNSUPPORTED;
  unsigned* amax = reinterpret_cast<unsigned*>(scales + 3 * BH);
  (void)hipGetLastError();
  hipLaunchKernelGGL(fp8_zero_kernel, dim3((3 * BH + 255) / 256), dim3(256), 0, stream, amax, 3 * BH);
  int rc = hip_status(hipGetLastError());
  if (rc != SVG_OK) return rc;
  const unsigned long long pieces = (unsigned long long)g.N * (kD / 8);
  const unsigned chunks = (unsigned)((pieces + 256 * kAmaxPieces - 1) / (256 * kAmaxPieces));
  hipLaunchKernelGGL(fp8_amax_kernel, dim3(chunks, BH, 3), dim3(256), 0, stream, static_cast<const u32x4*>(q),
                     static_cast<const u32x4*>(k), static_cast<const u32x4*>(v), pieces, amax, BH);
  rc = hip_status(hipGetLastError());
  if (rc != SVG_OK) return rc;
  QuantArgs a;
  a.in[0] = static_cast<const u32x4*>(q);
  a.in[1] = static_cast<const u32x4*>(k);
  a.in[2] = static_cast<const u32x4*>(v);
  a.q8 = static_cast<unsigned char*>(q8);
  a.k8 = static_cast<unsigned char*>(k8);
  a.v8t = static_cast<unsigned char*>(v8t);
  a.scales = scales;
  a.amax = amax;
  a.labels = labels;
  a.N = g.N; a.BH = BH; a.off = g.off; a.video_end = g.video_end; a.F = g.F; a.P = g.P; a.sink = g.sink;
  hipLaunchKernelGGL(fp8_quantize_kernel, dim3(g.nk, BH, 3), dim3(256), 0, stream, a);
  return hip_status(hipGetLastError());
}

int launch_fp8_attention(const Geo& g, const void* q8, const void* k8, const void* v8t, const float* scales,
                         void* o, const uint8_t* labels, const int32_t* row_ptr_s, const int32_t* col_idx_s,
                         const int32_t* row_ptr_t, const int32_t* col_idx_t, hipStream_t stream) {
  Fp8Args a = {};
  a.q8 = static_cast<const unsigned char*>(q8);
  a.k8 = static_cast<const unsigned char*>(k8);
  a.v8t = static_cast<const unsigned char*>(v8t);
  a.scales = scales;
  a.o = static_cast<__bf16*>(o);
  a.labels = labels;
  a.row_ptr[0] = row_ptr_s; a.col_idx[0] = col_idx_s;
  a.row_ptr[1] = row_ptr_t; a.col_idx[1] = col_idx_t;
  a.N = g.N; a.nk = g.nk; a.BH = g.B * g.H;
  a.nqt = g.nq;
  // (no stride in the dispatch order: this kernel starts the query tiles of a cohort at a common key tile
  // instead, which measured 0.6-1.8 % faster here than the stride with or without that start)
  a.so = sparse_order(a.BH, a.nqt, kBM, g.off, g.video_end, g.N, 1 << 24);
  a.scale_log2 = g.scale * 1.4426950408889634f;
  a.off = g.off; a.video_end = g.video_end; a.F = g.F; a.P = g.P; a.sink = g.sink;
  a.w_s = g.w_s; a.w_t = g.w_t;
  const unsigned grid = sparse_grid(a.so, a.BH);
  (void)hipGetLastError();
  if (a.BH > 64) hipLaunchKernelGGL(attn_fp8_kernel<kWideLabelWords>, dim3(grid), dim3(256), 0, stream, a);
  else hipLaunchKernelGGL(attn_fp8_kernel<1>, dim3(grid), dim3(256), 0, stream, a);
  return hip_status(hipGetLastError());
}

}  // namespace svg
