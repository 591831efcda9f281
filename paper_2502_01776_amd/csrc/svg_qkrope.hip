// QK-norm and rotary position embedding of q or k in one pass (Sec. 4.3 "Efficient kernel
// customization", Table 2).  HBM-bound: every element is read once and written once.
//
// The paper's point is the small head dimension (64 or 128): a token's head vector is
// only 128 or 256 bytes, far less than a wavefront.  Here D/8 consecutive lanes (8 or 16)
// own one token row, 16 bytes each, so a 64-lane wavefront covers 8 or 4 rows with full
// 16-byte accesses; the row statistics are reduced inside those lane groups with cross-lane
// moves (no LDS); the rotation of the interleaved channel pairs needs no other lane at all.
// A workgroup keeps its tokens and walks over the heads, so the angle tables and the norm
// weights are fetched once per token and reused for every head.
#include "svg_internal.h"

namespace svg {

namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

struct NormRopeArgs {
  const u32x4* in;
  u32x4* out;
  const float* weight;   // [D] or null
  const float* bias;     // [D] or null (LayerNorm form only)
  const float* cos;      // [F*P, D/2] or null: no rotation
  const float* sin;
  int N, BH, off, video_end;
  int norm, pairing;
  float eps;
  int heads_per_block;
};

template <int W>
__device__ __forceinline__ float group_sum(float x) {   // sum over W consecutive lanes (W = 8 or 16)
#pragma unroll
  for (int m = W / 2; m > 0; m >>= 1) x += __shfl_xor(x, m, W);
  return x;
}

template <int D>
__global__ __launch_bounds__(256) void norm_rope_kernel(NormRopeArgs a) {
  constexpr int CPR = D / 8;            // lanes per token row
  constexpr int ROWS = 256 / CPR;       // rows per workgroup
  const int c = threadIdx.x % CPR;      // this lane's channels: 8 c .. 8 c + 7
  const int n = blockIdx.x * ROWS + threadIdx.x / CPR;
  if (n >= a.N) return;                 // whole lane groups leave together
  const int h0 = blockIdx.y * a.heads_per_block;
  const int h1 = min(a.BH, h0 + a.heads_per_block);

  float w[8], b[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    w[e] = a.weight ? a.weight[8 * c + e] : 1.0f;
    b[e] = (a.bias && a.norm == SVG_NORM_LAYER) ? a.bias[8 * c + e] : 0.0f;
  }
  const bool rotate = a.cos != nullptr && n >= a.off && n < a.video_end;
  // interleaved pairing: pair p of this lane is channels (8 c + 2 p, 8 c + 2 p + 1), table column 4 c + p
  // half pairing: channel i < D/2 pairs with i + D/2, which the lane CPR/2 further on holds;
  //               both lanes use table columns 8 (c mod CPR/2) .. + 7
  float cs[8], sn[8];
  if (rotate) {
    const size_t base = (size_t)(n - a.off) * (D / 2);
    if (a.pairing == SVG_ROPE_INTERLEAVED) {
      const f32x4 c4 = *reinterpret_cast<const f32x4*>(a.cos + base + 4 * c);
      const f32x4 s4 = *reinterpret_cast<const f32x4*>(a.sin + base + 4 * c);
#pragma unroll
      for (int p = 0; p < 4; ++p) { cs[p] = c4[p]; sn[p] = s4[p]; }
    } else {
      const int col = 8 * (c % (CPR / 2));
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const f32x4 c4 = *reinterpret_cast<const f32x4*>(a.cos + base + col + 4 * q);
        const f32x4 s4 = *reinterpret_cast<const f32x4*>(a.sin + base + col + 4 * q);
#pragma unroll
        for (int p = 0; p < 4; ++p) { cs[4 * q + p] = c4[p]; sn[4 * q + p] = s4[p]; }
      }
    }
  }
  const float sign = c < CPR / 2 ? -1.0f : 1.0f;       // half pairing: a cos - b sin | b cos + a sin

  const size_t row = (size_t)n * CPR + c;
  const size_t head_stride = (size_t)a.N * CPR;
  auto process = [&](const u32x4 raw, int h) {
    float x[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      x[2 * e] = __uint_as_float(raw[e] << 16);
      x[2 * e + 1] = __uint_as_float(raw[e] & 0xffff0000u);
    }
    if (a.norm != SVG_NORM_NONE) {
      float mu = 0.f;
      if (a.norm == SVG_NORM_LAYER) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) s += x[e];
        mu = group_sum<CPR>(s) * (1.0f / D);
      }
      float ss = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        x[e] -= mu;
        ss = __builtin_fmaf(x[e], x[e], ss);
      }
      const float r = 1.0f / sqrtf(group_sum<CPR>(ss) * (1.0f / D) + a.eps);
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = __builtin_fmaf(x[e] * r, w[e], b[e]);
    }
    if (rotate) {
      if (a.pairing == SVG_ROPE_INTERLEAVED) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const float u = x[2 * p], v = x[2 * p + 1];
          x[2 * p] = u * cs[p] - v * sn[p];
          x[2 * p + 1] = v * cs[p] + u * sn[p];
        }
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float other = __shfl_xor(x[e], CPR / 2, CPR);
          x[e] = __builtin_fmaf(sign * other, sn[e], x[e] * cs[e]);
        }
      }
    }
    u32x4 o;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const f32x4 v4 = {x[4 * e], x[4 * e + 1], x[4 * e + 2], x[4 * e + 3]};
      const bf16x4 h4 = __builtin_convertvector(v4, bf16x4);
      const uint2 bits = *reinterpret_cast<const uint2*>(&h4);
      o[2 * e] = bits.x;
      o[2 * e + 1] = bits.y;
    }
    __builtin_nontemporal_store(o, &a.out[h * head_stride + row]);
  };
  // four heads at a time, their loads issued together
  constexpr int kUnroll = 4;
  for (int h = h0; h < h1; h += kUnroll) {
    u32x4 raw[kUnroll];
#pragma unroll
    for (int j = 0; j < kUnroll; ++j)
      if (h + j < h1) raw[j] = __builtin_nontemporal_load(&a.in[(h + j) * head_stride + row]);
#pragma unroll
    for (int j = 0; j < kUnroll; ++j)
      if (h + j < h1) process(raw[j], h + j);
  }
}

}  // namespace

int launch_norm_rope(const Geo& g, const void* x, void* y, int norm, const float* weight, const float* bias,
                     float eps, const float* cos, const float* sin, int pairing, hipStream_t stream) {
  NormRopeArgs a;
  a.in = static_cast<const u32x4*>(x);
  a.out = static_cast<u32x4*>(y);
  a.weight = weight; a.bias = bias; a.cos = cos; a.sin = sin;
  a.N = g.N; a.BH = g.B * g.H; a.off = g.off; a.video_end = g.video_end;
  a.norm = norm; a.pairing = pairing; a.eps = eps;
  const int rows = 256 / (g.D / 8);
  const unsigned gx = (unsigned)((g.N + rows - 1) / rows);
  // enough workgroups to fill the chip, and at most 8 heads per workgroup (measured best: the
  // tables are still reused 8 times, and the workgroups running at one time stay closer in memory)
  int splits = (int)((2048 + gx - 1) / gx);
  splits = splits < (a.BH + 7) / 8 ? (a.BH + 7) / 8 : splits;
  splits = splits > a.BH ? a.BH : splits;
  a.heads_per_block = (a.BH + splits - 1) / splits;
  const unsigned gy = (unsigned)((a.BH + a.heads_per_block - 1) / a.heads_per_block);
  if (gy > 65535u) return SVG_ERR_UNSUPPORTED;
  (void)hipGetLastError();
  if (g.D == 128) hipLaunchKernelGGL(norm_rope_kernel<128>, dim3(gx, gy), dim3(256), 0, stream, a);
  else hipLaunchKernelGGL(norm_rope_kernel<64>, dim3(gx, gy), dim3(256), 0, stream, a);
  return hip_status(hipGetLastError());
}

}  // namespace svg
