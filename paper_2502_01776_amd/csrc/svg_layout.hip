// Layout transformation between the F-outer and P-outer token orders (Sec. 4.2,
// Fig. 4) and its inverse.  Pure data movement, HBM-bound: each thread moves one
// 16-byte piece of a token row, a group of D/8 consecutive lanes moves one whole
// row (128 or 256 contiguous bytes on both the read and the write side), so every
// access is a full, aligned cache line.  Writes are linear in the output; reads
// are row-granular gathers.
#include "svg_internal.h"

namespace svg {

namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte piece

constexpr int kThreads = 256;
constexpr int kRowsPerThread = 4;   // independent 16-byte loads in flight per thread

struct LayoutArgs {
  const u32x4* in[2];      // one or two tensors per launch (blockIdx.z)
  u32x4* out[2];
  const uint8_t* labels;
  int temporal_only;       // heads labelled spatial are left alone (their slots of `out` are not written)
  int N, off, video_end, F, P, sink;
  int chunks_log2;     // log2(D/8): 16-byte pieces per row
  int inverse;
};

// Source row (in `in`) of output row n.
__device__ __forceinline__ int source_row(const LayoutArgs& a, int n) {
  if (n < a.off || n >= a.video_end) return n;         // text rows stay
  const unsigned v = (unsigned)(n - a.off);
  if (!a.inverse)              // out is in the transformed order: row v  <-  that row's token
    return a.off + (int)transformed_to_token(v, (unsigned)a.F, (unsigned)a.P, a.sink);
  return a.off + (int)token_to_transformed(v, (unsigned)a.F, (unsigned)a.P, a.sink);   // out is F-outer
}

__global__ __launch_bounds__(kThreads) void layout_kernel(LayoutArgs a) {
  const int bh = blockIdx.y;
  const int cpr = 1 << a.chunks_log2;
  const int rows_per_pass = kThreads >> a.chunks_log2;
  const int lane_row = threadIdx.x >> a.chunks_log2;
  const int c = threadIdx.x & (cpr - 1);
  const bool permute = a.labels == nullptr || a.labels[bh] == SVG_HEAD_TEMPORAL;
  if (a.temporal_only && !permute) return;
  const u32x4* in = a.in[blockIdx.z];
  u32x4* out = a.out[blockIdx.z];
  const size_t head = (size_t)bh * a.N;
  const int row0 = blockIdx.x * (rows_per_pass * kRowsPerThread) + lane_row;

  u32x4 val[kRowsPerThread];
#pragma unroll
  for (int i = 0; i < kRowsPerThread; ++i) {
    const int n = row0 + i * rows_per_pass;
    if (n < a.N) {
      const int src = permute ? source_row(a, n) : n;
      val[i] = __builtin_nontemporal_load(&in[((head + src) << a.chunks_log2) + c]);
    }
  }
#pragma unroll
  for (int i = 0; i < kRowsPerThread; ++i) {
    const int n = row0 + i * rows_per_pass;
    if (n < a.N) __builtin_nontemporal_store(val[i], &out[((head + n) << a.chunks_log2) + c]);
  }
}

}  // namespace

int launch_layout(const Geo& g, const void* in, void* out, const void* in2, void* out2, const uint8_t* labels,
                  bool inverse, bool temporal_only, hipStream_t stream) {
  LayoutArgs a;
  a.in[0] = static_cast<const u32x4*>(in);
  a.out[0] = static_cast<u32x4*>(out);
  a.in[1] = static_cast<const u32x4*>(in2);
  a.out[1] = static_cast<u32x4*>(out2);
  a.temporal_only = temporal_only ? 1 : 0;
  a.labels = labels;
  a.N = g.N; a.off = g.off; a.video_end = g.video_end; a.F = g.F; a.P = g.P; a.sink = g.sink;
  a.chunks_log2 = g.D == 128 ? 4 : 3;
  a.inverse = inverse ? 1 : 0;
  const int rows_per_block = (kThreads >> a.chunks_log2) * kRowsPerThread;
  dim3 grid((g.N + rows_per_block - 1) / rows_per_block, g.B * g.H, in2 ? 2 : 1);
  if (grid.y > 65535u) return SVG_ERR_UNSUPPORTED;
  (void)hipGetLastError();   // drop any stale error left by earlier runtime calls of the process
  hipLaunchKernelGGL(layout_kernel, grid, dim3(kThreads), 0, stream, a);
  return hip_status(hipGetLastError());
}

}  // namespace svg
