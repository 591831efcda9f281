// Measurement aids (no part of the method): what the bf16 matrix cores of this GPU sustain
// when nothing else limits them.  The attention kernels are priced against the published
// 2.5 PFLOP/s, which assumes 2.4 GHz; under a sustained matrix load with operands that look
// like real data (random signs and mantissas) the chip runs at a lower clock, and these
// loops show what is then left.  Form 0 issues only v_mfma_f32_32x32x16_bf16, operands in
// registers, two wavefronts per SIMD, four independent accumulators per wavefront.  Form 1
// adds, per product, what the D = 128 attention kernel needs per product besides the
// product: one 1 KB operand read from LDS, and for one score per lane one FMA, one
// exponential, one addition and half a bf16 pack -- and nothing else (no staging, no
// barriers, no global memory), so it bounds that kernel design from above.  Form 2 is the
// same for the D = 64 kernel: three wavefronts per SIMD, and per product the softmax
// instructions of TWO scores per lane (half the products per score): two FMAs, two
// exponentials, one bf16 pack and one packed dot product for the row sum.
#include "svg_internal.h"

namespace svg {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int kProbeThreads = 256;
constexpr int kProbeLds = 72 * 1024;          // keeps two workgroups (two wavefronts per SIMD) on a CU
constexpr int kProbeLds3 = 48 * 1024;         // form 2: three workgroups on a CU
constexpr int kProductsPerIteration = 16;
constexpr unsigned kOperandMask = 65535;      // operands: 65536 pieces of 16 bytes = 1 MiB

template <int FORM>
__global__ __launch_bounds__(kProbeThreads, FORM == 2 ? 3 : 2) void probe_kernel(const u32x4* data, float* sink, int iters) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[FORM == 2 ? kProbeLds3 : kProbeLds];
  const int tid = threadIdx.x, lane = tid & 63;
  for (int i = tid; i < 2048; i += kProbeThreads)
    reinterpret_cast<u32x4*>(lds)[i] = data[(blockIdx.x * 2048 + i) & kOperandMask];
  __syncthreads();
  bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = __builtin_bit_cast(bf16x8, data[(tid * 8 + i) & kOperandMask]);
    b[i] = __builtin_bit_cast(bf16x8, data[(tid * 8 + 4 + i + blockIdx.x) & kOperandMask]);
  }
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  float f[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) f[i] = (lane + i) * 1e-3f;
  unsigned packed = lane;
  float rowsum = 0.f;
  const unsigned char* base = lds + lane * 16;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < kProductsPerIteration; ++m) {
      bf16x8 av = a[m & 3];
      if (FORM != 0) av = *reinterpret_cast<const bf16x8*>(base + (m * 1024 + (it & 1) * 16384));
      __builtin_amdgcn_sched_barrier(0);
      acc[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, b[(m >> 2) & 3], acc[m & 3], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (FORM == 1) {
        f[m & 7] = __builtin_fmaf(f[m & 7], 0.999f, 1e-3f);
        f[(m + 1) & 7] = __builtin_amdgcn_exp2f(-f[(m + 1) & 7]);      // (negated: the chain stays finite)
        f[(m + 2) & 7] += f[(m + 3) & 7];
        if (m & 1) {
          const f32x2 two = {f[m & 7], f[(m + 1) & 7]};
          packed ^= __builtin_bit_cast(unsigned, __builtin_convertvector(two, bf16x2));
        }
      }
      if (FORM == 2) {
        f[m & 7] = __builtin_fmaf(f[m & 7], 0.999f, 1e-3f);
        f[(m + 4) & 7] = __builtin_fmaf(f[(m + 4) & 7], 0.999f, 1e-3f);
        f[(m + 1) & 7] = __builtin_amdgcn_exp2f(-f[(m + 1) & 7]);
        f[(m + 5) & 7] = __builtin_amdgcn_exp2f(-f[(m + 5) & 7]);
        const f32x2 two = {f[(m + 1) & 7], f[(m + 5) & 7]};
        const bf16x2 pair = __builtin_convertvector(two, bf16x2);
        const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
        rowsum = __builtin_amdgcn_fdot2_f32_bf16(pair, ones, rowsum, false);
      }
    }
  }
  float s = __uint_as_float(packed) + rowsum;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += f[i];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  sink[blockIdx.x * kProbeThreads + tid] = s;
}

}  // namespace

}  // namespace svg

extern "C" int svg_probe_mfma_bf16(int form, int32_t workgroups, int32_t iterations, const void* operands,
                                   float* sink, double* flop_out, void* stream) {
  if (form < 0 || form > 2 || workgroups <= 0 || workgroups > 65536 || iterations <= 0 || !operands || !sink)
    return SVG_ERR_INVALID_ARG;
  if (svg::misaligned16(operands) || svg::misaligned16(sink)) return SVG_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  (void)hipGetLastError();
  if (form == 0)
    hipLaunchKernelGGL((svg::probe_kernel<0>), dim3(workgroups), dim3(svg::kProbeThreads), 0, s,
                       static_cast<const svg::u32x4*>(operands), sink, iterations);
  else if (form == 1)
    hipLaunchKernelGGL((svg::probe_kernel<1>), dim3(workgroups), dim3(svg::kProbeThreads), 0, s,
                       static_cast<const svg::u32x4*>(operands), sink, iterations);
  else
    hipLaunchKernelGGL((svg::probe_kernel<2>), dim3(workgroups), dim3(svg::kProbeThreads), 0, s,
                       static_cast<const svg::u32x4*>(operands), sink, iterations);
  if (flop_out)
    *flop_out = (double)workgroups * (svg::kProbeThreads / 64) * (double)iterations * svg::kProductsPerIteration *
                (2.0 * 32 * 32 * 16);
  return svg::hip_status(hipGetLastError());
}
