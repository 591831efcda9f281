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

// What the LDS of one compute unit delivers for the access patterns of the attention kernels at
// head dimension 128: one workgroup of `waves` wavefronts issues `iters` x 16 LDS instructions of
// one kind per wavefront (the loaded values are consumed by empty statements, so nothing but the LDS
// instructions and their waits is timed) and every wavefront writes the shader clocks that took to
// ticks[wave].
//   form 0  ds_read_b128 of a K operand (rows padded by 16 bytes, 32 rows x 16 bytes per half wave)
//   form 1  ds_read_b64_tr_b16 of a V^T operand from row-major rows whose 32-byte slots are
//           XOR-swizzled with the row's two low bits (the layout the kernels stage V in)
//   form 2  the same read from plain row-major rows
//   form 3  ds_write_b128 in the staging pattern (16 lanes write one row)
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) i16x4 lds_i16x4;
typedef int i32x4 __attribute__((ext_vector_type(4)));
constexpr int kLdsProbeInstructions = 16;

template <int FORM>
__global__ __launch_bounds__(1024) void lds_probe_kernel(long long* ticks, int* sink, int iters) {
  constexpr int D = 128, V_ROW = D * 2, K_ROW = D * 2 + 16;
  __shared__ __attribute__((aligned(16))) unsigned char lds[64 * K_ROW];
  const int tid = threadIdx.x, lane = tid & 63;
  for (int i = tid; i < 64 * K_ROW / 4; i += blockDim.x) reinterpret_cast<unsigned*>(lds)[i] = i * 2654435761u;
  __syncthreads();
  const int g = lane >> 5, r = lane & 31;
  const int s = lane & 15, j = s >> 2, h = (lane >> 4) & 1;
  const int swizzle = FORM == 1 ? (2 * j) ^ (j >> 1) : 0;
  int v_off[4];
#pragma unroll
  for (int db = 0; db < 4; ++db) v_off[db] = (4 * g + j) * V_ROW + (((2 * db + h) ^ swizzle) << 5) + ((s & 3) << 3);
  const int k_off = r * K_ROW + (g << 4);
  const i32x4 payload = {tid, lane, g, r};
  __syncthreads();
  const long long t0 = clock64();
  for (int it = 0; it < iters; ++it) {
    // the array's address goes into the statement so that it counts as read and written there:
    // loads are not hoisted out of the loop and the stores of an iteration are not dropped
    asm volatile("" ::"v"(lds) : "memory");
    // all instructions of an iteration are issued before the first result is waited for
    i32x4 wide[FORM == 0 ? kLdsProbeInstructions : 1];
    i16x4 narrow[FORM == 1 || FORM == 2 ? kLdsProbeInstructions : 1];
#pragma unroll
    for (int u = 0; u < kLdsProbeInstructions; ++u) {
      if (FORM == 0) {        // operands (kb, s) of the first product: 2 key blocks x 8 channel steps
        wide[u] = *reinterpret_cast<const i32x4*>(lds + k_off + ((u & 1) * 32) * K_ROW + (u >> 1) * 32);
      } else if (FORM == 1 || FORM == 2) {   // operands (step, half, db) of the second product
        narrow[u] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (lds_i16x4*)(lds + v_off[u & 3] + ((u >> 2) & 1) * 8 * V_ROW + (u >> 3) * 16 * V_ROW));
      } else {                // 16 lanes write one row; 4 rows per instruction, 64 rows in all
        *reinterpret_cast<i32x4*>(lds + ((lane >> 4) + 4 * u) * K_ROW + ((lane & 15) << 4)) = payload;
      }
    }
#pragma unroll
    for (int u = 0; u < kLdsProbeInstructions; ++u) {
      if (FORM == 0) asm volatile("" ::"v"(wide[u]));
      if (FORM == 1 || FORM == 2) asm volatile("" ::"v"(narrow[u]));
    }
  }
  asm volatile("" ::"v"(lds) : "memory");
  const long long t1 = clock64();
  if (lane == 0) ticks[tid >> 6] = t1 - t0;
  sink[tid] = reinterpret_cast<const int*>(lds)[tid];
}

}  // namespace

}  // namespace svg

extern "C" int svg_probe_lds(int form, int32_t waves, int32_t iterations, void* scratch, size_t scratch_bytes,
                             void* stream) {
  if (form < 0 || form > 3 || waves <= 0 || waves > 16 || iterations <= 0 || !scratch) return SVG_ERR_INVALID_ARG;
  if (svg::misaligned16(scratch)) return SVG_ERR_INVALID_ARG;
  if (scratch_bytes < 16 * sizeof(long long) + 1024 * sizeof(int)) return SVG_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  long long* ticks = static_cast<long long*>(scratch);
  int* sink = reinterpret_cast<int*>(ticks + 16);
  (void)hipGetLastError();
  const dim3 grid(1), block(64 * waves);
  if (form == 0) hipLaunchKernelGGL((svg::lds_probe_kernel<0>), grid, block, 0, s, ticks, sink, iterations);
  else if (form == 1) hipLaunchKernelGGL((svg::lds_probe_kernel<1>), grid, block, 0, s, ticks, sink, iterations);
  else if (form == 2) hipLaunchKernelGGL((svg::lds_probe_kernel<2>), grid, block, 0, s, ticks, sink, iterations);
  else hipLaunchKernelGGL((svg::lds_probe_kernel<3>), grid, block, 0, s, ticks, sink, iterations);
  return svg::hip_status(hipGetLastError());
}

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
