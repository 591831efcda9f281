// Internal declarations shared by the host-side entry points and the kernel
// launchers of the sparse 3D attention library.  Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "svg.h"

namespace svg {

// Geometry after validation, passed by value to kernels.
struct Geo {
  int B, H, F, P, T, D, N;
  int off;          // first video row: T if text_first else 0
  int video_end;    // off + F*P
  int w_s, w_t, sink;
  int bm, bn, nq, nk;
  int text_first;
  float scale;      // softmax scale
};

// Checks sizes, D and tile shape.  Returns SVG_OK and fills g, or an error code.
int make_geo(const svg_shape_t* s, Geo* g);

// How the three passes of online profiling (Alg. 1) are cut into workgroups.  A (head, group of
// sampled rows) pair has one unmasked pass over all nk key tiles and two masked passes over the
// tiles their windows can reach; each pass is cut along its tile sequence into parts that run as
// separate workgroups and are merged afterwards from (output, maximum, row sum) triples.  The
// unmasked pass has n_full <= 6 parts with tile boundaries full_bound[] (the last parts are
// shorter, so that the workgroups finishing last are short ones), each masked pass n_masked <= 4
// equal parts.  The choice depends on the shape and t only (profile_plan in svg_host.cpp).
constexpr int kMaxProfileParts = 16;
struct ProfilePlan {
  int n_full, n_masked;
  int full_bound[kMaxProfileParts + 1];
  __host__ __device__ int slots() const { return n_full + 2 * n_masked; }
};
ProfilePlan profile_plan(const Geo& g, int t);

// Bytes of workspace svg_profile_heads uses for t rows: fp32 outputs [slots][BH][t][D], float2
// (maximum, row sum) [slots][BH][t], partial error sums float2 [BH][ceil(t/16)], row order int32 [t].
inline size_t profile_workspace_bytes(const Geo& g, int t) {
  const size_t bh = (size_t)g.B * g.H;
  const size_t slots = (size_t)profile_plan(g, t).slots();
  return slots * bh * t * g.D * sizeof(float) + slots * bh * t * 2 * sizeof(float) +
         bh * (size_t)((t + 15) / 16) * 2 * sizeof(float) + (((size_t)t * 4 + 15) & ~(size_t)15);
}

// The transformed ("P-outer") order of a temporal head, video part only; offsets are relative
// to the first video row.  Without the first-frame sink the token of frame f and position p
// sits at offset p*F + f (Sec. 4.2).  With the sink on (Sec. 3.1: every query also attends
// to the first frame) frame 0 comes first as one block in position order (offset p), and the
// position-outer order runs over the other frames: offset P + p*(F-1) + (f-1); the frame-0
// keys are then one contiguous run of key tiles instead of one key in every F rows.
// transformed_to_token returns the F-outer offset f*P + p of the token at transformed offset v.
__host__ __device__ inline unsigned transformed_to_token(unsigned v, unsigned F, unsigned P, int sink,
                                                         unsigned* pos = nullptr, unsigned* frame = nullptr) {
  unsigned p, f;
  if (sink) {
    if (v < P) {
      p = v;
      f = 0;
    } else {
      const unsigned w = v - P, rest = F > 1 ? F - 1 : 1;
      p = w / rest;
      f = w - p * rest + 1;
    }
  } else {
    p = v / F;
    f = v - p * F;
  }
  if (pos) *pos = p;
  if (frame) *frame = f;
  return f * P + p;
}
__host__ __device__ inline unsigned token_to_transformed(unsigned v, unsigned F, unsigned P, int sink) {
  const unsigned f = v / P, p = v - f * P;
  if (sink) return f == 0 ? p : P + p * (F - 1) + (f - 1);
  return p * F + f;
}

inline bool misaligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Argument checks shared by the profiling entry points (everything except the workspace).
inline int check_profile_args(const Geo& g, const void* q, const void* k, const void* v, const int32_t* rows,
                              int32_t t, const uint8_t* labels) {
  if (!q || !k || !v || !rows || !labels || t <= 0) return SVG_ERR_INVALID_ARG;
  if (misaligned16(q) || misaligned16(k) || misaligned16(v)) return SVG_ERR_INVALID_ARG;
  if ((int64_t)3 * g.B * g.H * ((t + g.bm - 1) / g.bm) > (int64_t)1 << 30) return SVG_ERR_UNSUPPORTED;
  if ((int64_t)g.B * g.H > 65535) return SVG_ERR_UNSUPPORTED;      // heads are a grid dimension of the error pass
  return SVG_OK;
}

// Remembers the most recent HIP error of the calling thread for svg_last_hip_error().
void note_hip_error(hipError_t e);
inline int hip_status(hipError_t e) {
  if (e == hipSuccess) return SVG_OK;
  note_hip_error(e);
  return SVG_ERR_HIP;
}

// Kernel launchers (defined in the .hip files).  All arguments validated by the caller.
// in2 / out2: optional second tensor moved by the same launch; temporal_only: heads labelled
// spatial are skipped instead of copied
int launch_layout(const Geo& g, const void* in, void* out, const void* in2, void* out2, const uint8_t* labels,
                  bool inverse, bool temporal_only, hipStream_t stream);
// k_t / v_t: optional P-outer copies of k and v that heads labelled temporal read instead of k / v
int launch_attention(const Geo& g, const void* q, const void* k, const void* v, const void* k_t, const void* v_t,
                     void* o, const uint8_t* labels, const int32_t* row_ptr_s, const int32_t* col_idx_s,
                     const int32_t* row_ptr_t, const int32_t* col_idx_t, bool sparse,
                     bool qo_token_order, bool element_mask, int32_t* row_table, hipStream_t stream);

// Bytes of workspace the sparse pass needs when k and v stay in token order (the row table).
inline size_t row_table_bytes(const Geo& g) { return 2 * (size_t)g.nk * g.bn * sizeof(int32_t); }
int launch_profile(const Geo& g, const void* q, const void* k, const void* v, const int32_t* rows,
                   int t, uint8_t* labels, float* mse, float* workspace, hipStream_t stream);

int launch_norm_rope(const Geo& g, const void* x, void* y, int norm, const float* weight, const float* bias,
                     float eps, const float* cos, const float* sin, int pairing, hipStream_t stream);
int launch_fp8_quantize(const Geo& g, const void* q, const void* k, const void* v, const uint8_t* labels,
                        void* q8, void* k8, void* v8t, float* scales, hipStream_t stream);
int launch_fp8_attention(const Geo& g, const void* q8, const void* k8, const void* v8t, const float* scales,
                         void* o, const uint8_t* labels, const int32_t* row_ptr_s, const int32_t* col_idx_s,
                         const int32_t* row_ptr_t, const int32_t* col_idx_t, hipStream_t stream);

}  // namespace svg
