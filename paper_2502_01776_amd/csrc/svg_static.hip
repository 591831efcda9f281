// Entry point for callers that cannot allocate device memory (HIP graph capture, tight
// serving loops, harnesses that forbid hipMalloc): online profiling with its workspace
// in an array that is part of the loaded code object instead of a caller's buffer.
#include <mutex>

#include "svg_internal.h"

namespace {

// Scratch of svg_profile_heads_static: one copy per GPU the library is loaded on, held until
// the process ends.  Every call on a GPU uses that GPU's copy, so calls that overlap in time
// on one GPU (different streams, different threads) race.
static __device__ __align__(256) unsigned char scratch[SVG_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of this GPU's copy of `scratch`.  In host code the array's name is only a
// handle for the runtime, not an address a kernel could use; the runtime translates it once per
// device (with that device current), and only the translated pointer is ever passed on.
int scratch_pointer(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return svg::hip_status(e);
  if (dev < 0 || dev >= kMaxDevices) return SVG_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return svg::hip_status(e);
    if (!p) return SVG_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return SVG_OK;
}

}  // namespace

extern "C" int svg_profile_heads_static(const svg_shape_t* shape, const void* q, const void* k, const void* v,
                                        const int32_t* rows, int32_t t, uint8_t* labels, float* mse,
                                        void* stream) {
  svg::Geo g;
  int rc = svg::make_geo(shape, &g);
  if (rc != SVG_OK) return rc;
  rc = svg::check_profile_args(g, q, k, v, rows, t, labels);
  if (rc != SVG_OK) return rc;
  // sizes beyond the array are refused before anything touches the device
  if (svg::profile_workspace_bytes(g, t) > (size_t)SVG_STATIC_SCRATCH_BYTES) return SVG_ERR_WORKSPACE;
  void* ws = nullptr;
  rc = scratch_pointer(&ws);
  if (rc != SVG_OK) return rc;
  // nothing in the workspace has to start at zero: every word a kernel of the profiling pass
  // reads was written earlier in the same call (outputs and statistics by the attention pass,
  // partial sums by the error pass, the row order by the ordering pass)
  return svg::launch_profile(g, q, k, v, rows, t, labels, mse, static_cast<float*>(ws),
                             static_cast<hipStream_t>(stream));
}
