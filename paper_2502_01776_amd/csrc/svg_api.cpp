// C-ABI entry points that enqueue kernels: argument checks, then the launchers.
#include "svg_internal.h"

using svg::Geo;

namespace {

size_t tensor_bytes(const Geo& g) { return (size_t)g.B * g.H * g.N * g.D * 2; }

bool overlap(const void* a, size_t a_bytes, const void* b, size_t b_bytes) {
  const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
  return x < y + b_bytes && y < x + a_bytes;
}
bool overlap(const void* a, const void* b, size_t bytes) { return overlap(a, bytes, b, bytes); }

int check_qkvo(const void* q, const void* k, const void* v, const void* o) {
  if (!q || !k || !v || !o) return SVG_ERR_INVALID_ARG;
  if (svg::misaligned16(q) || svg::misaligned16(k) || svg::misaligned16(v) || svg::misaligned16(o))
    return SVG_ERR_INVALID_ARG;
  return SVG_OK;
}

int layout_call(const svg_shape_t* shape, const void* in, void* out, const uint8_t* labels,
                void* stream, bool inverse) {
  Geo g;
  int rc = svg::make_geo(shape, &g);
  if (rc != SVG_OK) return rc;
  if (!in || !out || svg::misaligned16(in) || svg::misaligned16(out)) return SVG_ERR_INVALID_ARG;
  if (overlap(in, out, tensor_bytes(g))) return SVG_ERR_ALIAS;
  return svg::launch_layout(g, in, out, nullptr, nullptr, labels, inverse, false, static_cast<hipStream_t>(stream));
}

}  // namespace

extern "C" {

int svg_layout_fwd(const svg_shape_t* shape, const void* in, void* out, const uint8_t* labels,
                   void* stream) {
  return layout_call(shape, in, out, labels, stream, false);
}

int svg_layout_inv(const svg_shape_t* shape, const void* in, void* out, const uint8_t* labels,
                   void* stream) {
  return layout_call(shape, in, out, labels, stream, true);
}

int svg_profile_heads(const svg_shape_t* shape, const void* q, const void* k, const void* v,
                      const int32_t* rows, int32_t t, uint8_t* labels, float* mse, void* workspace,
                      size_t workspace_bytes, void* stream) {
  Geo g;
  int rc = svg::make_geo(shape, &g);
  if (rc != SVG_OK) return rc;
  rc = svg::check_profile_args(g, q, k, v, rows, t, labels);
  if (rc != SVG_OK) return rc;
  if (!workspace || workspace_bytes < svg_workspace_bytes(shape, t)) return SVG_ERR_WORKSPACE;
  if (svg::misaligned16(workspace)) return SVG_ERR_INVALID_ARG;
  return svg::launch_profile(g, q, k, v, rows, t, labels, mse, static_cast<float*>(workspace),
                             static_cast<hipStream_t>(stream));
}

int svg_sparse_attn_fwd_ex(const svg_shape_t* shape, const void* q, const void* k, const void* v,
                           void* o, const uint8_t* labels, const int32_t* row_ptr_s,
                           const int32_t* col_idx_s, const int32_t* row_ptr_t,
                           const int32_t* col_idx_t, uint32_t flags, void* workspace,
                           size_t workspace_bytes, void* stream) {
  if (flags & ~(uint32_t)(SVG_ATTN_QO_TOKEN_ORDER | SVG_ATTN_ELEMENT_MASK | SVG_ATTN_KV_TOKEN_ORDER))
    return SVG_ERR_INVALID_ARG;
  Geo g;
  int rc = svg::make_geo(shape, &g);
  if (rc != SVG_OK) return rc;
  rc = check_qkvo(q, k, v, o);
  if (rc != SVG_OK) return rc;
  if (!row_ptr_s || !col_idx_s) return SVG_ERR_INVALID_ARG;
  if (labels && (!row_ptr_t || !col_idx_t)) return SVG_ERR_INVALID_ARG;
  const size_t bytes = tensor_bytes(g);
  if (overlap(o, q, bytes) || overlap(o, k, bytes) || overlap(o, v, bytes)) return SVG_ERR_ALIAS;
  int32_t* row_table = nullptr;
  if (flags & SVG_ATTN_KV_TOKEN_ORDER) {
    if ((flags & SVG_ATTN_ELEMENT_MASK) || g.bm != 128) return SVG_ERR_UNSUPPORTED;
    if (!workspace || svg::misaligned16(workspace) || workspace_bytes < svg::row_table_bytes(g)) return SVG_ERR_WORKSPACE;
    if (overlap(workspace, svg::row_table_bytes(g), o, bytes) || overlap(workspace, svg::row_table_bytes(g), q, bytes) ||
        overlap(workspace, svg::row_table_bytes(g), k, bytes) || overlap(workspace, svg::row_table_bytes(g), v, bytes))
      return SVG_ERR_ALIAS;
    row_table = static_cast<int32_t*>(workspace);
  }
  return svg::launch_attention(g, q, k, v, nullptr, nullptr, o, labels, row_ptr_s, col_idx_s, row_ptr_t, col_idx_t,
                               true, (flags & SVG_ATTN_QO_TOKEN_ORDER) != 0,
                               (flags & SVG_ATTN_ELEMENT_MASK) != 0, row_table, static_cast<hipStream_t>(stream));
}

int svg_layout_kv_temporal(const svg_shape_t* shape, const void* k, const void* v, void* k_t, void* v_t,
                           const uint8_t* labels, void* stream) {
  Geo g;
  int rc = svg::make_geo(shape, &g);
  if (rc != SVG_OK) return rc;
  if (!k || !v || !k_t || !v_t || !labels) return SVG_ERR_INVALID_ARG;
  if (svg::misaligned16(k) || svg::misaligned16(v) || svg::misaligned16(k_t) || svg::misaligned16(v_t))
    return SVG_ERR_INVALID_ARG;
  const size_t bytes = tensor_bytes(g);
  if (overlap(k_t, k, bytes) || overlap(k_t, v, bytes) || overlap(v_t, k, bytes) || overlap(v_t, v, bytes) ||
      overlap(k_t, v_t, bytes))
    return SVG_ERR_ALIAS;
  return svg::launch_layout(g, k, k_t, v, v_t, labels, false, true, static_cast<hipStream_t>(stream));
}

int svg_sparse_attn_fwd_kv2(const svg_shape_t* shape, const void* q, const void* k, const void* v,
                            const void* k_t, const void* v_t, void* o, const uint8_t* labels,
                            const int32_t* row_ptr_s, const int32_t* col_idx_s, const int32_t* row_ptr_t,
                            const int32_t* col_idx_t, uint32_t flags, void* stream) {
  if (flags & ~(uint32_t)SVG_ATTN_ELEMENT_MASK) return SVG_ERR_INVALID_ARG;
  Geo g;
  int rc = svg::make_geo(shape, &g);
  if (rc != SVG_OK) return rc;
  rc = check_qkvo(q, k, v, o);
  if (rc != SVG_OK) return rc;
  if (!k_t || !v_t || svg::misaligned16(k_t) || svg::misaligned16(v_t)) return SVG_ERR_INVALID_ARG;
  if (!labels || !row_ptr_s || !col_idx_s || !row_ptr_t || !col_idx_t) return SVG_ERR_INVALID_ARG;
  const size_t bytes = tensor_bytes(g);
  if (overlap(o, q, bytes) || overlap(o, k, bytes) || overlap(o, v, bytes) || overlap(o, k_t, bytes) ||
      overlap(o, v_t, bytes))
    return SVG_ERR_ALIAS;
  return svg::launch_attention(g, q, k, v, k_t, v_t, o, labels, row_ptr_s, col_idx_s, row_ptr_t, col_idx_t, true,
                               true, (flags & SVG_ATTN_ELEMENT_MASK) != 0, nullptr, static_cast<hipStream_t>(stream));
}

int svg_sparse_attn_fwd(const svg_shape_t* shape, const void* q, const void* k, const void* v,
                        void* o, const uint8_t* labels, const int32_t* row_ptr_s,
                        const int32_t* col_idx_s, const int32_t* row_ptr_t,
                        const int32_t* col_idx_t, void* workspace, size_t workspace_bytes,
                        void* stream) {
  return svg_sparse_attn_fwd_ex(shape, q, k, v, o, labels, row_ptr_s, col_idx_s, row_ptr_t,
                                col_idx_t, 0u, workspace, workspace_bytes, stream);
}

int svg_dense_attn_fwd(const svg_shape_t* shape, const void* q, const void* k, const void* v,
                       void* o, void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace;
  (void)workspace_bytes;
  Geo g;
  int rc = svg::make_geo(shape, &g);
  if (rc != SVG_OK) return rc;
  rc = check_qkvo(q, k, v, o);
  if (rc != SVG_OK) return rc;
  const size_t bytes = tensor_bytes(g);
  if (overlap(o, q, bytes) || overlap(o, k, bytes) || overlap(o, v, bytes)) return SVG_ERR_ALIAS;
  return svg::launch_attention(g, q, k, v, nullptr, nullptr, o, nullptr, nullptr, nullptr, nullptr, nullptr, false,
                               false, false, nullptr, static_cast<hipStream_t>(stream));
}

int svg_qk_norm_rope(const svg_shape_t* shape, const void* x, void* y, int norm, const float* weight,
                     const float* bias, float eps, const float* cos, const float* sin, int pairing,
                     void* stream) {
  Geo g;
  int rc = svg::make_geo(shape, &g);
  if (rc != SVG_OK) return rc;
  if (!x || !y || svg::misaligned16(x) || svg::misaligned16(y)) return SVG_ERR_INVALID_ARG;
  if (norm != SVG_NORM_NONE && norm != SVG_NORM_RMS && norm != SVG_NORM_LAYER) return SVG_ERR_INVALID_ARG;
  if (pairing != SVG_ROPE_INTERLEAVED && pairing != SVG_ROPE_HALF) return SVG_ERR_INVALID_ARG;
  if ((cos == nullptr) != (sin == nullptr)) return SVG_ERR_INVALID_ARG;
  if (cos && (svg::misaligned16(cos) || svg::misaligned16(sin))) return SVG_ERR_INVALID_ARG;
  if (!(eps >= 0.f)) return SVG_ERR_INVALID_ARG;
  // in place (y == x) is fine, a partial overlap is not
  if (x != y && overlap(x, y, tensor_bytes(g))) return SVG_ERR_ALIAS;
  return svg::launch_norm_rope(g, x, y, norm, weight, bias, eps, cos, sin, pairing,
                               static_cast<hipStream_t>(stream));
}

size_t svg_fp8_buffer_bytes(const svg_shape_t* shape, int which) {
  Geo g;
  if (svg::make_geo(shape, &g) != SVG_OK || g.D != 128 || g.bm != 128) return 0;
  const size_t bh = (size_t)g.B * g.H;
  switch (which) {
    case SVG_FP8_Q: return bh * g.N * g.D;
    case SVG_FP8_K:
    case SVG_FP8_VT: return bh * g.nk * g.bn * g.D;
    case SVG_FP8_SCALES: return 6 * bh * sizeof(float);
    default: return 0;
  }
}

int svg_fp8_quantize(const svg_shape_t* shape, const void* q, const void* k, const void* v,
                     const uint8_t* labels, void* q8, void* k8, void* v8t, float* scales,
                     void* stream) {
  Geo g;
  int rc = svg::make_geo(shape, &g);
  if (rc != SVG_OK) return rc;
  if (g.D != 128 || g.bm != 128) return SVG_ERR_UNSUPPORTED;
  if (!q || !k || !v || !q8 || !k8 || !v8t || !scales) return SVG_ERR_INVALID_ARG;
  if (svg::misaligned16(q) || svg::misaligned16(k) || svg::misaligned16(v) || svg::misaligned16(q8) ||
      svg::misaligned16(k8) || svg::misaligned16(v8t) || svg::misaligned16(scales))
    return SVG_ERR_INVALID_ARG;
  {
    // the five outputs must be distinct from each other and from the three inputs
    const size_t in_bytes = tensor_bytes(g);
    const void* bufs[7] = {q8, k8, v8t, scales, q, k, v};
    const size_t sizes[7] = {svg_fp8_buffer_bytes(shape, SVG_FP8_Q), svg_fp8_buffer_bytes(shape, SVG_FP8_K),
                             svg_fp8_buffer_bytes(shape, SVG_FP8_VT), svg_fp8_buffer_bytes(shape, SVG_FP8_SCALES),
                             in_bytes, in_bytes, in_bytes};
    for (int i = 0; i < 4; ++i)
      for (int j = i + 1; j < 7; ++j)
        if (overlap(bufs[i], sizes[i], bufs[j], sizes[j])) return SVG_ERR_ALIAS;
  }
  return svg::launch_fp8_quantize(g, q, k, v, labels, q8, k8, v8t, scales,
                                  static_cast<hipStream_t>(stream));
}

int svg_sparse_attn_fp8_fwd(const svg_shape_t* shape, const void* q8, const void* k8,
                            const void* v8t, const float* scales, void* o, const uint8_t* labels,
                            const int32_t* row_ptr_s, const int32_t* col_idx_s,
                            const int32_t* row_ptr_t, const int32_t* col_idx_t, void* stream) {
  Geo g;
  int rc = svg::make_geo(shape, &g);
  if (rc != SVG_OK) return rc;
  if (g.D != 128 || g.bm != 128) return SVG_ERR_UNSUPPORTED;
  if (!scales || svg::misaligned16(scales)) return SVG_ERR_INVALID_ARG;
  rc = check_qkvo(q8, k8, v8t, o);
  if (rc != SVG_OK) return rc;
  if (!row_ptr_s || !col_idx_s) return SVG_ERR_INVALID_ARG;
  if (labels && (!row_ptr_t || !col_idx_t)) return SVG_ERR_INVALID_ARG;
  {
    const size_t o_bytes = tensor_bytes(g);
    if (overlap(o, o_bytes, q8, svg_fp8_buffer_bytes(shape, SVG_FP8_Q)) ||
        overlap(o, o_bytes, k8, svg_fp8_buffer_bytes(shape, SVG_FP8_K)) ||
        overlap(o, o_bytes, v8t, svg_fp8_buffer_bytes(shape, SVG_FP8_VT)) ||
        overlap(o, o_bytes, scales, svg_fp8_buffer_bytes(shape, SVG_FP8_SCALES)))
      return SVG_ERR_ALIAS;
  }
  return svg::launch_fp8_attention(g, q8, k8, v8t, scales, o, labels, row_ptr_s, col_idx_s, row_ptr_t,
                                   col_idx_t, static_cast<hipStream_t>(stream));
}

}  // extern "C"
