// Host side of the C ABI: argument validation, error strings, and the kept-tile
// list builder.  The tile list depends only on the geometry, so it is built on the
// host in closed form (interval arithmetic on frame / position groups) and the
// caller uploads it once per shape.
#include <algorithm>
#include <cmath>
#include <vector>

#include "svg_internal.h"

namespace svg {

static thread_local hipError_t g_last_hip_error = hipSuccess;
void note_hip_error(hipError_t e) { g_last_hip_error = e; }

// ---------------------------------------------------------------------------------------------
// Plan of the profiling passes (see ProfilePlan), from measurements on MI355X with 64 workgroups
// resident per XCD (96 at head dimension 64, where three fit a CU):
//  * Unmasked pass: four parts and two of half their length at the end, so that the workgroups
//    that finish last are short ones (1-3 % less time than eight equal parts; anything from
//    four to eight parts measured within 1 % of each other).  Fewer parts for short sequences,
//    and three when the sampled rows alone already give every XCD hundreds of workgroups.
//  * Masked passes: one part each, unless the (head, row group) pairs are so few that the two
//    masked workgroups per pair cannot fill an XCD; then as many parts (up to four) as keep
//    them within its resident places.  CogVideoX-v1 at 1 % (12 pairs per XCD): three parts,
//    -32 % time; 0.1 % of the rows at the 119k-token shape (3 pairs): four parts, 3.9 -> 1.3 ms;
//    with 15 or more pairs per XCD any cut of the masked passes measured slower (+4-20 %).
// ---------------------------------------------------------------------------------------------
namespace {

constexpr int kSlots = 64;            // workgroups resident on one XCD: 32 CUs x 2 (x 3 at D = 64)

void fill_bounds(ProfilePlan* p, int n_big, int n_small, int nk) {
  p->n_full = n_big + n_small;
  const int total = 2 * n_big + n_small;
  int cum = 0;
  for (int c = 0; c <= p->n_full; ++c) {
    p->full_bound[c] = (int)(((long long)nk * cum) / total);
    cum += c < n_big ? 2 : 1;
  }
  p->full_bound[p->n_full] = nk;
}

}  // namespace

ProfilePlan profile_plan(const Geo& g, int t) {
  const int groups = (t + g.bm - 1) / g.bm;
  const long long pairs = (long long)g.B * g.H * groups;
  const long long pairs_x = (pairs + 7) / 8;
  ProfilePlan plan = {};
  const int slots = g.D == 64 ? kSlots * 3 / 2 : kSlots;
  plan.n_masked = (int)std::max<long long>(1, std::min<long long>(4, (slots - 8) / (2 * pairs_x)));
  if (g.nk < 24) fill_bounds(&plan, 1, 0, g.nk);
  else if (pairs_x >= 4 * kSlots) fill_bounds(&plan, 1, 2, g.nk);
  else if (g.nk < 96) fill_bounds(&plan, 2, 2, g.nk);
  else fill_bounds(&plan, 4, 2, g.nk);
  return plan;
}

int make_geo(const svg_shape_t* s, Geo* g) {
  if (!s) return SVG_ERR_INVALID_ARG;
  if (s->B <= 0 || s->H <= 0 || s->F <= 0 || s->P <= 0 || s->T < 0) return SVG_ERR_INVALID_ARG;
  if (s->w_s < 0 || s->w_t < 0) return SVG_ERR_INVALID_ARG;
  if (s->text_first != 0 && s->text_first != 1) return SVG_ERR_INVALID_ARG;
  if (s->sink_first_frame != 0 && s->sink_first_frame != 1) return SVG_ERR_INVALID_ARG;
  if (!(s->softmax_scale == s->softmax_scale) || std::isinf(s->softmax_scale)) return SVG_ERR_INVALID_ARG;
  if (s->D != 64 && s->D != 128) return SVG_ERR_UNSUPPORTED;
  const bool big = s->block_m == 128 && s->block_n == 64;
  const bool small = s->block_m == 32 && s->block_n == 32;
  if (!big && !small) return SVG_ERR_UNSUPPORTED;
  const int64_t n = (int64_t)s->F * s->P + s->T;
  // row indices, tile indices and B*H*nq must fit comfortably in int32
  if (n > (1 << 22)) return SVG_ERR_UNSUPPORTED;
  const int64_t nq = (n + s->block_m - 1) / s->block_m;
  if ((int64_t)s->B * s->H * nq > (int64_t)1 << 30) return SVG_ERR_UNSUPPORTED;
  g->B = s->B; g->H = s->H; g->F = s->F; g->P = s->P; g->T = s->T; g->D = s->D;
  g->N = (int)n;
  g->text_first = s->text_first;
  g->off = s->text_first ? s->T : 0;
  g->video_end = g->off + s->F * s->P;
  g->w_s = s->w_s; g->w_t = s->w_t; g->sink = s->sink_first_frame;
  g->bm = s->block_m; g->bn = s->block_n;
  g->nq = (int)nq;
  g->nk = (int)((n + s->block_n - 1) / s->block_n);
  g->scale = s->softmax_scale > 0.f ? s->softmax_scale : 1.0f / std::sqrt((float)s->D);
  return SVG_OK;
}

}  // namespace svg

using svg::Geo;

extern "C" {

const char* svg_strerror(int status) {
  switch (status) {
    case SVG_OK: return "ok";
    case SVG_ERR_INVALID_ARG: return "invalid argument";
    case SVG_ERR_UNSUPPORTED: return "unsupported head dimension, tile shape or size";
    case SVG_ERR_WORKSPACE: return "workspace missing or too small";
    case SVG_ERR_ALIAS: return "input and output overlap";
    case SVG_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

const char* svg_version(void) { return "0.2"; }

const char* svg_last_hip_error(void) { return hipGetErrorString(svg::g_last_hip_error); }

size_t svg_workspace_bytes(const svg_shape_t* shape, int32_t t) {
  Geo g;
  if (svg::make_geo(shape, &g) != SVG_OK || t <= 0) return 0;
  const size_t a = svg::profile_workspace_bytes(g, t), b = svg::row_table_bytes(g);
  return a > b ? a : b;
}

int svg_profile_plan(const svg_shape_t* shape, int32_t t, int32_t* n_full, int32_t* n_masked,
                     int32_t* full_bound) {
  Geo g;
  int rc = svg::make_geo(shape, &g);
  if (rc != SVG_OK) return rc;
  if (t <= 0 || !n_full || !n_masked) return SVG_ERR_INVALID_ARG;
  const svg::ProfilePlan plan = svg::profile_plan(g, t);
  *n_full = plan.n_full;
  *n_masked = plan.n_masked;
  if (full_bound)
    for (int c = 0; c <= svg::kMaxProfileParts; ++c) full_bound[c] = plan.full_bound[c < plan.n_full ? c : plan.n_full];
  return SVG_OK;
}

int svg_tile_counts(const svg_shape_t* shape, int32_t* nq, int32_t* nk) {
  Geo g;
  int rc = svg::make_geo(shape, &g);
  if (rc != SVG_OK) return rc;
  if (!nq || !nk) return SVG_ERR_INVALID_ARG;
  *nq = g.nq;
  *nk = g.nk;
  return SVG_OK;
}

int svg_tile_list_build(const svg_shape_t* shape, int pattern, int32_t* row_ptr, int32_t* col_idx,
                        int64_t cap, int64_t* nnz_out) {
  Geo g;
  int rc = svg::make_geo(shape, &g);
  if (rc != SVG_OK) return rc;
  if (pattern != SVG_HEAD_SPATIAL && pattern != SVG_HEAD_TEMPORAL && pattern != SVG_LIST_TEMPORAL_FRAME_MAJOR)
    return SVG_ERR_INVALID_ARG;
  if (!row_ptr || !nnz_out || (col_idx && cap < 0)) return SVG_ERR_INVALID_ARG;
  const bool frame_major_temporal = pattern == SVG_LIST_TEMPORAL_FRAME_MAJOR;

  // In its own order a pattern groups `unit` consecutive video rows: a frame (P rows)
  // for spatial, a position (F rows) for temporal; `groups` of them; window w groups.
  const int unit = pattern == SVG_HEAD_SPATIAL ? g.P : g.F;
  const int groups = pattern == SVG_HEAD_SPATIAL ? g.F : g.P;
  const int w = pattern == SVG_HEAD_SPATIAL ? g.w_s : g.w_t;
  const int v0 = g.off, v1 = g.video_end;  // video rows [v0, v1)

  std::vector<uint8_t> keep(g.nk);
  // tiles kept by every video query: text keys, and frame-0 keys if the sink is on
  std::vector<uint8_t> always(g.nk, 0);
  auto mark = [&](std::vector<uint8_t>& m, int64_t lo, int64_t hi) {  // rows [lo, hi] inclusive
    if (lo > hi) return;
    for (int b = (int)(lo / g.bn); b <= (int)(hi / g.bn); ++b) m[b] = 1;
  };
  if (g.T > 0) {
    if (g.text_first) mark(always, 0, g.T - 1); else mark(always, v1, g.N - 1);
  }
  // first-frame sink: in every order frame 0 is the first P video rows (the transformed order of a
  // temporal head keeps it as a block in front, see transformed_to_token)
  if (g.sink) mark(always, v0, v0 + g.P - 1);
  const bool sink_temporal = g.sink && pattern == SVG_HEAD_TEMPORAL;

  int64_t nnz = 0;
  bool overflow = false;
  row_ptr[0] = 0;
  for (int a = 0; a < g.nq; ++a) {
    const int64_t r0 = (int64_t)a * g.bm;
    const int64_t r1 = std::min<int64_t>(r0 + g.bm, g.N) - 1;
    const bool has_text_query = g.T > 0 && (r0 < v0 || r1 >= v1);
    if (has_text_query) {
      std::fill(keep.begin(), keep.end(), (uint8_t)1);
    } else if (frame_major_temporal) {
      // Rows r0..r1 in F-outer order cover the in-frame positions [pa, pb] of one frame, or
      // wrap over a frame end ([pa, P) and [0, pb]), or every position; each position
      // interval keeps, in EVERY frame, the keys within w_t positions of it.
      keep = always;
      const int64_t pa = (r0 - v0) % g.P, pb = (r1 - v0) % g.P;
      const bool one_frame = (r0 - v0) / g.P == (r1 - v0) / g.P;
      auto keep_positions = [&](int64_t lo, int64_t hi) {
        lo = std::max<int64_t>(0, lo - g.w_t);
        hi = std::min<int64_t>(g.P - 1, hi + g.w_t);
        for (int f = 0; f < g.F; ++f) mark(keep, v0 + (int64_t)f * g.P + lo, v0 + (int64_t)f * g.P + hi);
      };
      if (one_frame) {
        keep_positions(pa, pb);
      } else if (r1 - r0 + 1 >= g.P) {
        keep_positions(0, g.P - 1);
      } else {
        keep_positions(pa, g.P - 1);
        keep_positions(0, pb);
      }
    } else if (sink_temporal) {
      // Transformed order with the sink: rows [v0, v0 + P) are frame 0 in position order, rows from
      // b0 = v0 + P on hold positions outer over the other F - 1 frames.  Frame-0 keys are kept
      // anyway; of the others a query at position p keeps the positions within w_t of it.  The
      // tile's rows may lie in either part or in both.
      keep = always;
      const int64_t b0 = v0 + g.P, rest = g.F - 1;
      auto keep_positions = [&](int64_t lo, int64_t hi) {
        if (rest <= 0) return;
        lo = std::max<int64_t>(0, lo - g.w_t);
        hi = std::min<int64_t>(g.P - 1, hi + g.w_t);
        mark(keep, b0 + lo * rest, b0 + (hi + 1) * rest - 1);
      };
      if (r0 < b0) keep_positions(r0 - v0, std::min<int64_t>(r1, b0 - 1) - v0);
      if (r1 >= b0 && rest > 0) keep_positions((std::max<int64_t>(r0, b0) - b0) / rest, (r1 - b0) / rest);
    } else {
      keep = always;
      const int64_t ga = (r0 - v0) / unit, gb = (r1 - v0) / unit;
      const int64_t lo = v0 + std::max<int64_t>(0, ga - w) * unit;
      const int64_t hi = v0 + std::min<int64_t>(groups, gb + w + 1) * unit - 1;
      mark(keep, lo, hi);
    }
    for (int b = 0; b < g.nk; ++b) {
      if (!keep[b]) continue;
      if (col_idx) {
        if (nnz < cap) col_idx[nnz] = b; else overflow = true;
      }
      ++nnz;
    }
    if (nnz > INT32_MAX) return SVG_ERR_UNSUPPORTED;
    row_ptr[a + 1] = (int32_t)nnz;
  }
  *nnz_out = nnz;
  return overflow ? SVG_ERR_INVALID_ARG : SVG_OK;
}

}  // extern "C"
