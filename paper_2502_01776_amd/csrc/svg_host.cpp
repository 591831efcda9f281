// Host side of the C ABI: argument validation, error strings, and the kept-tile
// list builder.  The tile list depends only on the geometry, so it is built on the
// host in closed form (interval arithmetic on frame / position groups) and the
// caller uploads it once per shape.
#include <algorithm>
#include <cmath>
#include <functional>
#include <mutex>
#include <queue>
#include <vector>

#include "svg_internal.h"

namespace svg {

static thread_local hipError_t g_last_hip_error = hipSuccess;
void note_hip_error(hipError_t e) { g_last_hip_error = e; }

// ---------------------------------------------------------------------------------------------
// Plan of the profiling passes (see ProfilePlan).  Cost model, in units of one unmasked key tile:
// a masked tile costs kMaskedTile (its waves also build and apply element masks, and wait for
// each other on tiles that only some of them need), every workgroup kStartTiles on top.  The
// masked passes of a group of rows visit the union of the windows of its rows: the sampled rows
// are taken to be spread evenly, so a group of a head's rows spans F / groups frames (spatial
// pass, rows in token order) or P / groups in-frame positions (temporal pass, rows grouped by
// position).  The workgroups of one XCD are dealt to its kSlots resident places in dispatch
// order (masked parts first, then the unmasked parts in order) and the plan with the smallest
// finishing time wins; more parts cost a little extra workspace and merging.
// ---------------------------------------------------------------------------------------------
namespace {

constexpr int kSlots = 64;            // workgroups resident on one XCD: 32 CUs x 2
constexpr double kMaskedTile = 1.5;
constexpr double kStartTiles = 10.0;

struct PlanKey {
  int v[12];
  bool operator==(const PlanKey& o) const { return std::equal(v, v + 12, o.v); }
};

double finish_time(const std::vector<std::pair<double, int>>& classes) {
  std::priority_queue<double, std::vector<double>, std::greater<double>> free_at;
  for (int i = 0; i < kSlots; ++i) free_at.push(0.0);
  double last = 0.0;
  for (const auto& c : classes)
    for (int i = 0; i < c.second; ++i) {
      const double t = free_at.top() + c.first;
      free_at.pop();
      free_at.push(t);
      last = std::max(last, t);
    }
  return last;
}

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

ProfilePlan search_plan(const Geo& g, int t) {
  const int groups = (t + g.bm - 1) / g.bm;
  const long long pairs = (long long)g.B * g.H * groups;
  const int pairs_x = (int)((pairs + 7) / 8);
  ProfilePlan best = {};
  best.n_masked = 1;
  if (g.nk < 4) {                       // a handful of tiles: nothing to cut
    fill_bounds(&best, 1, 0, g.nk);
    return best;
  }
  if (pairs_x >= 4 * kSlots) {          // many rounds of workgroups anyway: a short tail is all that is needed
    fill_bounds(&best, 1, 2, g.nk);
    return best;
  }
  const double tile_keys = g.bn;
  const double len_s = std::min<double>(g.nk, (((double)g.F / groups + 1 + 2 * g.w_s + 1) * g.P + g.T) / tile_keys);
  const double len_t = std::min<double>(g.nk, ((double)g.F * ((double)g.P / groups + 2 * g.w_t + 1) + g.T) / tile_keys);
  double best_time = -1.0;
  for (int nm = 1; nm <= 4; ++nm)
    for (int n_small = 0; n_small <= 2; n_small += 2)
      for (int n_big = 1; n_big + n_small <= kMaxProfileParts - 2; ++n_big) {
        if (2 * n_big + n_small > g.nk) break;
        std::vector<std::pair<double, int>> classes;
        classes.emplace_back(len_s * kMaskedTile / nm + kStartTiles, pairs_x * nm);
        classes.emplace_back(len_t * kMaskedTile / nm + kStartTiles, pairs_x * nm);
        const double unit = (double)g.nk / (2 * n_big + n_small);
        classes.emplace_back(2 * unit + kStartTiles, pairs_x * n_big);
        if (n_small) classes.emplace_back(unit + kStartTiles, pairs_x * n_small);
        const double time = finish_time(classes) * (1.0 + 0.002 * (n_big + n_small + 2 * nm));
        if (best_time < 0.0 || time < best_time) {
          best_time = time;
          best.n_masked = nm;
          fill_bounds(&best, n_big, n_small, g.nk);
        }
      }
  return best;
}

}  // namespace

ProfilePlan profile_plan(const Geo& g, int t) {
  static std::mutex mu;
  static std::vector<std::pair<PlanKey, ProfilePlan>> cache;
  static size_t next = 0;
  const PlanKey key = {{g.B * g.H, g.F, g.P, g.T, g.text_first, g.w_s, g.w_t, g.bm, g.bn, g.nk, t, 0}};
  std::lock_guard<std::mutex> lock(mu);
  for (const auto& e : cache)
    if (e.first == key) return e.second;
  const ProfilePlan plan = search_plan(g, t);
  if (cache.size() < 16) cache.emplace_back(key, plan);
  else cache[next++ % 16] = std::make_pair(key, plan);
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
