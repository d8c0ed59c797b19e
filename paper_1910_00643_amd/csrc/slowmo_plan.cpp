#include "slowmo_plan.h"

#include <algorithm>

namespace slowmo {

Layout make_layout(int32_t n_tensors, const int64_t *numel) {
  Layout L;
  L.arena_off.resize(n_tensors);
  int64_t off = 0;
  for (int32_t j = 0; j < n_tensors; ++j) {
    L.arena_off[j] = off;
    L.d += numel[j];
    off += (numel[j] + kArenaAlign - 1) / kArenaAlign * kArenaAlign;
  }
  L.d_pad = std::max<int64_t>(off, kArenaAlign);
  return L;
}

static int64_t tiles_of(int64_t n, int64_t tile) { return (n + tile - 1) / tile; }

int64_t count_local_tiles(int32_t m, int32_t n_tensors, const int64_t *numel) {
  int64_t per_worker = 0;
  for (int32_t j = 0; j < n_tensors; ++j) per_worker += tiles_of(numel[j], kLocalTile);
  return per_worker * m;
}

int64_t count_outer_tiles(int32_t n_tensors, const int64_t *numel) {
  int64_t t = 0;
  for (int32_t j = 0; j < n_tensors; ++j) t += tiles_of(numel[j], kOuterTile);
  return t;
}

static void cut(int32_t worker, int32_t n_tensors, const int64_t *numel, int64_t tile,
                std::vector<PlanRun> &runs) {
  for (int32_t j = 0; j < n_tensors; ++j) {
    for (int64_t off = 0; off < numel[j]; off += tile) {
      PlanRun r;
      r.tile = static_cast<int32_t>(runs.size());
      r.worker = worker;
      r.tensor = j;
      r.n = static_cast<int32_t>(std::min<int64_t>(tile, numel[j] - off));
      r.offset = off;
      runs.push_back(r);
    }
  }
}

void plan_local(int32_t m, int32_t n_tensors, const int64_t *numel, std::vector<PlanRun> &runs) {
  runs.clear();
  runs.reserve(static_cast<size_t>(count_local_tiles(m, n_tensors, numel)));
  for (int32_t w = 0; w < m; ++w) cut(w, n_tensors, numel, kLocalTile, runs);
}

void plan_outer(int32_t n_tensors, const int64_t *numel, std::vector<PlanRun> &runs) {
  runs.clear();
  runs.reserve(static_cast<size_t>(count_outer_tiles(n_tensors, numel)));
  cut(-1, n_tensors, numel, kOuterTile, runs);
}

}  // namespace slowmo
