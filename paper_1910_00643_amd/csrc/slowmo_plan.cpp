#include "slowmo_plan.h"

#include <algorithm>
#include <cstdlib>

namespace slowmo {

static int32_t env_int(const char *name, int32_t dflt, int32_t lo, int32_t hi) {
  const char *s = std::getenv(name);
  if (!s || !*s) return dflt;
  char *end = nullptr;
  long v = std::strtol(s, &end, 10);
  if (end == s || v < lo || v > hi) return dflt;
  return static_cast<int32_t>(v);
}

int32_t local_tile_elems() {
  // multiple of 4, at least one minimum-cost run
  int32_t t = env_int("SLOWMO_LOCAL_TILE", 16384, kMinRunCost, kMaxLocalTile);
  return t & ~3;
}

int32_t outer_tile_elems(int32_t m) {
  // The outer step moves 8m+16 bytes per element, so its tiles hold fewer
  // elements as m grows: about 512 KiB of traffic per tile.
  int32_t dflt = 4096;
  if (m >= 16) dflt = 2048;
  if (m <= 2) dflt = 8192;
  int32_t t = env_int("SLOWMO_OUTER_TILE", dflt, 256, 1 << 20);
  return t & ~3;
}

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

void plan_local(int32_t m, int32_t n_tensors, const int64_t *numel, int32_t tile_elems,
                std::vector<PlanRun> &runs, std::vector<int32_t> &tile_begin) {
  runs.clear();
  tile_begin.clear();
  tile_begin.push_back(0);
  int64_t fill = 0;  // budget used in the open tile
  auto close_tile = [&]() {
    if (static_cast<int32_t>(runs.size()) > tile_begin.back()) {
      tile_begin.push_back(static_cast<int32_t>(runs.size()));
    }
    fill = 0;
  };
  for (int32_t w = 0; w < m; ++w) {
    for (int32_t j = 0; j < n_tensors; ++j) {
      int64_t left = numel[j], off = 0;
      while (left > 0) {
        int64_t room = tile_elems - fill;
        if (room < kMinRunCost) {
          close_tile();
          continue;
        }
        int64_t n = std::min(left, room);
        if (n < left) n &= ~int64_t(3);  // the rest of the tensor continues 16-byte aligned
        PlanRun r;
        r.tile = static_cast<int32_t>(tile_begin.size()) - 1;
        r.worker = w;
        r.tensor = j;
        r.n = static_cast<int32_t>(n);
        r.offset = off;
        runs.push_back(r);
        fill += std::max<int64_t>(n, kMinRunCost);
        off += n;
        left -= n;
        if (tile_elems - fill < kMinRunCost) close_tile();
      }
    }
  }
  close_tile();
}

void plan_outer(int32_t n_tensors, const int64_t *numel, int32_t tile_elems,
                std::vector<PlanRun> &runs) {
  runs.clear();
  for (int32_t j = 0; j < n_tensors; ++j) {
    for (int64_t off = 0; off < numel[j]; off += tile_elems) {
      PlanRun r;
      r.tile = static_cast<int32_t>(runs.size());
      r.worker = -1;
      r.tensor = j;
      r.n = static_cast<int32_t>(std::min<int64_t>(tile_elems, numel[j] - off));
      r.offset = off;
      runs.push_back(r);
    }
  }
}

}  // namespace slowmo
