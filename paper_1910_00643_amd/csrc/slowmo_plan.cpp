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

int64_t count_big_tiles(int32_t n_tensors, const int64_t *numel) {
  int64_t t = 0;
  for (int32_t j = 0; j < n_tensors; ++j) t += numel[j] / kBigTile;
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

// Mixing step for any map with at most one in-neighbour per worker.  A sender
// j splits its mass evenly over itself and its outdeg(j) receivers, so
// p(i,j) = 1 / (1 + outdeg(j)) and P is column-stochastic (Algorithm C.1).
// The replicas are mixed in place: a worker is overwritten only after every
// worker that receives from it has been served.  Seen as "i points to
// in_peer[i]", the map is a forest of trees hanging off cycles and fixed
// points.  Each tree is listed receivers-first (post-order), a sender's
// receivers that have receivers of their own before those that have none:
// then a worker is mostly followed by its source, whose old value the kernel
// already holds in a register, and receivers of one sender that follow each
// other share that register.  A cycle comes after the trees of its members,
// each member before its source.
void plan_mix(int32_t m, const int32_t *in_peer, std::vector<MixEntry> &seq,
              std::vector<float> &share, bool with_idle) {
  std::vector<int32_t> outdeg(m, 0);
  for (int32_t i = 0; i < m; ++i)
    if (in_peer[i] != i) ++outdeg[in_peer[i]];
  share.resize(m);
  for (int32_t j = 0; j < m; ++j) share[j] = 1.0f / static_cast<float>(1 + outdeg[j]);

  // which workers lie on a cycle: peel those nobody (left) receives from
  std::vector<int32_t> pending = outdeg, queue;
  std::vector<char> in_tree(m, 0);
  queue.reserve(m);
  for (int32_t i = 0; i < m; ++i)
    if (pending[i] == 0) queue.push_back(i);
  for (size_t q = 0; q < queue.size(); ++q) {
    const int32_t i = queue[q];
    in_tree[i] = 1;
    const int32_t j = in_peer[i];
    if (j != i && --pending[j] == 0) queue.push_back(j);
  }
  // receivers of every worker that are tree workers: first those that have
  // receivers themselves, then those that have none (CSR layout)
  std::vector<int32_t> start(m + 1, 0), recv(m);
  for (int32_t i = 0; i < m; ++i)
    if (in_peer[i] != i && in_tree[i]) ++start[in_peer[i] + 1];
  for (int32_t j = 0; j < m; ++j) start[j + 1] += start[j];
  {
    std::vector<int32_t> fill(start.begin(), start.end() - 1);
    for (int pass = 0; pass < 2; ++pass)
      for (int32_t i = 0; i < m; ++i)
        if (in_peer[i] != i && in_tree[i] && (outdeg[i] == 0) == (pass == 1))
          recv[fill[in_peer[i]]++] = i;
  }

  seq.clear();
  seq.reserve(m);
  auto emit = [&](int32_t i) {
    if (in_peer[i] != i) {
      seq.push_back({i, in_peer[i], share[i], share[in_peer[i]], 0, 0});
    } else if (outdeg[i] > 0 || with_idle) {
      seq.push_back({i, i, share[i], 0.f, kMixNoSrc, 0});
    }  // else: an idle worker keeps its value
  };
  // post-order walk of the tree below `root`; the root itself is listed only
  // if it is a tree worker (cycle members wait for their cycle)
  std::vector<std::pair<int32_t, int32_t>> stack;  // (worker, next receiver to visit)
  auto walk = [&](int32_t root) {
    stack.push_back({root, start[root]});
    while (!stack.empty()) {
      auto &top = stack.back();
      if (top.second < start[top.first + 1]) {
        const int32_t c = recv[top.second++];
        stack.push_back({c, start[c]});
      } else {
        if (in_tree[top.first]) emit(top.first);
        stack.pop_back();
      }
    }
  };
  // One group per connected set of workers: a fixed point with everything that
  // hangs off it, or a cycle with the trees of its members.  Groups share no
  // worker, so they may run as separate launches.
  std::vector<size_t> group_start;
  for (int32_t r = 0; r < m; ++r) {
    if (!(in_tree[r] && in_peer[r] == r)) continue;
    const size_t at = seq.size();
    walk(r);
    if (seq.size() > at) group_start.push_back(at);
  }
  std::vector<char> seen(m, 0);
  for (int32_t i = 0; i < m; ++i) {
    if (in_tree[i] || seen[i]) continue;
    group_start.push_back(seq.size());
    for (int32_t j = i; !seen[j]; j = in_peer[j]) {
      seen[j] = 1;
      walk(j);  // the trees of the cycle's members first
    }
    const size_t first = seq.size();
    for (int32_t j = i; seen[j] == 1; j = in_peer[j]) {
      seen[j] = 2;
      emit(j);
    }
    seq[first].flags |= kMixSaveFirst;
    seq.back().flags |= kMixSrcFromFirst;
  }
  for (size_t at : group_start) seq[at].flags |= kMixGroupStart;
  // Operands the kernel still holds when an entry needs them.  `held`: the
  // worker whose old value is in the source register (the previous entry's
  // source).  saved[k]: the worker whose old value was copied into saved
  // register k when another source took its place in the source register,
  // because it is needed again (by a later receiver, or at its own turn, which
  // is always its last use); the register is free again after that turn.
  std::vector<int32_t> last_use(m, -1);
  for (size_t idx = 0; idx < seq.size(); ++idx) {
    if (!(seq[idx].flags & kMixNoSrc)) last_use[seq[idx].src] = static_cast<int32_t>(idx);
    last_use[seq[idx].node] = static_cast<int32_t>(idx);
  }
  int32_t held = -1, saved[kMixSaved];
  for (int32_t &w : saved) w = -1;
  auto saved_in = [&](int32_t w) {
    for (int k = 0; k < kMixSaved; ++k)
      if (w >= 0 && saved[k] == w) return k;
    return -1;
  };
  for (size_t idx = 0; idx < seq.size(); ++idx) {
    MixEntry &e = seq[idx];
    if (e.flags & kMixGroupStart) {
      held = -1;
      for (int32_t &w : saved) w = -1;
    }
    const int own_saved = saved_in(e.node);
    if (e.node == held) {
      e.flags |= kMixOwnFromS;
    } else if (own_saved >= 0) {
      e.flags |= (own_saved + 1) << kMixOwnSavedShift;
    }
    if (own_saved >= 0) saved[own_saved] = -1;  // the worker's own turn is its last use
    if (e.flags & kMixNoSrc) continue;
    const bool from_first = (e.flags & kMixSrcFromFirst) != 0;
    if (!from_first && e.src == held) {
      e.flags |= kMixSrcFromS;
      continue;
    }
    // the source register gets a new value: keep the old one if it is needed again
    if (held >= 0 && last_use[held] > static_cast<int32_t>(idx) && saved_in(held) < 0) {
      for (int k = 0; k < kMixSaved; ++k) {
        if (saved[k] < 0) {
          saved[k] = held;
          e.flags |= (k + 1) << kMixSaveShift;
          break;
        }
      }
    }
    const int src_saved = from_first ? -1 : saved_in(e.src);
    if (src_saved >= 0) e.flags |= (src_saved + 1) << kMixSrcSavedShift;
    held = e.src;
  }
}

}  // namespace slowmo
