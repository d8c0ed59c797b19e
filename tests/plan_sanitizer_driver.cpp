// Host-side planning code (tiling, mixing order) under AddressSanitizer and
// UBSan: built from csrc/slowmo_plan.cpp alone (no HIP), run on random tensor
// lists and random in-neighbour maps up to the largest worker count.  Prints
// OK; any out-of-bounds access, undefined operation or broken invariant aborts.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "slowmo_plan.h"

using namespace slowmo;

#define REQUIRE(c)                                                         \
  do {                                                                     \
    if (!(c)) {                                                            \
      std::fprintf(stderr, "line %d: requirement failed: %s\n", __LINE__, #c); \
      std::abort();                                                        \
    }                                                                      \
  } while (0)

static void check_tiling(std::mt19937_64 &rng) {
  const int sizes[] = {0, 1, 3, 4, 5, 255, 256, 257, 1023, 1024, 1025, 70001};
  for (int rep = 0; rep < 40; ++rep) {
    const int32_t m = 1 + static_cast<int32_t>(rng() % 5);
    const int32_t nt = 1 + static_cast<int32_t>(rng() % 9);
    std::vector<int64_t> numel(nt);
    for (auto &n : numel) n = sizes[rng() % (sizeof(sizes) / sizeof(sizes[0]))];
    const Layout L = make_layout(nt, numel.data());
    REQUIRE(L.d_pad % kArenaAlign == 0 && L.d_pad >= L.d);
    std::vector<PlanRun> lr, orr;
    plan_local(m, nt, numel.data(), lr);
    plan_outer(nt, numel.data(), orr);
    REQUIRE(static_cast<int64_t>(lr.size()) == count_local_tiles(m, nt, numel.data()));
    REQUIRE(static_cast<int64_t>(orr.size()) == count_outer_tiles(nt, numel.data()));
    std::vector<int64_t> covered(static_cast<size_t>(m) * nt, 0), covered_o(nt, 0);
    for (const PlanRun &r : lr) {
      REQUIRE(r.worker >= 0 && r.worker < m && r.tensor >= 0 && r.tensor < nt);
      REQUIRE(r.n > 0 && r.n <= kLocalTile && r.offset == covered[r.worker * nt + r.tensor]);
      covered[r.worker * nt + r.tensor] += r.n;
    }
    for (const PlanRun &r : orr) {
      REQUIRE(r.tensor >= 0 && r.tensor < nt && r.n > 0 && r.n <= kOuterTile);
      REQUIRE(r.offset == covered_o[r.tensor]);
      covered_o[r.tensor] += r.n;
    }
    for (int32_t w = 0; w < m; ++w)
      for (int32_t j = 0; j < nt; ++j) REQUIRE(covered[w * nt + j] == numel[j]);
    for (int32_t j = 0; j < nt; ++j) REQUIRE(covered_o[j] == numel[j]);
  }
}

// Replays the entries on one array the way the kernel does (its registers) and
// compares with the update computed from a saved copy.
static void check_mix(int32_t m, const std::vector<int32_t> &peer) {
  std::vector<MixEntry> seq;
  std::vector<float> share;
  plan_mix(m, peer.data(), seq, share);
  REQUIRE(static_cast<int32_t>(seq.size()) <= m && static_cast<int32_t>(share.size()) == m);
  std::vector<float> x(m), want(m);
  for (int32_t i = 0; i < m; ++i) x[i] = 1.0f + 0.37f * static_cast<float>(i % 97);
  for (int32_t i = 0; i < m; ++i) {
    float v = share[i] * x[i];
    if (peer[i] != i) v = v + share[peer[i]] * x[peer[i]];
    want[i] = v;
  }
  REQUIRE(seq.empty() || (seq[0].flags & kMixGroupStart));
  std::vector<char> written(m, 0);
  float S = 0.f, first = 0.f, H[kMixSaved + 1] = {};           // saved registers, numbered from 1
  bool s_valid = false, first_valid = false, h_valid[kMixSaved + 1] = {};
  int64_t reads = 0;
  for (const MixEntry &e : seq) {
    REQUIRE(e.node >= 0 && e.node < m && e.src >= 0 && e.src < m && !written[e.node]);
    if (e.flags & kMixGroupStart) {     // a launch of its own: registers start empty
      s_valid = first_valid = false;
      for (bool &v : h_valid) v = false;
    }
    REQUIRE(mix_save(e.flags) <= kMixSaved && mix_own_saved(e.flags) <= kMixSaved &&
            mix_src_saved(e.flags) <= kMixSaved);
    float own;
    if (e.flags & kMixOwnFromS) {
      REQUIRE(s_valid);
      own = S;
    } else if (mix_own_saved(e.flags)) {
      const int k = mix_own_saved(e.flags);
      REQUIRE(h_valid[k]);
      own = H[k];
    } else {
      own = x[e.node];
      ++reads;
    }
    if (e.flags & kMixSaveFirst) {
      first = own;
      first_valid = true;
    }
    if (e.flags & kMixNoSrc) {
      REQUIRE(peer[e.node] == e.node);
      x[e.node] = e.a * own;
    } else {
      REQUIRE(e.src == peer[e.node] && e.src != e.node);
      if (mix_save(e.flags)) {
        REQUIRE(s_valid);
        H[mix_save(e.flags)] = S;
        h_valid[mix_save(e.flags)] = true;
      }
      if (e.flags & kMixSrcFromFirst) {
        REQUIRE(first_valid);
        S = first;
      } else if (mix_src_saved(e.flags)) {
        const int k = mix_src_saved(e.flags);
        REQUIRE(h_valid[k]);
        S = H[k];
      } else if (e.flags & kMixSrcFromS) {
        REQUIRE(s_valid);
      } else {
        REQUIRE(!written[e.src]);
        S = x[e.src];
        ++reads;
      }
      s_valid = true;
      x[e.node] = e.a * own + e.b * S;
    }
    written[e.node] = 1;
  }
  REQUIRE(reads <= 2 * static_cast<int64_t>(seq.size()));
  for (int32_t i = 0; i < m; ++i) {
    REQUIRE(std::memcmp(&x[i], &want[i], sizeof(float)) == 0);
    if (!written[i]) {  // idle: no sender, no receiver
      REQUIRE(peer[i] == i);
      for (int32_t j = 0; j < m; ++j) REQUIRE(j == i || peer[j] != i);
    }
  }
}

int main() {
  std::mt19937_64 rng(1910);
  check_tiling(rng);
  const int32_t ms[] = {1, 2, 3, 4, 7, 8, 33, 64, 255, 1024};
  for (int32_t m : ms) {
    std::vector<int32_t> peer(m);
    for (int rep = 0; rep < 25; ++rep) {
      for (auto &p : peer) p = static_cast<int32_t>(rng() % m);  // any map
      check_mix(m, peer);
      for (int32_t i = 0; i < m; ++i) peer[i] = i;                // a permutation with fixed points
      for (int32_t i = m - 1; i > 0; --i)
        if (rng() % 4) std::swap(peer[i], peer[rng() % (i + 1)]);
      check_mix(m, peer);
    }
    for (int32_t i = 0; i < m; ++i) peer[i] = 0;                  // star
    check_mix(m, peer);
    for (int32_t i = 0; i < m; ++i) peer[i] = i + 1 < m ? i + 1 : i;  // chain
    check_mix(m, peer);
    for (int32_t i = 0; i < m; ++i) peer[i] = (i + 1) % m;        // one cycle
    check_mix(m, peer);
    for (int32_t i = 0; i < m; ++i) peer[i] = i;                  // everybody idle
    check_mix(m, peer);
  }
  std::puts("OK");
  return 0;
}
