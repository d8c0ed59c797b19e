// Host-side tiling of the tensor list into workgroup-sized units of work, and
// the device-visible descriptors the kernels read.  No HIP calls here.
#pragma once

#include <cstdint>
#include <vector>

namespace slowmo {

// Elements of padding granularity in the state arena: every tensor's slice of
// x0 / u / h / v starts at a multiple of 64 floats (256 bytes), so that the
// state side of a run is 16-byte aligned whenever the run starts at a
// multiple of 4 elements of its tensor.
constexpr int64_t kArenaAlign = 64;

// A run inside a local-step tile costs at least this many elements of the
// tile's budget, which bounds the number of runs per tile.
constexpr int32_t kMinRunCost = 512;
constexpr int32_t kMaxLocalTile = 65536;
constexpr int32_t kMaxRunsPerTile = kMaxLocalTile / kMinRunCost;  // LDS staging capacity

// One contiguous run of elements of one (worker, tensor) in the local step.
// 32 bytes; staged into LDS by the workgroup that owns the tile.
struct LocalRun {
  float *x;        // device: first element of the run in the worker's replica
  int64_t so;      // element offset of the run in the h / v arena (includes worker * d_pad)
  int64_t go;      // element offset of the run inside its tensor (for the gradient pointer)
  int32_t slot;    // worker * n_tensors + tensor: index into the per-call gradient table
  int32_t n;       // elements
};
static_assert(sizeof(LocalRun) == 32, "LocalRun layout");

// One tile of the outer step: a contiguous run of one tensor, all m replicas.
struct OuterRun {
  int64_t fo;      // element offset in the x0 / u arena
  int64_t eo;      // element offset inside the tensor (added to every replica pointer)
  int32_t tensor;
  int32_t n;
};
static_assert(sizeof(OuterRun) == 24, "OuterRun layout");

struct Layout {
  std::vector<int64_t> arena_off;  // per tensor, start in the per-worker arena (elements)
  int64_t d = 0;                   // total elements
  int64_t d_pad = 0;               // arena length per worker (elements, multiple of kArenaAlign)
};

struct PlanRun {  // host description of a run (mirrors slowmo_plan_run)
  int32_t tile, worker, tensor, n;
  int64_t offset;
};

Layout make_layout(int32_t n_tensors, const int64_t *numel);

// Packs all (worker, tensor) element ranges, worker-major, into tiles of
// about tile_elems elements.  A tile holds one or more runs; small tensors
// share a tile.  Splits inside a tensor fall on multiples of 4 elements.
void plan_local(int32_t m, int32_t n_tensors, const int64_t *numel, int32_t tile_elems,
                std::vector<PlanRun> &runs, std::vector<int32_t> &tile_begin);

// One run per tile: every tensor is cut into pieces of tile_elems elements.
void plan_outer(int32_t n_tensors, const int64_t *numel, int32_t tile_elems,
                std::vector<PlanRun> &runs);

// Tuned tile sizes (elements); environment variables SLOWMO_LOCAL_TILE and
// SLOWMO_OUTER_TILE override them (for tuning runs).
int32_t local_tile_elems();
int32_t outer_tile_elems(int32_t m);

}  // namespace slowmo
