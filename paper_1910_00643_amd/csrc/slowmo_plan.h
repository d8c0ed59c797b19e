// Host-side tiling of the tensor list into workgroup-sized units of work, and
// the device-visible descriptors the kernels read.  No HIP calls here.
//
// Measured on MI355X: the stream mix of this path (3-4 reads, 2-3 writes per
// element) runs fastest with many short-lived workgroups that each move one
// 16-byte vector per lane and retire, dispatched in memory order; looping
// (persistent) workgroups and larger tiles lose 15-20 % of bandwidth.  A tile
// is therefore small, and holds exactly one contiguous run of one tensor.
#pragma once

#include <cstdint>
#include <vector>

namespace slowmo {

// Every tensor's slice of x0 / u / h / v starts at a multiple of 64 floats
// (256 bytes) in the state arena, so the state side of a tile is 16-byte
// aligned (tiles start at multiples of 4 elements of their tensor).
constexpr int64_t kArenaAlign = 64;

constexpr int32_t kLocalBlock = 256;                 // threads per workgroup, local step
constexpr int32_t kLocalTile = 4 * kLocalBlock;      // elements per tile: one vec4 per lane
constexpr int32_t kOuterBlock = 256;
constexpr int32_t kOuterTile = 4 * kOuterBlock;

// Local step: one tile = up to kLocalTile elements of one (worker, tensor).
struct LocalTile {
  int64_t go;      // element offset of the tile inside its tensor
  int32_t slot;    // worker * n_tensors + tensor
  int32_t n;       // elements in the tile (1..kLocalTile)
};
static_assert(sizeof(LocalTile) == 16, "LocalTile layout");

// Per (worker, tensor), fixed at create.
struct SlotInfo {
  float *x;        // device: the worker's replica of the tensor
  int64_t so;      // element offset of the tensor in the h / v arena (includes worker * d_pad)
};
static_assert(sizeof(SlotInfo) == 16, "SlotInfo layout");

// Outer step: one tile = up to kOuterTile elements of one tensor, all m replicas.
struct OuterTile {
  int64_t fo;      // element offset in the x0 / u arena
  int64_t eo;      // element offset inside the tensor (added to every replica pointer)
  int32_t tensor;
  int32_t n;       // elements; bit 30 set: some replica pointer of this tensor is not
                   // 16-byte aligned (element-wise path)
};
static_assert(sizeof(OuterTile) == 24, "OuterTile layout");
constexpr int32_t kOuterUnalignedBit = 1 << 30;

struct Layout {
  std::vector<int64_t> arena_off;  // per tensor, start in the per-worker arena (elements)
  int64_t d = 0;                   // total elements
  int64_t d_pad = 0;               // arena length per worker (elements, multiple of kArenaAlign)
};

struct PlanRun {  // host description of a tile (mirrors slowmo_plan_run)
  int32_t tile, worker, tensor, n;
  int64_t offset;
};

Layout make_layout(int32_t n_tensors, const int64_t *numel);

// Number of tiles of each kind (no allocation).
int64_t count_local_tiles(int32_t m, int32_t n_tensors, const int64_t *numel);
int64_t count_outer_tiles(int32_t n_tensors, const int64_t *numel);

// Tiles in launch order: worker-major, tensors in list order, offsets ascending.
void plan_local(int32_t m, int32_t n_tensors, const int64_t *numel, std::vector<PlanRun> &runs);
void plan_outer(int32_t n_tensors, const int64_t *numel, std::vector<PlanRun> &runs);

}  // namespace slowmo
