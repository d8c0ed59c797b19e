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

#ifndef SLOWMO_LOCAL_BLOCK
#define SLOWMO_LOCAL_BLOCK 64
#endif
#ifndef SLOWMO_OUTER_BLOCK
#define SLOWMO_OUTER_BLOCK 64
#endif
// Threads per workgroup; a tile is one vec4 per lane.  Single-wavefront
// workgroups measured best for both kernels (64 > 128 > 256 > 512).
constexpr int32_t kLocalBlock = SLOWMO_LOCAL_BLOCK;
constexpr int32_t kLocalTile = 4 * kLocalBlock;
constexpr int32_t kOuterBlock = SLOWMO_OUTER_BLOCK;
constexpr int32_t kOuterTile = 4 * kOuterBlock;

// Big tiles of the outer step and of the fused last step: one 1024-thread
// workgroup takes kBigVpt vectors per lane, i.e. 256 KiB of every stream it
// walks (its 16 waves start together and move from replica to replica
// together).  Measured in one process on the same replicas against the
// single-wave tiles: the fused last step is 10-14 % faster at m = 32, 6-7 % at
// m = 16, 3-5 % at m = 8 and no faster at m = 4; the plain outer step 8 % faster
// at m = 32 and within +-4 % at m = 8.  Smaller shapes (128 or 64 KiB per stream
// and workgroup) gain half of that or nothing.  Under "maintain" the fused
// kernel stores every worker's buffers inside the walk and is 2-10 % slower in
// this shape than in single waves, so it takes big tiles only under "reset".
// Used for the whole kBigTile pieces of aligned tensors from these worker
// counts on:
constexpr int32_t kBigBlock = 1024;
constexpr int32_t kBigVpt = 16;
constexpr int32_t kBigTile = 4 * kBigBlock * kBigVpt;
constexpr int32_t kBigFusedFromWorkers = 8;
constexpr int32_t kBigOuterFromWorkers = 16;
// ... and only when there are enough of them to occupy the chip: one big tile
// keeps one of the 256 CUs busy.  Measured on one tensor of k big tiles (m = 8
// and 32): twice as slow as single-wave tiles at k = 64, 6-17 % slower at
// k = 128, 4-15 % faster from k = 173 on.
constexpr int32_t kBigMinTiles = 160;
static_assert(kBigTile % kOuterTile == 0, "a big tile is a whole number of ordinary tiles");

// One tile of either kernel: the k-th piece of a tensor.  For the local step
// `owner` is the slot (worker * n_tensors + tensor); for the outer step it is
// the tensor.  8 bytes, read with one scalar load.
struct TileRef {
  int32_t owner;
  int32_t k;
};
static_assert(sizeof(TileRef) == 8, "TileRef layout");

// Per (worker, tensor), fixed at create.
struct SlotInfo {
  float *x;        // device: the worker's replica of the tensor
  int64_t so;      // element offset of the tensor in the h / v arena (includes worker * d_pad)
  int64_t numel;   // elements in the tensor
  float wd;        // weight decay of this tensor
  float lr_scale;  // the tensor's fast learning rate is lr * lr_scale
};
static_assert(sizeof(SlotInfo) == 32, "SlotInfo layout");

// Per tensor, fixed at create (outer step).
struct TensorInfo {
  int64_t fo;         // element offset of the tensor in the x0 / u arena
  int64_t numel;
  int64_t unaligned;  // non-zero: some replica of this tensor is not 16-byte aligned
  float lr_scale;     // the tensor's fast learning rate is lr * lr_scale
  float wd;           // weight decay of this tensor
};
static_assert(sizeof(TensorInfo) == 32, "TensorInfo layout");

struct Layout {
  std::vector<int64_t> arena_off;  // per tensor, start in the per-worker arena (elements)
  int64_t d = 0;                   // total elements
  int64_t d_pad = 0;               // arena length per worker (elements, multiple of kArenaAlign)
};

struct PlanRun {  // host description of a tile (mirrors slowmo_plan_run)
  int32_t tile, worker, tensor, n;
  int64_t offset;
};

// Mixing step of gradient push (any in-neighbour map, column-stochastic weights).  The
// workers are listed in an order in which every worker comes before the worker
// it receives from, so that old values are still in memory when they are
// needed; the members of a cycle follow each other, each before its source,
// and the last one takes the first one's old value from a register.  Where an
// operand is the previous entry's source it is taken from a register too.
// Two more registers ("saved" operands) keep a sender whose later receivers or
// own turn come only after other senders have passed through the source
// register, so that it is not read (in the fused kernel: stepped) again.
constexpr int32_t kMixSaved = 4;
enum MixFlag : int32_t {
  kMixOwnFromS = 1,      // the worker's old value is the previous entry's source value
  kMixSrcFromS = 2,      // same source as the previous entry
  kMixSrcFromFirst = 4,  // the source is the worker that opened the cycle
  kMixSaveFirst = 8,     // this worker opens a cycle: keep its old value
  kMixNoSrc = 16,        // receives from nobody: x <- a * x
  kMixGroupStart = 32,   // first entry of a connected group of workers (for the launcher only)
};
// Three 3-bit fields above the flag bits, each 0 (no) or 1 + the number of a
// saved register:
//   save : before this entry's source replaces the held source value, the held
//          one is copied into that saved register;
//   own  : the worker's old value is in that saved register;
//   src  : the source value is in that saved register (and becomes the held
//          source value again).
constexpr int32_t kMixSaveShift = 6, kMixOwnSavedShift = 9, kMixSrcSavedShift = 12;
constexpr int32_t kMixFieldMask = 7;
constexpr int32_t mix_save(int32_t flags) { return (flags >> kMixSaveShift) & kMixFieldMask; }
constexpr int32_t mix_own_saved(int32_t flags) { return (flags >> kMixOwnSavedShift) & kMixFieldMask; }
constexpr int32_t mix_src_saved(int32_t flags) { return (flags >> kMixSrcSavedShift) & kMixFieldMask; }
static_assert(kMixSaved <= kMixFieldMask, "register numbers must fit the fields");
struct MixEntry {
  int32_t node;    // worker updated by this entry
  int32_t src;     // worker it receives from (the worker itself with kMixNoSrc)
  float a;         // p(node, node) = 1 / (1 + outdeg(node))
  float b;         // p(node, src)  = 1 / (1 + outdeg(src))
  int32_t flags;   // MixFlag bits
  int32_t pad_;
};
static_assert(sizeof(MixEntry) == 24, "MixEntry layout");
// The update order of one mixing step for the in-neighbour map in_peer (m
// entries in 0..m-1); share[j] = 1 / (1 + outdeg(j)).  Workers that neither
// send nor receive get no entry unless with_idle is set (then: a = 1, kMixNoSrc).
void plan_mix(int32_t m, const int32_t *in_peer, std::vector<MixEntry> &seq,
              std::vector<float> &share, bool with_idle = false);

Layout make_layout(int32_t n_tensors, const int64_t *numel);

// Number of tiles of each kind (no allocation).
int64_t count_local_tiles(int32_t m, int32_t n_tensors, const int64_t *numel);
int64_t count_outer_tiles(int32_t n_tensors, const int64_t *numel);
// Whole kBigTile pieces over all tensors (an upper bound on the big tiles in use).
int64_t count_big_tiles(int32_t n_tensors, const int64_t *numel);

// Tiles in launch order: worker-major, tensors in list order, offsets ascending.
void plan_local(int32_t m, int32_t n_tensors, const int64_t *numel, std::vector<PlanRun> &runs);
void plan_outer(int32_t n_tensors, const int64_t *numel, std::vector<PlanRun> &runs);

}  // namespace slowmo
