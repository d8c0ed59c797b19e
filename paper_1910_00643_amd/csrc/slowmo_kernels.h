// Launch interface between the C ABI (host logic) and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "slowmo_plan.h"

namespace slowmo {

struct LocalArgs {
  const TileRef *tiles;        // device, ntiles entries (owner = slot)
  const SlotInfo *slots;       // device, m * n_tensors entries
  const void *const *gtab;     // device: m * n_tensors gradient pointers of this call
  int32_t ntiles;
  float *h;                    // device: h arena, m * d_pad
  float *v;                    // device: v arena (Adam) or nullptr
  float lr;
  float wd;
  // SGD with Nesterov momentum
  float mu;
  // Adam: factors and reciprocal bias corrections 1 / (1 - beta^l)
  float b1, b2, omb1, omb2, rc1, rc2, eps;
};

struct OuterArgs {
  const TileRef *tiles;        // device, ntiles entries (owner = tensor)
  const TensorInfo *tensors;   // device, n_tensors entries
  float *const *xtab_t;        // device: replica pointers, tensor-major: [tensor * m + worker]
  int32_t ntiles;
  int32_t m;
  float *x0;                   // device: arena d_pad
  float *u;                    // device: arena d_pad
  float lr;                    // gamma_t (scaled per tensor in the kernel)
  float alpha;                 // slow learning rate; (alpha * gamma_t) is rounded once to fp32
  float beta;
  float m_f;                   // (float) m
  // buffer strategy "average": arenas to average over the workers (nullptr = skip)
  float *avg_h;
  float *avg_v;
  int64_t d_pad;               // worker stride of the arenas, elements
};

// Outer step without the exact average: lines 7-8 per (worker, element) with
// per-worker x0 and u arenas (m * d_pad each), over the local-step tiles.
struct OuterNoAvgArgs {
  const TileRef *tiles;        // device (owner = slot)
  const SlotInfo *slots;       // device
  int32_t ntiles;
  float *x0;                   // device: m * d_pad
  float *u;                    // device: m * d_pad
  float lr, alpha, beta;
};

struct MixArgs {
  const TileRef *tiles;        // device: outer-step tiles (owner = tensor)
  const TensorInfo *tensors;   // device
  float *const *xtab_t;        // device: replica pointers, tensor-major
  int32_t ntiles;
  int32_t m;
  const MixEntry *seq;         // device: len entries
  int32_t len;
};

// De-biased parameters of push-sum: z^{(i)} = x^{(i)} / w_i, over the local tiles.
struct DebiasArgs {
  const TileRef *tiles;        // device (owner = slot)
  const SlotInfo *slots;       // device
  float *const *ztab;          // device: m * n_tensors destination pointers (worker-major)
  const float *w;              // device: m push-sum weights
  int32_t ntiles;
  int32_t n_tensors;
};

struct LaunchTuning {
  int32_t xcd_remap;    // 1: consecutive tiles go to the same XCD
  int32_t xcd_run;      // tiles an XCD takes in a row before the next XCD's run; 0 = one
                        // contiguous eighth of all tiles per XCD
  int32_t nontemporal;  // 1: streaming (non-temporal) loads and stores
  int32_t fuse_last;    // 1: slowmo_local_outer_step runs one fused kernel when it can
  int32_t fuse_mix;     // 1: slowmo_local_mix_step runs one fused kernel when it can
  int32_t big_tiles;    // 1: whole kBigTile pieces of aligned tensors go to the big-tile kernels
  int32_t outer_lds;    // bytes of (unused) dynamic LDS per outer-step workgroup: caps the
                        // number of resident wavefronts per CU (160 KiB / outer_lds); 0 = no cap
};

// base: 0 SGD-Nesterov, 1 Adam.  bf16: gradient dtype.  first: the stored
// h (and v) are to be read as zero (first step after a reset / after create).
// last: h (and v) are dead after this step and are not written.
hipError_t launch_local_step(const LocalArgs &a, int base, bool bf16, bool first, bool last,
                             const LaunchTuning &tune, hipStream_t stream);
hipError_t launch_outer_step(const OuterArgs &a, const LaunchTuning &tune, hipStream_t stream);
// The last local step of an outer iteration and the outer step in one pass
// (one workgroup = 256 elements of one tensor, all workers).  Requires every
// replica and gradient pointer to be 16-byte aligned (8 for bf16).  policy:
// 0 reset (buffers not stored), 1 maintain (stored), 2 average (their mean
// over the workers is stored).
hipError_t launch_local_outer_step(const LocalArgs &l, const OuterArgs &o, int32_t n_tensors,
                                   int base, bool bf16, bool first, int policy,
                                   const LaunchTuning &tune, hipStream_t stream);
// The same two operations on BIG tiles (a.tiles / o.tiles list whole kBigTile
// pieces, every one full and 16-byte aligned in every stream).  Results are
// bit-identical to the ordinary tiles'.  launch_outer_big handles no buffer
// average (a.avg_h must be NULL); launch_local_outer_big handles policies 0 and 1.
hipError_t launch_outer_big(const OuterArgs &a, const LaunchTuning &tune, hipStream_t stream);
hipError_t launch_local_outer_big(const LocalArgs &l, const OuterArgs &o, int32_t n_tensors,
                                  int base, bool bf16, bool first, int policy,
                                  const LaunchTuning &tune, hipStream_t stream);
// Copies worker 0's replica into x0 (x0_copies copies, d_pad apart) and into the
// replicas of workers 1..m-1; uses a.tiles, a.tensors, a.xtab_t, a.x0, a.d_pad, a.m.
hipError_t launch_init_broadcast(const OuterArgs &a, int32_t x0_copies, const LaunchTuning &tune,
                                 hipStream_t stream);
hipError_t launch_mix_step(const MixArgs &a, const LaunchTuning &tune,
                              hipStream_t stream);
// The local step and the mixing step that follows it in one kernel; x.seq must
// list EVERY worker (plan_mix with idle workers).  Needs 16-byte aligned
// replicas and gradient pointers that allow vector loads.
hipError_t launch_local_mix_step(const LocalArgs &l, const MixArgs &x, int64_t d_pad,
                                 int32_t n_tensors, int base, bool bf16, bool first,
                                 const LaunchTuning &tune, hipStream_t stream);
hipError_t launch_debias(const DebiasArgs &a, const LaunchTuning &tune, hipStream_t stream);

// Static device memory for the entry point that allocates nothing: room for
// the de-bias table (destination pointers, then the push-sum weights) of up to
// kStaticMaxPointers (worker, tensor) pairs.
constexpr size_t kStaticMaxPointers = 65536;
constexpr size_t kStaticMaxWorkers = 1024;
constexpr size_t kStaticScratchBytes =
    kStaticMaxPointers * sizeof(void *) + kStaticMaxWorkers * sizeof(float);
// Address of that memory on `device`.  The first call for a device must be made
// with that device current (it asks the runtime for the symbol's address
// there); later calls return the remembered address without any HIP call.
hipError_t static_scratch(int device, void **ptr);
hipError_t launch_outer_noavg_step(const OuterNoAvgArgs &a, const LaunchTuning &tune,
                                   hipStream_t stream);

}  // namespace slowmo
