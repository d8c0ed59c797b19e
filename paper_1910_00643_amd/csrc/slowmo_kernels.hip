// gfx950 kernels of the Slow Momentum hot path.
//
// k_local_step         Algorithm 1 lines 3-5 for all workers (Table C.1 rows SGD, Adam)
// k_outer_step         lines 6-8 + copy into every replica (+ "average" buffer strategy)
// k_local_outer_step   the last local step of an outer iteration fused with the outer step
// k_outer_big, k_local_outer_big   the same two on 65 536-element pieces (many workers)
// k_init_broadcast     Algorithm 1 "Input": x_{0,0} into x0 and every replica
// k_outer_noavg        lines 7-8 per worker, without line 6 (Section 6)
// k_mix_step        mixing step of stochastic gradient push (Algorithm C.1)
// k_local_mix_step     a local step and the mixing step that follows it, fused
// k_debias             de-biased parameters of stochastic gradient push (Algorithm C.1)
//
// All of them are pure streams: every byte is read once and written once, no
// element is reused, so there is no dense contraction and the matrix cores are
// not involved.  The shape that measured fastest on MI355X for this read/write
// mix:
//   * one 16-byte vector per lane and per stream -- a wavefront instruction is
//     one contiguous 1 KiB burst;
//   * small workgroups that load, compute, store and retire (no loop): their
//     stores do not hold a wave slot, reads and writes of neighbouring
//     workgroups interleave, and the set of addresses in flight is a compact
//     window that moves through memory in order;
//   * non-temporal loads and stores (nothing is reused);
//   * workgroup -> tile mapping that gives each XCD one contiguous range of
//     tiles (workgroups are dealt to the 8 XCDs round-robin);
//   * tile descriptors and pointer tables read with scalar loads: they are
//     uniform over the workgroup, so they live in SGPRs, not in LDS.
//
// Compiled with -ffp-contract=off: products and sums are rounded separately,
// in the order written here, which is the order of Table C.1 and Eq. (2)-(3).
#include "slowmo_kernels.h"

#include <mutex>

// Device memory of the allocation-free entry point (slowmo_debias_static): the
// table its kernel reads.  One copy per GPU, held until the process ends.  In
// host code this name is only a handle for hipGetSymbolAddress -- the address
// kernels and copies use is the one static_scratch() returns.
static __device__ __align__(256) unsigned char scratch[slowmo::kStaticScratchBytes];

namespace slowmo {

namespace {

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

}  // namespace

hipError_t static_scratch(int device, void **ptr) {
  *ptr = nullptr;
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    int current = -1;
    hipError_t e = hipGetDevice(&current);
    if (e != hipSuccess) return e;
    if (current != device) return hipErrorInvalidDevice;  // each GPU has its own copy and address
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[device] = p;
  }
  *ptr = g_scratch_ptr[device];
  return hipSuccess;
}

namespace {

constexpr int kXcd = 8;  // XCDs per MI355X; workgroups are dealt to them round-robin

typedef float V4 __attribute__((ext_vector_type(4)));
typedef uint32_t U2 __attribute__((ext_vector_type(2)));

// Pointers that were themselves loaded from memory (replica and gradient
// tables) have no known address space, and the compiler would use flat
// accesses for them.  They are global memory: say so, to get global_load /
// global_store.
#define SLOWMO_GLOBAL __attribute__((address_space(1)))
typedef SLOWMO_GLOBAL V4 GV4;
typedef SLOWMO_GLOBAL U2 GU2;

template <typename T>
__device__ __forceinline__ SLOWMO_GLOBAL T *as_global(const void *p) {
  return (SLOWMO_GLOBAL T *)(reinterpret_cast<uintptr_t>(p));
}

template <bool NT>
__device__ __forceinline__ V4 ld4(const float *p) {
  const GV4 *q = as_global<V4>(p);
  if constexpr (NT) return __builtin_nontemporal_load(q);
  return *q;
}
template <bool NT>
__device__ __forceinline__ void st4(float *p, V4 v) {
  GV4 *q = as_global<V4>(p);
  if constexpr (NT) {
    __builtin_nontemporal_store(v, q);
  } else {
    *q = v;
  }
}
__device__ __forceinline__ float ld1(const float *p) { return *as_global<float>(p); }
__device__ __forceinline__ void st1(float *p, float v) { *as_global<float>(p) = v; }

// Gradient access: fp32 as is, bf16 widened exactly (the 16 bits become the
// high half of an fp32 word).
template <bool BF16>
__device__ __forceinline__ float ldg1(const void *g, int j) {
  if constexpr (BF16) {
    uint32_t w = as_global<uint16_t>(g)[j];
    return __uint_as_float(w << 16);
  } else {
    return as_global<float>(g)[j];
  }
}
template <bool BF16, bool NT>
__device__ __forceinline__ V4 ldg4(const void *g, int vec) {
  if constexpr (BF16) {
    const GU2 *p = as_global<U2>(g) + vec;
    U2 w = NT ? __builtin_nontemporal_load(p) : *p;
    V4 r;
    r.x = __uint_as_float(w.x << 16);
    r.y = __uint_as_float(w.x & 0xffff0000u);
    r.z = __uint_as_float(w.y << 16);
    r.w = __uint_as_float(w.y & 0xffff0000u);
    return r;
  } else {
    return ld4<NT>(reinterpret_cast<const float *>(g) + 4 * vec);
  }
}

// Tile of workgroup b.  Workgroup b runs on XCD b mod 8; with the remap, XCD c
// walks the contiguous tile range [c * chunk, (c + 1) * chunk), so each XCD's
// L2 and TLB see one compact window of every stream instead of a 1-in-8 comb.
__device__ __forceinline__ int tile_of(int b, int chunk, int run) {
  // run == 0: workgroup b takes tile b.  Otherwise the workgroups of one XCD
  // (b % 8) take runs of `run` consecutive tiles, the 8 XCDs side by side;
  // run == chunk gives every XCD one contiguous eighth of the tiles.
  if (run == 0) return b;
  const int q = b / kXcd, x = b % kXcd;
  return (q / run) * (kXcd * run) + x * run + q % run;
}

// ---- per-element arithmetic -------------------------------------------------

struct SgdP {
  float lr, mu, wd;
};
// Table C.1, SGD row, with the coupled weight-decay term.
template <bool FIRST>
__device__ __forceinline__ void sgd_elem(float &x, float &h, float g, const SgdP &p) {
  float grad = g + p.wd * x;
  float hn = FIRST ? grad : p.mu * h + grad;
  float dir = p.mu * hn + grad;
  h = hn;
  x = x - p.lr * dir;
}

struct AdamP {
  float lr, wd, b1, b2, omb1, omb2, rc1, rc2, eps;
};
// Table C.1, Adam row.  The two bias corrections are multiplications by
// reciprocals computed on the host in fp64; the root and the final quotient
// use the hardware's 1-ulp approximations, which keeps the kernel far from
// the VALU limit (an error of a few 1e-7 relative on the step, i.e. below
// 1e-9 absolute per step at the learning rates in use).
template <bool FIRST>
__device__ __forceinline__ void adam_elem(float &x, float &h, float &v, float g, const AdamP &p) {
  float grad = g + p.wd * x;
  float gsq = grad * grad;
  float hn = FIRST ? p.omb1 * grad : p.b1 * h + p.omb1 * grad;
  float vn = FIRST ? p.omb2 * gsq : p.b2 * v + p.omb2 * gsq;
  float hhat = hn * p.rc1;
  float vhat = vn * p.rc2;
  float den = __builtin_amdgcn_sqrtf(vhat) + p.eps;
  float dir = hhat * __builtin_amdgcn_rcpf(den);
  h = hn;
  v = vn;
  x = x - p.lr * dir;
}

struct OuterP {
  float lr, alpha_lr, beta, m_f, alpha;
};
// gamma_t of one tensor: lr * lr_scale, and (alpha * gamma_t), each rounded once.
__device__ __forceinline__ OuterP for_tensor(OuterP p, float lr_scale) {
  p.lr = p.lr * lr_scale;
  p.alpha_lr = p.alpha * p.lr;
  return p;
}
// Algorithm 1 lines 6-8 for one element, given the ordered sum s of the
// replicas.  Returns x_{t+1,0}.
__device__ __forceinline__ float outer_elem(float s, float x0, float &u, const OuterP &p) {
  float xbar = s / p.m_f;
  float diff = x0 - xbar;
  float un = p.beta * u + diff / p.lr;
  u = un;
  return x0 - p.alpha_lr * un;
}

// ---- local step ---------------------------------------------------------------
// One workgroup = one tile = up to 4 * blockDim elements of one (worker,
// tensor).  Lane t owns elements [4t, 4t + 4) of the tile.

// FIRST: the stored buffers are to be read as zero (not loaded).  LAST: the
// buffers are dead after this step (the reset policy discards them before
// their next use), so they are not stored.
template <int BASE, bool BF16, bool FIRST, bool LAST, bool NT>
__global__ __launch_bounds__(kLocalBlock) void k_local_step(
    const TileRef *__restrict__ tiles, const SlotInfo *__restrict__ slots,
    const void *const *__restrict__ gtab, float *__restrict__ hbase, float *__restrict__ vbase,
    int ntiles, int chunk, int remap, SgdP sp, AdamP ap) {
  const int tile = tile_of(blockIdx.x, chunk, remap);
  if (tile >= ntiles) return;
  const TileRef t = tiles[tile];         // uniform: scalar loads
  const SlotInfo s = slots[t.owner];
  // per-tensor hyper-parameters (uniform over the workgroup)
  sp.lr = sp.lr * s.lr_scale;
  sp.wd = s.wd;
  ap.lr = ap.lr * s.lr_scale;
  ap.wd = s.wd;
  constexpr int gsize = BF16 ? 2 : 4;
  const int64_t go = static_cast<int64_t>(t.k) * kLocalTile;  // offset of the tile in its tensor
  const void *g = static_cast<const char *>(gtab[t.owner]) + go * gsize;
  float *x = s.x + go;
  float *h = hbase + s.so + go;
  float *v = BASE == 1 ? vbase + s.so + go : nullptr;
  const int64_t left = s.numel - go;
  const int n = left < kLocalTile ? static_cast<int>(left) : kLocalTile;
  // h and v are 16-byte aligned by construction of the arena
  uintptr_t bits = reinterpret_cast<uintptr_t>(x) |
                   (BF16 ? reinterpret_cast<uintptr_t>(g) << 1 : reinterpret_cast<uintptr_t>(g));
  const int e0 = 4 * static_cast<int>(threadIdx.x);
  if (e0 >= n) return;
  if ((bits & 15) == 0 && e0 + 4 <= n) {
    const int idx = threadIdx.x;
    V4 xv = ld4<NT>(x + e0), hv, vv;
    // With only two loads per wave (buffers read as zero) the step measures 2.5 %
    // faster when the second load is issued after the first has returned
    // (2.125 -> 2.072 ms, m = 32, 25.6 M elements, four alternating runs); with
    // three or four loads the same wait changes nothing or costs 1-2 %.
    if constexpr (FIRST) asm volatile("s_waitcnt vmcnt(0)" : "+v"(xv)::"memory");
    if constexpr (!FIRST) hv = ld4<NT>(h + e0);
    if constexpr (!FIRST && BASE == 1) vv = ld4<NT>(v + e0);
    V4 gv = ldg4<BF16, NT>(g, idx);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float xe = xv[c], he = FIRST ? 0.f : hv[c];
      if constexpr (BASE == 0) {
        sgd_elem<FIRST>(xe, he, gv[c], sp);
      } else {
        float ve = FIRST ? 0.f : vv[c];
        adam_elem<FIRST>(xe, he, ve, gv[c], ap);
        vv[c] = ve;
      }
      xv[c] = xe;
      hv[c] = he;
    }
    st4<NT>(x + e0, xv);
    if constexpr (!LAST) st4<NT>(h + e0, hv);
    if constexpr (!LAST && BASE == 1) st4<NT>(v + e0, vv);
  } else {
    // element-wise: the ragged tail of a tensor, or pointers that are not
    // 16-byte aligned
    const int e1 = e0 + 4 < n ? e0 + 4 : n;
    for (int j = e0; j < e1; ++j) {
      float xe = ld1(x + j), he = FIRST ? 0.f : ld1(h + j);
      float ge = ldg1<BF16>(g, j);
      if constexpr (BASE == 0) {
        sgd_elem<FIRST>(xe, he, ge, sp);
      } else {
        float ve = FIRST ? 0.f : ld1(v + j);
        adam_elem<FIRST>(xe, he, ve, ge, ap);
        if constexpr (!LAST) st1(v + j, ve);
      }
      st1(x + j, xe);
      if constexpr (!LAST) st1(h + j, he);
    }
  }
}

// ---- outer step -----------------------------------------------------------------
// One workgroup = one tile = up to 4 * blockDim elements of one tensor; lane t
// owns elements [4t, 4t + 4) in all m replicas, x0 and u.

#ifndef SLOWMO_OUTER_UNROLL
#define SLOWMO_OUTER_UNROLL 8
#endif
#ifndef SLOWMO_OUTER_NTL
#define SLOWMO_OUTER_NTL 1
#endif
#ifndef SLOWMO_OUTER_NTS
#define SLOWMO_OUTER_NTS 1
#endif
#define SLOWMO_STR2(x) #x
#define SLOWMO_STR(x) SLOWMO_STR2(x)
#define SLOWMO_PRAGMA_UNROLL_OUTER _Pragma(SLOWMO_STR(unroll SLOWMO_OUTER_UNROLL))

// Buffer strategy "average" for this lane's elements of one arena (h or v):
// every worker's value becomes the ordered mean over the workers.  The arena
// is 16-byte aligned by construction, so only a ragged tail is element-wise.
template <bool NTL, bool NTS>
__device__ __forceinline__ void average_arena(float *__restrict__ b0, int64_t stride, int m,
                                              float m_f, int e0, int n) {
  if (e0 + 4 <= n) {
    V4 acc = ld4<NTL>(b0 + e0);
    SLOWMO_PRAGMA_UNROLL_OUTER
    for (int i = 1; i < m; ++i) acc = acc + ld4<NTL>(b0 + i * stride + e0);
    V4 mean;
#pragma unroll
    for (int c = 0; c < 4; ++c) mean[c] = acc[c] / m_f;
    SLOWMO_PRAGMA_UNROLL_OUTER
    for (int i = 0; i < m; ++i) st4<NTS>(b0 + i * stride + e0, mean);
  } else {
    for (int j = e0; j < n; ++j) {
      float s = ld1(b0 + j);
      for (int i = 1; i < m; ++i) s = s + ld1(b0 + i * stride + j);
      float mean = s / m_f;
      for (int i = 0; i < m; ++i) st1(b0 + i * stride + j, mean);
    }
  }
}

// AVG: 0 = lines 6-8 only; 1 = also average h over the workers; 2 = h and v.
template <bool NT, int AVG>
__global__ __launch_bounds__(kOuterBlock) void k_outer_step(
    const TileRef *__restrict__ tiles, const TensorInfo *__restrict__ tensors,
    float *const *__restrict__ xtab_t, float *__restrict__ x0base, float *__restrict__ ubase,
    float *__restrict__ hbase, float *__restrict__ vbase, int64_t d_pad, int ntiles, int chunk,
    int remap, int m, OuterP p0) {
  const int tile = tile_of(blockIdx.x, chunk, remap);
  if (tile >= ntiles) return;
  const TileRef t = tiles[tile];         // uniform: scalar loads
  const TensorInfo ti = tensors[t.owner];
  const OuterP p = for_tensor(p0, ti.lr_scale);
  const int64_t eo = static_cast<int64_t>(t.k) * kOuterTile;  // offset of the tile in its tensor
  const int64_t left = ti.numel - eo;
  const int n = left < kOuterTile ? static_cast<int>(left) : kOuterTile;
  const bool aligned = ti.unaligned == 0;
  float *const *__restrict__ xp = xtab_t + static_cast<int64_t>(t.owner) * m;  // m replica pointers
  float *x0 = x0base + ti.fo + eo;
  float *u = ubase + ti.fo + eo;
  const int e0 = 4 * static_cast<int>(threadIdx.x);
  if (e0 >= n) return;
  constexpr bool NTL = NT && SLOWMO_OUTER_NTL, NTS = NT && SLOWMO_OUTER_NTS;
  if (aligned && e0 + 4 <= n) {
    // line 6: ordered sum over the replicas, i = 0, 1, ..., m-1
    V4 acc = ld4<NTL>(xp[0] + eo + e0);
    SLOWMO_PRAGMA_UNROLL_OUTER
    for (int i = 1; i < m; ++i) acc = acc + ld4<NTL>(xp[i] + eo + e0);
    V4 x0v = ld4<NTL>(x0 + e0);
    V4 uv = ld4<NTL>(u + e0);
    V4 xn;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float ue = uv[c];
      xn[c] = outer_elem(acc[c], x0v[c], ue, p);
      uv[c] = ue;
    }
    st4<NTS>(u + e0, uv);
    st4<NTS>(x0 + e0, xn);
    SLOWMO_PRAGMA_UNROLL_OUTER
    for (int i = 0; i < m; ++i) st4<NTS>(xp[i] + eo + e0, xn);
  } else {
    const int e1 = e0 + 4 < n ? e0 + 4 : n;
    for (int j = e0; j < e1; ++j) {
      float s = ld1(xp[0] + eo + j);
      for (int i = 1; i < m; ++i) s = s + ld1(xp[i] + eo + j);
      float ue = ld1(u + j);
      float xn = outer_elem(s, ld1(x0 + j), ue, p);
      st1(u + j, ue);
      st1(x0 + j, xn);
      for (int i = 0; i < m; ++i) st1(xp[i] + eo + j, xn);
    }
  }
  // line 2 of the next outer iteration, strategy "average"
  if constexpr (AVG >= 1) average_arena<NTL, NTS>(hbase + ti.fo + eo, d_pad, m, p.m_f, e0, n);
  if constexpr (AVG >= 2) average_arena<NTL, NTS>(vbase + ti.fo + eo, d_pad, m, p.m_f, e0, n);
}

// ---- common starting point (Algorithm 1, "Input") ------------------------------
// x_{0,0} is worker 0's replica: copy it into x0 (one copy, or one per worker
// when every worker keeps its own) and into the replicas of workers 1..m-1.
template <bool NT>
__global__ __launch_bounds__(kOuterBlock) void k_init_broadcast(
    const TileRef *__restrict__ tiles, const TensorInfo *__restrict__ tensors,
    float *const *__restrict__ xtab_t, float *__restrict__ x0base, int64_t d_pad, int x0_copies,
    int ntiles, int chunk, int remap, int m) {
  const int tile = tile_of(blockIdx.x, chunk, remap);
  if (tile >= ntiles) return;
  const TileRef t = tiles[tile];
  const TensorInfo ti = tensors[t.owner];
  const int64_t eo = static_cast<int64_t>(t.k) * kOuterTile;
  const int64_t left = ti.numel - eo;
  const int n = left < kOuterTile ? static_cast<int>(left) : kOuterTile;
  float *const *__restrict__ xp = xtab_t + static_cast<int64_t>(t.owner) * m;
  float *x0 = x0base + ti.fo + eo;
  const int e0 = 4 * static_cast<int>(threadIdx.x);
  if (e0 >= n) return;
  if (ti.unaligned == 0 && e0 + 4 <= n) {
    const V4 v = ld4<NT>(xp[0] + eo + e0);
    for (int c = 0; c < x0_copies; ++c) st4<NT>(x0 + c * d_pad + e0, v);
#pragma unroll 8
    for (int i = 1; i < m; ++i) st4<NT>(xp[i] + eo + e0, v);
  } else {
    const int e1 = e0 + 4 < n ? e0 + 4 : n;
    for (int j = e0; j < e1; ++j) {
      const float v = ld1(xp[0] + eo + j);
      for (int c = 0; c < x0_copies; ++c) st1(x0 + c * d_pad + j, v);
      for (int i = 1; i < m; ++i) st1(xp[i] + eo + j, v);
    }
  }
}

// ---- outer step without the exact average (Section 6) ---------------------------
// Same tiling as the local step: one workgroup = 256 elements of one (worker,
// tensor); 3 streams read, 3 written.  "xbar" is the worker's own replica
// (a one-term sum divided by 1, which is exact).
template <bool NT>
__global__ __launch_bounds__(kLocalBlock) void k_outer_noavg(
    const TileRef *__restrict__ tiles, const SlotInfo *__restrict__ slots,
    float *__restrict__ x0base, float *__restrict__ ubase, int ntiles, int chunk, int remap,
    OuterP p0) {
  const int tile = tile_of(blockIdx.x, chunk, remap);
  if (tile >= ntiles) return;
  const TileRef t = tiles[tile];
  const SlotInfo s = slots[t.owner];
  const OuterP p = for_tensor(p0, s.lr_scale);
  const int64_t go = static_cast<int64_t>(t.k) * kLocalTile;
  float *x = s.x + go;
  float *x0 = x0base + s.so + go;
  float *u = ubase + s.so + go;
  const int64_t left = s.numel - go;
  const int n = left < kLocalTile ? static_cast<int>(left) : kLocalTile;
  const int e0 = 4 * static_cast<int>(threadIdx.x);
  if (e0 >= n) return;
  if ((reinterpret_cast<uintptr_t>(x) & 15) == 0 && e0 + 4 <= n) {
    V4 xv = ld4<NT>(x + e0), x0v = ld4<NT>(x0 + e0), uv = ld4<NT>(u + e0);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float ue = uv[c];
      xv[c] = outer_elem(xv[c], x0v[c], ue, p);
      uv[c] = ue;
    }
    st4<NT>(u + e0, uv);
    st4<NT>(x0 + e0, xv);
    st4<NT>(x + e0, xv);
  } else {
    const int e1 = e0 + 4 < n ? e0 + 4 : n;
    for (int j = e0; j < e1; ++j) {
      float ue = ld1(u + j);
      float xn = outer_elem(ld1(x + j), ld1(x0 + j), ue, p);
      st1(u + j, ue);
      st1(x0 + j, xn);
      st1(x + j, xn);
    }
  }
}

// ---- last local step + outer step, fused ---------------------------------------
// For one tile (256 elements of one tensor): for every worker in order, the
// base-optimizer step on that worker's (x, h[, v], g) -- the same arithmetic
// as k_local_step -- with the new x kept in registers and added to the ordered
// sum; then lines 6-8 and the write of x_{t+1,0} into all replicas.  The
// replicas are read once and written once (the unfused pair writes and
// re-reads them), and under "reset" / "average" the per-worker buffers of this
// step are never written.
template <int BASE, bool BF16, bool FIRST, int POLICY, bool NT>
__global__ __launch_bounds__(kOuterBlock) void k_local_outer_step(
    const TileRef *__restrict__ tiles, const TensorInfo *__restrict__ tensors,
    float *const *__restrict__ xtab_t, const void *const *__restrict__ gtab,
    float *__restrict__ x0base, float *__restrict__ ubase, float *__restrict__ hbase,
    float *__restrict__ vbase, int64_t d_pad, int n_tensors, int ntiles, int chunk, int remap,
    int m, SgdP sp, AdamP ap, OuterP p0) {
  const int tile = tile_of(blockIdx.x, chunk, remap);
  if (tile >= ntiles) return;
  const TileRef t = tiles[tile];
  const TensorInfo ti = tensors[t.owner];
  const OuterP p = for_tensor(p0, ti.lr_scale);
  sp.lr = sp.lr * ti.lr_scale;
  sp.wd = ti.wd;
  ap.lr = ap.lr * ti.lr_scale;
  ap.wd = ti.wd;
  const int64_t eo = static_cast<int64_t>(t.k) * kOuterTile;
  const int64_t left = ti.numel - eo;
  const int n = left < kOuterTile ? static_cast<int>(left) : kOuterTile;
  float *const *__restrict__ xp = xtab_t + static_cast<int64_t>(t.owner) * m;
  const void *const *__restrict__ gp = gtab + t.owner;       // worker i: gp[i * n_tensors]
  float *x0 = x0base + ti.fo + eo;
  float *u = ubase + ti.fo + eo;
  float *h0 = hbase + ti.fo + eo;                              // worker i: h0 + i * d_pad
  float *v0 = BASE == 1 ? vbase + ti.fo + eo : nullptr;
  constexpr int gsize = BF16 ? 2 : 4;
  const int e0 = 4 * static_cast<int>(threadIdx.x);
  if (e0 >= n) return;
  if (e0 + 4 <= n) {
    V4 acc, acch, accv;
#ifndef SLOWMO_FUSED_NTL
#define SLOWMO_FUSED_NTL 1
#endif
#ifndef SLOWMO_FUSED_UNROLL
#define SLOWMO_FUSED_UNROLL 8
#endif
    _Pragma(SLOWMO_STR(unroll SLOWMO_FUSED_UNROLL))
    for (int i = 0; i < m; ++i) {
      float *xi = xp[i] + eo + e0;
      float *hi = h0 + i * d_pad + e0;
      float *vi = BASE == 1 ? v0 + i * d_pad + e0 : nullptr;
      const void *gi = static_cast<const char *>(gp[static_cast<int64_t>(i) * n_tensors]) + eo * gsize;
      V4 xv = ld4<NT && SLOWMO_FUSED_NTL>(xi), hv, vv;
      if constexpr (!FIRST) hv = ld4<NT && SLOWMO_FUSED_NTL>(hi);
      if constexpr (!FIRST && BASE == 1) vv = ld4<NT && SLOWMO_FUSED_NTL>(vi);
      V4 gv = ldg4<BF16, NT && SLOWMO_FUSED_NTL>(gi, threadIdx.x);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        float xe = xv[c], he = FIRST ? 0.f : hv[c];
        if constexpr (BASE == 0) {
          sgd_elem<FIRST>(xe, he, gv[c], sp);
        } else {
          float ve = FIRST ? 0.f : vv[c];
          adam_elem<FIRST>(xe, he, ve, gv[c], ap);
          vv[c] = ve;
        }
        xv[c] = xe;
        hv[c] = he;
      }
      if constexpr (POLICY == 1) {
        st4<NT>(hi, hv);
        if constexpr (BASE == 1) st4<NT>(vi, vv);
      }
      if constexpr (POLICY == 2) {
        acch = (i == 0) ? hv : acch + hv;
        if constexpr (BASE == 1) accv = (i == 0) ? vv : accv + vv;
      }
      acc = (i == 0) ? xv : acc + xv;
    }
    V4 x0v = ld4<NT>(x0 + e0), uv = ld4<NT>(u + e0), xn;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float ue = uv[c];
      xn[c] = outer_elem(acc[c], x0v[c], ue, p);
      uv[c] = ue;
    }
    st4<NT>(u + e0, uv);
    st4<NT>(x0 + e0, xn);
#pragma unroll 8
    for (int i = 0; i < m; ++i) st4<NT>(xp[i] + eo + e0, xn);
    if constexpr (POLICY == 2) {
      V4 mh, mv;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        mh[c] = acch[c] / p.m_f;
        if constexpr (BASE == 1) mv[c] = accv[c] / p.m_f;
      }
#pragma unroll 8
      for (int i = 0; i < m; ++i) {
        st4<NT>(h0 + i * d_pad + e0, mh);
        if constexpr (BASE == 1) st4<NT>(v0 + i * d_pad + e0, mv);
      }
    }
  } else {
    for (int j = e0; j < n; ++j) {        // ragged tail of the tensor
      float s = 0.f, sh = 0.f, sv = 0.f;
      for (int i = 0; i < m; ++i) {
        float *xi = xp[i] + eo + j;
        float *hi = h0 + i * d_pad + j;
        float *vi = BASE == 1 ? v0 + i * d_pad + j : nullptr;
        const void *gi = static_cast<const char *>(gp[static_cast<int64_t>(i) * n_tensors]) + eo * gsize;
        float xe = ld1(xi), he = FIRST ? 0.f : ld1(hi), ve = 0.f;
        float ge = ldg1<BF16>(gi, j);
        if constexpr (BASE == 0) {
          sgd_elem<FIRST>(xe, he, ge, sp);
        } else {
          ve = FIRST ? 0.f : ld1(vi);
          adam_elem<FIRST>(xe, he, ve, ge, ap);
        }
        if constexpr (POLICY == 1) {
          st1(hi, he);
          if constexpr (BASE == 1) st1(vi, ve);
        }
        sh = (i == 0) ? he : sh + he;
        sv = (i == 0) ? ve : sv + ve;
        s = (i == 0) ? xe : s + xe;
      }
      float ue = ld1(u + j);
      float xn = outer_elem(s, ld1(x0 + j), ue, p);
      st1(u + j, ue);
      st1(x0 + j, xn);
      for (int i = 0; i < m; ++i) st1(xp[i] + eo + j, xn);
      if constexpr (POLICY == 2) {
        for (int i = 0; i < m; ++i) {
          st1(h0 + i * d_pad + j, sh / p.m_f);
          if constexpr (BASE == 1) st1(v0 + i * d_pad + j, sv / p.m_f);
        }
      }
    }
  }
}

// ---- big tiles: the two kernels above on whole 65 536-element pieces ---------------
// One 1024-thread workgroup = kBigTile elements of one tensor, all workers;
// lane t owns the vectors [v * 4096 + 4t, + 4), v = 0..15, of every stream.  All
// 16 waves of the workgroup read 256 KiB of replica 0, then of replica 1, ...:
// measured, a memory region that is visited in pieces of this size serves the
// many-stream walk about 10 % faster than 1 KiB pieces from unrelated waves
// (m = 32).  The pieces are full and 16-byte aligned in every stream, so there
// is no element-wise path.  Same arithmetic, same order of the sum, same
// results as the ordinary tiles.  Streams are addressed as a uniform base (the
// piece of vector v) plus the lane's offset, which keeps the addresses in
// scalar registers: the 128 vector registers a 1024-thread workgroup can have
// per lane hold the 16 accumulators and the operands of a few vectors.
constexpr int kBigStride = 4 * kBigBlock;  // floats between a lane's consecutive vectors

__global__ __launch_bounds__(kBigBlock) void k_outer_big(
    const TileRef *__restrict__ tiles, const TensorInfo *__restrict__ tensors,
    float *const *__restrict__ xtab_t, float *__restrict__ x0base, float *__restrict__ ubase,
    int ntiles, int chunk, int remap, int m, OuterP p0) {
  const int tile = tile_of(blockIdx.x, chunk, remap);
  if (tile >= ntiles) return;
  const TileRef t = tiles[tile];
  const TensorInfo ti = tensors[t.owner];
  const OuterP p = for_tensor(p0, ti.lr_scale);
  const int64_t eo = static_cast<int64_t>(t.k) * kBigTile;
  float *const *__restrict__ xp = xtab_t + static_cast<int64_t>(t.owner) * m;
  float *x0 = x0base + ti.fo + eo;
  float *u = ubase + ti.fo + eo;
  const int lane = 4 * static_cast<int>(threadIdx.x);
  constexpr int HALF = kBigVpt / 2;
  V4 acc[kBigVpt];
  for (int i = 0; i < m; ++i) {       // line 6: ordered sum, i = 0, 1, ..., m-1
    const float *x = xp[i] + eo;
#pragma unroll
    for (int v0 = 0; v0 < kBigVpt; v0 += HALF) {
      V4 xv[HALF];
#pragma unroll
      for (int v = 0; v < HALF; ++v) xv[v] = ld4<true>(x + (v0 + v) * kBigStride + lane);
#pragma unroll
      for (int v = 0; v < HALF; ++v) acc[v0 + v] = (i == 0) ? xv[v] : acc[v0 + v] + xv[v];
    }
  }
#pragma unroll
  for (int v = 0; v < kBigVpt; ++v) {
    const V4 x0v = ld4<true>(x0 + v * kBigStride + lane);
    V4 uv = ld4<true>(u + v * kBigStride + lane), xn;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float ue = uv[c];
      xn[c] = outer_elem(acc[v][c], x0v[c], ue, p);
      uv[c] = ue;
    }
    st4<true>(u + v * kBigStride + lane, uv);
    st4<true>(x0 + v * kBigStride + lane, xn);
    acc[v] = xn;
  }
  for (int i = 0; i < m; ++i) {
    float *x = xp[i] + eo;
#pragma unroll
    for (int v = 0; v < kBigVpt; ++v) st4<true>(x + v * kBigStride + lane, acc[v]);
  }
}

// POLICY 0 (reset: the buffers of this step are not stored) or 1 (maintain).
// A worker's step runs over SUB vectors at a time: their operands are loaded,
// stepped, added to the sum and dropped before the next SUB are loaded.
template <int BASE, bool BF16, bool FIRST, int POLICY>
__global__ __launch_bounds__(kBigBlock) void k_local_outer_big(
    const TileRef *__restrict__ tiles, const TensorInfo *__restrict__ tensors,
    float *const *__restrict__ xtab_t, const void *const *__restrict__ gtab,
    float *__restrict__ x0base, float *__restrict__ ubase, float *__restrict__ hbase,
    float *__restrict__ vbase, int64_t d_pad, int n_tensors, int ntiles, int chunk, int remap,
    int m, SgdP sp, AdamP ap, OuterP p0) {
  static_assert(POLICY == 0 || POLICY == 1, "no buffer average on big tiles");
  const int tile = tile_of(blockIdx.x, chunk, remap);
  if (tile >= ntiles) return;
  const TileRef t = tiles[tile];
  const TensorInfo ti = tensors[t.owner];
  const OuterP p = for_tensor(p0, ti.lr_scale);
  sp.lr = sp.lr * ti.lr_scale;
  sp.wd = ti.wd;
  ap.lr = ap.lr * ti.lr_scale;
  ap.wd = ti.wd;
  const int64_t eo = static_cast<int64_t>(t.k) * kBigTile;
  float *const *__restrict__ xp = xtab_t + static_cast<int64_t>(t.owner) * m;
  const void *const *__restrict__ gp = gtab + t.owner;       // worker i: gp[i * n_tensors]
  float *x0 = x0base + ti.fo + eo;
  float *u = ubase + ti.fo + eo;
  float *h0 = hbase + ti.fo + eo;                              // worker i: h0 + i * d_pad
  float *v0 = BASE == 1 ? vbase + ti.fo + eo : nullptr;
  constexpr int gsize = BF16 ? 2 : 4;
  constexpr int SUB = 2;
  const int lane = 4 * static_cast<int>(threadIdx.x);
  V4 acc[kBigVpt];
  for (int i = 0; i < m; ++i) {
    const float *xi = xp[i] + eo;
    float *hi = h0 + i * d_pad;
    float *vi = BASE == 1 ? v0 + i * d_pad : nullptr;
    const char *gi = static_cast<const char *>(gp[static_cast<int64_t>(i) * n_tensors]) + eo * gsize;
#pragma unroll
    for (int s0 = 0; s0 < kBigVpt; s0 += SUB) {
      V4 xv[SUB], hv[SUB], vv[SUB], gv[SUB];
#pragma unroll
      for (int v = 0; v < SUB; ++v) {
        const int off = (s0 + v) * kBigStride;
        xv[v] = ld4<true>(xi + off + lane);
        if constexpr (!FIRST) hv[v] = ld4<true>(hi + off + lane);
        if constexpr (!FIRST && BASE == 1) vv[v] = ld4<true>(vi + off + lane);
        gv[v] = ldg4<BF16, true>(gi + static_cast<int64_t>(off) * gsize, threadIdx.x);
      }
#pragma unroll
      for (int v = 0; v < SUB; ++v) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          float xe = xv[v][c], he = FIRST ? 0.f : hv[v][c];
          if constexpr (BASE == 0) {
            sgd_elem<FIRST>(xe, he, gv[v][c], sp);
          } else {
            float ve = FIRST ? 0.f : vv[v][c];
            adam_elem<FIRST>(xe, he, ve, gv[v][c], ap);
            vv[v][c] = ve;
          }
          xv[v][c] = xe;
          hv[v][c] = he;
        }
        if constexpr (POLICY == 1) {
          const int off = (s0 + v) * kBigStride;
          st4<true>(hi + off + lane, hv[v]);
          if constexpr (BASE == 1) st4<true>(vi + off + lane, vv[v]);
        }
        acc[s0 + v] = (i == 0) ? xv[v] : acc[s0 + v] + xv[v];
      }
    }
  }
#pragma unroll
  for (int v = 0; v < kBigVpt; ++v) {
    const V4 x0v = ld4<true>(x0 + v * kBigStride + lane);
    V4 uv = ld4<true>(u + v * kBigStride + lane), xn;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float ue = uv[c];
      xn[c] = outer_elem(acc[v][c], x0v[c], ue, p);
      uv[c] = ue;
    }
    st4<true>(u + v * kBigStride + lane, uv);
    st4<true>(x0 + v * kBigStride + lane, xn);
    acc[v] = xn;
  }
  for (int i = 0; i < m; ++i) {
    float *x = xp[i] + eo;
#pragma unroll
    for (int v = 0; v < kBigVpt; ++v) st4<true>(x + v * kBigStride + lane, acc[v]);
  }
}

// ---- mixing step of stochastic gradient push (Algorithm C.1) ---------------------
// x^{(i)} <- p(i,i) x^{(i)} + p(i,j) x^{(j)}, j = in_peer(i), in place; one
// workgroup = 256 elements of one tensor, all workers.  See MixEntry.  Every entry overwrites one worker
// with a * own + b * src, both operands being values from before the step.
// An operand that the previous entry already loaded (it is the previous
// entry's source) or that opened the current cycle is taken from a register
// instead of memory, so a replica is read once unless a sender has several
// receivers that are not neighbours in the order.  The loads of a batch of
// entries are issued together; all of them read old values, which stay in
// memory until their own entry comes, so issuing them early is safe.  Plain
// (cached) loads for the source operand measured faster than non-temporal ones.
#ifndef SLOWMO_MIX_BATCH
#define SLOWMO_MIX_BATCH 4
#endif
#ifndef SLOWMO_MIX_OWN_NT
#define SLOWMO_MIX_OWN_NT 1
#endif
#ifndef SLOWMO_MIX_SRC_NT
#define SLOWMO_MIX_SRC_NT 0
#endif
constexpr int kMixBatch = SLOWMO_MIX_BATCH;

// The saved registers of the mixing kernels: kMixSaved values of type T, read
// and written with a register number 1..kMixSaved that is uniform over the
// workgroup (named members, so that they live in registers).
template <typename T>
struct SavedRegs {
  T r1, r2, r3, r4;
  __device__ __forceinline__ void clear(const T &z) { r1 = r2 = r3 = r4 = z; }
  __device__ __forceinline__ void put(int k, const T &v) {
    if (k == 1) {
      r1 = v;
    } else if (k == 2) {
      r2 = v;
    } else if (k == 3) {
      r3 = v;
    } else if (k == 4) {
      r4 = v;
    }
  }
  __device__ __forceinline__ T get(int k, T v) const {   // v: the result for k == 0
    if (k == 1) {
      v = r1;
    } else if (k == 2) {
      v = r2;
    } else if (k == 3) {
      v = r3;
    } else if (k == 4) {
      v = r4;
    }
    return v;
  }
};
static_assert(kMixSaved == 4, "SavedRegs has four members");
// an entry's operand that is in a register already (not read from memory)
__device__ __forceinline__ bool mix_own_in_register(int32_t flags) {
  return (flags & kMixOwnFromS) || mix_own_saved(flags);
}
__device__ __forceinline__ bool mix_src_in_register(int32_t flags) {
  return (flags & (kMixSrcFromS | kMixSrcFromFirst)) || mix_src_saved(flags);
}

template <bool NT>
__global__ __launch_bounds__(kOuterBlock) void k_mix_step(
    const TileRef *__restrict__ tiles, const TensorInfo *__restrict__ tensors,
    float *const *__restrict__ xtab_t, const MixEntry *__restrict__ seq, int len, int ntiles,
    int chunk, int remap, int m) {
  const int tile = tile_of(blockIdx.x, chunk, remap);
  if (tile >= ntiles) return;
  const TileRef t = tiles[tile];
  const TensorInfo ti = tensors[t.owner];
  const int64_t eo = static_cast<int64_t>(t.k) * kOuterTile;
  const int64_t left = ti.numel - eo;
  const int n = left < kOuterTile ? static_cast<int>(left) : kOuterTile;
  float *const *__restrict__ xp = xtab_t + static_cast<int64_t>(t.owner) * m;
  const int e0 = 4 * static_cast<int>(threadIdx.x);
  if (e0 >= n) return;
  if (ti.unaligned == 0 && e0 + 4 <= n) {
    V4 S = {0.f, 0.f, 0.f, 0.f}, first = S;
    SavedRegs<V4> H;
    H.clear(S);
    for (int base = 0; base < len; base += kMixBatch) {
      V4 own[kMixBatch], sv[kMixBatch];
      float *ptr[kMixBatch];
#pragma unroll
      for (int q = 0; q < kMixBatch; ++q) {
        if (base + q < len) {
          const MixEntry en = seq[base + q];
          ptr[q] = xp[en.node] + eo + e0;
          if (!mix_own_in_register(en.flags)) own[q] = ld4<NT && SLOWMO_MIX_OWN_NT>(ptr[q]);
          if (!(en.flags & kMixNoSrc) && !mix_src_in_register(en.flags))
            sv[q] = ld4<NT && SLOWMO_MIX_SRC_NT>(xp[en.src] + eo + e0);
        }
      }
#pragma unroll
      for (int q = 0; q < kMixBatch; ++q) {
        if (base + q < len) {
          const MixEntry en = seq[base + q];
          const V4 o = (en.flags & kMixOwnFromS) ? S : H.get(mix_own_saved(en.flags), own[q]);
          if (en.flags & kMixSaveFirst) first = o;
          if (en.flags & kMixNoSrc) {
            st4<NT>(ptr[q], en.a * o);
          } else {
            H.put(mix_save(en.flags), S);
            if (en.flags & kMixSrcFromFirst) {
              S = first;
            } else if (!(en.flags & kMixSrcFromS)) {
              S = H.get(mix_src_saved(en.flags), sv[q]);
            }
            st4<NT>(ptr[q], en.a * o + en.b * S);
          }
        }
      }
    }
  } else {
    const int e1 = e0 + 4 < n ? e0 + 4 : n;
    for (int j = e0; j < e1; ++j) {
      float S = 0.f, first = 0.f;
      SavedRegs<float> H;
      H.clear(0.f);
      for (int i = 0; i < len; ++i) {
        const MixEntry en = seq[i];
        float *ptr = xp[en.node] + eo + j;
        const float o = (en.flags & kMixOwnFromS)       ? S
                        : mix_own_saved(en.flags) != 0 ? H.get(mix_own_saved(en.flags), 0.f)
                                                       : ld1(ptr);
        if (en.flags & kMixSaveFirst) first = o;
        if (en.flags & kMixNoSrc) {
          st1(ptr, en.a * o);
        } else {
          H.put(mix_save(en.flags), S);
          if (en.flags & kMixSrcFromFirst) {
            S = first;
          } else if (mix_src_saved(en.flags)) {
            S = H.get(mix_src_saved(en.flags), 0.f);
          } else if (!(en.flags & kMixSrcFromS)) {
            S = ld1(xp[en.src] + eo + j);
          }
          st1(ptr, en.a * o + en.b * S);
        }
      }
    }
  }
}

// ---- local step + mixing step, fused ---------------------------------------------
// Stochastic gradient push as base optimizer runs a mixing step after every
// local step (Algorithm C.1).  Done as two kernels, the replicas are written by
// the first and read again by the second.  Here one workgroup takes a tile of
// one tensor through all workers in the mixing order: a worker's base-optimizer
// step (the arithmetic of k_local_step) is computed when its value is first
// needed and the stepped x stays in registers for the mix, so x is read once
// and written once per step (8 bytes per worker and element less).  A worker
// whose stepped value is needed as a source before its own turn, and is not
// the next in the order, is stepped again from memory at its own turn: its x,
// h and v in memory stay untouched until then.
template <int BASE, bool BF16, bool FIRST, bool NT>
__device__ __forceinline__ void step_vec4(const float *xi, const float *hi, const float *vi,
                                          const void *gi, int lane, const SgdP &sp,
                                          const AdamP &ap, V4 &xv, V4 &hv, V4 &vv) {
  xv = ld4<NT>(xi);
  if constexpr (!FIRST) hv = ld4<NT>(hi);
  if constexpr (!FIRST && BASE == 1) vv = ld4<NT>(vi);
  const V4 gv = ldg4<BF16, NT>(gi, lane);
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    float xe = xv[c], he = FIRST ? 0.f : hv[c];
    if constexpr (BASE == 0) {
      sgd_elem<FIRST>(xe, he, gv[c], sp);
    } else {
      float ve = FIRST ? 0.f : vv[c];
      adam_elem<FIRST>(xe, he, ve, gv[c], ap);
      vv[c] = ve;
    }
    xv[c] = xe;
    hv[c] = he;
  }
}

template <int BASE, bool BF16, bool FIRST>
__device__ __forceinline__ void step_1(const float *xi, const float *hi, const float *vi,
                                       const void *gi, int j, const SgdP &sp, const AdamP &ap,
                                       float &xe, float &he, float &ve) {
  xe = ld1(xi);
  he = FIRST ? 0.f : ld1(hi);
  ve = 0.f;
  const float ge = ldg1<BF16>(gi, j);
  if constexpr (BASE == 0) {
    sgd_elem<FIRST>(xe, he, ge, sp);
  } else {
    ve = FIRST ? 0.f : ld1(vi);
    adam_elem<FIRST>(xe, he, ve, ge, ap);
  }
}

template <int BASE, bool BF16, bool FIRST, bool NT>
__global__ __launch_bounds__(kOuterBlock) void k_local_mix_step(
    const TileRef *__restrict__ tiles, const TensorInfo *__restrict__ tensors,
    float *const *__restrict__ xtab_t, const void *const *__restrict__ gtab,
    float *__restrict__ hbase, float *__restrict__ vbase, const MixEntry *__restrict__ seq, int len,
    int64_t d_pad, int n_tensors, int ntiles, int chunk, int remap, int m, SgdP sp, AdamP ap) {
  const int tile = tile_of(blockIdx.x, chunk, remap);
  if (tile >= ntiles) return;
  const TileRef t = tiles[tile];
  const TensorInfo ti = tensors[t.owner];
  sp.lr = sp.lr * ti.lr_scale;
  sp.wd = ti.wd;
  ap.lr = ap.lr * ti.lr_scale;
  ap.wd = ti.wd;
  const int64_t eo = static_cast<int64_t>(t.k) * kOuterTile;
  const int64_t left = ti.numel - eo;
  const int n = left < kOuterTile ? static_cast<int>(left) : kOuterTile;
  float *const *__restrict__ xp = xtab_t + static_cast<int64_t>(t.owner) * m;
  const void *const *__restrict__ gp = gtab + t.owner;       // worker i: gp[i * n_tensors]
  float *h0 = hbase + ti.fo + eo;                              // worker i: h0 + i * d_pad
  float *v0 = BASE == 1 ? vbase + ti.fo + eo : nullptr;
  constexpr int gsize = BF16 ? 2 : 4;
  const int e0 = 4 * static_cast<int>(threadIdx.x);
  if (e0 >= n) return;
  if (e0 + 4 <= n) {
    V4 Sx = {0.f, 0.f, 0.f, 0.f}, Sh = Sx, Sv = Sx, first = Sx;
    SavedRegs<V4> Hx, Hh, Hv;       // saved stepped workers: new x, h and v
    Hx.clear(Sx);
    Hh.clear(Sx);
    Hv.clear(Sx);
#pragma unroll 1
    for (int i = 0; i < len; ++i) {
      const MixEntry en = seq[i];
      float *xi = xp[en.node] + eo + e0;
      float *hi = h0 + en.node * d_pad + e0;
      float *vi = BASE == 1 ? v0 + en.node * d_pad + e0 : nullptr;
      V4 xo, ho, vo;
      if (mix_own_in_register(en.flags)) {       // in a saved register, else held in S
        xo = Hx.get(mix_own_saved(en.flags), Sx);
        ho = Hh.get(mix_own_saved(en.flags), Sh);
        vo = Hv.get(mix_own_saved(en.flags), Sv);
      } else {
        const void *gi =
            static_cast<const char *>(gp[static_cast<int64_t>(en.node) * n_tensors]) + eo * gsize;
        step_vec4<BASE, BF16, FIRST, NT>(xi, hi, vi, gi, threadIdx.x, sp, ap, xo, ho, vo);
      }
      st4<NT>(hi, ho);
      if constexpr (BASE == 1) st4<NT>(vi, vo);
      if (en.flags & kMixSaveFirst) first = xo;
      if (en.flags & kMixNoSrc) {
        st4<NT>(xi, en.a * xo);
      } else {
        Hx.put(mix_save(en.flags), Sx);
        Hh.put(mix_save(en.flags), Sh);
        Hv.put(mix_save(en.flags), Sv);
        if (en.flags & kMixSrcFromFirst) {
          Sx = first;
        } else if (mix_src_saved(en.flags)) {
          Sx = Hx.get(mix_src_saved(en.flags), Sx);
          Sh = Hh.get(mix_src_saved(en.flags), Sh);
          Sv = Hv.get(mix_src_saved(en.flags), Sv);
        } else if (!(en.flags & kMixSrcFromS)) {
          const void *gs =
              static_cast<const char *>(gp[static_cast<int64_t>(en.src) * n_tensors]) + eo * gsize;
          step_vec4<BASE, BF16, FIRST, NT>(xp[en.src] + eo + e0, h0 + en.src * d_pad + e0,
                                           BASE == 1 ? v0 + en.src * d_pad + e0 : nullptr, gs,
                                           threadIdx.x, sp, ap, Sx, Sh, Sv);
        }
        st4<NT>(xi, en.a * xo + en.b * Sx);
      }
    }
  } else {
    for (int j = e0; j < n; ++j) {        // ragged tail of the tensor
      float Sx = 0.f, Sh = 0.f, Sv = 0.f, first = 0.f;
      SavedRegs<float> Hx, Hh, Hv;
      Hx.clear(0.f);
      Hh.clear(0.f);
      Hv.clear(0.f);
      for (int i = 0; i < len; ++i) {
        const MixEntry en = seq[i];
        float *xi = xp[en.node] + eo + j;
        float *hi = h0 + en.node * d_pad + j;
        float *vi = BASE == 1 ? v0 + en.node * d_pad + j : nullptr;
        float xo, ho, vo;
        if (mix_own_in_register(en.flags)) {
          xo = Hx.get(mix_own_saved(en.flags), Sx);
          ho = Hh.get(mix_own_saved(en.flags), Sh);
          vo = Hv.get(mix_own_saved(en.flags), Sv);
        } else {
          const void *gi =
              static_cast<const char *>(gp[static_cast<int64_t>(en.node) * n_tensors]) + eo * gsize;
          step_1<BASE, BF16, FIRST>(xi, hi, vi, gi, j, sp, ap, xo, ho, vo);
        }
        st1(hi, ho);
        if constexpr (BASE == 1) st1(vi, vo);
        if (en.flags & kMixSaveFirst) first = xo;
        if (en.flags & kMixNoSrc) {
          st1(xi, en.a * xo);
        } else {
          Hx.put(mix_save(en.flags), Sx);
          Hh.put(mix_save(en.flags), Sh);
          Hv.put(mix_save(en.flags), Sv);
          if (en.flags & kMixSrcFromFirst) {
            Sx = first;
          } else if (mix_src_saved(en.flags)) {
            Sx = Hx.get(mix_src_saved(en.flags), Sx);
            Sh = Hh.get(mix_src_saved(en.flags), Sh);
            Sv = Hv.get(mix_src_saved(en.flags), Sv);
          } else if (!(en.flags & kMixSrcFromS)) {
            const void *gs =
                static_cast<const char *>(gp[static_cast<int64_t>(en.src) * n_tensors]) + eo * gsize;
            step_1<BASE, BF16, FIRST>(xp[en.src] + eo + j, h0 + en.src * d_pad + j,
                                      BASE == 1 ? v0 + en.src * d_pad + j : nullptr, gs, j, sp, ap,
                                      Sx, Sh, Sv);
          }
          st1(xi, en.a * xo + en.b * Sx);
        }
      }
    }
  }
}

// z^{(i)} = x^{(i)} / w_i (Algorithm C.1, last line), one workgroup per local tile.
template <bool NT>
__global__ __launch_bounds__(kLocalBlock) void k_debias(
    const TileRef *__restrict__ tiles, const SlotInfo *__restrict__ slots,
    float *const *__restrict__ ztab, const float *__restrict__ w, int n_tensors, int ntiles,
    int chunk, int remap) {
  const int tile = tile_of(blockIdx.x, chunk, remap);
  if (tile >= ntiles) return;
  const TileRef t = tiles[tile];
  const SlotInfo s = slots[t.owner];
  const float wi = w[t.owner / n_tensors];
  const int64_t go = static_cast<int64_t>(t.k) * kLocalTile;
  const float *x = s.x + go;
  float *z = ztab[t.owner] + go;
  const int64_t left = s.numel - go;
  const int n = left < kLocalTile ? static_cast<int>(left) : kLocalTile;
  const int e0 = 4 * static_cast<int>(threadIdx.x);
  if (e0 >= n) return;
  if (((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(z)) & 15) == 0 && e0 + 4 <= n) {
    V4 xv = ld4<NT>(x + e0);
#pragma unroll
    for (int c = 0; c < 4; ++c) xv[c] = xv[c] / wi;
    st4<NT>(z + e0, xv);
  } else {
    const int e1 = e0 + 4 < n ? e0 + 4 : n;
    for (int j = e0; j < e1; ++j) st1(z + j, ld1(x + j) / wi);
  }
}

struct Grid {
  int chunk;
  int run;  // tiles per XCD turn; 0 = no remap
  unsigned blocks;
};
Grid make_grid(int ntiles, const LaunchTuning &t) {
  Grid g;
  g.chunk = (ntiles + kXcd - 1) / kXcd;
  g.run = !t.xcd_remap ? 0 : (t.xcd_run > 0 && t.xcd_run < g.chunk ? t.xcd_run : g.chunk);
  if (g.run == 0) {
    g.blocks = static_cast<unsigned>(ntiles);
  } else {
    int64_t span = static_cast<int64_t>(kXcd) * g.run;
    if ((ntiles + span - 1) / span * span > INT32_MAX) {  // keep workgroup ids within int
      g.run = g.chunk;
      span = static_cast<int64_t>(kXcd) * g.run;
    }
    g.blocks = static_cast<unsigned>((ntiles + span - 1) / span * span);
  }
  return g;
}

template <int BASE, bool BF16, bool FIRST, bool LAST>
hipError_t launch_local_t(const LocalArgs &a, const LaunchTuning &t, hipStream_t s) {
  const Grid g = make_grid(a.ntiles, t);
  const SgdP sp{a.lr, a.mu, a.wd};
  const AdamP ap{a.lr, a.wd, a.b1, a.b2, a.omb1, a.omb2, a.rc1, a.rc2, a.eps};
  if (t.nontemporal) {
    hipLaunchKernelGGL((k_local_step<BASE, BF16, FIRST, LAST, true>), dim3(g.blocks),
                       dim3(kLocalBlock), 0, s, a.tiles, a.slots, a.gtab, a.h, a.v, a.ntiles,
                       g.chunk, g.run, sp, ap);
  } else {
    hipLaunchKernelGGL((k_local_step<BASE, BF16, FIRST, LAST, false>), dim3(g.blocks),
                       dim3(kLocalBlock), 0, s, a.tiles, a.slots, a.gtab, a.h, a.v, a.ntiles,
                       g.chunk, g.run, sp, ap);
  }
  return hipGetLastError();
}

template <int BASE, bool BF16>
hipError_t launch_local_b(const LocalArgs &a, bool first, bool last, const LaunchTuning &t,
                          hipStream_t s) {
  if (first) {
    return last ? launch_local_t<BASE, BF16, true, true>(a, t, s)
                : launch_local_t<BASE, BF16, true, false>(a, t, s);
  }
  return last ? launch_local_t<BASE, BF16, false, true>(a, t, s)
              : launch_local_t<BASE, BF16, false, false>(a, t, s);
}

}  // namespace

hipError_t launch_local_step(const LocalArgs &a, int base, bool bf16, bool first, bool last,
                             const LaunchTuning &t, hipStream_t s) {
  if (a.ntiles <= 0) return hipSuccess;
  if (base == 0) {
    return bf16 ? launch_local_b<0, true>(a, first, last, t, s)
                : launch_local_b<0, false>(a, first, last, t, s);
  }
  return bf16 ? launch_local_b<1, true>(a, first, last, t, s)
              : launch_local_b<1, false>(a, first, last, t, s);
}

template <bool NT, int AVG>
hipError_t launch_outer_t(const OuterArgs &a, const LaunchTuning &t, hipStream_t s) {
  const Grid g = make_grid(a.ntiles, t);
  const OuterP p{a.lr, 0.f, a.beta, a.m_f, a.alpha};
  hipLaunchKernelGGL((k_outer_step<NT, AVG>), dim3(g.blocks), dim3(kOuterBlock), t.outer_lds, s,
                     a.tiles, a.tensors, a.xtab_t, a.x0, a.u, a.avg_h, a.avg_v, a.d_pad, a.ntiles,
                     g.chunk, g.run, a.m, p);
  return hipGetLastError();
}

hipError_t launch_outer_step(const OuterArgs &a, const LaunchTuning &t, hipStream_t s) {
  if (a.ntiles <= 0) return hipSuccess;
  const int avg = a.avg_h ? (a.avg_v ? 2 : 1) : 0;
  if (t.nontemporal) {
    return avg == 0 ? launch_outer_t<true, 0>(a, t, s)
                    : avg == 1 ? launch_outer_t<true, 1>(a, t, s) : launch_outer_t<true, 2>(a, t, s);
  }
  return avg == 0 ? launch_outer_t<false, 0>(a, t, s)
                  : avg == 1 ? launch_outer_t<false, 1>(a, t, s) : launch_outer_t<false, 2>(a, t, s);
}

hipError_t launch_outer_big(const OuterArgs &a, const LaunchTuning &t, hipStream_t s) {
  if (a.ntiles <= 0) return hipSuccess;
  if (a.avg_h || a.avg_v || !t.nontemporal) return hipErrorInvalidValue;
  const Grid g = make_grid(a.ntiles, t);
  const OuterP p{a.lr, 0.f, a.beta, a.m_f, a.alpha};
  hipLaunchKernelGGL(k_outer_big, dim3(g.blocks), dim3(kBigBlock), 0, s, a.tiles, a.tensors,
                     a.xtab_t, a.x0, a.u, a.ntiles, g.chunk, g.run, a.m, p);
  return hipGetLastError();
}

namespace {

template <int BASE, bool BF16, bool FIRST>
hipError_t launch_fused_big_t(const LocalArgs &l, const OuterArgs &o, int n_tensors, int policy,
                              const LaunchTuning &t, hipStream_t s) {
  const Grid g = make_grid(o.ntiles, t);
  const SgdP sp{l.lr, l.mu, l.wd};
  const AdamP ap{l.lr, l.wd, l.b1, l.b2, l.omb1, l.omb2, l.rc1, l.rc2, l.eps};
  const OuterP p{o.lr, 0.f, o.beta, o.m_f, o.alpha};
  if (policy == 0) {
    hipLaunchKernelGGL((k_local_outer_big<BASE, BF16, FIRST, 0>), dim3(g.blocks), dim3(kBigBlock),
                       0, s, o.tiles, o.tensors, o.xtab_t, l.gtab, o.x0, o.u, l.h, l.v, o.d_pad,
                       n_tensors, o.ntiles, g.chunk, g.run, o.m, sp, ap, p);
  } else {
    hipLaunchKernelGGL((k_local_outer_big<BASE, BF16, FIRST, 1>), dim3(g.blocks), dim3(kBigBlock),
                       0, s, o.tiles, o.tensors, o.xtab_t, l.gtab, o.x0, o.u, l.h, l.v, o.d_pad,
                       n_tensors, o.ntiles, g.chunk, g.run, o.m, sp, ap, p);
  }
  return hipGetLastError();
}

template <int BASE, bool BF16>
hipError_t launch_fused_big_f(const LocalArgs &l, const OuterArgs &o, int n_tensors, bool first,
                              int policy, const LaunchTuning &t, hipStream_t s) {
  return first ? launch_fused_big_t<BASE, BF16, true>(l, o, n_tensors, policy, t, s)
               : launch_fused_big_t<BASE, BF16, false>(l, o, n_tensors, policy, t, s);
}

}  // namespace

hipError_t launch_local_outer_big(const LocalArgs &l, const OuterArgs &o, int32_t n_tensors,
                                  int base, bool bf16, bool first, int policy,
                                  const LaunchTuning &t, hipStream_t s) {
  if (o.ntiles <= 0) return hipSuccess;
  if ((policy != 0 && policy != 1) || !t.nontemporal) return hipErrorInvalidValue;
  if (base == 0) {
    return bf16 ? launch_fused_big_f<0, true>(l, o, n_tensors, first, policy, t, s)
                : launch_fused_big_f<0, false>(l, o, n_tensors, first, policy, t, s);
  }
  return bf16 ? launch_fused_big_f<1, true>(l, o, n_tensors, first, policy, t, s)
              : launch_fused_big_f<1, false>(l, o, n_tensors, first, policy, t, s);
}

namespace {

template <int BASE, bool BF16, bool FIRST, int POLICY>
hipError_t launch_fused_t(const LocalArgs &l, const OuterArgs &o, int n_tensors,
                          const LaunchTuning &t, hipStream_t s) {
  const Grid g = make_grid(o.ntiles, t);
  const SgdP sp{l.lr, l.mu, l.wd};
  const AdamP ap{l.lr, l.wd, l.b1, l.b2, l.omb1, l.omb2, l.rc1, l.rc2, l.eps};
  const OuterP p{o.lr, 0.f, o.beta, o.m_f, o.alpha};
  if (t.nontemporal) {
    hipLaunchKernelGGL((k_local_outer_step<BASE, BF16, FIRST, POLICY, true>), dim3(g.blocks),
                       dim3(kOuterBlock), 0, s, o.tiles, o.tensors, o.xtab_t, l.gtab, o.x0, o.u, l.h,
                       l.v, o.d_pad, n_tensors, o.ntiles, g.chunk, g.run, o.m, sp, ap, p);
  } else {
    hipLaunchKernelGGL((k_local_outer_step<BASE, BF16, FIRST, POLICY, false>), dim3(g.blocks),
                       dim3(kOuterBlock), 0, s, o.tiles, o.tensors, o.xtab_t, l.gtab, o.x0, o.u, l.h,
                       l.v, o.d_pad, n_tensors, o.ntiles, g.chunk, g.run, o.m, sp, ap, p);
  }
  return hipGetLastError();
}

template <int BASE, bool BF16, bool FIRST>
hipError_t launch_fused_p(const LocalArgs &l, const OuterArgs &o, int n_tensors, int policy,
                          const LaunchTuning &t, hipStream_t s) {
  switch (policy) {
    case 0: return launch_fused_t<BASE, BF16, FIRST, 0>(l, o, n_tensors, t, s);
    case 1: return launch_fused_t<BASE, BF16, FIRST, 1>(l, o, n_tensors, t, s);
    default: return launch_fused_t<BASE, BF16, FIRST, 2>(l, o, n_tensors, t, s);
  }
}

template <int BASE, bool BF16>
hipError_t launch_fused_f(const LocalArgs &l, const OuterArgs &o, int n_tensors, bool first,
                          int policy, const LaunchTuning &t, hipStream_t s) {
  return first ? launch_fused_p<BASE, BF16, true>(l, o, n_tensors, policy, t, s)
               : launch_fused_p<BASE, BF16, false>(l, o, n_tensors, policy, t, s);
}

}  // namespace

hipError_t launch_local_outer_step(const LocalArgs &l, const OuterArgs &o, int32_t n_tensors,
                                   int base, bool bf16, bool first, int policy,
                                   const LaunchTuning &t, hipStream_t s) {
  if (o.ntiles <= 0) return hipSuccess;
  if (base == 0) {
    return bf16 ? launch_fused_f<0, true>(l, o, n_tensors, first, policy, t, s)
                : launch_fused_f<0, false>(l, o, n_tensors, first, policy, t, s);
  }
  return bf16 ? launch_fused_f<1, true>(l, o, n_tensors, first, policy, t, s)
              : launch_fused_f<1, false>(l, o, n_tensors, first, policy, t, s);
}

hipError_t launch_init_broadcast(const OuterArgs &a, int32_t x0_copies, const LaunchTuning &t,
                                 hipStream_t s) {
  if (a.ntiles <= 0) return hipSuccess;
  const Grid g = make_grid(a.ntiles, t);
  if (t.nontemporal) {
    hipLaunchKernelGGL((k_init_broadcast<true>), dim3(g.blocks), dim3(kOuterBlock), 0, s, a.tiles,
                       a.tensors, a.xtab_t, a.x0, a.d_pad, x0_copies, a.ntiles, g.chunk,
                       g.run, a.m);
  } else {
    hipLaunchKernelGGL((k_init_broadcast<false>), dim3(g.blocks), dim3(kOuterBlock), 0, s, a.tiles,
                       a.tensors, a.xtab_t, a.x0, a.d_pad, x0_copies, a.ntiles, g.chunk,
                       g.run, a.m);
  }
  return hipGetLastError();
}

hipError_t launch_mix_step(const MixArgs &a, const LaunchTuning &t, hipStream_t s) {
  if (a.ntiles <= 0 || a.len <= 0) return hipSuccess;
  const Grid g = make_grid(a.ntiles, t);
  if (t.nontemporal) {
    hipLaunchKernelGGL((k_mix_step<true>), dim3(g.blocks), dim3(kOuterBlock), 0, s, a.tiles,
                       a.tensors, a.xtab_t, a.seq, a.len, a.ntiles, g.chunk, g.run, a.m);
  } else {
    hipLaunchKernelGGL((k_mix_step<false>), dim3(g.blocks), dim3(kOuterBlock), 0, s, a.tiles,
                       a.tensors, a.xtab_t, a.seq, a.len, a.ntiles, g.chunk, g.run, a.m);
  }
  return hipGetLastError();
}

namespace {

template <int BASE, bool BF16, bool FIRST>
hipError_t launch_local_mix_t(const LocalArgs &l, const MixArgs &x, int64_t d_pad, int n_tensors,
                              const LaunchTuning &t, hipStream_t s) {
  const Grid g = make_grid(x.ntiles, t);
  const SgdP sp{l.lr, l.mu, l.wd};
  const AdamP ap{l.lr, l.wd, l.b1, l.b2, l.omb1, l.omb2, l.rc1, l.rc2, l.eps};
  if (t.nontemporal) {
    hipLaunchKernelGGL((k_local_mix_step<BASE, BF16, FIRST, true>), dim3(g.blocks),
                       dim3(kOuterBlock), 0, s, x.tiles, x.tensors, x.xtab_t, l.gtab, l.h, l.v, x.seq,
                       x.len, d_pad, n_tensors, x.ntiles, g.chunk, g.run, x.m, sp, ap);
  } else {
    hipLaunchKernelGGL((k_local_mix_step<BASE, BF16, FIRST, false>), dim3(g.blocks),
                       dim3(kOuterBlock), 0, s, x.tiles, x.tensors, x.xtab_t, l.gtab, l.h, l.v, x.seq,
                       x.len, d_pad, n_tensors, x.ntiles, g.chunk, g.run, x.m, sp, ap);
  }
  return hipGetLastError();
}

template <int BASE, bool BF16>
hipError_t launch_local_mix_f(const LocalArgs &l, const MixArgs &x, int64_t d_pad, int n_tensors,
                              bool first, const LaunchTuning &t, hipStream_t s) {
  return first ? launch_local_mix_t<BASE, BF16, true>(l, x, d_pad, n_tensors, t, s)
               : launch_local_mix_t<BASE, BF16, false>(l, x, d_pad, n_tensors, t, s);
}

}  // namespace

hipError_t launch_local_mix_step(const LocalArgs &l, const MixArgs &x, int64_t d_pad,
                                 int32_t n_tensors, int base, bool bf16, bool first,
                                 const LaunchTuning &t, hipStream_t s) {
  if (x.ntiles <= 0 || x.len <= 0) return hipSuccess;
  if (base == 0) {
    return bf16 ? launch_local_mix_f<0, true>(l, x, d_pad, n_tensors, first, t, s)
                : launch_local_mix_f<0, false>(l, x, d_pad, n_tensors, first, t, s);
  }
  return bf16 ? launch_local_mix_f<1, true>(l, x, d_pad, n_tensors, first, t, s)
              : launch_local_mix_f<1, false>(l, x, d_pad, n_tensors, first, t, s);
}

hipError_t launch_debias(const DebiasArgs &a, const LaunchTuning &t, hipStream_t s) {
  if (a.ntiles <= 0) return hipSuccess;
  const Grid g = make_grid(a.ntiles, t);
  if (t.nontemporal) {
    hipLaunchKernelGGL((k_debias<true>), dim3(g.blocks), dim3(kLocalBlock), 0, s, a.tiles, a.slots,
                       a.ztab, a.w, a.n_tensors, a.ntiles, g.chunk, g.run);
  } else {
    hipLaunchKernelGGL((k_debias<false>), dim3(g.blocks), dim3(kLocalBlock), 0, s, a.tiles, a.slots,
                       a.ztab, a.w, a.n_tensors, a.ntiles, g.chunk, g.run);
  }
  return hipGetLastError();
}

hipError_t launch_outer_noavg_step(const OuterNoAvgArgs &a, const LaunchTuning &t, hipStream_t s) {
  if (a.ntiles <= 0) return hipSuccess;
  const Grid g = make_grid(a.ntiles, t);
  const OuterP p{a.lr, 0.f, a.beta, 1.0f, a.alpha};
  if (t.nontemporal) {
    hipLaunchKernelGGL((k_outer_noavg<true>), dim3(g.blocks), dim3(kLocalBlock), 0, s, a.tiles,
                       a.slots, a.x0, a.u, a.ntiles, g.chunk, g.run, p);
  } else {
    hipLaunchKernelGGL((k_outer_noavg<false>), dim3(g.blocks), dim3(kLocalBlock), 0, s, a.tiles,
                       a.slots, a.x0, a.u, a.ntiles, g.chunk, g.run, p);
  }
  return hipGetLastError();
}

}  // namespace slowmo
