// gfx950 kernels of the Slow Momentum hot path.
//
// Both kernels are pure streams: every byte is read once and written once, no
// element is reused, so there is no dense contraction and the matrix cores are
// not involved.  What matters is (i) 16-byte per-lane accesses that make each
// wavefront instruction one contiguous 1 KiB burst, (ii) enough independent
// loads in flight per CU to cover HBM latency, (iii) tiles of equal cost so
// that all 256 CUs drain together, and (iv) a tile -> workgroup mapping that
// keeps neighbouring tiles on one XCD.
//
// Compiled with -ffp-contract=off: products and sums are rounded separately,
// in the order written here, which is the order of Table C.1 and Eq. (2)-(3).
#include "slowmo_kernels.h"

#include "../../include/slowmo.h"

namespace slowmo {

namespace {

constexpr int kBlock = 256;  // 4 wavefronts of 64 lanes
constexpr int kXcd = 8;      // XCDs per MI355X; workgroups are dealt to them round-robin

typedef float V4 __attribute__((ext_vector_type(4)));
typedef uint32_t U2 __attribute__((ext_vector_type(2)));

template <bool NT>
__device__ __forceinline__ V4 ld4(const float *p) {
  if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const V4 *>(p));
  return *reinterpret_cast<const V4 *>(p);
}
template <bool NT>
__device__ __forceinline__ void st4(float *p, V4 v) {
  if constexpr (NT) {
    __builtin_nontemporal_store(v, reinterpret_cast<V4 *>(p));
  } else {
    *reinterpret_cast<V4 *>(p) = v;
  }
}

// Gradient access: fp32 as is, bf16 widened exactly (the 16 bits become the
// high half of an fp32 word).
template <bool BF16>
__device__ __forceinline__ float ldg1(const void *g, int j) {
  if constexpr (BF16) {
    uint32_t w = reinterpret_cast<const uint16_t *>(g)[j];
    return __uint_as_float(w << 16);
  } else {
    return reinterpret_cast<const float *>(g)[j];
  }
}
template <bool BF16, bool NT>
__device__ __forceinline__ V4 ldg4(const void *g, int vec) {
  if constexpr (BF16) {
    const U2 *p = reinterpret_cast<const U2 *>(g) + vec;
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

// Tile visited by the v-th unit of the launch.  Workgroup b runs on XCD
// b mod 8; with the remap, XCD c walks the contiguous tile range
// [c * chunk, (c + 1) * chunk), so each XCD's L2 and TLB see one compact
// window of every stream instead of a 1-in-8 comb over all of it.
__device__ __forceinline__ int tile_of(int v, int chunk, int remap) {
  return remap ? (v % kXcd) * chunk + v / kXcd : v;
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
  float lr, alpha_lr, beta, m_f;
};
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

template <int BASE, bool BF16, bool FIRST, bool NT, int U>
__device__ __forceinline__ void local_run(float *__restrict__ x, float *__restrict__ h,
                                          float *__restrict__ v, const void *__restrict__ g, int n,
                                          const SgdP &sp, const AdamP &ap) {
  const int tid = threadIdx.x;
  uintptr_t bits = reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(h);
  if constexpr (BASE == 1) bits |= reinterpret_cast<uintptr_t>(v);
  bits |= BF16 ? (reinterpret_cast<uintptr_t>(g) << 1) : reinterpret_cast<uintptr_t>(g);
  int done = 0;
  if ((bits & 15) == 0) {
    const int nv = n >> 2;
    for (int base = 0; base < nv; base += kBlock * U) {
      V4 xv[U], hv[U], vv[U], gv[U];
#pragma unroll
      for (int q = 0; q < U; ++q) {
        int idx = base + q * kBlock + tid;
        if (idx < nv) {
          xv[q] = ld4<NT>(x + 4 * idx);
          if constexpr (!FIRST) hv[q] = ld4<NT>(h + 4 * idx);
          if constexpr (!FIRST && BASE == 1) vv[q] = ld4<NT>(v + 4 * idx);
          gv[q] = ldg4<BF16, NT>(g, idx);
        }
      }
#pragma unroll
      for (int q = 0; q < U; ++q) {
        int idx = base + q * kBlock + tid;
        if (idx < nv) {
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            float xe = xv[q][c], he = FIRST ? 0.f : hv[q][c];
            if constexpr (BASE == 0) {
              sgd_elem<FIRST>(xe, he, gv[q][c], sp);
            } else {
              float ve = FIRST ? 0.f : vv[q][c];
              adam_elem<FIRST>(xe, he, ve, gv[q][c], ap);
              vv[q][c] = ve;
            }
            xv[q][c] = xe;
            hv[q][c] = he;
          }
          st4<NT>(x + 4 * idx, xv[q]);
          st4<NT>(h + 4 * idx, hv[q]);
          if constexpr (BASE == 1) st4<NT>(v + 4 * idx, vv[q]);
        }
      }
    }
    done = nv << 2;
  }
  // element-wise path: the ragged tail of an aligned run, or a whole run
  // whose pointers are not 16-byte aligned
  for (int j = done + tid; j < n; j += kBlock) {
    float xe = x[j], he = FIRST ? 0.f : h[j];
    float ge = ldg1<BF16>(g, j);
    if constexpr (BASE == 0) {
      sgd_elem<FIRST>(xe, he, ge, sp);
    } else {
      float ve = FIRST ? 0.f : v[j];
      adam_elem<FIRST>(xe, he, ve, ge, ap);
      v[j] = ve;
    }
    x[j] = xe;
    h[j] = he;
  }
}

template <int BASE, bool BF16, bool FIRST, bool NT, int U>
__global__ __launch_bounds__(kBlock) void k_local_step(LocalArgs a, int chunk, int nunits,
                                                       int remap) {
  // The descriptors of the runs in this workgroup's tile, staged once in LDS
  // and then read by all four wavefronts as broadcasts.
  __shared__ LocalRun s_run[kMaxRunsPerTile];
  __shared__ const void *s_g[kMaxRunsPerTile];
  const SgdP sp{a.lr, a.mu, a.wd};
  const AdamP ap{a.lr, a.wd, a.b1, a.b2, a.omb1, a.omb2, a.rc1, a.rc2, a.eps};
  constexpr int gsize = BF16 ? 2 : 4;
  for (int unit = blockIdx.x; unit < nunits; unit += gridDim.x) {
    const int tile = tile_of(unit, chunk, remap);
    if (tile >= a.ntiles) continue;  // uniform over the workgroup
    const int rb = a.tile_begin[tile];
    const int nr = a.tile_begin[tile + 1] - rb;
    if (static_cast<int>(threadIdx.x) < nr) {
      LocalRun r = a.runs[rb + threadIdx.x];
      s_run[threadIdx.x] = r;
      s_g[threadIdx.x] = static_cast<const char *>(a.gtab[r.slot]) + r.go * gsize;
    }
    __syncthreads();
    for (int i = 0; i < nr; ++i) {
      const LocalRun r = s_run[i];
      local_run<BASE, BF16, FIRST, NT, U>(r.x, a.h + r.so, BASE == 1 ? a.v + r.so : nullptr,
                                          s_g[i], r.n, sp, ap);
    }
    __syncthreads();  // LDS is rewritten by the next tile
  }
}

// ---- outer step -----------------------------------------------------------------

template <bool NT, int U>
__global__ __launch_bounds__(kBlock) void k_outer_step(OuterArgs a, int chunk, int nunits,
                                                       int remap) {
  __shared__ float *s_xp[SLOWMO_MAX_WORKERS];  // replica pointers of this tile's run
  __shared__ int s_unaligned;
  const int tid = threadIdx.x;
  const int m = a.m;
  const OuterP p{a.lr, a.alpha_lr, a.beta, a.m_f};
  for (int unit = blockIdx.x; unit < nunits; unit += gridDim.x) {
    const int tile = tile_of(unit, chunk, remap);
    if (tile >= a.ntiles) continue;  // uniform over the workgroup
    const OuterRun r = a.runs[tile];
    if (tid == 0) s_unaligned = 0;
    __syncthreads();
    for (int i = tid; i < m; i += kBlock) {
      float *xp = a.xtab[static_cast<int64_t>(i) * a.n_tensors + r.tensor] + r.eo;
      s_xp[i] = xp;
      if (reinterpret_cast<uintptr_t>(xp) & 15) s_unaligned = 1;
    }
    __syncthreads();
    float *__restrict__ x0 = a.x0 + r.fo;  // 16-byte aligned by construction of the arena
    float *__restrict__ u = a.u + r.fo;
    const int n = r.n;
    int done = 0;
    if (!s_unaligned) {
      const int nv = n >> 2;
      for (int base = 0; base < nv; base += kBlock * U) {
        V4 acc[U];
        // line 6: ordered sum over the replicas, i = 0, 1, ..., m-1
#pragma unroll 4
        for (int i = 0; i < m; ++i) {
          const float *xp = s_xp[i];
#pragma unroll
          for (int q = 0; q < U; ++q) {
            int idx = base + q * kBlock + tid;
            if (idx < nv) {
              V4 t = ld4<NT>(xp + 4 * idx);
              acc[q] = (i == 0) ? t : acc[q] + t;
            }
          }
        }
        V4 xn[U];
#pragma unroll
        for (int q = 0; q < U; ++q) {
          int idx = base + q * kBlock + tid;
          if (idx < nv) {
            V4 x0v = ld4<NT>(x0 + 4 * idx);
            V4 uv = ld4<NT>(u + 4 * idx);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              float ue = uv[c];
              xn[q][c] = outer_elem(acc[q][c], x0v[c], ue, p);
              uv[c] = ue;
            }
            st4<NT>(u + 4 * idx, uv);
            st4<NT>(x0 + 4 * idx, xn[q]);
          }
        }
        for (int i = 0; i < m; ++i) {
          float *xp = s_xp[i];
#pragma unroll
          for (int q = 0; q < U; ++q) {
            int idx = base + q * kBlock + tid;
            if (idx < nv) st4<NT>(xp + 4 * idx, xn[q]);
          }
        }
      }
      done = nv << 2;
    }
    for (int j = done + tid; j < n; j += kBlock) {
      float s = s_xp[0][j];
      for (int i = 1; i < m; ++i) s = s + s_xp[i][j];
      float ue = u[j];
      float xn = outer_elem(s, x0[j], ue, p);
      u[j] = ue;
      x0[j] = xn;
      for (int i = 0; i < m; ++i) s_xp[i][j] = xn;
    }
    __syncthreads();  // s_xp is rewritten by the next tile
  }
}

struct Grid {
  int chunk, nunits, blocks;
};
Grid make_grid(int ntiles, int persistent, int remap) {
  Grid g;
  g.chunk = (ntiles + kXcd - 1) / kXcd;
  g.nunits = remap ? g.chunk * kXcd : ntiles;
  g.blocks = (persistent > 0 && persistent < g.nunits) ? persistent : g.nunits;
  return g;
}

template <int BASE, bool BF16, bool FIRST>
hipError_t launch_local_t(const LocalArgs &a, const LaunchTuning &t, hipStream_t s) {
  Grid g = make_grid(a.ntiles, t.local_grid, t.xcd_remap);
  if (t.nontemporal) {
    hipLaunchKernelGGL((k_local_step<BASE, BF16, FIRST, true, 4>), dim3(g.blocks), dim3(kBlock), 0,
                       s, a, g.chunk, g.nunits, t.xcd_remap);
  } else {
    hipLaunchKernelGGL((k_local_step<BASE, BF16, FIRST, false, 4>), dim3(g.blocks), dim3(kBlock),
                       0, s, a, g.chunk, g.nunits, t.xcd_remap);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_local_step(const LocalArgs &a, int base, bool bf16, bool first,
                             const LaunchTuning &t, hipStream_t s) {
  if (a.ntiles <= 0) return hipSuccess;
  if (base == 0) {
    if (bf16) {
      return first ? launch_local_t<0, true, true>(a, t, s) : launch_local_t<0, true, false>(a, t, s);
    }
    return first ? launch_local_t<0, false, true>(a, t, s) : launch_local_t<0, false, false>(a, t, s);
  }
  if (bf16) {
    return first ? launch_local_t<1, true, true>(a, t, s) : launch_local_t<1, true, false>(a, t, s);
  }
  return first ? launch_local_t<1, false, true>(a, t, s) : launch_local_t<1, false, false>(a, t, s);
}

hipError_t launch_outer_step(const OuterArgs &a, const LaunchTuning &t, hipStream_t s) {
  if (a.ntiles <= 0) return hipSuccess;
  Grid g = make_grid(a.ntiles, t.outer_grid, t.xcd_remap);
  if (t.nontemporal) {
    hipLaunchKernelGGL((k_outer_step<true, 2>), dim3(g.blocks), dim3(kBlock), 0, s, a, g.chunk,
                       g.nunits, t.xcd_remap);
  } else {
    hipLaunchKernelGGL((k_outer_step<false, 2>), dim3(g.blocks), dim3(kBlock), 0, s, a, g.chunk,
                       g.nunits, t.xcd_remap);
  }
  return hipGetLastError();
}

}  // namespace slowmo
