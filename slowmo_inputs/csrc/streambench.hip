// Stream microbenchmark: the access shapes the optimizer kernels choose among,
// as one parameterised kernel, so that their bandwidth ceilings on this chip can
// be measured side by side (bench.py --ladder).  Measurement infrastructure: no
// optimizer arithmetic, not part of the library.
//
// Memory is seen as `units` x S streams of n floats each, stream s of unit u at
// base + (u * S + s) * stride.  A tile is B * VPT consecutive 16-byte vectors of
// one unit; its workgroup reads the tile from the first R streams of the unit,
// adds them up and writes the sum to W streams -- the first W (in place) or
// streams R .. R+W-1 (out of place).  (units, S, R, W) = (m, 3, 3, 2) in place
// is the traffic of the SGD local step, (1, m+2, m+2, m+2) that of the outer
// step, (m, 1, 1, 0) / (m, 1, 0, 1) a plain read / write.
#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

typedef float V4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) V4 GV4;

template <bool NT>
__device__ __forceinline__ V4 ld(const float *p) {
  const GV4 *q = (const GV4 *)(reinterpret_cast<uintptr_t>(p));
  if constexpr (NT) return __builtin_nontemporal_load(q);
  return *q;
}
template <bool NT>
__device__ __forceinline__ void st(float *p, V4 v) {
  GV4 *q = (GV4 *)(reinterpret_cast<uintptr_t>(p));
  if constexpr (NT) {
    __builtin_nontemporal_store(v, q);
  } else {
    *q = v;
  }
}

struct Shape {
  int64_t stride;          // floats between streams
  int64_t tiles_per_unit;
  int64_t total;           // units * tiles_per_unit
  int S, R, W, wfirst;     // wfirst: first stream written (0 in place, R out of place)
  int units;
  int order;               // 0: unit-major (all tiles of unit 0, then unit 1, ...); 1: unit-minor
  int remap;               // 1: each XCD (workgroup id mod 8) takes one contiguous eighth
  int iters;               // tiles per workgroup, consecutive (1: load, store, retire)
};

template <int B, int VPT, bool NTL, bool NTS>
__global__ __launch_bounds__(B) void k_streams(float *base, Shape sh) {
  int64_t b = blockIdx.x;
  if (sh.remap) {
    const int64_t chunk = (static_cast<int64_t>(gridDim.x) + 7) / 8;
    b = (b % 8) * chunk + b / 8;
  }
  for (int it = 0; it < sh.iters; ++it) {
    const int64_t L = b * sh.iters + it;
    if (L >= sh.total) return;
    // one 64-bit division, not four: it is expanded inline and a wave that
    // moves a few KiB feels the length of what runs before its first load
    int64_t u, k;
    if (sh.order) {
      k = L / sh.units;
      u = L - k * sh.units;
    } else {
      u = L / sh.tiles_per_unit;
      k = L - u * sh.tiles_per_unit;
    }
    float *p = base + u * sh.S * sh.stride + (k * (B * VPT) + threadIdx.x) * 4;
    V4 acc[VPT];
#pragma unroll
    for (int v = 0; v < VPT; ++v) acc[v] = V4{1.f, 2.f, 3.f, 4.f};
#pragma unroll 8
    for (int s = 0; s < sh.R; ++s) {
#pragma unroll
      for (int v = 0; v < VPT; ++v) acc[v] += ld<NTL>(p + s * sh.stride + v * (B * 4));
    }
    if (sh.W == 0) {  // read-only: a store that never happens keeps the loads alive
      V4 t = acc[0];
#pragma unroll
      for (int v = 1; v < VPT; ++v) t += acc[v];
      if (t.x == 1.2345e30f) st<NTS>(p, t);
    }
#pragma unroll 8
    for (int s = 0; s < sh.W; ++s) {
#pragma unroll
      for (int v = 0; v < VPT; ++v) st<NTS>(p + (sh.wfirst + s) * sh.stride + v * (B * 4), acc[v]);
    }
  }
}

// lds: bytes of (unused) dynamic LDS per workgroup -- caps how many workgroups
// share a CU (160 KiB per CU).
template <int B, int VPT, bool NTL, bool NTS>
hipError_t launch_nt(float *base, const Shape &sh, int lds, dim3 g, hipStream_t s) {
  if (lds > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_streams<B, VPT, NTL, NTS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((k_streams<B, VPT, NTL, NTS>), g, dim3(B), lds, s, base, sh);
  return hipGetLastError();
}

template <int B, int VPT>
hipError_t launch(float *base, const Shape &sh, int nt, int lds, hipStream_t s) {
  const int64_t blocks = (sh.total + sh.iters - 1) / sh.iters;
  const int64_t grid = sh.remap ? (blocks + 7) / 8 * 8 : blocks;
  if (grid > INT32_MAX) return hipErrorInvalidValue;
  const dim3 g(static_cast<unsigned>(grid));
  switch (nt & 3) {  // bit 0: non-temporal loads, bit 1: non-temporal stores
    case 0: return launch_nt<B, VPT, false, false>(base, sh, lds, g, s);
    case 1: return launch_nt<B, VPT, true, false>(base, sh, lds, g, s);
    case 2: return launch_nt<B, VPT, false, true>(base, sh, lds, g, s);
    default: return launch_nt<B, VPT, true, true>(base, sh, lds, g, s);
  }
}

}  // namespace

// One launch of the stream kernel.  base: device buffer of at least
// units * S * stride floats; n (floats per stream, <= stride) must be a multiple
// of 4 * B * VPT and stride a multiple of 4.  Supported (B, VPT): see the switch
// below.  nt: bit 0 =
// non-temporal loads, bit 1 = non-temporal stores.  lds: bytes of unused
// dynamic LDS per workgroup (0 .. 160 KiB), to cap the workgroups per CU.  Returns 0 or a
// hipError_t value (hipErrorInvalidValue for an unsupported shape).
extern "C" int slowmo_inputs_streambench(void *base, int64_t stride, int32_t units, int32_t S,
                                         int32_t R, int32_t W, int32_t in_place, int64_t n,
                                         int32_t B, int32_t VPT, int32_t nt, int32_t order,
                                         int32_t remap, int32_t iters, int32_t lds, void *stream) {
  const int64_t tile = static_cast<int64_t>(4) * B * VPT;
  if (!base || units < 1 || S < 1 || R < 0 || W < 0 || R > S || W > S || R + W == 0 ||
      (!in_place && R + W > S) || n <= 0 || n > stride || stride % 4 || tile <= 0 || n % tile ||
      iters < 1 || lds < 0 || lds > 160 * 1024)
    return static_cast<int>(hipErrorInvalidValue);
  Shape sh{};
  sh.stride = stride;
  sh.tiles_per_unit = n / tile;
  sh.total = sh.tiles_per_unit * units;
  sh.S = S;
  sh.R = R;
  sh.W = W;
  sh.wfirst = in_place ? 0 : R;
  sh.units = units;
  sh.order = order ? 1 : 0;
  sh.remap = remap ? 1 : 0;
  sh.iters = iters;
  float *p = static_cast<float *>(base);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipErrorInvalidValue;
  const int key = B * 100 + VPT;
  switch (key) {
    case 6401: e = launch<64, 1>(p, sh, nt, lds, s); break;
    case 6402: e = launch<64, 2>(p, sh, nt, lds, s); break;
    case 6404: e = launch<64, 4>(p, sh, nt, lds, s); break;
    case 6408: e = launch<64, 8>(p, sh, nt, lds, s); break;
    case 12801: e = launch<128, 1>(p, sh, nt, lds, s); break;
    case 12804: e = launch<128, 4>(p, sh, nt, lds, s); break;
    case 25601: e = launch<256, 1>(p, sh, nt, lds, s); break;
    case 25602: e = launch<256, 2>(p, sh, nt, lds, s); break;
    case 25604: e = launch<256, 4>(p, sh, nt, lds, s); break;
    case 25608: e = launch<256, 8>(p, sh, nt, lds, s); break;
    case 25616: e = launch<256, 16>(p, sh, nt, lds, s); break;
    case 25632: e = launch<256, 32>(p, sh, nt, lds, s); break;
    case 51201: e = launch<512, 1>(p, sh, nt, lds, s); break;
    case 51204: e = launch<512, 4>(p, sh, nt, lds, s); break;
    case 51208: e = launch<512, 8>(p, sh, nt, lds, s); break;
    case 51216: e = launch<512, 16>(p, sh, nt, lds, s); break;
    case 51232: e = launch<512, 32>(p, sh, nt, lds, s); break;
    case 102401: e = launch<1024, 1>(p, sh, nt, lds, s); break;
    case 102402: e = launch<1024, 2>(p, sh, nt, lds, s); break;
    case 102404: e = launch<1024, 4>(p, sh, nt, lds, s); break;
    case 102408: e = launch<1024, 8>(p, sh, nt, lds, s); break;
    case 102416: e = launch<1024, 16>(p, sh, nt, lds, s); break;
    case 102432: e = launch<1024, 32>(p, sh, nt, lds, s); break;
    default: break;
  }
  return static_cast<int>(e);
}
