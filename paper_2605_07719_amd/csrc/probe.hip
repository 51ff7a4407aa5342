// Measurement aids (not part of the method): a plain streaming read and a plain copy of a device
// buffer.  The benchmark uses them to state the HBM read rate this machine reaches with no arithmetic at
// all, and to scale hardware-counter readings against a transfer of known size.
#include "../../include/fluxion.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fx_kernels.hpp"

namespace {

constexpr int kUnroll = 8;

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

template <bool kNonTemporal>
__device__ __forceinline__ uint4 load16(const uint4* p) {
  if (kNonTemporal) {
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
  }
  return *p;
}

// Every wave reads one contiguous share of the buffer, kUnroll wave-wide 1 KiB loads in flight (grid-stride
// loops with power-of-two strides were measured up to 20% slower at some launch shapes).
template <bool kNonTemporal>
__global__ __launch_bounds__(256) void probe_read_kernel(const uint4* __restrict__ src, size_t n16,
                                                         uint32_t* __restrict__ sink) {
  const size_t n_waves = (size_t)gridDim.x * 4;
  const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const size_t per = (n16 + n_waves - 1) / n_waves;
  const size_t lo = wave * per, hi = lo + per < n16 ? lo + per : n16;
  const int lane = threadIdx.x & 63;
  uint4 acc = make_uint4(0, 0, 0, 0);
  size_t i = lo + lane;
  for (; i + (kUnroll - 1) * 64 < hi; i += kUnroll * 64) {
    uint4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) v[u] = load16<kNonTemporal>(src + i + u * 64);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w;
    }
  }
  for (; i < hi; i += 64) {
    uint4 v = load16<kNonTemporal>(src + i);
    acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
  }
  // data-dependent, practically never true: keeps the loads alive without a store per thread
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = acc.x;
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                         size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

int grid_for(int wg_per_cu) {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
    n = 256;
  if (wg_per_cu < 1) wg_per_cu = 1;
  if (wg_per_cu > 32) wg_per_cu = 32;
  return n * wg_per_cu;
}

}  // namespace

extern "C" {

fx_status fx_probe_read(const void* src, size_t bytes, void* sink, int wg_per_cu, void* stream) {
  if (!src || !sink || bytes < 16 || (reinterpret_cast<uintptr_t>(src) & 15u)) return FX_ERR_INVALID_ARG;
  return fx::launch(probe_read_kernel<false>, dim3(grid_for(wg_per_cu)), dim3(256), 0, static_cast<hipStream_t>(stream),
                    static_cast<const uint4*>(src), bytes / 16, static_cast<uint32_t*>(sink)) == hipSuccess
             ? FX_OK
             : FX_ERR_HIP;
}

fx_status fx_probe_read_streaming(const void* src, size_t bytes, void* sink, int wg_per_cu, void* stream) {
  if (!src || !sink || bytes < 16 || (reinterpret_cast<uintptr_t>(src) & 15u)) return FX_ERR_INVALID_ARG;
  return fx::launch(probe_read_kernel<true>, dim3(grid_for(wg_per_cu)), dim3(256), 0, static_cast<hipStream_t>(stream),
                    static_cast<const uint4*>(src), bytes / 16, static_cast<uint32_t*>(sink)) == hipSuccess
             ? FX_OK
             : FX_ERR_HIP;
}

fx_status fx_probe_copy(void* dst, const void* src, size_t bytes, int wg_per_cu, void* stream) {
  if (!src || !dst || bytes < 16 || (reinterpret_cast<uintptr_t>(src) & 15u) ||
      (reinterpret_cast<uintptr_t>(dst) & 15u))
    return FX_ERR_INVALID_ARG;
  return fx::launch(probe_copy_kernel, dim3(grid_for(wg_per_cu)), dim3(256), 0, static_cast<hipStream_t>(stream),
                    static_cast<const uint4*>(src), static_cast<uint4*>(dst), bytes / 16) == hipSuccess
             ? FX_OK
             : FX_ERR_HIP;
}

}  // extern "C"
