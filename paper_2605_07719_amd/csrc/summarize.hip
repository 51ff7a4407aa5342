// Block key summaries (Sec. 2.1 of the paper: every block is represented by the dimension-wise
// minima and maxima of its token keys).  One pass over K, no arithmetic: an HBM stream.
//
// Mapping: a thread owns 8 consecutive channels (one 16-byte load per token) of one block and walks
// the block's tokens; the d/8 threads of a block sit in consecutive lanes, so each load instruction
// of a wave covers whole 128/256-byte key rows and each store covers a whole summary row.
#include "fx_device.hpp"
#include "fx_kernels.hpp"

namespace fx {

template <int kD>
__global__ __launch_bounds__(256) void summarize_kernel(Params P, const uint16_t* __restrict__ K,
                                                        uint16_t* __restrict__ S) {
  constexpr int kLanes = kD / 8;         // lanes per token row
  constexpr int kBlocksPerWg = 256 / kLanes;
  const int b = blockIdx.z, j = blockIdx.y;
  const Geo geo = geometry(P, b, j);
  const int i = blockIdx.x * kBlocksPerWg + threadIdx.x / kLanes;
  if (i >= geo.n_blocks) return;
  const int chunk = threadIdx.x % kLanes;
  const int t_lo = i * geo.g;
  const int t_hi = min(t_lo + geo.g, geo.n_tokens);
  const uint16_t* src = K + P.seq_base[b] + (int64_t)j * P.kv_head_stride + chunk * 8;

  float mn[8], mx[8];
  {
    uint4 r = *reinterpret_cast<const uint4*>(src + (int64_t)t_lo * P.token_stride);
    unpack8(r, mn);
#pragma unroll
    for (int c = 0; c < 8; ++c) mx[c] = mn[c];
  }
#pragma unroll 4
  for (int t = t_lo + 1; t < t_hi; ++t) {
    uint4 r = *reinterpret_cast<const uint4*>(src + (int64_t)t * P.token_stride);
    float x[8];
    unpack8(r, x);
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      mn[c] = fminf(mn[c], x[c]);
      mx[c] = fmaxf(mx[c], x[c]);
    }
  }
  const int64_t blk = P.sum_base[(int64_t)b * P.n_kv_heads + j] + i;
  uint16_t* dst = S + (blk * 2) * kD + chunk * 8;
  *reinterpret_cast<uint4*>(dst) = pack8(mn);
  *reinterpret_cast<uint4*>(dst + kD) = pack8(mx);
}

hipError_t launch_summarize(const Params& P, const void* K, void* S, hipStream_t stream) {
  const int lanes = P.head_dim / 8;
  const int blocks_per_wg = 256 / lanes;
  dim3 grid((P.nb_stride + blocks_per_wg - 1) / blocks_per_wg, P.n_kv_heads, P.batch);
  if (P.head_dim == 128)
    hipLaunchKernelGGL(summarize_kernel<128>, grid, dim3(256), 0, stream, P, (const uint16_t*)K, (uint16_t*)S);
  else
    hipLaunchKernelGGL(summarize_kernel<64>, grid, dim3(256), 0, stream, P, (const uint16_t*)K, (uint16_t*)S);
  return hipGetLastError();
}

}  // namespace fx
