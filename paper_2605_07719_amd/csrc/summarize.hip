// Block key summaries (Sec. 2.1 of the paper: every block is represented by the dimension-wise
// minima and maxima of its token keys).  One pass over K, no arithmetic: an HBM stream.
//
// Mapping: a thread owns 8 consecutive channels (one 16-byte load per token) of one block and walks
// the block's tokens; the d/8 threads of a block sit in consecutive lanes, so each load instruction
// of a wave covers whole 128/256-byte key rows and each store covers a whole summary row.
#include "fx_device.hpp"
#include "fx_kernels.hpp"

namespace fx {

// With `prev_len` (append mode) only the blocks that hold tokens at or after prev_len[b] are redone.
template <int kD>
__global__ __launch_bounds__(256) void summarize_kernel(Params P, const uint16_t* __restrict__ K,
                                                        uint16_t* __restrict__ S,
                                                        const int32_t* __restrict__ prev_len) {
  constexpr int kLanes = kD / 8;         // lanes per token row
  constexpr int kBlocksPerWg = 256 / kLanes;
  const int b = blockIdx.z, j = blockIdx.y;
  const Geo geo = geometry(P, b, j);
  int first_block = 0;
  if (prev_len) {
    const int p = prev_len[b];
    first_block = (p < 0 ? 0 : p) / geo.g;
  }
  const int i = first_block + blockIdx.x * kBlocksPerWg + threadIdx.x / kLanes;
  if (i >= geo.n_blocks) return;
  const int chunk = threadIdx.x % kLanes;
  const int t_lo = i * geo.g;
  const int t_hi = min(t_lo + geo.g, geo.n_tokens);
  const uint16_t* src = K + P.seq_base[b] + (int64_t)j * P.kv_head_stride + chunk * 8;

  float mn[8], mx[8];
  {
    uint4 r = stream_load16(src + (int64_t)t_lo * P.token_stride);
    unpack8(r, mn);
#pragma unroll
    for (int c = 0; c < 8; ++c) mx[c] = mn[c];
  }
#pragma unroll 8
  for (int t = t_lo + 1; t < t_hi; ++t) {
    uint4 r = stream_load16(src + (int64_t)t * P.token_stride);
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

// Summary pyramid: one coarse block = `ratio` consecutive fine blocks; same thread mapping as above,
// reading summary rows instead of key rows.
template <int kD>
__global__ __launch_bounds__(256) void coarsen_kernel(Params Pf, Params Pc, const uint16_t* __restrict__ Sf,
                                                      uint16_t* __restrict__ Sc) {
  constexpr int kLanes = kD / 8;
  constexpr int kBlocksPerWg = 256 / kLanes;
  const int b = blockIdx.z, j = blockIdx.y;
  const Geo gc = geometry(Pc, b, j);
  const Geo gf = geometry(Pf, b, j);
  const int i = blockIdx.x * kBlocksPerWg + threadIdx.x / kLanes;
  if (i >= gc.n_blocks) return;
  const int chunk = threadIdx.x % kLanes;
  const int ratio = gc.g / gf.g;
  const int f_lo = i * ratio;
  const int f_hi = min(f_lo + ratio, gf.n_blocks);
  const uint16_t* src = Sf + Pf.sum_base[(int64_t)b * Pf.n_kv_heads + j] * 2 * (int64_t)kD + chunk * 8;
  float mn[8], mx[8];
  unpack8(stream_load16(src + (int64_t)f_lo * 2 * kD), mn);
  unpack8(stream_load16(src + (int64_t)f_lo * 2 * kD + kD), mx);
  for (int f = f_lo + 1; f < f_hi; ++f) {
    float a[8], c[8];
    unpack8(stream_load16(src + (int64_t)f * 2 * kD), a);
    unpack8(stream_load16(src + (int64_t)f * 2 * kD + kD), c);
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      mn[t] = fminf(mn[t], a[t]);
      mx[t] = fmaxf(mx[t], c[t]);
    }
  }
  uint16_t* dst = Sc + (Pc.sum_base[(int64_t)b * Pc.n_kv_heads + j] + i) * 2 * (int64_t)kD + chunk * 8;
  *reinterpret_cast<uint4*>(dst) = pack8(mn);
  *reinterpret_cast<uint4*>(dst + kD) = pack8(mx);
}

hipError_t launch_coarsen(const Params& Pf, const Params& Pc, const void* Sf, void* Sc, hipStream_t stream) {
  const int blocks_per_wg = 256 / (Pc.head_dim / 8);
  dim3 grid((Pc.nb_stride + blocks_per_wg - 1) / blocks_per_wg, Pc.n_kv_heads, Pc.batch);
  if (Pc.head_dim == 128)
    return launch(coarsen_kernel<128>, grid, dim3(256), 0, stream, Pf, Pc, (const uint16_t*)Sf, (uint16_t*)Sc);
  return launch(coarsen_kernel<64>, grid, dim3(256), 0, stream, Pf, Pc, (const uint16_t*)Sf, (uint16_t*)Sc);
}

hipError_t launch_summarize(const Params& P, const void* K, void* S, const int32_t* prev_len, int max_new_tokens,
                            hipStream_t stream) {
  const int lanes = P.head_dim / 8;
  const int blocks_per_wg = 256 / lanes;
  // append mode: at most ceil(max_new / 16) + 1 blocks per (sequence, KV head) change
  const int blocks = prev_len ? (max_new_tokens + 15) / 16 + 1 : P.nb_stride;
  dim3 grid((blocks + blocks_per_wg - 1) / blocks_per_wg, P.n_kv_heads, P.batch);
  if (P.head_dim == 128)
    return launch(summarize_kernel<128>, grid, dim3(256), 0, stream, P, (const uint16_t*)K, (uint16_t*)S, prev_len);
  return launch(summarize_kernel<64>, grid, dim3(256), 0, stream, P, (const uint16_t*)K, (uint16_t*)S, prev_len);
}

}  // namespace fx
