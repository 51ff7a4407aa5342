// Shared device-side definitions of the fluxion HIP kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fx {

constexpr int kMaxKvHeads = 64;
constexpr int kMaxGroup = 8;
constexpr int kWave = 64;
constexpr int kMaxSeqLen = 1 << 19;
constexpr float kNegBig = -1.0e30f;  // "no token seen yet" running maximum (finite, so differences stay finite)

// Everything a kernel needs to know about the cache placement; passed by value (kernarg).
struct Params {
  int32_t batch, n_q_heads, n_kv_heads, head_dim, group, max_seq_len;
  const int32_t* seq_len;
  const int64_t* seq_base;
  int64_t kv_head_stride, token_stride;
  const int64_t* sum_base;
  uint8_t gran[kMaxKvHeads];  // block size g_j of KV head j, in tokens (16..128)
  int32_t sink_tokens, window_tokens, k_max;
  int32_t nb_stride;  // row length of per-(b,h) block arrays: max over j of ceil(max_seq_len / g_j)
  int32_t group_union;  // decode only: every head of a group attends to the union of the group's selections
};

// Block geometry of one (sequence, KV head): see the header of the C ABI.
struct Geo {
  int32_t n_tokens, g, n_blocks, n_sink, w0, n_cand;
};

__device__ __forceinline__ Geo geometry(const Params& P, int b, int j) {
  Geo G;
  int n = P.seq_len[b];
  n = n < 0 ? 0 : (n > P.max_seq_len ? P.max_seq_len : n);
  G.n_tokens = n;
  G.g = P.gran[j];
  G.n_blocks = (n + G.g - 1) / G.g;
  G.n_sink = (P.sink_tokens + G.g - 1) / G.g;
  int first_window = n - P.window_tokens;
  first_window = first_window < 0 ? 0 : first_window;
  G.w0 = first_window / G.g;
  int nc = G.w0 - G.n_sink;
  G.n_cand = nc < 0 ? 0 : nc;
  return G;
}

// 16-byte load of data that is read once per step (K/V rows, summary rows): a non-temporal load, which
// streams through the caches without displacing what is reused (q, union entries, partial results).
// Measured on the attention kernel at 128K context: 0.72 -> 0.80 of the HBM peak from this hint alone.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 stream_load16(const void* p) {
  const u32x4_t v = __builtin_nontemporal_load(static_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// 8 consecutive bf16 values (one 16-byte load) -> 8 floats.
__device__ __forceinline__ void unpack8(const uint4& r, float* f) {
  f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x);
  f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
  f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z);
  f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
}

// Values that are bf16-exact floats -> 8 packed bf16.
__device__ __forceinline__ uint4 pack8(const float* f) {
  uint4 r;
  r.x = (__float_as_uint(f[0]) >> 16) | (__float_as_uint(f[1]) & 0xffff0000u);
  r.y = (__float_as_uint(f[2]) >> 16) | (__float_as_uint(f[3]) & 0xffff0000u);
  r.z = (__float_as_uint(f[4]) >> 16) | (__float_as_uint(f[5]) & 0xffff0000u);
  r.w = (__float_as_uint(f[6]) >> 16) | (__float_as_uint(f[7]) & 0xffff0000u);
  return r;
}

// acc + a.lo * b.lo + a.hi * b.hi on two packed bf16 pairs (v_dot2c_f32_bf16): exact products, fp32 sum.
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), acc, false);
}

// Operand and result vectors of the matrix-core instructions used here (v_mfma_f32_16x16x32_bf16: 8 bf16 per
// lane and operand; v_mfma_f32_16x16x16_bf16: 4 bf16 per lane and operand; both: 4 floats per lane).
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

// Cross-lane moves inside a row of 16 lanes (DPP): every lane reads a partner, so "old" is unused.
template <int kCtrl>
__device__ __forceinline__ float dpp_f(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), kCtrl, 0xf, 0xf, false));
}
constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7 - i within each 8
constexpr int kDppMirror = 0x140;      // lane i <-> 15 - i within each 16

// Sum over the kLanes (8 or 16) consecutive lanes that share one token row; every lane gets the sum.
template <int kLanes>
__device__ __forceinline__ float group_sum(float x) {
  x += dpp_f<kDppXor1>(x);
  x += dpp_f<kDppXor2>(x);
  x += dpp_f<kDppHalfMirror>(x);
  if (kLanes == 16) x += dpp_f<kDppMirror>(x);
  return x;
}

constexpr int kMaxWaves = 16;  // waves of the largest workgroup (1024 threads)

// Block-wide exclusive prefix count of a predicate over a workgroup of kW waves.
// `scratch` is kW ints of LDS reserved for this call site; two barriers per call.
template <int kW = 4>
__device__ __forceinline__ int block_excl_count(bool flag, int* scratch, int& total) {
  unsigned long long ball = __ballot(flag);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int before = __popcll(ball & ((1ull << lane) - 1ull));
  __syncthreads();  // previous users of scratch are done
  if (lane == 0) scratch[wave] = __popcll(ball);
  __syncthreads();
  int off = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kW; ++w) {
    int c = scratch[w];
    if (w < wave) off += c;
    tot += c;
  }
  total = tot;
  return off + before;
}

// Inclusive prefix sum over the threads of a workgroup of kW waves.  `scratch`: kW ints of LDS.
template <int kW = 4>
__device__ __forceinline__ int block_incl_scan(int v, int* scratch) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    int up = __shfl_up(v, off, kWave);
    if (lane >= off) v += up;
  }
  __syncthreads();
  if (lane == 63) scratch[wave] = v;
  __syncthreads();
  int add = 0;
#pragma unroll
  for (int w = 0; w < kW - 1; ++w)
    if (w < wave) add += scratch[w];
  return v + add;
}

}  // namespace fx
