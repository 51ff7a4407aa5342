// Block scoring and per-head top-k (Sec. 2.1 of the paper: the query is compared with the metadata
// of all key blocks and the top-k blocks are selected; Sec. 5.3: one block size per GQA group, one
// budget per head).
//
// Stage 1 (score_kernel) streams the candidate summaries of one (sequence, KV head) once and scores
// them for up to 4 query heads of the group at a time:
//     score = sum_c max(q_c * mn_c, q_c * mx_c) = sum_c (max(q_c,0) * mx_c + min(q_c,0) * mn_c),
// every product is exact and the sum is accumulated in fp64, so the ranking agrees with an fp64
// evaluation except for candidates that are equal to ~1e-15.  Scores leave the kernel as 64-bit
// keys whose unsigned order is the order of the scores.
// Stage 2 (topk_kernel) finds, per (sequence, query head), the k-th largest key by a most-significant
// -digit-first radix select (8 passes of 8 bits), then writes the kept block indices in ascending
// order; among keys equal to the k-th the lowest block indices are kept.
#include "fx_device.hpp"
#include "fx_kernels.hpp"

namespace fx {

__device__ __forceinline__ uint64_t ordered_key(double s) {
  uint64_t u = (uint64_t)__double_as_longlong(s);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}

template <int kD, int kHP>
__global__ __launch_bounds__(256) void score_kernel(Params P, const uint16_t* __restrict__ q,
                                                    const uint16_t* __restrict__ S, uint64_t* __restrict__ keys) {
  constexpr int kLanes = kD / 8;
  constexpr int kCandPerIter = 256 / kLanes;
  constexpr int kIters = 4;
  constexpr int kTile = kCandPerIter * kIters;
  const int n_pass = (P.group + kHP - 1) / kHP;
  const int b = blockIdx.z, j = blockIdx.y / n_pass, pass = blockIdx.y % n_pass;
  const Geo geo = geometry(P, b, j);
  const int tile0 = blockIdx.x * kTile;
  if (tile0 >= geo.n_cand) return;
  const int chunk = threadIdx.x % kLanes;
  const int slot = threadIdx.x / kLanes;
  const int h0 = j * P.group + pass * kHP;
  const int nh = min(kHP, P.group - pass * kHP);

  double qp[kHP][8], qn[kHP][8];
#pragma unroll
  for (int r = 0; r < kHP; ++r) {
    float x[8];
    if (r < nh) {
      uint4 raw = *reinterpret_cast<const uint4*>(q + ((int64_t)b * P.n_q_heads + h0 + r) * kD + chunk * 8);
      unpack8(raw, x);
    } else {
#pragma unroll
      for (int c = 0; c < 8; ++c) x[c] = 0.f;
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      qp[r][c] = (double)fmaxf(x[c], 0.f);
      qn[r][c] = (double)fminf(x[c], 0.f);
    }
  }

  const uint16_t* sum_row =
      S + (P.sum_base[(int64_t)b * P.n_kv_heads + j] + geo.n_sink) * 2 * (int64_t)kD + chunk * 8;
  uint4 raw_mn[kIters], raw_mx[kIters];
#pragma unroll
  for (int it = 0; it < kIters; ++it) {
    const int r = tile0 + it * kCandPerIter + slot;
    const int rc = min(r, geo.n_cand - 1);  // clamped: stays inside the candidate range
    const uint16_t* p = sum_row + (int64_t)rc * 2 * kD;
    raw_mn[it] = *reinterpret_cast<const uint4*>(p);
    raw_mx[it] = *reinterpret_cast<const uint4*>(p + kD);
  }
#pragma unroll
  for (int it = 0; it < kIters; ++it) {
    const int r = tile0 + it * kCandPerIter + slot;
    float fmn[8], fmx[8];
    unpack8(raw_mn[it], fmn);
    unpack8(raw_mx[it], fmx);
    double dmn[8], dmx[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      dmn[c] = (double)fmn[c];
      dmx[c] = (double)fmx[c];
    }
#pragma unroll
    for (int hh = 0; hh < kHP; ++hh) {
      if (hh < nh) {
        double acc = 0.0;
#pragma unroll
        for (int c = 0; c < 8; ++c) acc = fma(qp[hh][c], dmx[c], fma(qn[hh][c], dmn[c], acc));
#pragma unroll
        for (int off = 1; off < kLanes; off <<= 1) acc += __shfl_xor(acc, off, kWave);
        if (chunk == 0 && r < geo.n_cand)
          keys[((int64_t)b * P.n_q_heads + h0 + hh) * P.nb_stride + geo.n_sink + r] = ordered_key(acc);
      }
    }
  }
}

__global__ __launch_bounds__(256) void topk_kernel(Params P, const uint64_t* __restrict__ keys,
                                                   const float* __restrict__ budget_frac,
                                                   const int32_t* __restrict__ budget_blocks,
                                                   int32_t* __restrict__ idx, int32_t* __restrict__ cnt) {
  __shared__ int hist[256];
  __shared__ int scan_scratch[4];
  __shared__ int count_scratch_a[4];
  __shared__ int count_scratch_b[4];
  __shared__ int s_digit, s_krem;

  const int b = blockIdx.y, h = blockIdx.x, j = h / P.group;
  const int tid = threadIdx.x;
  const Geo geo = geometry(P, b, j);
  const int64_t slot = (int64_t)b * P.n_q_heads + h;
  double want;
  if (budget_blocks)
    want = (double)budget_blocks[slot];
  else
    want = ceil((double)budget_frac[slot] * (double)geo.n_cand);
  const int limit = geo.n_cand < P.k_max ? geo.n_cand : P.k_max;
  const int k = want > 0.0 ? (want < (double)limit ? (int)want : limit) : 0;  // NaN falls to 0
  int32_t* out = idx + slot * P.k_max;
  const uint64_t* kh = keys + slot * P.nb_stride + geo.n_sink;
  const int n = geo.n_cand;

  if (tid == 0) cnt[slot] = k;
  if (k == 0) {
    for (int r = tid; r < P.k_max; r += 256) out[r] = -1;
    return;
  }
  if (k == n) {
    for (int r = tid; r < P.k_max; r += 256) out[r] = r < k ? geo.n_sink + r : -1;
    return;
  }

  // Radix select of the k-th largest key: `prefix` holds the digits fixed so far.
  uint64_t prefix = 0;
  int krem = k;
  for (int pass = 7; pass >= 0; --pass) {
    const int shift = pass * 8;
    const uint64_t hi_mask = pass == 7 ? 0ull : (~0ull << (shift + 8));
    hist[tid] = 0;
    __syncthreads();
    for (int base = 0; base < n; base += 256) {
      const int r = base + tid;
      bool match = false;
      unsigned digit = 0;
      if (r < n) {
        const uint64_t key = kh[r];
        match = (key & hi_mask) == prefix;
        digit = (unsigned)(key >> shift) & 255u;
      }
      // One LDS atomic per wave when all matching lanes agree on the digit (the usual case for the
      // sign/exponent digits), else one per lane.
      const unsigned long long mball = __ballot(match);
      if (mball) {
        const int leader = __ffsll((long long)mball) - 1;
        const unsigned d0 = __shfl(digit, leader, kWave);
        const unsigned long long same = __ballot(match && digit == d0);
        if (same == mball) {
          if ((tid & 63) == leader) atomicAdd(&hist[d0], __popcll(mball));
        } else if (match) {
          atomicAdd(&hist[digit], 1);
        }
      }
    }
    __syncthreads();
    const int dg = 255 - tid;  // thread t owns digit 255 - t, so a prefix sum over threads is a suffix sum over digits
    const int c = hist[dg];
    const int incl = block_incl_scan(c, scan_scratch);
    const int excl = incl - c;
    if (excl < krem && krem <= incl) {
      s_digit = dg;
      s_krem = krem - excl;
    }
    __syncthreads();
    prefix |= (uint64_t)s_digit << shift;
    krem = s_krem;
    __syncthreads();
  }
  const uint64_t kth = prefix;  // the k-th largest key; `krem` of the keys equal to it are kept

  int run_sel = 0, run_eq = 0;
  for (int base = 0; base < n; base += 256) {
    const int r = base + tid;
    const uint64_t key = r < n ? kh[r] : 0ull;
    const bool gt = r < n && key > kth;
    const bool eq = r < n && key == kth;
    int tot_eq, tot_sel;
    const int eq_before = run_eq + block_excl_count(eq, count_scratch_a, tot_eq);
    const bool sel = gt || (eq && eq_before < krem);
    const int pos = run_sel + block_excl_count(sel, count_scratch_b, tot_sel);
    if (sel && pos < P.k_max) out[pos] = geo.n_sink + r;
    run_eq += tot_eq;
    run_sel += tot_sel;
  }
  for (int r = k + tid; r < P.k_max; r += 256) out[r] = -1;
}

hipError_t launch_select(const Params& P, const void* q, const void* S, const float* budget_frac,
                         const int32_t* budget_blocks, int32_t* idx, int32_t* cnt, void* workspace,
                         hipStream_t stream) {
  const SelectWorkspace W = carve_select(P);
  uint64_t* keys = reinterpret_cast<uint64_t*>(static_cast<char*>(workspace) + W.keys_off);
  constexpr int kHP = 4;
  const int n_pass = (P.group + kHP - 1) / kHP;
  const int lanes = P.head_dim / 8;
  const int tile = (256 / lanes) * 4;
  dim3 sgrid((P.nb_stride + tile - 1) / tile, P.n_kv_heads * n_pass, P.batch);
  {
  ScopedSlot prof(kSlotScore, stream);
  if (P.head_dim == 128)
    hipLaunchKernelGGL((score_kernel<128, kHP>), sgrid, dim3(256), 0, stream, P, (const uint16_t*)q,
                       (const uint16_t*)S, keys);
  else
    hipLaunchKernelGGL((score_kernel<64, kHP>), sgrid, dim3(256), 0, stream, P, (const uint16_t*)q,
                       (const uint16_t*)S, keys);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  ScopedSlot prof(kSlotTopk, stream);
  hipLaunchKernelGGL(topk_kernel, dim3(P.n_q_heads, P.batch), dim3(256), 0, stream, P, (const uint64_t*)keys,
                     budget_frac, budget_blocks, idx, cnt);
  return hipGetLastError();
}

}  // namespace fx
