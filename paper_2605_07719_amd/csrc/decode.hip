// Split-K sparse decode attention with an online-softmax merge (App. A.1 of the paper:
// s = q K^T / sqrt(D), O = softmax(s) V over the kept tokens; Sec. 2.2 and Sec. 4 step 4: the result
// over the chosen blocks is fused with the result over the retained sink and window tokens; Sec. 5.3
// and Sec. 6.2: the unit of work is one GQA group of one sequence).
//
// Three kernels on one stream:
//   plan_kernel    per (sequence, KV head): OR the chosen-block lists of the group's heads into a
//                  per-block head mask, add the sink and window blocks for every head, and compact
//                  the non-empty blocks into an ascending "union list" of (block, head mask) entries.
//                  A block that several heads of the group want is then read from HBM once.
//   attend_kernel  persistent workgroups walk work items; an item is a chunk of one group's union
//                  list.  Each wave takes 16-token slices of the chunk: coalesced 16-byte-per-lane
//                  loads of K and V rows, fp32 dot products reduced inside the 8/16 lanes that share
//                  a token, running (max, sum, accumulator) per head in registers.  Per item one
//                  partial triple per head is written.  The chunk length adapts to the total amount
//                  of selected work so that small steps still spread over the whole chip.
//   merge_kernel   per (sequence, query head): fuse the partial triples of the group's items in
//                  item order (fixed order => reproducible results).
// Logits are kept in the log2 domain (q is pre-multiplied by log2(e)/sqrt(D)) so the exponentials
// are single v_exp_f32 instructions.
#include "fx_device.hpp"
#include "fx_kernels.hpp"

namespace fx {

__global__ __launch_bounds__(256) void plan_kernel(Params P, const int32_t* __restrict__ idx,
                                                   const int32_t* __restrict__ cnt, uint32_t* __restrict__ uni,
                                                   int32_t* __restrict__ ucount, int union_cap) {
  extern __shared__ uint32_t mask_words[];  // one byte of head mask per block, 4 blocks per word
  __shared__ int scratch[4];
  const int b = blockIdx.y, j = blockIdx.x, tid = threadIdx.x;
  const int grp = b * P.n_kv_heads + j;
  int counts[kMaxGroup];  // requested before the geometry so they arrive together with the sequence length
#pragma unroll
  for (int r = 0; r < kMaxGroup; ++r) {
    counts[r] = 0;
    if (r < P.group) {
      const int c = cnt[(int64_t)b * P.n_q_heads + j * P.group + r];
      counts[r] = c < 0 ? 0 : (c > P.k_max ? P.k_max : c);
    }
  }
  const Geo geo = geometry(P, b, j);
  const int n_words = (geo.n_blocks + 3) >> 2;
  for (int w = tid; w < n_words; w += 256) mask_words[w] = 0u;
  __syncthreads();
  // The heads' index lists are cut into pieces of 512 entries and the pieces are dealt to the 4 waves
  // round-robin, so short lists of different heads are walked concurrently and a long list is shared by
  // all waves; a lane keeps eight index loads in flight before the LDS atomics that consume them.
  {
    const int wave = tid >> 6, lane = tid & 63;
    int piece_no = 0;
#pragma unroll
    for (int r = 0; r < kMaxGroup; ++r) {
      if (r >= P.group) break;
      const int64_t slot = (int64_t)b * P.n_q_heads + j * P.group + r;
      const int c = counts[r];
      const int32_t* list = idx + slot * P.k_max;
      for (int base = 0; base < c; base += 512, ++piece_no) {
        if ((piece_no & 3) != wave) continue;
        int i[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int e = base + u * 64 + lane;
          i[u] = e < c ? list[e] : -1;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (i[u] >= 0 && i[u] < geo.n_blocks) atomicOr(&mask_words[i[u] >> 2], (1u << r) << ((i[u] & 3) * 8));
      }
    }
  }
  __syncthreads();
  // ordered compaction: thread t owns the consecutive blocks [t * per, (t + 1) * per), so one block
  // scan of the per-thread counts gives every thread its write position
  const uint32_t all = (1u << P.group) - 1u;
  const int per = (geo.n_blocks + 255) >> 8;
  const int i0 = min(tid * per, geo.n_blocks), i1 = min(i0 + per, geo.n_blocks);
  auto mask_of = [&](int i) -> uint32_t {
    if (i < geo.n_sink || i >= geo.w0) return all;
    const uint32_t m = (mask_words[i >> 2] >> ((i & 3) * 8)) & 255u;
    return (P.group_union && m) ? all : m;
  };
  int mine = 0;
  for (int i = i0; i < i1; ++i) mine += mask_of(i) != 0u;
  const int incl = block_incl_scan(mine, scratch);
  int pos = incl - mine;
  uint32_t* dst = uni + (int64_t)grp * union_cap;
  for (int i = i0; i < i1; ++i) {
    const uint32_t m = mask_of(i);
    if (m != 0u) {
      if (pos < union_cap) dst[pos] = ((uint32_t)i << 8) | m;
      ++pos;
    }
  }
  if (tid == 255) ucount[grp] = incl < union_cap ? incl : union_cap;
}

template <int kD, int kG>
__global__ __launch_bounds__(256) void attend_kernel(Params P, const uint16_t* __restrict__ q,
                                                     const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
                                                     const uint32_t* __restrict__ uni,
                                                     const int32_t* __restrict__ ucount, int union_cap,
                                                     int32_t* __restrict__ sched, float* __restrict__ acc_part,
                                                     float* __restrict__ ml_part, int items_cap) {
  constexpr int kLanes = kD / 8;        // lanes that share one token row
  constexpr int kTPL = 64 / kLanes;     // token rows per wave-wide load
  constexpr int kLoads = 16 / kTPL;     // loads per 16-token slice
  // register budget: prefetching pays only where it does not cost a resident wave (measured)
  constexpr bool kPrefetch = kD == 128 ? (kG == 6 || kG == 7) : (kG >= 7);
  extern __shared__ int s_prefix[];     // [n_groups + 1] exclusive prefix of items per group
  __shared__ float s_red[4][kG][kD + 2];
  __shared__ int s_scan[4];
  __shared__ unsigned long long s_total;
  __shared__ uint32_t s_ent[kMaxChunkEntries];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int chunk = lane % kLanes, tslot = lane / kLanes;
  const int n_groups = P.batch * P.n_kv_heads;

  // ---- split sizing, computed identically by every workgroup -------------------------------------
  if (tid == 0) s_total = 0ull;
  __syncthreads();
  {
    unsigned long long local = 0;
    for (int g = tid; g < n_groups; g += 256) local += (unsigned long long)ucount[g] * P.gran[g % P.n_kv_heads];
    if (local) atomicAdd(&s_total, local);
  }
  __syncthreads();
  const unsigned long long total_tokens = s_total;
  int shift = 0;
  while (shift < kMaxChunkShift && total_tokens > (unsigned long long)kTargetItems * (kMinChunkTokens << shift)) ++shift;
  const int chunk_tokens = kMinChunkTokens << shift;
  {
    const int per = (n_groups + 255) / 256;
    const int g_lo = min(tid * per, n_groups), g_hi = min(g_lo + per, n_groups);
    int local = 0;
    for (int g = g_lo; g < g_hi; ++g) {
      const int cb = max(1, chunk_tokens / (int)P.gran[g % P.n_kv_heads]);
      local += (ucount[g] + cb - 1) / cb;
    }
    const int incl = block_incl_scan(local, s_scan);
    int run = incl - local;
    for (int g = g_lo; g < g_hi; ++g) {
      s_prefix[g] = run;
      const int cb = max(1, chunk_tokens / (int)P.gran[g % P.n_kv_heads]);
      run += (ucount[g] + cb - 1) / cb;
    }
    if (tid == 255) s_prefix[n_groups] = incl;  // the last thread's inclusive sum is the item total
  }
  __syncthreads();
  const int n_items = min(s_prefix[n_groups], items_cap);
  if (blockIdx.x == 0) {
    for (int g = tid; g <= n_groups; g += 256) sched[g] = s_prefix[g];
    if (tid == 0) sched[n_groups + 1] = chunk_tokens;
  }

  const float q_scale = 1.4426950408889634f * rsqrtf((float)kD);

  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    // group of this item: the last g with s_prefix[g] <= item
    int lo = 0, hi = n_groups - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (s_prefix[mid] <= item) lo = mid; else hi = mid - 1;
    }
    const int grp = lo, b = grp / P.n_kv_heads, j = grp % P.n_kv_heads;
    const Geo geo = geometry(P, b, j);
    const int cb = max(1, chunk_tokens / geo.g);
    const int n_union = ucount[grp];
    const int e0 = (item - s_prefix[grp]) * cb;
    const int e1 = min(e0 + cb, n_union);
    const int spb = geo.g >> 4;  // 16-token slices per block
    const int n_slices = (e1 - e0) * spb;
    const uint32_t* entries = uni + (int64_t)grp * union_cap;
    const int64_t head_base = P.seq_base[b] + (int64_t)j * P.kv_head_stride + chunk * 8;
    const uint16_t* Kb = K + head_base;
    const uint16_t* Vb = V + head_base;

    // the item's union entries go to LDS once, so the per-slice address chain starts from LDS
    if (tid < e1 - e0) s_ent[tid] = entries[e0 + tid];
    __syncthreads();

    // q stays packed (2 bf16 per register); the 1/sqrt(D) and log2(e) factors are applied to the dot product
    uint4 qp[kG];
    float acc[kG][8], m_run[kG], l_run[kG];
#pragma unroll
    for (int r = 0; r < kG; ++r) {
      qp[r] = *reinterpret_cast<const uint4*>(q + ((int64_t)b * P.n_q_heads + j * kG + r) * kD + chunk * 8);
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[r][c] = 0.f;
      m_run[r] = kNegBig;
      l_run[r] = 0.f;
    }

    // With kPrefetch the K/V rows of the wave's next slice are requested before the current slice is
    // consumed (one slice, 8 KiB at d = 128, always in flight per wave) at the price of 32 registers;
    // without it the kernel relies on more resident waves per SIMD.
    uint4 kraw[kLoads], vraw[kLoads], knext[kLoads], vnext[kLoads];
    uint32_t mask_next = 0;
    int t0_next = 0;
    auto issue = [&](int sl, uint4* kr, uint4* vr, uint32_t& mask_out, int& t0_out) {
      const uint32_t ent = __builtin_amdgcn_readfirstlane(s_ent[sl / spb]);
      mask_out = ent & 255u;
      t0_out = (int)(ent >> 8) * geo.g + (sl % spb) * 16 + tslot;
#pragma unroll
      for (int i = 0; i < kLoads; ++i) {
        const int64_t row = (int64_t)min(t0_out + i * kTPL, geo.n_tokens - 1) * P.token_stride;
        kr[i] = *reinterpret_cast<const uint4*>(Kb + row);
        vr[i] = *reinterpret_cast<const uint4*>(Vb + row);
      }
    };
    if (kPrefetch && wave < n_slices) issue(wave, knext, vnext, mask_next, t0_next);

    for (int sl = wave; sl < n_slices; sl += 4) {
      if (kPrefetch) {
#pragma unroll
        for (int i = 0; i < kLoads; ++i) {
          kraw[i] = knext[i];
          vraw[i] = vnext[i];
        }
      } else {
        issue(sl, kraw, vraw, mask_next, t0_next);
      }
      const uint32_t mask = mask_next;
      const int t0 = t0_next;
      if (kPrefetch && sl + 4 < n_slices) issue(sl + 4, knext, vnext, mask_next, t0_next);

      // logits (log2 domain) of the slice's tokens for every head that wants this block
      float sp[kG][kLoads];
#pragma unroll
      for (int i = 0; i < kLoads; ++i) {
        const bool valid = t0 + i * kTPL < geo.n_tokens;
#pragma unroll
        for (int r = 0; r < kG; ++r) {
          if (mask & (1u << r)) {
            float dot = dot2_bf16(qp[r].x, kraw[i].x, 0.f);
            dot = dot2_bf16(qp[r].y, kraw[i].y, dot);
            dot = dot2_bf16(qp[r].z, kraw[i].z, dot);
            dot = dot2_bf16(qp[r].w, kraw[i].w, dot);
            dot = group_sum<kLanes>(dot) * q_scale;
            sp[r][i] = valid ? dot : kNegBig;
          }
        }
      }
      // online-softmax update per head: new maximum, rescale, probabilities
#pragma unroll
      for (int r = 0; r < kG; ++r) {
        if (mask & (1u << r)) {
          float mx = sp[r][0];
#pragma unroll
          for (int i = 1; i < kLoads; ++i) mx = fmaxf(mx, sp[r][i]);
          const float m_new = fmaxf(m_run[r], mx);
          const float alpha = __builtin_amdgcn_exp2f(m_run[r] - m_new);
          float psum = 0.f;
#pragma unroll
          for (int i = 0; i < kLoads; ++i) {
            const bool valid = t0 + i * kTPL < geo.n_tokens;
            sp[r][i] = valid ? __builtin_amdgcn_exp2f(sp[r][i] - m_new) : 0.f;
            psum += sp[r][i];
          }
          l_run[r] = l_run[r] * alpha + psum;
          m_run[r] = m_new;
          if (__ballot(alpha != 1.f)) {  // the maximum moved somewhere in the wave (rare once warmed up)
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[r][c] *= alpha;
          }
        }
      }
      // acc += p * v
#pragma unroll
      for (int i = 0; i < kLoads; ++i) {
        float vf[8];
        unpack8(vraw[i], vf);
#pragma unroll
        for (int r = 0; r < kG; ++r) {
          if (mask & (1u << r)) {
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[r][c] = fmaf(sp[r][i], vf[c], acc[r][c]);
          }
        }
      }
    }

    // ---- fuse the token slots of the wave, then the 4 waves, then write the item's partial --------
#pragma unroll
    for (int r = 0; r < kG; ++r) {
      float M = m_run[r];
#pragma unroll
      for (int off = kLanes; off < 64; off <<= 1) M = fmaxf(M, __shfl_xor(M, off, kWave));
      const float w = __builtin_amdgcn_exp2f(m_run[r] - M);
      float lw = l_run[r] * w;
#pragma unroll
      for (int off = kLanes; off < 64; off <<= 1) lw += __shfl_xor(lw, off, kWave);
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        float a = acc[r][c] * w;
#pragma unroll
        for (int off = kLanes; off < 64; off <<= 1) a += __shfl_xor(a, off, kWave);
        acc[r][c] = a;
      }
      if (tslot == 0) {
#pragma unroll
        for (int c = 0; c < 8; ++c) s_red[wave][r][chunk * 8 + c] = acc[r][c];
        if (chunk == 0) {
          s_red[wave][r][kD] = M;
          s_red[wave][r][kD + 1] = lw;
        }
      }
    }
    __syncthreads();
    for (int x = tid; x < kG * kD; x += 256) {
      const int r = x / kD, c = x % kD;
      float M = s_red[0][r][kD];
#pragma unroll
      for (int w = 1; w < 4; ++w) M = fmaxf(M, s_red[w][r][kD]);
      float o = 0.f, L = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float sc = __builtin_amdgcn_exp2f(s_red[w][r][kD] - M);
        o += s_red[w][r][c] * sc;
        L += s_red[w][r][kD + 1] * sc;
      }
      acc_part[((int64_t)item * kG + r) * kD + c] = o;
      if (c == 0) {
        ml_part[((int64_t)item * kG + r) * 2] = M;
        ml_part[((int64_t)item * kG + r) * 2 + 1] = L;
      }
    }
    __syncthreads();
  }
}

// One workgroup per (sequence, query head).  The group's items are spread over 256 / (kD/4) slices of
// threads, each thread owning 4 channels; a slice folds its items into a running (max, sum, accumulator)
// in item order, and the slices are then fused in slice order (fixed order => reproducible results).
template <int kD>
__global__ __launch_bounds__(256) void merge_kernel(Params P, const int32_t* __restrict__ sched,
                                                    const float* __restrict__ acc_part,
                                                    const float* __restrict__ ml_part, float* __restrict__ out,
                                                    int items_cap) {
  constexpr int kLanesC = kD / 4;          // threads per item (4 channels each)
  constexpr int kSlices = 256 / kLanesC;   // items in flight per iteration
  __shared__ float s_o[kSlices][kD];
  __shared__ float s_m[kSlices], s_l[kSlices];
  const int b = blockIdx.y, h = blockIdx.x, tid = threadIdx.x;
  const int G = P.group, j = h / G, r = h % G;
  const int grp = b * P.n_kv_heads + j;
  const int p0 = min(sched[grp], items_cap), p1 = min(sched[grp + 1], items_cap);

  const int slice = tid / kLanesC, cl = tid % kLanesC;
  float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
  float m_run = kNegBig, L = 0.f;
  // loads are unconditional (an item in which this head took no part contributes exact zeros), so
  // the compiler can keep several iterations in flight
#pragma unroll 4
  for (int it = p0 + slice; it < p1; it += kSlices) {
    const float2 ml = *reinterpret_cast<const float2*>(ml_part + ((int64_t)it * G + r) * 2);
    const float4 a = *reinterpret_cast<const float4*>(acc_part + ((int64_t)it * G + r) * kD + cl * 4);
    const float m_new = fmaxf(m_run, ml.x);
    const float keep = __builtin_amdgcn_exp2f(m_run - m_new), w = __builtin_amdgcn_exp2f(ml.x - m_new);
    L = L * keep + ml.y * w;
    o.x = o.x * keep + a.x * w; o.y = o.y * keep + a.y * w; o.z = o.z * keep + a.z * w; o.w = o.w * keep + a.w * w;
    m_run = m_new;
  }
  *reinterpret_cast<float4*>(&s_o[slice][cl * 4]) = o;
  if (cl == 0) {
    s_m[slice] = m_run;
    s_l[slice] = L;
  }
  __syncthreads();
  if (tid < kD) {
    float M = s_m[0];
#pragma unroll
    for (int sl = 1; sl < kSlices; ++sl) M = fmaxf(M, s_m[sl]);
    float acc = 0.f, Lt = 0.f;
#pragma unroll
    for (int sl = 0; sl < kSlices; ++sl) {
      const float w = __builtin_amdgcn_exp2f(s_m[sl] - M);
      acc += s_o[sl][tid] * w;
      Lt += s_l[sl] * w;
    }
    out[((int64_t)b * P.n_q_heads + h) * kD + tid] = Lt > 0.f ? acc / Lt : 0.f;
  }
}

template <int kD, int kG>
static hipError_t launch_attend(const Params& P, const void* q, const void* K, const void* V, const uint32_t* uni,
                                const int32_t* ucount, const DecodeWorkspace& W, int32_t* sched, float* acc_part,
                                float* ml_part, int n_cu, hipStream_t stream) {
  static int wg_per_cu = 0;  // occupancy of this instantiation, queried once
  const size_t lds = (size_t)(P.batch * P.n_kv_heads + 1) * sizeof(int);
  if (wg_per_cu == 0) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attend_kernel<kD, kG>, 256, lds) != hipSuccess || n < 1) n = 1;
    wg_per_cu = n > 8 ? 8 : n;
  }
  int grid = n_cu * wg_per_cu;
  if (grid > W.items_cap) grid = W.items_cap;
  hipLaunchKernelGGL((attend_kernel<kD, kG>), dim3(grid), dim3(256), lds, stream, P, (const uint16_t*)q,
                     (const uint16_t*)K, (const uint16_t*)V, uni, ucount, W.union_cap, sched, acc_part, ml_part,
                     W.items_cap);
  return hipGetLastError();
}

template <int kD>
static hipError_t dispatch_group(const Params& P, const void* q, const void* K, const void* V, const uint32_t* uni,
                                 const int32_t* ucount, const DecodeWorkspace& W, int32_t* sched, float* acc_part,
                                 float* ml_part, int n_cu, hipStream_t stream) {
  switch (P.group) {
#define FX_CASE(G) \
  case G:          \
    return launch_attend<kD, G>(P, q, K, V, uni, ucount, W, sched, acc_part, ml_part, n_cu, stream);
    FX_CASE(1) FX_CASE(2) FX_CASE(3) FX_CASE(4) FX_CASE(5) FX_CASE(6) FX_CASE(7) FX_CASE(8)
#undef FX_CASE
  }
  return hipErrorInvalidValue;
}

hipError_t launch_decode(const Params& P, const void* q, const void* K, const void* V, const int32_t* idx,
                         const int32_t* cnt, float* out, void* workspace, int n_cu, hipStream_t stream) {
  const DecodeWorkspace W = carve_decode(P);
  char* ws = static_cast<char*>(workspace);
  uint32_t* uni = reinterpret_cast<uint32_t*>(ws + W.union_off);
  int32_t* ucount = reinterpret_cast<int32_t*>(ws + W.ucount_off);
  int32_t* sched = reinterpret_cast<int32_t*>(ws + W.sched_off);
  float* acc_part = reinterpret_cast<float*>(ws + W.acc_off);
  float* ml_part = reinterpret_cast<float*>(ws + W.ml_off);

  const size_t plan_lds = (size_t)((P.nb_stride + 3) / 4) * sizeof(uint32_t);
  {
    ScopedSlot prof(kSlotPlan, stream);
    hipLaunchKernelGGL(plan_kernel, dim3(P.n_kv_heads, P.batch), dim3(256), plan_lds, stream, P, idx, cnt, uni,
                       ucount, W.union_cap);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  {
    ScopedSlot prof(kSlotAttend, stream);
    e = P.head_dim == 128
            ? dispatch_group<128>(P, q, K, V, uni, ucount, W, sched, acc_part, ml_part, n_cu, stream)
            : dispatch_group<64>(P, q, K, V, uni, ucount, W, sched, acc_part, ml_part, n_cu, stream);
  }
  if (e != hipSuccess) return e;
  ScopedSlot prof(kSlotMerge, stream);
  if (P.head_dim == 128)
    hipLaunchKernelGGL(merge_kernel<128>, dim3(P.n_q_heads, P.batch), dim3(256), 0, stream, P, (const int32_t*)sched,
                       (const float*)acc_part, (const float*)ml_part, out, W.items_cap);
  else
    hipLaunchKernelGGL(merge_kernel<64>, dim3(P.n_q_heads, P.batch), dim3(256), 0, stream, P, (const int32_t*)sched,
                       (const float*)acc_part, (const float*)ml_part, out, W.items_cap);
  return hipGetLastError();
}

}  // namespace fx
