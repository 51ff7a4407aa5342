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
//   attend_kernel  the union lists of all groups, cut into 16-token slices, form one global slice
//                  sequence; every workgroup of the launch takes an equal contiguous share of it (a
//                  "unit"), so the work per workgroup is balanced whatever the budgets, block sizes
//                  and sequence lengths are.  Where a unit crosses from one group into the next it
//                  is cut into segments; the tail of the sequence is cut into small units that
//                  workgroups claim from a counter as they finish.  Within a segment each wave takes
//                  every fourth slice: coalesced, non-temporal 16-byte-per-lane loads of K and V rows
//                  (each row is read once per step), running (max, sum, accumulator) per head in
//                  registers.  The arithmetic comes in two forms: a vector form (fp32 dot products
//                  reduced inside the 8/16 lanes that share a token; head_dim 64 and groups of fewer
//                  than 4 heads) and a matrix-core form (K Q^T and P V on bf16 MFMA with fp32
//                  accumulation; head_dim 128, 4 to 8 heads per group), described where it starts.
//                  Per segment one partial triple per head is written, to slot
//                  unit + group (strictly increasing along the slice sequence, hence unique).
//   merge_kernel   per (sequence, query head): fuse the partial triples of the group's segments in
//                  slot order (fixed order => reproducible results).
// The exponentials are single v_exp_f32 instructions (base 2): dot products stay unscaled and the factor
// log2(e)/sqrt(D) is folded into the exponent's fused multiply-add; the running maxima are scaled when a
// partial is written, so the partials and the merge work in the scaled log2 domain.
#include <atomic>

#include "fx_device.hpp"
#include "fx_kernels.hpp"

namespace fx {

#ifndef FX_PLAN_PIECE
#define FX_PLAN_PIECE 512
#endif

#ifndef FX_PLAN_WAVES
#define FX_PLAN_WAVES 8
#endif
constexpr int kPlanWaves = FX_PLAN_WAVES;  // a group is one workgroup's job; 8 waves measured best (4: long lists serialise, 16: slow start)
constexpr int kPlanThreads = 64 * kPlanWaves;

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(Params P, const int32_t* __restrict__ idx,
                                                   const int32_t* __restrict__ cnt, uint32_t* __restrict__ uni,
                                                   int32_t* __restrict__ ucount, int union_cap,
                                                   int32_t* __restrict__ claim_counter, int direct_w, int piece_cap) {
  extern __shared__ uint32_t mask_words[];  // one byte of head mask per block, 4 blocks per word
  __shared__ int scratch[kPlanWaves];
  __shared__ uint32_t s_not_dense;
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
  // The first piece of every head's list is requested here, by the wave that will walk it (wave r: head r), before
  // the counts and the sequence length have arrived: its addresses need only k_max, so the entries travel together
  // with them instead of one round trip later.  Entries past a list's count are dropped when the piece is used.
  constexpr int kPiece = FX_PLAN_PIECE;
  const int wave = tid >> 6, lane = tid & 63;
  int first_piece[kPiece / 64];
  {
    const bool mine = wave < P.group;
    const int32_t* list = idx + ((int64_t)b * P.n_q_heads + j * P.group + (mine ? wave : 0)) * P.k_max;
#pragma unroll
    for (int u = 0; u < kPiece / 64; ++u) {
      const int e = u * 64 + lane;
      first_piece[u] = (mine && e < P.k_max) ? list[e] : -1;
    }
  }
  const Geo geo = geometry(P, b, j);
  const int n_words = (geo.n_blocks + 3) >> 2;
  for (int w = tid; w < n_words; w += kPlanThreads) mask_words[w] = 0u;
  // A head whose list is exactly the candidates in ascending order (what fx_select writes for a dense head) gets
  // its bit from the block's position.  The list is still read once and compared entry by entry -- any other
  // list of that length (duplicates, junk, an external selector's fixed-size list on a short sequence) fails the
  // comparison and is walked like every other list -- but the comparison needs no LDS atomics.
  uint32_t maybe_dense = 0u;
#pragma unroll
  for (int r = 0; r < kMaxGroup; ++r)
    if (r < P.group && geo.n_cand > 0 && counts[r] == geo.n_cand) maybe_dense |= 1u << r;
  if (tid == 0) s_not_dense = 0u;
  __syncthreads();
  // The heads' index lists are cut into pieces of FX_PLAN_PIECE entries.  The first piece of head r belongs to
  // wave r (above); the further pieces of long lists are dealt to the waves round-robin, so a long list is shared
  // by all waves; a lane keeps all index loads of a piece in flight before the LDS atomics that consume them.
  // piece entries i[u] (entry number base + 64 u + lane of head r's list, -1 past the count c) -> head masks,
  // or, for a list that may be the whole candidate range, the comparison with that range
  auto consume = [&](int r, bool check, int base, int c, const int* i) {
    if (check) {
      bool ok = true;
#pragma unroll
      for (int u = 0; u < kPiece / 64; ++u) {
        const int e = base + u * 64 + lane;
        ok = ok && (e >= c || i[u] == geo.n_sink + e);
      }
      if (!ok) atomicOr(&s_not_dense, 1u << r);
    } else {
#pragma unroll
      for (int u = 0; u < kPiece / 64; ++u)
        if (i[u] >= 0 && i[u] < geo.n_blocks) atomicOr(&mask_words[i[u] >> 2], (1u << r) << ((i[u] & 3) * 8));
    }
  };
  auto walk = [&](uint32_t heads, uint32_t verify) {
    int piece_no = 0;
#pragma unroll
    for (int r = 0; r < kMaxGroup; ++r) {
      if (r >= P.group) break;
      if (!((heads >> r) & 1u)) continue;
      const bool check = (verify >> r) & 1u;
      const int64_t slot = (int64_t)b * P.n_q_heads + j * P.group + r;
      const int c = counts[r];
      const int32_t* list = idx + slot * P.k_max;
      int base = 0;
      if (r < kPlanWaves) {  // the first piece is already in wave r's registers
        if (wave == r && c > 0) {
          int i[kPiece / 64];
#pragma unroll
          for (int u = 0; u < kPiece / 64; ++u) i[u] = u * 64 + lane < c ? first_piece[u] : -1;
          consume(r, check, 0, c, i);
        }
        base = kPiece;
      }
      for (; base < c; base += kPiece, ++piece_no) {
        if (piece_no % kPlanWaves != wave) continue;
        int i[kPiece / 64];
#pragma unroll
        for (int u = 0; u < kPiece / 64; ++u) {
          const int e = base + u * 64 + lane;
          i[u] = e < c ? list[e] : -1;
        }
        consume(r, check, base, c, i);
      }
    }
  };
  walk((1u << P.group) - 1u, maybe_dense);
  __syncthreads();
  const uint32_t failed = s_not_dense;  // workgroup-uniform
  const uint32_t dense_heads = maybe_dense & ~failed;
  if (failed) {
    walk(failed, 0u);
    __syncthreads();
  }
  // Ordered compaction in two sweeps.  A wave owns a contiguous share of the blocks and walks it 64
  // blocks at a time: the first sweep counts the kept blocks (ballot + popcount, no barrier), one barrier
  // exchanges the wave totals, the second sweep writes each kept block at wave base + running count
  // + its rank inside the ballot, so every store instruction writes one contiguous run of entries.
  const uint32_t all = (1u << P.group) - 1u;
  const bool as_union = P.group_union != 0;
  // head mask of block i, 0 past `end`; branch-free with an unconditional (clamped) LDS read so that the
  // reads of an unrolled step are all in flight together
  auto mask_of = [&](int i, int end) -> uint32_t {
    const int ic = min(i, geo.n_blocks - 1);
    uint32_t m = (mask_words[ic >> 2] >> ((ic & 3) * 8)) & 255u;
    m |= dense_heads;  // (sink and window blocks are overridden below)
    m = (as_union && m != 0u) ? all : m;
    m = (ic < geo.n_sink || ic >= geo.w0) ? all : m;
    return i < end ? m : 0u;
  };
  const int per_wave = (geo.n_blocks + kPlanThreads - 1) / kPlanThreads * 64;  // a multiple of 64; all waves together cover n_blocks
  const int w_lo = min(wave * per_wave, geo.n_blocks), w_hi = min(w_lo + per_wave, geo.n_blocks);
  // four 64-block steps per iteration keep four LDS reads in flight
  int count = 0;
  for (int base = w_lo; base < w_hi; base += 256) {
    uint32_t m[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) m[u] = mask_of(base + u * 64 + lane, w_hi);
#pragma unroll
    for (int u = 0; u < 4; ++u) count += __popcll(__ballot(m[u] != 0u));
  }
  if (lane == 0) scratch[wave] = count;
  __syncthreads();
  int pos = 0, total = 0;
#pragma unroll
  for (int w = 0; w < kPlanWaves; ++w) {
    if (w < wave) pos += scratch[w];
    total += scratch[w];
  }
  // Direct mode (small steps): the list is stored cut into pieces of S = ceil(n / direct_w) entries (n = min(total,
  // union_cap) kept entries; at most direct_w pieces, the last one shorter), piece w at the fixed place
  // (grp * direct_w + w) * piece_cap, so that workgroup w of the attention kernel finds its work without a prefix
  // over the groups.  S <= ceil(union_cap / direct_w) = piece_cap.
  const int n_kept = total < union_cap ? total : union_cap;
  const int piece_len = direct_w > 0 ? (n_kept + direct_w - 1) / direct_w : 1;
  const float inv_piece_len = 1.0f / (float)(piece_len > 0 ? piece_len : 1);
  uint32_t* dst = uni + (direct_w > 0 ? (int64_t)grp * direct_w * piece_cap : (int64_t)grp * union_cap);
  for (int base = w_lo; base < w_hi; base += 256) {
    uint32_t m[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) m[u] = mask_of(base + u * 64 + lane, w_hi);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const unsigned long long kept = __ballot(m[u] != 0u);
      const int at = pos + __popcll(kept & ((1ull << lane) - 1ull));
      if (m[u] != 0u && at < union_cap) {
        int where = at;
        if (direct_w > 0) {  // at / piece_len: a float estimate, then exact integer corrections
          int w = (int)((float)at * inv_piece_len);
          w -= (w * piece_len > at);
          w += ((w + 1) * piece_len <= at);
          where = w * piece_cap + (at - w * piece_len);
        }
        dst[where] = ((uint32_t)(base + u * 64 + lane) << 8) | m[u];
      }
      pos += __popcll(kept);
    }
  }
  if (tid == 0) ucount[grp] = total < union_cap ? total : union_cap;
  if (grp == 0 && tid == 0) *claim_counter = 0;  // the attention kernel that follows claims units from it
}

// Division of the global slice sequence into units (a slice is 16 tokens of a union list).
//
// Throughput regime (at least FX_MIN_SHARE slices per workgroup): the first `n_static` units, one per
// workgroup of the launch and taken by workgroup number, are equal shares of the leading part of the
// sequence; the rest is cut into small units that workgroups claim from a counter as they become free.
// The claimed part evens out the differences in speed between workgroups (equal shares finish up to
// +-12% apart: waves of an older workgroup are served first on a CU, and the XCDs do not get identical
// bandwidth).  Units may span several groups; a unit is then processed in one segment per group.
//
// Latency regime (fewer slices): the step is cut into units of one workgroup's share, at least 4 slices
// (one per wave), and every group is padded to a whole number of units (`align`), so that no unit spans
// two groups and no workgroup pays two segment latencies.  Nothing is claimed.
//
// Unit boundaries depend only on the slice counts and the launch size, never on which workgroup takes a
// unit, so the partial results and their merge order are reproducible.
struct Split {
  int unit_s;      // slices per static unit
  int static_end;  // first slice of the claimed part
  int unit_d;      // slices per claimed unit
  int n_static;
  int n_claimed;
  int align;       // groups start at multiples of this many slices in the (padded) sequence
  __device__ __forceinline__ int unit_of(int slice) const {
    return slice < static_end ? slice / unit_s : n_static + (slice - static_end) / unit_d;
  }
  __device__ __forceinline__ int unit_begin(int u) const {
    return u < n_static ? u * unit_s : static_end + (u - n_static) * unit_d;
  }
  __device__ __forceinline__ int unit_len(int u) const { return u < n_static ? unit_s : unit_d; }
};
#ifndef FX_CLAIMED_PCT
#define FX_CLAIMED_PCT 25   // share of the sequence that is claimed
#endif
#ifndef FX_MIN_SHARE
#define FX_MIN_SHARE 64     // slices per workgroup from which the throughput regime applies
#endif
#ifndef FX_CLAIMED_UNIT
#define FX_CLAIMED_UNIT 20  // slices per claimed unit (5 per wave); measured optimum between 12 and 28
#endif
__device__ __forceinline__ Split make_split(int total_slices, int n_wg) {
  Split sp;
  const int share = (total_slices + n_wg - 1) / n_wg;  // slices per workgroup if all were static
  if (share < FX_MIN_SHARE) {
    sp.unit_s = share < 4 ? 4 : ((share + 3) & ~3);
    sp.align = sp.unit_s;
    sp.unit_d = 4;
    sp.n_claimed = 0;
    sp.n_static = 0;    // both set by finish_split() once the padded total is known
    sp.static_end = 0;
    return sp;
  }
  sp.align = 1;
  sp.n_static = n_wg;
  sp.unit_s = ((int)((int64_t)share * (100 - FX_CLAIMED_PCT) / 100) + 3) & ~3;
  sp.static_end = min(total_slices, sp.unit_s * n_wg);
  const int rest = total_slices - sp.static_end;
  // larger claimed units only where a workgroup would otherwise take more than kClaimedPerWg of them
  const int d = ((rest + kClaimedPerWg * n_wg - 1) / (kClaimedPerWg * n_wg) + 3) & ~3;
  sp.unit_d = d < FX_CLAIMED_UNIT ? FX_CLAIMED_UNIT : d;
  sp.n_claimed = (rest + sp.unit_d - 1) / sp.unit_d;
  return sp;
}
__device__ __forceinline__ void finish_split(Split& sp, int padded_total) {
  if (sp.align > 1) {
    sp.static_end = padded_total;
    sp.n_static = padded_total / sp.unit_s;  // padded_total is a multiple of unit_s
  }
}

struct FullSlice { static constexpr bool value = true; };
struct PartialSlice { static constexpr bool value = false; };

template <int kD, int kG, bool kMfma>
__global__ __launch_bounds__(256) void attend_kernel(Params P, const uint16_t* __restrict__ q,
                                                     const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
                                                     const uint32_t* __restrict__ uni,
                                                     const int32_t* __restrict__ ucount, int union_cap,
                                                     int32_t* __restrict__ sched, float* __restrict__ acc_part,
                                                     float* __restrict__ ml_part, int slots_cap, int direct_w,
                                                     int piece_cap) {
  constexpr int kLanes = kD / 8;        // lanes that share one token row
  constexpr int kTPL = 64 / kLanes;     // token rows per wave-wide load
  constexpr int kLoads = 16 / kTPL;     // loads per 16-token slice
  // Register budget of the vector form.  Up to 5 heads per group every head's logits are computed first, then the softmax
  // updates, then the accumulation (most independent work in flight; 3-5 resident waves per SIMD).  From 6
  // heads on that order needs > 200 registers (2 resident waves), so a slice is processed one head at a
  // time (only one head's probabilities live) and q is re-read from LDS per head: 142-160 registers,
  // 3 resident waves (measured +4% at 7 heads per group; at 4 heads the LDS reads cost 3%).
  constexpr bool kHeadMajor = kG >= 6 && !kMfma;
  // (In the vector form, requesting the next slice before the current one is consumed costs 32 more registers
  // and never paid for the resident wave it takes away; the matrix-core form has the registers to spare.)
  extern __shared__ int s_prefix[];     // [n_groups + 1] exclusive prefix of (padded) slices per group, then
                                        // [n_groups] per group: slices it really has | slices per block << 24
  __shared__ float s_red[4][kG][kD + 2];
  __shared__ int s_scan[4];
  __shared__ uint32_t s_ent[kEntriesPerPiece];
  __shared__ int s_claim;
  __shared__ uint4 s_q[kHeadMajor ? kG : 1][kD / 8];
  constexpr int kStageStride = kD / 8 + 1;  // 16-byte pieces per staged K row: the row plus one piece of padding
  __shared__ uint4 s_kstage[kMfma ? 4 : 1][kMfma ? 16 * kStageStride : 1];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int chunk = lane % kLanes, tslot = lane / kLanes;
  const int n_groups = P.batch * P.n_kv_heads;
  int* s_real = s_prefix + n_groups + 1;  // a segment then starts without a round trip to list lengths and block sizes

  // ---- the global slice sequence and its division, computed identically by every workgroup --------
  // (not in direct mode, where the plan kernel has already cut every group's list into one piece per workgroup)
  Split split{};
  int total_slices = 0;
  if (direct_w == 0) {
  {
    const int per = (n_groups + 255) / 256;
    const int g_lo = min(tid * per, n_groups), g_hi = min(g_lo + per, n_groups);
    // one round trip to global memory (list lengths and block sizes together); the later passes read LDS
    int local = 0;
    for (int g = g_lo; g < g_hi; ++g) {
      const int spb = (int)P.gran[g % P.n_kv_heads] >> 4;
      const int n = ucount[g] * spb;
      s_real[g] = n | (spb << 24);
      local += n;
    }
    auto slices_of = [&](int g) { return s_real[g] & 0xffffff; };  // this thread's own writes
    int incl = block_incl_scan(local, s_scan);
    split = make_split(s_scan[0] + s_scan[1] + s_scan[2] + s_scan[3], (int)gridDim.x);
    const int al = split.align;
    if (al > 1) {  // second pass over the padded counts
      local = 0;
      for (int g = g_lo; g < g_hi; ++g) local += (slices_of(g) + al - 1) / al * al;
      incl = block_incl_scan(local, s_scan);
    }
    int run = incl - local;
    for (int g = g_lo; g < g_hi; ++g) {
      s_prefix[g] = run;
      run += (slices_of(g) + al - 1) / al * al;
    }
    if (tid == 255) s_prefix[n_groups] = incl;  // the last thread's inclusive sum is the (padded) total
  }
  __syncthreads();
  total_slices = s_prefix[n_groups];
  finish_split(split, total_slices);
  if (blockIdx.x == 0) {
    for (int g = tid; g <= n_groups; g += 256) sched[g] = s_prefix[g];
    if (tid == 0) {
      sched[n_groups + 1] = split.unit_s;
      sched[n_groups + 2] = split.static_end;
      sched[n_groups + 3] = split.unit_d;
      sched[n_groups + 4] = split.n_static;
    }
  }
  }
  int32_t* claim_counter = sched + n_groups + 5;  // zeroed by plan_kernel
  const float q_scale = 1.4426950408889634f * rsqrtf((float)kD);

  int claimed = 0;
  // ---- one segment: slices [l0, l1) of group `grp`, counted from the start of `entries` (spb slices per entry);
  // the segment's partial goes to `slot`.  The first entries are requested up to entry `e_load_end` (exclusive),
  // which in direct mode does not depend on the list's length, so they travel together with it.  `claim_next`:
  // the segment ends a unit while units are being claimed (the claim is issued before the reduction).
  auto segment = [&](int grp, const uint32_t* entries, int l0, int l1, int spb, int e_load_end, int slot,
                     bool claim_next) {
    const int b = grp / P.n_kv_heads, j = grp % P.n_kv_heads;
    const int e_lo = l0 / spb, e_hi = (l1 - 1) / spb;                  // union entries touched (inclusive)
    // The first 256 union entries are requested here, together with q and the sequence's length and base
    // (everything a segment needs from global memory before its K/V rows: one round trip).
    uint32_t ent_next = e_lo + tid < e_load_end ? entries[e_lo + tid] : 0u;
    struct { int g, n_tokens; } geo;
    geo.g = spb << 4;
    {
      const int n = P.seq_len[b];
      geo.n_tokens = n < 0 ? 0 : (n > P.max_seq_len ? P.max_seq_len : n);
    }
    const int64_t head_base = P.seq_base[b] + (int64_t)j * P.kv_head_stride + chunk * 8;
    const uint16_t* Kb = K + head_base;
    const uint16_t* Vb = V + head_base;

    if constexpr (kMfma) {
    // ---- matrix-core form of the segment (head_dim 128) ----------------------------------------------------
    // Lane (row r = lane / 16, column c = lane % 16).  The K/V loads are the same as in the vector form: load i
    // gives this lane channels 8c .. 8c+7 of token 4i + r of the slice.
    //   S^T = K Q^T  (v_mfma_f32_16x16x32_bf16, 4 steps of 32 channels): the 16 K rows pass through a private,
    //     row-padded LDS region of the wave (written as loaded, read back with lane (r, c) taking 16 bytes of
    //     the row of token 4(c % 4) + c / 4 at piece 4 step + r), B = Q^T with head c % 8 in column c (heads
    //     twice: columns 8..15 repeat columns 0..7).  Result register i of lane (r, c): logit of token 4i + r
    //     for head c % 8 -- the same tokens whose V rows the lane holds.
    //   softmax: every lane works on its own head's 4 logits; the running maximum of a head is common to all
    //     its lanes and is only raised (one cross-row exchange, accumulators rescaled) when some logit exceeds it.
    //   O = P V  (v_mfma_f32_16x16x16_bf16, k = 4r + i <-> token 4i + r, one instruction per channel e of the
    //     lane's 8: column c <-> channel 8c + e): A = P, rows 0..7 the upper 16 bits of p of head c, rows 8..15
    //     the bf16 of what that cut off (so p enters with 16 mantissa bits and the two partial outputs add up
    //     at the end of the segment); B = V straight from the load registers (two byte permutes per channel).
    // The arithmetic per slice does not depend on how many heads want the block.
    static_assert(!kMfma || (kD == 128 && kG <= 8), "matrix-core path: head_dim 128, at most 8 heads per group");
    const int r = lane >> 4, c = lane & 15;
    const int my_head = c & 7;
    const bool is_lo = c >= 8;
    uint4* stage = s_kstage[wave];
    uint4 q_op[4];
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      q_op[st] = make_uint4(0u, 0u, 0u, 0u);
      if (my_head < kG)
        q_op[st] = *reinterpret_cast<const uint4*>(q + ((int64_t)b * P.n_q_heads + j * kG + my_head) * kD + 32 * st + 8 * r);
    }
    f32x4_t o_acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o_acc[e] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    float m_run = kNegBig, l_run = 0.f;
    const int tau_row = (4 * (c & 3) + (c >> 2)) * kStageStride;  // LDS row of the token that MFMA row c stands for

    for (int pe = e_lo; pe <= e_hi; pe += kEntriesPerPiece) {
    __syncthreads();  // the previous piece's readers are done
    s_ent[tid] = ent_next;
    __syncthreads();
    if (pe + kEntriesPerPiece + tid <= e_hi) ent_next = entries[pe + kEntriesPerPiece + tid];  // in flight during this piece
    const int p_lo = max(l0, pe * spb), p_hi = min(l1, (pe + kEntriesPerPiece) * spb);

    // The rows of the wave's next slice are requested before the current slice is worked on (two slices, 16 KiB,
    // in flight per wave; 162 registers, two resident workgroups per compute unit: +2% at the dense point,
    // where the kernel then streams as fast as a plain read of the same bytes, no change elsewhere).
    uint4 kraw_n[kLoads], vraw_n[kLoads];
    uint32_t ent_n = 0u;
    auto request = [&](int sl_) {
      const int e_ = sl_ / spb;
      ent_n = __builtin_amdgcn_readfirstlane(s_ent[e_ - pe]);
      const int tf_ = (int)(ent_n >> 8) * geo.g + (sl_ - e_ * spb) * 16;
#pragma unroll
      for (int i = 0; i < kLoads; ++i) {
        const int64_t row = (int64_t)min(tf_ + tslot + i * kTPL, geo.n_tokens - 1) * P.token_stride;
        kraw_n[i] = stream_load16(Kb + row);
        vraw_n[i] = stream_load16(Vb + row);
      }
    };
    if (p_lo + wave < p_hi) request(p_lo + wave);
    for (int sl = p_lo + wave; sl < p_hi; sl += 4) {
      const int e = sl / spb;
      const uint32_t ent = ent_n;
      const uint32_t mask = ent & 255u;
      const int t_first = (int)(ent >> 8) * geo.g + (sl - e * spb) * 16;  // first token of the slice
      const int t0 = t_first + tslot;                                      // tslot == r at head_dim 128
      uint4 kraw[kLoads], vraw[kLoads];
#pragma unroll
      for (int i = 0; i < kLoads; ++i) {
        kraw[i] = kraw_n[i];
        vraw[i] = vraw_n[i];
      }
      if (sl + 4 < p_hi) request(sl + 4);
      // K rows -> LDS -> A operand.  Only this wave touches its region and a wave's LDS instructions execute in
      // order: the fences keep the compiler from reordering across them; no barrier instruction is needed.
#pragma unroll
      for (int i = 0; i < kLoads; ++i) stage[(4 * i + r) * kStageStride + c] = kraw[i];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      f32x4_t d = {0.f, 0.f, 0.f, 0.f};
      uint4 k_op[4];
#pragma unroll
      for (int st = 0; st < 4; ++st) k_op[st] = stage[tau_row + 4 * st + r];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int st = 0; st < 4; ++st)
        d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, k_op[st]),
                                                    __builtin_bit_cast(bf16x8_t, q_op[st]), d, 0, 0, 0);
      // softmax of this lane's head over its 4 tokens
      const bool active = ((mask >> my_head) & 1u) != 0u && my_head < kG;
      bool ok[4];
      float sp[4];
      float mx = kNegBig;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ok[i] = active && (t0 + i * kTPL < geo.n_tokens);
        sp[i] = ok[i] ? d[i] : kNegBig;
        mx = fmaxf(mx, sp[i]);
      }
      if (__ballot(mx > m_run)) {  // some head's maximum moves (rare once warmed up): raise it for all its lanes
        mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
        mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * q_scale);
        l_run *= alpha;
        m_run = m_new;
        // accumulator register i of this lane belongs to head-row 4r + i, i.e. head (4r + i) % 8, whose factor
        // sits in the lanes of column (4r + i) % 8
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float a = __shfl(alpha, (4 * r + i) & 7, kWave);
#pragma unroll
          for (int e8 = 0; e8 < 8; ++e8) o_acc[e8][i] *= a;
        }
      }
      const float m_scaled = m_run * q_scale;
      uint32_t pbits[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float pv = ok[i] ? __builtin_amdgcn_exp2f(fmaf(sp[i], q_scale, -m_scaled)) : 0.f;
        l_run += pv;
        const float hi = __uint_as_float(__float_as_uint(pv) & 0xffff0000u);
        pbits[i] = __float_as_uint(is_lo ? pv - hi : pv);  // the upper halves are packed below
      }
      uint2 p_op;
      p_op.x = __builtin_amdgcn_perm(pbits[1], pbits[0], 0x07060302u);
      p_op.y = __builtin_amdgcn_perm(pbits[3], pbits[2], 0x07060302u);
      const s16x4_t p_vec = __builtin_bit_cast(s16x4_t, p_op);
#pragma unroll
      for (int w = 0; w < 4; ++w) {  // dword w of the V registers holds channels 2w (low half) and 2w + 1
        const uint32_t v0 = w == 0 ? vraw[0].x : w == 1 ? vraw[0].y : w == 2 ? vraw[0].z : vraw[0].w;
        const uint32_t v1 = w == 0 ? vraw[1].x : w == 1 ? vraw[1].y : w == 2 ? vraw[1].z : vraw[1].w;
        const uint32_t v2 = w == 0 ? vraw[2].x : w == 1 ? vraw[2].y : w == 2 ? vraw[2].z : vraw[2].w;
        const uint32_t v3 = w == 0 ? vraw[3].x : w == 1 ? vraw[3].y : w == 2 ? vraw[3].z : vraw[3].w;
        uint2 even, odd;
        even.x = __builtin_amdgcn_perm(v1, v0, 0x05040100u);
        even.y = __builtin_amdgcn_perm(v3, v2, 0x05040100u);
        odd.x = __builtin_amdgcn_perm(v1, v0, 0x07060302u);
        odd.y = __builtin_amdgcn_perm(v3, v2, 0x07060302u);
        o_acc[2 * w] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(p_vec, __builtin_bit_cast(s16x4_t, even), o_acc[2 * w], 0, 0, 0);
        o_acc[2 * w + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(p_vec, __builtin_bit_cast(s16x4_t, odd), o_acc[2 * w + 1], 0, 0, 0);
      }
    }
    }  // pieces

    // the claim of the next unit is requested before the last segment's reduction, which hides its latency
    if (claim_next && tid == 0) claimed = atomicAdd(claim_counter, 1);

    // ---- the wave's partial: add the two halves of p's split, sum l over the rows, hand over to the 4-wave fuse --
    {
      float lt = l_run;
      lt += __shfl_xor(lt, 16, kWave);
      lt += __shfl_xor(lt, 32, kWave);
#pragma unroll
      for (int e8 = 0; e8 < 8; ++e8) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float x = o_acc[e8][i];
          x += __shfl_xor(x, 32, kWave);  // head-row 4r + i (upper bits of p) + head-row 4r + i + 8 (the rest)
          o_acc[e8][i] = x;
        }
      }
      if (r < 2) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int head = 4 * r + i;
          if (head < kG) {
#pragma unroll
            for (int e8 = 0; e8 < 8; ++e8) s_red[wave][head][c * 8 + e8] = o_acc[e8][i];
          }
        }
      }
      if (r == 0 && c < kG) {
        s_red[wave][c][kD] = m_run;
        s_red[wave][c][kD + 1] = lt;
      }
    }
    } else {
    // q stays packed (2 bf16 per register) and unscaled (the softmax scale is applied in the exponent)
    uint4 qp[kHeadMajor ? 1 : kG];
    if constexpr (kHeadMajor) {  // visible to all waves after the barrier that precedes the first piece
      if (tid < kG * kLanes)
        s_q[tid / kLanes][tid % kLanes] = *reinterpret_cast<const uint4*>(
            q + ((int64_t)b * P.n_q_heads + j * kG + tid / kLanes) * kD + (tid % kLanes) * 8);
    }
    float acc[kG][8], m_run[kG], l_run[kG];
#pragma unroll
    for (int r = 0; r < kG; ++r) {
      if constexpr (!kHeadMajor)
        qp[r] = *reinterpret_cast<const uint4*>(q + ((int64_t)b * P.n_q_heads + j * kG + r) * kD + chunk * 8);
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[r][c] = 0.f;
      m_run[r] = kNegBig;
      l_run[r] = 0.f;
    }

    // the segment's union entries pass through LDS in pieces, so the per-slice address chain starts from LDS
    for (int pe = e_lo; pe <= e_hi; pe += kEntriesPerPiece) {
    __syncthreads();  // the previous piece's readers are done
    s_ent[tid] = ent_next;
    __syncthreads();
    if (pe + kEntriesPerPiece + tid <= e_hi) ent_next = entries[pe + kEntriesPerPiece + tid];  // in flight during this piece
    const int p_lo = max(l0, pe * spb), p_hi = min(l1, (pe + kEntriesPerPiece) * spb);

    for (int sl = p_lo + wave; sl < p_hi; sl += 4) {
      // the slice's 16 K rows and 16 V rows: kLoads wave-wide loads each, 16 bytes per lane
      const int e = sl / spb;
      const uint32_t ent = __builtin_amdgcn_readfirstlane(s_ent[e - pe]);
      const uint32_t mask = ent & 255u;
      const int t_first = (int)(ent >> 8) * geo.g + (sl - e * spb) * 16;  // first token of the slice
      const int t0 = t_first + tslot;
      const bool full = t_first + 16 <= geo.n_tokens;  // wave-uniform; false only in a sequence's last block
      uint4 kraw[kLoads], vraw[kLoads];
#pragma unroll
      for (int i = 0; i < kLoads; ++i) {
        const int64_t row = (int64_t)min(t0 + i * kTPL, geo.n_tokens - 1) * P.token_stride;
        kraw[i] = stream_load16(Kb + row);
        vraw[i] = stream_load16(Vb + row);
      }

      // The slice's arithmetic, compiled twice: kFull drops every per-row validity test.  Logits stay
      // unscaled (log2(e)/sqrt(D) is folded into the exponent's fused multiply-add); the running maxima
      // m_run are therefore unscaled too and are scaled when the partial is written.
      auto compute = [&](auto full_tag) {
      constexpr bool kFull = decltype(full_tag)::value;
      if constexpr (kHeadMajor) {
#pragma unroll
        for (int r = 0; r < kG; ++r) {
          if (mask & (1u << r)) {
            __asm__ volatile("" ::: "memory");  // keeps the LDS read of q inside the loop instead of in registers
            const uint4 qv = s_q[r][chunk];
            float sp[kLoads];
#pragma unroll
            for (int i = 0; i < kLoads; ++i) {
              const bool valid = kFull || t0 + i * kTPL < geo.n_tokens;
              float dot = dot2_bf16(qv.x, kraw[i].x, 0.f);
              dot = dot2_bf16(qv.y, kraw[i].y, dot);
              dot = dot2_bf16(qv.z, kraw[i].z, dot);
              dot = dot2_bf16(qv.w, kraw[i].w, dot);
              dot = group_sum<kLanes>(dot);
              sp[i] = valid ? dot : kNegBig;
            }
            float mx = sp[0];
#pragma unroll
            for (int i = 1; i < kLoads; ++i) mx = fmaxf(mx, sp[i]);
            const float m_new = fmaxf(m_run[r], mx);
            const float alpha = __builtin_amdgcn_exp2f((m_run[r] - m_new) * q_scale);
            const float m_scaled = m_new * q_scale;
            float psum = 0.f;
#pragma unroll
            for (int i = 0; i < kLoads; ++i) {
              const bool valid = kFull || t0 + i * kTPL < geo.n_tokens;
              sp[i] = valid ? __builtin_amdgcn_exp2f(fmaf(sp[i], q_scale, -m_scaled)) : 0.f;
              psum += sp[i];
            }
            l_run[r] = l_run[r] * alpha + psum;
            m_run[r] = m_new;
            if (__ballot(alpha != 1.f)) {  // the maximum moved somewhere in the wave (rare once warmed up)
#pragma unroll
              for (int c = 0; c < 8; ++c) acc[r][c] *= alpha;
            }
#pragma unroll
            for (int i = 0; i < kLoads; ++i) {
              float vf[8];
              unpack8(vraw[i], vf);
#pragma unroll
              for (int c = 0; c < 8; ++c) acc[r][c] = fmaf(sp[i], vf[c], acc[r][c]);
            }
          }
        }
      } else {
        // logits (log2 domain) of the slice's tokens for every head that wants this block
        float sp[kG][kLoads];
#pragma unroll
        for (int i = 0; i < kLoads; ++i) {
          const bool valid = kFull || t0 + i * kTPL < geo.n_tokens;
#pragma unroll
          for (int r = 0; r < kG; ++r) {
            if (mask & (1u << r)) {
              float dot = dot2_bf16(qp[r].x, kraw[i].x, 0.f);
              dot = dot2_bf16(qp[r].y, kraw[i].y, dot);
              dot = dot2_bf16(qp[r].z, kraw[i].z, dot);
              dot = dot2_bf16(qp[r].w, kraw[i].w, dot);
              dot = group_sum<kLanes>(dot);
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
            const float alpha = __builtin_amdgcn_exp2f((m_run[r] - m_new) * q_scale);
            const float m_scaled = m_new * q_scale;
            float psum = 0.f;
#pragma unroll
            for (int i = 0; i < kLoads; ++i) {
              const bool valid = kFull || t0 + i * kTPL < geo.n_tokens;
              sp[r][i] = valid ? __builtin_amdgcn_exp2f(fmaf(sp[r][i], q_scale, -m_scaled)) : 0.f;
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
      };  // compute
      if (full) compute(FullSlice{}); else compute(PartialSlice{});
    }
    }  // pieces

    // the claim of the next unit is requested before the last segment's reduction, which hides its latency
    if (claim_next && tid == 0) claimed = atomicAdd(claim_counter, 1);

    // ---- fuse the token slots of the wave, then the 4 waves, then write the segment's partial -----
#pragma unroll
    for (int r = 0; r < kG; ++r) {
      float M = m_run[r];
#pragma unroll
      for (int off = kLanes; off < 64; off <<= 1) M = fmaxf(M, __shfl_xor(M, off, kWave));
      const float w = __builtin_amdgcn_exp2f((m_run[r] - M) * q_scale);
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
    }  // vector form
    __syncthreads();
    for (int x = tid; x < kG * kD; x += 256) {
      const int r = x / kD, c = x % kD;
      float M = s_red[0][r][kD];
#pragma unroll
      for (int w = 1; w < 4; ++w) M = fmaxf(M, s_red[w][r][kD]);
      float o = 0.f, L = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float sc = __builtin_amdgcn_exp2f((s_red[w][r][kD] - M) * q_scale);
        o += s_red[w][r][c] * sc;
        L += s_red[w][r][kD + 1] * sc;
      }
      acc_part[((int64_t)slot * kG + r) * kD + c] = o;
      if (c == 0) {
        ml_part[((int64_t)slot * kG + r) * 2] = M * q_scale;  // the merge works in the scaled log2 domain
        ml_part[((int64_t)slot * kG + r) * 2 + 1] = L;
      }
    }
    __syncthreads();
  };  // segment

  // ---- direct mode (small steps): workgroup w of group grp takes the w-th of direct_w pieces of the group's list,
  // which the plan kernel stored at a fixed place: no prefix over the groups, one segment, one partial.
  if (direct_w > 0) {
    const int grp = blockIdx.x / direct_w, w = blockIdx.x - grp * direct_w;
    const int spb = (int)P.gran[grp % P.n_kv_heads] >> 4;
    const int total = ucount[grp];
    const int piece_len = (total + direct_w - 1) / direct_w;  // as the plan kernel cut the list
    const int n_mine = max(min(total - w * piece_len, piece_len), 0);
    segment(grp, uni + ((int64_t)grp * direct_w + w) * piece_cap, 0, n_mine * spb, spb, piece_cap, (int)blockIdx.x,
            false);
    return;
  }

  int unit = blockIdx.x;
  for (;;) {
  int s0 = 0, s1 = 0;
  if (unit < split.n_static + split.n_claimed) {
    s0 = split.unit_begin(unit);
    s1 = min(s0 + split.unit_len(unit), unit < split.n_static ? split.static_end : total_slices);
  }
  const bool had_work = s0 < s1;
  int grp = 0;  // group of slice s0: the last g with s_prefix[g] <= s0 (groups without slices are skipped)
  if (s0 < s1) {
    int lo = 0, hi = n_groups - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (s_prefix[mid] <= s0) lo = mid; else hi = mid - 1;
    }
    grp = lo;
  }

  while (s0 < s1) {
    const int seg_end = min(s1, s_prefix[grp + 1]);
    const int spb = s_real[grp] >> 24;  // 16-token slices per block
    // slices relative to the group's list (the end of a padded group is clipped to the list's length)
    const int l0 = s0 - s_prefix[grp], l1 = min(seg_end - s_prefix[grp], s_real[grp] & 0xffffff);
    segment(grp, uni + (int64_t)grp * union_cap, l0, l1, spb, (l1 - 1) / spb + 1,
            min(unit + grp, slots_cap - 1),  // the clamp never binds (slots_cap >= units + groups)
            seg_end == s1 && split.n_claimed > 0);
    s0 = seg_end;
    do ++grp; while (grp < n_groups && s_prefix[grp + 1] <= s0);  // next group that has slices
  }

  // ---- next unit: claimed from the counter (every workgroup ends with a claim beyond the last unit) ----
  if (unit < split.n_static && unit + (int)gridDim.x < split.n_static) {  // latency regime: units beyond one per workgroup
    unit += gridDim.x;
    continue;
  }
  if (split.n_claimed == 0) break;
  if (tid == 0) s_claim = had_work ? claimed : atomicAdd(claim_counter, 1);
  __syncthreads();
  const int u = s_claim;
  __syncthreads();
  if (u >= split.n_claimed) break;
  unit = split.n_static + u;
  }
}

// One workgroup per (sequence, query head, 32 output channels).  The group's partials (slots unit + group
// of the units that overlap the group's part of the slice sequence) are spread over 32 rows of 8 threads,
// each thread owning 4 channels; a row folds its partials into a running (max, sum, accumulator) in slot
// order, and the rows are then fused in row order (fixed order => reproducible results).  A group with a
// long union list (a dense head) has thousands of partials: hence 32 of them in flight per step.
constexpr int kMergeCols = 32;
template <int kD>
__global__ __launch_bounds__(256) void merge_kernel(Params P, const int32_t* __restrict__ sched,
                                                    const float* __restrict__ acc_part,
                                                    const float* __restrict__ ml_part, float* __restrict__ out,
                                                    int slots_cap, int direct_w) {
  constexpr int kLanesC = kMergeCols / 4;  // threads per partial (4 channels each)
  constexpr int kRows = 256 / kLanesC;     // partials in flight per iteration
  __shared__ float s_o[kRows][kMergeCols + 1];
  __shared__ float s_m[kRows], s_l[kRows];
  const int b = blockIdx.y, h = blockIdx.x, c0 = blockIdx.z * kMergeCols, tid = threadIdx.x;
  const int G = P.group, j = h / G, r = h % G;
  const int grp = b * P.n_kv_heads + j;
  int p0 = 0, p1 = 0;
  if (direct_w > 0) {  // one partial per workgroup of the attention kernel, direct_w of them per group
    p0 = grp * direct_w;
    p1 = p0 + direct_w;
  } else if (const int first = sched[grp], last = sched[grp + 1]; last > first) {
    const int32_t* sp_raw = sched + P.batch * P.n_kv_heads + 1;
    Split split;
    split.unit_s = sp_raw[0];
    split.static_end = sp_raw[1];
    split.unit_d = sp_raw[2];
    split.n_static = sp_raw[3];
    p0 = min(split.unit_of(first) + grp, slots_cap);
    p1 = min(split.unit_of(last - 1) + grp + 1, slots_cap);
  }

  const int row = tid / kLanesC, cl = tid % kLanesC;
  float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
  float m_run = kNegBig, L = 0.f;
  // loads are unconditional (a segment in which this head took no part contributes exact zeros), so
  // the compiler can keep several iterations in flight
#pragma unroll 4
  for (int it = p0 + row; it < p1; it += kRows) {
    const float2 ml = *reinterpret_cast<const float2*>(ml_part + ((int64_t)it * G + r) * 2);
    const float4 a = *reinterpret_cast<const float4*>(acc_part + ((int64_t)it * G + r) * kD + c0 + cl * 4);
    const float m_new = fmaxf(m_run, ml.x);
    const float keep = __builtin_amdgcn_exp2f(m_run - m_new), w = __builtin_amdgcn_exp2f(ml.x - m_new);
    L = L * keep + ml.y * w;
    o.x = o.x * keep + a.x * w; o.y = o.y * keep + a.y * w; o.z = o.z * keep + a.z * w; o.w = o.w * keep + a.w * w;
    m_run = m_new;
  }
  s_o[row][cl * 4 + 0] = o.x; s_o[row][cl * 4 + 1] = o.y; s_o[row][cl * 4 + 2] = o.z; s_o[row][cl * 4 + 3] = o.w;
  if (cl == 0) {
    s_m[row] = m_run;
    s_l[row] = L;
  }
  __syncthreads();
  if (tid < kMergeCols) {
    float M = s_m[0];
#pragma unroll
    for (int i = 1; i < kRows; ++i) M = fmaxf(M, s_m[i]);
    float acc = 0.f, Lt = 0.f;
#pragma unroll
    for (int i = 0; i < kRows; ++i) {
      const float w = __builtin_amdgcn_exp2f(s_m[i] - M);
      acc += s_o[i][tid] * w;
      Lt += s_l[i] * w;
    }
    out[((int64_t)b * P.n_q_heads + h) * kD + c0 + tid] = Lt > 0.f ? acc / Lt : 0.f;
  }
}

// Which groups take the matrix-core form of the attention kernel (head_dim 128 only).  Its arithmetic per slice
// does not depend on the number of heads that want a block, so it wins clearly where many heads share blocks
// (7 heads on every block: 0.58 -> 0.81 of the HBM peak) and by 0-3% at 4 heads per group with one head per
// block; below 4 heads per group the vector form stays.
#ifndef FX_MFMA_MIN_GROUP
#define FX_MFMA_MIN_GROUP 4
#endif
template <int kD, int kG>
constexpr bool kUseMfma = kD == 128 && kG >= FX_MFMA_MIN_GROUP;

// Resident workgroups of attend_kernel<kD, kG> per compute unit on the current device (queried once per device).
template <int kD, int kG>
static int attend_wg_per_cu(size_t lds) {
  static std::atomic<int> cached[kMaxDevices];
  const int dev = current_device();
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attend_kernel<kD, kG, kUseMfma<kD, kG>>, 256, lds) != hipSuccess || n < 1) n = 1;
    n = n > 8 ? 8 : n;
    cached[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

static size_t attend_lds_bytes(const Params& P) { return (size_t)(2 * P.batch * P.n_kv_heads + 1) * sizeof(int); }

template <int kD, int kG>
static int attend_grid(const Params& P, int n_cu) {
  const int grid = n_cu * attend_wg_per_cu<kD, kG>(attend_lds_bytes(P));
  return grid > kMaxUnits ? kMaxUnits : grid;
}

// Direct mode of the decode stage, for small steps: the host can bound every group's slice count from k_max alone
// (union_cap entries of at most max_spb slices); if that bound leaves at most kDirectMaxSlices slices to each of
// the `w` workgroups a group can have, the plan kernel stores every group's list cut into w pieces at fixed
// places and the attention kernel needs neither the prefix over the groups nor the slice-sequence split: one
// dependent round trip less before the first K/V rows, and the merge kernel finds its partials without the
// split description.  w = 0: not used.
constexpr int kDirectMaxSlices = 32;
struct DirectMode {
  int w = 0, piece_cap = 0;
};
static DirectMode direct_mode(const Params& P, const DecodeWorkspace& W, int n_wg) {
  const int n_groups = P.batch * P.n_kv_heads;
  if (n_groups > n_wg) return {};
  int max_spb = 1;
  for (int j = 0; j < P.n_kv_heads; ++j) max_spb = max_spb > (P.gran[j] >> 4) ? max_spb : (P.gran[j] >> 4);
  const int64_t bound = (int64_t)W.union_cap * max_spb;  // slices a group can have at most
  int w = n_wg / n_groups;
  const int64_t enough = (bound + 3) / 4;                // pieces of at least 4 slices at the bound
  if (w > enough) w = (int)enough;
  if (w < 1) w = 1;
  const int piece_cap = (W.union_cap + w - 1) / w;
  if ((int64_t)piece_cap * max_spb > kDirectMaxSlices || piece_cap > kEntriesPerPiece) return {};
  return {w, piece_cap};
}

template <int kD, int kG>
static hipError_t launch_attend(const Params& P, const void* q, const void* K, const void* V, const uint32_t* uni,
                                const int32_t* ucount, const DecodeWorkspace& W, int32_t* sched, float* acc_part,
                                float* ml_part, int n_cu, DirectMode dm, hipStream_t stream) {
  const int grid = dm.w > 0 ? P.batch * P.n_kv_heads * dm.w : attend_grid<kD, kG>(P, n_cu);
  return launch(attend_kernel<kD, kG, kUseMfma<kD, kG>>, dim3(grid), dim3(256), attend_lds_bytes(P), stream, P,
                (const uint16_t*)q, (const uint16_t*)K, (const uint16_t*)V, uni, ucount, W.union_cap, sched, acc_part,
                ml_part, W.slots_cap, dm.w, dm.piece_cap);
}

template <int kD>
static hipError_t dispatch_group(const Params& P, const void* q, const void* K, const void* V, const uint32_t* uni,
                                 const int32_t* ucount, const DecodeWorkspace& W, int32_t* sched, float* acc_part,
                                 float* ml_part, int n_cu, DirectMode dm, hipStream_t stream) {
  switch (P.group) {
#define FX_CASE(G) \
  case G:          \
    return launch_attend<kD, G>(P, q, K, V, uni, ucount, W, sched, acc_part, ml_part, n_cu, dm, stream);
    FX_CASE(1) FX_CASE(2) FX_CASE(3) FX_CASE(4) FX_CASE(5) FX_CASE(6) FX_CASE(7) FX_CASE(8)
#undef FX_CASE
  }
  return hipErrorInvalidValue;
}

int attend_launch_size(const Params& P, int n_cu) {
  switch (P.group) {
#define FX_CASE(G) \
  case G:          \
    return P.head_dim == 128 ? attend_grid<128, G>(P, n_cu) : attend_grid<64, G>(P, n_cu);
    FX_CASE(1) FX_CASE(2) FX_CASE(3) FX_CASE(4) FX_CASE(5) FX_CASE(6) FX_CASE(7) FX_CASE(8)
#undef FX_CASE
  }
  return kMaxUnits;
}

hipError_t launch_decode(const Params& P, const void* q, const void* K, const void* V, const int32_t* idx,
                         const int32_t* cnt, float* out, void* workspace, int carve_units, int n_cu,
                         hipStream_t stream) {
  const DecodeWorkspace W = carve_decode(P, carve_units);
  char* ws = static_cast<char*>(workspace);
  uint32_t* uni = reinterpret_cast<uint32_t*>(ws + W.union_off);
  int32_t* ucount = reinterpret_cast<int32_t*>(ws + W.ucount_off);
  int32_t* sched = reinterpret_cast<int32_t*>(ws + W.sched_off);
  float* acc_part = reinterpret_cast<float*>(ws + W.acc_off);
  float* ml_part = reinterpret_cast<float*>(ws + W.ml_off);

  const size_t plan_lds = (size_t)((P.nb_stride + 3) / 4) * sizeof(uint32_t);
  const DirectMode dm = direct_mode(P, W, attend_launch_size(P, n_cu));
  hipError_t e;
  {
    ScopedSlot prof(kSlotPlan, stream);
    e = launch(plan_kernel, dim3(P.n_kv_heads, P.batch), dim3(kPlanThreads), plan_lds, stream, P, idx, cnt, uni, ucount,
               W.union_cap, sched + P.batch * P.n_kv_heads + 5, dm.w, dm.piece_cap);
  }
  if (e != hipSuccess) return e;
  {
    ScopedSlot prof(kSlotAttend, stream);
    e = P.head_dim == 128
            ? dispatch_group<128>(P, q, K, V, uni, ucount, W, sched, acc_part, ml_part, n_cu, dm, stream)
            : dispatch_group<64>(P, q, K, V, uni, ucount, W, sched, acc_part, ml_part, n_cu, dm, stream);
  }
  if (e != hipSuccess) return e;
  ScopedSlot prof(kSlotMerge, stream);
  if (P.head_dim == 128)
    return launch(merge_kernel<128>, dim3(P.n_q_heads, P.batch, 128 / kMergeCols), dim3(256), 0, stream, P,
                  (const int32_t*)sched, (const float*)acc_part, (const float*)ml_part, out, W.slots_cap, dm.w);
  return launch(merge_kernel<64>, dim3(P.n_q_heads, P.batch, 64 / kMergeCols), dim3(256), 0, stream, P,
                (const int32_t*)sched, (const float*)acc_part, (const float*)ml_part, out, W.slots_cap, dm.w);
}

}  // namespace fx
