// Block scoring and per-head top-k (Sec. 2.1 of the paper: the query is compared with the metadata
// of all key blocks and the top-k blocks are selected; Sec. 5.3: one block size per GQA group, one
// budget per head).
//
// The score of a block for a head is  s = sum_c max(q_c mn_c, q_c mx_c)
//                                       = sum_c (min(q_c,0) mn_c + max(q_c,0) mx_c),
// i.e. one row of a dense product  [q- | q+] (G x 2d)  times  [mn | mx]^T (2d x n_cand): the summary
// rows are stored exactly as [mn | mx], so the stream of summaries feeds the matrix cores directly.
//
// Stage 1 (score_grid_kernel / score_stream_kernel): per (sequence, KV head) stream the candidate summaries once; bf16 MFMA
//   (16x16x32, fp32 accumulate) gives, for all heads of the group at once, an approximate score
//   s~ and the magnitude sum a~ = sum_c (|q-_c| |mn_c| + |q+_c| |mx_c|) that bounds its rounding error.
// Stage 2 (topk_reg_kernel / topk_kernel): per (sequence, query head) a radix select on the fp32 keys finds the k-th
//   largest s~ = T.  With eps = gamma * max a~, every candidate above T + 2 eps is certainly among
//   the exact top-k and every candidate below T - 2 eps certainly is not.  Only the few candidates
//   inside the band are re-scored exactly (exact products, fp64 accumulation) and ranked by
//   (exact score descending, index ascending).  The result therefore equals the selection made on
//   fp64 scores (up to fp64 summation order, ~1e-16), while the bulk of the work runs at the speed
//   the summaries stream from HBM.  If the band holds more candidates than fit in LDS (masses of
//   identical blocks) the head falls back to exact scores for all candidates and a 64-bit radix select.
#include <atomic>

#include "fx_device.hpp"
#include "fx_kernels.hpp"

namespace fx {


// Bound on |s~ - s| / a~.  Products of bf16 pairs are exact in fp32; a chain of 2d <= 256 fp32
// accumulations is off by at most 256 * 2^-24 a~ = 2^-16 a~ with round-to-nearest adds and 2^-15 a~
// with truncating adds.  2^-14 leaves a factor of two over the worse case; the GPU tests check the
// measured error of every candidate against this bound.
constexpr float kGamma = 1.0f / 16384.0f;
constexpr int kAmbCap = 256;  // band candidates re-scored in LDS; more => fallback

__device__ __forceinline__ uint64_t ordered_key64(double s) {
  uint64_t u = (uint64_t)__double_as_longlong(s);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}
__device__ __forceinline__ uint32_t ordered_key32(float s) {
  uint32_t u = __float_as_uint(s);
  return (u >> 31) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key32_to_float(uint32_t k) {
  return __uint_as_float((k >> 31) ? (k & 0x7fffffffu) : ~k);
}

// ---------------------------------------------------------------------------------------------------
// Stage 1
// ---------------------------------------------------------------------------------------------------
// MFMA operand layout (v_mfma_f32_16x16x32_bf16): lane l supplies A[m = l % 16][k = 8 (l / 16) .. + 8]
// and B[k = 8 (l / 16) .. + 8][n = l % 16]; it receives D[m = 4 (l / 16) + i][n = l % 16], i = 0..3.
// Here n = candidate within a tile of 16, k = position in the [mn | mx] row, and A row
//   m = 4 (h % 4) + 2 (h / 4)     is [q- | q+] of head h of the group       (-> s~, from B)
//   m = 4 (h % 4) + 2 (h / 4) + 1 is [|q-| | |q+|] of head h                (-> a~, from |B|)
// so that result register 0 of the lanes 16 x .. 16 x + 15 is head x's score of the tile's 16 candidates
// (register 2: head x + 4; registers 1 and 3: the magnitude sums): one store instruction of the whole
// wave writes the scores of four heads, and one cross-lane reduction per register serves four heads.
// Small steps load the summaries straight into the B layout (each lane 16 bytes of its own row: 64-byte
// pieces of 16 rows per instruction, so two instructions share every 128-byte line).  The stream kernel
// instead loads a tile as 8 KiB of whole lines with non-temporal loads (1 KiB contiguous per instruction)
// and turns it into the B layout through a private, padded LDS region of the wave: 62 -> 53 us at 128K
// context, batch 16.  (The same staging with ordinary loads is twice slower than no staging; four neighbouring
// lanes per row followed by a wave-wide permutation made no difference.)
// The magnitude sums are reduced to one maximum per tile and head before they leave the kernel (the
// selection only needs their maximum per head).  The scores are stored tile-major,
// [sequence][KV head][tile][head of the group][16], so that a wave's stores for a tile form one
// contiguous run of G * 64 bytes (scattered 64-byte pieces cost ~10% of the kernel).

// LDS of one wave for the staged tile walk: 16 rows of 2 kD bf16, each padded by 16 bytes so that the 16 lanes
// that read the same piece of 16 different rows hit different banks.
template <int kD>
struct TileStage {
  static constexpr int kPieces = kD / 4;      // 16-byte pieces per [mn | mx] row
  static constexpr int kStride = kPieces + 1;  // row stride in pieces
  uint4 piece[16 * kStride];
};

// One wave scores tiles [tile_first, tile_end) of group (b, j): it requests the next tile's rows before it
// multiplies the current one.  `rows_base` points at the group's first candidate row.  With `stage` (the wave's
// own LDS region) the rows arrive as whole lines and pass through LDS; without, they are loaded in the B layout.
template <int kD, bool kStaged>
__device__ __forceinline__ void score_tiles(const Params& P, const uint16_t* __restrict__ q,
                                            const uint16_t* __restrict__ rows_base, int n_cand, int b, int j,
                                            int tile_first, int tile_end, float* __restrict__ approx,
                                            float* __restrict__ mag_tile, int mag_stride, int lane,
                                            TileStage<kD>* stage = nullptr) {
  constexpr int kRow = 2 * kD;       // elements of one [mn | mx] row
  constexpr int kSlabs = kRow / 32;  // MFMA k-steps per row = 1 KiB load instructions per tile
  constexpr int kPieces = TileStage<kD>::kPieces, kStride = TileStage<kD>::kStride;
  const int n = lane & 15, r = lane >> 4;
  uint4 cur[kSlabs], nxt[kSlabs];
  auto fetch = [&](int tile, uint4* dst) {
    if constexpr (kStaged) {
      // instruction i takes pieces 64 i .. 64 i + 63 of the tile: rows are contiguous, so 1 KiB of whole lines
#pragma unroll
      for (int i = 0; i < kSlabs; ++i) {
        const int f = i * 64 + lane;
        const int cand = min(tile * 16 + f / kPieces, n_cand - 1);  // clamped: stays inside the candidates
        dst[i] = stream_load16(rows_base + (int64_t)cand * kRow + (f % kPieces) * 8);
      }
    } else {
      const int cand = min(tile * 16 + n, n_cand - 1);  // clamped: stays inside the candidates
      const uint16_t* p = rows_base + r * 8 + (int64_t)cand * kRow;
#pragma unroll
      for (int s = 0; s < kSlabs; ++s) dst[s] = *reinterpret_cast<const uint4*>(p + 32 * s);
    }
  };
  fetch(tile_first, nxt);

  // A operand, built once per group from q with bit operations on the packed bf16 pairs:
  // q- keeps the negative elements, q+ the others; the magnitude rows drop the sign.
  uint4 a_op[kSlabs];
  {
    const int head = (n >> 2) + 4 * ((n >> 1) & 1);
    const bool want_abs = (n & 1) != 0;
    auto part = [&](uint32_t v, bool is_mx) -> uint32_t {
      const uint32_t neg = ((v >> 15) & 0x00010001u) * 0xffffu;  // 0xffff in every half whose sign bit is set
      const uint32_t kept = is_mx ? (v & ~neg) : (v & neg);
      return want_abs ? (kept & 0x7fff7fffu) : kept;
    };
#pragma unroll
    for (int s = 0; s < kSlabs; ++s) {
      const int e = 32 * s + 8 * r;  // first row element of this lane's k-chunk
      const int c = e % kD;
      const bool is_mx = e >= kD;
      uint4 raw = make_uint4(0u, 0u, 0u, 0u);
      if (head < P.group)
        raw = *reinterpret_cast<const uint4*>(q + ((int64_t)b * P.n_q_heads + j * P.group + head) * kD + c);
      a_op[s] = make_uint4(part(raw.x, is_mx), part(raw.y, is_mx), part(raw.z, is_mx), part(raw.w, is_mx));
    }
  }

  for (int tile = tile_first; tile < tile_end; ++tile) {
    if constexpr (kStaged) {
      // Only this wave touches its region, and a wave's LDS instructions execute in order: the fences keep the
      // compiler from moving the reads of other lanes' data above the writes (and the next tile's writes above
      // these reads); no barrier instruction is needed.
#pragma unroll
      for (int i = 0; i < kSlabs; ++i) {
        const int f = i * 64 + lane;
        stage->piece[(f / kPieces) * kStride + f % kPieces] = nxt[i];
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int s = 0; s < kSlabs; ++s) cur[s] = stage->piece[n * kStride + 4 * s + r];  // pieces 4 s + r of row n
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    } else {
#pragma unroll
      for (int s = 0; s < kSlabs; ++s) cur[s] = nxt[s];
    }
    if (tile + 1 < tile_end) fetch(tile + 1, nxt);
    f32x4_t d_s = {0.f, 0.f, 0.f, 0.f}, d_a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < kSlabs; ++s) {
      const uint4 v = cur[s];
      const uint4 va = make_uint4(v.x & 0x7fff7fffu, v.y & 0x7fff7fffu, v.z & 0x7fff7fffu, v.w & 0x7fff7fffu);
      d_s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a_op[s]),
                                                    __builtin_bit_cast(bf16x8_t, v), d_s, 0, 0, 0);
      d_a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a_op[s]),
                                                    __builtin_bit_cast(bf16x8_t, va), d_a, 0, 0, 0);
    }
    const int cand = tile * 16 + n;
#pragma unroll
    for (int half = 0; half < 2; ++half) {  // heads r and r + 4
      if (4 * half >= P.group) break;  // wave-uniform
      const int head = r + 4 * half;
      if (head < P.group && cand < n_cand)
        approx[((((int64_t)b * P.n_kv_heads + j) * mag_stride + tile) * P.group + head) * 16 + n] = d_s[2 * half];
      // maximum magnitude over the tile's 16 candidates (clamped duplicates repeat a real candidate)
      float m = d_a[2 * half + 1];
      m = fmaxf(m, dpp_f<kDppXor1>(m));
      m = fmaxf(m, dpp_f<kDppXor2>(m));
      m = fmaxf(m, dpp_f<kDppHalfMirror>(m));
      m = fmaxf(m, dpp_f<kDppMirror>(m));
      if (n == 0 && head < P.group) mag_tile[((int64_t)b * P.n_q_heads + j * P.group + head) * mag_stride + tile] = m;
    }
  }
}

// Does any head of group (b, j) select blocks at all?  A group of streaming heads (Sec. 3.2: budget 0)
// needs no scores and its summaries are never read.  Unrolled so that the loads go out together.
__device__ __forceinline__ bool group_selects(const Params& P, const float* __restrict__ budget_frac,
                                              const int32_t* __restrict__ budget_blocks, int b, int j) {
  bool any = false;
#pragma unroll
  for (int h = 0; h < kMaxGroup; ++h) {
    if (h < P.group) {
      const int64_t slot = (int64_t)b * P.n_q_heads + j * P.group + h;
      any |= budget_blocks ? budget_blocks[slot] > 0 : budget_frac[slot] > 0.f;
    }
  }
  return any;
}

// Small steps (at most one tile per wave slot of the chip): the grid enumerates (sequence, KV head, tile
// range) directly and a wave needs nothing but its own group's length, so its first loads go out at once.
template <int kD>
__global__ __launch_bounds__(256) void score_grid_kernel(Params P, const uint16_t* __restrict__ q,
                                                         const uint16_t* __restrict__ S, float* __restrict__ approx,
                                                         float* __restrict__ mag_tile,
                                                         const float* __restrict__ budget_frac,
                                                         const int32_t* __restrict__ budget_blocks, int mag_stride) {
  const int b = blockIdx.z, j = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // budgets, summary offset and sequence length are requested together (one round trip, not three)
  const bool any = group_selects(P, budget_frac, budget_blocks, b, j);
  const int64_t first_block = P.sum_base[(int64_t)b * P.n_kv_heads + j];
  const Geo geo = geometry(P, b, j);
  const int tile = blockIdx.x * 4 + wave;
  if (tile * 16 >= geo.n_cand || !any) return;  // whole wave leaves
  const uint16_t* rows = S + (first_block + geo.n_sink) * (int64_t)(2 * kD);
  score_tiles<kD, false>(P, q, rows, geo.n_cand, b, j, tile, tile + 1, approx, mag_tile, mag_stride, lane);
}

// Larger steps: the tiles of all groups that need scores form one global tile sequence (its prefix over
// the groups is computed by every workgroup from the sequence lengths and budgets); every wave of the
// launch walks an equal contiguous share of it and rebuilds its A operand where the share crosses into
// the next group.  Ragged batches, mixed block sizes and streaming groups therefore cost nothing in
// balance (a grid over the longest sequence leaves most workgroups of a short one without work).
// kStaged: whole-line loads through LDS (see above); the host falls back to the unstaged form where the group
// tables leave no room for the stage.
template <int kD, bool kStaged>
__global__ __launch_bounds__(256) void score_stream_kernel(Params P, const uint16_t* __restrict__ q,
                                                           const uint16_t* __restrict__ S, float* __restrict__ approx,
                                                           float* __restrict__ mag_tile,
                                                           const float* __restrict__ budget_frac,
                                                           const int32_t* __restrict__ budget_blocks, int mag_stride) {
  // per group, filled by the prologue so that a wave entering a group starts its first loads at once:
  extern __shared__ long long s_rowbase[];  // [n_groups] first candidate's row (in blocks) inside the summaries
  __shared__ int s_scan[4];
  __shared__ TileStage<kD> s_stage[kStaged ? 4 : 1];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_groups = P.batch * P.n_kv_heads;
  int* s_tiles = reinterpret_cast<int*>(s_rowbase + n_groups);  // [n_groups + 1] exclusive prefix of tiles
  uint16_t* s_ncand = reinterpret_cast<uint16_t*>(s_tiles + n_groups + 1);  // [n_groups] candidates (at most 2^15)
  {
    auto tiles_of = [&](int g) -> int {
      const int b = g / P.n_kv_heads, j = g - b * P.n_kv_heads;
      const bool any = group_selects(P, budget_frac, budget_blocks, b, j);
      const Geo geo = geometry(P, b, j);
      s_ncand[g] = (uint16_t)geo.n_cand;
      s_rowbase[g] = P.sum_base[g] + geo.n_sink;
      return any ? (geo.n_cand + 15) >> 4 : 0;
    };
    const int per = (n_groups + 255) / 256;
    const int g_lo = min(tid * per, n_groups), g_hi = min(g_lo + per, n_groups);
    int local = 0;
    for (int g = g_lo; g < g_hi; ++g) {
      const int c = tiles_of(g);
      s_tiles[g] = c;  // replaced by the prefix below (same thread)
      local += c;
    }
    const int incl = block_incl_scan(local, s_scan);
    int run = incl - local;
    for (int g = g_lo; g < g_hi; ++g) {
      const int c = s_tiles[g];
      s_tiles[g] = run;
      run += c;
    }
    if (tid == 255) s_tiles[n_groups] = incl;
  }
  __syncthreads();
  const int total_tiles = s_tiles[n_groups];
  const int n_waves = gridDim.x * 4;
  const int share = (total_tiles + n_waves - 1) / n_waves;
  int t = (blockIdx.x * 4 + wave) * share;
  const int t_end = min(t + share, total_tiles);
  if (t >= t_end) return;  // whole wave leaves

  int grp;  // group of tile t: the last g with s_tiles[g] <= t (groups without tiles are skipped)
  {
    int lo = 0, hi = n_groups - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (s_tiles[mid] <= t) lo = mid; else hi = mid - 1;
    }
    grp = lo;
  }
  while (t < t_end) {
    const int b = grp / P.n_kv_heads, j = grp - b * P.n_kv_heads;
    const int tile_first = t - s_tiles[grp];
    const int tile_end = min(t_end, s_tiles[grp + 1]) - s_tiles[grp];
    score_tiles<kD, kStaged>(P, q, S + s_rowbase[grp] * (int64_t)(2 * kD), s_ncand[grp], b, j, tile_first, tile_end,
                             approx, mag_tile, mag_stride, lane, &s_stage[kStaged ? wave : 0]);
    t = s_tiles[grp] + tile_end;
    do ++grp; while (grp < n_groups && s_tiles[grp + 1] <= t);  // next group that has tiles
  }
}

// ---------------------------------------------------------------------------------------------------
// Stage 2
// ---------------------------------------------------------------------------------------------------

// Exact score of one candidate for one head, computed by a whole wave: exact products, fp64 sums.
// Every lane returns the same value.
template <int kD>
__device__ __forceinline__ double exact_score_wave(const uint16_t* __restrict__ q_h, const uint16_t* __restrict__ row,
                                                   int lane) {
  constexpr int kPer = kD / 64;  // channels per lane (1 or 2)
  double acc = 0.0;
#pragma unroll
  for (int t = 0; t < kPer; ++t) {
    const int c = lane * kPer + t;
    const double qc = (double)__uint_as_float((uint32_t)q_h[c] << 16);
    const double mn = (double)__uint_as_float((uint32_t)row[c] << 16);
    const double mx = (double)__uint_as_float((uint32_t)row[kD + c] << 16);
    acc = fma(fmax(qc, 0.0), mx, fma(fmin(qc, 0.0), mn, acc));
  }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) acc += __shfl_xor(acc, off, kWave);
  return acc;
}

// Most-significant-digit-first radix select over `n` keys read through `load(r)`: returns the k-th
// largest key and how many of the keys equal to it belong to the top k.  Any multiple of 256 threads; `hist`
// is 256 ints of LDS, `scan_scratch` one int per wave, `s_pair` 2 ints.
template <typename KeyT, int kT, typename Load>
__device__ __forceinline__ void radix_select(Load load, int n, int k, int* hist, int* scan_scratch, int* s_pair,
                                             KeyT& kth_out, int& krem_out) {
  constexpr int kPasses = sizeof(KeyT);
  const int tid = threadIdx.x;
  KeyT prefix = 0;
  int krem = k;
  for (int pass = kPasses - 1; pass >= 0; --pass) {
    const int shift = pass * 8;
    const KeyT hi_mask = pass == kPasses - 1 ? (KeyT)0 : (KeyT)(~(KeyT)0 << (shift + 8));
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int base = 0; base < n; base += kT) {
      const int r = base + tid;
      bool match = false;
      unsigned digit = 0;
      if (r < n) {
        const KeyT key = load(r);
        match = (key & hi_mask) == prefix;
        digit = (unsigned)(key >> shift) & 255u;
      }
      // one LDS atomic per wave when all matching lanes agree on the digit (usual for the sign and
      // exponent digits), else one per lane
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
    const int dg = 255 - tid;  // thread t < 256 owns digit 255 - t: a prefix sum over threads is a suffix sum over digits
    const int c = tid < 256 ? hist[dg] : 0;
    const int incl = block_incl_scan<kT / 64>(c, scan_scratch);
    const int excl = incl - c;
    if (tid < 256 && excl < krem && krem <= incl) {
      s_pair[0] = dg;
      s_pair[1] = krem - excl;
    }
    __syncthreads();
    prefix |= (KeyT)s_pair[0] << shift;
    krem = s_pair[1];
    __syncthreads();
  }
  kth_out = prefix;
  krem_out = krem;
}

// LDS of one top-k workgroup.
struct TopkShared {
  int hist[256];
  int scan[kMaxWaves];
  int count_a[kMaxWaves];
  int count_b[kMaxWaves];
  int pair[2];
  int total;
  float wmax[kMaxWaves];
  uint32_t kmin[kMaxWaves], kmax[kMaxWaves];
  int amb_idx[kAmbCap];         // band candidates, ascending
  uint64_t amb_key[kAmbCap];    // their exact keys
  unsigned char amb_chosen[kAmbCap];
};

// out[from .. to) = -1 (the padding behind a head's index list), 16 bytes per store where alignment allows.
template <int kT>
__device__ __forceinline__ void pad_minus_one(int32_t* out, int from, int to) {
  const int tid = threadIdx.x;
  const int shift = (int)((reinterpret_cast<uintptr_t>(out) >> 2) & 3);  // elements past a 16-byte boundary
  int lo = ((from + shift + 3) & ~3) - shift;                            // first index whose address is aligned
  lo = lo < to ? lo : to;
  const int n_vec = (to - lo) >> 2;
  for (int r = from + tid; r < lo; r += kT) out[r] = -1;
  int4* v = reinterpret_cast<int4*>(out + lo);
  for (int x = tid; x < n_vec; x += kT) v[x] = make_int4(-1, -1, -1, -1);
  for (int r = lo + 4 * n_vec + tid; r < to; r += kT) out[r] = -1;
}

// Everything the top-k of one (sequence, query head) needs.
struct HeadTask {
  int k, n, n_sink;           // blocks to keep, candidates, index of the first candidate block
  int32_t* out;               // idx row of this head
  const float* ap_base;       // approximate scores: candidate r at ap_base[(r / 16) * tile_step + r % 16]
  int tile_step;
  const float* mag;           // one magnitude maximum per tile of 16 candidates
  const uint16_t* q_h;        // the head's query
  const uint16_t* rows;       // [mn | mx] row of candidate 0
  uint64_t* keys64;           // exact keys of the fallback path, candidate 0 first
};

struct TopkArgs {
  const uint16_t* q;
  const uint16_t* S;
  const float* approx;
  const float* mag;
  uint64_t* keys64;
  const float* budget_frac;
  const int32_t* budget_blocks;
  int32_t* idx;
  int32_t* cnt;
  int mag_stride;
};

// Fills the task of head blockIdx.x of sequence blockIdx.y, writes cnt, and finishes the two trivial
// cases (nothing kept / everything kept) on the spot.  Returns false when the head is done.
template <int kD, int kT>
__device__ __forceinline__ bool begin_head(const Params& P, const TopkArgs& A, HeadTask& t) {
  const int b = blockIdx.y, h = blockIdx.x, j = h / P.group, tid = threadIdx.x;
  const Geo geo = geometry(P, b, j);
  const int64_t slot = (int64_t)b * P.n_q_heads + h;
  double want;
  if (A.budget_blocks)
    want = (double)A.budget_blocks[slot];
  else
    want = ceil((double)A.budget_frac[slot] * (double)geo.n_cand);
  const int limit = geo.n_cand < P.k_max ? geo.n_cand : P.k_max;
  t.k = want > 0.0 ? (want < (double)limit ? (int)want : limit) : 0;  // NaN falls to 0
  t.n = geo.n_cand;
  t.n_sink = geo.n_sink;
  t.out = A.idx + slot * P.k_max;
  t.ap_base = A.approx + (((int64_t)b * P.n_kv_heads + j) * A.mag_stride * P.group + (h - j * P.group)) * 16;
  t.tile_step = P.group * 16;
  t.mag = A.mag + slot * A.mag_stride;
  t.q_h = A.q + slot * kD;
  t.rows = A.S + (P.sum_base[(int64_t)b * P.n_kv_heads + j] + geo.n_sink) * (int64_t)(2 * kD);
  t.keys64 = A.keys64 + slot * P.nb_stride + geo.n_sink;
  if (tid == 0) A.cnt[slot] = t.k;
  if (t.k == 0 || t.k == t.n) {
    for (int r = tid; r < P.k_max; r += kT) t.out[r] = r < t.k ? t.n_sink + r : -1;
    return false;
  }
  return true;
}

// 2 * gamma * (largest magnitude sum of the head): half-width of the band around the k-th approximate score.
// `amax` is this thread's partial maximum over the head's tile magnitudes.
__device__ __forceinline__ float band_width_from_max(float amax) { return 2.0f * kGamma * amax * 1.001f + 1e-30f; }

template <int kT>
__device__ __forceinline__ float band_half_width(float amax, TopkShared& sh) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) amax = fmaxf(amax, __shfl_xor(amax, off, kWave));
  __syncthreads();
  if ((tid & 63) == 0) sh.wmax[tid >> 6] = amax;
  __syncthreads();
  amax = sh.wmax[0];
#pragma unroll
  for (int w = 1; w < kT / 64; ++w) amax = fmaxf(amax, sh.wmax[w]);
  return band_width_from_max(amax);
}

// Exact path for a head whose band holds more candidates than LDS takes: exact fp64 scores for every
// candidate, 64-bit radix select, ordered compaction (ties: lowest indices).
template <int kD, int kT>
__device__ __forceinline__ void exact_fallback(const Params& P, const HeadTask& t, TopkShared& sh) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int n_waves = kT / 64;
  for (int r = wave; r < t.n; r += n_waves) {
    const double s = exact_score_wave<kD>(t.q_h, t.rows + (int64_t)r * 2 * kD, lane);
    if (lane == 0) t.keys64[r] = ordered_key64(s);
  }
  __threadfence_block();
  __syncthreads();
  uint64_t kth;
  int krem;
  radix_select<uint64_t, kT>([&](int r) { return t.keys64[r]; }, t.n, t.k, sh.hist, sh.scan, sh.pair, kth, krem);
  int run_sel = 0, run_eq = 0;
  for (int base = 0; base < t.n; base += kT) {
    const int r = base + tid;
    const uint64_t key = r < t.n ? t.keys64[r] : 0ull;
    const bool gt = r < t.n && key > kth;
    const bool eq = r < t.n && key == kth;
    int tot_eq, tot_sel;
    const int eq_before = run_eq + block_excl_count<n_waves>(eq, sh.count_a, tot_eq);
    const bool sel = gt || (eq && eq_before < krem);
    const int pos = run_sel + block_excl_count<n_waves>(sel, sh.count_b, tot_sel);
    if (sel && pos < P.k_max) t.out[pos] = t.n_sink + r;
    run_eq += tot_eq;
    run_sel += tot_sel;
  }
  pad_minus_one<kT>(t.out, t.k, P.k_max);
}

// Band candidates sh.amb_idx[0 .. n_amb) (ascending) -> sh.amb_chosen: the `need` best by (exact score
// descending, index ascending).
template <int kD, int kT>
__device__ __forceinline__ void resolve_band(const HeadTask& t, TopkShared& sh, int n_amb, int need) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  __syncthreads();  // amb_idx is complete
  for (int a = wave; a < n_amb; a += kT / 64) {
    const double s = exact_score_wave<kD>(t.q_h, t.rows + (int64_t)sh.amb_idx[a] * 2 * kD, lane);
    if (lane == 0) sh.amb_key[a] = ordered_key64(s);
  }
  __syncthreads();
  if (tid < n_amb) {
    const uint64_t mine = sh.amb_key[tid];
    int rank = 0;
    for (int a = 0; a < n_amb; ++a) {
      const uint64_t other = sh.amb_key[a];
      rank += (other > mine) || (other == mine && a < tid);
    }
    sh.amb_chosen[tid] = rank < need;
  }
  __syncthreads();
}

// Generic variant: any number of candidates, keys re-read from the workspace in every pass.
template <int kD>
__global__ __launch_bounds__(256) void topk_kernel(Params P, TopkArgs A) {
  __shared__ TopkShared sh;
  HeadTask t;
  if (!begin_head<kD, 256>(P, A, t)) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  auto ap = [&](int r) { return t.ap_base[(int64_t)(r >> 4) * t.tile_step + (r & 15)]; };
  float amax = 0.f;
  for (int r = tid; r < (t.n + 15) >> 4; r += 256) amax = fmaxf(amax, t.mag[r]);
  const float eps2 = band_half_width<256>(amax, sh);

  uint32_t kth32;
  int krem32;
  radix_select<uint32_t, 256>([&](int r) { return ordered_key32(ap(r)); }, t.n, t.k, sh.hist, sh.scan, sh.pair, kth32,
                         krem32);
  const float T = key32_to_float(kth32);
  const float hi = T + eps2, lo = T - eps2;

  // classify: certainly kept (above the band) / ambiguous (inside the band)
  int c_sure = 0, c_amb = 0;
  for (int r = tid; r < t.n; r += 256) {
    const float s = ap(r);
    c_sure += s > hi;
    c_amb += (s <= hi) && (s >= lo);
  }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    c_sure += __shfl_xor(c_sure, off, kWave);
    c_amb += __shfl_xor(c_amb, off, kWave);
  }
  __syncthreads();
  if (lane == 0) {
    sh.count_a[wave] = c_sure;
    sh.count_b[wave] = c_amb;
  }
  __syncthreads();
  const int n_sure = sh.count_a[0] + sh.count_a[1] + sh.count_a[2] + sh.count_a[3];
  const int n_amb = sh.count_b[0] + sh.count_b[1] + sh.count_b[2] + sh.count_b[3];
  const int need = t.k - n_sure;  // 1 <= need <= n_amb by construction of the band around the k-th key

  if (need < n_amb && n_amb > kAmbCap) {
    exact_fallback<kD, 256>(P, t, sh);
    return;
  }
  const bool resolve = need < n_amb;  // otherwise every band candidate is kept and no exact score is needed
  if (resolve) {
    int run = 0;
    for (int base = 0; base < t.n; base += 256) {
      const int r = base + tid;
      const float s = r < t.n ? ap(r) : 0.f;
      const bool amb = r < t.n && s <= hi && s >= lo;
      int tot;
      const int pos = run + block_excl_count(amb, sh.count_a, tot);
      if (amb) sh.amb_idx[pos] = r;
      run += tot;
    }
    resolve_band<kD, 256>(t, sh, n_amb, need);
  }

  // ordered compaction of the kept candidates
  int run_sel = 0, run_amb = 0;
  for (int base = 0; base < t.n; base += 256) {
    const int r = base + tid;
    const float s = r < t.n ? ap(r) : 0.f;
    const bool sure = r < t.n && s > hi;
    const bool amb = r < t.n && s <= hi && s >= lo;
    int tot_amb, tot_sel;
    const int a = run_amb + block_excl_count(amb, sh.count_a, tot_amb);
    const bool sel = sure || (amb && (!resolve || sh.amb_chosen[a]));
    const int pos = run_sel + block_excl_count(sel, sh.count_b, tot_sel);
    if (sel && pos < P.k_max) t.out[pos] = t.n_sink + r;
    run_amb += tot_amb;
    run_sel += tot_sel;
  }
  pad_minus_one<256>(t.out, t.k, P.k_max);
}

// Register-resident variant for n_cand <= kT * KPT (kT threads): thread t owns the KPT consecutive candidates
// t * KPT .. so that index order is thread order and every ordered compaction costs one block scan.
// Keys are reduced to (key - smallest key) before the radix passes, which removes the sign/exponent
// digits all candidates share: the select takes ceil(log2(span) / 8) passes, usually 3.
template <int kD, int KPT, int kT>
__global__ __launch_bounds__(kT) void topk_reg_kernel(Params P, TopkArgs A) {
  constexpr int kW = kT / 64;                 // waves
  constexpr int kMagPer = (512 + kT - 1) / kT;  // tile magnitudes per thread (at most 512 tiles)
  __shared__ TopkShared sh;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r0 = tid * KPT;
  // The approximate scores and tile magnitudes of this thread are requested first: their addresses do not
  // depend on the sequence length, so they travel together with the loads the geometry waits for instead
  // of after them.  Slots past the last candidate hold stale data and are masked below.
  float4 raw[KPT / 4];
  float mag_raw[kMagPer];
  {
    const int h = blockIdx.x, j = h / P.group;
    const float* ap_base =
        A.approx + (((int64_t)blockIdx.y * P.n_kv_heads + j) * A.mag_stride * P.group + (h - j * P.group)) * 16;
#pragma unroll
    for (int i4 = 0; i4 < KPT; i4 += 4) {  // KPT and r0 are multiples of 4: four candidates never straddle a tile
      const int r = r0 + i4;
      raw[i4 / 4] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (r < A.mag_stride * 16)
        raw[i4 / 4] = *reinterpret_cast<const float4*>(ap_base + (int64_t)(r >> 4) * (P.group * 16) + (r & 15));
    }
    const float* mg = A.mag + ((int64_t)blockIdx.y * P.n_q_heads + h) * A.mag_stride;
#pragma unroll
    for (int u = 0; u < kMagPer; ++u) mag_raw[u] = tid + u * kT < A.mag_stride ? mg[tid + u * kT] : 0.f;
  }
  HeadTask t;
  if (!begin_head<kD, kT>(P, A, t)) return;
  float amax = 0.f;
#pragma unroll
  for (int u = 0; u < kMagPer; ++u)
    if (tid + u * kT < (t.n + 15) >> 4) amax = fmaxf(amax, mag_raw[u]);
  // keys of this thread's candidates (0 = no candidate: below every real key) and the key range; the
  // largest magnitude, the smallest and the largest key are reduced together behind one barrier
  uint32_t key[KPT];
  uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
  for (int i4 = 0; i4 < KPT; i4 += 4) {
    const float f[4] = {raw[i4 / 4].x, raw[i4 / 4].y, raw[i4 / 4].z, raw[i4 / 4].w};
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      key[i4 + u] = 0u;
      if (r0 + i4 + u < t.n) {
        key[i4 + u] = ordered_key32(f[u]);
        kmin = min(kmin, key[i4 + u]);
        kmax = max(kmax, key[i4 + u]);
      }
    }
  }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, off, kWave));
    kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, off, kWave));
    amax = fmaxf(amax, __shfl_xor(amax, off, kWave));
  }
  if (lane == 0) {
    sh.kmin[wave] = kmin;
    sh.kmax[wave] = kmax;
    sh.wmax[wave] = amax;
  }
  if (tid < 256) sh.hist[tid] = 0;  // for the first radix pass
  __syncthreads();
  kmin = sh.kmin[0];
  kmax = sh.kmax[0];
  amax = sh.wmax[0];
#pragma unroll
  for (int w = 1; w < kW; ++w) {
    kmin = min(kmin, sh.kmin[w]);
    kmax = max(kmax, sh.kmax[w]);
    amax = fmaxf(amax, sh.wmax[w]);
  }
  const float eps2 = band_width_from_max(amax);

  // radix select of the k-th largest key on u = key - kmin, most significant digit first
  const uint32_t span = kmax - kmin;
  const int n_bits = span ? 32 - __clz((int)span) : 0;
  uint32_t prefix = 0;
  int krem = t.k;
  for (int pass = (n_bits + 7) / 8 - 1; pass >= 0; --pass) {
    const int shift = pass * 8;
    const uint32_t hi_mask = shift + 8 >= 32 ? 0u : (~0u << (shift + 8));
    // four barriers per pass: the histogram is empty on entry (its owner clears each bin right after reading
    // it), and `pair` is not rewritten before three barriers of the next pass have passed
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
      const uint32_t u = key[i] - kmin;
      if (key[i] != 0u && (u & hi_mask) == prefix) atomicAdd(&sh.hist[(u >> shift) & 255u], 1);
    }
    __syncthreads();
    const int dg = 255 - tid;  // threads 0..255 own one digit each
    int c = 0;
    if (tid < 256) {
      c = sh.hist[dg];
      sh.hist[dg] = 0;
    }
    const int incl = block_incl_scan<kW>(c, sh.scan);
    const int excl = incl - c;
    if (tid < 256 && excl < krem && krem <= incl) {
      sh.pair[0] = dg;
      sh.pair[1] = krem - excl;
    }
    __syncthreads();
    prefix |= (uint32_t)sh.pair[0] << shift;
    krem = sh.pair[1];
  }
  const float T = key32_to_float(kmin + prefix);
  const uint32_t hi_key = ordered_key32(T + eps2), lo_key = ordered_key32(T - eps2);

  // classify this thread's candidates: certainly kept / inside the band
  int c_sure = 0, c_amb = 0;
#pragma unroll
  for (int i = 0; i < KPT; ++i) {
    c_sure += key[i] > hi_key;
    c_amb += key[i] >= lo_key && key[i] <= hi_key;
  }
  // both counts in one scan: low half = certainly kept, high half = band (each at most 8192: no carry)
  const int packed_incl = block_incl_scan<kW>(c_sure | (c_amb << 16), sh.scan);
  if (tid == kT - 1) sh.total = packed_incl;
  __syncthreads();
  const int n_sure = sh.total & 0xffff, n_amb = sh.total >> 16;
  const int amb_base = (packed_incl >> 16) - c_amb;
  const int need = t.k - n_sure;  // 1 <= need <= n_amb by construction of the band around the k-th key

  if (need < n_amb && n_amb > kAmbCap) {
    exact_fallback<kD, kT>(P, t, sh);
    return;
  }
  const bool resolve = need < n_amb;  // otherwise every band candidate is kept and no exact score is needed
  if (resolve) {
    int a = amb_base;
#pragma unroll
    for (int i = 0; i < KPT; ++i)
      if (key[i] >= lo_key && key[i] <= hi_key) sh.amb_idx[a++] = r0 + i;
    resolve_band<kD, kT>(t, sh, n_amb, need);
  }

  // ordered compaction of the kept candidates
  int c_sel = 0;
  uint32_t sel_bits = 0;
  {
    int a = amb_base;
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
      bool sel = key[i] > hi_key;
      if (key[i] >= lo_key && key[i] <= hi_key) {
        sel = !resolve || sh.amb_chosen[a];
        ++a;
      }
      sel_bits |= (uint32_t)sel << i;
      c_sel += sel;
    }
  }
  int pos = block_incl_scan<kW>(c_sel, sh.scan) - c_sel;
#pragma unroll
  for (int i = 0; i < KPT; ++i)
    if ((sel_bits >> i) & 1u) {
      if (pos < P.k_max) t.out[pos] = t.n_sink + r0 + i;
      ++pos;
    }
  pad_minus_one<kT>(t.out, t.k, P.k_max);
}

float select_error_gamma() { return kGamma; }

// Resident workgroups of the stream score kernel per CU on the current device, queried once per device.
template <int kD, bool kStaged>
static int score_wg_per_cu(size_t lds) {
  static std::atomic<int> cached[kMaxDevices];
  const int dev = current_device();
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    const hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, score_stream_kernel<kD, kStaged>, 256, lds);
    if (e != hipSuccess || n < 1) n = 1;
    n = n > 8 ? 8 : n;
    cached[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

// Launches the score stage: the grid kernel for small steps, else the stream kernel.
template <int kD, bool kStaged>
static hipError_t launch_score(const Params& P, const uint16_t* q, const uint16_t* S, float* approx, float* mag,
                         const float* budget_frac, const int32_t* budget_blocks, int mag_stride, size_t lds, int n_cu,
                         hipStream_t stream) {
  const int64_t max_tiles = (int64_t)P.batch * P.n_kv_heads * mag_stride;
  const int64_t slots = (int64_t)n_cu * score_wg_per_cu<kD, kStaged>(lds);  // resident workgroups of the chip
  if (max_tiles <= 4 * slots) {  // at most one tile per wave slot
    const dim3 grid((mag_stride + 3) / 4, P.n_kv_heads, P.batch);
    return launch(score_grid_kernel<kD>, grid, dim3(256), 0, stream, P, q, S, approx, mag, budget_frac, budget_blocks,
                  mag_stride);
  }
  return launch(score_stream_kernel<kD, kStaged>, dim3((unsigned)slots), dim3(256), lds, stream, P, q, S, approx, mag,
                budget_frac, budget_blocks, mag_stride);
}

hipError_t launch_select(const Params& P, const void* q, const void* S, const float* budget_frac,
                         const int32_t* budget_blocks, int32_t* idx, int32_t* cnt, void* workspace, int n_cu,
                         hipStream_t stream) {
  const SelectWorkspace W = carve_select(P);
  char* ws = static_cast<char*>(workspace);
  float* approx = reinterpret_cast<float*>(ws + W.approx_off);
  float* mag = reinterpret_cast<float*>(ws + W.mag_off);
  uint64_t* keys = reinterpret_cast<uint64_t*>(ws + W.keys_off);
  const int mag_stride = W.mag_stride;
  hipError_t e;
  {
    ScopedSlot prof(kSlotScore, stream);
    // Group tables of the stream kernel: 14 bytes per group, 56 KiB at the largest supported batch * n_kv_heads
    // (4096).  A workgroup may use 64 KiB: the four waves' tile stages (33 KiB at d = 128, 17 KiB at d = 64) are
    // used where they fit beside the tables (up to about 2200 / 3400 groups) and a wave has a stream to speak of
    // (4 tiles or more; with fewer the extra LDS pass is pure latency: +0.6 us on the Qwen-shaped ragged batch).
    const size_t lds = (size_t)P.batch * P.n_kv_heads * (sizeof(long long) + sizeof(int) + sizeof(uint16_t)) + sizeof(int);
    const size_t stage = 4 * (P.head_dim == 128 ? sizeof(TileStage<128>) : sizeof(TileStage<64>));
    const int64_t waves = (int64_t)n_cu * 4 * (P.head_dim == 128 ? score_wg_per_cu<128, true>(lds) : score_wg_per_cu<64, true>(lds));
    const bool staged = lds + stage + 64 <= 65536 && (int64_t)P.batch * P.n_kv_heads * mag_stride >= 4 * waves;
    const uint16_t* q16 = (const uint16_t*)q;
    const uint16_t* S16 = (const uint16_t*)S;
    if (P.head_dim == 128) {
      if (staged) e = launch_score<128, true>(P, q16, S16, approx, mag, budget_frac, budget_blocks, mag_stride, lds, n_cu, stream);
      else e = launch_score<128, false>(P, q16, S16, approx, mag, budget_frac, budget_blocks, mag_stride, lds, n_cu, stream);
    } else {
      if (staged) e = launch_score<64, true>(P, q16, S16, approx, mag, budget_frac, budget_blocks, mag_stride, lds, n_cu, stream);
      else e = launch_score<64, false>(P, q16, S16, approx, mag, budget_frac, budget_blocks, mag_stride, lds, n_cu, stream);
    }
  }
  if (e != hipSuccess) return e;
  ScopedSlot prof(kSlotTopk, stream);
  const dim3 tgrid(P.n_q_heads, P.batch);
  const TopkArgs A{(const uint16_t*)q, (const uint16_t*)S, approx, mag, keys, budget_frac, budget_blocks, idx, cnt,
                   mag_stride};
  // keys per thread x threads per head: 4 x 256 for up to 1024 blocks, then wider workgroups before longer
  // per-thread key lists (every phase of the kernel is a chain of barriers and per-thread loops over the keys)
#ifndef FX_TOPK_T2
#define FX_TOPK_T2 256   // threads up to 2048 blocks (512 measured no better)
#endif
#ifndef FX_TOPK_T4
#define FX_TOPK_T4 512   // threads up to 4096 blocks (256: +1.4 us, 1024: +9 us at 512 heads)
#endif
#ifndef FX_TOPK_T8
#define FX_TOPK_T8 1024  // threads up to 8192 blocks (256: +4.5 us, 512: +0.6 us)
#endif
#define FX_TOPK_REG(D, KPT, T) e = launch(topk_reg_kernel<D, KPT, T>, tgrid, dim3(T), 0, stream, P, A)
  if (P.head_dim == 128) {
    if (P.nb_stride <= 1024) FX_TOPK_REG(128, 4, 256);
    else if (P.nb_stride <= 2048) FX_TOPK_REG(128, 2048 / FX_TOPK_T2, FX_TOPK_T2);
    else if (P.nb_stride <= 4096) FX_TOPK_REG(128, 4096 / FX_TOPK_T4, FX_TOPK_T4);
    else if (P.nb_stride <= 8192) FX_TOPK_REG(128, 8192 / FX_TOPK_T8, FX_TOPK_T8);
    else e = launch(topk_kernel<128>, tgrid, dim3(256), 0, stream, P, A);
  } else {
    if (P.nb_stride <= 1024) FX_TOPK_REG(64, 4, 256);
    else if (P.nb_stride <= 2048) FX_TOPK_REG(64, 2048 / FX_TOPK_T2, FX_TOPK_T2);
    else if (P.nb_stride <= 4096) FX_TOPK_REG(64, 4096 / FX_TOPK_T4, FX_TOPK_T4);
    else if (P.nb_stride <= 8192) FX_TOPK_REG(64, 8192 / FX_TOPK_T8, FX_TOPK_T8);
    else e = launch(topk_kernel<64>, tgrid, dim3(256), 0, stream, P, A);
  }
#undef FX_TOPK_REG
  return e;
}

}  // namespace fx
