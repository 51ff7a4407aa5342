// Host-side launch entry points of the kernel files and the carving of the caller's workspace.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <tuple>
#include <type_traits>
#include <utility>

#include "fx_device.hpp"

namespace fx {

constexpr size_t kAlign = 256;

// Per-device caches (occupancy, compute units) are indexed by the current device ordinal.
constexpr int kMaxDevices = 64;
inline int current_device() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) dev = 0;
  return dev;
}
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Kernel launch that returns this launch's own status (the return value of hipLaunchKernel) and leaves the
// runtime's sticky "last error" alone: an error the caller has not yet looked at is neither cleared nor taken
// for one of ours.  Arguments are converted to the kernel's parameter types before their addresses are taken.
template <typename Tuple, size_t... I>
inline void arg_pointers(Tuple& vals, void** ptrs, std::index_sequence<I...>) {
  ((ptrs[I] = static_cast<void*>(&std::get<I>(vals))), ...);
}
template <typename... KArgs, typename... Args>
inline hipError_t launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t stream,
                         Args&&... args) {
  static_assert(sizeof...(KArgs) == sizeof...(Args), "argument count differs from the kernel's parameter count");
  std::tuple<std::decay_t<KArgs>...> vals{static_cast<std::decay_t<KArgs>>(std::forward<Args>(args))...};
  void* ptrs[sizeof...(KArgs) > 0 ? sizeof...(KArgs) : 1];
  arg_pointers(vals, ptrs, std::index_sequence_for<KArgs...>{});
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds, stream);
}

// fx_select scratch: the approximate scores (fp32, tile-major [sequence][KV head][tile][head of group][16]),
// per (sequence, query head, tile of 16 candidates) the largest magnitude sum (fp32), and for the exact
// fallback path one order-preserving 64-bit key per (sequence, query head, block).
struct SelectWorkspace {
  size_t approx_off, mag_off, keys_off, total;
  int32_t mag_stride;  // tiles per (sequence, query head) row of the magnitude array
};
inline SelectWorkspace carve_select(const Params& P) {
  SelectWorkspace W;
  const size_t n = (size_t)P.batch * P.n_q_heads * P.nb_stride;
  W.mag_stride = (P.nb_stride + 15) / 16;
  size_t off = 0;
  W.approx_off = off; off += align_up((size_t)P.batch * P.n_q_heads * W.mag_stride * 16 * sizeof(float));
  W.mag_off = off;    off += align_up((size_t)P.batch * P.n_q_heads * W.mag_stride * sizeof(float));
  W.keys_off = off;   off += align_up(n * sizeof(uint64_t));
  W.total = off;
  return W;
}

// Work split of the decode stage.  The union lists of all groups, cut into 16-token slices, form one
// sequence that is divided into units: one static unit per workgroup of the launch (at most kMaxUnits)
// followed by up to kClaimedPerWg smaller units per workgroup that are claimed from a counter.  A unit
// that spans several groups writes one partial result per group it touches, to slot unit + group.
constexpr int kMaxUnits = 2048;
#ifndef FX_CLAIMED_PER_WG
#define FX_CLAIMED_PER_WG 8
#endif
constexpr int kClaimedPerWg = FX_CLAIMED_PER_WG;
constexpr int kMaxGroups = 4096;
constexpr int kEntriesPerPiece = 256;  // union entries staged in LDS at a time

// fx_sparse_decode scratch.
struct DecodeWorkspace {
  int32_t union_cap;  // entries per group in the union list
  int32_t slots_cap;  // partial-result slots: units + groups
  size_t union_off;   // uint32 [n_groups][union_cap]   (block << 8) | head mask, ascending by block
                      // (direct mode: [n_groups][w][piece_cap], the same entries cut into w pieces per group)
  size_t ucount_off;  // int32  [n_groups]              entries per group
  size_t sched_off;   // int32  [n_groups + 8]          exclusive slice prefix, total, the split (4 values), claim counter
  size_t acc_off;     // float  [slots_cap][group][d]   un-normalised partial outputs
  size_t ml_off;      // float  [slots_cap][group][2]   partial running maximum (log2 domain) and sum
  size_t total;
};
// `max_units`: upper bound of the attention kernel's launch size the carving must hold partial results for
// (the public size query cannot ask the device and uses kMaxUnits).
inline DecodeWorkspace carve_decode(const Params& P, int max_units = kMaxUnits) {
  DecodeWorkspace W;
  const int n_groups = P.batch * P.n_kv_heads;
  int64_t ucap = 0;
  for (int j = 0; j < P.n_kv_heads; ++j) {
    const int64_t g = P.gran[j];
    const int64_t nb = (P.max_seq_len + g - 1) / g;
    const int64_t always = (P.sink_tokens + g - 1) / g + (P.window_tokens + g - 1) / g + 1;
    const int64_t u = nb < always + (int64_t)P.group * P.k_max ? nb : always + (int64_t)P.group * P.k_max;
    if (u > ucap) ucap = u;
  }
  if (ucap < 1) ucap = 1;
  const int64_t slots = (int64_t)max_units * (1 + kClaimedPerWg) + 2 * n_groups + 8;
  W.union_cap = (int32_t)ucap;
  W.slots_cap = (int32_t)slots;
  size_t off = 0;
  // (+ room for rounding: in direct mode the lists are stored in w pieces of ceil(ucap / w) entries per group)
  W.union_off = off;  off += align_up(((size_t)n_groups * ucap + 2 * (size_t)kMaxUnits) * sizeof(uint32_t));
  W.ucount_off = off; off += align_up((size_t)n_groups * sizeof(int32_t));
  W.sched_off = off;  off += align_up((size_t)(n_groups + 8) * sizeof(int32_t));
  W.acc_off = off;    off += align_up((size_t)slots * P.group * P.head_dim * sizeof(float));
  W.ml_off = off;     off += align_up((size_t)slots * P.group * 2 * sizeof(float));
  W.total = off;
  return W;
}

// Optional per-kernel timing (benchmarks only): slots are recorded around launches when enabled.
enum ProfileSlot { kSlotScore = 0, kSlotTopk = 1, kSlotPlan = 2, kSlotAttend = 3, kSlotMerge = 4, kNumSlots = 5 };
struct Profiler {
  bool enabled = false;
  hipEvent_t start[kNumSlots] = {}, stop[kNumSlots] = {};
  bool recorded[kNumSlots] = {};
};
Profiler& profiler();
struct ScopedSlot {  // records start on construction and stop on destruction, on `stream`
  int slot;
  hipStream_t stream;
  ScopedSlot(int s, hipStream_t st) : slot(s), stream(st) {
    if (profiler().enabled) (void)hipEventRecord(profiler().start[slot], stream);
  }
  ~ScopedSlot() {
    if (profiler().enabled) {
      (void)hipEventRecord(profiler().stop[slot], stream);
      profiler().recorded[slot] = true;
    }
  }
};

float select_error_gamma();
hipError_t launch_summarize(const Params& P, const void* K, void* S, const int32_t* prev_len, int max_new_tokens,
                            hipStream_t stream);
hipError_t launch_coarsen(const Params& Pf, const Params& Pc, const void* Sf, void* Sc, hipStream_t stream);
hipError_t launch_select(const Params& P, const void* q, const void* S, const float* budget_frac,
                         const int32_t* budget_blocks, int32_t* idx, int32_t* cnt, void* workspace, int n_cu,
                         hipStream_t stream);
// Workgroups the attention kernel is launched with on the current device (resident slots, at most kMaxUnits).
int attend_launch_size(const Params& P, int n_cu);
// `carve_units`: the max_units the caller sized `workspace` with (>= attend_launch_size).
hipError_t launch_decode(const Params& P, const void* q, const void* K, const void* V, const int32_t* idx,
                         const int32_t* cnt, float* out, void* workspace, int carve_units, int n_cu,
                         hipStream_t stream);

}  // namespace fx
