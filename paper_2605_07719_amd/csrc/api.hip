// C ABI of libfluxion: argument validation on the host, then kernel launches on the caller's stream.
// Every check that does not need the device happens before the first HIP call.
#include "../../include/fluxion.h"

#include <atomic>
#include <mutex>

#include "fx_device.hpp"
#include "fx_kernels.hpp"

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Validates the host-visible part of a layout and fills the kernel parameter block.
fx_status make_params(const fx_layout* L, int32_t sink_tokens, int32_t window_tokens, int32_t k_max, fx::Params* P) {
  if (!L) return FX_ERR_INVALID_ARG;
  if (!L->seq_len || !L->seq_base || !L->sum_base || !L->gran) return FX_ERR_INVALID_ARG;
  if (L->batch < 1 || L->n_q_heads < 1 || L->n_kv_heads < 1 || L->max_seq_len < 0) return FX_ERR_INVALID_ARG;
  if (L->n_q_heads % L->n_kv_heads != 0) return FX_ERR_INVALID_ARG;
  if (sink_tokens < 0 || window_tokens < 0 || k_max < 1) return FX_ERR_INVALID_ARG;
  if (L->token_stride < L->head_dim || L->token_stride % 8 != 0 || L->kv_head_stride % 8 != 0 || L->kv_head_stride < 0)
    return FX_ERR_INVALID_ARG;
  if (L->head_dim != 64 && L->head_dim != 128) return FX_ERR_UNSUPPORTED;
  const int group = L->n_q_heads / L->n_kv_heads;
  if (group > fx::kMaxGroup || L->n_kv_heads > fx::kMaxKvHeads) return FX_ERR_UNSUPPORTED;
  if (L->max_seq_len > fx::kMaxSeqLen || L->batch > 65535) return FX_ERR_UNSUPPORTED;
  if ((int64_t)L->batch * L->n_kv_heads > fx::kMaxGroups) return FX_ERR_UNSUPPORTED;
  P->batch = L->batch;
  P->n_q_heads = L->n_q_heads;
  P->n_kv_heads = L->n_kv_heads;
  P->head_dim = L->head_dim;
  P->group = group;
  P->max_seq_len = L->max_seq_len;
  P->seq_len = L->seq_len;
  P->seq_base = L->seq_base;
  P->kv_head_stride = L->kv_head_stride;
  P->token_stride = L->token_stride;
  P->sum_base = L->sum_base;
  int nb_stride = 1;
  for (int j = 0; j < fx::kMaxKvHeads; ++j) P->gran[j] = 16;
  for (int j = 0; j < L->n_kv_heads; ++j) {
    const int g = L->gran[j];
    if (g < 16 || g > 128 || g % 16 != 0) return FX_ERR_UNSUPPORTED;
    P->gran[j] = (uint8_t)g;
    const int nb = (L->max_seq_len + g - 1) / g;
    if (nb > nb_stride) nb_stride = nb;
  }
  P->nb_stride = nb_stride;
  P->sink_tokens = sink_tokens;
  P->window_tokens = window_tokens;
  P->k_max = k_max;
  P->group_union = 0;
  return FX_OK;
}

// Compute units of the current device (queried once per device).
int compute_units() {
  static std::atomic<int> cached[fx::kMaxDevices];
  const int dev = fx::current_device();
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
    cached[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

}  // namespace

namespace fx {
Profiler& profiler() {
  static Profiler p;
  return p;
}
}  // namespace fx

extern "C" {

fx_status fx_profile_enable(int enable) {
  fx::Profiler& p = fx::profiler();
  if ((enable != 0) == p.enabled) return FX_OK;
  if (enable) {
    for (int s = 0; s < fx::kNumSlots; ++s) {
      if (hipEventCreate(&p.start[s]) != hipSuccess || hipEventCreate(&p.stop[s]) != hipSuccess) return FX_ERR_HIP;
      p.recorded[s] = false;
    }
    p.enabled = true;
  } else {
    p.enabled = false;
    for (int s = 0; s < fx::kNumSlots; ++s) {
      (void)hipEventDestroy(p.start[s]);
      (void)hipEventDestroy(p.stop[s]);
      p.recorded[s] = false;
    }
  }
  return FX_OK;
}

fx_status fx_profile_read(float* ms, int n) {
  fx::Profiler& p = fx::profiler();
  if (!ms || n != fx::kNumSlots || !p.enabled) return FX_ERR_INVALID_ARG;
  for (int s = 0; s < fx::kNumSlots; ++s) {
    ms[s] = -1.f;
    if (!p.recorded[s]) continue;
    if (hipEventSynchronize(p.stop[s]) != hipSuccess) return FX_ERR_HIP;
    if (hipEventElapsedTime(&ms[s], p.start[s], p.stop[s]) != hipSuccess) return FX_ERR_HIP;
  }
  return FX_OK;
}

const char* fx_status_string(fx_status status) {
  switch (status) {
    case FX_OK: return "ok";
    case FX_ERR_INVALID_ARG: return "invalid argument";
    case FX_ERR_UNSUPPORTED: return "unsupported shape or size";
    case FX_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case FX_ERR_HIP: return "HIP launch failed";
    case FX_ERR_SCRATCH_LIMIT: return "problem exceeds the built-in scratch buffer";
  }
  return "unknown status";
}

fx_status fx_summarize(const fx_layout* layout, const void* K, void* summaries, void* stream) {
  fx::Params P;
  fx_status st = make_params(layout, 0, 0, 1, &P);
  if (st != FX_OK) return st;
  if (!K || !summaries || !aligned16(K) || !aligned16(summaries)) return FX_ERR_INVALID_ARG;
  if (P.max_seq_len == 0) return FX_OK;
  return fx::launch_summarize(P, K, summaries, nullptr, 0, static_cast<hipStream_t>(stream)) == hipSuccess
             ? FX_OK
             : FX_ERR_HIP;
}

fx_status fx_summarize_append(const fx_layout* layout, const void* K, void* summaries, const int32_t* prev_len,
                              int32_t max_new_tokens, void* stream) {
  fx::Params P;
  fx_status st = make_params(layout, 0, 0, 1, &P);
  if (st != FX_OK) return st;
  if (!K || !summaries || !prev_len || !aligned16(K) || !aligned16(summaries) || max_new_tokens < 0)
    return FX_ERR_INVALID_ARG;
  if (P.max_seq_len == 0) return FX_OK;
  if (max_new_tokens > P.max_seq_len) max_new_tokens = P.max_seq_len;
  return fx::launch_summarize(P, K, summaries, prev_len, max_new_tokens, static_cast<hipStream_t>(stream)) ==
                 hipSuccess
             ? FX_OK
             : FX_ERR_HIP;
}

fx_status fx_coarsen_summaries(const fx_layout* fine, const void* fine_summaries, const fx_layout* coarse,
                               void* coarse_summaries, void* stream) {
  fx::Params Pf, Pc;
  fx_status st = make_params(fine, 0, 0, 1, &Pf);
  if (st != FX_OK) return st;
  st = make_params(coarse, 0, 0, 1, &Pc);
  if (st != FX_OK) return st;
  if (!fine_summaries || !coarse_summaries || !aligned16(fine_summaries) || !aligned16(coarse_summaries))
    return FX_ERR_INVALID_ARG;
  if (Pf.batch != Pc.batch || Pf.n_q_heads != Pc.n_q_heads || Pf.n_kv_heads != Pc.n_kv_heads ||
      Pf.head_dim != Pc.head_dim || Pf.max_seq_len != Pc.max_seq_len)
    return FX_ERR_INVALID_ARG;
  for (int j = 0; j < Pf.n_kv_heads; ++j)
    if (Pc.gran[j] % Pf.gran[j] != 0) return FX_ERR_INVALID_ARG;
  if (Pc.max_seq_len == 0) return FX_OK;
  return fx::launch_coarsen(Pf, Pc, fine_summaries, coarse_summaries, static_cast<hipStream_t>(stream)) == hipSuccess
             ? FX_OK
             : FX_ERR_HIP;
}

size_t fx_select_workspace_bytes(const fx_layout* layout) {
  fx::Params P;
  if (make_params(layout, 0, 0, 1, &P) != FX_OK) return 0;
  return fx::carve_select(P).total;
}

fx_status fx_select(const fx_layout* layout, const void* q, const void* summaries, const float* budget_frac,
                    const int32_t* budget_blocks, int32_t sink_tokens, int32_t window_tokens, int32_t k_max,
                    int32_t* idx, int32_t* cnt, void* workspace, size_t workspace_bytes, void* stream) {
  fx::Params P;
  fx_status st = make_params(layout, sink_tokens, window_tokens, k_max, &P);
  if (st != FX_OK) return st;
  if (!q || !summaries || !idx || !cnt || !workspace) return FX_ERR_INVALID_ARG;
  if ((budget_frac == nullptr) == (budget_blocks == nullptr)) return FX_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(summaries) || !aligned16(workspace)) return FX_ERR_INVALID_ARG;
  if (workspace_bytes < fx::carve_select(P).total) return FX_ERR_WORKSPACE_TOO_SMALL;
  return fx::launch_select(P, q, summaries, budget_frac, budget_blocks, idx, cnt, workspace, compute_units(),
                           static_cast<hipStream_t>(stream)) == hipSuccess
             ? FX_OK
             : FX_ERR_HIP;
}

fx_status fx_select_workspace_view(const fx_layout* layout, size_t* approx_offset, size_t* mag_offset,
                                   int64_t* row_stride, int64_t* mag_stride, float* gamma) {
  fx::Params P;
  fx_status st = make_params(layout, 0, 0, 1, &P);
  if (st != FX_OK) return st;
  if (!approx_offset || !mag_offset || !row_stride || !mag_stride || !gamma) return FX_ERR_INVALID_ARG;
  const fx::SelectWorkspace W = fx::carve_select(P);
  *approx_offset = W.approx_off;
  *mag_offset = W.mag_off;
  *row_stride = P.nb_stride;
  *mag_stride = W.mag_stride;
  *gamma = fx::select_error_gamma();
  return FX_OK;
}

size_t fx_decode_workspace_bytes(const fx_layout* layout, int32_t k_max, int32_t sink_tokens, int32_t window_tokens) {
  fx::Params P;
  if (make_params(layout, sink_tokens, window_tokens, k_max, &P) != FX_OK) return 0;
  return fx::carve_decode(P).total;
}

static fx_status sparse_decode_impl(const fx_layout* layout, const void* q, const void* K, const void* V,
                                    const int32_t* idx, const int32_t* cnt, int32_t k_max, int32_t sink_tokens,
                                    int32_t window_tokens, float* out, void* workspace, size_t workspace_bytes,
                                    void* stream, int group_union) {
  fx::Params P;
  fx_status st = make_params(layout, sink_tokens, window_tokens, k_max, &P);
  if (st != FX_OK) return st;
  if (!q || !K || !V || !idx || !cnt || !out || !workspace) return FX_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(K) || !aligned16(V) || !aligned16(workspace)) return FX_ERR_INVALID_ARG;
  if (workspace_bytes < fx::carve_decode(P).total) return FX_ERR_WORKSPACE_TOO_SMALL;
  P.group_union = group_union;
  return fx::launch_decode(P, q, K, V, idx, cnt, out, workspace, fx::kMaxUnits, compute_units(),
                           static_cast<hipStream_t>(stream)) == hipSuccess
             ? FX_OK
             : FX_ERR_HIP;
}

fx_status fx_sparse_decode(const fx_layout* layout, const void* q, const void* K, const void* V, const int32_t* idx,
                           const int32_t* cnt, int32_t k_max, int32_t sink_tokens, int32_t window_tokens, float* out,
                           void* workspace, size_t workspace_bytes, void* stream) {
  return sparse_decode_impl(layout, q, K, V, idx, cnt, k_max, sink_tokens, window_tokens, out, workspace,
                            workspace_bytes, stream, 0);
}

fx_status fx_sparse_decode_union(const fx_layout* layout, const void* q, const void* K, const void* V,
                                 const int32_t* idx, const int32_t* cnt, int32_t k_max, int32_t sink_tokens,
                                 int32_t window_tokens, float* out, void* workspace, size_t workspace_bytes,
                                 void* stream) {
  return sparse_decode_impl(layout, q, K, V, idx, cnt, k_max, sink_tokens, window_tokens, out, workspace,
                            workspace_bytes, stream, 1);
}

// ---- fx_sparse_decode for callers that cannot allocate ---------------------------------------------------------
// The scratch of the decode stage (union lists, split description, claim counter, partial results) lives in a
// file-scope device array instead of a caller-supplied workspace.  Every GPU the library runs on holds its own
// copy of the array at its own address; the address is looked up once per device and that pointer -- never the
// array's name, which in host code is only a stand-in -- is what the kernels receive.
static __device__ __align__(256) unsigned char scratch[FX_STATIC_SCRATCH_BYTES];

namespace {
std::mutex g_scratch_mutex;
void* g_scratch_ptr[fx::kMaxDevices];  // device address of `scratch` per device ordinal; guarded by the mutex

// Device address of `scratch` on the current device, or nullptr.
void* static_scratch() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= fx::kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

fx_status fx_sparse_decode_static(const fx_layout* layout, const void* q, const void* K, const void* V,
                                  const int32_t* idx, const int32_t* cnt, int32_t k_max, int32_t sink_tokens,
                                  int32_t window_tokens, float* out, void* stream) {
  fx::Params P;
  fx_status st = make_params(layout, sink_tokens, window_tokens, k_max, &P);
  if (st != FX_OK) return st;
  if (!q || !K || !V || !idx || !cnt || !out) return FX_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(K) || !aligned16(V)) return FX_ERR_INVALID_ARG;
  // smallest possible carving (one unit): a problem that cannot fit at any launch size is refused on the host
  if (fx::carve_decode(P, 1).total > (size_t)FX_STATIC_SCRATCH_BYTES) return FX_ERR_SCRATCH_LIMIT;
  void* ws = static_scratch();
  if (!ws) return FX_ERR_HIP;
  const int n_cu = compute_units();
  const int units = fx::attend_launch_size(P, n_cu);  // the attention kernel's launch size on this device
  if (fx::carve_decode(P, units).total > (size_t)FX_STATIC_SCRATCH_BYTES) return FX_ERR_SCRATCH_LIMIT;
  return fx::launch_decode(P, q, K, V, idx, cnt, out, ws, units, n_cu, static_cast<hipStream_t>(stream)) == hipSuccess
             ? FX_OK
             : FX_ERR_HIP;
}

}  // extern "C"
