// C ABI of libfluxion: argument validation on the host, then kernel launches on the caller's stream.
// Every check that does not need the device happens before the first HIP call.
#include "../../include/fluxion.h"

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
  return FX_OK;
}

int compute_units() {
  static int n_cu = 0;
  if (n_cu == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
      n = 256;
    n_cu = n;
  }
  return n_cu;
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
  }
  return "unknown status";
}

fx_status fx_summarize(const fx_layout* layout, const void* K, void* summaries, void* stream) {
  fx::Params P;
  fx_status st = make_params(layout, 0, 0, 1, &P);
  if (st != FX_OK) return st;
  if (!K || !summaries || !aligned16(K) || !aligned16(summaries)) return FX_ERR_INVALID_ARG;
  if (P.max_seq_len == 0) return FX_OK;
  return fx::launch_summarize(P, K, summaries, static_cast<hipStream_t>(stream)) == hipSuccess ? FX_OK : FX_ERR_HIP;
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
  return fx::launch_select(P, q, summaries, budget_frac, budget_blocks, idx, cnt, workspace,
                           static_cast<hipStream_t>(stream)) == hipSuccess
             ? FX_OK
             : FX_ERR_HIP;
}

fx_status fx_select_workspace_view(const fx_layout* layout, size_t* approx_offset, size_t* mag_offset,
                                   int64_t* row_stride, float* gamma) {
  fx::Params P;
  fx_status st = make_params(layout, 0, 0, 1, &P);
  if (st != FX_OK) return st;
  if (!approx_offset || !mag_offset || !row_stride || !gamma) return FX_ERR_INVALID_ARG;
  const fx::SelectWorkspace W = fx::carve_select(P);
  *approx_offset = W.approx_off;
  *mag_offset = W.mag_off;
  *row_stride = P.nb_stride;
  *gamma = fx::select_error_gamma();
  return FX_OK;
}

size_t fx_decode_workspace_bytes(const fx_layout* layout, int32_t k_max, int32_t sink_tokens, int32_t window_tokens) {
  fx::Params P;
  if (make_params(layout, sink_tokens, window_tokens, k_max, &P) != FX_OK) return 0;
  return fx::carve_decode(P).total;
}

fx_status fx_sparse_decode(const fx_layout* layout, const void* q, const void* K, const void* V, const int32_t* idx,
                           const int32_t* cnt, int32_t k_max, int32_t sink_tokens, int32_t window_tokens, float* out,
                           void* workspace, size_t workspace_bytes, void* stream) {
  fx::Params P;
  fx_status st = make_params(layout, sink_tokens, window_tokens, k_max, &P);
  if (st != FX_OK) return st;
  if (!q || !K || !V || !idx || !cnt || !out || !workspace) return FX_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(K) || !aligned16(V) || !aligned16(workspace)) return FX_ERR_INVALID_ARG;
  if (workspace_bytes < fx::carve_decode(P).total) return FX_ERR_WORKSPACE_TOO_SMALL;
  return fx::launch_decode(P, q, K, V, idx, cnt, out, workspace, compute_units(), static_cast<hipStream_t>(stream)) ==
                 hipSuccess
             ? FX_OK
             : FX_ERR_HIP;
}

}  // extern "C"
