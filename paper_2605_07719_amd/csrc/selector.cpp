// Granularity-budget selector (host control logic; Sec. 5.2 Eq. 1 and Sec. 5.3 Eq. 3 of the paper).
// It only fills the gran[] / budget[] tables the kernels consume.
#include "../../include/fluxion.h"

#include <cmath>

extern "C" fx_status fx_choose_granularity(int32_t n_q_heads, int32_t n_kv_heads, const float* bgt0,
                                           const float* slope, const uint8_t* streaming, int64_t l_cpu,
                                           const int32_t* candidates, int32_t n_candidates, int32_t* gran,
                                           float* budget, double* volume) {
  if (n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads != 0) return FX_ERR_INVALID_ARG;
  if (!bgt0 || !slope || !candidates || !gran || !budget || n_candidates < 1 || l_cpu < 0) return FX_ERR_INVALID_ARG;
  for (int c = 0; c < n_candidates; ++c)
    if (candidates[c] < 1) return FX_ERR_INVALID_ARG;
  const int G = n_q_heads / n_kv_heads;
  auto head_budget = [&](int h, int blk) -> double {  // Eq. 1, kept inside [0, 1]; streaming heads keep nothing
    if (streaming && streaming[h]) return 0.0;
    const double b = (double)bgt0[h] + (double)slope[h] * std::log2((double)blk);
    return b < 0.0 ? 0.0 : (b > 1.0 ? 1.0 : b);
  };
  for (int j = 0; j < n_kv_heads; ++j) {
    bool any_retrieval = false;
    for (int r = 0; r < G; ++r) any_retrieval |= !(streaming && streaming[j * G + r]);
    int best = candidates[0];
    double best_v = 0.0;
    if (any_retrieval) {
      for (int c = 0; c < n_candidates; ++c) {
        const int blk = candidates[c];
        double sum = 0.0;
        for (int r = 0; r < G; ++r) sum += head_budget(j * G + r, blk);
        const double v = 2.0 * (double)l_cpu / (double)blk + 2.0 * (double)l_cpu * sum;  // Eq. 3
        if (c == 0 || v < best_v) {  // ties keep the earlier candidate
          best = blk;
          best_v = v;
        }
      }
    }
    gran[j] = best;
    if (volume) volume[j] = best_v;
    for (int r = 0; r < G; ++r) budget[j * G + r] = (float)head_budget(j * G + r, best);
  }
  return FX_OK;
}
