// fx_oracle.cpp -- CPU oracle for block-sparse decode attention (TEST INFRASTRUCTURE ONLY).
//
// This file is the slow, plain, fp64 statement of what the hot path computes.  It exists so that
// tests, the smoke check and the benchmark's cpu_baseline leg have something independent to compare
// the HIP kernels with.  It shares no code, header, table or helper with the HIP library and the
// product never calls it.
//
// What it follows (the paper, by section):
//   * Sec. 2.1  -- two-stage block-sparse attention: logical blocks of `g` tokens, Quest-style block
//                  metadata (per-channel minimum and maximum of the block's keys), query-vs-metadata
//                  relevance estimate, top-k blocks, attention over the selected blocks' tokens.
//   * Sec. 2.2 / Sec. 4 step 4 -- the output over selected blocks is fused with the output over the
//                  always-retained initial (sink) and most recent (local window) tokens.
//   * Sec. 3.2 / Sec. 7.1 -- the retained set is counted in tokens (64 initial, 256 recent there).
//   * Sec. 5.3  -- under GQA all heads of a group share one block size; each head has its own budget.
//   * App. A.1  -- segment scores s = q K^T / sqrt(D), LSE, and O = softmax(s) V.
//
// Readings taken where the paper is silent (each is listed in the design notes of the repository):
//   block score = sum_c max(q_c * mn_c, q_c * mx_c)   (the per-channel upper bound the min/max
//   metadata exists for); budget fraction applies to the candidate blocks (those that are neither
//   sink nor window blocks), k = ceil(frac * n_cand) evaluated in double; ties go to the lower block
//   index; each head attends to its own selection, not the group union; a partial tail block covers
//   only its valid tokens; a sink/window size that is not a whole number of blocks is rounded
//   outwards to whole blocks.
//
// Parity pins (tests/test_oracle_*.py): dense special case against a library softmax-attention,
// two-token closed form, uniform-key closed form, softmax weights summing to 1, budget 1.0 == dense,
// budget 0 == dense over the retained tokens, chunked online-softmax merge == two-pass, rank-counting
// brute force and planted exact ties for top-k, min/max bracketing and coarsening identities for the
// summaries, upper-bound invariant for the score, single-token blocks giving score == q.k.
// End-to-end numeric values: parity unpinned (the paper prints no q/K/V -> output example).
//
// All tensors are bf16 bit patterns (uint16_t) decoded exactly to double; all arithmetic is fp64.

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <thread>
#include <vector>

namespace {

struct Layout {
  int32_t batch, n_q_heads, n_kv_heads, head_dim;
  const int32_t* seq_len;   // [batch] valid tokens of each sequence
  const int64_t* seq_base;  // [batch] element offset of token 0, KV head 0 of each sequence in K and V
  int64_t kv_head_stride;   // elements between consecutive KV heads of one sequence
  int64_t token_stride;     // elements between consecutive tokens
  const int64_t* sum_base;  // [batch * n_kv_heads] offset, in blocks, of block 0 in the summaries
  const int32_t* gran;      // [n_kv_heads] logical block size g_j in tokens
};

inline double bf16_to_double(uint16_t bits) {
  uint32_t u = static_cast<uint32_t>(bits) << 16;
  float f;
  std::memcpy(&f, &u, sizeof f);
  return static_cast<double>(f);
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Block geometry of one (sequence, KV head): number of blocks, number of leading sink blocks and the
// first window block.  Candidates for selection are the blocks i with n_sink <= i < w0.
struct Geometry {
  int64_t n_tokens, g, n_blocks, n_sink, w0, n_cand;
};

Geometry geometry(const Layout& L, int b, int j, int sink_tokens, int window_tokens) {
  Geometry G;
  G.n_tokens = L.seq_len[b];
  G.g = L.gran[j];
  G.n_blocks = ceil_div(G.n_tokens, G.g);
  G.n_sink = ceil_div(sink_tokens, G.g);
  int64_t first_window_token = std::max<int64_t>(G.n_tokens - window_tokens, 0);
  G.w0 = first_window_token / G.g;
  G.n_cand = std::max<int64_t>(G.w0 - G.n_sink, 0);
  return G;
}

inline const uint16_t* key_row(const Layout& L, const uint16_t* T, int b, int j, int64_t t) {
  return T + L.seq_base[b] + static_cast<int64_t>(j) * L.kv_head_stride + t * L.token_stride;
}

// Summary of block i of (b, j): S[(sum_base + i) * 2 * d + 0 * d + c] = min, [... + 1 * d + c] = max.
inline const uint16_t* summary_row(const Layout& L, const uint16_t* S, int b, int j, int64_t i, int which) {
  int64_t blk = L.sum_base[static_cast<int64_t>(b) * L.n_kv_heads + j] + i;
  return S + (blk * 2 + which) * L.head_dim;
}

template <class F>
void parallel_for(int64_t n_tasks, int n_threads, F&& body) {
  if (n_threads <= 1 || n_tasks <= 1) {
    for (int64_t i = 0; i < n_tasks; ++i) body(i);
    return;
  }
  std::atomic<int64_t> next{0};
  std::vector<std::thread> pool;
  for (int w = 0; w < n_threads; ++w)
    pool.emplace_back([&] {
      for (;;) {
        int64_t i = next.fetch_add(1);
        if (i >= n_tasks) return;
        body(i);
      }
    });
  for (auto& th : pool) th.join();
}

// Quest-style relevance estimate of one block for one query head (Sec. 2.1): per channel the larger
// of q*min and q*max, summed over channels.  No 1/sqrt(D): ranking does not depend on a positive scale.
double block_score(const Layout& L, const uint16_t* q_h, const uint16_t* S, int b, int j, int64_t i) {
  const uint16_t* mn = summary_row(L, S, b, j, i, 0);
  const uint16_t* mx = summary_row(L, S, b, j, i, 1);
  double s = 0.0;
  for (int c = 0; c < L.head_dim; ++c) {
    double qc = bf16_to_double(q_h[c]);
    s += std::max(qc * bf16_to_double(mn[c]), qc * bf16_to_double(mx[c]));
  }
  return s;
}

// Number of blocks head h keeps among n_cand candidates.
int64_t budget_to_k(const float* budget_frac, const int32_t* budget_blocks, int64_t slot, int64_t n_cand) {
  int64_t k;
  if (budget_blocks)
    k = budget_blocks[slot];
  else
    k = static_cast<int64_t>(std::ceil(static_cast<double>(budget_frac[slot]) * static_cast<double>(n_cand)));
  return std::min(std::max<int64_t>(k, 0), n_cand);
}

// Tokens head h of sequence b attends to: valid tokens of its selected blocks, of the sink blocks and
// of the window blocks, in ascending order, each once.
// With group_union the selected blocks of every head of h's GQA group count (Sec. 5.3 discusses the
// union of a group's selections as the data that is actually moved).
std::vector<int64_t> token_set(const Layout& L, int b, int h, const int32_t* idx, const int32_t* cnt,
                               int k_max, int sink_tokens, int window_tokens, bool group_union = false) {
  int G = L.n_q_heads / L.n_kv_heads;
  int j = h / G;
  Geometry geo = geometry(L, b, j, sink_tokens, window_tokens);
  std::vector<char> keep(static_cast<size_t>(geo.n_blocks), 0);
  for (int64_t i = 0; i < geo.n_blocks; ++i)
    if (i < geo.n_sink || i >= geo.w0) keep[i] = 1;
  for (int hh = group_union ? j * G : h; hh < (group_union ? (j + 1) * G : h + 1); ++hh) {
    int64_t slot = static_cast<int64_t>(b) * L.n_q_heads + hh;
    for (int r = 0; r < cnt[slot]; ++r) {
      int64_t i = idx[slot * k_max + r];
      if (i >= 0 && i < geo.n_blocks) keep[i] = 1;
    }
  }
  std::vector<int64_t> tokens;
  for (int64_t i = 0; i < geo.n_blocks; ++i) {
    if (!keep[i]) continue;
    int64_t hi = std::min((i + 1) * geo.g, geo.n_tokens);
    for (int64_t t = i * geo.g; t < hi; ++t) tokens.push_back(t);
  }
  return tokens;
}

// App. A.1: s_t = <q, k_t> / sqrt(D).
double logit(const Layout& L, const uint16_t* q_h, const uint16_t* k_t) {
  double dot = 0.0;
  for (int c = 0; c < L.head_dim; ++c) dot += bf16_to_double(q_h[c]) * bf16_to_double(k_t[c]);
  return dot / std::sqrt(static_cast<double>(L.head_dim));
}

// Two-pass softmax attention over an explicit token list.  Optionally returns the weights and the LSE.
void attend_two_pass(const Layout& L, const uint16_t* q_h, const uint16_t* K, const uint16_t* V, int b, int j,
                     const std::vector<int64_t>& tokens, double* out, double* weights, double* lse) {
  int d = L.head_dim;
  std::vector<double> s(tokens.size());
  double m = -std::numeric_limits<double>::infinity();
  for (size_t n = 0; n < tokens.size(); ++n) {
    s[n] = logit(L, q_h, key_row(L, K, b, j, tokens[n]));
    m = std::max(m, s[n]);
  }
  double denom = 0.0;
  for (size_t n = 0; n < tokens.size(); ++n) {
    s[n] = std::exp(s[n] - m);
    denom += s[n];
  }
  for (int c = 0; c < d; ++c) out[c] = 0.0;
  for (size_t n = 0; n < tokens.size(); ++n) {
    double p = s[n] / denom;
    if (weights) weights[n] = p;
    const uint16_t* v = key_row(L, V, b, j, tokens[n]);
    for (int c = 0; c < d; ++c) out[c] += p * bf16_to_double(v[c]);
  }
  if (lse) *lse = tokens.empty() ? -std::numeric_limits<double>::infinity() : m + std::log(denom);
}

// Split-K form: the token list is cut into chunks of `chunk` tokens; each chunk yields a partial
// (m, l, acc) and partials are fused by M = max m_i, L = sum l_i e^{m_i - M}, o = sum acc_i e^{m_i - M} / L.
void attend_chunked(const Layout& L, const uint16_t* q_h, const uint16_t* K, const uint16_t* V, int b, int j,
                    const std::vector<int64_t>& tokens, int64_t chunk, double* out) {
  int d = L.head_dim;
  struct Partial {
    double m, l;
    std::vector<double> acc;
  };
  std::vector<Partial> parts;
  for (size_t lo = 0; lo < tokens.size(); lo += static_cast<size_t>(chunk)) {
    size_t hi = std::min(tokens.size(), lo + static_cast<size_t>(chunk));
    Partial P{-std::numeric_limits<double>::infinity(), 0.0, std::vector<double>(d, 0.0)};
    std::vector<double> s(hi - lo);
    for (size_t n = lo; n < hi; ++n) {
      s[n - lo] = logit(L, q_h, key_row(L, K, b, j, tokens[n]));
      P.m = std::max(P.m, s[n - lo]);
    }
    for (size_t n = lo; n < hi; ++n) {
      double e = std::exp(s[n - lo] - P.m);
      P.l += e;
      const uint16_t* v = key_row(L, V, b, j, tokens[n]);
      for (int c = 0; c < d; ++c) P.acc[c] += e * bf16_to_double(v[c]);
    }
    parts.push_back(std::move(P));
  }
  double M = -std::numeric_limits<double>::infinity();
  for (auto& P : parts) M = std::max(M, P.m);
  double Lsum = 0.0;
  for (int c = 0; c < d; ++c) out[c] = 0.0;
  for (auto& P : parts) {
    double w = std::exp(P.m - M);
    Lsum += P.l * w;
    for (int c = 0; c < d; ++c) out[c] += P.acc[c] * w;
  }
  for (int c = 0; c < d; ++c) out[c] = parts.empty() ? 0.0 : out[c] / Lsum;
}

}  // namespace

extern "C" {

struct fxo_layout {
  int32_t batch, n_q_heads, n_kv_heads, head_dim;
  const int32_t* seq_len;
  const int64_t* seq_base;
  int64_t kv_head_stride, token_stride;
  const int64_t* sum_base;
  const int32_t* gran;
};

static Layout to_layout(const fxo_layout* l) {
  return Layout{l->batch,    l->n_q_heads,      l->n_kv_heads,   l->head_dim, l->seq_len,
                l->seq_base, l->kv_head_stride, l->token_stride, l->sum_base, l->gran};
}

// Sec. 2.1: per block and channel, minimum and maximum of the block's valid keys (kept as the bf16
// bit pattern of the winning key element; among equal values the first token's pattern is kept).
void fxo_summarize(const fxo_layout* l, const uint16_t* K, uint16_t* S, int n_threads) {
  Layout L = to_layout(l);
  int64_t n_tasks = static_cast<int64_t>(L.batch) * L.n_kv_heads;
  parallel_for(n_tasks, n_threads, [&](int64_t task) {
    int b = static_cast<int>(task / L.n_kv_heads), j = static_cast<int>(task % L.n_kv_heads);
    Geometry geo = geometry(L, b, j, 0, 0);
    for (int64_t i = 0; i < geo.n_blocks; ++i) {
      uint16_t* mn = const_cast<uint16_t*>(summary_row(L, S, b, j, i, 0));
      uint16_t* mx = const_cast<uint16_t*>(summary_row(L, S, b, j, i, 1));
      int64_t lo = i * geo.g, hi = std::min((i + 1) * geo.g, geo.n_tokens);
      for (int c = 0; c < L.head_dim; ++c) {
        uint16_t best_mn = key_row(L, K, b, j, lo)[c], best_mx = best_mn;
        for (int64_t t = lo + 1; t < hi; ++t) {
          uint16_t x = key_row(L, K, b, j, t)[c];
          if (bf16_to_double(x) < bf16_to_double(best_mn)) best_mn = x;
          if (bf16_to_double(x) > bf16_to_double(best_mx)) best_mx = x;
        }
        mn[c] = best_mn;
        mx[c] = best_mx;
      }
    }
  });
}

// Scores of every candidate block: scores[(b * Hq + h) * nb_stride + i] for n_sink <= i < w0; other
// entries are left untouched.
void fxo_scores(const fxo_layout* l, const uint16_t* q, const uint16_t* S, int sink_tokens, int window_tokens,
                double* scores, int64_t nb_stride, int n_threads) {
  Layout L = to_layout(l);
  int G = L.n_q_heads / L.n_kv_heads;
  int64_t n_tasks = static_cast<int64_t>(L.batch) * L.n_q_heads;
  parallel_for(n_tasks, n_threads, [&](int64_t task) {
    int b = static_cast<int>(task / L.n_q_heads), h = static_cast<int>(task % L.n_q_heads);
    int j = h / G;
    Geometry geo = geometry(L, b, j, sink_tokens, window_tokens);
    const uint16_t* q_h = q + task * L.head_dim;
    for (int64_t i = geo.n_sink; i < geo.w0; ++i) scores[task * nb_stride + i] = block_score(L, q_h, S, b, j, i);
  });
}

// Top-k block selection per head (Sec. 2.1): order candidates by (score descending, index ascending),
// keep the first k_h, report them ascending in idx[(b*Hq+h)*k_max + r], pad with -1, count in cnt.
// tie_gap[b*Hq+h] (optional) = |s_k - s_{k+1}| / max(|s_k|, |s_{k+1}|) for the last kept and the first
// dropped candidate in that order, +inf when there is no such pair.  kth_score (optional) = s_k.
// Returns 0, or -1 if some k_h exceeds k_max (nothing is truncated silently).
int fxo_select(const fxo_layout* l, const uint16_t* q, const uint16_t* S, const float* budget_frac,
               const int32_t* budget_blocks, int sink_tokens, int window_tokens, int k_max, int32_t* idx,
               int32_t* cnt, double* tie_gap, double* kth_score, int n_threads) {
  Layout L = to_layout(l);
  int G = L.n_q_heads / L.n_kv_heads;
  int64_t n_tasks = static_cast<int64_t>(L.batch) * L.n_q_heads;
  std::atomic<int> status{0};
  parallel_for(n_tasks, n_threads, [&](int64_t task) {
    int b = static_cast<int>(task / L.n_q_heads), h = static_cast<int>(task % L.n_q_heads);
    int j = h / G;
    Geometry geo = geometry(L, b, j, sink_tokens, window_tokens);
    int64_t k = budget_to_k(budget_frac, budget_blocks, task, geo.n_cand);
    for (int r = 0; r < k_max; ++r) idx[task * k_max + r] = -1;
    cnt[task] = 0;
    if (tie_gap) tie_gap[task] = std::numeric_limits<double>::infinity();
    if (kth_score) kth_score[task] = std::numeric_limits<double>::quiet_NaN();
    if (k > k_max) {
      status = -1;
      return;
    }
    const uint16_t* q_h = q + task * L.head_dim;
    std::vector<std::pair<double, int64_t>> cand;
    for (int64_t i = geo.n_sink; i < geo.w0; ++i) cand.emplace_back(block_score(L, q_h, S, b, j, i), i);
    std::sort(cand.begin(), cand.end(), [](const auto& a, const auto& c) {
      if (a.first != c.first) return a.first > c.first;
      return a.second < c.second;
    });
    std::vector<int64_t> chosen;
    for (int64_t r = 0; r < k; ++r) chosen.push_back(cand[r].second);
    std::sort(chosen.begin(), chosen.end());
    for (int64_t r = 0; r < k; ++r) idx[task * k_max + r] = static_cast<int32_t>(chosen[r]);
    cnt[task] = static_cast<int32_t>(k);
    if (k > 0 && kth_score) kth_score[task] = cand[k - 1].first;
    if (k > 0 && k < static_cast<int64_t>(cand.size()) && tie_gap) {
      double a = cand[k - 1].first, c = cand[k].first;
      double scale = std::max(std::fabs(a), std::fabs(c));
      tie_gap[task] = scale > 0.0 ? std::fabs(a - c) / scale : 0.0;
    }
  });
  return status.load();
}

// Sparse attention of every head over its own token set (App. A.1 restricted to the kept tokens).
// mode 0: two-pass softmax.  mode 1: split into chunks of `chunk_tokens` and merged.
// group_union != 0: every head attends to the union of its group's selections.
// out[(b*Hq+h)*d + c] in fp64; lse (optional) [b*Hq+h], mode 0 only.
void fxo_sparse_attention(const fxo_layout* l, const uint16_t* q, const uint16_t* K, const uint16_t* V,
                          const int32_t* idx, const int32_t* cnt, int k_max, int sink_tokens, int window_tokens,
                          int mode, int64_t chunk_tokens, int group_union, double* out, double* lse, int n_threads) {
  Layout L = to_layout(l);
  int G = L.n_q_heads / L.n_kv_heads;
  int64_t n_tasks = static_cast<int64_t>(L.batch) * L.n_q_heads;
  parallel_for(n_tasks, n_threads, [&](int64_t task) {
    int b = static_cast<int>(task / L.n_q_heads), h = static_cast<int>(task % L.n_q_heads);
    int j = h / G;
    std::vector<int64_t> tokens = token_set(L, b, h, idx, cnt, k_max, sink_tokens, window_tokens, group_union != 0);
    const uint16_t* q_h = q + task * L.head_dim;
    if (mode == 0)
      attend_two_pass(L, q_h, K, V, b, j, tokens, out + task * L.head_dim, nullptr, lse ? lse + task : nullptr);
    else
      attend_chunked(L, q_h, K, V, b, j, tokens, chunk_tokens, out + task * L.head_dim);
  });
}

// Dense attention over all valid tokens of the sequence (App. A.1 with S = everything).
void fxo_dense_attention(const fxo_layout* l, const uint16_t* q, const uint16_t* K, const uint16_t* V, double* out,
                         double* lse, int n_threads) {
  Layout L = to_layout(l);
  int G = L.n_q_heads / L.n_kv_heads;
  int64_t n_tasks = static_cast<int64_t>(L.batch) * L.n_q_heads;
  parallel_for(n_tasks, n_threads, [&](int64_t task) {
    int b = static_cast<int>(task / L.n_q_heads), h = static_cast<int>(task % L.n_q_heads);
    int j = h / G;
    std::vector<int64_t> tokens(static_cast<size_t>(L.seq_len[b]));
    for (size_t t = 0; t < tokens.size(); ++t) tokens[t] = static_cast<int64_t>(t);
    attend_two_pass(L, q + task * L.head_dim, K, V, b, j, tokens, out + task * L.head_dim, nullptr,
                    lse ? lse + task : nullptr);
  });
}

// Token set and softmax weights of one (b, h), for inspection by tests.  Writes at most `capacity`
// tokens/weights and returns the size of the set.
int64_t fxo_token_weights(const fxo_layout* l, const uint16_t* q, const uint16_t* K, const uint16_t* V,
                          const int32_t* idx, const int32_t* cnt, int k_max, int sink_tokens, int window_tokens,
                          int b, int h, int group_union, int64_t capacity, int64_t* tokens_out,
                          double* weights_out) {
  Layout L = to_layout(l);
  int G = L.n_q_heads / L.n_kv_heads;
  std::vector<int64_t> tokens = token_set(L, b, h, idx, cnt, k_max, sink_tokens, window_tokens, group_union != 0);
  std::vector<double> w(tokens.size()), o(static_cast<size_t>(L.head_dim));
  int64_t task = static_cast<int64_t>(b) * L.n_q_heads + h;
  attend_two_pass(L, q + task * L.head_dim, K, V, b, h / G, tokens, o.data(), w.data(), nullptr);
  int64_t n = std::min<int64_t>(capacity, static_cast<int64_t>(tokens.size()));
  for (int64_t r = 0; r < n; ++r) {
    tokens_out[r] = tokens[r];
    weights_out[r] = w[r];
  }
  return static_cast<int64_t>(tokens.size());
}

// One decode layer-step as the baseline times it: selection followed by sparse attention.
int fxo_layer_step(const fxo_layout* l, const uint16_t* q, const uint16_t* K, const uint16_t* V, const uint16_t* S,
                   const float* budget_frac, const int32_t* budget_blocks, int sink_tokens, int window_tokens,
                   int k_max, int32_t* idx, int32_t* cnt, double* out, int n_threads) {
  int rc = fxo_select(l, q, S, budget_frac, budget_blocks, sink_tokens, window_tokens, k_max, idx, cnt, nullptr,
                      nullptr, n_threads);
  if (rc != 0) return rc;
  fxo_sparse_attention(l, q, K, V, idx, cnt, k_max, sink_tokens, window_tokens, 0, 0, 0, out, nullptr, n_threads);
  return 0;
}

}  // extern "C"
