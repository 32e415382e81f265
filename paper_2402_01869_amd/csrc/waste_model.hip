// Host-side arithmetic of the scheduler that drives the kernels: the GPU-memory-waste model
// (Section 3.2, Eq. 1-3; Section 4.2, Eq. 4; Section 4.3, Eq. 5), recomputation chunk sizing and
// the saturation point (Section 4.2), and the interception schedule (Section 4.3).  fp64, no GPU.
#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>
#include <vector>

#include "../../include/infercept_hot.h"

namespace {

const double kNaN = std::numeric_limits<double>::quiet_NaN();

bool table_ok(const ic_tfwd_table* t) {
  if (!t || t->n < 1 || !t->tokens || !t->seconds) return false;
  for (int k = 0; k < t->n; ++k) {
    if (!(t->tokens[k] > 0.0) || !(t->seconds[k] >= 0.0)) return false;
    if (k && !(t->tokens[k] > t->tokens[k - 1])) return false;
  }
  return true;
}

// Piecewise-linear profile; below the first point the ray from the origin, past the last point the
// last segment continued.
double eval(const ic_tfwd_table* t, double x) {
  const double* tk = t->tokens;
  const double* sc = t->seconds;
  if (t->n == 1 || x <= tk[0]) return sc[0] * (x / tk[0]);
  const double* hi = std::lower_bound(tk + 1, tk + t->n - 1, x);  // first point >= x, capped at the last
  const int k = (int)(hi - tk);
  const double w = (x - tk[k - 1]) / (tk[k] - tk[k - 1]);
  return sc[k - 1] + w * (sc[k] - sc[k - 1]);
}

}  // namespace

extern "C" {

double ic_tfwd_eval(const ic_tfwd_table* table, double tokens) {
  if (!table_ok(table) || !(tokens >= 0.0)) return kNaN;
  return eval(table, tokens);
}

double ic_waste_discard(const ic_tfwd_table* table, double ctx_tokens, double other_tokens, double token_bytes) {
  const double t = ic_tfwd_eval(table, ctx_tokens);
  return t * ctx_tokens * token_bytes + t * other_tokens * token_bytes;
}

double ic_waste_preserve(double t_int_s, double ctx_tokens, double token_bytes) {
  return t_int_s * ctx_tokens * token_bytes;
}

double ic_waste_swap(double t_swap_s, double batch_tokens, double token_bytes) {
  return 2.0 * t_swap_s * batch_tokens * token_bytes;
}

double ic_waste_chunked_discard(const ic_tfwd_table* table, double ctx_tokens, double other_tokens,
                                double token_bytes, int32_t n_chunks) {
  if (n_chunks < 1) return kNaN;
  const double whole = ic_tfwd_eval(table, ctx_tokens);
  const double chunk = ic_tfwd_eval(table, ctx_tokens / n_chunks);
  return whole * ctx_tokens * token_bytes / 2.0 + n_chunks * chunk * other_tokens * token_bytes;
}

int64_t ic_chunk_tokens(int64_t saturation_point, int64_t running_tokens) {
  return std::max<int64_t>(0, saturation_point - running_tokens);
}

int64_t ic_chunk_count(int64_t ctx_tokens, int64_t chunk_tokens) {
  if (ctx_tokens < 0 || chunk_tokens < 1) return -1;
  return ctx_tokens / chunk_tokens + (ctx_tokens % chunk_tokens != 0);
}

int64_t ic_saturation_point(const double* query_tokens, const double* seconds, int32_t n, double frac) {
  if (!query_tokens || !seconds || n < 1 || !(frac > 0.0) || frac > 1.0) return -1;
  double best = 0.0;
  for (int k = 0; k < n; ++k) {
    if (!(query_tokens[k] > 0.0) || !(seconds[k] > 0.0) || (k && !(query_tokens[k] > query_tokens[k - 1]))) return -1;
    best = std::max(best, query_tokens[k] / seconds[k]);
  }
  for (int k = 0; k < n; ++k)
    if (query_tokens[k] / seconds[k] >= frac * best) return (int64_t)query_tokens[k];
  return -1;
}

int ic_schedule_intercepted(int32_t n, const double* waste_preserve, const double* waste_chunked_discard,
                            const int64_t* ctx_tokens, int64_t swap_out_budget_tokens, int64_t* swap_tokens,
                            int32_t* action) {
  if (n < 0 || swap_out_budget_tokens < 0) return IC_EINVAL;
  if (n == 0) return IC_OK;
  if (!waste_preserve || !waste_chunked_discard || !ctx_tokens || !swap_tokens || !action) return IC_ENULL;
  std::vector<double> waste((size_t)n);
  for (int i = 0; i < n; ++i) {
    if (ctx_tokens[i] < 0 || !(waste_preserve[i] >= 0.0) || !(waste_chunked_discard[i] >= 0.0)) return IC_EINVAL;
    waste[i] = std::min(waste_preserve[i], waste_chunked_discard[i]);  // Eq. 5
  }
  std::vector<int32_t> order((size_t)n);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return waste[a] > waste[b]; });
  int64_t budget = swap_out_budget_tokens;
  for (int32_t i : order) {
    const int64_t out = std::min(ctx_tokens[i], budget);
    budget -= out;
    swap_tokens[i] = out;
    action[i] = ctx_tokens[i] == out ? IC_ACT_NONE
                : waste_preserve[i] <= waste_chunked_discard[i] ? IC_ACT_PRESERVE : IC_ACT_DISCARD;
  }
  return IC_OK;
}

}  // extern "C"
