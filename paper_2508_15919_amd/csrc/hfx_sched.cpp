// Step composition on the host (HFX Section 3.3.1): token budget (Eq. 3), maturity time, the
// linear prefill-latency model and a one-instance form of the four dispatching steps.  Plain
// double arithmetic; no device calls in this file.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <numeric>
#include <vector>

#include "../../include/hfxattn.h"

namespace {

bool finite_all(std::initializer_list<double> xs) {
  for (double x : xs)
    if (!std::isfinite(x)) return false;
  return true;
}

hfx_status check_model(double ttft, double tpot, const hfx_latency_model* m) {
  if (!m) return HFX_ERR_NULL;
  if (!finite_all({ttft, tpot, m->a, m->b, m->e_d})) return HFX_ERR_MODEL;
  if (ttft <= 0.0 || tpot <= 0.0 || m->b <= 0.0 || m->a < 0.0 || m->e_d < 0.0) return HFX_ERR_MODEL;
  return HFX_OK;
}

const int64_t kBudgetCap = INT64_MAX / 2;

}  // namespace

extern "C" {

hfx_status hfx_token_budget(double ttft, double tpot, const hfx_latency_model* model, int64_t* n_token) {
  if (!n_token) return HFX_ERR_NULL;
  hfx_status st = check_model(ttft, tpot, model);
  if (st != HFX_OK) return st;
  const double slack = tpot - model->e_d;   // what one decode iteration saves against its TPOT
  if (slack <= 0.0) {
    *n_token = 0;
    return HFX_OK;
  }
  // 2 E_p + k E_d <= TTFT with k = E_p / slack  <=>  E_p <= TTFT * slack / (2 TPOT - E_d)
  const double bound = slack * ttft / ((2.0 * tpot - model->e_d) * model->b) - model->a / model->b;
  if (!(bound >= 0.0)) {
    *n_token = 0;
  } else if (bound >= (double)kBudgetCap) {
    *n_token = kBudgetCap;
  } else {
    *n_token = (int64_t)std::floor(bound);
  }
  return HFX_OK;
}

hfx_status hfx_maturity_time(double e_p, double tpot, double e_d, double* k, double* maturity) {
  if (!finite_all({e_p, tpot, e_d}) || e_p < 0.0 || tpot <= 0.0 || e_d < 0.0) return HFX_ERR_MODEL;
  if (tpot - e_d <= 0.0) return HFX_ERR_MODEL;
  const double iters = e_p / (tpot - e_d);
  if (k) *k = iters;
  if (maturity) *maturity = e_p + iters * e_d;
  return HFX_OK;
}

hfx_status hfx_fit_latency_model(int32_t count, const int64_t* n_token, const double* seconds,
                                 hfx_latency_model* model, double* r_squared) {
  if (!n_token || !seconds || !model) return HFX_ERR_NULL;
  if (count < 2) return HFX_ERR_MODEL;
  double mx = 0.0, my = 0.0;
  for (int i = 0; i < count; ++i) {
    if (!std::isfinite(seconds[i])) return HFX_ERR_MODEL;
    mx += (double)n_token[i];
    my += seconds[i];
  }
  mx /= count;
  my /= count;
  double sxx = 0.0, sxy = 0.0, syy = 0.0;
  for (int i = 0; i < count; ++i) {
    const double dx = (double)n_token[i] - mx, dy = seconds[i] - my;
    sxx += dx * dx;
    sxy += dx * dy;
    syy += dy * dy;
  }
  if (!(sxx > 0.0)) return HFX_ERR_MODEL;
  double b = sxy / sxx;
  double a = my - b * mx;
  if (!(b > 0.0)) return HFX_ERR_MODEL;
  if (a < 0.0) a = 0.0;
  model->a = a;
  model->b = b;
  if (r_squared) {
    double sse = 0.0;
    for (int i = 0; i < count; ++i) {
      const double e = seconds[i] - (a + b * (double)n_token[i]);
      sse += e * e;
    }
    *r_squared = syy > 0.0 ? 1.0 - sse / syy : 1.0;
  }
  return HFX_OK;
}

hfx_status hfx_compose_step(double ttft, double tpot, const hfx_latency_model* model, int32_t n_running,
                            const int32_t* running_ctx, int32_t n_waiting, const int32_t* prompt_len,
                            const double* urgency, int32_t mixed, int32_t* admitted, int32_t* kind,
                            int32_t* q_len, int32_t* ctx_len, int32_t* n_step, hfx_decision* decision) {
  if (!n_step || (n_running > 0 && !running_ctx) || (n_waiting > 0 && (!prompt_len || !admitted))) return HFX_ERR_NULL;
  if ((n_running > 0 || n_waiting > 0) && (!kind || !q_len || !ctx_len)) return HFX_ERR_NULL;
  if (n_running < 0 || n_waiting < 0) return HFX_ERR_LEN;
  int64_t budget = 0;
  hfx_status st = hfx_token_budget(ttft, tpot, model, &budget);
  if (st != HFX_OK) return st;
  for (int i = 0; i < n_running; ++i)
    if (running_ctx[i] < 1 || running_ctx[i] == INT32_MAX) return HFX_ERR_LEN;
  for (int i = 0; i < n_waiting; ++i) {
    if (prompt_len[i] < 1) return HFX_ERR_LEN;
    if (urgency && std::isnan(urgency[i])) return HFX_ERR_MODEL;
  }

  // step 3: most urgent first; a request that does not fit is passed over, the scan goes on
  std::vector<int32_t> order((size_t)n_waiting);
  std::iota(order.begin(), order.end(), 0);
  if (urgency)
    std::stable_sort(order.begin(), order.end(), [urgency](int32_t x, int32_t y) { return urgency[x] < urgency[y]; });
  int64_t left = budget, taken = 0;
  std::vector<int32_t> chosen;
  for (int i = 0; i < n_waiting; ++i) admitted[i] = 0;
  for (int32_t w : order) {
    if ((int64_t)prompt_len[w] <= left) {
      admitted[w] = 1;
      chosen.push_back(w);
      left -= prompt_len[w];
      taken += prompt_len[w];
    }
  }

  // the step: with nothing admitted the instance simply decodes on
  int32_t n = 0;
  if (mixed || chosen.empty())
    for (int i = 0; i < n_running; ++i, ++n) {
      kind[n] = HFX_DECODE;
      q_len[n] = 1;
      ctx_len[n] = running_ctx[i] + 1;
    }
  for (int32_t w : chosen) {
    kind[n] = HFX_PREFILL;
    q_len[n] = prompt_len[w];
    ctx_len[n] = prompt_len[w];
    ++n;
  }
  *n_step = n;

  // step 4: the instance's next maturity time
  if (decision) {
    decision->budget = budget;
    decision->n_token = taken;
    decision->e_p = taken > 0 ? model->a + model->b * (double)taken : 0.0;
    decision->k = 0.0;
    decision->maturity = 0.0;
    if (taken > 0) {
      st = hfx_maturity_time(decision->e_p, tpot, model->e_d, &decision->k, &decision->maturity);
      if (st != HFX_OK) return st;
    }
  }
  return HFX_OK;
}

}  // extern "C"
