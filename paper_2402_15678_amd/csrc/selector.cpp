// Adaptive speculation length selector (paper section 3.3): host-side bookkeeping between verification
// steps.  Every step contributes one sample t_LLM / vl (verification time over the average number of
// tokens a request gained from it, the quantity equation s_optimal minimises).  Once
// decision_threshold samples have been collected since the last change of s, a straight line is fitted
// to them by least squares: a rising trend means the last change went past the optimum and s is
// lowered by s_penalty, otherwise s is raised by s_reward; the samples are then discarded.
#include "../../include/minions_verify.h"

#include <cmath>
#include <new>
#include <vector>

struct mn_selector {
  int s, s_min, s_max, decision_threshold, s_penalty, s_reward;
  std::vector<double> samples;
  long adjustments;
};

extern "C" mn_status mn_selector_create(mn_selector** out, int s_init, int s_min, int s_max, int decision_threshold,
                                        int s_penalty, int s_reward) {
  if (!out) return MN_ENULL;
  *out = nullptr;
  if (s_min < 0 || s_max < s_min || s_init < s_min || s_init > s_max) return MN_EINVAL;
  if (decision_threshold < 2 || s_penalty < 0 || s_reward < 0) return MN_EINVAL;
  mn_selector* p = new (std::nothrow) mn_selector();
  if (!p) return MN_ECAPACITY;
  p->s = s_init;
  p->s_min = s_min;
  p->s_max = s_max;
  p->decision_threshold = decision_threshold;
  p->s_penalty = s_penalty;
  p->s_reward = s_reward;
  p->adjustments = 0;
  *out = p;
  return MN_OK;
}

extern "C" void mn_selector_destroy(mn_selector* p) { delete p; }

extern "C" int mn_selector_current(const mn_selector* p) { return p ? p->s : -1; }

extern "C" long mn_selector_adjustments(const mn_selector* p) { return p ? p->adjustments : -1; }

// slope of the least-squares line through (0, y_0) .. (m-1, y_{m-1}), m >= 2
static double fit_slope(const std::vector<double>& y) {
  const size_t m = y.size();
  double xm = 0.0, ym = 0.0;
  for (size_t i = 0; i < m; ++i) {
    xm += (double)i;
    ym += y[i];
  }
  xm /= (double)m;
  ym /= (double)m;
  double sxy = 0.0, sxx = 0.0;
  for (size_t i = 0; i < m; ++i) {
    const double dx = (double)i - xm;
    sxy += dx * (y[i] - ym);
    sxx += dx * dx;
  }
  return sxy / sxx;
}

extern "C" mn_status mn_selector_observe(mn_selector* p, double t_llm, double vl, int* s_out, double* slope_out) {
  if (!p) return MN_ENULL;
  if (slope_out) *slope_out = std::nan("");
  if (s_out) *s_out = p->s;
  if (!(t_llm >= 0.0) || !(vl > 0.0) || !std::isfinite(t_llm) || !std::isfinite(vl)) return MN_EINVAL;
  p->samples.push_back(t_llm / vl);
  if ((int)p->samples.size() >= p->decision_threshold) {
    const double slope = fit_slope(p->samples);
    int s = p->s;
    if (slope > 0.0) s -= p->s_penalty;
    else s += p->s_reward;
    if (s < p->s_min) s = p->s_min;
    if (s > p->s_max) s = p->s_max;
    p->s = s;
    p->samples.clear();
    ++p->adjustments;
    if (slope_out) *slope_out = slope;
  }
  if (s_out) *s_out = p->s;
  return MN_OK;
}
