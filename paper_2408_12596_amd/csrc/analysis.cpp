// Offline analysis: per-device speed curves (natural cubic spline, Appendix
// "Cubic Spline Interpolation") and Algorithm 2 ("Optimal Batch Size
// Searching").  Host only, double precision, no device work.
#include "common.h"
#include <algorithm>
#include <cmath>
#include <limits>
#include <vector>

namespace {

// Second derivatives of the natural spline through (x, y): tridiagonal system
// from C2 continuity with zero curvature at both ends, solved by elimination.
std::vector<double> spline_second_derivs(const std::vector<double>& x, const std::vector<double>& y) {
  const int n = (int)x.size() - 1;  // intervals
  std::vector<double> M(n + 1, 0.0);
  if (n < 2) return M;
  std::vector<double> diag(n + 1), rhs(n + 1), upper(n + 1);
  for (int i = 1; i < n; ++i) {
    double h0 = x[i] - x[i - 1], h1 = x[i + 1] - x[i];
    diag[i] = 2.0 * (h0 + h1);
    upper[i] = h1;
    rhs[i] = 6.0 * ((y[i + 1] - y[i]) / h1 - (y[i] - y[i - 1]) / h0);
  }
  for (int i = 2; i < n; ++i) {
    double h0 = x[i] - x[i - 1];
    double w = h0 / diag[i - 1];
    diag[i] -= w * upper[i - 1];
    rhs[i] -= w * rhs[i - 1];
  }
  for (int i = n - 1; i >= 1; --i) {
    double next = (i + 1 < n) ? upper[i] * M[i + 1] : 0.0;
    M[i] = (rhs[i] - next) / diag[i];
  }
  return M;
}

double spline_eval(const std::vector<double>& x, const std::vector<double>& y, const std::vector<double>& M, double q) {
  const int n = (int)x.size() - 1;
  int i = (int)(std::upper_bound(x.begin(), x.end(), q) - x.begin()) - 1;
  i = std::max(0, std::min(i, n - 1));
  double h = x[i + 1] - x[i], t = q - x[i];
  double b = (y[i + 1] - y[i]) / h - h * (2.0 * M[i] + M[i + 1]) / 6.0;
  double c = M[i] / 2.0, d = (M[i + 1] - M[i]) / (6.0 * h);
  return y[i] + b * t + c * t * t + d * t * t * t;
}

int check_curve(const poplar_curve* c) {
  if (!c) return poplar_fail(POPLAR_ERR_INVALID, "curve is null");
  if (c->mbs < 0) return poplar_fail(POPLAR_ERR_INVALID, "negative mbs");
  if (c->mbs == 0) return POPLAR_OK;
  if (c->n_pts < 1 || !c->batch || !c->time) return poplar_fail(POPLAR_ERR_INVALID, "curve needs at least one sample");
  for (int i = 0; i < c->n_pts; ++i)
    if (c->batch[i] < 1 || !(c->time[i] > 0.0)) return poplar_fail(POPLAR_ERR_INVALID, "curve sample %d: batch %d time %g", i, c->batch[i], c->time[i]);
  return POPLAR_OK;
}

// speed[0..mbs]; speed[0] = 0.
void build_speed(const poplar_curve& c, std::vector<double>& speed) {
  speed.assign(c.mbs + 1, 0.0);
  if (c.mbs == 0) return;
  std::vector<std::pair<int, double>> pts;
  for (int i = 0; i < c.n_pts; ++i) pts.push_back({c.batch[i], (double)c.batch[i] / c.time[i]});
  std::stable_sort(pts.begin(), pts.end(), [](const std::pair<int, double>& a, const std::pair<int, double>& b) { return a.first < b.first; });
  std::vector<double> xs, ys;
  for (size_t i = 0; i < pts.size();) {
    size_t j = i;
    double sum = 0.0;
    while (j < pts.size() && pts[j].first == pts[i].first) sum += pts[j++].second;
    xs.push_back((double)pts[i].first);
    ys.push_back(sum / (double)(j - i));
    i = j;
  }
  double ymax = *std::max_element(ys.begin(), ys.end());
  std::vector<double> M;
  if (xs.size() > 1) M = spline_second_derivs(xs, ys);
  for (int b = 1; b <= c.mbs; ++b) {
    double q = std::min(std::max((double)b, xs.front()), xs.back());
    double s = xs.size() == 1 ? ys[0] : spline_eval(xs, ys, M, q);
    speed[b] = std::max(s, 1e-9 * ymax);
  }
}

void build_time(const std::vector<double>& speed, std::vector<double>& tm) {
  tm.assign(speed.size(), 0.0);
  for (size_t b = 1; b < speed.size(); ++b) tm[b] = std::max(tm[b - 1], (double)b / speed[b]);
}

}  // namespace

// Communication volume per device and its time on a given link (Appendix "Analysis of Experiments",
// Appendix "Details about ZeRO"): a collective over P elements moves P elements per device.
extern "C" int poplar_comm_model(int64_t P, int32_t world, int32_t stage, double param_bytes, double grad_bytes,
                                 double bytes_per_second, double* micro_bytes, double* step_bytes, double* total_micro_elements,
                                 double* t_micro, double* t_step) {
  if (P < 0 || world < 1 || stage < 0 || stage > 3) return poplar_fail(POPLAR_ERR_INVALID, "need P >= 0, world >= 1, stage 0..3");
  if (!(param_bytes > 0.0) || !(grad_bytes > 0.0) || !(bytes_per_second > 0.0))
    return poplar_fail(POPLAR_ERR_INVALID, "element sizes and bandwidth must be positive");
  int64_t mp = 0, mg = 0, sp = 0, sg = 0;   // elements per micro-step / per step, parameters / gradients
  if (world > 1) {
    switch (stage) {
      case 0: sg = 2 * P; break;
      case 1: sp = P; sg = 2 * P; break;
      case 2: mg = P; sp = P; break;
      default: mp = 2 * P; mg = P; break;
    }
  }
  const double mb = (double)mp * param_bytes + (double)mg * grad_bytes;
  const double sb = (double)sp * param_bytes + (double)sg * grad_bytes;
  if (micro_bytes) *micro_bytes = mb;
  if (step_bytes) *step_bytes = sb;
  if (total_micro_elements) *total_micro_elements = (double)((mp + mg) * (int64_t)world);
  if (t_micro) *t_micro = mb / bytes_per_second;
  if (t_step) *t_step = sb / bytes_per_second;
  return POPLAR_OK;
}

extern "C" int poplar_speed_curve(const poplar_curve* curve, double* speed) {
  POPLAR_TRY(check_curve(curve));
  if (!speed) return poplar_fail(POPLAR_ERR_INVALID, "speed is null");
  std::vector<double> s;
  build_speed(*curve, s);
  std::copy(s.begin(), s.end(), speed);
  return POPLAR_OK;
}

static int allocate_stage01(int n, const poplar_curve* curves, int64_t gbs, double peak_frac, poplar_alloc* out) {
  std::vector<std::vector<double>> sp(n);
  std::vector<double> speed(n, 0.0);
  double speed_cluster = 0.0;
  for (int i = 0; i < n; ++i) {
    build_speed(curves[i], sp[i]);
    for (int b = 1; b <= curves[i].mbs; ++b) speed[i] = std::max(speed[i], sp[i][b]);
    speed_cluster += speed[i];
  }
  if (!(speed_cluster > 0.0)) return poplar_fail(POPLAR_ERR_INVALID, "no device can run a single sample");
  const double time_optimal = (double)gbs / speed_cluster;
  std::vector<int64_t> gmbs(n);
  int64_t remain = gbs;
  for (int i = 0; i < n; ++i) {
    gmbs[i] = (int64_t)std::floor(time_optimal * speed[i]);
    remain -= gmbs[i];
  }
  while (remain > 0) {
    int best = -1;
    double best_t = std::numeric_limits<double>::infinity();
    for (int i = 0; i < n; ++i) {
      if (!(speed[i] > 0.0)) continue;
      double t = (double)(gmbs[i] + 1) / speed[i];
      if (t < best_t) { best = i; best_t = t; }
    }
    gmbs[best] += 1;
    remain -= 1;
  }
  double T = 0.0, T_steps = 0.0;
  for (int i = 0; i < n; ++i) {
    if (gmbs[i] > std::numeric_limits<int32_t>::max()) return poplar_fail(POPLAR_ERR_INVALID, "gmbs overflows int32");
    out->gmbs[i] = (int32_t)gmbs[i];
    if (gmbs[i] == 0) { out->b[i] = out->gas[i] = out->lbs[i] = 0; continue; }
    int64_t top = 1;
    for (int b = 1; b <= curves[i].mbs; ++b)
      if (sp[i][b] >= peak_frac * speed[i]) top = b;
    int64_t bi = std::min(gmbs[i], top);
    int64_t gi = (gmbs[i] + bi - 1) / bi;
    out->b[i] = (int32_t)bi;
    out->gas[i] = (int32_t)gi;
    out->lbs[i] = (int32_t)(gmbs[i] - (gi - 1) * bi);
    T = std::max(T, (double)gmbs[i] / speed[i]);
    const int64_t li = gmbs[i] - (gi - 1) * bi;
    T_steps = std::max(T_steps, (double)(gi - 1) * ((double)bi / sp[i][bi]) + (double)li / sp[i][li]);
  }
  out->T = T;
  out->T_steps = T_steps;
  out->t = time_optimal;
  return POPLAR_OK;
}

static int allocate_stage23(int n, const poplar_curve* curves, int64_t gbs, double t_comm, poplar_alloc* out) {
  std::vector<std::vector<double>> tm(n);
  std::vector<double> cand;
  for (int i = 0; i < n; ++i) {
    std::vector<double> sp;
    build_speed(curves[i], sp);
    build_time(sp, tm[i]);
    for (size_t b = 1; b < tm[i].size(); ++b) cand.push_back(tm[i][b]);
  }
  std::sort(cand.begin(), cand.end());
  cand.erase(std::unique(cand.begin(), cand.end()), cand.end());
  bool have = false;
  double best_wall = 0.0, best_t = 0.0;
  int64_t best_gas = 0;
  std::vector<int> best_b(n, 0), bs(n);
  for (double t : cand) {
    int64_t mb = 0;
    for (int i = 0; i < n; ++i) {
      int k = 0;
      while (k + 1 < (int)tm[i].size() && tm[i][k + 1] <= t) ++k;
      bs[i] = k;
      mb += k;
    }
    if (mb == 0) continue;
    int64_t gas = (gbs + mb - 1) / mb;
    double wall = (t + t_comm) * (double)gas;
    if (!have || wall < best_wall) { have = true; best_wall = wall; best_t = t; best_gas = gas; best_b = bs; }
  }
  if (!have) return poplar_fail(POPLAR_ERR_INVALID, "no device can run a single sample");
  if (best_gas > std::numeric_limits<int32_t>::max()) return poplar_fail(POPLAR_ERR_INVALID, "gas overflows int32");
  int64_t mb = 0;
  for (int i = 0; i < n; ++i) mb += best_b[i];
  int64_t R = gbs - (best_gas - 1) * mb;
  std::vector<int> lbs(n, 0);
  for (int64_t k = 0; k < R; ++k) {
    int pick = -1;
    double pick_t = std::numeric_limits<double>::infinity();
    for (int i = 0; i < n; ++i)
      if (lbs[i] < best_b[i] && tm[i][lbs[i] + 1] < pick_t) { pick = i; pick_t = tm[i][lbs[i] + 1]; }
    lbs[pick] += 1;
  }
  for (int i = 0; i < n; ++i) {
    out->b[i] = best_b[i];
    out->gas[i] = (int32_t)best_gas;
    out->lbs[i] = lbs[i];
    int64_t g = (best_gas - 1) * best_b[i] + lbs[i];
    if (g > std::numeric_limits<int32_t>::max()) return poplar_fail(POPLAR_ERR_INVALID, "gmbs overflows int32");
    out->gmbs[i] = (int32_t)g;
  }
  out->T = best_wall;
  out->T_steps = best_wall;
  out->t = best_t;
  return POPLAR_OK;
}

extern "C" int poplar_allocate(int32_t stage, int32_t n_dev, const poplar_curve* curves, int64_t gbs,
                               double time_communication, double peak_frac, poplar_alloc* out) {
  if (stage < 0 || stage > 3) return poplar_fail(POPLAR_ERR_INVALID, "stage %d outside 0..3", stage);
  if (n_dev < 1 || !curves) return poplar_fail(POPLAR_ERR_INVALID, "need at least one device curve");
  if (gbs < 1) return poplar_fail(POPLAR_ERR_INVALID, "gbs must be positive");
  if (!out || !out->gmbs || !out->b || !out->gas || !out->lbs) return poplar_fail(POPLAR_ERR_INVALID, "output arrays missing");
  if (!(peak_frac > 0.0 && peak_frac <= 1.0)) return poplar_fail(POPLAR_ERR_INVALID, "peak_frac must be in (0, 1]");
  if (!(time_communication >= 0.0)) return poplar_fail(POPLAR_ERR_INVALID, "time_communication must be >= 0");
  for (int i = 0; i < n_dev; ++i) POPLAR_TRY(check_curve(&curves[i]));
  if (stage <= 1) return allocate_stage01(n_dev, curves, gbs, peak_frac, out);
  return allocate_stage23(n_dev, curves, gbs, time_communication, out);
}
