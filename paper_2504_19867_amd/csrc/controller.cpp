// SLO-aware partition adjuster (host logic, no GPU work).
//
// Paper, "Dynamic Adjusting Method": Algorithm 1 raises the share of the phase whose observed
// latency misses its objective, guided by the latency models of Eq. 4 (whose shape follows from
// Eq. 1, latency inversely proportional to the share, and the M/M/1 waiting time of Eq. 2-3).
// The repairs to the printed listing and the choices the paper leaves open are stated with the
// declarations in semipd.h.
#include "semipd.h"

#include <math.h>

#include <algorithm>
#include <limits>
#include <mutex>
#include <new>
#include <vector>

namespace {
struct Point { double share, latency; };
struct Line { double a, b, sse; };

// least squares latency = a u + b over the points' regressors u
Line fit_line(const std::vector<double>& u, const std::vector<Point>& pts) {
  const size_t n = pts.size();
  double mu = 0.0, mv = 0.0;
  for (size_t i = 0; i < n; ++i) mu += u[i];
  for (size_t i = 0; i < n; ++i) mv += pts[i].latency;
  mu /= (double)n;
  mv /= (double)n;
  double suu = 0.0, suv = 0.0;
  for (size_t i = 0; i < n; ++i) suu += (u[i] - mu) * (u[i] - mu);
  for (size_t i = 0; i < n; ++i) suv += (u[i] - mu) * (pts[i].latency - mv);
  Line l;
  l.a = suv / suu;
  l.b = mv - l.a * mu;
  l.sse = 0.0;
  for (size_t i = 0; i < n; ++i) {
    const double r = l.a * u[i] + l.b - pts[i].latency;
    l.sse += r * r;
  }
  return l;
}

bool one_share_only(const std::vector<Point>& pts) {
  for (const Point& p : pts)
    if (p.share != pts[0].share) return false;
  return true;
}

// nearest rank: the smallest sample with at least p percent of the samples at or below it
double percentile(std::vector<double>& w, double p) {
  std::sort(w.begin(), w.end());
  long k = (long)ceil(p / 100.0 * (double)w.size());
  if (k < 1) k = 1;
  return w[(size_t)k - 1];
}
}  // namespace

struct spd_ctrl {
  spd_ctrl_config cfg;
  std::mutex mu;
  std::vector<double> win_ttft, win_tpot;
  std::vector<Point> pts_ttft, pts_tpot;        // one point per closed window, latest last
  double a1 = 0.0, lambda = 0.0, b1 = 0.0, a2 = 0.0, b2 = 0.0;

  void refit() {
    std::vector<double> u;
    if (one_share_only(pts_tpot)) {             // Eq. 1 alone
      a2 = pts_tpot.back().latency * pts_tpot.back().share;
      b2 = 0.0;
    } else {
      u.resize(pts_tpot.size());
      for (size_t i = 0; i < u.size(); ++i) u[i] = 1.0 / pts_tpot[i].share;
      const Line l = fit_line(u, pts_tpot);
      a2 = l.a;
      b2 = l.b;
    }
    if (one_share_only(pts_ttft)) {
      a1 = pts_ttft.back().latency * pts_ttft.back().share;
      lambda = 0.0;
      b1 = 0.0;
    } else {
      double lowest = pts_ttft[0].share;
      for (const Point& p : pts_ttft) lowest = std::min(lowest, p.share);
      u.resize(pts_ttft.size());
      bool have = false;
      double best_sse = 0.0;
      for (int cand = 0; (double)cand < lowest; ++cand) {
        for (size_t i = 0; i < u.size(); ++i) u[i] = 1.0 / (pts_ttft[i].share - (double)cand);
        const Line l = fit_line(u, pts_ttft);
        if (!have || l.sse < best_sse - 1e-12 * (1.0 + best_sse)) {
          have = true;
          best_sse = l.sse;
          a1 = l.a;
          lambda = (double)cand;
          b1 = l.b;
        }
      }
    }
  }
  double est_ttft(double x) const {             // Eq. 4; at or below lambda the queue never drains
    return x <= lambda ? std::numeric_limits<double>::infinity() : a1 / (x - lambda) + b1;
  }
  double est_tpot(double y) const { return a2 / y + b2; }
};

extern "C" int spd_ctrl_create(const spd_ctrl_config* cfg, spd_ctrl** out) {
  if (!cfg || !out) return SPD_EINVAL;
  if (!(cfg->slo_ttft > 0.0) || !(cfg->slo_tpot > 0.0) || !isfinite(cfg->slo_ttft) || !isfinite(cfg->slo_tpot)) return SPD_EINVAL;
  if (!(cfg->p_slo > 0.0) || !(cfg->p_slo <= 100.0)) return SPD_EINVAL;
  if (cfg->window_size <= 0 || cfg->max_step <= 0 || cfg->step_size <= 0 || cfg->step_size > 50 || cfg->history < 1)
    return SPD_EINVAL;
  spd_ctrl* c = new (std::nothrow) spd_ctrl();
  if (!c) return SPD_EINVAL;
  c->cfg = *cfg;
  *out = c;
  return SPD_OK;
}

extern "C" int spd_ctrl_destroy(spd_ctrl* c) {
  if (!c) return SPD_EINVAL;
  delete c;
  return SPD_OK;
}

extern "C" int spd_ctrl_observe_ttft(spd_ctrl* c, double latency) {
  if (!c || !isfinite(latency) || latency < 0.0) return SPD_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  c->win_ttft.push_back(latency);
  return SPD_OK;
}

extern "C" int spd_ctrl_observe_tpot(spd_ctrl* c, double latency) {
  if (!c || !isfinite(latency) || latency < 0.0) return SPD_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  c->win_tpot.push_back(latency);
  return SPD_OK;
}

extern "C" int spd_ctrl_step(spd_ctrl* c, int64_t iter, int32_t x0, int32_t y0, int32_t* x_out, int32_t* y_out) {
  if (!c || !x_out || !y_out || iter < 0) return SPD_EINVAL;
  const int32_t ss = c->cfg.step_size;
  if (x0 < ss || x0 > 100 || y0 < ss || y0 > 100) return SPD_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  *x_out = x0;
  *y_out = y0;
  if (iter % c->cfg.window_size > 0) return SPD_OK;
  const bool empty = c->win_ttft.empty() || c->win_tpot.empty();
  double ttft = 0.0, tpot = 0.0;
  if (!empty) {
    ttft = percentile(c->win_ttft, c->cfg.p_slo);
    tpot = percentile(c->win_tpot, c->cfg.p_slo);
  }
  c->win_ttft.clear();
  c->win_tpot.clear();
  if (empty) return SPD_OK;
  c->pts_ttft.push_back(Point{(double)x0, ttft});
  c->pts_tpot.push_back(Point{(double)y0, tpot});
  if ((int64_t)c->pts_ttft.size() > c->cfg.history) c->pts_ttft.erase(c->pts_ttft.begin());
  if ((int64_t)c->pts_tpot.size() > c->cfg.history) c->pts_tpot.erase(c->pts_tpot.begin());
  c->refit();
  const bool ttft_fails = ttft > c->cfg.slo_ttft, tpot_fails = tpot > c->cfg.slo_tpot;
  if (ttft_fails == tpot_fails) return SPD_OK;  // both fail: no room to move; both pass: nothing to do
  // the failing phase is `up`, the other one `dn`
  int32_t up = ttft_fails ? x0 : y0, dn = ttft_fails ? y0 : x0;
  for (int step = 0; step < c->cfg.max_step; ++step) {
    const double share = 100.0 * (double)up / (double)(up + dn);
    const double est = ttft_fails ? c->est_ttft(share) : c->est_tpot(share);
    if (!(est > (ttft_fails ? c->cfg.slo_ttft : c->cfg.slo_tpot))) break;
    if (up + ss <= 100) up += ss;
    else dn = std::max(ss, dn - ss);
  }
  *x_out = ttft_fails ? up : dn;
  *y_out = ttft_fails ? dn : up;
  return SPD_OK;
}

extern "C" int spd_ctrl_model(spd_ctrl* c, double* out) {
  if (!c || !out) return SPD_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  out[0] = c->a1; out[1] = c->lambda; out[2] = c->b1; out[3] = c->a2; out[4] = c->b2;
  return SPD_OK;
}
