// State monitor and chunk-size rule of the cloud (paper Sec. 3.2 Eq. 1-2, Sec. 3.3 Eq. 3,
// Sec. 3.5): host code beside the GPU library; see include/hat_sched.h for the contract and
// for how g(.) is kept (a table over fixed knots, linear in between).
#include <cmath>
#include <vector>

#include "../../include/hat_sched.h"

struct hat_sched {
  std::vector<int32_t> knots;
  std::vector<double> g;
  std::vector<char> seen;
  double alpha = 0.8;
  double mu = 0.0;
  bool have_mu = false;
};

namespace {

struct Point { double x, y; };

std::vector<Point> observed(const hat_sched* s) {
  std::vector<Point> p;
  for (size_t k = 0; k < s->knots.size(); ++k)
    if (s->seen[k]) p.push_back({(double)s->knots[k], s->g[k]});
  return p;
}

double eval(const std::vector<Point>& p, double x) {
  if (p.empty()) return 0.0;
  if (p.size() == 1) return p[0].y;
  size_t j = 0;
  while (j + 2 < p.size() && x > p[j + 1].x) ++j;
  return p[j].y + (p[j + 1].y - p[j].y) * (x - p[j].x) / (p[j + 1].x - p[j].x);
}

}  // namespace

extern "C" {

int32_t hat_sched_create(const int32_t* knots, int32_t n_knots, double alpha, hat_sched_t** out) {
  if (out) *out = nullptr;
  if (!out || !knots || n_knots < 1 || !(alpha >= 0.0 && alpha <= 1.0)) return -1;
  for (int32_t k = 0; k < n_knots; ++k)
    if (knots[k] < 0 || (k > 0 && knots[k] <= knots[k - 1])) return -1;
  hat_sched* s = new hat_sched;
  s->knots.assign(knots, knots + n_knots);
  s->g.assign(n_knots, 0.0);
  s->seen.assign(n_knots, 0);
  s->alpha = alpha;
  *out = s;
  return 0;
}

void hat_sched_destroy(hat_sched_t* s) { delete s; }

int32_t hat_sched_observe(hat_sched_t* s, double mu_hat, double eta_hat) {
  if (!s || !std::isfinite(mu_hat) || !std::isfinite(eta_hat) || mu_hat < 0.0 || eta_hat < 0.0) return -1;
  const double a = s->alpha;
  s->mu = s->have_mu ? a * s->mu + (1.0 - a) * mu_hat : mu_hat;
  s->have_mu = true;
  size_t best = 0;
  for (size_t k = 1; k < s->knots.size(); ++k)
    if (std::fabs(s->knots[k] - mu_hat) < std::fabs(s->knots[best] - mu_hat)) best = k;
  s->g[best] = s->seen[best] ? a * s->g[best] + (1.0 - a) * eta_hat : eta_hat;
  s->seen[best] = 1;
  return 0;
}

double hat_sched_mu(const hat_sched_t* s) { return s ? s->mu : 0.0; }

double hat_sched_predict(const hat_sched_t* s, double tokens) {
  if (!s) return 0.0;
  return eval(observed(s), tokens);
}

int32_t hat_sched_chunk_size(const hat_sched_t* s, double bytes_per_token, double beta_up, int32_t pipeline_len,
                             int32_t x_min, int32_t x_max) {
  if (!s || !(bytes_per_token > 0.0) || !(beta_up > 0.0) || pipeline_len < 1 || x_min < 1 || x_max < x_min) return -1;
  const std::vector<Point> p = observed(s);
  const double mu = s->mu, P = (double)pipeline_len;
  const double wait = eval(p, mu);
  // f(X) >= 0 with f(X) = X A / beta - (g(mu) + g(mu + X)) / P, evaluated exactly as the rule states it
  auto ok = [&](int32_t X) { return (double)X * bytes_per_token / beta_up >= (wait + eval(p, mu + X)) / P; };
  // g(mu + X) is linear in X between the observed knots, so on each piece f is linear and its
  // sign change is found in closed form; the integer next to the real root is then settled by
  // evaluating the rule itself (rounding of the division could put the root a hair off).
  const size_t npiece = p.size() < 2 ? 1 : p.size() - 1;
  for (size_t j = 0; j < npiece; ++j) {
    // X range of piece j: mu + X in (p[j].x, p[j+1].x], the first and last pieces open-ended
    double lo_x = (j == 0) ? -INFINITY : p[j].x - mu;
    double hi_x = (j + 1 == npiece) ? INFINITY : p[j + 1].x - mu;
    int32_t Lo = x_min, Hi = x_max;
    if (lo_x >= (double)x_min) Lo = (int32_t)std::floor(lo_x) + 1;   // X > lo_x
    if (hi_x < (double)x_max) Hi = (int32_t)std::floor(hi_x);        // X <= hi_x
    if (Lo > Hi) continue;
    double slope = 0.0, y_at_mu = p.empty() ? 0.0 : p[0].y;          // g(mu + X) = y_at_mu + slope X on this piece
    if (p.size() >= 2) {
      slope = (p[j + 1].y - p[j].y) / (p[j + 1].x - p[j].x);
      y_at_mu = p[j].y + slope * (mu - p[j].x);
    }
    const double c = bytes_per_token / beta_up - slope / P;          // df/dX
    const double rhs = (wait + y_at_mu) / P;                         // f(X) = c X - rhs
    int32_t X;
    if (c > 0.0) {
      const double root = rhs / c;
      if (root > (double)Hi + 1.0) continue;                         // not on this piece
      X = root <= (double)Lo ? Lo : (int32_t)std::ceil(root);
      if (X > Hi) X = Hi;
      while (X > Lo && ok(X - 1)) --X;
      while (X <= Hi && !ok(X)) ++X;
      if (X <= Hi) return X;
    } else {
      // f does not grow with X on this piece: if it holds anywhere here it holds at the left end first
      if (ok(Lo)) return Lo;
      if (c < 0.0) continue;
    }
  }
  return x_max;
}

int32_t hat_sched_parallel_draft_steps(const hat_sched_t* s, double draft_len, double bytes_per_token,
                                       double beta_up, double beta_down, double gamma) {
  if (!s || !(draft_len >= 0.0) || !(bytes_per_token > 0.0) || !(beta_up > 0.0) || !(beta_down > 0.0) || !(gamma > 0.0))
    return -1;
  const double t = draft_len * bytes_per_token / beta_up + eval(observed(s), s->mu) + draft_len * bytes_per_token / beta_down;
  const double steps = std::floor(t / gamma);
  return steps > 0.0 ? (int32_t)std::fmin(steps, 2147483647.0) : 0;   // a count of steps: not below zero
}

}  // extern "C"
