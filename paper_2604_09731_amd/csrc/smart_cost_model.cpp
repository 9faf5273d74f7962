// Device cost models of the paper's Sec. 3.1 ("Cost Modeling") on the host:
//   C_draft(x)  = lambda x                              (Eq. "linear_model", beta = 0)
//   C_verify(x) = gamma (exp(delta x^rho) - 1)          (Eq. "exp_model", eta = 0)
// fitted to a handful of timed forward passes, and the cost / marginal-cost tables
// (Eq. "marginal_cost") that smart_select_tree takes.
//
// The fit is least squares.  For fixed (delta, rho) the best gamma is a ratio of two
// sums, which leaves a two-dimensional search; it runs over rho and over
// s = delta * x_max^rho (the exponent at the largest sample), so it does not depend
// on the units of x: a coarse grid, then
// a Levenberg-Marquardt iteration from the best cell.
#include <math.h>
#include <stdint.h>

#include <algorithm>
#include <limits>
#include <vector>

#include "smart_tree.h"

namespace {

struct Samples {
  const double* x;
  const double* t;
  int n;
  double x_max;
};

// sum of squared residuals at (rho, log s) with the best gamma; also returns that gamma
double reduced_sse(const Samples& S, double rho, double log_s, double* gamma_out) {
  const double s = exp(log_s);
  double ff = 0.0, ft = 0.0, tt = 0.0;
  for (int i = 0; i < S.n; ++i) {
    const double f = expm1(s * pow(S.x[i] / S.x_max, rho));
    ff += f * f;
    ft += f * S.t[i];
    tt += S.t[i] * S.t[i];
  }
  if (!(ff > 0.0) || !std::isfinite(ff)) {
    if (gamma_out) *gamma_out = 0.0;
    return std::numeric_limits<double>::infinity();
  }
  const double gamma = ft / ff;
  if (gamma_out) *gamma_out = gamma;
  double sse = 0.0;
  for (int i = 0; i < S.n; ++i) {
    const double r = gamma * expm1(s * pow(S.x[i] / S.x_max, rho)) - S.t[i];
    sse += r * r;
  }
  (void)tt;
  return sse;
}

constexpr double kRhoLo = 0.05, kRhoHi = 4.0;
constexpr double kLogSLo = -13.815510557964274 /* log 1e-6 */, kLogSHi = 3.6888794541139363 /* log 40 */;

}  // namespace

extern "C" int32_t smart_cost_tables_biased(double lambda, double beta, double gamma, double delta, double rho,
                                            double eta, double c_T, double tokens_per_node,
                                            int32_t undrafted_nodes, int32_t n_max, double* h_cost,
                                            double* h_dcost) {
  if (!h_cost || n_max < 0 || undrafted_nodes < 0 || !(c_T > 0.0) || !(tokens_per_node > 0.0) || !(rho > 0.0) ||
      !(delta >= 0.0) || !(gamma >= 0.0) || !(lambda >= 0.0) || !(beta >= 0.0) || !(eta >= 0.0) ||
      !std::isfinite(beta) || !std::isfinite(eta))
    return SMART_EINVAL;
  auto tokens = [&](int n) { return tokens_per_node * (double)(n > undrafted_nodes ? n - undrafted_nodes : 0); };
  for (int n = 0; n <= n_max + 1; ++n) {
    const double x = tokens(n);
    h_cost[n] = (lambda * x + gamma * expm1(delta * pow(x, rho)) + beta + eta) / c_T;
  }
  if (h_dcost) {
    for (int n = 0; n <= n_max; ++n) {
      const double x = tokens(n);
      if (x == 0.0 && rho < 1.0)
        h_dcost[n] = std::numeric_limits<double>::infinity();
      else
        h_dcost[n] = tokens_per_node * (lambda + gamma * delta * rho * pow(x, rho - 1.0) * exp(delta * pow(x, rho))) / c_T;
    }
  }
  return SMART_OK;
}

extern "C" int32_t smart_cost_tables(double lambda, double gamma, double delta, double rho, double c_T,
                                     double tokens_per_node, int32_t n_max, double* h_cost,
                                     double* h_dcost) {
  return smart_cost_tables_biased(lambda, 0.0, gamma, delta, rho, 0.0, c_T, tokens_per_node, 0, n_max, h_cost, h_dcost);
}

extern "C" int32_t smart_fit_cost_models(int32_t n_points, const double* h_x, const double* h_t_draft,
                                         const double* h_t_verify, double* h_lambda, double* h_gamma,
                                         double* h_delta, double* h_rho, double* h_sse) {
  if (n_points < 1 || !h_x) return SMART_EINVAL;
  if (!h_t_draft && !h_t_verify) return SMART_EINVAL;
  if (h_t_draft && !h_lambda) return SMART_EINVAL;
  if (h_t_verify && (!h_gamma || !h_delta || !h_rho)) return SMART_EINVAL;
  double x_max = 0.0;
  for (int i = 0; i < n_points; ++i) {
    if (!(h_x[i] > 0.0) || !std::isfinite(h_x[i])) return SMART_EINVAL;
    x_max = std::max(x_max, h_x[i]);
  }
  if (h_t_draft) {  // line through the origin
    double xx = 0.0, xt = 0.0;
    for (int i = 0; i < n_points; ++i) {
      if (!std::isfinite(h_t_draft[i])) return SMART_EINVAL;
      xx += h_x[i] * h_x[i];
      xt += h_x[i] * h_t_draft[i];
    }
    *h_lambda = xt / xx;
  }
  if (!h_t_verify) return SMART_OK;
  if (n_points < 3) return SMART_EINVAL;  // three parameters
  for (int i = 0; i < n_points; ++i)
    if (!std::isfinite(h_t_verify[i])) return SMART_EINVAL;
  const Samples S{h_x, h_t_verify, n_points, x_max};
  // coarse grid
  const int NR = 80, NS = 120;
  double best = std::numeric_limits<double>::infinity(), rho = 1.0, ls = 0.0;
  for (int i = 0; i < NR; ++i) {
    const double r = kRhoLo + (kRhoHi - kRhoLo) * i / (NR - 1);
    for (int j = 0; j < NS; ++j) {
      const double l = kLogSLo + (kLogSHi - kLogSLo) * j / (NS - 1);
      const double v = reduced_sse(S, r, l, nullptr);
      if (v < best) { best = v; rho = r; ls = l; }
    }
  }
  if (!std::isfinite(best)) return SMART_EINVAL;
  // Levenberg-Marquardt on the two remaining parameters (gamma is projected out at every
  // evaluation), Jacobian by central differences.
  std::vector<double> r0(n_points), rp(n_points), rm(n_points), J(2 * (size_t)n_points);
  auto residuals = [&](double r, double l, std::vector<double>& out) {
    double g;
    const double v = reduced_sse(S, r, l, &g);
    const double s = exp(l);
    for (int i = 0; i < n_points; ++i) out[i] = g * expm1(s * pow(h_x[i] / x_max, r)) - h_t_verify[i];
    return v;
  };
  double mu = 1e-3;
  for (int it = 0; it < 400; ++it) {
    residuals(rho, ls, r0);
    const double hr = 1e-6, hl = 1e-6;
    residuals(rho + hr, ls, rp);
    residuals(rho - hr, ls, rm);
    for (int i = 0; i < n_points; ++i) J[2 * i] = (rp[i] - rm[i]) / (2 * hr);
    residuals(rho, ls + hl, rp);
    residuals(rho, ls - hl, rm);
    for (int i = 0; i < n_points; ++i) J[2 * i + 1] = (rp[i] - rm[i]) / (2 * hl);
    double a00 = 0, a01 = 0, a11 = 0, g0 = 0, g1 = 0;
    for (int i = 0; i < n_points; ++i) {
      a00 += J[2 * i] * J[2 * i];
      a01 += J[2 * i] * J[2 * i + 1];
      a11 += J[2 * i + 1] * J[2 * i + 1];
      g0 += J[2 * i] * r0[i];
      g1 += J[2 * i + 1] * r0[i];
    }
    bool moved = false;
    for (int tries = 0; tries < 40 && !moved; ++tries) {
      const double b00 = a00 * (1 + mu) + 1e-300, b11 = a11 * (1 + mu) + 1e-300;
      const double det = b00 * b11 - a01 * a01;
      if (!(det > 0.0) || !std::isfinite(det)) { mu *= 10; continue; }
      const double dr = -(b11 * g0 - a01 * g1) / det, dl = -(b00 * g1 - a01 * g0) / det;
      const double r_new = std::min(kRhoHi, std::max(kRhoLo, rho + dr));
      const double l_new = std::min(kLogSHi, std::max(kLogSLo, ls + dl));
      const double v = reduced_sse(S, r_new, l_new, nullptr);
      if (v < best) {
        moved = true;
        const double gain = best - v;
        best = v; rho = r_new; ls = l_new;
        mu = std::max(mu * 0.3, 1e-12);
        if (gain <= 1e-16 * (best + 1e-300) && fabs(dr) < 1e-12 && fabs(dl) < 1e-12) it = 1 << 30;
      } else {
        mu *= 10;
      }
    }
    if (!moved) break;
    if (it >= (1 << 30)) break;
  }
  double gamma = 0.0;
  best = reduced_sse(S, rho, ls, &gamma);
  *h_gamma = gamma;
  *h_rho = rho;
  *h_delta = exp(ls) / pow(x_max, rho);
  if (h_sse) *h_sse = best;
  return SMART_OK;
}
