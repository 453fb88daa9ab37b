// Host-side Lloyd-Max codebook construction (eq. (4) of the paper) for the
// coordinate density of Lemma 1,
//     f_X(x) = Gamma(d/2) / (sqrt(pi) Gamma((d-1)/2)) * (1 - x^2)^((d-3)/2).
//
// All integrals are taken in the angle t = asin(x): f_X(x) dx becomes
// C cos^(d-2)(t) dt, which is smooth on the closed interval for every d >= 3,
// and are evaluated by composite 16-point Gauss-Legendre quadrature on panels
// no wider than one standard deviation (1/sqrt(d)).  The first moment has the
// closed form  -C/(d-1) (1-x^2)^((d-1)/2).  fp64 throughout; the results are
// rounded to fp32 once at the end.
#include <cmath>
#include <cstdint>
#include <vector>

#include "../../include/turboquant.h"

namespace {

constexpr int kGL = 16;

struct GaussLegendre {
  double node[kGL];
  double weight[kGL];
  GaussLegendre() {
    // roots of the Legendre polynomial P_16 by Newton iteration from the
    // Chebyshev-like first guess; weights 2 / ((1 - x^2) P'_n(x)^2)
    const double pi = 3.14159265358979323846;
    for (int i = 0; i < kGL; ++i) {
      double x = std::cos(pi * (i + 0.75) / (kGL + 0.5));
      double dp = 0.0;
      for (int it = 0; it < 100; ++it) {
        double p0 = 1.0, p1 = x;
        for (int k = 2; k <= kGL; ++k) {
          double pk = ((2.0 * k - 1.0) * x * p1 - (k - 1.0) * p0) / k;
          p0 = p1;
          p1 = pk;
        }
        dp = kGL * (x * p1 - p0) / (x * x - 1.0);
        double dx = p1 / dp;
        x -= dx;
        if (std::fabs(dx) < 1e-16) break;
      }
      node[i] = x;
      weight[i] = 2.0 / ((1.0 - x * x) * dp * dp);
    }
  }
};

struct CoordLaw {
  int d;
  double log_c;    // log of the normalising constant of Lemma 1
  double sigma;    // 1/sqrt(d)
  double t_clip;   // |angle| beyond which the density is below 1e-40 of its peak
  GaussLegendre gl;

  explicit CoordLaw(int dim) : d(dim) {
    log_c = std::lgamma(0.5 * d) - 0.5 * std::log(3.14159265358979323846) -
            std::lgamma(0.5 * (d - 1));
    sigma = 1.0 / std::sqrt((double)d);
    const double half_pi = 1.57079632679489661923;
    t_clip = std::fmin(half_pi, 14.0 * sigma);
  }

  // moments 0 and 2 of f_X over x in [lo, hi]
  void moments02(double lo, double hi, double* m0, double* m2) const {
    double a = std::asin(std::fmax(-1.0, lo)), b = std::asin(std::fmin(1.0, hi));
    a = std::fmax(a, -t_clip);
    b = std::fmin(b, t_clip);
    *m0 = 0.0;
    *m2 = 0.0;
    if (!(b > a)) return;
    int panels = (int)std::ceil((b - a) / sigma);
    if (panels < 1) panels = 1;
    const double h = (b - a) / panels;
    double s0 = 0.0, s2 = 0.0;
    for (int p = 0; p < panels; ++p) {
      const double mid = a + (p + 0.5) * h;
      for (int i = 0; i < kGL; ++i) {
        const double t = mid + 0.5 * h * gl.node[i];
        const double ct = std::cos(t);
        double w = 0.0;
        if (ct > 0.0) w = std::exp(log_c + (d - 2.0) * std::log(ct));
        w *= gl.weight[i];
        const double st = std::sin(t);
        s0 += w;
        s2 += w * st * st;
      }
    }
    *m0 = 0.5 * h * s0;
    *m2 = 0.5 * h * s2;
  }

  // first moment of f_X over [lo, hi], closed form
  double moment1(double lo, double hi) const {
    auto g = [this](double x) {
      const double u = 1.0 - x * x;
      if (u <= 0.0) return 0.0;
      return std::exp(log_c - std::log(d - 1.0) + 0.5 * (d - 1.0) * std::log(u));
    };
    return g(lo) - g(hi);
  }
};

}  // namespace

extern "C" tq_status tq_build_codebook(int32_t d, int32_t bits, float* centroids, float* bounds,
                                       double* cost_per_coord) {
  if (d < 3 || bits < 0 || bits > 8 || centroids == nullptr) return TQ_ERR_INVALID_ARG;
  if (bits > 0 && bounds == nullptr) return TQ_ERR_INVALID_ARG;
  const int K = 1 << bits;
  if (K == 1) {
    centroids[0] = 0.0f;
    if (cost_per_coord) *cost_per_coord = 1.0 / d;  // E[X^2] of a unit vector's coordinate
    return TQ_OK;
  }
  const CoordLaw law(d);
  std::vector<double> c(K), cn(K), edge(K + 1), m0(K), m1(K), m2(K);
  // evenly spaced start inside the bulk of the law; Lloyd's iteration has a
  // single fixed point for a log-concave density, so the start only sets speed
  const double span = std::fmin(0.95, 3.0 * law.sigma);
  for (int k = 0; k < K; ++k) c[k] = span * (-1.0 + (2.0 * k + 1.0) / K);

  auto cells = [&](const std::vector<double>& cc) {
    edge[0] = -1.0;
    edge[K] = 1.0;
    for (int k = 1; k < K; ++k) edge[k] = 0.5 * (cc[k - 1] + cc[k]);  // Voronoi: midpoints
    for (int k = 0; k < K; ++k) {
      law.moments02(edge[k], edge[k + 1], &m0[k], &m2[k]);
      m1[k] = law.moment1(edge[k], edge[k + 1]);
    }
  };

  // stop when the update is below 1e-13 sigma, or when it has stopped shrinking
  // (rounding noise of the quadrature sets a floor that grows slowly with d)
  const int max_iter = 2000000;
  double best_delta = 1e300;
  int since_best = 0;
  for (int it = 0; it < max_iter; ++it) {
    cells(c);
    double delta = 0.0;
    for (int k = 0; k < K; ++k) cn[k] = (m0[k] > 0.0) ? m1[k] / m0[k] : c[k];
    for (int k = 0; k < K / 2; ++k) {  // the law is even: keep the codebook antisymmetric
      const double v = 0.5 * (cn[K - 1 - k] - cn[k]);
      cn[k] = -v;
      cn[K - 1 - k] = v;
    }
    for (int k = 0; k < K; ++k) delta = std::fmax(delta, std::fabs(cn[k] - c[k]));
    c.swap(cn);
    if (delta < 1e-13 * law.sigma) break;
    if (delta < 0.5 * best_delta) {
      best_delta = delta;
      since_best = 0;
    } else if (++since_best > 2000 && best_delta < 1e-10 * law.sigma) {
      break;
    }
  }
  cells(c);
  double cost = 0.0;
  for (int k = 0; k < K; ++k) cost += m2[k] - 2.0 * c[k] * m1[k] + c[k] * c[k] * m0[k];
  for (int k = 0; k < K; ++k) centroids[k] = (float)c[k];
  for (int k = 0; k + 1 < K; ++k) bounds[k] = (float)(0.5 * (c[k] + c[k + 1]));
  if (cost_per_coord) *cost_per_coord = cost;
  return TQ_OK;
}

extern "C" tq_status tq_bucket_masses(int32_t d, int32_t bits, const float* centroids, double* p) {
  if (d < 3 || bits < 0 || bits > 8 || centroids == nullptr || p == nullptr) return TQ_ERR_INVALID_ARG;
  const int K = 1 << bits;
  const CoordLaw law(d);
  double total = 0.0;
  for (int k = 0; k < K; ++k) {
    if (k > 0 && !(centroids[k] > centroids[k - 1])) return TQ_ERR_INVALID_ARG;
    const double lo = k == 0 ? -1.0 : 0.5 * ((double)centroids[k - 1] + (double)centroids[k]);
    const double hi = k == K - 1 ? 1.0 : 0.5 * ((double)centroids[k] + (double)centroids[k + 1]);
    double m2;
    law.moments02(lo, hi, &p[k], &m2);
    total += p[k];
  }
  for (int k = 0; k < K; ++k) p[k] /= total;  // the quadrature leaves 1e-15; the clipped far tails 1e-40
  return TQ_OK;
}
