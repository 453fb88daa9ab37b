// Host-side construction of the global parameters that need no GPU: the
// random rotation of Sec. 3.1 (orthogonal factor of a QR decomposition of a
// Gaussian matrix) and the block-diagonal parameter matrices of two instances
// over a channel split (Sec. 4.3).  fp64 inside, run once per (d, b), off the
// timed path.
#include <atomic>
#include <cmath>
#include <cstring>
#include <thread>
#include <vector>

#include "../../include/turboquant.h"

namespace {

// w[0..len) -= 2 (v . w) v   for a unit vector v: the reflection I - 2 v v^T
inline void reflect(const double* v, double* w, int64_t len) {
  double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
  int64_t i = 0;
  for (; i + 4 <= len; i += 4) {
    s0 += v[i] * w[i];
    s1 += v[i + 1] * w[i + 1];
    s2 += v[i + 2] * w[i + 2];
    s3 += v[i + 3] * w[i + 3];
  }
  for (; i < len; ++i) s0 += v[i] * w[i];
  const double s = 2.0 * ((s0 + s1) + (s2 + s3));
  for (i = 0; i < len; ++i) w[i] -= s * v[i];
}

// Turns row k of `a` (entries k..d-1: column k of the matrix being factorised,
// below and on the diagonal) into the unit vector of the Householder
// reflection that maps it to R_kk e_1, and returns R_kk.
double make_reflector(double* x, int64_t len) {
  double ss = 0.0;
  for (int64_t i = 0; i < len; ++i) ss += x[i] * x[i];
  const double nx = std::sqrt(ss);
  if (nx == 0.0) return 0.0;  // a zero column: H = I (v = 0)
  const double alpha = x[0] >= 0.0 ? -nx : nx;
  x[0] -= alpha;
  // |v|^2 = |x|^2 - 2 alpha x0 + alpha^2 with the old x0; recomputed plainly
  double vv = 0.0;
  for (int64_t i = 0; i < len; ++i) vv += x[i] * x[i];
  const double inv = 1.0 / std::sqrt(vv);
  for (int64_t i = 0; i < len; ++i) x[i] *= inv;
  return alpha;
}

}  // namespace

extern "C" {

tq_status tq_build_rotation(int32_t d, const double* gaussian, float* Pi) {
  if (d <= 0 || gaussian == nullptr || Pi == nullptr) return TQ_ERR_INVALID_ARG;
  if (d > 16384) return TQ_ERR_UNSUPPORTED;
  const int64_t n = d;
  // a[j] = column j of the input: every reflection then works on contiguous memory
  std::vector<double> a((size_t)n * n);
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j < n; ++j) a[(size_t)j * n + i] = gaussian[(size_t)i * n + j];
  std::vector<double> rdiag((size_t)n, 0.0);
  std::vector<std::atomic<int>> ready((size_t)n);
  for (auto& r : ready) r.store(0, std::memory_order_relaxed);

  unsigned hw = std::thread::hardware_concurrency();
  int T = (int)(hw == 0 ? 1 : hw);
  if (T > 16) T = 16;
  if (T > d / 64 + 1) T = d / 64 + 1;

  // Factorisation, columns dealt round-robin to the threads.  Reflection k is
  // published (ready[k]) by the owner of column k as soon as reflections
  // 0..k-1 have been applied to that column; every thread then applies it to
  // its own later columns, the one that owns column k+1 doing that column first.
  auto factor = [&](int t) {
    for (int64_t k = 0; k < n; ++k) {
      if (k % T == t) {
        rdiag[(size_t)k] = make_reflector(&a[(size_t)k * n + k], n - k);
        ready[(size_t)k].store(1, std::memory_order_release);
      } else {
        while (ready[(size_t)k].load(std::memory_order_acquire) == 0) std::this_thread::yield();
      }
      const double* v = &a[(size_t)k * n + k];
      // own columns after k, the next one to be published first
      int64_t first = k + 1;
      if (first < n && first % T == t) reflect(v, &a[(size_t)first * n + k], n - k);
      for (int64_t j = k + 2; j < n; ++j)
        if (j % T == t) reflect(v, &a[(size_t)j * n + k], n - k);
      // (the owner of column k+1 publishes it at the top of its next iteration)
    }
  };
  {
    std::vector<std::thread> pool;
    for (int t = 1; t < T; ++t) pool.emplace_back(factor, t);
    factor(0);
    for (auto& th : pool) th.join();
  }

  // Q = H_0 H_1 ... H_{d-1}.  Column c of Q is H_0 ... H_c e_c (later
  // reflections leave e_c alone), built innermost first; the columns are
  // independent.  Column j is negated where R_jj < 0, which makes the
  // factorisation unique (R with a positive diagonal).
  auto form = [&](int t) {
    std::vector<double> w((size_t)n);
    for (int64_t c = t; c < n; c += T) {
      std::memset(w.data(), 0, sizeof(double) * (size_t)n);
      w[(size_t)c] = 1.0;
      for (int64_t k = c; k >= 0; --k) reflect(&a[(size_t)k * n + k], &w[(size_t)k], n - k);
      const double sgn = rdiag[(size_t)c] < 0.0 ? -1.0 : 1.0;
      for (int64_t i = 0; i < n; ++i) Pi[(size_t)i * n + c] = (float)(sgn * w[(size_t)i]);
    }
  };
  {
    std::vector<std::thread> pool;
    for (int t = 1; t < T; ++t) pool.emplace_back(form, t);
    form(0);
    for (auto& th : pool) th.join();
  }
  return TQ_OK;
}

tq_status tq_compose_split(int32_t d, int32_t d_hi, const int32_t* hi_channels, const float* block_hi,
                           const float* block_lo, float* out) {
  if (d <= 0 || d_hi <= 0 || d_hi >= d || hi_channels == nullptr || block_hi == nullptr || block_lo == nullptr ||
      out == nullptr)
    return TQ_ERR_INVALID_ARG;
  std::vector<int32_t> order;
  std::vector<char> is_hi((size_t)d, 0);
  int32_t prev = -1;
  for (int32_t i = 0; i < d_hi; ++i) {
    const int32_t c = hi_channels[i];
    if (c <= prev || c >= d) return TQ_ERR_INVALID_ARG;  // ascending, distinct, in range
    prev = c;
    is_hi[(size_t)c] = 1;
    order.push_back(c);
  }
  for (int32_t c = 0; c < d; ++c)
    if (!is_hi[(size_t)c]) order.push_back(c);
  const int32_t d_lo = d - d_hi;
  std::memset(out, 0, sizeof(float) * (size_t)d * d);
  // column c of blockdiag(hi, lo) acts on channel order[c]
  for (int32_t r = 0; r < d_hi; ++r)
    for (int32_t c = 0; c < d_hi; ++c) out[(size_t)r * d + order[(size_t)c]] = block_hi[(size_t)r * d_hi + c];
  for (int32_t r = 0; r < d_lo; ++r)
    for (int32_t c = 0; c < d_lo; ++c)
      out[(size_t)(d_hi + r) * d + order[(size_t)(d_hi + c)]] = block_lo[(size_t)r * d_lo + c];
  return TQ_OK;
}

}  // extern "C"
