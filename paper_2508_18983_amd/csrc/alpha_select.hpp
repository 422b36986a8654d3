// Choosing the substitution threshold alpha from a latency budget (Section V-C,
// Eq. 5): a low-degree polynomial T(alpha) is fitted to measured (alpha, TPOT)
// pairs by least squares, and a one-dimensional scan from the low end returns
// the smallest alpha whose predicted TPOT meets the budget (the accuracy loss
// grows with alpha, so the smallest feasible alpha is the minimiser).  Plain
// C++ with no HIP dependency: part of libsmoe and of the CPU test shim.
#pragma once
#include <cmath>

namespace smoe {

constexpr int kMaxPolyDegree = 6;

// Least-squares coefficients c[0..degree] (constant term first) of
// T(a) = sum_i c[i] a^i through the n samples; false when the system is
// singular (fewer distinct alphas than coefficients).  The abscissae are
// centred and scaled to [-1, 1] for the solve and the result is expanded back.
inline bool fit_polynomial(const double* a, const double* t, int n, int degree, double* c) {
  if (degree < 0 || degree > kMaxPolyDegree || n <= degree) return false;
  const int m = degree + 1;
  double lo = a[0], hi = a[0];
  for (int i = 1; i < n; ++i) { lo = a[i] < lo ? a[i] : lo; hi = a[i] > hi ? a[i] : hi; }
  if (!(hi > lo) && degree > 0) return false;
  const double mid = 0.5 * (lo + hi), half = degree > 0 ? 0.5 * (hi - lo) : 1.0;
  // normal equations in the scaled variable u = (a - mid) / half
  double M[kMaxPolyDegree + 1][kMaxPolyDegree + 2] = {};
  for (int s = 0; s < n; ++s) {
    const double u = (a[s] - mid) / half;
    double pw[2 * kMaxPolyDegree + 1];
    pw[0] = 1.0;
    for (int i = 1; i <= 2 * degree; ++i) pw[i] = pw[i - 1] * u;
    for (int i = 0; i < m; ++i) {
      for (int j = 0; j < m; ++j) M[i][j] += pw[i + j];
      M[i][m] += pw[i] * t[s];
    }
  }
  // Gaussian elimination with partial pivoting
  for (int col = 0; col < m; ++col) {
    int piv = col;
    for (int r = col + 1; r < m; ++r)
      if (std::fabs(M[r][col]) > std::fabs(M[piv][col])) piv = r;
    if (std::fabs(M[piv][col]) < 1e-13 * (1.0 + std::fabs(M[0][0]))) return false;
    if (piv != col)
      for (int j = 0; j <= m; ++j) { const double x = M[col][j]; M[col][j] = M[piv][j]; M[piv][j] = x; }
    for (int r = col + 1; r < m; ++r) {
      const double f = M[r][col] / M[col][col];
      for (int j = col; j <= m; ++j) M[r][j] -= f * M[col][j];
    }
  }
  double d[kMaxPolyDegree + 1];
  for (int i = m - 1; i >= 0; --i) {
    double s = M[i][m];
    for (int j = i + 1; j < m; ++j) s -= M[i][j] * d[j];
    d[i] = s / M[i][i];
  }
  // expand sum_i d[i] ((a - mid) / half)^i into powers of a
  for (int i = 0; i < m; ++i) c[i] = 0.0;
  double basis[kMaxPolyDegree + 1] = {1.0};         // coefficients of ((a - mid) / half)^i, built up by i
  int blen = 1;
  for (int i = 0; i < m; ++i) {
    for (int j = 0; j < blen; ++j) c[j] += d[i] * basis[j];
    if (i + 1 < m) {                                 // basis *= (a - mid) / half
      double next[kMaxPolyDegree + 1] = {};
      for (int j = 0; j < blen; ++j) {
        next[j] += basis[j] * (-mid / half);
        next[j + 1] += basis[j] / half;
      }
      ++blen;
      for (int j = 0; j < blen; ++j) basis[j] = next[j];
    }
  }
  return true;
}

inline double eval_polynomial(const double* c, int degree, double a) {
  double v = c[degree];
  for (int i = degree - 1; i >= 0; --i) v = v * a + c[i];
  return v;
}

// Smallest point of the uniform grid lo + i (hi - lo) / (resolution - 1) over the
// sampled range [min a, max a] with T(point) <= budget.  Returns 0 and the point
// in *alpha; 1 when no grid point meets the budget; -1 on bad arguments.
inline int select_alpha(const double* a, const double* t, int n, double budget, int degree, int resolution,
                        double* alpha, double* coef) {
  if (!a || !t || !alpha || !coef || n < 1 || resolution < 2) return -1;
  if (!fit_polynomial(a, t, n, degree, coef)) return -1;
  double lo = a[0], hi = a[0];
  for (int i = 1; i < n; ++i) { lo = a[i] < lo ? a[i] : lo; hi = a[i] > hi ? a[i] : hi; }
  for (int i = 0; i < resolution; ++i) {
    const double x = lo + (hi - lo) * (double)i / (double)(resolution - 1);
    if (eval_polynomial(coef, degree, x) <= budget) { *alpha = x; return 0; }
  }
  return 1;
}

}  // namespace smoe
