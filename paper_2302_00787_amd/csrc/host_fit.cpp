// Closed-form DERF parameter fits on d x d statistics, in fp64 on the host.
//
// Input: the data statistics of one parameter group (mu4 = mean x, mu5 = mean y,
// M1 = mean x x^T, M2 = mean y y^T; Theorems on ADERF and SDERF).  Output: one
// theta block in the layout documented in favorsharp.h.  The matrix
// decompositions are cyclic Jacobi iterations written here (symmetric
// eigenproblem: two-sided rotations; SVD: one-sided Hestenes rotations).
#include "host_fit.h"

#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>
#include <vector>

namespace fs {

// Scalar minimiser of log(1-4A) - 1/2 log(1-8A) + phi/(1-8A)  (appendix lemma).
static double a_star(double phi) {
  const double t = 2.0 * phi + 1.0;
  return (1.0 - 2.0 * phi - std::sqrt(t * t + 8.0 * phi)) / 16.0;
}

// Symmetric eigendecomposition a = v diag(w) v^T, cyclic Jacobi.  a: n*n row-major (destroyed),
// v: n*n, column j is the eigenvector of w[j].  Eigenvalues are returned in non-ascending order and each
// eigenvector has its largest-magnitude component positive (lowest index on ties).
void jacobi_eigh(int n, std::vector<double>& a, std::vector<double>& w, std::vector<double>& v) {
  v.assign((size_t)n * n, 0.0);
  for (int i = 0; i < n; ++i) v[(size_t)i * n + i] = 1.0;
  double scale = 0.0;
  for (double x : a) scale = std::max(scale, std::fabs(x));
  for (int sweep = 0; sweep < 60; ++sweep) {
    double off = 0.0;
    for (int p = 0; p < n; ++p)
      for (int q = p + 1; q < n; ++q) off += a[(size_t)p * n + q] * a[(size_t)p * n + q];
    if (std::sqrt(off) <= 1e-30 + 1e-17 * scale * n) break;
    for (int p = 0; p < n - 1; ++p) {
      for (int q = p + 1; q < n; ++q) {
        const double apq = a[(size_t)p * n + q];
        if (std::fabs(apq) < 1e-300) continue;
        const double app = a[(size_t)p * n + p], aqq = a[(size_t)q * n + q];
        const double zeta = (aqq - app) / (2.0 * apq);
        const double t = (zeta >= 0 ? 1.0 : -1.0) / (std::fabs(zeta) + std::sqrt(1.0 + zeta * zeta));
        const double c = 1.0 / std::sqrt(1.0 + t * t), s = c * t;
        for (int k = 0; k < n; ++k) {      // columns p, q
          const double akp = a[(size_t)k * n + p], akq = a[(size_t)k * n + q];
          a[(size_t)k * n + p] = c * akp - s * akq;
          a[(size_t)k * n + q] = s * akp + c * akq;
        }
        for (int k = 0; k < n; ++k) {      // rows p, q
          const double apk = a[(size_t)p * n + k], aqk = a[(size_t)q * n + k];
          a[(size_t)p * n + k] = c * apk - s * aqk;
          a[(size_t)q * n + k] = s * apk + c * aqk;
        }
        for (int k = 0; k < n; ++k) {
          const double vkp = v[(size_t)k * n + p], vkq = v[(size_t)k * n + q];
          v[(size_t)k * n + p] = c * vkp - s * vkq;
          v[(size_t)k * n + q] = s * vkp + c * vkq;
        }
      }
    }
  }
  std::vector<int> order(n);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(),
                   [&](int i, int j) { return a[(size_t)i * n + i] > a[(size_t)j * n + j]; });
  std::vector<double> vs((size_t)n * n);
  w.resize(n);
  for (int j = 0; j < n; ++j) {
    const int src = order[j];
    w[j] = a[(size_t)src * n + src];
    int big = 0;
    for (int k = 1; k < n; ++k)
      if (std::fabs(v[(size_t)k * n + src]) > std::fabs(v[(size_t)big * n + src])) big = k;
    const double sg = v[(size_t)big * n + src] < 0 ? -1.0 : 1.0;
    for (int k = 0; k < n; ++k) vs[(size_t)k * n + j] = sg * v[(size_t)k * n + src];
  }
  v.swap(vs);
}

// Singular value decomposition z = u diag(s) vt^T of a square matrix by one-sided Jacobi rotations.
// Only u and s are returned (the ADERF closed form uses nothing else); s is non-ascending.
static void jacobi_svd_us(int n, const std::vector<double>& z, std::vector<double>& u, std::vector<double>& s) {
  std::vector<double> g = z;
  for (int sweep = 0; sweep < 60; ++sweep) {
    bool rotated = false;
    for (int p = 0; p < n - 1; ++p) {
      for (int q = p + 1; q < n; ++q) {
        double al = 0, be = 0, ga = 0;
        for (int k = 0; k < n; ++k) {
          const double gp = g[(size_t)k * n + p], gq = g[(size_t)k * n + q];
          al += gp * gp; be += gq * gq; ga += gp * gq;
        }
        if (std::fabs(ga) <= 1e-16 * std::sqrt(al * be) || ga == 0.0) continue;
        rotated = true;
        const double zeta = (be - al) / (2.0 * ga);
        const double t = (zeta >= 0 ? 1.0 : -1.0) / (std::fabs(zeta) + std::sqrt(1.0 + zeta * zeta));
        const double c = 1.0 / std::sqrt(1.0 + t * t), sn = c * t;
        for (int k = 0; k < n; ++k) {
          const double gp = g[(size_t)k * n + p], gq = g[(size_t)k * n + q];
          g[(size_t)k * n + p] = c * gp - sn * gq;
          g[(size_t)k * n + q] = sn * gp + c * gq;
        }
      }
    }
    if (!rotated) break;
  }
  std::vector<double> norms(n);
  for (int j = 0; j < n; ++j) {
    double t = 0;
    for (int k = 0; k < n; ++k) t += g[(size_t)k * n + j] * g[(size_t)k * n + j];
    norms[j] = std::sqrt(t);
  }
  std::vector<int> order(n);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int i, int j) { return norms[i] > norms[j]; });
  u.assign((size_t)n * n, 0.0);
  s.resize(n);
  for (int j = 0; j < n; ++j) {
    const int src = order[j];
    s[j] = norms[src];
    for (int k = 0; k < n; ++k) u[(size_t)k * n + j] = norms[src] > 0 ? g[(size_t)k * n + src] / norms[src] : 0.0;
  }
}

static void write_header(float* th, double logD, double lbar, int flags, int variant) {
  th[0] = (float)logD;
  th[1] = (float)lbar;
  th[2] = (float)flags;
  th[3] = (float)variant;
  th[4] = th[5] = th[6] = th[7] = 0.f;
}

// GERF-shaped theta (A = a I, B1 = b diag(p), B2 = b diag(1/p), C1 = -1/2 diag(p^2), C2 = -1/2 diag(p^-2)).
static void write_scalar_family(float* th, int d, double a, const std::vector<double>& psi, double lbar, int variant) {
  const double b = std::sqrt(1.0 - 4.0 * a);
  bool unit = true;
  for (double p : psi) unit = unit && (p == 1.0);
  write_header(th, 0.25 * d * std::log(1.0 - 4.0 * a), lbar, unit ? 3 : 0, variant);
  float* A = th + 8; float* B1 = A + d; float* B2 = B1 + (size_t)d * d;
  float* C1 = B2 + (size_t)d * d; float* C2 = C1 + (size_t)d * d;
  std::fill(B1, C2 + (size_t)d * d, 0.f);
  for (int l = 0; l < d; ++l) {
    A[l] = (float)a;
    B1[(size_t)l * d + l] = (float)(b * psi[l]);
    B2[(size_t)l * d + l] = (float)(b / psi[l]);
    C1[(size_t)l * d + l] = (float)(-0.5 * psi[l] * psi[l]);
    C2[(size_t)l * d + l] = (float)(-0.5 / (psi[l] * psi[l]));
  }
}

int fit_group(int variant, int d, const double* M1, const double* M2, const double* mu4, const double* mu5,
              double ridge, float* th) {
  const size_t dd = (size_t)d * d;
  double tr1 = 0, tr2 = 0, dot = 0;
  for (int l = 0; l < d; ++l) { tr1 += M1[(size_t)l * d + l]; tr2 += M2[(size_t)l * d + l]; dot += mu4[l] * mu5[l]; }
  const double nan = std::numeric_limits<double>::quiet_NaN();
  std::vector<double> ones(d, 1.0);

  if (variant == 0) {                                   // PosRF: A = 0
    write_scalar_family(th, d, 0.0, ones, nan, variant);
    return 0;
  }
  if (variant == 1 || variant == 2) {                   // GERF, SADERF
    std::vector<double> psi = ones;
    double s = tr1 + tr2 + 2.0 * dot;                   // mean |x + y|^2
    if (variant == 2) {
      s = 2.0 * dot;
      for (int l = 0; l < d; ++l) {
        const double m1 = M1[(size_t)l * d + l], m2 = M2[(size_t)l * d + l];
        if (!(m1 > 0.0) || !(m2 > 0.0)) return 3;
        psi[l] = std::pow(m2 / m1, 0.25);
        s += psi[l] * psi[l] * m1 + m2 / (psi[l] * psi[l]);
      }
    }
    const double a = a_star(s / d);
    double sx = tr1, sy = tr2;
    if (variant == 2) {
      sx = sy = 0;
      for (int l = 0; l < d; ++l) {
        sx += psi[l] * psi[l] * M1[(size_t)l * d + l];
        sy += M2[(size_t)l * d + l] / (psi[l] * psi[l]);
      }
    }
    const double lbar = d * std::log((1.0 - 4.0 * a) / std::sqrt(1.0 - 8.0 * a))
                        + (2.0 - 8.0 * a) / (1.0 - 8.0 * a) * s - sx - sy;
    write_scalar_family(th, d, a, psi, lbar, variant);
    return 0;
  }
  float* A = th + 8; float* B1 = A + d; float* B2 = B1 + dd; float* C1 = B2 + dd; float* C2 = C1 + dd;

  if (variant == 4) {                                   // SDERF
    std::vector<double> N(dd), w, Q;
    for (int r = 0; r < d; ++r)
      for (int c = 0; c < d; ++c)
        N[(size_t)r * d + c] = M1[(size_t)r * d + c] + mu4[r] * mu5[c] + mu5[r] * mu4[c] + M2[(size_t)r * d + c];
    jacobi_eigh(d, N, w, Q);
    double logD = 0, lbar = -tr1 - tr2;
    std::fill(C1, C1 + 2 * dd, 0.f);
    for (int l = 0; l < d; ++l) {
      const double lam = std::max(w[l], 0.0);
      const double a = a_star(lam);
      A[l] = (float)a;
      logD += 0.25 * std::log(1.0 - 4.0 * a);
      lbar += std::log(1.0 - 4.0 * a) - 0.5 * std::log(1.0 - 8.0 * a) + (1.0 + 1.0 / (1.0 - 8.0 * a)) * lam;
      const double b = std::sqrt(1.0 - 4.0 * a);
      for (int c = 0; c < d; ++c) {                     // B = (I - 4A)^(1/2) Q3^T: row l is the scaled eigenvector l
        B1[(size_t)l * d + c] = B2[(size_t)l * d + c] = (float)(b * Q[(size_t)c * d + l]);
      }
      C1[(size_t)l * d + l] = C2[(size_t)l * d + l] = -0.5f;
    }
    write_header(th, logD, lbar, 3, variant);
    return 0;
  }
  if (variant == 3) {                                   // ADERF
    std::vector<double> m1(M1, M1 + dd), m2(M2, M2 + dd), l1, l2, Q1, Q2;
    for (int l = 0; l < d; ++l) { m1[(size_t)l * d + l] += ridge; m2[(size_t)l * d + l] += ridge; }
    jacobi_eigh(d, m1, l1, Q1);
    jacobi_eigh(d, m2, l2, Q2);
    if (!(l1[d - 1] > 1e-12 * l1[0]) || !(l2[d - 1] > 1e-12 * l2[0])) return 3;
    // Z = L1^(1/2) Q1^T Q2 L2^(1/2)
    std::vector<double> Z(dd), U, sig;
    for (int r = 0; r < d; ++r)
      for (int c = 0; c < d; ++c) {
        double t = 0;
        for (int k = 0; k < d; ++k) t += Q1[(size_t)k * d + r] * Q2[(size_t)k * d + c];
        Z[(size_t)r * d + c] = std::sqrt(l1[r]) * t * std::sqrt(l2[c]);
      }
    jacobi_svd_us(d, Z, U, sig);
    double trs = 0;
    for (double s : sig) trs += s;
    if (!(sig[d - 1] > 0.0)) return 3;
    const double mu3 = dot / d;
    const double a = a_star(2.0 * trs / d + 2.0 * mu3);
    const double b = std::sqrt(1.0 - 4.0 * a);
    // B1 = b S^(1/2) U^T L1^(-1/2) Q1^T,  B2 = b S^(-1/2) U^T L1^(1/2) Q1^T
    std::vector<double> b1(dd), b2(dd);
    for (int r = 0; r < d; ++r)
      for (int c = 0; c < d; ++c) {
        double t1 = 0, t2 = 0;
        for (int k = 0; k < d; ++k) {
          const double uq = U[(size_t)k * d + r] * Q1[(size_t)c * d + k];
          t1 += uq / std::sqrt(l1[k]);
          t2 += uq * std::sqrt(l1[k]);
        }
        b1[(size_t)r * d + c] = b * std::sqrt(sig[r]) * t1;
        b2[(size_t)r * d + c] = b / std::sqrt(sig[r]) * t2;
      }
    for (int r = 0; r < d; ++r)
      for (int c = 0; c < d; ++c) {
        double t1 = 0, t2 = 0;
        for (int k = 0; k < d; ++k) {
          t1 += b1[(size_t)k * d + r] * b1[(size_t)k * d + c];
          t2 += b2[(size_t)k * d + r] * b2[(size_t)k * d + c];
        }
        C1[(size_t)r * d + c] = (float)(-t1 / (2.0 * (1.0 - 4.0 * a)));
        C2[(size_t)r * d + c] = (float)(-t2 / (2.0 * (1.0 - 4.0 * a)));
        B1[(size_t)r * d + c] = (float)b1[(size_t)r * d + c];
        B2[(size_t)r * d + c] = (float)b2[(size_t)r * d + c];
      }
    for (int l = 0; l < d; ++l) A[l] = (float)a;
    const double lbar = d * (std::log(1.0 - 4.0 * a) - 0.5 * std::log(1.0 - 8.0 * a)
                             + 2.0 / (1.0 - 8.0 * a) * (trs / d + mu3) + 2.0 * mu3);
    write_header(th, 0.25 * d * std::log(1.0 - 4.0 * a), lbar, 0, variant);
    return 0;
  }
  return 1;
}

bool orthogonal_rows(int n, int d, const double* g, const double* len, double* out) {
  std::vector<double> q((size_t)n * d);
  for (int i = 0; i < n; ++i) {
    double* qi = &q[(size_t)i * d];
    double n0 = 0.0;
    for (int c = 0; c < d; ++c) { qi[c] = g[(size_t)i * d + c]; n0 += qi[c] * qi[c]; }
    for (int pass = 0; pass < 2; ++pass)
      for (int j = 0; j < i; ++j) {
        const double* qj = &q[(size_t)j * d];
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += qi[c] * qj[c];
        for (int c = 0; c < d; ++c) qi[c] -= dot * qj[c];
      }
    double n1 = 0.0;
    for (int c = 0; c < d; ++c) n1 += qi[c] * qi[c];
    if (!(n1 > 1e-24 * n0) || !(n0 > 0.0)) return false;
    const double inv = 1.0 / std::sqrt(n1);
    for (int c = 0; c < d; ++c) qi[c] *= inv;
    for (int c = 0; c < d; ++c) out[(size_t)i * d + c] = len[i] * qi[c];
  }
  return true;
}

}  // namespace fs
