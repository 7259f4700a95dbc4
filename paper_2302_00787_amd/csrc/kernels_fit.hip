// Closed-form DERF parameter fits on the device: one workgroup per parameter group, fp64, no host round trip.
//
// Input: the data statistics of a group (mu4 = mean x, mu5 = mean y, M1 = mean x x^T, M2 = mean y y^T; Theorems on
// ADERF and SDERF), as the statistics kernels leave them.  Output: one theta block per group (layout in
// favorsharp.h) and one status word per group.
//
// The symmetric eigenproblems (M1, M2, and N = M1 + mu4 mu5^T + mu5 mu4^T + M2) are solved by the two-sided Jacobi
// iteration, the singular value problem of the ADERF matrix Lambda1^(1/2) Q1^T Q2 Lambda2^(1/2) by the one-sided
// (Hestenes) iteration on its columns, whose normalised columns are the left singular vectors.  Both use the
// round-robin ordering: a round rotates d/2 disjoint index pairs at once, a few lanes per pair, one or two barriers
// per round.  The matrix lives in LDS during the iteration, and so do the accumulated rotations when both fit
// (d <= 96).
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace fs {

namespace {

constexpr int FIT_NT = 512;      // threads per workgroup (256 and 1024 were measured: 30 % slower / no faster)
constexpr int FIT_DMAX = 128;
// A pair of columns counts as orthogonal below this cosine.  The statistics carry fp32 rounding of the inputs'
// products, so nothing is gained by iterating to the last bits of fp64.
constexpr double kJacobiEps = 1e-13;
// A sweep is followed by another one only if it met a pair above this cosine: the iteration converges quadratically,
// so a sweep whose largest cosine is below 1e-8 leaves nothing above 1e-15 behind, and the sweep that would only
// confirm that is not run.
constexpr double kJacobiAgain = 1e-8;

// Scalar minimiser of log(1-4A) - 1/2 log(1-8A) + phi/(1-8A)  (appendix lemma on the scalar objective).
__device__ __forceinline__ double a_star(double phi) {
  const double t = 2.0 * phi + 1.0;
  return (1.0 - 2.0 * phi - sqrt(t * t + 8.0 * phi)) / 16.0;
}

// Sum over a group of w consecutive lanes (w a power of two, groups aligned); every lane gets the same bits.
__device__ __forceinline__ double lanes_sum(double v, int w) {
  for (int m = w >> 1; m > 0; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}

struct FitShared {
  double nrm[3][FIT_DMAX];   // column norms after an iteration (eigenvalues / singular values, unsorted)
  double sgn[3][FIT_DMAX];   // sign that makes the largest component of an eigenvector positive
  int ord[3][FIT_DMAX];      // ord[k] = column with the k-th largest norm
  double red[8];             // scalars shared by the workgroup
  int flag;
};

// Tangent of the Jacobi rotation that annihilates the off-diagonal entry `off` of a 2 x 2 block whose diagonal
// entries differ by `diff`: t = sign(z) / (|z| + sqrt(1 + z^2)), z = diff / (2 off).  The rotation must be orthogonal
// to fp64 accuracy, its angle need not be (an error of 1e-6 of the angle leaves 1e-6 of the pair's off-diagonal entry
// for the next sweep): fp32 with the hardware reciprocal and square root.  0, inf or NaN when there is nothing to
// rotate (the callers skip those).
__device__ __forceinline__ float rotation_tangent(float diff, float off) {
  const float zeta = diff * __builtin_amdgcn_rcpf(2.f * off);
  return copysignf(1.f, zeta) * __builtin_amdgcn_rcpf(fabsf(zeta) + __builtin_amdgcn_sqrtf(1.f + zeta * zeta));
}

// Cosine 1 / sqrt(1 + t^2) of the rotation with tangent t, |t| <= 1, to fp64 accuracy: the fp32 hardware estimate
// and two Newton steps (relative error 1e-7 -> 1e-14 -> below the rounding of fp64).
__device__ __forceinline__ double rotation_cosine(double t) {
  const double x = 1.0 + t * t;
  double c = (double)__builtin_amdgcn_rsqf((float)x);
  c = c * (1.5 - 0.5 * x * c * c);
  c = c * (1.5 - 0.5 * x * c * c);
  return c;
}

// Batched access to a pair of strided vectors for the sizes where every lane of a pair handles exactly NI elements
// (n = NI x lanes per pair: 32, 64, 128 with 512 threads).  Every request is issued before the first use, so a pair
// costs one memory latency, not one per element as in the general loops (whose stores may alias the next loads).
template <int NI>
__device__ __forceinline__ void fetch_pair(const double* xp, const double* xq, int stride, int r0, int tpp,
                                           double (&x)[NI], double (&y)[NI]) {
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const size_t r = (size_t)(r0 + i * tpp) * stride;
    x[i] = xp[r];
    y[i] = xq[r];
  }
}
// (xp, xq) <- (c xp - s xq, s xp + c xq) on those elements.
template <int NI>
__device__ __forceinline__ void store_rotated(double* xp, double* xq, int stride, int r0, int tpp, const double (&x)[NI],
                                              const double (&y)[NI], double c, double s) {
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const size_t r = (size_t)(r0 + i * tpp) * stride;
    xp[r] = c * x[i] - s * y[i];
    xq[r] = s * x[i] + c * y[i];
  }
}

// One-sided Jacobi on the columns of g (n x n, column c at g + c * ldg): g <- g R with mutually orthogonal columns,
// v <- v R if v != nullptr (column c at v + c * ldv).  All FIT_NT threads must call; n <= FIT_DMAX.  The function is
// inlined at each call site so that the address spaces of g and v (LDS or global) are known to the compiler.
// NI > 0: n = NI x (lanes per pair), batched accesses; NI = 0: any n.
template <int NI>
__device__ __forceinline__ void jacobi_columns(double* g, double* v, int n, int ldg, int ldv, FitShared& sh) {
  const int np = (n + 1) / 2;        // pairs per round
  const int m = 2 * np;              // players of the tournament (player n is a bye when n is odd)
  int tpp = 64;                      // lanes per pair
  while (tpp * np > FIT_NT) tpp >>= 1;
  const int t = threadIdx.x, pair = t / tpp, r0 = t % tpp;
  constexpr int NA = NI > 0 ? NI : 1;
  for (int sweep = 0; sweep < 40; ++sweep) {
    if (t == 0) sh.flag = 0;
    __syncthreads();
    // round-robin: player m-1 stays, the others walk round a circle of m-1 seats; in round `round` pair 0 is
    // (m-1, round), pair k is (round + k, round - k) modulo m-1.  The two seats advance by one per round.
    int pa = pair % (m - 1), pb = (m - 1 - pair) % (m - 1);
    for (int round = 0; round < m - 1; ++round) {
      if (pair < np) {
        int p = pair == 0 ? m - 1 : pa;
        int q = pair == 0 ? round : pb;
        if (p > q) { const int s = p; p = q; q = s; }
        if (q < n) {
          double* gp = g + (size_t)p * ldg;
          double* gq = g + (size_t)q * ldg;
          double al = 0.0, be = 0.0, ga = 0.0;
          double x[NA], y[NA];
          if constexpr (NI > 0) {
            fetch_pair<NA>(gp, gq, 1, r0, tpp, x, y);
#pragma unroll
            for (int i = 0; i < NA; ++i) { al += x[i] * x[i]; be += y[i] * y[i]; ga += x[i] * y[i]; }
          } else {
            for (int r = r0; r < n; r += tpp) {
              const double a = gp[r], b = gq[r];
              al += a * a; be += b * b; ga += a * b;
            }
          }
          al = lanes_sum(al, tpp); be = lanes_sum(be, tpp); ga = lanes_sum(ga, tpp);
          // tangent in fp32, cosine and sine from it in fp64
          const float tn32 = rotation_tangent((float)(be - al), (float)ga);
          if (ga * ga > kJacobiEps * kJacobiEps * al * be && tn32 != 0.f && isfinite(tn32)) {
            const double tn = (double)tn32;
            const double c = rotation_cosine(tn), s = c * tn;
            if constexpr (NI > 0) {
              double vx[NA], vy[NA];
              if (v != nullptr) fetch_pair<NA>(v + (size_t)p * ldv, v + (size_t)q * ldv, 1, r0, tpp, vx, vy);
              store_rotated<NA>(gp, gq, 1, r0, tpp, x, y, c, s);
              if (v != nullptr) store_rotated<NA>(v + (size_t)p * ldv, v + (size_t)q * ldv, 1, r0, tpp, vx, vy, c, s);
            } else {
              for (int r = r0; r < n; r += tpp) {
                const double a = gp[r], b = gq[r];
                gp[r] = c * a - s * b;
                gq[r] = s * a + c * b;
              }
              if (v != nullptr) {
                double* vp = v + (size_t)p * ldv;
                double* vq = v + (size_t)q * ldv;
                for (int r = r0; r < n; r += tpp) {
                  const double a = vp[r], b = vq[r];
                  vp[r] = c * a - s * b;
                  vq[r] = s * a + c * b;
                }
              }
            }
            if (r0 == 0 && ga * ga > kJacobiAgain * kJacobiAgain * al * be) sh.flag = 1;
          }
        }
      }
      pa = pa + 1 == m - 1 ? 0 : pa + 1;
      pb = pb + 1 == m - 1 ? 0 : pb + 1;
      __syncthreads();
    }
    const int again = sh.flag;
    __syncthreads();
    if (!again) break;
  }
}

// Two-sided Jacobi for a symmetric matrix a (n x n in column-major with stride lda): a <- J^T a J until the
// off-diagonal part vanishes, v <- v J.  The rotation of pair (p, q) is fixed by the 2 x 2 block (a_pp, a_pq, a_qq),
// which no other pair of the round touches; the round applies all column rotations, a barrier, all row rotations.
// No inner products and no cross-lane sums are needed, and the sweep count follows the conditioning of a itself
// (the one-sided iteration on a symmetric matrix works on its square).  `scale`: largest |a_ii| at the start.
// NI as above; with NI > 0 the columns of a and of v are requested together with the 2 x 2 block, before the
// rotation is known, so that a round is a chain of two memory latencies and two barriers.
template <int NI>
__device__ __forceinline__ void jacobi_symmetric(double* a, double* v, int n, int lda, int ldv, double scale, FitShared& sh) {
  const int np = (n + 1) / 2;
  const int m = 2 * np;
  int tpp = 64;
  while (tpp * np > FIT_NT) tpp >>= 1;
  const int t = threadIdx.x, pair = t / tpp, r0 = t % tpp;
  constexpr int NA = NI > 0 ? NI : 1;
  for (int sweep = 0; sweep < 40; ++sweep) {
    if (t == 0) sh.flag = 0;
    __syncthreads();
    int pa = pair % (m - 1), pb = (m - 1 - pair) % (m - 1);
    for (int round = 0; round < m - 1; ++round) {
      bool rot = false, big = false;
      double c = 1.0, s = 0.0;
      int p = 0, q = 0;
      double x[NA], y[NA], vx[NA], vy[NA];
      if (pair < np) {
        p = pair == 0 ? m - 1 : pa;
        q = pair == 0 ? round : pb;
        if (p > q) { const int w = p; p = q; q = w; }
        if (q < n) {
          if constexpr (NI > 0) {
            fetch_pair<NA>(a + (size_t)p * lda, a + (size_t)q * lda, 1, r0, tpp, x, y);
            if (v != nullptr) fetch_pair<NA>(v + (size_t)p * ldv, v + (size_t)q * ldv, 1, r0, tpp, vx, vy);
          }
          const double app = a[(size_t)p * lda + p], aqq = a[(size_t)q * lda + q], apq = a[(size_t)q * lda + p];
          const float tn32 = rotation_tangent((float)(aqq - app), (float)apq);
          if (apq * apq > kJacobiEps * kJacobiEps * fabs(app * aqq) && fabs(apq) > 1e-18 * scale && tn32 != 0.f && isfinite(tn32)) {
            const double tn = (double)tn32;
            c = rotation_cosine(tn);
            s = c * tn;
            rot = true;
            big = apq * apq > kJacobiAgain * kJacobiAgain * fabs(app * aqq);
          }
        }
      }
      if (rot) {
        double* ap = a + (size_t)p * lda;
        double* aq = a + (size_t)q * lda;
        if constexpr (NI > 0) {
          store_rotated<NA>(ap, aq, 1, r0, tpp, x, y, c, s);
          if (v != nullptr) store_rotated<NA>(v + (size_t)p * ldv, v + (size_t)q * ldv, 1, r0, tpp, vx, vy, c, s);
        } else {
          for (int r = r0; r < n; r += tpp) {
            const double xx = ap[r], yy = aq[r];
            ap[r] = c * xx - s * yy;
            aq[r] = s * xx + c * yy;
          }
          if (v != nullptr) {
            double* vp = v + (size_t)p * ldv;
            double* vq = v + (size_t)q * ldv;
            for (int r = r0; r < n; r += tpp) {
              const double xx = vp[r], yy = vq[r];
              vp[r] = c * xx - s * yy;
              vq[r] = s * xx + c * yy;
            }
          }
        }
      }
      __syncthreads();
      if (rot) {
        if constexpr (NI > 0) {
          fetch_pair<NA>(a + p, a + q, lda, r0, tpp, x, y);
          store_rotated<NA>(a + p, a + q, lda, r0, tpp, x, y, c, s);
        } else {
          for (int k = r0; k < n; k += tpp) {
            const double xx = a[(size_t)k * lda + p], yy = a[(size_t)k * lda + q];
            a[(size_t)k * lda + p] = c * xx - s * yy;
            a[(size_t)k * lda + q] = s * xx + c * yy;
          }
        }
        if (r0 == 0 && big) sh.flag = 1;
      }
      pa = pa + 1 == m - 1 ? 0 : pa + 1;
      pb = pb + 1 == m - 1 ? 0 : pb + 1;
      __syncthreads();
    }
    const int again = sh.flag;
    __syncthreads();
    if (!again) break;
  }
}

// The iteration for the sizes with a batched form (n = 64: 4 elements per lane, n = 128: 16), else the general one.
__device__ __forceinline__ void jacobi_any(double* a, double* v, int n, int lda, int ldv, bool symmetric, double scale,
                                           FitShared& sh) {
  if (n == 64) {
    if (symmetric) jacobi_symmetric<4>(a, v, n, lda, ldv, scale, sh);
    else jacobi_columns<4>(a, v, n, lda, ldv, sh);
  } else if (n == 128) {
    if (symmetric) jacobi_symmetric<16>(a, v, n, lda, ldv, scale, sh);
    else jacobi_columns<16>(a, v, n, lda, ldv, sh);
  } else {
    if (symmetric) jacobi_symmetric<0>(a, v, n, lda, ldv, scale, sh);
    else jacobi_columns<0>(a, v, n, lda, ldv, sh);
  }
}

// Column norms (one-sided iteration) or diagonal entries (two-sided), their non-ascending order and (with v) the
// eigenvector signs into slot k of the shared block.
__device__ __forceinline__ void rank_columns(const double* wg, const double* wv, int n, int ldg, int ldv, int k, bool symmetric, FitShared& sh) {
  const int t = threadIdx.x;
  if (t < n) {
    if (symmetric) {
      sh.nrm[k][t] = wg[(size_t)t * ldg + t];
    } else {
      double s2 = 0.0;
      for (int r = 0; r < n; ++r) s2 += wg[(size_t)t * ldg + r] * wg[(size_t)t * ldg + r];
      sh.nrm[k][t] = sqrt(s2);
    }
    if (wv != nullptr) {
      int big = 0;
      for (int r = 1; r < n; ++r)
        if (fabs(wv[(size_t)t * ldv + r]) > fabs(wv[(size_t)t * ldv + big])) big = r;
      sh.sgn[k][t] = wv[(size_t)t * ldv + big] < 0.0 ? -1.0 : 1.0;
    }
  }
  __syncthreads();
  if (t < n) {
    int rank = 0;
    const double mine = sh.nrm[k][t];
    for (int i = 0; i < n; ++i) rank += (sh.nrm[k][i] > mine || (sh.nrm[k][i] == mine && i < t)) ? 1 : 0;
    sh.ord[k][rank] = t;
  }
  __syncthreads();
}

// Decomposes a d x d matrix held in global memory (g, column-major with stride n, overwritten): the two-sided
// iteration when `symmetric` (eigenvalues = final diagonal), else the one-sided one (singular values = final column
// norms, left singular vectors = normalised columns); v (overwritten; nullptr: none) accumulates the rotations.
// Values, order and signs go to slot k.  The matrix is copied to LDS for the iteration (column stride n + 1: columns
// start in different banks) and back afterwards; the rotations join it there when both fit (n <= kLdsBoth), else
// they stay in global memory.
constexpr int kLdsBoth = 96;
__device__ __forceinline__ void decompose(double* g, double* v, int n, int k, bool symmetric, FitShared& sh, double* lds) {
  const int t = threadIdx.x, nn = n * n, ld = n + 1;
  double* wg = lds;
  for (int e = t; e < nn; e += FIT_NT) wg[(e / n) * ld + e % n] = g[e];
  if (t == 0 && symmetric) {
    double sc = 0.0;
    for (int l = 0; l < n; ++l) sc = fmax(sc, fabs(g[(size_t)l * n + l]));
    sh.red[1] = sc;
  }
  if (v == nullptr) {
    __syncthreads();
    jacobi_any(wg, nullptr, n, ld, 0, symmetric, sh.red[1], sh);
    rank_columns(wg, nullptr, n, ld, 0, k, symmetric, sh);
  } else if (n <= kLdsBoth) {
    double* wv = lds + (size_t)n * ld;
    for (int e = t; e < nn; e += FIT_NT) wv[(e / n) * ld + e % n] = (e / n == e % n) ? 1.0 : 0.0;
    __syncthreads();
    jacobi_any(wg, wv, n, ld, ld, symmetric, sh.red[1], sh);
    rank_columns(wg, wv, n, ld, ld, k, symmetric, sh);
    for (int e = t; e < nn; e += FIT_NT) v[e] = wv[(e / n) * ld + e % n];
  } else {
    for (int e = t; e < nn; e += FIT_NT) v[e] = (e / n == e % n) ? 1.0 : 0.0;
    __syncthreads();
    jacobi_any(wg, v, n, ld, n, symmetric, sh.red[1], sh);
    rank_columns(wg, v, n, ld, n, k, symmetric, sh);
  }
  for (int e = t; e < nn; e += FIT_NT) g[e] = wg[(e / n) * ld + e % n];
  __syncthreads();
}

__device__ void write_header(float* th, double logD, double lbar, int flags, int variant) {
  th[0] = (float)logD;
  th[1] = (float)lbar;
  th[2] = (float)flags;
  th[3] = (float)variant;
  th[4] = th[5] = th[6] = th[7] = 0.f;
}

// grid (groups), block FIT_NT.  stats: per group [M1 d*d, mu4 d][M2 d*d, mu5 d]; ws: per group 7 d*d doubles.
__global__ void __launch_bounds__(FIT_NT) k_fit_device(int variant, int d, const double* stats, double ridge, double* ws,
                                                       float* theta, int* status, size_t theta_floats) {
  extern __shared__ __align__(16) unsigned char fit_lds[];
  __shared__ FitShared sh;
  const int t = threadIdx.x, grp = blockIdx.x, n = d, nn = d * d;
  const size_t per = (size_t)nn + d;
  const double* M1 = stats + (size_t)grp * 2 * per;
  const double* mu4 = M1 + nn;
  const double* M2 = M1 + per;
  const double* mu5 = M2 + nn;
  float* th = theta + (size_t)grp * theta_floats;
  float* A = th + 8;
  float* B1 = A + d;
  float* B2 = B1 + nn;
  float* C1 = B2 + nn;
  float* C2 = C1 + nn;
  double* w = ws + (size_t)grp * 7 * nn;
  double* lds = (double*)fit_lds;
  const double nan = __builtin_nan("");

  // traces and mu4 . mu5 (every thread computes them: d <= 128 terms)
  double tr1 = 0.0, tr2 = 0.0, dot = 0.0;
  for (int l = 0; l < d; ++l) { tr1 += M1[(size_t)l * d + l]; tr2 += M2[(size_t)l * d + l]; dot += mu4[l] * mu5[l]; }

  if (variant <= 2) {                                   // PosRF, GERF, SADERF: A = a I, diagonal B and C
    // psi_l = (M2_ll / M1_ll)^(1/4) for SADERF, 1 otherwise
    bool bad = false;
    double s = variant == 2 ? 2.0 * dot : tr1 + tr2 + 2.0 * dot, sx = tr1, sy = tr2;
    if (variant == 2) {
      sx = sy = 0.0;
      for (int l = 0; l < d; ++l) {
        const double m1 = M1[(size_t)l * d + l], m2 = M2[(size_t)l * d + l];
        if (!(m1 > 0.0) || !(m2 > 0.0)) { bad = true; break; }
        const double p2 = sqrt(m2 / m1);
        sx += p2 * m1; sy += m2 / p2;
      }
      s += sx + sy;
    }
    if (bad) {
      if (t == 0) status[grp] = 3;
      return;
    }
    const double a = variant == 0 ? 0.0 : a_star(s / d);
    const double b = sqrt(1.0 - 4.0 * a);
    for (int e = t; e < 4 * nn; e += FIT_NT) B1[e] = 0.f;
    __syncthreads();
    if (t < d) {
      const double psi = variant == 2 ? sqrt(sqrt(M2[(size_t)t * d + t] / M1[(size_t)t * d + t])) : 1.0;
      A[t] = (float)a;
      B1[(size_t)t * d + t] = (float)(b * psi);
      B2[(size_t)t * d + t] = (float)(b / psi);
      C1[(size_t)t * d + t] = (float)(-0.5 * psi * psi);
      C2[(size_t)t * d + t] = (float)(-0.5 / (psi * psi));
    }
    if (t == 0) {
      const double lbar = variant == 0 ? nan
                                       : d * log((1.0 - 4.0 * a) / sqrt(1.0 - 8.0 * a)) + (2.0 - 8.0 * a) / (1.0 - 8.0 * a) * s - sx - sy;
      write_header(th, 0.25 * d * log(1.0 - 4.0 * a), lbar, variant == 2 ? 0 : 3, variant);
      status[grp] = 0;
    }
    return;
  }

  if (variant == 4) {                                   // SDERF: one eigendecomposition of N
    double* N = w;
    double* V = w + nn;
    for (int e = t; e < nn; e += FIT_NT) {
      const int r = e / d, c = e % d;
      N[e] = M1[e] + mu4[r] * mu5[c] + mu5[r] * mu4[c] + M2[e];
    }
    __syncthreads();
    decompose(N, V, n, 0, true, sh, lds);
    for (int e = t; e < nn; e += FIT_NT) {              // B = (I - 4A)^(1/2) Q3^T: row l is the scaled eigenvector l
      const int l = e / d, c = e % d, src = sh.ord[0][l];
      const double a = a_star(fmax(sh.nrm[0][src], 0.0));
      const float bv = (float)(sqrt(1.0 - 4.0 * a) * sh.sgn[0][src] * V[(size_t)src * d + c]);
      B1[e] = bv;
      B2[e] = bv;
      C1[e] = C2[e] = l == c ? -0.5f : 0.f;
      if (c == 0) A[l] = (float)a;
    }
    // the per-eigenvalue terms of log D and of the objective in parallel (the logarithms are the expensive part),
    // their sums in eigenvalue order by one thread
    if (t < d) {
      const double lam = fmax(sh.nrm[0][sh.ord[0][t]], 0.0), a = a_star(lam);
      sh.nrm[1][t] = 0.25 * log(1.0 - 4.0 * a);
      sh.nrm[2][t] = log(1.0 - 4.0 * a) - 0.5 * log(1.0 - 8.0 * a) + (1.0 + 1.0 / (1.0 - 8.0 * a)) * lam;
    }
    __syncthreads();
    if (t == 0) {
      double logD = 0.0, lbar = -tr1 - tr2;
      for (int l = 0; l < d; ++l) { logD += sh.nrm[1][l]; lbar += sh.nrm[2][l]; }
      write_header(th, logD, lbar, 3, variant);
      status[grp] = 0;
    }
    return;
  }

  // ADERF: eig M1, eig M2, SVD of Z = L1^(1/2) Q1^T Q2 L2^(1/2)
  double* G1 = w;
  double* V1 = w + nn;
  double* G2 = w + 2 * (size_t)nn;
  double* V2 = w + 3 * (size_t)nn;
  double* Z = w + 4 * (size_t)nn;      // column-major
  double* b1 = w + 5 * (size_t)nn;     // row-major
  double* b2 = w + 6 * (size_t)nn;
  for (int e = t; e < nn; e += FIT_NT) {
    const double rd = (e / d == e % d) ? ridge : 0.0;
    G1[e] = M1[e] + rd;
    G2[e] = M2[e] + rd;
  }
  __syncthreads();
  decompose(G1, V1, n, 0, true, sh, lds);
  decompose(G2, V2, n, 1, true, sh, lds);
  {
    const double l1max = sh.nrm[0][sh.ord[0][0]], l1min = sh.nrm[0][sh.ord[0][d - 1]];
    const double l2max = sh.nrm[1][sh.ord[1][0]], l2min = sh.nrm[1][sh.ord[1][d - 1]];
    if (!(l1min > 1e-12 * l1max) || !(l2min > 1e-12 * l2max)) {
      if (t == 0) status[grp] = 3;
      return;
    }
  }
  for (int e = t; e < nn; e += FIT_NT) {
    const int c = e / d, r = e % d;                     // Z[r][c] at Z[c * d + r]
    const int s1 = sh.ord[0][r], s2 = sh.ord[1][c];
    double acc = 0.0;
    for (int k = 0; k < d; ++k) acc += V1[(size_t)s1 * d + k] * V2[(size_t)s2 * d + k];
    Z[e] = sqrt(sh.nrm[0][s1]) * sh.sgn[0][s1] * acc * sh.sgn[1][s2] * sqrt(sh.nrm[1][s2]);
  }
  __syncthreads();
  decompose(Z, nullptr, n, 2, false, sh, lds);
  if (t == 0) {
    double trs = 0.0;
    for (int l = 0; l < d; ++l) trs += sh.nrm[2][l];
    sh.red[0] = trs;
  }
  __syncthreads();
  const double trs = sh.red[0], sigmin = sh.nrm[2][sh.ord[2][d - 1]];
  if (!(sigmin > 0.0)) {
    if (t == 0) status[grp] = 3;
    return;
  }
  const double mu3 = dot / d;
  const double a = a_star(2.0 * trs / d + 2.0 * mu3);
  const double b = sqrt(1.0 - 4.0 * a);
  // B1 = b S^(1/2) U^T L1^(-1/2) Q1^T,  B2 = b S^(-1/2) U^T L1^(1/2) Q1^T
  for (int e = t; e < nn; e += FIT_NT) {
    const int r = e / d, c = e % d, s3 = sh.ord[2][r];
    const double sig = sh.nrm[2][s3];
    double t1 = 0.0, t2 = 0.0;
    for (int k = 0; k < d; ++k) {
      const int s1 = sh.ord[0][k];
      const double uq = Z[(size_t)s3 * d + k] / sig * sh.sgn[0][s1] * V1[(size_t)s1 * d + c];
      const double rl = sqrt(sh.nrm[0][s1]);
      t1 += uq / rl;
      t2 += uq * rl;
    }
    b1[e] = b * sqrt(sig) * t1;
    b2[e] = b / sqrt(sig) * t2;
    B1[e] = (float)b1[e];
    B2[e] = (float)b2[e];
  }
  __syncthreads();
  for (int e = t; e < nn; e += FIT_NT) {                // C^(k) = -B^(k)T B^(k) / (2 (1 - 4a))
    const int r = e / d, c = e % d;
    double t1 = 0.0, t2 = 0.0;
    for (int k = 0; k < d; ++k) {
      t1 += b1[(size_t)k * d + r] * b1[(size_t)k * d + c];
      t2 += b2[(size_t)k * d + r] * b2[(size_t)k * d + c];
    }
    C1[e] = (float)(-t1 / (2.0 * (1.0 - 4.0 * a)));
    C2[e] = (float)(-t2 / (2.0 * (1.0 - 4.0 * a)));
  }
  if (t < d) A[t] = (float)a;
  if (t == 0) {
    const double lbar = d * (log(1.0 - 4.0 * a) - 0.5 * log(1.0 - 8.0 * a) + 2.0 / (1.0 - 8.0 * a) * (trs / d + mu3) + 2.0 * mu3);
    write_header(th, 0.25 * d * log(1.0 - 4.0 * a), lbar, 0, variant);
    status[grp] = 0;
  }
}

}  // namespace

size_t fit_device_workspace_doubles(int d, int groups) { return (size_t)groups * 7 * d * d; }

int launch_fit_device(int variant, int d, int groups, const double* stats, double ridge, double* ws, float* theta,
                      int* status, size_t theta_floats, hipStream_t st) {
  if (d < 1 || d > FIT_DMAX) return 2;
  const size_t lds = (size_t)(d <= 96 ? 2 : 1) * d * (d + 1) * sizeof(double);
  if (lds > 0 && hipFuncSetAttribute((const void*)k_fit_device, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
    (void)hipGetLastError();
    return 2;
  }
  hipLaunchKernelGGL(k_fit_device, dim3(groups), dim3(FIT_NT), lds, st, variant, d, stats, ridge, ws, theta, status,
                     theta_floats);
  if (hipGetLastError() != hipSuccess) return 5;
  return 0;
}

}  // namespace fs
