// Kernel operator K^(alpha)(X, Y) C for a few right-hand sides (Section 2.1, the problem statement): out = P (S^T C)
// with fp32 rows, fp32 arithmetic on v_mfma_f32_16x16x4_f32 tiles and every scale kept (Section 2.3: the
// exp(alpha |.|^2) factors, D, M^-1/2).  Shapes: d a multiple of 4 up to 64, M a multiple of 16, n <= 16 columns.
//
// Four launches: k_op_pre (projection constants, per-feature norms), k_op_state (one workgroup per 64 key rows:
// S^T C of those rows on the workgroup's own shift), k_op_reduce (sum over the workgroups on the common shift),
// k_op_apply (one workgroup per 64 query rows: P T, scaled back).
//
// A workgroup is eight waves; a wave owns every eighth 16-feature tile.  The 64 rows of the workgroup sit in LDS once
// (scaled by qk_scale) and from there in registers as MFMA operands for the whole kernel (lane l <-> row l % 16 of a
// 16-row tile, contraction index 4 k4 + l / 16); the projection slice of a feature tile is eight registers read
// straight from global memory one tile ahead.  With MFMA operand layout A[l%16][l/16], B[l/16][l%16], D[4(l/16)+r][l%16]:
//   key side    E = X W^T      (A = rows, B = W~)     -> lane <-> feature, registers <-> rows 4g .. 4g+3: S^T as A operand
//               T_tile += S^T C (B = C rows 4g + r, one MFMA per register r)
//   query side  E^T = W X^T    (A = W~, B = rows; the same two register images with their roles exchanged)
//                                                      -> lane <-> row, registers <-> features: P^T as B operand
//               out^T += T^T P^T (A = T rows 4g + r of the tile)
// Exponents live in the log2 domain.  Shifts come from the Cauchy-Schwarz bounds bias_m + |W~_m| |x|, maximised over
// the features from their norms alone (no projection pass to find exact maxima): any shift that keeps the factors in
// range is exact, because it is applied back at the end (through the exponent field: the sum of two bounds may
// leave the fp32 exponent range although the result does not).  What the bounds cannot see is the angle between x
// and W~_m: a row all of whose true exponents lie more than about 2^120 below its bound flushes to zero.
#include <algorithm>

#include "fast_common.h"

namespace fs {
namespace op {

constexpr int RW = 64;          // rows per workgroup
constexpr int NTH = 512;        // threads per workgroup: eight waves, two per SIMD
constexpr int NWV = NTH / 64;
constexpr int NC = 16;          // right-hand-side columns (padded)
constexpr int DMAX = 64;
// (the kernels are instantiated for 8 and 16 contraction steps of a projection: d <= 32 and d <= 64; operands of
// the steps past d / 4 are zero)

__device__ __forceinline__ f32x4 mfma4(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

struct OpArgs {
  TensorDev X;            // rows of this side ([N, d] f32)
  const float* theta;     // one parameter set
  const float* W;         // [2][M][d] fp32, log2e folded in
  const float* bias;      // [2][M]
  const float* wnorm;     // [2][M]: |W~_m|
  const float* C;         // [Ny][n]
  float* Tpart;           // [nwg][M][NC]
  float* tshift;          // [nwg]
  float* T;               // [M][NC]
  float* tstar;           // [1]
  float* out;             // [Nx][n]
  int N, d, M, n, nwg;
  float scale, alpha;
};

// ---------------------------------------------------------------------------------------------------
// Projection constants (Section 4, evaluation recipe): W~[side][m,:] = log2e omega_m^T B_side, bias[side][m] = log2e
// (omega_m^T A omega_m + log D - 1/2 log M), wnorm[side][m] = |W~[side][m,:]|.  grid (M/4, 2), block 256: a wave per
// feature, lane c handles column c.
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_op_pre(const float* theta, const float* Omega, int M, int d, float* W,
                                                float* bias, float* wnorm) {
  const int m = blockIdx.x * 4 + (threadIdx.x >> 6), side = blockIdx.y, c = threadIdx.x & 63;
  const float* om = Omega + (size_t)m * d;
  const float* Bm = theta + FS_THETA_HEADER_ + d + (side ? (size_t)d * d : 0);
  const float* A = theta + FS_THETA_HEADER_;
  float acc = 0.f, q = 0.f;
  if (c < d) {
    // eight rows of B requested at a time (d is a multiple of 4): the loop is a chain of memory latencies otherwise
    for (int l0 = 0; l0 < d; l0 += 8) {
      float o[8], bv[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int l = min(l0 + i, d - 1);
        o[i] = l0 + i < d ? om[l] : 0.f;
        bv[i] = Bm[l * d + c];
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) acc += o[i] * bv[i];
    }
    acc *= kLog2e;
    W[((size_t)side * M + m) * d + c] = acc;
    q = A[c] * om[c] * om[c];
  }
  float n2 = acc * acc;
#pragma unroll
  for (int s = 1; s < 64; s <<= 1) { n2 += __shfl_xor(n2, s); q += __shfl_xor(q, s); }
  if (c == 0) {
    bias[(size_t)side * M + m] = kLog2e * (q + theta[0] - 0.5f * logf((float)M));
    wnorm[(size_t)side * M + m] = sqrtf(n2);
  }
}

// Largest of n floats, as the same value in every thread of the workgroup (red: one float of LDS per wave).
__device__ __forceinline__ float block_max(const float* p, int n, float* red) {
  float v = -INFINITY;
  for (int i = threadIdx.x; i < n; i += NTH) v = fmaxf(v, p[i]);
  v = fast::wave_max(v);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  v = red[0];
#pragma unroll
  for (int i = 1; i < NWV; ++i) v = fmaxf(v, red[i]);
  __syncthreads();
  return v;
}

struct SmemOp {
  float x[RW][DMAX + 1];          // rows, scaled by qk_scale (zero past the end)
  float c[RW][NC];                // right-hand-side rows (key side) / partial outputs of one wave (query side)
  float xo[NWV][RW][NC + 1];      // partial out^T tiles of the waves: [wave][row][column]
  float rt[RW];                   // row term log2e (x^T C x + alpha |x|^2) - shift of the row / of the workgroup
  float sh[RW];                   // per-row shift (query side)
  float cs[RW];                   // largest Cauchy-Schwarz term |W~_m| |x| of the row (-inf past the end)
  float red[NWV];
};

// Rows to LDS, row terms and shifts.  Fills sm.x, sm.rt (row term) and sm.sh = row term + max over the features m of
// (bias_m + row_shift(|x|, |W~_m|)), -inf past the end.  By Cauchy-Schwarz no exponent of the row exceeds its shift by
// more than 120 binary orders, and ordinary rows end up near zero.  The maximum is taken feature by feature (not
// largest bias + largest norm): features with a long W~_m have a very negative bias when A is far from zero, and
// a bound that ignores that can sit hundreds of binary orders above every actual exponent, which would flush the
// whole row to zero.  What no norm can see is the angle between x and W~_m: the shift of a row lies at most 1.5 x its
// largest Cauchy-Schwarz term (sm.cs) above the row's largest exponent.  Workgroups with a row beyond kSafeCs = 60
// (90 binary orders at most: safe) replace the shifts by exact maxima found in a projection pass of their own.
constexpr float kSafeCs = 60.f;
__device__ __forceinline__ void stage_rows(SmemOp& sm, const OpArgs& a, int side, int row0, const float* wnorm, const float* bias) {
  const float* Xp = (const float*)a.X.ptr;
  for (int idx = threadIdx.x; idx < RW * a.d; idx += NTH) {
    const int r = idx / a.d, c = idx - r * a.d;
    sm.x[r][c] = row0 + r < a.N ? a.scale * Xp[(long long)(row0 + r) * a.X.sl + c] : 0.f;
  }
  __syncthreads();
  // eight threads per row
  const int r = threadIdx.x >> 3, part = threadIdx.x & 7;
  const bool iso = ((int)a.theta[2]) & 1;
  const float* Cm = a.theta + FS_THETA_HEADER_ + a.d + (2 + (side ? 1 : 0)) * (size_t)a.d * a.d;
  float n2 = 0.f, qf = 0.f;
  for (int i = part; i < a.d; i += 8) {
    const float xi = sm.x[r][i];
    n2 += xi * xi;
    if (!iso) {
      float t = 0.f;
      for (int j = 0; j < a.d; ++j) t += Cm[i * a.d + j] * sm.x[r][j];
      qf += xi * t;
    }
  }
  n2 += __shfl_xor(n2, 1); n2 += __shfl_xor(n2, 2); n2 += __shfl_xor(n2, 4);
  qf += __shfl_xor(qf, 1); qf += __shfl_xor(qf, 2); qf += __shfl_xor(qf, 4);
  const float len = __builtin_amdgcn_sqrtf(n2);
  float bound = -INFINITY, csmax = 0.f;
  for (int m0 = 0; m0 < a.M; m0 += 64) {
    // eight features per thread and trip, all sixteen loads in flight together (indices past the end are clamped:
    // a feature counted twice does not change a maximum)
    float wn[8], bs[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int m = min(m0 + part + 8 * u, a.M - 1);
      wn[u] = wnorm[m];
      bs[u] = bias[m];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const float cs = wn[u] * len;
      csmax = fmaxf(csmax, cs);
      bound = fmaxf(bound, bs[u] + fmaxf(fast::kBeta * cs, cs - 120.f));
    }
  }
  bound = fmaxf(bound, __shfl_xor(bound, 1)); bound = fmaxf(bound, __shfl_xor(bound, 2)); bound = fmaxf(bound, __shfl_xor(bound, 4));
  csmax = fmaxf(csmax, __shfl_xor(csmax, 1)); csmax = fmaxf(csmax, __shfl_xor(csmax, 2)); csmax = fmaxf(csmax, __shfl_xor(csmax, 4));
  if (part == 0) {
    const float rt = kLog2e * ((iso ? -0.5f * n2 : qf) + a.alpha * n2);
    sm.rt[r] = rt;
    sm.sh[r] = row0 + r < a.N ? bound + rt : -INFINITY;
    sm.cs[r] = row0 + r < a.N ? csmax : -INFINITY;
  }
  __syncthreads();
}

// ---------------------------------------------------------------------------------------------------
// Key side: Tpart[wg] = sum over the workgroup's rows j of exp2(E2_jm - t_wg) C_j, t_wg = largest row bound.
// grid ceil(Ny / 64), block 256.
// ---------------------------------------------------------------------------------------------------
template <int KMAX>
__global__ void __launch_bounds__(NTH) k_op_state(OpArgs a) {
  __shared__ SmemOp sm;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  const int row0 = blockIdx.x * RW, nk = a.d >> 2, ntile = a.M >> 4;
  const float* W2 = a.W + (size_t)a.M * a.d;
  const float* b2 = a.bias + a.M;
  stage_rows(sm, a, 1, row0, a.wnorm + a.M, b2);
  for (int idx = threadIdx.x; idx < RW * NC; idx += NTH) {
    const int r = idx / NC, col = idx - r * NC;
    sm.c[r][col] = (row0 + r < a.N && col < a.n) ? a.C[(size_t)(row0 + r) * a.n + col] : 0.f;
  }
  float twg = block_max(sm.sh, RW, sm.red);            // (its barriers also publish sm.c)
  const bool exact = block_max(sm.cs, RW, sm.red) > kSafeCs;
  // row operands, right-hand-side operands and the per-row part of the exponent, for the whole kernel
  float xr[4][KMAX], cr[4][4];
  f32x4 add[4];
#pragma unroll
  for (int tt = 0; tt < 4; ++tt) {
#pragma unroll
    for (int k4 = 0; k4 < KMAX; ++k4) xr[tt][k4] = k4 < nk ? sm.x[16 * tt + c][4 * k4 + g] : 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) cr[tt][r] = sm.c[16 * tt + 4 * g + r][c];
  }
  float wr[KMAX], wn[KMAX];
  if (exact) {
    // the workgroup's largest exponent itself: one projection pass without the exponentials
    float emax = -INFINITY;
    for (int ft = w; ft < ntile; ft += NWV) {
#pragma unroll
      for (int k4 = 0; k4 < KMAX; ++k4) wr[k4] = k4 < nk ? W2[(size_t)(16 * ft + c) * a.d + 4 * k4 + g] : 0.f;
      const float bm = b2[16 * ft + c];
      f32x4 e[4];
#pragma unroll
      for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          e[tt][r] = row0 + 16 * tt + 4 * g + r < a.N ? sm.rt[16 * tt + 4 * g + r] + bm : -INFINITY;
#pragma unroll
      for (int k4 = 0; k4 < KMAX; ++k4)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) e[tt] = mfma4(xr[tt][k4], wr[k4], e[tt]);
#pragma unroll
      for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int r = 0; r < 4; ++r) emax = fmaxf(emax, e[tt][r]);
    }
    emax = fast::wave_max(emax);
    if (lane == 0) sm.red[w] = emax;
    __syncthreads();
    twg = sm.red[0];
#pragma unroll
    for (int i = 1; i < NWV; ++i) twg = fmaxf(twg, sm.red[i]);
    __syncthreads();
  }
#pragma unroll
  for (int tt = 0; tt < 4; ++tt)
#pragma unroll
    for (int r = 0; r < 4; ++r)   // rows past the end: -inf, their features are exactly zero
      add[tt][r] = row0 + 16 * tt + 4 * g + r < a.N ? sm.rt[16 * tt + 4 * g + r] - twg : -INFINITY;
  int ft = w;
  if (ft < ntile) {
#pragma unroll
    for (int k4 = 0; k4 < KMAX; ++k4) wr[k4] = k4 < nk ? W2[(size_t)(16 * ft + c) * a.d + 4 * k4 + g] : 0.f;
  }
  for (; ft < ntile; ft += NWV) {
    const float bm = b2[16 * ft + c];
    if (ft + NWV < ntile) {
#pragma unroll
      for (int k4 = 0; k4 < KMAX; ++k4) wn[k4] = k4 < nk ? W2[(size_t)(16 * (ft + NWV) + c) * a.d + 4 * k4 + g] : 0.f;
    }
    // four independent chains (one per 16-row tile), summed at the end
    f32x4 e[4], tq[4];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) { e[tt] = add[tt] + bm; tq[tt] = f32x4{0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
    for (int k4 = 0; k4 < KMAX; ++k4)
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) e[tt] = mfma4(xr[tt][k4], wr[k4], e[tt]);
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) tq[tt] = mfma4(fast_exp2(e[tt][r]), cr[tt][r], tq[tt]);
    const f32x4 t = (tq[0] + tq[1]) + (tq[2] + tq[3]);
    float* out = a.Tpart + ((size_t)blockIdx.x * a.M + 16 * ft + 4 * g) * NC + c;
#pragma unroll
    for (int r = 0; r < 4; ++r) out[(size_t)r * NC] = t[r];
#pragma unroll
    for (int k4 = 0; k4 < KMAX; ++k4) wr[k4] = wn[k4];
  }
  if (threadIdx.x == 0) a.tshift[blockIdx.x] = twg;
}

// T = sum_wg Tpart[wg] 2^(t_wg - t*), t* = max t_wg.  grid ceil(M * NC / 64), block 256: 64 consecutive elements per
// workgroup, the workgroups' partial states dealt to the four waves.
__global__ void __launch_bounds__(256) k_op_reduce(const float* Tpart, const float* tshift, float* T, float* tstar,
                                                   int nwg, int total) {
  __shared__ float red[4], part[4][64];
  float ts = -INFINITY;
  for (int i = threadIdx.x; i < nwg; i += 256) ts = fmaxf(ts, tshift[i]);
  ts = fast::wave_max(ts);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ts;
  __syncthreads();
  ts = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  const int e = blockIdx.x * 64 + (threadIdx.x & 63), q = threadIdx.x >> 6;
  float acc = 0.f;
  if (e < total) {
#pragma unroll 8
    for (int i = q; i < nwg; i += 4) acc += Tpart[(size_t)i * total + e] * fast_exp2(tshift[i] - ts);
  }
  part[q][threadIdx.x & 63] = acc;
  __syncthreads();
  if (q == 0 && e < total) T[e] = (part[0][threadIdx.x] + part[1][threadIdx.x]) + (part[2][threadIdx.x] + part[3][threadIdx.x]);
  if (blockIdx.x == 0 && threadIdx.x == 0) tstar[0] = ts;
}

// ---------------------------------------------------------------------------------------------------
// Query side: out_i = 2^(s_i + t*) sum_m exp2(E1_im - s_i) T_m, s_i = the row's bound.  grid ceil(Nx / 64), block 256.
// ---------------------------------------------------------------------------------------------------
template <int KMAX>
__global__ void __launch_bounds__(NTH) k_op_apply(OpArgs a) {
  __shared__ SmemOp sm;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  const int row0 = blockIdx.x * RW, nk = a.d >> 2, ntile = a.M >> 4;
  stage_rows(sm, a, 0, row0, a.wnorm, a.bias);
  const bool exact = block_max(sm.cs, RW, sm.red) > kSafeCs;
  float xr[4][KMAX], add[4];
#pragma unroll
  for (int tt = 0; tt < 4; ++tt) {
#pragma unroll
    for (int k4 = 0; k4 < KMAX; ++k4) xr[tt][k4] = k4 < nk ? sm.x[16 * tt + c][4 * k4 + g] : 0.f;
  }
  float wr[KMAX], wn[KMAX];
  if (exact) {
    // every row's largest exponent itself: one projection pass without the exponentials; a wave's maxima of row
    // 16 tt + c end up in its lanes (., c), the waves meet in LDS
    float rmax[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    for (int ft = w; ft < ntile; ft += NWV) {
#pragma unroll
      for (int k4 = 0; k4 < KMAX; ++k4) wr[k4] = k4 < nk ? a.W[(size_t)(16 * ft + c) * a.d + 4 * k4 + g] : 0.f;
      f32x4 bm;
#pragma unroll
      for (int r = 0; r < 4; ++r) bm[r] = a.bias[16 * ft + 4 * g + r];
      f32x4 e[4];
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) e[tt] = bm + sm.rt[16 * tt + c];
#pragma unroll
      for (int k4 = 0; k4 < KMAX; ++k4)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) e[tt] = mfma4(wr[k4], xr[tt][k4], e[tt]);
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) rmax[tt] = fmaxf(rmax[tt], fmaxf(fmaxf(e[tt][0], e[tt][1]), fmaxf(e[tt][2], e[tt][3])));
    }
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
      rmax[tt] = fmaxf(rmax[tt], __shfl_xor(rmax[tt], 16));
      rmax[tt] = fmaxf(rmax[tt], __shfl_xor(rmax[tt], 32));
      if (g == 0) sm.xo[w][16 * tt + c][0] = rmax[tt];
    }
    __syncthreads();
    if (threadIdx.x < RW) {
      float m = sm.xo[0][threadIdx.x][0];
#pragma unroll
      for (int wv = 1; wv < NWV; ++wv) m = fmaxf(m, sm.xo[wv][threadIdx.x][0]);
      sm.sh[threadIdx.x] = m;
    }
    __syncthreads();
  }
#pragma unroll
  for (int tt = 0; tt < 4; ++tt)   // the row's own part of the exponent minus its shift (rows past the end: their results are not stored)
    add[tt] = row0 + 16 * tt + c < a.N ? sm.rt[16 * tt + c] - sm.sh[16 * tt + c] : 0.f;
  f32x4 o[4];
#pragma unroll
  for (int tt = 0; tt < 4; ++tt) o[tt] = f32x4{0.f, 0.f, 0.f, 0.f};
  f32x4 tr, tn;
  int ft = w;
  if (ft < ntile) {
#pragma unroll
    for (int k4 = 0; k4 < KMAX; ++k4) wr[k4] = k4 < nk ? a.W[(size_t)(16 * ft + c) * a.d + 4 * k4 + g] : 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) tr[r] = a.T[(size_t)(16 * ft + 4 * g + r) * NC + c];
  }
  for (; ft < ntile; ft += NWV) {
    f32x4 bm;
#pragma unroll
    for (int r = 0; r < 4; ++r) bm[r] = a.bias[16 * ft + 4 * g + r];
    if (ft + NWV < ntile) {
#pragma unroll
      for (int k4 = 0; k4 < KMAX; ++k4) wn[k4] = k4 < nk ? a.W[(size_t)(16 * (ft + NWV) + c) * a.d + 4 * k4 + g] : 0.f;
#pragma unroll
      for (int r = 0; r < 4; ++r) tn[r] = a.T[(size_t)(16 * (ft + NWV) + 4 * g + r) * NC + c];
    }
    f32x4 e[4];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) e[tt] = bm + add[tt];
#pragma unroll
    for (int k4 = 0; k4 < KMAX; ++k4)
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) e[tt] = mfma4(wr[k4], xr[tt][k4], e[tt]);
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) o[tt] = mfma4(tr[r], fast_exp2(e[tt][r]), o[tt]);
#pragma unroll
    for (int k4 = 0; k4 < KMAX; ++k4) wr[k4] = wn[k4];
    tr = tn;
  }
  // o[tt]: rows = columns 4g + r of the right-hand side, column = row 16 tt + c of the workgroup
#pragma unroll
  for (int tt = 0; tt < 4; ++tt)
#pragma unroll
    for (int r = 0; r < 4; ++r) sm.xo[w][16 * tt + c][4 * g + r] = o[tt][r];
  __syncthreads();
  const float ts = a.tstar[0];
  for (int idx = threadIdx.x; idx < RW * a.n; idx += NTH) {
    const int r = idx / a.n, col = idx - r * a.n;
    if (row0 + r < a.N) {
      float v = 0.f;
#pragma unroll
      for (int wv = 0; wv < NWV; ++wv) v += sm.xo[wv][r][col];
      // v 2^(s_i + t*): the two shifts are bounds and may add up to more than the fp32 exponent range although the
      // result is representable, so the power of two is applied through the exponent field, not as a factor
      const float sft = sm.sh[r] + ts, whole = floorf(sft);
      a.out[(size_t)(row0 + r) * a.n + col] = ldexpf(v * fast_exp2(sft - whole), (int)fminf(fmaxf(whole, -1000.f), 1000.f));
    }
  }
}

}  // namespace op

bool op_supported(int dtype_x, int dtype_y, int d, int M, int n) {
  return dtype_x == 0 && dtype_y == 0 && d % 4 == 0 && d <= op::DMAX && M % 16 == 0 && n <= op::NC;
}

// Floats of workspace: W, bias, wnorm, partial states and their shifts, the state and its shift.
size_t op_workspace_floats(int Ny, int d, int M) {
  const size_t nwg = (Ny + op::RW - 1) / op::RW;
  return (size_t)2 * M * d + 4 * (size_t)M + nwg * M * op::NC + nwg + (size_t)M * op::NC + 64;
}

#define FS_LAUNCH_CHECK() do { if (hipGetLastError() != hipSuccess) return 5; } while (0)

int launch_op_matvec(const float* theta, const TensorDev& X, const TensorDev& Y, int Nx, int Ny, int d, float scale,
                     float alpha, const float* Omega, int M, const float* C, int n, float* out, float* ws, hipStream_t st) {
  const int nwg = (Ny + op::RW - 1) / op::RW;
  float* W = ws;
  float* bias = W + (size_t)2 * M * d;
  float* wnorm = bias + (size_t)2 * M;
  float* Tpart = wnorm + (size_t)2 * M;
  float* tshift = Tpart + (size_t)nwg * M * op::NC;
  float* T = tshift + nwg;
  float* tstar = T + (size_t)M * op::NC;
  hipLaunchKernelGGL(op::k_op_pre, dim3(M / 4, 2), dim3(256), 0, st, theta, Omega, M, d, W, bias, wnorm);
  FS_LAUNCH_CHECK();
  op::OpArgs a;
  a.theta = theta; a.W = W; a.bias = bias; a.wnorm = wnorm; a.C = C; a.Tpart = Tpart; a.tshift = tshift; a.T = T;
  a.tstar = tstar; a.out = out; a.d = d; a.M = M; a.n = n; a.nwg = nwg; a.scale = scale; a.alpha = alpha;
  a.X = Y; a.N = Ny;
  if (d <= 32) hipLaunchKernelGGL(op::k_op_state<8>, dim3(nwg), dim3(op::NTH), 0, st, a);
  else hipLaunchKernelGGL(op::k_op_state<16>, dim3(nwg), dim3(op::NTH), 0, st, a);
  FS_LAUNCH_CHECK();
  const int total = M * op::NC;
  hipLaunchKernelGGL(op::k_op_reduce, dim3((total + 63) / 64), dim3(256), 0, st, Tpart, tshift, T, tstar, nwg, total);
  FS_LAUNCH_CHECK();
  a.X = X; a.N = Nx;
  if (d <= 32) hipLaunchKernelGGL(op::k_op_apply<8>, dim3((Nx + op::RW - 1) / op::RW), dim3(op::NTH), 0, st, a);
  else hipLaunchKernelGGL(op::k_op_apply<16>, dim3((Nx + op::RW - 1) / op::RW), dim3(op::NTH), 0, st, a);
  FS_LAUNCH_CHECK();
  return 0;
}

}  // namespace fs
