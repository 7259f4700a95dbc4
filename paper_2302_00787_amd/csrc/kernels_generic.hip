// General-shape FAVOR# kernels: fp32 arithmetic on fp32 MFMA tiles (v_mfma_f32_16x16x4_f32), any d <= 128,
// any M, any sequence length, f32 or bf16 storage.  They serve the fp32 workloads and every shape the
// bf16 fast path does not cover.  All exponents are kept in the log2 domain: the projection matrices and
// biases arrive pre-multiplied by log2(e), so a feature is exp2(E2 - shift).
//
// Tile shape everywhere: 32 rows (tokens) x 32 features per step, 256 threads = 4 waves.
// MFMA 16x16x4 f32 operand layout used below: lane l supplies A[l%16][l/16] and B[l/16][l%16];
// accumulator register r of lane l is D[4*(l/16) + r][l%16].
#include "fs_common.h"
#include "kernels.h"

namespace fs {

constexpr int TR = 32;     // rows per tile
constexpr int MB = 32;     // features per block
constexpr int NT = 256;    // threads per workgroup

constexpr int ACC_PER_WAVE = 5;   // ceil(2 * MAXVT / 4)

// This side's C matrix, or nullptr when the parameter set says C = -I/2 (flag bit 0 of the theta header).
__device__ __forceinline__ const float* side_cmat(const GenSide& s, int b, int h, int H) {
  const float* th = s.theta + (size_t)group_of(s.groups, b, h, H) * s.theta_stride;
  return (((int)th[2]) & 1) ? nullptr : th + s.c_offset;
}

__device__ __forceinline__ f32x4 mfma4(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// dst[r][c] = scale * T[row0 + r][c] for r < 32; zero outside [0, nrows) x [0, ncols); columns up to ncols_pad written.
__device__ void load_rows(float* dst, int ld, const TensorDev& t, long long base, int row0, int nrows,
                          int ncols, int ncols_pad, float scale) {
  for (int idx = threadIdx.x; idx < TR * ncols_pad; idx += NT) {
    const int r = idx / ncols_pad, c = idx - r * ncols_pad;
    float v = 0.f;
    if (row0 + r < nrows && c < ncols) v = scale * load_elem(t, base + (long long)(row0 + r) * t.sl + c);
    dst[r * ld + c] = v;
  }
}

// Value tile with an optional column of ones at index ncols (the normaliser column of attention).
__device__ void load_values(float* dst, int ld, const TensorDev& t, long long base, int row0, int nrows,
                            int ncols, int ncols_pad, int append_ones) {
  for (int idx = threadIdx.x; idx < TR * ncols_pad; idx += NT) {
    const int r = idx / ncols_pad, c = idx - r * ncols_pad;
    float v = 0.f;
    if (row0 + r < nrows) {
      if (c < ncols) v = load_elem(t, base + (long long)(row0 + r) * t.sl + c);
      else if (c == ncols && append_ones) v = 1.f;
    }
    dst[r * ld + c] = v;
  }
}

// Ws[f][c] = W[m0 + f][c] (zero rows past M), bias_s[f] = bias[m0 + f].
__device__ void load_wblock(float* Ws, float* bias_s, int ld, const float* W, const float* bias, int m0, int M,
                            int d, int dpad) {
  for (int idx = threadIdx.x; idx < MB * dpad; idx += NT) {
    const int f = idx / dpad, c = idx - f * dpad;
    Ws[f * ld + c] = (m0 + f < M && c < d) ? W[(long long)(m0 + f) * d + c] : 0.f;
  }
  if (threadIdx.x < MB) bias_s[threadIdx.x] = (m0 + threadIdx.x < M) ? bias[m0 + threadIdx.x] : 0.f;
}

// The same block travelling global -> registers -> LDS, so that the load of the next block is in flight while the
// current one is used: thread t carries row f = t/8 of the block, columns t%8 + 8i (dpad <= 128: at most 16).
struct WRegs { float w[16]; float b; };
__device__ __forceinline__ void wblock_fetch(WRegs& r, const float* W, const float* bias, int m0, int M, int d, int dpad) {
  const int f = threadIdx.x >> 3, c0 = threadIdx.x & 7;
  const float* row = W + (long long)(m0 + f) * d;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int c = c0 + 8 * i;
    r.w[i] = 0.f;
    if (8 * i < dpad && m0 + f < M && c < d) r.w[i] = row[c];
  }
  r.b = (threadIdx.x < MB && m0 + threadIdx.x < M) ? bias[m0 + threadIdx.x] : 0.f;
}
__device__ __forceinline__ void wblock_put(const WRegs& r, float* Ws, float* bias_s, int ld, int dpad) {
  const int f = threadIdx.x >> 3, c0 = threadIdx.x & 7;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int c = c0 + 8 * i;
    if (8 * i < dpad && c < dpad) Ws[f * ld + c] = r.w[i];
  }
  if (threadIdx.x < MB) bias_s[threadIdx.x] = r.b;
}

// ((C + C^T) x)[c] for a dense C (four partial sums and several loads in flight: a plain loop is a chain of cache
// latencies).
__device__ __forceinline__ float sym_row_dot(const float* Cmat, int d, int c, const float* x) {
  const float* crow = Cmat + (size_t)c * d;
  const float* ccol = Cmat + c;
  float t0 = 0.f, t1 = 0.f, t2 = 0.f, t3 = 0.f;
  int a = 0;
#pragma unroll 2
  for (; a + 4 <= d; a += 4) {
    t0 += (crow[a] + ccol[(size_t)a * d]) * x[a];
    t1 += (crow[a + 1] + ccol[(size_t)(a + 1) * d]) * x[a + 1];
    t2 += (crow[a + 2] + ccol[(size_t)(a + 2) * d]) * x[a + 2];
    t3 += (crow[a + 3] + ccol[(size_t)(a + 3) * d]) * x[a + 3];
  }
  for (; a < d; ++a) t0 += (crow[a] + ccol[(size_t)a * d]) * x[a];
  return (t0 + t1) + (t2 + t3);
}

// rterm[r] = log2e * (x_r^T C x_r + alpha |x_r|^2); Cmat == nullptr means C = -I/2.
__device__ void row_terms(float* rterm, const float* Xs, int ld, int d, const float* Cmat, float alpha) {
  const int r = threadIdx.x >> 3, part = threadIdx.x & 7;
  const float* x = Xs + r * ld;
  float acc = 0.f;
  if (Cmat == nullptr) {
    for (int a = part; a < d; a += 8) acc += x[a] * x[a];
    acc *= (alpha - 0.5f);
  } else {
    // (eight loads of the row of C in flight and four partial sums: the loop is a chain of cache latencies otherwise)
    for (int a = part; a < d; a += 8) {
      const float* crow = Cmat + (size_t)a * d;
      float t0 = 0.f, t1 = 0.f, t2 = 0.f, t3 = 0.f;
      int b = 0;
#pragma unroll 2
      for (; b + 4 <= d; b += 4) {
        t0 += crow[b] * x[b];
        t1 += crow[b + 1] * x[b + 1];
        t2 += crow[b + 2] * x[b + 2];
        t3 += crow[b + 3] * x[b + 3];
      }
      for (; b < d; ++b) t0 += crow[b] * x[b];
      acc += x[a] * ((t0 + t1) + (t2 + t3) + alpha * x[a]);
    }
  }
  acc += __shfl_xor(acc, 1);
  acc += __shfl_xor(acc, 2);
  acc += __shfl_xor(acc, 4);
  if (part == 0) rterm[r] = kLog2e * acc;
}

// Row terms of the 32-row tile at row0 of (b,h): from the side's table when the call keeps one, else computed.
__device__ void row_terms_of(float* rterm, const GenSide& sd, int bh, int L, int row0, int row_end, const float* Xs,
                             int ld, int d, const float* Cmat, float alpha) {
  if (sd.rk != nullptr) {
    if (threadIdx.x < TR) rterm[threadIdx.x] = row0 + (int)threadIdx.x < row_end ? sd.rk[(size_t)bh * L + row0 + threadIdx.x] : 0.f;
  } else {
    row_terms(rterm, Xs, ld, d, Cmat, alpha);
  }
}

// Wave w computes the 16x16 tile (row tile w>>1, feature tile w&1) of Xs * Ws^T.
__device__ __forceinline__ f32x4 proj_tile(const float* Xs, const float* Ws, int ld, int dpad) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const float* ap = Xs + ((w >> 1) * 16 + (lane & 15)) * ld + (lane >> 4);
  const float* bp = Ws + ((w & 1) * 16 + (lane & 15)) * ld + (lane >> 4);
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int k = 0; k < dpad; k += 4) acc = mfma4(ap[k], bp[k], acc);
  return acc;
}

// Max of e[0..3] over the 16 lanes that share lane>>4, combined into LDS (ordered-uint image) per row.
__device__ __forceinline__ void rowmax_update(uint32_t* rowmax_u, const float e[4]) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    float v = e[r];
    v = fmaxf(v, __shfl_xor(v, 1));
    v = fmaxf(v, __shfl_xor(v, 2));
    v = fmaxf(v, __shfl_xor(v, 4));
    v = fmaxf(v, __shfl_xor(v, 8));
    if ((lane & 15) == 0) atomicMax(&rowmax_u[(w >> 1) * 16 + 4 * (lane >> 4) + r], float_to_ordered(v));
  }
}

// One pass over all feature blocks computing, per row, max_m (W_m . x + bias_m) (+ rterm is added by the caller).
__device__ void rowmax_pass(uint32_t* rowmax_u, const float* Xs, float* Ws, float* bias_s, int ld, const float* W,
                            const float* bias, int M, int d, int dpad) {
  if (threadIdx.x < TR) rowmax_u[threadIdx.x] = 0u;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  WRegs wr;
  wblock_fetch(wr, W, bias, 0, M, d, dpad);
  for (int m0 = 0; m0 < M; m0 += MB) {
    __syncthreads();
    wblock_put(wr, Ws, bias_s, ld, dpad);
    __syncthreads();
    if (m0 + MB < M) wblock_fetch(wr, W, bias, m0 + MB, M, d, dpad);
    const f32x4 acc = proj_tile(Xs, Ws, ld, dpad);
    const int f = (w & 1) * 16 + (lane & 15);
    float e[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) e[r] = (m0 + f < M) ? acc[r] + bias_s[f] : -INFINITY;
    rowmax_update(rowmax_u, e);
  }
  __syncthreads();
}

// ---------------------------------------------------------------------------------------------------
// Projection constants (Section 4, evaluation recipe): W~[m,:] = log2e * omega_m^T B, bias_m = log2e *
// (omega_m^T A omega_m + log D - 1/2 log M).  grid (M, 2 sides, pgroups), block 128.
// ---------------------------------------------------------------------------------------------------
__global__ void k_prep(const float* theta, int groups, const float* Omega, int omega_groups, int pgroups,
                       int B, int H, int M, int d, float* W, uint16_t* Wbf, float* bias) {
  const int m = blockIdx.x, side = blockIdx.y, pg = blockIdx.z;
  int b = 0, h = 0;
  if (pgroups == H && pgroups != 1) h = pg;
  else if (pgroups != 1) { b = pg / H; h = pg % H; }
  const size_t tf = FS_THETA_HEADER_ + (size_t)d + 4 * (size_t)d * d;
  const float* th = theta + (size_t)group_of(groups, b, h, H) * tf;
  const float* om = Omega + ((size_t)group_of(omega_groups, b, h, H) * M + m) * d;
  const float* Bm = th + FS_THETA_HEADER_ + d + (side ? (size_t)d * d : 0);
  const size_t o = (((size_t)pg * 2 + side) * M + m);
  const int c = threadIdx.x;
  if (c < d) {
    float acc = 0.f;
    for (int l = 0; l < d; ++l) acc += om[l] * Bm[l * d + c];
    acc *= kLog2e;
    W[o * d + c] = acc;
    Wbf[o * d + c] = f32_to_bf16_bits(acc);
  }
  if (c == 0) {
    const float* A = th + FS_THETA_HEADER_;
    float q = 0.f;
    for (int l = 0; l < d; ++l) q += A[l] * om[l] * om[l];
    bias[o] = kLog2e * (q + th[0] - 0.5f * logf((float)M));
  }
}

__global__ void k_fill_u32(uint32_t* p, uint32_t v, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// ---------------------------------------------------------------------------------------------------
// Materialised features (Section 2.1, rows of P or S).  grid (ceil(n/32)), dynamic LDS.
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(NT) k_gen_features(TensorDev X, int n, int d, float scale, float alpha,
                                                     const float* W, const float* bias, const float* theta,
                                                     long long c_offset, int M, float* out, float* row_logscale) {
  extern __shared__ float smem[];
  const int dpad = (d + 3) & ~3, ld = dpad + 1;
  float* Xs = smem;
  float* Ws = Xs + TR * ld;
  float* bias_s = Ws + MB * ld;
  float* rterm = bias_s + MB;
  uint32_t* rowmax_u = (uint32_t*)(rterm + TR);
  const int row0 = blockIdx.x * TR;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const float* Cmat = (((int)theta[2]) & 1) ? nullptr : theta + c_offset;

  load_rows(Xs, ld, X, 0, row0, n, d, dpad, scale);
  __syncthreads();
  row_terms(rterm, Xs, ld, d, Cmat, alpha);
  __syncthreads();
  if (row_logscale != nullptr) {
    rowmax_pass(rowmax_u, Xs, Ws, bias_s, ld, W, bias, M, d, dpad);
    if (threadIdx.x < TR && row0 + threadIdx.x < n)
      row_logscale[row0 + threadIdx.x] = (ordered_to_float(rowmax_u[threadIdx.x]) + rterm[threadIdx.x]) * kLn2;
  }
  for (int m0 = 0; m0 < M; m0 += MB) {
    __syncthreads();
    load_wblock(Ws, bias_s, ld, W, bias, m0, M, d, dpad);
    __syncthreads();
    const f32x4 acc = proj_tile(Xs, Ws, ld, dpad);
    const int f = (w & 1) * 16 + (lane & 15);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = (w >> 1) * 16 + 4 * (lane >> 4) + r;
      float e = acc[r] + bias_s[f];
      e = (row_logscale != nullptr) ? e - ordered_to_float(rowmax_u[row]) : e + rterm[row];
      if (row0 + row < n && m0 + f < M) out[(size_t)(row0 + row) * M + m0 + f] = fast_exp2(e);
    }
  }
}

// ---------------------------------------------------------------------------------------------------
// Key-side maximum of the exponent per (b, h): kmax[bh] = max_{j,m} E2[j,m] (ordered-uint image, atomicMax).
// grid (ceil(Lk/32), B*H).
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(NT) k_gen_kmax(GenSide ks, int Lk, int H, int M, int d, uint32_t* kmax_u) {
  extern __shared__ float smem[];
  const int dpad = (d + 3) & ~3, ld = dpad + 1;
  float* Xs = smem;
  float* Ws = Xs + TR * ld;
  float* bias_s = Ws + MB * ld;
  float* rterm = bias_s + MB;
  uint32_t* rowmax_u = (uint32_t*)(rterm + TR);
  const int bh = blockIdx.y, b = bh / H, h = bh % H;
  const int row0 = blockIdx.x * TR;
  const int pg = group_of(ks.pgroups, b, h, H);
  const float* W = ks.W + ((size_t)pg * 2 + 1) * M * d;
  const float* bias = ks.bias + ((size_t)pg * 2 + 1) * M;
  const float* Cmat = side_cmat(ks, b, h, H);

  load_rows(Xs, ld, ks.X, b * ks.X.sb + h * ks.X.sh, row0, Lk, d, dpad, ks.scale);
  __syncthreads();
  row_terms(rterm, Xs, ld, d, Cmat, ks.alpha);
  rowmax_pass(rowmax_u, Xs, Ws, bias_s, ld, W, bias, M, d, dpad);
  if (threadIdx.x < 64) {
    float v = (threadIdx.x < TR && row0 + threadIdx.x < Lk)
                  ? ordered_to_float(rowmax_u[threadIdx.x]) + rterm[threadIdx.x] : -INFINITY;
    for (int s = 1; s < 64; s <<= 1) v = fmaxf(v, __shfl_xor(v, s));
    if (threadIdx.x == 0) atomicMax(&kmax_u[bh], float_to_ordered(v));
    if (ks.rk != nullptr && threadIdx.x < TR && row0 + (int)threadIdx.x < Lk) ks.rk[(size_t)bh * Lk + row0 + threadIdx.x] = rterm[threadIdx.x];
  }
}

// ---------------------------------------------------------------------------------------------------
// Key-side partial states (Section 2.1, S^T C): Tpart[bh][seg][m][v] = sum_{j in seg} exp2(E2[j,m] - kmax) * V1[j,v].
// grid (nseg, ceil(M/32), B*H).
// ---------------------------------------------------------------------------------------------------
// With row_shift != nullptr the kernel serves the backward pass on the query side: features of side 1 with the
// per-row shifts the forward pass used (no row term in the exponent), "values" = the rows of the output gradient.
__global__ void __launch_bounds__(NT) k_gen_state(GenSide ks, TensorDev V, int Lk, int H, int M, int d, int nv,
                                                  int append_ones, int ldt, int rows_per_seg, int nseg,
                                                  const uint32_t* kmax_u, const float* row_shift, float* Tpart) {
  extern __shared__ float smem[];
  const int dpad = (d + 3) & ~3, ld = dpad + 1, ldv = ldt + 1, lds = MB + 1;
  float* Xs = smem;
  float* Ws = Xs + TR * ld;
  float* Vs = Ws + MB * ld;
  float* Ss = Vs + TR * ldv;
  float* bias_s = Ss + TR * lds;
  float* rterm = bias_s + MB;
  const int seg = blockIdx.x, m0 = blockIdx.y * MB, bh = blockIdx.z, b = bh / H, h = bh % H;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int pg = group_of(ks.pgroups, b, h, H);
  const int side = row_shift == nullptr ? 1 : 0;
  const float* W = ks.W + ((size_t)pg * 2 + side) * M * d;
  const float* bias = ks.bias + ((size_t)pg * 2 + side) * M;
  const float* Cmat = side_cmat(ks, b, h, H);
  const float c = row_shift == nullptr ? ordered_to_float(kmax_u[bh]) : 0.f;
  const int nvt = ldt / 16, ntiles = 2 * nvt;

  load_wblock(Ws, bias_s, ld, W, bias, m0, M, d, dpad);
  f32x4 acc[ACC_PER_WAVE];
#pragma unroll
  for (int t = 0; t < ACC_PER_WAVE; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int row_end = min(Lk, (seg + 1) * rows_per_seg);
  for (int row0 = seg * rows_per_seg; row0 < row_end; row0 += TR) {
    __syncthreads();
    load_rows(Xs, ld, ks.X, b * ks.X.sb + h * ks.X.sh, row0, row_end, d, dpad, ks.scale);
    load_values(Vs, ldv, V, b * V.sb + h * V.sh, row0, row_end, nv, ldt, append_ones);
    __syncthreads();
    if (row_shift == nullptr) row_terms_of(rterm, ks, bh, Lk, row0, row_end, Xs, ld, d, Cmat, ks.alpha);
    else if (threadIdx.x < TR) rterm[threadIdx.x] = row0 + threadIdx.x < row_end ? -row_shift[(size_t)bh * Lk + row0 + threadIdx.x] : 0.f;
    __syncthreads();
    const f32x4 e = proj_tile(Xs, Ws, ld, dpad);
    const int f = (w & 1) * 16 + (lane & 15);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = (w >> 1) * 16 + 4 * (lane >> 4) + r;
      Ss[row * lds + f] = (m0 + f < M) ? fast_exp2(e[r] + bias_s[f] + rterm[row] - c) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int tl = 0; tl < ACC_PER_WAVE; ++tl) {
      const int t = w + 4 * tl;
      if (t < ntiles) {
        const int mt = t & 1, vt = t >> 1;
        const float* ap = Ss + (lane >> 4) * lds + mt * 16 + (lane & 15);      // A[i=m][k=j] = Ss[j][m]
        const float* bp = Vs + (lane >> 4) * ldv + vt * 16 + (lane & 15);      // B[k=j][n=v] = Vs[j][v]
        for (int k = 0; k < TR; k += 4) acc[tl] = mfma4(ap[k * lds], bp[k * ldv], acc[tl]);
      }
    }
  }
  float* out = Tpart + (((size_t)bh * nseg + seg) * M) * ldt;
#pragma unroll
  for (int tl = 0; tl < ACC_PER_WAVE; ++tl) {
    const int t = w + 4 * tl;
    if (t < ntiles) {
      const int mt = t & 1, vt = t >> 1;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = m0 + mt * 16 + 4 * (lane >> 4) + r;
        if (m < M) out[(size_t)m * ldt + vt * 16 + (lane & 15)] = acc[tl][r];
      }
    }
  }
}

// Sum (prefix = 0: result in segment 0's slot), exclusive prefix (prefix = 1, in place) or exclusive suffix
// (prefix = 2, in place) over the segments.  block (64, 4): 64 consecutive elements, and for the plain sum four
// interleaved groups of segments that are added up through LDS (the scans run on the first group alone).
__global__ void __launch_bounds__(256) k_gen_reduce(float* Tpart, int nseg, size_t per_state, size_t total, int prefix) {
  __shared__ float part[4][64];
  const size_t i = (size_t)blockIdx.x * 64 + threadIdx.x;
  const int grp = threadIdx.y;
  const bool live = i < total;
  const size_t bh = live ? i / per_state : 0, e = live ? i - bh * per_state : 0;
  float* p = Tpart + bh * nseg * per_state + e;
  if (prefix == 0) {
    float run = 0.f;
    if (live)
      for (int s = grp; s < nseg; s += 4) run += p[(size_t)s * per_state];
    part[grp][threadIdx.x] = run;
    __syncthreads();
    if (live && grp == 0) p[0] = (part[0][threadIdx.x] + part[1][threadIdx.x]) + (part[2][threadIdx.x] + part[3][threadIdx.x]);
    return;
  }
  if (!live || grp != 0) return;
  float run = 0.f;
  if (prefix == 2) {
    for (int s = nseg - 1; s >= 0; --s) {
      const float v = p[(size_t)s * per_state];
      p[(size_t)s * per_state] = run;
      run += v;
    }
  } else {
    for (int s = 0; s < nseg; ++s) {
      const float v = p[(size_t)s * per_state];
      p[(size_t)s * per_state] = run;
      run += v;
    }
  }
}

// Normalise (attention) or rescale (operator) an accumulated 32 x ldt tile held in LDS and store it.  Attention
// rows whose normaliser is not positive are written as zeros and, with a counter, counted (once per row).
__device__ void store_result(const float* Os, int ldo, const TensorDev& Y, long long ybase, int row0, int nrows,
                             int nv, int matvec, const float* row_log2scale, unsigned* flushed = nullptr) {
  for (int idx = threadIdx.x; idx < TR * nv; idx += NT) {
    const int r = idx / nv, c = idx - r * nv;
    if (row0 + r >= nrows) continue;
    float v = Os[r * ldo + c];
    if (matvec) v *= fast_exp2(row_log2scale[r]);
    else {
      const float den = Os[r * ldo + nv];
      v = den > 0.f ? v / den : 0.f;
      if (flushed != nullptr && c == 0 && !(den > 0.f)) atomicAdd(flushed, 1u);
    }
    store_elem(Y, ybase + (long long)(row0 + r) * Y.sl + c, v);
  }
}

// ---------------------------------------------------------------------------------------------------
// Query side of the non-causal contraction (Section 2.1, P (S^T C); Section 2.2 for the row normalisation).
// grid (ceil(Lq/32), B*H).  T: [bh][M][ldt] with stride state_stride between (b,h).
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(NT) k_gen_apply(GenSide qs, int Lq, int H, int M, int d, int nv, int ldt,
                                                  const float* T, size_t state_stride, const uint32_t* kmax_u,
                                                  int matvec, TensorDev Y, float* den_out, float* shift_out,
                                                  unsigned* flushed) {
  extern __shared__ float smem[];
  const int dpad = (d + 3) & ~3, ld = dpad + 1, ldts = ldt + 1, lds = MB + 1;
  float* Xs = smem;
  float* Ws = Xs + TR * ld;
  float* Ts = Ws + MB * ld;          // also reused as the output tile (32 x ldts)
  float* Ps = Ts + MB * ldts;
  float* bias_s = Ps + TR * lds;
  float* rterm = bias_s + MB;
  float* rscale = rterm + TR;
  uint32_t* rowmax_u = (uint32_t*)(rscale + TR);
  const int bh = blockIdx.y, b = bh / H, h = bh % H, row0 = blockIdx.x * TR;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int pg = group_of(qs.pgroups, b, h, H);
  const float* W = qs.W + ((size_t)pg * 2) * M * d;
  const float* bias = qs.bias + ((size_t)pg * 2) * M;
  const float* Cmat = side_cmat(qs, b, h, H);
  const float* Tb = T + (size_t)bh * state_stride;
  const int nvt = ldt / 16, ntiles = 2 * nvt;

  load_rows(Xs, ld, qs.X, b * qs.X.sb + h * qs.X.sh, row0, Lq, d, dpad, qs.scale);
  __syncthreads();
  // (the query row terms matter in operator mode only: in attention they cancel in the normalisation)
  if (matvec) row_terms(rterm, Xs, ld, d, Cmat, qs.alpha);
  else if (threadIdx.x < TR) rterm[threadIdx.x] = 0.f;
  rowmax_pass(rowmax_u, Xs, Ws, bias_s, ld, W, bias, M, d, dpad);
  // operator mode multiplies the shifts back: exp2(rowmax + rterm + kmax)
  if (threadIdx.x < TR)
    rscale[threadIdx.x] = ordered_to_float(rowmax_u[threadIdx.x]) + rterm[threadIdx.x] + ordered_to_float(kmax_u[bh]);

  f32x4 acc[ACC_PER_WAVE];
#pragma unroll
  for (int t = 0; t < ACC_PER_WAVE; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  // the projection block and the state block of the next step are fetched while the current step computes: thread
  // t carries row t/8 of the state block, columns t%8 + 8i (ldt <= 144: at most 18)
  WRegs wr;
  float tr[18];
  auto fetch_t = [&](int m0) {
    const int f = threadIdx.x >> 3, c0 = threadIdx.x & 7;
    const float* row = Tb + (size_t)(m0 + f) * ldt;
#pragma unroll
    for (int i = 0; i < 18; ++i) {
      tr[i] = 0.f;
      if (8 * i < ldt && m0 + f < M) tr[i] = row[c0 + 8 * i];
    }
  };
  wblock_fetch(wr, W, bias, 0, M, d, dpad);
  fetch_t(0);
  for (int m0 = 0; m0 < M; m0 += MB) {
    __syncthreads();
    wblock_put(wr, Ws, bias_s, ld, dpad);
    {
      const int f = threadIdx.x >> 3, c0 = threadIdx.x & 7;
#pragma unroll
      for (int i = 0; i < 18; ++i)
        if (8 * i < ldt) Ts[f * ldts + c0 + 8 * i] = tr[i];
    }
    __syncthreads();
    if (m0 + MB < M) {
      wblock_fetch(wr, W, bias, m0 + MB, M, d, dpad);
      fetch_t(m0 + MB);
    }
    const f32x4 e = proj_tile(Xs, Ws, ld, dpad);
    const int f = (w & 1) * 16 + (lane & 15);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = (w >> 1) * 16 + 4 * (lane >> 4) + r;
      Ps[row * lds + f] = (m0 + f < M) ? fast_exp2(e[r] + bias_s[f] - ordered_to_float(rowmax_u[row])) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int tl = 0; tl < ACC_PER_WAVE; ++tl) {
      const int t = w + 4 * tl;
      if (t < ntiles) {
        const int rt = t & 1, vt = t >> 1;
        const float* ap = Ps + (rt * 16 + (lane & 15)) * lds + (lane >> 4);    // A[i][k=m] = Ps[i][m]
        const float* bp = Ts + (lane >> 4) * ldts + vt * 16 + (lane & 15);     // B[k=m][n=v] = Ts[m][v]
        for (int k = 0; k < MB; k += 4) acc[tl] = mfma4(ap[k], bp[k * ldts], acc[tl]);
      }
    }
  }
  __syncthreads();
  float* Os = Ts;
#pragma unroll
  for (int tl = 0; tl < ACC_PER_WAVE; ++tl) {
    const int t = w + 4 * tl;
    if (t < ntiles) {
      const int rt = t & 1, vt = t >> 1;
#pragma unroll
      for (int r = 0; r < 4; ++r) Os[(rt * 16 + 4 * (lane >> 4) + r) * ldts + vt * 16 + (lane & 15)] = acc[tl][r];
    }
  }
  __syncthreads();
  store_result(Os, ldts, Y, b * Y.sb + h * Y.sh, row0, Lq, nv, matvec, rscale, flushed);
  // for the backward pass: the (shifted) denominators and the shifts themselves, so that it rebuilds the same features
  if (den_out != nullptr && threadIdx.x < TR && row0 + threadIdx.x < Lq) {
    den_out[(size_t)bh * Lq + row0 + threadIdx.x] = Os[threadIdx.x * ldts + nv];
    shift_out[(size_t)bh * Lq + row0 + threadIdx.x] = ordered_to_float(rowmax_u[threadIdx.x]);
  }
}

// ---------------------------------------------------------------------------------------------------
// Causal contraction over one segment of one sequence, 32 rows per step, running state in global memory
// (initialised with the exclusive prefix of the segment states).  For each step:
//   Y_c = (tril(P_c S_c^T) [V_c 1] + P_c T_prev) normalised by its last column;  T += S_c^T [V_c 1].
// grid (nseg, B*H).
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(NT) k_gen_causal(GenSide qs, GenSide ks, TensorDev V, int L, int H, int M, int d,
                                                   int nv, int ldt, int rows_per_seg, int nseg,
                                                   const uint32_t* kmax_u, float* Tstate, TensorDev Y, float* den_out,
                                                   float* shift_out, unsigned* flushed) {
  extern __shared__ float smem[];
  const int dpad = (d + 3) & ~3, ld = dpad + 1, ldv = ldt + 1, lds = MB + 1;
  float* Qs = smem;
  float* Ks = Qs + TR * ld;
  float* Ws = Ks + TR * ld;
  float* Vs = Ws + MB * ld;
  float* Ts = Vs + TR * ldv;          // state block, later the output tile
  float* Ps = Ts + MB * ldv;
  float* Ss = Ps + TR * lds;
  float* As = Ss + TR * lds;
  float* bias_s = As + TR * lds;
  float* rterm = bias_s + MB;
  uint32_t* rowmax_u = (uint32_t*)(rterm + TR);
  const int seg = blockIdx.x, bh = blockIdx.y, b = bh / H, h = bh % H;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int pgq = group_of(qs.pgroups, b, h, H);
  const float* W1 = qs.W + ((size_t)pgq * 2) * M * d;
  const float* bias1 = qs.bias + ((size_t)pgq * 2) * M;
  const float* W2 = ks.W + ((size_t)pgq * 2 + 1) * M * d;
  const float* bias2 = ks.bias + ((size_t)pgq * 2 + 1) * M;
  const float* Cmat2 = side_cmat(ks, b, h, H);
  const float c = ordered_to_float(kmax_u[bh]);
  float* Tg = Tstate + ((size_t)bh * nseg + seg) * M * ldt;
  const int nvt = ldt / 16, ntiles = 2 * nvt;
  const long long qbase = b * qs.X.sb + h * qs.X.sh, kbase = b * ks.X.sb + h * ks.X.sh;

  const int row_end = min(L, (seg + 1) * rows_per_seg);
  for (int row0 = seg * rows_per_seg; row0 < row_end; row0 += TR) {
    __syncthreads();
    load_rows(Qs, ld, qs.X, qbase, row0, row_end, d, dpad, qs.scale);
    load_rows(Ks, ld, ks.X, kbase, row0, row_end, d, dpad, ks.scale);
    load_values(Vs, ldv, V, b * V.sb + h * V.sh, row0, row_end, nv, ldt, 1);
    __syncthreads();
    row_terms_of(rterm, ks, bh, L, row0, row_end, Ks, ld, d, Cmat2, 0.f);
    rowmax_pass(rowmax_u, Qs, Ws, bias_s, ld, W1, bias1, M, d, dpad);

    f32x4 acc[ACC_PER_WAVE];
#pragma unroll
    for (int t = 0; t < ACC_PER_WAVE; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    f32x4 sc = {0.f, 0.f, 0.f, 0.f};          // scores tile (query tile w>>1, key tile w&1)
    for (int m0 = 0; m0 < M; m0 += MB) {
      const int f = (w & 1) * 16 + (lane & 15);
      __syncthreads();
      load_wblock(Ws, bias_s, ld, W1, bias1, m0, M, d, dpad);
      for (int idx = threadIdx.x; idx < MB * ldt; idx += NT) {
        const int ff = idx / ldt, cc = idx - ff * ldt;
        Ts[ff * ldv + cc] = (m0 + ff < M) ? Tg[(size_t)(m0 + ff) * ldt + cc] : 0.f;
      }
      __syncthreads();
      {
        const f32x4 e = proj_tile(Qs, Ws, ld, dpad);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = (w >> 1) * 16 + 4 * (lane >> 4) + r;
          Ps[row * lds + f] = (m0 + f < M) ? fast_exp2(e[r] + bias_s[f] - ordered_to_float(rowmax_u[row])) : 0.f;
        }
      }
      __syncthreads();
      load_wblock(Ws, bias_s, ld, W2, bias2, m0, M, d, dpad);
      __syncthreads();
      {
        const f32x4 e = proj_tile(Ks, Ws, ld, dpad);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = (w >> 1) * 16 + 4 * (lane >> 4) + r;
          Ss[row * lds + f] = (m0 + f < M) ? fast_exp2(e[r] + bias_s[f] + rterm[row] - c) : 0.f;
        }
      }
      __syncthreads();
      {   // scores: A[i][k=m] = Ps[i][m], B[k=m][n=j] = Ss[j][m]
        const float* ap = Ps + ((w >> 1) * 16 + (lane & 15)) * lds + (lane >> 4);
        const float* bp = Ss + ((w & 1) * 16 + (lane & 15)) * lds + (lane >> 4);
        for (int k = 0; k < MB; k += 4) sc = mfma4(ap[k], bp[k], sc);
      }
#pragma unroll
      for (int tl = 0; tl < ACC_PER_WAVE; ++tl) {
        const int t = w + 4 * tl;
        if (t < ntiles) {
          const int rt = t & 1, vt = t >> 1;
          {   // inter-chunk term with the state before this step
            const float* ap = Ps + (rt * 16 + (lane & 15)) * lds + (lane >> 4);
            const float* bp = Ts + (lane >> 4) * ldv + vt * 16 + (lane & 15);
            for (int k = 0; k < MB; k += 4) acc[tl] = mfma4(ap[k], bp[k * ldv], acc[tl]);
          }
          {   // state update for feature tile rt: T[m][v] += sum_j Ss[j][m] Vs[j][v]
            f32x4 up = {0.f, 0.f, 0.f, 0.f};
            const float* ap = Ss + (lane >> 4) * lds + rt * 16 + (lane & 15);
            const float* bp = Vs + (lane >> 4) * ldv + vt * 16 + (lane & 15);
            for (int k = 0; k < TR; k += 4) up = mfma4(ap[k * lds], bp[k * ldv], up);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int m = m0 + rt * 16 + 4 * (lane >> 4) + r;
              if (m < M) Tg[(size_t)m * ldt + vt * 16 + (lane & 15)] += up[r];
            }
          }
        }
      }
    }
    // causal mask inside the step (key j <= query i), then the intra-chunk product
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int i = (w >> 1) * 16 + 4 * (lane >> 4) + r, j = (w & 1) * 16 + (lane & 15);
      As[i * lds + j] = (j <= i) ? sc[r] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int tl = 0; tl < ACC_PER_WAVE; ++tl) {
      const int t = w + 4 * tl;
      if (t < ntiles) {
        const int rt = t & 1, vt = t >> 1;
        const float* ap = As + (rt * 16 + (lane & 15)) * lds + (lane >> 4);
        const float* bp = Vs + (lane >> 4) * ldv + vt * 16 + (lane & 15);
        for (int k = 0; k < TR; k += 4) acc[tl] = mfma4(ap[k], bp[k * ldv], acc[tl]);
      }
    }
    __syncthreads();
    float* Os = Ts;
#pragma unroll
    for (int tl = 0; tl < ACC_PER_WAVE; ++tl) {
      const int t = w + 4 * tl;
      if (t < ntiles) {
        const int rt = t & 1, vt = t >> 1;
#pragma unroll
        for (int r = 0; r < 4; ++r) Os[(rt * 16 + 4 * (lane >> 4) + r) * ldv + vt * 16 + (lane & 15)] = acc[tl][r];
      }
    }
    __syncthreads();
    store_result(Os, ldv, Y, b * Y.sb + h * Y.sh, row0, row_end, nv, 0, nullptr, flushed);
    if (den_out != nullptr && threadIdx.x < TR && row0 + threadIdx.x < row_end) {   // for the backward pass
      den_out[(size_t)bh * L + row0 + threadIdx.x] = Os[threadIdx.x * ldv + nv];
      shift_out[(size_t)bh * L + row0 + threadIdx.x] = ordered_to_float(rowmax_u[threadIdx.x]);
    }
  }
}

// ---------------------------------------------------------------------------------------------------
// Statistics scan for the fits: per (b,h) and row chunk, sum x and sum x x^T of the scaled rows (fp32 MFMA,
// fp32 partials), then a second kernel adds the partials of all (b,h) of a group in fp64.
// grid (nchunks, B*H, 2 tensors).  part: [2][B*H][nchunks][d*d + d].
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(NT) k_stats_partial(TensorDev X, TensorDev Yt, int Lx, int Ly, int H, int d,
                                                      float scale, int rows_per_chunk, int nchunks, float* part) {
  extern __shared__ float smem[];
  const int dpad = (d + 15) & ~15, ld = dpad + 1;
  float* Xs = smem;
  const int which = blockIdx.z, bh = blockIdx.y, b = bh / H, h = bh % H, chunk = blockIdx.x;
  const TensorDev& T = which ? Yt : X;
  const int L = which ? Ly : Lx;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int nt = dpad / 16, ntiles = nt * nt;      // <= 64 tiles, 16 per wave
  f32x4 acc[16];
#pragma unroll
  for (int t = 0; t < 16; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  float colsum = 0.f;
  const int row_end = min(L, (chunk + 1) * rows_per_chunk);
  for (int row0 = chunk * rows_per_chunk; row0 < row_end; row0 += TR) {
    __syncthreads();
    load_rows(Xs, ld, T, b * T.sb + h * T.sh, row0, row_end, d, dpad, scale);
    __syncthreads();
    if (threadIdx.x < d)
      for (int r = 0; r < TR; ++r) colsum += Xs[r * ld + threadIdx.x];
#pragma unroll
    for (int tl = 0; tl < 16; ++tl) {
      const int t = w + 4 * tl;
      if (t < ntiles) {
        const int at = t / nt, bt = t - at * nt;
        const float* ap = Xs + (lane >> 4) * ld + at * 16 + (lane & 15);      // A[i=a][k=row] = Xs[row][a]
        const float* bp = Xs + (lane >> 4) * ld + bt * 16 + (lane & 15);
        for (int k = 0; k < TR; k += 4) acc[tl] = mfma4(ap[k * ld], bp[k * ld], acc[tl]);
      }
    }
  }
  float* out = part + (((size_t)which * gridDim.y + bh) * nchunks + chunk) * ((size_t)d * d + d);
#pragma unroll
  for (int tl = 0; tl < 16; ++tl) {
    const int t = w + 4 * tl;
    if (t < ntiles) {
      const int at = t / nt, bt = t - at * nt;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int a = at * 16 + 4 * (lane >> 4) + r, bb = bt * 16 + (lane & 15);
        if (a < d && bb < d) out[(size_t)a * d + bb] = acc[tl][r];
      }
    }
  }
  if (threadIdx.x < d) out[(size_t)d * d + threadIdx.x] = colsum;
}

// stats: [groups][2][d*d + d] doubles: mean x x^T then mean x, for X (0) and Y (1).
__global__ void k_stats_final(const float* part, int B, int H, int nchunks, int d, int groups, int Lx, int Ly,
                              double* stats) {
  const size_t per = (size_t)d * d + d;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)groups * 2 * per) return;
  const int g = (int)(i / (2 * per));
  const int which = (int)((i / per) & 1);
  const size_t e = i % per;
  double s = 0.0;
  long long rows = 0;
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < H; ++h) {
      if (group_of(groups, b, h, H) != g) continue;
      rows += which ? Ly : Lx;
      const float* p = part + (((size_t)which * B * H + (size_t)b * H + h) * nchunks) * per + e;
      // four independent partial sums: the loads of a whole group of chunks are in flight together
      double s4[4] = {0.0, 0.0, 0.0, 0.0};
      int c = 0;
      for (; c + 4 <= nchunks; c += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) s4[u] += (double)p[(size_t)(c + u) * per];
      }
      for (; c < nchunks; ++c) s4[0] += (double)p[(size_t)c * per];
      s += (s4[0] + s4[1]) + (s4[2] + s4[3]);
    }
  stats[i] = s / (double)rows;
}

// ---------------------------------------------------------------------------------------------------
// Backward pass of non-causal attention (chain rule on Section 2.2's attention equation with K_hat = P S^T;
// theta and omega are constants).  With V1 = [V 1], T = S^T V1, Yhat = P T:
//   G1_i = [dY_i / den_i, -(dY_i . Y_i) / den_i],  dP = G1 T^T,  R = P^T G1,  dV1 = S R,  dS = V1 R^T,
//   dE = F * dF  (F = P or S),   dx = dE W + rowsum(dE) (C + C^T) x,   d(input) = qk_scale dx.
// The exponent shifts of the forward pass (one per query row, one per sequence for the keys) cancel in every
// product above, so the kernels work on the shifted quantities throughout.
// ---------------------------------------------------------------------------------------------------

// In place: row i of `buf` ([bh][L][ldt], holding Y_i in its first nv columns) becomes G1_i (zero padded).
// Sixteen lanes per row (consecutive columns: coalesced), 16 rows per workgroup of 256 threads.
__global__ void k_bwd_ghat(TensorDev dY, float* buf, const float* den, int L, int H, int nv, int ldt, size_t rows) {
  const size_t i = (size_t)blockIdx.x * 16 + (threadIdx.x >> 4);
  const int l = threadIdx.x & 15;
  const bool live = i < rows;
  const size_t ii = live ? i : 0;
  const int bh = (int)(ii / L), row = (int)(ii - (size_t)bh * L), b = bh / H, h = bh % H;
  float* g = buf + ii * ldt;
  const float dn = den[ii];
  const float inv = dn > 0.f ? 1.f / dn : 0.f;
  const long long base = b * dY.sb + h * dY.sh + (long long)row * dY.sl;
  float dot = 0.f;
  for (int c = l; c < nv; c += 16) dot += load_elem(dY, base + c) * g[c];
  dot += __shfl_xor(dot, 1);
  dot += __shfl_xor(dot, 2);
  dot += __shfl_xor(dot, 4);
  dot += __shfl_xor(dot, 8);
  if (!live) return;
  for (int c = l; c < ldt; c += 16) g[c] = c < nv ? load_elem(dY, base + c) * inv : (c == nv ? -dot * inv : 0.f);
}

// One side of the backward pass for a tile of 32 rows.  F = this side's features (query side: per-row shifts from
// the forward pass, no row term; key side: the sequence's key shift and the row term), A = the rows' "left" factor
// (query side: G1; key side: V1), St = the state it is contracted with (query side: T; key side: R).
//   out1 = F St          (key side only: its first nv columns are dV)
//   dF   = A St^T,  dE = F * dF,  grad = scale (dE W / log2e + rowsum(dE) (C + C^T) x)
// grid (ceil(L/32), B*H).
__global__ void __launch_bounds__(NT) k_gen_bwd_side(GenSide sd, int side, TensorDev A, int a_cols, int append_ones, int L,
                                                     int H, int M, int d, int nv, int ldt, const float* St,
                                                     size_t state_stride, const uint32_t* kmax_u, const float* row_shift,
                                                     TensorDev out1, int want_out1, TensorDev grad) {
  extern __shared__ float smem[];
  const int dpad = (d + 3) & ~3, ld = dpad + 1, ldts = ldt + 1, lds = MB + 1;
  float* Xs = smem;
  float* Ws = Xs + TR * ld;          // also the gradient tile (32 x ld) at the end
  float* As = Ws + MB * ld;
  float* Sts = As + TR * ldts;       // also the out1 tile (32 x ldts) at the end
  float* Fs = Sts + MB * ldts;
  float* dEs = Fs + TR * lds;
  float* bias_s = dEs + TR * lds;
  float* rterm = bias_s + MB;        // what is added to the exponent per row (row term - shift)
  float* rsum = rterm + TR;
  const int bh = blockIdx.y, b = bh / H, h = bh % H, row0 = blockIdx.x * TR;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int pg = group_of(sd.pgroups, b, h, H);
  const float* W = sd.W + ((size_t)pg * 2 + side) * M * d;
  const float* bias = sd.bias + ((size_t)pg * 2 + side) * M;
  const float* Cmat = side_cmat(sd, b, h, H);
  const float* Sb = St + (size_t)bh * state_stride;
  const int nvt = ldt / 16, ntiles = 2 * nvt, nct = dpad / 16 + ((dpad & 15) ? 1 : 0), ngt = 2 * nct;

  load_rows(Xs, ld, sd.X, b * sd.X.sb + h * sd.X.sh, row0, L, d, dpad, sd.scale);
  load_values(As, ldts, A, b * A.sb + h * A.sh, row0, L, a_cols, ldt, append_ones);
  __syncthreads();
  if (side == 1) {
    row_terms_of(rterm, sd, bh, L, row0, L, Xs, ld, d, Cmat, sd.alpha);
    __syncthreads();
    if (threadIdx.x < TR) rterm[threadIdx.x] -= ordered_to_float(kmax_u[bh]);
  } else if (threadIdx.x < TR) {
    rterm[threadIdx.x] = row0 + threadIdx.x < L ? -row_shift[(size_t)bh * L + row0 + threadIdx.x] : 0.f;
  }

  f32x4 acc_o[ACC_PER_WAVE], acc_g[4];
#pragma unroll
  for (int t = 0; t < ACC_PER_WAVE; ++t) acc_o[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int t = 0; t < 4; ++t) acc_g[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  float rs_part = 0.f;               // thread (row = tid / 8, part = tid % 8): its share of rowsum(dE)

  for (int m0 = 0; m0 < M; m0 += MB) {
    __syncthreads();
    load_wblock(Ws, bias_s, ld, W, bias, m0, M, d, dpad);
    for (int idx = threadIdx.x; idx < MB * ldt; idx += NT) {
      const int f = idx / ldt, c = idx - f * ldt;
      Sts[f * ldts + c] = (m0 + f < M) ? Sb[(size_t)(m0 + f) * ldt + c] : 0.f;
    }
    __syncthreads();
    const f32x4 e = proj_tile(Xs, Ws, ld, dpad);
    const int f = (w & 1) * 16 + (lane & 15);
    float fv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = (w >> 1) * 16 + 4 * (lane >> 4) + r;
      fv[r] = (m0 + f < M && row0 + row < L) ? fast_exp2(e[r] + bias_s[f] + rterm[row]) : 0.f;
      Fs[row * lds + f] = fv[r];
    }
    // dF tile of this wave (rows (w>>1)*16.., features (w&1)*16..): A[i][k=v] = As[i][v], B[k=v][n=m] = Sts[m][v]
    {
      const float* ap = As + ((w >> 1) * 16 + (lane & 15)) * ldts + (lane >> 4);
      const float* bp = Sts + ((w & 1) * 16 + (lane & 15)) * ldts + (lane >> 4);
      f32x4 df = {0.f, 0.f, 0.f, 0.f};
      for (int k = 0; k < ldt; k += 4) df = mfma4(ap[k], bp[k], df);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = (w >> 1) * 16 + 4 * (lane >> 4) + r;
        dEs[row * lds + f] = fv[r] * df[r];
      }
    }
    __syncthreads();
    if (want_out1) {
#pragma unroll
      for (int tl = 0; tl < ACC_PER_WAVE; ++tl) {
        const int t = w + 4 * tl;
        if (t < ntiles) {
          const int rt = t & 1, vt = t >> 1;
          const float* ap = Fs + (rt * 16 + (lane & 15)) * lds + (lane >> 4);     // A[i][k=m] = Fs[i][m]
          const float* bp = Sts + (lane >> 4) * ldts + vt * 16 + (lane & 15);     // B[k=m][n=v] = Sts[m][v]
          for (int k = 0; k < MB; k += 4) acc_o[tl] = mfma4(ap[k], bp[k * ldts], acc_o[tl]);
        }
      }
    }
#pragma unroll
    for (int tl = 0; tl < 4; ++tl) {
      const int t = w + 4 * tl;
      if (t < ngt) {
        const int rt = t & 1, ct = t >> 1;
        const float* ap = dEs + (rt * 16 + (lane & 15)) * lds + (lane >> 4);      // A[i][k=m] = dEs[i][m]
        const float* bp = Ws + (lane >> 4) * ld + ct * 16 + (lane & 15);          // B[k=m][n=c] = Ws[m][c]
        f32x4 a = acc_g[tl];
        for (int k = 0; k < MB; k += 4) a = mfma4(ap[k], (ct * 16 + (lane & 15) < dpad) ? bp[k * ld] : 0.f, a);
        acc_g[tl] = a;
      }
    }
    {
      const int row = threadIdx.x >> 3, part = threadIdx.x & 7;
#pragma unroll
      for (int q = 0; q < 4; ++q) rs_part += dEs[row * lds + part * 4 + q];
    }
  }
  __syncthreads();
  // tiles back to LDS
  float* Gs = Ws;
  float* Os = Sts;
#pragma unroll
  for (int tl = 0; tl < 4; ++tl) {
    const int t = w + 4 * tl;
    if (t < ngt) {
      const int rt = t & 1, ct = t >> 1, col = ct * 16 + (lane & 15);
      if (col < dpad) {
#pragma unroll
        for (int r = 0; r < 4; ++r) Gs[(rt * 16 + 4 * (lane >> 4) + r) * ld + col] = acc_g[tl][r];
      }
    }
  }
  if (want_out1) {
#pragma unroll
    for (int tl = 0; tl < ACC_PER_WAVE; ++tl) {
      const int t = w + 4 * tl;
      if (t < ntiles) {
        const int rt = t & 1, vt = t >> 1;
#pragma unroll
        for (int r = 0; r < 4; ++r) Os[(rt * 16 + 4 * (lane >> 4) + r) * ldts + vt * 16 + (lane & 15)] = acc_o[tl][r];
      }
    }
  }
  rs_part += __shfl_xor(rs_part, 1);
  rs_part += __shfl_xor(rs_part, 2);
  rs_part += __shfl_xor(rs_part, 4);
  if ((threadIdx.x & 7) == 0) rsum[threadIdx.x >> 3] = rs_part;
  __syncthreads();
  // grad[i][c] = scale (Gs[i][c] / log2e + rsum_i ((C + C^T) x_i)[c]);  C = -I/2: (C + C^T) x = -x
  for (int idx = threadIdx.x; idx < TR * d; idx += NT) {
    const int r = idx / d, c = idx - r * d;
    if (row0 + r >= L) continue;
    float cx;
    if (Cmat == nullptr) cx = -Xs[r * ld + c];
    else {
      cx = sym_row_dot(Cmat, d, c, Xs + r * ld);
    }
    const float v = sd.scale * (Gs[r * ld + c] * kLn2 + rsum[r] * (cx + 2.f * sd.alpha * Xs[r * ld + c]));
    store_elem(grad, b * grad.sb + h * grad.sh + (long long)(row0 + r) * grad.sl + c, v);
  }
  if (want_out1) {
    for (int idx = threadIdx.x; idx < TR * nv; idx += NT) {
      const int r = idx / nv, c = idx - r * nv;
      if (row0 + r < L) store_elem(out1, b * out1.sb + h * out1.sh + (long long)(row0 + r) * out1.sl + c, Os[r * ldts + c]);
    }
  }
}

// ---------------------------------------------------------------------------------------------------
// Backward pass of causal attention.  With T_i the prefix state (keys j <= i) and R_j the suffix sum
// sum_{i >= j} P_i^T G1_i, per chunk c of 32 rows (A = tril(G1_c V1_c^T), B = tril(P_c S_c^T)):
//   dP_c  = G1_c T_{c-1}^T + A S_c                 dV1_c = S_c R_{c+1} + B^T G1_c
//   dS_c  = V1_c R_{c+1}^T + A^T P_c               and dE = F * dF, dx = dE W + rowsum(dE) (C + C^T) x as above.
// The query kernel walks a segment forwards with the running prefix state (initialised with the exclusive prefix
// of the segment states), the key kernel walks it backwards with the running suffix sum (initialised with the
// exclusive suffix of the segments' P^T G1).  G1, the denominators and the query shifts come from a forward pass.
// grid (nseg, B*H) both.
// ---------------------------------------------------------------------------------------------------
struct BwdCausalSmem {
  float *Qs, *Ks, *Ws, *Vs, *Gs, *Ts, *Ps, *Ss, *dEs, *As, *Bs, *bias_s, *rterm, *qsh, *rsum;
};
__device__ __forceinline__ BwdCausalSmem bwd_causal_carve(float* smem, int ld, int ldv, int lds) {
  BwdCausalSmem m;
  m.Qs = smem;
  m.Ks = m.Qs + TR * ld;
  m.Ws = m.Ks + TR * ld;
  m.Vs = m.Ws + MB * ld;
  m.Gs = m.Vs + TR * ldv;
  m.Ts = m.Gs + TR * ldv;
  m.Ps = m.Ts + MB * ldv;
  m.Ss = m.Ps + TR * lds;
  m.dEs = m.Ss + TR * lds;
  m.As = m.dEs + TR * lds;
  m.Bs = m.As + TR * lds;
  m.bias_s = m.Bs + TR * lds;
  m.rterm = m.bias_s + MB;
  m.qsh = m.rterm + TR;
  m.rsum = m.qsh + TR;
  return m;
}

// As[i][j] = (j <= i) ? G1_i . V1_j : 0 for the chunk's 32 x 32 (query, key) pairs; wave w owns tile (w>>1, w&1).
__device__ __forceinline__ void bwd_causal_amat(float* As, const float* Gs, const float* Vs, int ldv, int lds, int ldt) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const float* ap = Gs + ((w >> 1) * 16 + (lane & 15)) * ldv + (lane >> 4);   // A[i][k=v] = Gs[i][v]
  const float* bp = Vs + ((w & 1) * 16 + (lane & 15)) * ldv + (lane >> 4);    // B[k=v][n=j] = Vs[j][v]
  f32x4 a = {0.f, 0.f, 0.f, 0.f};
  for (int k = 0; k < ldt; k += 4) a = mfma4(ap[k], bp[k], a);
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int i = (w >> 1) * 16 + 4 * (lane >> 4) + r, j = (w & 1) * 16 + (lane & 15);
    As[i * lds + j] = (j <= i) ? a[r] : 0.f;
  }
}

// grad rows of a 32-row tile from the accumulated dE W tile (Gsrc, stride ld), the row sums and x.
__device__ __forceinline__ void bwd_store_grad(const TensorDev& grad, long long base, int row0, int row_end, int d, int ld,
                                               const float* Gsrc, const float* rsum, const float* Xs, const float* Cmat,
                                               float scale, float alpha) {
  for (int idx = threadIdx.x; idx < TR * d; idx += NT) {
    const int r = idx / d, c = idx - r * d;
    if (row0 + r >= row_end) continue;
    float cx;
    if (Cmat == nullptr) cx = -Xs[r * ld + c];
    else {
      cx = sym_row_dot(Cmat, d, c, Xs + r * ld);
    }
    const float v = scale * (Gsrc[r * ld + c] * kLn2 + rsum[r] * (cx + 2.f * alpha * Xs[r * ld + c]));
    store_elem(grad, base + (long long)(row0 + r) * grad.sl + c, v);
  }
}

__global__ void __launch_bounds__(NT) k_gen_bwd_causal_q(GenSide qs, GenSide ks, TensorDev V, const float* ghat, int L,
                                                         int H, int M, int d, int nv, int ldt, int rows_per_seg, int nseg,
                                                         const uint32_t* kmax_u, const float* row_shift, float* Tstate,
                                                         TensorDev dQ) {
  extern __shared__ float smem[];
  const int dpad = (d + 3) & ~3, ld = dpad + 1, ldv = ldt + 1, lds = MB + 1;
  const BwdCausalSmem m = bwd_causal_carve(smem, ld, ldv, lds);
  const int seg = blockIdx.x, bh = blockIdx.y, b = bh / H, h = bh % H;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int pg = group_of(qs.pgroups, b, h, H);
  const float* W1 = qs.W + ((size_t)pg * 2) * M * d;
  const float* bias1 = qs.bias + ((size_t)pg * 2) * M;
  const float* W2 = ks.W + ((size_t)pg * 2 + 1) * M * d;
  const float* bias2 = ks.bias + ((size_t)pg * 2 + 1) * M;
  const float* Cmat1 = side_cmat(qs, b, h, H);
  const float* Cmat2 = side_cmat(ks, b, h, H);
  const float c = ordered_to_float(kmax_u[bh]);
  float* Tg = Tstate + ((size_t)bh * nseg + seg) * M * ldt;
  const TensorDev G{ghat, 0, (long long)H * L * ldt, (long long)L * ldt, (long long)ldt};
  const int nvt = ldt / 16, ntiles = 2 * nvt, nct = (dpad + 15) / 16, ngt = 2 * nct;
  const long long qbase = b * qs.X.sb + h * qs.X.sh, kbase = b * ks.X.sb + h * ks.X.sh;

  const int row_end = min(L, (seg + 1) * rows_per_seg);
  for (int row0 = seg * rows_per_seg; row0 < row_end; row0 += TR) {
    __syncthreads();
    load_rows(m.Qs, ld, qs.X, qbase, row0, row_end, d, dpad, qs.scale);
    load_rows(m.Ks, ld, ks.X, kbase, row0, row_end, d, dpad, ks.scale);
    load_values(m.Vs, ldv, V, b * V.sb + h * V.sh, row0, row_end, nv, ldt, 1);
    load_values(m.Gs, ldv, G, b * G.sb + h * G.sh, row0, row_end, ldt, ldt, 0);
    if (threadIdx.x < TR) m.qsh[threadIdx.x] = row0 + threadIdx.x < row_end ? -row_shift[(size_t)bh * L + row0 + threadIdx.x] : 0.f;
    __syncthreads();
    row_terms_of(m.rterm, ks, bh, L, row0, row_end, m.Ks, ld, d, Cmat2, 0.f);
    bwd_causal_amat(m.As, m.Gs, m.Vs, ldv, lds, ldt);

    f32x4 acc_g[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) acc_g[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    float rs_part = 0.f;
    for (int m0 = 0; m0 < M; m0 += MB) {
      const int f = (w & 1) * 16 + (lane & 15);
      __syncthreads();
      load_wblock(m.Ws, m.bias_s, ld, W2, bias2, m0, M, d, dpad);
      for (int idx = threadIdx.x; idx < MB * ldt; idx += NT) {
        const int ff = idx / ldt, cc = idx - ff * ldt;
        m.Ts[ff * ldv + cc] = (m0 + ff < M) ? Tg[(size_t)(m0 + ff) * ldt + cc] : 0.f;
      }
      __syncthreads();
      {
        const f32x4 e = proj_tile(m.Ks, m.Ws, ld, dpad);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = (w >> 1) * 16 + 4 * (lane >> 4) + r;
          m.Ss[row * lds + f] = (m0 + f < M && row0 + row < row_end) ? fast_exp2(e[r] + m.bias_s[f] + m.rterm[row] - c) : 0.f;
        }
      }
      __syncthreads();
      load_wblock(m.Ws, m.bias_s, ld, W1, bias1, m0, M, d, dpad);
      __syncthreads();
      {
        const f32x4 e = proj_tile(m.Qs, m.Ws, ld, dpad);
        float fv[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = (w >> 1) * 16 + 4 * (lane >> 4) + r;
          fv[r] = (m0 + f < M && row0 + row < row_end) ? fast_exp2(e[r] + m.bias_s[f] + m.qsh[row]) : 0.f;
        }
        // dP tile (rows (w>>1)*16.., features (w&1)*16..) = G1 T_prev^T + A S
        f32x4 df = {0.f, 0.f, 0.f, 0.f};
        {
          const float* ap = m.Gs + ((w >> 1) * 16 + (lane & 15)) * ldv + (lane >> 4);   // A[i][k=v] = Gs[i][v]
          const float* bp = m.Ts + ((w & 1) * 16 + (lane & 15)) * ldv + (lane >> 4);    // B[k=v][n=m] = Ts[m][v]
          for (int k = 0; k < ldt; k += 4) df = mfma4(ap[k], bp[k], df);
        }
        {
          const float* ap = m.As + ((w >> 1) * 16 + (lane & 15)) * lds + (lane >> 4);   // A[i][k=j] = As[i][j]
          const float* bp = m.Ss + (lane >> 4) * lds + (w & 1) * 16 + (lane & 15);      // B[k=j][n=m] = Ss[j][m]
          for (int k = 0; k < TR; k += 4) df = mfma4(ap[k], bp[k * lds], df);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = (w >> 1) * 16 + 4 * (lane >> 4) + r;
          m.dEs[row * lds + f] = fv[r] * df[r];
        }
      }
      __syncthreads();
#pragma unroll
      for (int tl = 0; tl < 4; ++tl) {
        const int t = w + 4 * tl;
        if (t < ngt) {
          const int rt = t & 1, ct = t >> 1;
          const float* ap = m.dEs + (rt * 16 + (lane & 15)) * lds + (lane >> 4);        // A[i][k=m] = dEs[i][m]
          const float* bp = m.Ws + (lane >> 4) * ld + ct * 16 + (lane & 15);            // B[k=m][n=c] = Ws[m][c]
          const bool in = ct * 16 + (lane & 15) < dpad;
          f32x4 a = acc_g[tl];
          for (int k = 0; k < MB; k += 4) a = mfma4(ap[k], in ? bp[k * ld] : 0.f, a);
          acc_g[tl] = a;
        }
      }
      {
        const int row = threadIdx.x >> 3, part = threadIdx.x & 7;
#pragma unroll
        for (int q = 0; q < 4; ++q) rs_part += m.dEs[row * lds + part * 4 + q];
      }
      // the state takes this chunk's keys (after its last use above): T[m][v] += sum_j Ss[j][m] Vs[j][v]
#pragma unroll
      for (int tl = 0; tl < ACC_PER_WAVE; ++tl) {
        const int t = w + 4 * tl;
        if (t < ntiles) {
          const int rt = t & 1, vt = t >> 1;
          f32x4 up = {0.f, 0.f, 0.f, 0.f};
          const float* ap = m.Ss + (lane >> 4) * lds + rt * 16 + (lane & 15);
          const float* bp = m.Vs + (lane >> 4) * ldv + vt * 16 + (lane & 15);
          for (int k = 0; k < TR; k += 4) up = mfma4(ap[k * lds], bp[k * ldv], up);
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int mm = m0 + rt * 16 + 4 * (lane >> 4) + r;
            if (mm < M) Tg[(size_t)mm * ldt + vt * 16 + (lane & 15)] += up[r];
          }
        }
      }
    }
    __syncthreads();
    float* Gd = m.Ws;
#pragma unroll
    for (int tl = 0; tl < 4; ++tl) {
      const int t = w + 4 * tl;
      if (t < ngt) {
        const int rt = t & 1, ct = t >> 1, col = ct * 16 + (lane & 15);
        if (col < dpad) {
#pragma unroll
          for (int r = 0; r < 4; ++r) Gd[(rt * 16 + 4 * (lane >> 4) + r) * ld + col] = acc_g[tl][r];
        }
      }
    }
    rs_part += __shfl_xor(rs_part, 1);
    rs_part += __shfl_xor(rs_part, 2);
    rs_part += __shfl_xor(rs_part, 4);
    if ((threadIdx.x & 7) == 0) m.rsum[threadIdx.x >> 3] = rs_part;
    __syncthreads();
    bwd_store_grad(dQ, b * dQ.sb + h * dQ.sh, row0, row_end, d, ld, Gd, m.rsum, m.Qs, Cmat1, qs.scale, 0.f);
  }
}

__global__ void __launch_bounds__(NT) k_gen_bwd_causal_k(GenSide qs, GenSide ks, TensorDev V, const float* ghat, int L,
                                                         int H, int M, int d, int nv, int ldt, int rows_per_seg, int nseg,
                                                         const uint32_t* kmax_u, const float* row_shift, float* Rstate,
                                                         TensorDev dK, TensorDev dV) {
  extern __shared__ float smem[];
  const int dpad = (d + 3) & ~3, ld = dpad + 1, ldv = ldt + 1, lds = MB + 1;
  const BwdCausalSmem m = bwd_causal_carve(smem, ld, ldv, lds);
  const int seg = blockIdx.x, bh = blockIdx.y, b = bh / H, h = bh % H;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int pg = group_of(qs.pgroups, b, h, H);
  const float* W1 = qs.W + ((size_t)pg * 2) * M * d;
  const float* bias1 = qs.bias + ((size_t)pg * 2) * M;
  const float* W2 = ks.W + ((size_t)pg * 2 + 1) * M * d;
  const float* bias2 = ks.bias + ((size_t)pg * 2 + 1) * M;
  const float* Cmat2 = side_cmat(ks, b, h, H);
  const float c = ordered_to_float(kmax_u[bh]);
  float* Rg = Rstate + ((size_t)bh * nseg + seg) * M * ldt;
  const TensorDev G{ghat, 0, (long long)H * L * ldt, (long long)L * ldt, (long long)ldt};
  const int nvt = ldt / 16, ntiles = 2 * nvt, nct = (dpad + 15) / 16, ngt = 2 * nct;
  const long long qbase = b * qs.X.sb + h * qs.X.sh, kbase = b * ks.X.sb + h * ks.X.sh;

  const int row_beg = seg * rows_per_seg, row_end = min(L, (seg + 1) * rows_per_seg);
  const int nchunk = (row_end - row_beg + TR - 1) / TR;
  for (int ch = nchunk - 1; ch >= 0; --ch) {
    const int row0 = row_beg + ch * TR;
    __syncthreads();
    load_rows(m.Qs, ld, qs.X, qbase, row0, row_end, d, dpad, qs.scale);
    load_rows(m.Ks, ld, ks.X, kbase, row0, row_end, d, dpad, ks.scale);
    load_values(m.Vs, ldv, V, b * V.sb + h * V.sh, row0, row_end, nv, ldt, 1);
    load_values(m.Gs, ldv, G, b * G.sb + h * G.sh, row0, row_end, ldt, ldt, 0);
    if (threadIdx.x < TR) m.qsh[threadIdx.x] = row0 + threadIdx.x < row_end ? -row_shift[(size_t)bh * L + row0 + threadIdx.x] : 0.f;
    __syncthreads();
    row_terms_of(m.rterm, ks, bh, L, row0, row_end, m.Ks, ld, d, Cmat2, 0.f);
    bwd_causal_amat(m.As, m.Gs, m.Vs, ldv, lds, ldt);

    f32x4 acc_o[ACC_PER_WAVE], acc_g[4];
#pragma unroll
    for (int t = 0; t < ACC_PER_WAVE; ++t) acc_o[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 4; ++t) acc_g[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    f32x4 sc = {0.f, 0.f, 0.f, 0.f};      // scores tile (query tile w>>1, key tile w&1)
    float rs_part = 0.f;
    for (int m0 = 0; m0 < M; m0 += MB) {
      const int f = (w & 1) * 16 + (lane & 15);
      __syncthreads();
      load_wblock(m.Ws, m.bias_s, ld, W1, bias1, m0, M, d, dpad);
      for (int idx = threadIdx.x; idx < MB * ldt; idx += NT) {
        const int ff = idx / ldt, cc = idx - ff * ldt;
        m.Ts[ff * ldv + cc] = (m0 + ff < M) ? Rg[(size_t)(m0 + ff) * ldt + cc] : 0.f;
      }
      __syncthreads();
      {
        const f32x4 e = proj_tile(m.Qs, m.Ws, ld, dpad);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = (w >> 1) * 16 + 4 * (lane >> 4) + r;
          m.Ps[row * lds + f] = (m0 + f < M && row0 + row < row_end) ? fast_exp2(e[r] + m.bias_s[f] + m.qsh[row]) : 0.f;
        }
      }
      __syncthreads();
      load_wblock(m.Ws, m.bias_s, ld, W2, bias2, m0, M, d, dpad);
      __syncthreads();
      {
        const f32x4 e = proj_tile(m.Ks, m.Ws, ld, dpad);
        float fv[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = (w >> 1) * 16 + 4 * (lane >> 4) + r;
          fv[r] = (m0 + f < M && row0 + row < row_end) ? fast_exp2(e[r] + m.bias_s[f] + m.rterm[row] - c) : 0.f;
          m.Ss[row * lds + f] = fv[r];
        }
        // dS tile (keys (w>>1)*16.., features (w&1)*16..) = V1 R_next^T + A^T P
        f32x4 ds = {0.f, 0.f, 0.f, 0.f};
        {
          const float* ap = m.Vs + ((w >> 1) * 16 + (lane & 15)) * ldv + (lane >> 4);   // A[j][k=v] = Vs[j][v]
          const float* bp = m.Ts + ((w & 1) * 16 + (lane & 15)) * ldv + (lane >> 4);    // B[k=v][n=m] = Rs[m][v]
          for (int k = 0; k < ldt; k += 4) ds = mfma4(ap[k], bp[k], ds);
        }
        {
          const float* ap = m.As + (lane >> 4) * lds + (w >> 1) * 16 + (lane & 15);     // A[j][k=i] = As[i][j]
          const float* bp = m.Ps + (lane >> 4) * lds + (w & 1) * 16 + (lane & 15);      // B[k=i][n=m] = Ps[i][m]
          for (int k = 0; k < TR; k += 4) ds = mfma4(ap[k * lds], bp[k * lds], ds);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = (w >> 1) * 16 + 4 * (lane >> 4) + r;
          m.dEs[row * lds + f] = fv[r] * ds[r];
        }
      }
      __syncthreads();
      {   // scores: A[i][k=m] = Ps[i][m], B[k=m][n=j] = Ss[j][m]
        const float* ap = m.Ps + ((w >> 1) * 16 + (lane & 15)) * lds + (lane >> 4);
        const float* bp = m.Ss + ((w & 1) * 16 + (lane & 15)) * lds + (lane >> 4);
        for (int k = 0; k < MB; k += 4) sc = mfma4(ap[k], bp[k], sc);
      }
#pragma unroll
      for (int tl = 0; tl < ACC_PER_WAVE; ++tl) {
        const int t = w + 4 * tl;
        if (t < ntiles) {
          const int rt = t & 1, vt = t >> 1;
          {   // dV1 += S R_next: A[j][k=m] = Ss[j][m], B[k=m][n=v] = Rs[m][v]
            const float* ap = m.Ss + (rt * 16 + (lane & 15)) * lds + (lane >> 4);
            const float* bp = m.Ts + (lane >> 4) * ldv + vt * 16 + (lane & 15);
            for (int k = 0; k < MB; k += 4) acc_o[tl] = mfma4(ap[k], bp[k * ldv], acc_o[tl]);
          }
          {   // the suffix sum takes this chunk's queries (after its last use): R[m][v] += sum_i Ps[i][m] Gs[i][v]
            f32x4 up = {0.f, 0.f, 0.f, 0.f};
            const float* ap = m.Ps + (lane >> 4) * lds + rt * 16 + (lane & 15);
            const float* bp = m.Gs + (lane >> 4) * ldv + vt * 16 + (lane & 15);
            for (int k = 0; k < TR; k += 4) up = mfma4(ap[k * lds], bp[k * ldv], up);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int mm = m0 + rt * 16 + 4 * (lane >> 4) + r;
              if (mm < M) Rg[(size_t)mm * ldt + vt * 16 + (lane & 15)] += up[r];
            }
          }
        }
      }
#pragma unroll
      for (int tl = 0; tl < 4; ++tl) {
        const int t = w + 4 * tl;
        if (t < ngt) {
          const int rt = t & 1, ct = t >> 1;
          const float* ap = m.dEs + (rt * 16 + (lane & 15)) * lds + (lane >> 4);
          const float* bp = m.Ws + (lane >> 4) * ld + ct * 16 + (lane & 15);
          const bool in = ct * 16 + (lane & 15) < dpad;
          f32x4 a = acc_g[tl];
          for (int k = 0; k < MB; k += 4) a = mfma4(ap[k], in ? bp[k * ld] : 0.f, a);
          acc_g[tl] = a;
        }
      }
      {
        const int row = threadIdx.x >> 3, part = threadIdx.x & 7;
#pragma unroll
        for (int q = 0; q < 4; ++q) rs_part += m.dEs[row * lds + part * 4 + q];
      }
    }
    // B = tril(P S^T); dV1 += B^T G1: A[j][k=i] = Bs[i][j], B[k=i][n=v] = Gs[i][v]
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int i = (w >> 1) * 16 + 4 * (lane >> 4) + r, j = (w & 1) * 16 + (lane & 15);
      m.Bs[i * lds + j] = (j <= i) ? sc[r] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int tl = 0; tl < ACC_PER_WAVE; ++tl) {
      const int t = w + 4 * tl;
      if (t < ntiles) {
        const int rt = t & 1, vt = t >> 1;
        const float* ap = m.Bs + (lane >> 4) * lds + rt * 16 + (lane & 15);
        const float* bp = m.Gs + (lane >> 4) * ldv + vt * 16 + (lane & 15);
        for (int k = 0; k < TR; k += 4) acc_o[tl] = mfma4(ap[k * lds], bp[k * ldv], acc_o[tl]);
      }
    }
    __syncthreads();
    float* Gd = m.Ws;
    float* Os = m.Ts;
#pragma unroll
    for (int tl = 0; tl < 4; ++tl) {
      const int t = w + 4 * tl;
      if (t < ngt) {
        const int rt = t & 1, ct = t >> 1, col = ct * 16 + (lane & 15);
        if (col < dpad) {
#pragma unroll
          for (int r = 0; r < 4; ++r) Gd[(rt * 16 + 4 * (lane >> 4) + r) * ld + col] = acc_g[tl][r];
        }
      }
    }
#pragma unroll
    for (int tl = 0; tl < ACC_PER_WAVE; ++tl) {
      const int t = w + 4 * tl;
      if (t < ntiles) {
        const int rt = t & 1, vt = t >> 1;
#pragma unroll
        for (int r = 0; r < 4; ++r) Os[(rt * 16 + 4 * (lane >> 4) + r) * ldv + vt * 16 + (lane & 15)] = acc_o[tl][r];
      }
    }
    rs_part += __shfl_xor(rs_part, 1);
    rs_part += __shfl_xor(rs_part, 2);
    rs_part += __shfl_xor(rs_part, 4);
    if ((threadIdx.x & 7) == 0) m.rsum[threadIdx.x >> 3] = rs_part;
    __syncthreads();
    bwd_store_grad(dK, b * dK.sb + h * dK.sh, row0, row_end, d, ld, Gd, m.rsum, m.Ks, Cmat2, ks.scale, 0.f);
    for (int idx = threadIdx.x; idx < TR * nv; idx += NT) {
      const int r = idx / nv, cc = idx - r * nv;
      if (row0 + r < row_end) store_elem(dV, b * dV.sb + h * dV.sh + (long long)(row0 + r) * dV.sl + cc, Os[r * ldv + cc]);
    }
  }
}

// ---------------------------------------------------------------------------------------------------
// host launchers
// ---------------------------------------------------------------------------------------------------
static size_t lds_floats_basic(int d) { const int ld = ((d + 3) & ~3) + 1; return (size_t)(TR + MB) * ld + MB + 2 * TR + TR; }

size_t gen_lds_features(int d) { return lds_floats_basic(d) * 4; }
size_t gen_lds_state(int d, int ldt) {
  const int ld = ((d + 3) & ~3) + 1;
  return ((size_t)(TR + MB) * ld + (size_t)TR * (ldt + 1) + (size_t)TR * (MB + 1) + MB + TR) * 4;
}
size_t gen_lds_apply(int d, int ldt) {
  const int ld = ((d + 3) & ~3) + 1;
  return ((size_t)(TR + MB) * ld + (size_t)MB * (ldt + 1) + (size_t)TR * (MB + 1) + MB + 3 * TR) * 4;
}
size_t gen_lds_causal(int d, int ldt) {
  const int ld = ((d + 3) & ~3) + 1;
  return ((size_t)(2 * TR + MB) * ld + (size_t)(TR + MB) * (ldt + 1) + (size_t)3 * TR * (MB + 1) + MB + 2 * TR) * 4;
}
size_t gen_lds_stats(int d) { return (size_t)TR * (((d + 15) & ~15) + 1) * 4; }

#define FS_LAUNCH_CHECK() do { if (hipGetLastError() != hipSuccess) return 5; } while (0)

static int set_lds(const void* fn, size_t bytes) {
  if (bytes > 48 * 1024) {
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) {
      (void)hipGetLastError();
      return 2;
    }
  }
  return 0;
}

int launch_prep(const float* theta, int groups, const float* Omega, int omega_groups, int pgroups, int B, int H,
                int M, int d, float* W, uint16_t* Wbf, float* bias, hipStream_t st) {
  hipLaunchKernelGGL(k_prep, dim3(M, 2, pgroups), dim3(128), 0, st, theta, groups, Omega, omega_groups, pgroups, B, H,
                     M, d, W, Wbf, bias);
  FS_LAUNCH_CHECK();
  return 0;
}

int launch_fill_u32(uint32_t* p, uint32_t v, size_t n, hipStream_t st) {
  if (n == 0) return 0;
  hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, v, n);
  FS_LAUNCH_CHECK();
  return 0;
}

int launch_gen_features(const TensorDev& X, int n, int d, float scale, float alpha, const float* W, const float* bias,
                        const float* theta, long long c_offset, int M, float* out, float* row_logscale,
                        hipStream_t st) {
  const size_t lds = gen_lds_features(d);
  if (int rc = set_lds((const void*)k_gen_features, lds)) return rc;
  hipLaunchKernelGGL(k_gen_features, dim3((n + TR - 1) / TR), dim3(NT), lds, st, X, n, d, scale, alpha, W, bias, theta,
                     c_offset, M, out, row_logscale);
  FS_LAUNCH_CHECK();
  return 0;
}

int launch_gen_kmax(const GenSide& ks, int Lk, int BH, int H, int M, int d, uint32_t* kmax_u, hipStream_t st) {
  const size_t lds = gen_lds_features(d);
  if (int rc = set_lds((const void*)k_gen_kmax, lds)) return rc;
  hipLaunchKernelGGL(k_gen_kmax, dim3((Lk + TR - 1) / TR, BH), dim3(NT), lds, st, ks, Lk, H, M, d, kmax_u);
  FS_LAUNCH_CHECK();
  return 0;
}

int launch_gen_state(const GenSide& ks, const TensorDev& V, int Lk, int BH, int H, int M, int d, int nv,
                     int append_ones, int ldt, int rows_per_seg, int nseg, const uint32_t* kmax_u,
                     const float* row_shift, float* Tpart, hipStream_t st) {
  const size_t lds = gen_lds_state(d, ldt);
  if (int rc = set_lds((const void*)k_gen_state, lds)) return rc;
  hipLaunchKernelGGL(k_gen_state, dim3(nseg, (M + MB - 1) / MB, BH), dim3(NT), lds, st, ks, V, Lk, H, M, d, nv,
                     append_ones, ldt, rows_per_seg, nseg, kmax_u, row_shift, Tpart);
  FS_LAUNCH_CHECK();
  return 0;
}

int launch_gen_reduce(float* Tpart, int BH, int nseg, size_t per_state, int prefix, hipStream_t st) {
  const size_t total = (size_t)BH * per_state;
  hipLaunchKernelGGL(k_gen_reduce, dim3((unsigned)((total + 63) / 64)), dim3(64, 4), 0, st, Tpart, nseg, per_state,
                     total, prefix);
  FS_LAUNCH_CHECK();
  return 0;
}

int launch_gen_apply(const GenSide& qs, int Lq, int BH, int H, int M, int d, int nv, int ldt, const float* T,
                     size_t state_stride, const uint32_t* kmax_u, int matvec, const TensorDev& Y, float* den_out,
                     float* shift_out, hipStream_t st, unsigned* flushed) {
  const size_t lds = gen_lds_apply(d, ldt);
  if (int rc = set_lds((const void*)k_gen_apply, lds)) return rc;
  hipLaunchKernelGGL(k_gen_apply, dim3((Lq + TR - 1) / TR, BH), dim3(NT), lds, st, qs, Lq, H, M, d, nv, ldt, T,
                     state_stride, kmax_u, matvec, Y, den_out, shift_out, flushed);
  FS_LAUNCH_CHECK();
  return 0;
}

size_t gen_lds_bwd_side(int d, int ldt) {
  const int ld = ((d + 3) & ~3) + 1;
  return ((size_t)(TR + MB) * ld + (size_t)(TR + MB) * (ldt + 1) + (size_t)2 * TR * (MB + 1) + MB + 2 * TR) * 4;
}

int launch_bwd_ghat(const TensorDev& dY, float* buf, const float* den, int L, int BH, int H, int nv, int ldt,
                    hipStream_t st) {
  const size_t rows = (size_t)BH * L;
  hipLaunchKernelGGL(k_bwd_ghat, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, st, dY, buf, den, L, H, nv, ldt, rows);
  FS_LAUNCH_CHECK();
  return 0;
}

int launch_gen_bwd_side(const GenSide& sd, int side, const TensorDev& A, int a_cols, int append_ones, int L, int BH,
                        int H, int M, int d, int nv, int ldt, const float* St, size_t state_stride,
                        const uint32_t* kmax_u, const float* row_shift, const TensorDev& out1, int want_out1,
                        const TensorDev& grad, hipStream_t st) {
  const size_t lds = gen_lds_bwd_side(d, ldt);
  if (int rc = set_lds((const void*)k_gen_bwd_side, lds)) return rc;
  hipLaunchKernelGGL(k_gen_bwd_side, dim3((L + TR - 1) / TR, BH), dim3(NT), lds, st, sd, side, A, a_cols, append_ones, L,
                     H, M, d, nv, ldt, St, state_stride, kmax_u, row_shift, out1, want_out1, grad);
  FS_LAUNCH_CHECK();
  return 0;
}

size_t gen_lds_bwd_causal(int d, int ldt) {
  const int ld = ((d + 3) & ~3) + 1;
  return ((size_t)(2 * TR + MB) * ld + (size_t)(2 * TR + MB) * (ldt + 1) + (size_t)5 * TR * (MB + 1) + MB + 3 * TR) * 4;
}

int launch_gen_bwd_causal(const GenSide& qs, const GenSide& ks, const TensorDev& V, const float* ghat, int L, int BH, int H,
                          int M, int d, int nv, int ldt, int rows_per_seg, int nseg, const uint32_t* kmax_u,
                          const float* row_shift, float* Tstate, float* Rstate, const TensorDev& dQ, const TensorDev& dK,
                          const TensorDev& dV, hipStream_t st) {
  const size_t lds = gen_lds_bwd_causal(d, ldt);
  if (int rc = set_lds((const void*)k_gen_bwd_causal_q, lds)) return rc;
  if (int rc = set_lds((const void*)k_gen_bwd_causal_k, lds)) return rc;
  hipLaunchKernelGGL(k_gen_bwd_causal_q, dim3(nseg, BH), dim3(NT), lds, st, qs, ks, V, ghat, L, H, M, d, nv, ldt,
                     rows_per_seg, nseg, kmax_u, row_shift, Tstate, dQ);
  FS_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_gen_bwd_causal_k, dim3(nseg, BH), dim3(NT), lds, st, qs, ks, V, ghat, L, H, M, d, nv, ldt,
                     rows_per_seg, nseg, kmax_u, row_shift, Rstate, dK, dV);
  FS_LAUNCH_CHECK();
  return 0;
}

int launch_gen_causal(const GenSide& qs, const GenSide& ks, const TensorDev& V, int L, int BH, int H, int M, int d,
                      int nv, int ldt, int rows_per_seg, int nseg, const uint32_t* kmax_u, float* Tstate,
                      const TensorDev& Y, float* den_out, float* shift_out, hipStream_t st, unsigned* flushed) {
  const size_t lds = gen_lds_causal(d, ldt);
  if (int rc = set_lds((const void*)k_gen_causal, lds)) return rc;
  hipLaunchKernelGGL(k_gen_causal, dim3(nseg, BH), dim3(NT), lds, st, qs, ks, V, L, H, M, d, nv, ldt, rows_per_seg,
                     nseg, kmax_u, Tstate, Y, den_out, shift_out, flushed);
  FS_LAUNCH_CHECK();
  return 0;
}

int launch_stats(const TensorDev& X, const TensorDev& Y, int B, int H, int Lx, int Ly, int d, float scale, int groups,
                 int rows_per_chunk, int nchunks, float* part, double* stats, hipStream_t st) {
  if (stats_bf16_supported(X, Y, d)) {
    if (int rc = launch_stats_bf16(X, Y, B * H, H, Lx, Ly, scale, rows_per_chunk, nchunks, part, st)) return rc;
  } else if (stats_wide_supported(X, Y, d)) {
    if (int rc = launch_stats_wide(X, Y, B * H, H, Lx, Ly, scale, rows_per_chunk, nchunks, part, st)) return rc;
  } else {
    const size_t lds = gen_lds_stats(d);
    if (int rc = set_lds((const void*)k_stats_partial, lds)) return rc;
    hipLaunchKernelGGL(k_stats_partial, dim3(nchunks, B * H, 2), dim3(NT), lds, st, X, Y, Lx, Ly, H, d, scale,
                       rows_per_chunk, nchunks, part);
    FS_LAUNCH_CHECK();
  }
  const size_t total = (size_t)groups * 2 * ((size_t)d * d + d);
  hipLaunchKernelGGL(k_stats_final, dim3((unsigned)((total + 127) / 128)), dim3(128), 0, st, part, B, H, nchunks, d,
                     groups, Lx, Ly, stats);
  FS_LAUNCH_CHECK();
  return 0;
}

}  // namespace fs
