// Backward pass of non-causal attention on the bf16 path (d = dv = 64, M = 256): gradients of sum(Y * dY) with
// respect to Q, K, V, theta and omega held fixed (chain rule on Section 2.2's attention equation with K_hat = P S^T).
//
// With V1 = [V 1], T = S^T V1 (the forward state, 256 x 65) and Yhat = P T (numerators and normaliser):
//   G1_i = [dY_i / den_i, -(dY_i . Y_i) / den_i]      (65 numbers per query, stored as rows of 80 bf16)
//   R    = P^T G1                                     (256 x 65, the query-side twin of the state)
//   dV   = (S R)[:, :64]
//   dP   = G1 T^T,  dE1 = P * dP,  dQ = dE1 (d E1 / d q)
//   dS   = V1 R^T,  dE2 = S * dS,  dK = dE2 (d E2 / d k)
// Exponents are in the log2 domain with W~ carrying log2(e) and qk_scale, so d E / d (raw row) = ln2 W~ plus, on
// the key side, the derivative of the row term y^T C2 y (y = qk_scale k): qk_scale^2 (C2 + C2^T) k times the row
// sum of dE2.  On the query side that row sum vanishes identically (Y does not depend on a per-row factor of P).
// The exponent shifts and the placement of the bias on the query side cancel in every product above, so the
// kernels work on the same shifted features as the forward pass.
//
// Kernels (one attention_backward call = forward state and reduction, then):
//   k_bwd_apply<1>   queries: Yhat = P T, normalise, G1 rows                         -> gh
//   k_bwd_rstate     queries: segment sums of P^T G1                                 -> Rpart (k_fast_reduce sums them)
//   k_bwd_apply<2>   keys:    dV = S R
//   k_bwd_grad<0/1>  queries / keys: dF = (state) (left rows)^T, dE = F * dF, gradient rows
//   k_bwd_whole      many or short sequences: all of the above (and the forward state) for one (b,h) per workgroup
// All of them keep a wave's 64 features of every operand in registers, as the forward kernels do.
#include "fast_bwd.h"
#include "fast_state.h"

namespace fs {

using namespace fast;

namespace bwd {

// ---------------------------------------------------------------------------------------------------------------
// MODE 1 (queries): rows of G1.  MODE 2 (keys): dV = S R.  Structure of k_fast_apply.  grid (nblk, B*H).
// ---------------------------------------------------------------------------------------------------------------
// Rows [row_beg, row_end) of one (b,h) against the state image tb (state^T as A operand: row v = 16 vt + c, k <->
// features 64w + 32 mb + 16 (e/4) + 4g + e%4); cs: the key shift of the sequence (MODE 2).  Returns the number of
// rows this wave finished with a zero normaliser (MODE 1).
template <int MODE>
__device__ __forceinline__ int apply_rows_b(const BwdArgs& ba, SmemApply& sm, int bh, const bf16x8 (&tb)[NVT][2], float cs,
                                            int row_beg, int row_end) {
  const FastArgs& a = ba.f;
  const int b = bh / a.H, h = bh % a.H;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  const int pg = group_of(a.pgroups, b, h, a.H);
  constexpr int side = MODE == 1 ? 0 : 1;
  const TensorDev& X = MODE == 1 ? a.Q : a.K;
  const float wmax = max256(a.wnorm + ((size_t)pg * 2 + side) * M), amax = max256(a.bias + ((size_t)pg * 2) * M);
  const uint16_t* Xb = (const uint16_t*)X.ptr + b * X.sb + h * X.sh;
  const float* th = a.theta + (size_t)group_of(a.groups, b, h, a.H) * (FS_THETA_HEADER_ + (size_t)D + 4 * (size_t)D * D);
  const bool isoC = ((int)th[2]) & 1;

  WSlice wx;
  load_wslice(wx, a.Wbf + ((size_t)pg * 2 + side) * M * D);
  QBias qb;
  load_qbias(qb, a.bias + ((size_t)pg * 2) * M, amax);
  int nzero = 0;                   // (MODE 1) rows this wave finished with a zero normaliser

  // staged rows -> LDS with what is added to their exponents: - row_shift (queries), row term - key shift (keys)
  auto stage = [&](const RowRegs& r, int buf, int row0) {
    float n2[2];
    store_rows_s(r, sm.q[buf], n2);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int q = threadIdx.x + NT * i, row = q >> 3;
      if ((q & 7) == 0) {
        float add;
        if (MODE == 1) add = -row_shift(n2[i], wmax);
        else {
          float rt = -0.5f * kLog2e * a.scale * a.scale * n2[i];
          if (!isoC) rt = row0 + row < row_end ? a.rk[(size_t)bh * a.L + row0 + row] : 0.f;
          add = rt - cs;
        }
        sm.qadd[buf][row] = add;
      }
    }
  };

  RowRegs xr;
  load_rows_g(xr, Xb, X.sl, row_beg, row_end);
  stage(xr, 0, row_beg);
  __syncthreads();
  int buf = 0;
  for (int row0 = row_beg; row0 < row_end; row0 += TC, buf ^= 1) {
    const bool more = row0 + TC < row_end;
    if (more) load_rows_g(xr, Xb, X.sl, row0 + TC, row_end);
    // (MODE 1) this wave's rows of dY are requested before the chunk's feature tiles and used after them
    f32x4 gpre[4] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
    if (MODE == 1 && row0 + 16 * w + c < row_end) {
      const long long go = b * ba.dY.sb + h * ba.dY.sh + (long long)(row0 + 16 * w + c) * ba.dY.sl + 4 * g;
      if (ba.dY.dtype == 1) {
#pragma unroll
        for (int vt = 0; vt < 4; ++vt) gpre[vt] = __builtin_convertvector(*(const bf16x4*)((const uint16_t*)ba.dY.ptr + go + 16 * vt), f32x4);
      } else {
#pragma unroll
        for (int vt = 0; vt < 4; ++vt) gpre[vt] = *(const f32x4*)((const float*)ba.dY.ptr + go + 16 * vt);
      }
    }
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      bf16x8 p[2];
      feature_tile<MODE == 1>(wx, &qb, sm.q[buf], it, sm.qadd[buf][16 * it + c], p);
      f32x4 y[NVT];
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) {
        y[vt] = mfma(tb[vt][0], p[0], f32x4{0.f, 0.f, 0.f, 0.f});
        y[vt] = mfma(tb[vt][1], p[1], y[vt]);
      }
      exchange_put_bf16(sm, y, it, w, lane);
    }
    __syncthreads();
    {
      f32x4 fs[4] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
      finish_tiles(fs, sm, w, 0, lane);
      finish_tiles(fs, sm, w, 2, lane);
      const int token = row0 + 16 * w + c;
      const bool valid = token < row_end;
      if (MODE == 1) {
        unsigned zt;
        const float inv = finish_norm(fs, sm, w, lane, &zt);      // fs = Y rows now
        nzero += count_zero_tokens(zt, w, row_end - row0);
        f32x4 gv[4];
        float dot = 0.f;
#pragma unroll
        for (int vt = 0; vt < 4; ++vt) {
          gv[vt] = gpre[vt];
#pragma unroll
          for (int r = 0; r < 4; ++r) dot += gv[vt][r] * fs[vt][r];
        }
        dot += __shfl_xor(dot, 16);
        dot += __shfl_xor(dot, 32);
        if (valid) {
          uint16_t* go = ba.gh + ((size_t)bh * ba.Lq + token) * DVP + 4 * g;
#pragma unroll
          for (int vt = 0; vt < 4; ++vt) *(bf16x4*)(go + 16 * vt) = __builtin_convertvector(gv[vt] * inv, bf16x4);
          const f32x4 last = {g == 0 ? -dot * inv : 0.f, 0.f, 0.f, 0.f};
          *(bf16x4*)(go + D) = __builtin_convertvector(last, bf16x4);
        }
      } else if (valid) {
        if (ba.dV.dtype == 1) {
          uint16_t* yp = (uint16_t*)ba.dV.ptr + b * ba.dV.sb + h * ba.dV.sh + (long long)token * ba.dV.sl + 4 * g;
#pragma unroll
          for (int vt = 0; vt < 4; ++vt) *(bf16x4*)(yp + 16 * vt) = __builtin_convertvector(fs[vt], bf16x4);
        } else {
          float* yp = (float*)ba.dV.ptr + b * ba.dV.sb + h * ba.dV.sh + (long long)token * ba.dV.sl + 4 * g;
#pragma unroll
          for (int vt = 0; vt < 4; ++vt) *(f32x4*)(yp + 16 * vt) = fs[vt];
        }
      }
    }
    if (more) stage(xr, buf ^ 1, row0 + TC);
    __syncthreads();
  }
  return nzero;
}

template <int MODE>
__global__ void __launch_bounds__(NT, 2) k_bwd_apply(BwdArgs ba, int rows_per_blk) {
  __shared__ SmemApply sm;
  const FastArgs& a = ba.f;
  const int blk = blockIdx.x, bh = blockIdx.y;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  const int L = MODE == 1 ? ba.Lq : ba.Lk;
  bf16x8 tb[NVT][2];
  const float* Sg = MODE == 1 ? a.Tpart + (size_t)bh * a.nslot * M * DVP : ba.Rpart + (size_t)bh * ba.rslots * M * DVP;
#pragma unroll
  for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      f32x8 t;
#pragma unroll
      for (int e = 0; e < 8; ++e) t[e] = Sg[(size_t)(64 * w + 32 * mb + 16 * (e >> 2) + 4 * g + (e & 3)) * DVP + 16 * vt + c];
      tb[vt][mb] = __builtin_convertvector(t, bf16x8);
    }
  const int row_beg = blk * rows_per_blk;
  const int nzero = apply_rows_b<MODE>(ba, sm, bh, tb, a.cstar[bh], row_beg, min(L, row_beg + rows_per_blk));
  if (MODE == 1) report_zero_rows(a.flushed, nzero, lane);
}

// ---------------------------------------------------------------------------------------------------------------
// Segment sums of P^T G1 (structure of k_fast_state: query features with their per-row shifts, "values" = rows of
// G1, all 80 columns).  grid (rslots, B*H); LDS: Smem (rows, transposed values, shifts).
// ---------------------------------------------------------------------------------------------------------------
__device__ __forceinline__ void rstate_rows(const BwdArgs& ba, Smem& sm, int bh, int row_beg, int row_end, f32x4 (&R)[4][NVT]) {
  const FastArgs& a = ba.f;
  const int b = bh / a.H, h = bh % a.H;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, c = lane & 15;
  const int pg = group_of(a.pgroups, b, h, a.H);
  const float wmax = max256(a.wnorm + ((size_t)pg * 2) * M), amax = max256(a.bias + ((size_t)pg * 2) * M);
  const uint16_t* Qb = (const uint16_t*)a.Q.ptr + b * a.Q.sb + h * a.Q.sh;
  const uint16_t* Gb = ba.gh + (size_t)bh * ba.Lq * DVP;

  WSlice wq;
  load_wslice(wq, a.Wbf + ((size_t)pg * 2) * M * D);
  float bcol[4];         // 2 (bias - largest bias) of feature 64w + 16 mt + c
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) bcol[mt] = 2.f * (a.bias[((size_t)pg * 2) * M + 64 * w + 16 * mt + c] - amax);
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt) R[mt][vt] = f32x4{0.f, 0.f, 0.f, 0.f};

  auto stage = [&](const RowRegs& qr, const RowRegs3& gr, int buf) {
    float n2[2];
    store_rows_s(qr, sm.k[buf], n2);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int q = threadIdx.x + NT * i;
      if ((q & 7) == 0) sm.kadd[buf][q >> 3] = -row_shift(n2[i], wmax);
    }
    store_g80_s(gr, sm.vt[buf]);
  };

  RowRegs qr;
  RowRegs3 gr;
  load_rows_g(qr, Qb, a.Q.sl, row_beg, row_end);
  load_g80_g(gr, Gb, row_beg, row_end);
  stage(qr, gr, 0);
  __syncthreads();

  int buf = 0;
  for (int row0 = row_beg; row0 < row_end; row0 += TC, buf ^= 1) {
    const bool more = row0 + TC < row_end;
    if (more) {
      load_rows_g(qr, Qb, a.Q.sl, row0 + TC, row_end);
      load_g80_g(gr, Gb, row0 + TC, row_end);
    }
#pragma unroll
    for (int jp = 0; jp < 2; ++jp) {
      bf16x8 st[4];
      feature_pair_major<true>(wq, bcol, sm.k[buf], sm.kadd[buf], jp, 0.f, st);
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) {
        const bf16x8 vop = load_vop(sm.vt[buf], jp, vt);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) R[mt][vt] = mfma(st[mt], vop, R[mt][vt]);
      }
    }
    if (more) stage(qr, gr, buf ^ 1);
    __syncthreads();
  }
}

__global__ void __launch_bounds__(NT) k_bwd_rstate(BwdArgs ba) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int slot = blockIdx.x, bh = blockIdx.y;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  const int row_beg = slot * ba.rows_per_rslot;
  f32x4 R[4][NVT];
  rstate_rows(ba, *reinterpret_cast<Smem*>(smem_raw), bh, row_beg, min(ba.Lq, row_beg + ba.rows_per_rslot), R);
  float* out = ba.Rpart + ((size_t)bh * ba.rslots + slot) * M * DVP;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
      for (int r = 0; r < 4; ++r) out[(size_t)(64 * w + 16 * mt + 4 * g + r) * DVP + 16 * vt + c] = R[mt][vt][r];
  if (threadIdx.x == 0) ba.rcpart[(size_t)bh * ba.rslots + slot] = 0.f;
}

// ---------------------------------------------------------------------------------------------------------------
// Gradient rows.  KEY = 0: dQ from (queries, left rows = G1, state = T).  KEY = 1: dK from (keys, left rows = [V 1],
// state = R).  Per 16-token tile: F (feature tile), dF = state x (left rows)^T in the same accumulator layout
// (rows = features, column = token), dE = F * dF, gradient tile = W~^T (A operand: rows = coordinates, k <->
// features; a row of ones appended: row sum of dE) x dE.  The four waves' partial gradient tiles are summed through
// LDS on the MFMA pipe.  grid (nblk, B*H); 74 kB of dynamic LDS: two workgroups per CU.
// ---------------------------------------------------------------------------------------------------------------
struct SmemGrad {
  __attribute__((aligned(16))) uint16_t q[1][TC][LDR];            // rows of the chunk (one buffer)
  float qadd[TC];
  __attribute__((aligned(16))) uint16_t lam[TC][LDL];             // left rows: G1 (queries) or [V 1 0..] (keys)
  __attribute__((aligned(16))) uint16_t xch[NW][NW][16][LDXB];
  // C2 + C2^T as A operands of the keys' row term when C2 is dense: [16-row tile][k-step][lane] (rows = gradient columns)
  __attribute__((aligned(16))) uint16_t csym[4][KS][64][8];
};

// Rows [row_beg, row_end) of one (b,h); sa: the state as A operand of dF (row f = 64w + 16mt + c, k = 32kk + 8g + e
// <-> column v, zero from 80 on); cs: the key shift of the sequence (KEY).
template <int KEY>
__device__ __forceinline__ void grad_rows(const BwdArgs& ba, SmemGrad& sm, int bh, const bf16x8 (&sa)[4][3], float cs,
                                          int row_beg, int row_end) {
  const FastArgs& a = ba.f;
  const int b = bh / a.H, h = bh % a.H;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  const int pg = group_of(a.pgroups, b, h, a.H);
  const TensorDev& X = KEY ? a.K : a.Q;
  const TensorDev& G = KEY ? ba.dK : ba.dQ;
  const float wmax = max256(a.wnorm + ((size_t)pg * 2 + KEY) * M), amax = max256(a.bias + ((size_t)pg * 2) * M);
  const uint16_t* Xb = (const uint16_t*)X.ptr + b * X.sb + h * X.sh;
  const uint16_t* Vb = (const uint16_t*)a.V.ptr + b * a.V.sb + h * a.V.sh;
  const uint16_t* Gb = ba.gh + (size_t)bh * ba.Lq * DVP;
  const float* th = a.theta + (size_t)group_of(a.groups, b, h, a.H) * (FS_THETA_HEADER_ + (size_t)D + 4 * (size_t)D * D);
  const bool isoC = ((int)th[2]) & 1;
  const float* C2 = th + FS_THETA_HEADER_ + D + 3 * (size_t)D * D;
  const uint16_t* Wg = a.Wbf + ((size_t)pg * 2 + KEY) * M * D;

  WSlice wx;
  load_wslice(wx, Wg);
  QBias qb;
  load_qbias(qb, a.bias + ((size_t)pg * 2) * M, amax);
  // W~^T as A operand of the gradient tile: row = coordinate 16dt + c, k <-> feature 64w + 32blk + 16(e/4) + 4g + e%4;
  // tile dt = 4 has ones in its row 0 (coordinate "64" = the row sum of dE) and zeros elsewhere
  bf16x8 wt[NVT][2];
#pragma unroll
  for (int dt = 0; dt < NVT; ++dt)
#pragma unroll
    for (int bk = 0; bk < 2; ++bk) {
      u32x4 v = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int f = 64 * w + 32 * bk + 16 * (e >> 2) + 4 * g + (e & 3);
        uint32_t bits;
        if (dt < 4) bits = Wg[(size_t)f * D + 16 * dt + c];
        else bits = c == 0 ? 0x3f80u : 0u;
        v[e >> 1] |= bits << (16 * (e & 1));
      }
      wt[dt][bk] = __builtin_bit_cast(bf16x8, v);
    }

  if (KEY && !isoC) {
    for (int piece = threadIdx.x; piece < 4 * KS * 64; piece += NT) {
      const int l = piece & 63, ks = (piece >> 6) % KS, dt = piece / (64 * KS);
      const int dd = 16 * dt + (l & 15), e0 = 32 * ks + 8 * (l >> 4);
      f32x8 cv;
#pragma unroll
      for (int e = 0; e < 8; ++e) cv[e] = C2[dd * D + e0 + e] + C2[(e0 + e) * D + dd];
      *(bf16x8*)(&sm.csym[dt][ks][l][0]) = __builtin_convertvector(cv, bf16x8);
    }
  }
  // zero padding of the left-rows tile (columns the staging never writes)
  for (int idx = threadIdx.x; idx < TC * (KL - (KEY ? D : DVP)); idx += NT) {
    const int n = KL - (KEY ? D : DVP);
    sm.lam[idx / n][(KEY ? D : DVP) + idx % n] = 0;
  }

  auto load_left = [&](RowRegs3& r, int row0) {
    if (KEY) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int q = threadIdx.x + NT * i, row = q >> 3, pc = q & 7;
        r.p[i] = u32x4{0u, 0u, 0u, 0u};
        if (row0 + row < row_end) r.p[i] = *(const u32x4*)(Vb + (long long)(row0 + row) * a.V.sl + pc * 8);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 3; ++i) {
        const int q = threadIdx.x + NT * i, row = q / 10, pc = q - 10 * row;
        r.p[i] = u32x4{0u, 0u, 0u, 0u};
        if (q < TC * 10 && row0 + row < row_end) r.p[i] = *(const u32x4*)(Gb + (size_t)(row0 + row) * DVP + pc * 8);
      }
    }
  };
  auto stage = [&](const RowRegs& xr, const RowRegs3& lr, int row0) {
    float n2[2];
    store_rows_s(xr, sm.q[0], n2);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int q = threadIdx.x + NT * i, row = q >> 3;
      if ((q & 7) == 0) {
        float add;
        if (!KEY) add = -row_shift(n2[i], wmax);
        else {
          float rt = -0.5f * kLog2e * a.scale * a.scale * n2[i];
          if (!isoC) rt = row0 + row < row_end ? a.rk[(size_t)bh * a.L + row0 + row] : 0.f;
          add = rt - cs;
        }
        sm.qadd[row] = add;
      }
    }
    if (KEY) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int q = threadIdx.x + NT * i, row = q >> 3, pc = q & 7;
        *(u32x4*)(&sm.lam[row][pc * 8]) = lr.p[i];
      }
      if (threadIdx.x < TC) sm.lam[threadIdx.x][D] = row0 + (int)threadIdx.x < row_end ? 0x3f80u : 0u;   // the ones column
    } else {
#pragma unroll
      for (int i = 0; i < 3; ++i) {
        const int q = threadIdx.x + NT * i, row = q / 10, pc = q - 10 * row;
        if (q < TC * 10) *(u32x4*)(&sm.lam[row][pc * 8]) = lr.p[i];
      }
    }
  };

  RowRegs xr;
  RowRegs3 lr;
  load_rows_g(xr, Xb, X.sl, row_beg, row_end);
  load_left(lr, row_beg);
  __syncthreads();                 // the zero padding is in place
  stage(xr, lr, row_beg);
  __syncthreads();
  for (int row0 = row_beg; row0 < row_end; row0 += TC) {
    const bool more = row0 + TC < row_end;
    if (more) {
      load_rows_g(xr, Xb, X.sl, row0 + TC, row_end);
      load_left(lr, row0 + TC);
    }
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      bf16x8 s[2];
      feature_tile<!KEY>(wx, &qb, sm.q[0], it, sm.qadd[16 * it + c], s);
      // dF: rows = features 16mt + 4g + r, column = token c
      f32x4 df[4] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
      for (int kk = 0; kk < 3; ++kk) {
        const bf16x8 lop = *(const bf16x8*)(&sm.lam[16 * it + c][32 * kk + 8 * g]);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) df[mt] = mfma(sa[mt][kk], lop, df[mt]);
      }
      // dE = F * dF, F from its bf16 image (element e of block bk <-> feature tile 2bk + e/4, row e%4)
      bf16x8 eimg[2];
#pragma unroll
      for (int bk = 0; bk < 2; ++bk) {
        const f32x8 fv = __builtin_convertvector(s[bk], f32x8);
        const f32x4 lo = {fv[0] * df[2 * bk][0], fv[1] * df[2 * bk][1], fv[2] * df[2 * bk][2], fv[3] * df[2 * bk][3]};
        const f32x4 hi = {fv[4] * df[2 * bk + 1][0], fv[5] * df[2 * bk + 1][1], fv[6] * df[2 * bk + 1][2], fv[7] * df[2 * bk + 1][3]};
        eimg[bk] = pack8(lo, hi);
      }
      f32x4 gt[NVT];
#pragma unroll
      for (int dt = 0; dt < NVT; ++dt) {
        if (dt < 4 || KEY) {
          gt[dt] = mfma(wt[dt][0], eimg[0], f32x4{0.f, 0.f, 0.f, 0.f});
          gt[dt] = mfma(wt[dt][1], eimg[1], gt[dt]);
        } else {
          gt[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
      }
      exchange_put_bf16(sm, gt, it, w, lane);
    }
    __syncthreads();
    {
      f32x4 fs[4] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
      finish_tiles(fs, sm, w, 0, lane);
      finish_tiles(fs, sm, w, 2, lane);
      const int trow = 16 * w + c, token = row0 + trow;
      if (KEY) {
        // derivative of the row term: rowsum(dE2) qk_scale^2 (C2 + C2^T) k   (C2 = -I/2: - qk_scale^2 k)
        const float rs = finish_col64(sm, w, lane) * a.scale * a.scale;
        if (isoC) {
#pragma unroll
          for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r = 0; r < 4; ++r)
              fs[dt][r] = kLn2 * fs[dt][r] - rs * bf16_bits_to_f32(sm.q[0][trow][16 * dt + 4 * g + r]);
        } else {
          // dense C2 (ADERF, SADERF): the matrix as A operand (rows = gradient columns), the key rows as B operand
          bf16x8 kop[KS];
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) kop[ks] = *(const bf16x8*)(&sm.q[0][trow][32 * ks + 8 * g]);
#pragma unroll
          for (int dt = 0; dt < 4; ++dt) {
            f32x4 u = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) u = mfma(*(const bf16x8*)(&sm.csym[dt][ks][lane][0]), kop[ks], u);
            fs[dt] = kLn2 * fs[dt] + rs * u;
          }
        }
      } else {
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) fs[dt] *= kLn2;
      }
      if (token < row_end) {
        if (G.dtype == 1) {
          uint16_t* yp = (uint16_t*)G.ptr + b * G.sb + h * G.sh + (long long)token * G.sl + 4 * g;
#pragma unroll
          for (int dt = 0; dt < 4; ++dt) *(bf16x4*)(yp + 16 * dt) = __builtin_convertvector(fs[dt], bf16x4);
        } else {
          float* yp = (float*)G.ptr + b * G.sb + h * G.sh + (long long)token * G.sl + 4 * g;
#pragma unroll
          for (int dt = 0; dt < 4; ++dt) *(f32x4*)(yp + 16 * dt) = fs[dt];
        }
      }
    }
    __syncthreads();               // every wave is done with the rows and the exchange buffer
    if (more) stage(xr, lr, row0 + TC);
    __syncthreads();
  }
}

template <int KEY>
__global__ void __launch_bounds__(NT, 2) k_bwd_grad(BwdArgs ba, int rows_per_blk) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const FastArgs& a = ba.f;
  const int blk = blockIdx.x, bh = blockIdx.y;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  const int L = KEY ? ba.Lk : ba.Lq;
  bf16x8 sa[4][3];
  {
    const float* Sg = KEY ? ba.Rpart + (size_t)bh * ba.rslots * M * DVP : a.Tpart + (size_t)bh * a.nslot * M * DVP;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int kk = 0; kk < 3; ++kk) {
        f32x8 t;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int v = 32 * kk + 8 * g + e;
          t[e] = v < DVP ? Sg[(size_t)(64 * w + 16 * mt + c) * DVP + v] : 0.f;
        }
        sa[mt][kk] = __builtin_convertvector(t, bf16x8);
      }
  }
  const int row_beg = blk * rows_per_blk;
  grad_rows<KEY>(ba, *reinterpret_cast<SmemGrad*>(smem_raw), bh, sa, a.cstar[bh], row_beg, min(L, row_beg + rows_per_blk));
}

// ---------------------------------------------------------------------------------------------------------------
// The whole backward pass of one (b,h) in one workgroup (non-causal calls with many or short sequences): the states T
// and R never leave the workgroup.  In the kernels above each of them goes to memory once per slot, through a
// reduction, and back twice, 80 kB a time, while a sequence of 128 tokens is 150 kB of rows altogether.  Phases, each
// the loop of one of the kernels above over all rows of the sequence:
//   keys:    T = S^T [V 1]                (state_rows)
//   queries: G1 rows -> gh                (apply_rows_b<1>, T as operand image)
//   queries: dQ                           (grad_rows<0>; T's image turned into the row operand through LDS)
//   queries: R = P^T G1                   (rstate_rows; gh read back: written by this workgroup, behind a barrier)
//   keys:    dV = S R                     (apply_rows_b<2>)
//   keys:    dK                           (grad_rows<1>)
// T is dead before R is built, so no phase holds more than its kernel does.  grid (B*H), block 256, two per CU.
// ---------------------------------------------------------------------------------------------------------------
union SmemBwdWhole {
  SmemState s;
  SmemApply q;
  Smem r;
  SmemGrad g;
  uint16_t tr[NW][64][LDL];        // a wave's state slice as rows of 96 columns (transposition of the operand image)
};

// Operand image of a state slice (apply kernels: tb[vt][mb] element e <-> feature 32 mb + 16 (e/4) + 4g + e%4, column
// 16 vt + c) -> rows operand of the gradient kernels (sa[mt][kk] element e <-> feature 16 mt + c, column 32 kk + 8g + e;
// columns 80 .. 95 zero), through the wave's own LDS rows.  Barriers on both sides: the region overlays the buffers
// of the phases before and after.
__device__ __forceinline__ void image_to_rows(const bf16x8 (&tb)[NVT][2], uint16_t (*tr)[LDL], bf16x8 (&sa)[4][3]) {
  const int lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
  __syncthreads();
#pragma unroll
  for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      const u32x4 bits = __builtin_bit_cast(u32x4, tb[vt][mb]);
#pragma unroll
      for (int e = 0; e < 8; ++e)
        tr[32 * mb + 16 * (e >> 2) + 4 * g + (e & 3)][16 * vt + c] = (uint16_t)(bits[e >> 1] >> (16 * (e & 1)));
    }
  *(u32x4*)(&tr[lane][DVP]) = u32x4{0u, 0u, 0u, 0u};
  *(u32x4*)(&tr[lane][DVP + 8]) = u32x4{0u, 0u, 0u, 0u};
  __syncthreads();
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int kk = 0; kk < 3; ++kk) sa[mt][kk] = *(const bf16x8*)(&tr[16 * mt + c][32 * kk + 8 * g]);
  __syncthreads();
}

__device__ __forceinline__ void pack_state(const f32x4 (&T)[4][NVT], bf16x8 (&tb)[NVT][2]) {
#pragma unroll
  for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) tb[vt][mb] = pack8(T[2 * mb][vt], T[2 * mb + 1][vt]);
}

__global__ void __launch_bounds__(NT, 2) k_bwd_whole(BwdArgs ba) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  SmemBwdWhole& sm = *reinterpret_cast<SmemBwdWhole*>(smem_raw);
  const FastArgs& a = ba.f;
  const int bh = blockIdx.x, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  bf16x8 tb[NVT][2];
  float cs;
  {
    f32x4 T[4][NVT];
    state_rows(a, sm.s, bh, 0, ba.Lk, T, cs);
    pack_state(T, tb);
  }
  const int nzero = apply_rows_b<1>(ba, sm.q, bh, tb, cs, 0, ba.Lq);
  report_zero_rows(a.flushed, nzero, lane);
  {
    bf16x8 sa[4][3];
    image_to_rows(tb, sm.tr[w], sa);
    grad_rows<0>(ba, sm.g, bh, sa, cs, 0, ba.Lq);
  }
  {
    f32x4 R[4][NVT];
    rstate_rows(ba, sm.r, bh, 0, ba.Lq, R);
    pack_state(R, tb);
  }
  apply_rows_b<2>(ba, sm.q, bh, tb, cs, 0, ba.Lk);
  {
    bf16x8 sa[4][3];
    image_to_rows(tb, sm.tr[w], sa);
    grad_rows<1>(ba, sm.g, bh, sa, cs, 0, ba.Lk);
  }
}

#define FS_LAUNCH_CHECK_() do { if (hipGetLastError() != hipSuccess) return 5; } while (0)
int launch_bwd_rstate(const BwdArgs& ba, int BH, hipStream_t st) {
  hipLaunchKernelGGL(k_bwd_rstate, dim3(ba.rslots, BH), dim3(NT), sizeof(Smem), st, ba);
  FS_LAUNCH_CHECK_();
  return 0;
}

}  // namespace bwd

using namespace bwd;

#define FS_LAUNCH_CHECK() do { if (hipGetLastError() != hipSuccess) return 5; } while (0)

size_t fast_bwd_lds_bytes() { return sizeof(SmemBwdWhole); }

// One non-causal backward call with a workgroup per sequence (after the constants; no state pass before it).
int launch_fast_backward_whole(const FastLaunch& f, const FastArgs& a, const TensorDev& dY, const TensorDev& dQ,
                               const TensorDev& dK, const TensorDev& dV, uint16_t* gh, hipStream_t st) {
  static_assert(sizeof(SmemBwdWhole) <= 80 * 1024, "k_bwd_whole: two workgroups per CU");
  BwdArgs ba;
  ba.f = a;
  ba.dY = dY; ba.dQ = dQ; ba.dK = dK; ba.dV = dV;
  ba.gh = gh; ba.Rpart = nullptr; ba.rcpart = nullptr;
  ba.Lq = f.Lq; ba.Lk = f.Lk; ba.rslots = 0; ba.rows_per_rslot = 0;
  if (hipFuncSetAttribute((const void*)k_bwd_whole, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(SmemBwdWhole)) != hipSuccess) {
    (void)hipGetLastError();
    return 2;
  }
  hipLaunchKernelGGL(k_bwd_whole, dim3(f.B * f.H), dim3(NT), sizeof(SmemBwdWhole), st, ba);
  FS_LAUNCH_CHECK();
  return 0;
}

// One non-causal backward call after the forward state pass (f.Tpart slot 0 = total state, f.cstar = key shifts).
int launch_fast_backward(const FastLaunch& f, const FastArgs& a, const TensorDev& dY, const TensorDev& dQ,
                         const TensorDev& dK, const TensorDev& dV, uint16_t* gh, float* Rpart, float* rcpart,
                         float* rcstar, int rslots, int rows_per_rslot, hipStream_t st) {
  BwdArgs ba;
  ba.f = a;
  ba.dY = dY; ba.dQ = dQ; ba.dK = dK; ba.dV = dV;
  ba.gh = gh; ba.Rpart = Rpart; ba.rcpart = rcpart;
  ba.Lq = f.Lq; ba.Lk = f.Lk; ba.rslots = rslots; ba.rows_per_rslot = rows_per_rslot;
  const int BH = f.B * f.H;
  auto blocks = [&](int L, int* rows_per_blk) {
    const int want = std::max(1, std::min((512 + BH - 1) / BH, (L + TC - 1) / TC));
    *rows_per_blk = (((L + want - 1) / want) + TC - 1) / TC * TC;
    return (L + *rows_per_blk - 1) / *rows_per_blk;
  };
  int rq, rk;
  const int nq = blocks(f.Lq, &rq), nk = blocks(f.Lk, &rk);
  if (hipFuncSetAttribute((const void*)k_bwd_grad<0>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(SmemGrad)) != hipSuccess ||
      hipFuncSetAttribute((const void*)k_bwd_grad<1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(SmemGrad)) != hipSuccess) {
    (void)hipGetLastError();
    return 2;
  }
  hipLaunchKernelGGL(k_bwd_apply<1>, dim3(nq, BH), dim3(NT), 0, st, ba, rq);
  FS_LAUNCH_CHECK();
  if (int rc = launch_bwd_rstate(ba, BH, st)) return rc;
  launch_fast_reduce_sum(Rpart, rcpart, rcstar, rslots, BH, st);
  FS_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_bwd_apply<2>, dim3(nk, BH), dim3(NT), 0, st, ba, rk);
  FS_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_bwd_grad<0>, dim3(nq, BH), dim3(NT), sizeof(SmemGrad), st, ba, rq);
  FS_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_bwd_grad<1>, dim3(nk, BH), dim3(NT), sizeof(SmemGrad), st, ba, rk);
  FS_LAUNCH_CHECK();
  return 0;
}

}  // namespace fs
