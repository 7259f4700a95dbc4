// Key-side state pass of the bf16 path (d = dv = 64, M = 256), shared by the forward kernels (kernels_bf16.hip) and
// the backward kernel that takes a whole sequence per workgroup (kernels_bf16_bwd.hip).
#pragma once
#include "fast_pc.h"

namespace fs {

using namespace fast;

// ---------------------------------------------------------------------------------------------------
// Key-side state of a range of rows: T = sum_j S'_j [V_j 1]^T / 2^dk, S' = features without the bias (Section 2.1,
// S^T C with C = [V 1]), for a workgroup of 256 threads (two per CU).
//
// Four waves of 64 features; per 64-token chunk every wave builds its feature tiles feature-major (A = token rows,
// B = W~; the per-token part of the exponent is the accumulator's initial value, read from LDS as a 16-byte vector)
// and adds S^T [V 1] to its state slice in registers.  Key and value rows stay row-major in LDS as they are in
// memory (global -> registers -> LDS, no arithmetic on the way): the value operand is a transposing LDS read, the
// squared row norms (row term -|y|^2/2 and the bound for the running shift) are the diagonal of Y Y^T on the MFMA
// pipe, computed by wave w for token tile w ONE CHUNK AHEAD, so that a single barrier per chunk orders everything:
// iteration c computes the constants of chunk c+1 (its key rows arrived in iteration c-1: three key buffers),
// contracts chunk c, and stores the value rows of chunk c+1 and the key rows of chunk c+2.  The largest bound of a
// chunk is gathered with an LDS float maximum, so the chunk starts with one broadcast read instead of a reduction.
// A wave executes in order, so every LDS read of a chunk is issued at the top of the iteration, ahead of the MFMA
// and exp2 streams that consume them.
// ---------------------------------------------------------------------------------------------------
struct SmemState {
  uint16_t k[3][TC][LDR];                                   // key rows of three consecutive chunks
  __attribute__((aligned(16))) uint16_t v[2][TC][LDV];      // value rows (columns 64.. are constant: 1, 0, ..)
  __attribute__((aligned(16))) float kadd[2][TC];           // per key token: row term (-inf past the end)
  float kmax[4];                                            // largest row_shift + row term of a chunk, at chunk index % 3
};

// The state of the key rows [row_beg, row_end) of one (b,h), left in the registers of the workgroup's four waves
// (wave w: features 64w .. 64w+63 x 80 columns) on the shift dk.  Ends behind a barrier: the caller may reuse the LDS.
// BOUND_ONLY: nothing but dk, the largest bound of the rows (the shift such a state would have): no projections, no
// values, T untouched.
template <bool BOUND_ONLY = false>
__device__ __forceinline__ void state_rows(const FastArgs& a, SmemState& sm, int bh, int row_beg, int row_end,
                                           f32x4 (&T)[4][NVT], float& dk) {
  const int b = bh / a.H, h = bh % a.H;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, g = lane >> 4, c = lane & 15;
  const int pg = group_of(a.pgroups, b, h, a.H);
  const float* th = a.theta + (size_t)group_of(a.groups, b, h, a.H) * (FS_THETA_HEADER_ + (size_t)D + 4 * (size_t)D * D);
  const bool isoC = ((int)th[2]) & 1;
  const float wmax = max256(a.wnorm + ((size_t)pg * 2 + 1) * M);
  const uint16_t* Kb = (const uint16_t*)a.K.ptr + b * a.K.sb + h * a.K.sh + (long long)row_beg * a.K.sl;
  const uint16_t* Vb = (const uint16_t*)a.V.ptr + b * a.V.sb + h * a.V.sh + (long long)row_beg * a.V.sl;
  const float* rkb = a.rk + (size_t)bh * a.L + row_beg;
  const int nrows = row_end - row_beg;

  WSlice wk;
  if (!BOUND_ONLY) {
    load_wslice(wk, a.Wbf + ((size_t)pg * 2 + 1) * M * D);
    init_value_pad(sm.v[0], 2 * TC, NT);
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) T[mt][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  if (tid < 3) sm.kmax[tid] = -INFINITY;
  dk = -INFINITY;

  // staging: thread -> rows tid/8 and tid/8 + 32 of a chunk, bytes 16 (tid%8); rows past the end read as zero
  // (a fresh descriptor per chunk: uniform base = the chunk's first row, 32-bit offsets inside the chunk)
  const int srow = tid >> 3, spc = tid & 7;
  u32x4 kr[2], vr[2];
  auto load_k = [&](int r0) {
    const __amdgpu_buffer_rsrc_t rk_ = pc::chunk_rsrc(Kb + (long long)r0 * a.K.sl, 2 * (int)a.K.sl, nrows - r0, 2 * D);
#pragma unroll
    for (int i = 0; i < 2; ++i) kr[i] = __builtin_amdgcn_raw_buffer_load_b128(rk_, 2 * ((srow + 32 * i) * (int)a.K.sl + spc * 8), 0, 0);
  };
  auto load_v = [&](int r0) {
    if (BOUND_ONLY) return;
    const __amdgpu_buffer_rsrc_t rv_ = pc::chunk_rsrc(Vb + (long long)r0 * a.V.sl, 2 * (int)a.V.sl, nrows - r0, 2 * D);
#pragma unroll
    for (int i = 0; i < 2; ++i) vr[i] = __builtin_amdgcn_raw_buffer_load_b128(rv_, 2 * ((srow + 32 * i) * (int)a.V.sl + spc * 8), 0, 0);
  };
  auto store_k = [&](int kb) {
#pragma unroll
    for (int i = 0; i < 2; ++i) *(u32x4*)(&sm.k[kb][srow + 32 * i][spc * 8]) = kr[i];
  };
  auto store_v = [&](int vb) {
    if (BOUND_ONLY) return;
#pragma unroll
    for (int i = 0; i < 2; ++i) *(u32x4*)(&sm.v[vb][srow + 32 * i][spc * 8]) = vr[i];
  };
  // Per-token constants of token tile w of a chunk (first row r0 of the slot) from the squared norms n2 of its rows
  // (valid in the lanes (g, c) = (c / 4, c)): row terms to kadd[cb], the largest bound into kmax[mb].
  // (`rkv`: the token's row term from memory, for parameter sets with a dense C2: requested by the caller ahead of time)
  auto row_term_of = [&](int r0) {
    float v = 0.f;
    if (!isoC && g == (c >> 2) && r0 + 16 * w + c < nrows) v = rkb[r0 + 16 * w + c];
    return v;
  };
  auto constants = [&](float n2, float rkv, int cb, int mb, int r0) {
    if (g == (c >> 2)) {
      const int t = 16 * w + c;
      const bool valid = r0 + t < nrows;
      float rt = -0.5f * kLog2e * a.scale * a.scale * n2;
      if (!isoC) rt = valid ? rkv : 0.f;
      // rows past the end get -inf: their features are exactly zero whatever the key shift is
      sm.kadd[cb][t] = valid ? rt : -INFINITY;
      if (valid) lds_fmax(&sm.kmax[mb], row_shift(n2, wmax) + rt);
    }
  };
  auto tile_op = [&](int kb, int jt, int ks) { return *(const bf16x8*)(&sm.k[kb][16 * jt + c][32 * ks + 8 * g]); };

  // the first two chunks' key rows and the first chunk's value rows in one round trip
  {
    load_k(0);
    load_v(0);
    const u32x4 k0[2] = {kr[0], kr[1]};
    load_k(TC);
    store_k(1);
    kr[0] = k0[0]; kr[1] = k0[1];
    store_k(0);
    store_v(0);
  }
  __syncthreads();
  constants(tile_row_norms(tile_op(0, w, 0), tile_op(0, w, 1), lane), row_term_of(0), 0, 0, 0);
  load_v(TC);
  load_k(2 * TC);
  __syncthreads();

  int kcur = 0, knext = 1, kfree = 2;
  for (int r0 = 0, ci = 0; r0 < nrows; r0 += TC, ++ci) {
    const int cb = ci & 1;
    if constexpr (BOUND_ONLY) {
      // the constants of the next chunk and the running maximum only
      const float dnew = sm.kmax[kcur];
      const bf16x8 xn0 = tile_op(knext, w, 0), xn1 = tile_op(knext, w, 1);
      const float rk_next = row_term_of(r0 + TC);
      dk = fmaxf(dk, dnew);
      const float n2 = tile_row_norms(xn0, xn1, lane);
      if (tid == 0) sm.kmax[kfree] = -INFINITY;
      constants(n2, rk_next, cb ^ 1, knext, r0 + TC);
      store_k(kfree);
      load_k(r0 + 3 * TC);
      __syncthreads();
      const int t = kcur; kcur = knext; knext = kfree; kfree = t;
      continue;
    }
    // ---- every LDS read of the chunk, up front
    const float dnew = sm.kmax[kcur];
    bf16x8 x[4][KS];
    f32x4 kadd4[4];
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) x[jt][ks] = tile_op(kcur, jt, ks);
      kadd4[jt] = *(const f32x4*)(&sm.kadd[cb][16 * jt + 4 * g]);
    }
    const bf16x8 xn0 = tile_op(knext, w, 0), xn1 = tile_op(knext, w, 1);     // token tile w of the next chunk
    const float rk_next = row_term_of(r0 + TC);      // (dense C2) requested here, used at the end of the iteration
    // ---- running key shift: the state is rebased when the chunk's largest bound exceeds the current shift
    if (dnew > dk) {
      const float f = fast_exp2(dk - dnew);
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt) T[mt][vt] *= f;
      dk = dnew;
    }
    // ---- projections of both token pairs (32 MFMAs); the value operands are requested behind them, the exp2 /
    // convert stream of a pair runs beside the MFMAs of the other one
    f32x4 acc[2][4][2];            // [pair][feature tile][tile of the pair]
    bf16x8 vop[2][NVT];
#pragma unroll
    for (int jp = 0; jp < 2; ++jp) {
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
          acc[jp][mt][jj] = mfma(x[2 * jp + jj][0], wk.w[mt][0], kadd4[2 * jp + jj] - dk);
#pragma unroll
          for (int ks = 1; ks < KS; ++ks) acc[jp][mt][jj] = mfma(x[2 * jp + jj][ks], wk.w[mt][ks], acc[jp][mt][jj]);
        }
      if (jp == 0) {
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt) vop[0][vt] = load_vop_tr(sm.v[cb], 0, vt, lane);
      }
    }
    const float n2 = tile_row_norms(xn0, xn1, lane);
    if (tid == 0) sm.kmax[kfree] = -INFINITY;    // last read in the previous iteration, gathered again in the next one
#pragma unroll
    for (int jp = 0; jp < 2; ++jp) {
      bf16x8 st[4];
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) st[mt] = pack8(exp2v(acc[jp][mt][0]), exp2v(acc[jp][mt][1]));
      if (jp == 0) {
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt) vop[1][vt] = load_vop_tr(sm.v[cb], 1, vt, lane);
      }
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) T[mt][vt] = mfma(st[mt], vop[jp][vt], T[mt][vt]);
    }
    constants(n2, rk_next, cb ^ 1, knext, r0 + TC);
    store_v(cb ^ 1);
    store_k(kfree);
    load_v(r0 + 2 * TC);
    load_k(r0 + 3 * TC);
    __syncthreads();
    const int t = kcur; kcur = knext; knext = kfree; kfree = t;
  }
}

}  // namespace fs
