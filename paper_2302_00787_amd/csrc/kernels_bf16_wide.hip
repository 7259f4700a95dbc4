// bf16 path of FAVOR# attention for d = dv = 128, M = 512 (the long-context shape): causal and non-causal (the same
// kernels: the reduction then leaves the sum of all slot states, and the walk has no first side and its own
// division of the queries into slots).
//
// The kernels for d = dv = 64, M = 256 keep 64 features x 80 state columns per wave in registers.  This shape is
// four such problems: the sums over features that make up numerator and normaliser split into two halves of 256
// features, and the value columns into [V_0..63, 1] and [V_64..127, 1] (the normaliser column rides along in both:
// the fifth value tile of a wave is there anyway).  Every (feature half, column half) combination is the producer /
// consumer walk of the forward pass (fast_pc.h) with projections of depth 128.  Two launches: the first runs both
// column halves of feature half 0 and leaves UNNORMALISED partial rows (fp32) and partial normalisers; the second
// runs feature half 1, adds the first launch's partial rows to its own in the finishing step, divides by the sum
// of the two partial normalisers and stores Y.  All combinations share every shift (the per-row query shift and the
// per-slot key shift are bounds over all 512 features), so their partial rows are on one scale.
//
//   k_wide_pre     projection constants for both sides (Section 4, evaluation recipe)
//   (k_key_row_terms of the d = 64 file: the key row terms of parameter sets with a dense C2)
//   k_wide_state   per (slot, feature half): S^T [V 1] over the slot (eight waves of 32 features, all 129 columns)
//   k_wide_reduce  exclusive prefix over the slots, each on the running maximum of the slots' shifts
//   k_wide_walk    per (slot, column half), once per feature half: the causal walk; the second launch finishes Y
#include <hip/hip_ext.h>

#include <algorithm>

#include "fast_pc.h"

namespace fs {

using namespace fast;

namespace wide {

using namespace pc;

constexpr int DW = 128;            // head and value dimension
constexpr int MW = 512;            // random features
constexpr int KSW = DW / 32;       // MFMA k-steps of a projection
constexpr int LDRW = DW + 8;       // row stride (bf16) of a token tile in LDS: 68 dwords
constexpr int NVW = 9;             // value tiles of the state kernel: 128 columns + the ones column + padding
constexpr int TLD = NVW * 16;      // row stride (floats) of a state: 144; column 128 = normaliser
constexpr int YLD = 132;           // row stride (floats) of a partial output row: 128 columns, partial normaliser of column half ch at 128 + ch

struct WideArgs {
  TensorDev Q, K, V, Y;
  const float* theta;
  const float* Omega;
  uint16_t* Wbf;     // [pg][2][512][128]
  float* bias;       // [pg][2][512]
  float* wnorm;      // [pg][2][512]
  float* rk;         // [BH][L]
  float* Tpart;      // [BH][2][nslot][256][144]
  float* cpart;      // [BH][nslot]
  float* cstar;      // [BH] largest shift of each sequence, then [BH][nslot] the key shift of each slot
  float* Ypart;      // [BH][Lq][132]: partial rows of feature half 0
  int groups, omega_groups, pgroups, B, H, L, nslot, rows_per_slot;   // L keys in nslot slots (state kernel, reduction)
  int Lq, rows_per_slot_q;   // the walk's rows and its slots (causal calls: the same numbers as the key side's)
  int fh;            // feature half of this launch of the walk
  float scale;
  unsigned* flushed; // counter of output rows with a zero normaliser (nullptr: not counted)
  const float* zero_state;   // causal call with one slot per sequence: a state of zeros, the start of every walk
};

__device__ __forceinline__ float max512(const float* p) {
  const int lane = threadIdx.x & 63;
  const f32x4 a = *(const f32x4*)(p + 4 * lane), b = *(const f32x4*)(p + 256 + 4 * lane);
  const float m = wave_max(fmaxf(fmaxf(fmaxf(a[0], a[1]), fmaxf(a[2], a[3])), fmaxf(fmaxf(b[0], b[1]), fmaxf(b[2], b[3]))));
  return __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, m)));
}
// Sum over the row of 16 lanes the lane belongs to.
__device__ __forceinline__ float sum16(float v) {
  v = sum8(v);
  v += dpp_f<0x128>(v);
  return v;
}

// ---------------------------------------------------------------------------------------------------
// Projection constants: grid 32 * 2 * pgroups workgroups of 256 threads; see k_fast_pre.  A wave computes four
// features at a time (every number of B it requests serves all four: the kernel is bound by those requests), lane c
// handles columns c and c + 64.
// ---------------------------------------------------------------------------------------------------
constexpr int PREF = 4;            // features per wave
__global__ void __launch_bounds__(256) k_wide_pre(WideArgs a, int* dense_flag) {
  const size_t tf = FS_THETA_HEADER_ + (size_t)DW + 4 * (size_t)DW * DW;
  const int H = a.H, block = blockIdx.x;
  const int c = threadIdx.x & 63;
  constexpr int per_side = MW / (4 * PREF);
  const int pg = block / (per_side * 2), rem = block % (per_side * 2), side = rem / per_side;
  const int m0 = (rem % per_side) * 4 * PREF + (threadIdx.x >> 6) * PREF;
  int b = 0, h = 0;
  if (a.pgroups == H && a.pgroups != 1) h = pg;
  else if (a.pgroups != 1) { b = pg / H; h = pg % H; }
  const float* th = a.theta + (size_t)group_of(a.groups, b, h, H) * tf;
  if (dense_flag != nullptr && rem == 0 && threadIdx.x == 0 && !(((int)th[2]) & 1)) atomicOr(dense_flag, 1);
  const float* om = a.Omega + ((size_t)group_of(a.omega_groups, b, h, H) * MW + m0) * DW;
  const float* Bm = th + FS_THETA_HEADER_ + DW + (side ? (size_t)DW * DW : 0);
  const float* A = th + FS_THETA_HEADER_;
  float acc0[PREF], acc1[PREF];
#pragma unroll
  for (int f = 0; f < PREF; ++f) acc0[f] = acc1[f] = 0.f;
#pragma unroll 4
  for (int l = 0; l < DW; ++l) {
    const float v0 = Bm[l * DW + c], v1 = Bm[l * DW + c + 64];
#pragma unroll
    for (int f = 0; f < PREF; ++f) {
      const float o = om[f * DW + l];
      acc0[f] += o * v0;
      acc1[f] += o * v1;
    }
  }
#pragma unroll
  for (int f = 0; f < PREF; ++f) {
    const size_t o = ((size_t)pg * 2 + side) * MW + m0 + f;
    const uint16_t b0 = f32_to_bf16_bits(acc0[f] * kLog2e * a.scale), b1 = f32_to_bf16_bits(acc1[f] * kLog2e * a.scale);
    a.Wbf[o * DW + c] = b0;
    a.Wbf[o * DW + c + 64] = b1;
    const float r0 = bf16_bits_to_f32(b0), r1 = bf16_bits_to_f32(b1);
    const float* of = om + f * DW;
    float n2 = r0 * r0 + r1 * r1, q = A[c] * of[c] * of[c] + A[c + 64] * of[c + 64] * of[c + 64];
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) { n2 += __shfl_xor(n2, s); q += __shfl_xor(q, s); }
    if (c == 0) {
      a.bias[o] = kLog2e * (q + th[0] - 0.5f * logf((float)MW));
      a.wnorm[o] = sqrtf(n2);
    }
  }
}

// Rows of 128 numbers: 16 pieces of 16 bytes; returns in every lane of the 16 that share the row its squared norm.
__device__ __forceinline__ float store_row_piece_w(u32x4 p, uint16_t (*tile)[LDRW], int row, int pc) {
  *(u32x4*)(&tile[row][pc * 8]) = p;
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float lo = __uint_as_float(p[e] << 16), hi = __uint_as_float(p[e] & 0xffff0000u);
    s += lo * lo + hi * hi;
  }
  return sum16(s);
}

// ---------------------------------------------------------------------------------------------------
// Key-side state of one slot and one feature half: Tpart = sum_j S'_j [V_j 1]^T / 2^cpart.  Eight waves of 32
// features; feature tiles feature-major (projection MFMA with swapped operands).  grid (nslot, B*H, 2), block 512.
// ---------------------------------------------------------------------------------------------------
struct SmemWState {
  __attribute__((aligned(16))) uint16_t k[2][TC][LDRW];
  __attribute__((aligned(16))) uint16_t vt[2][TLD][LDJ];     // [column][token]; row 128 = ones, rows 129.. = 0
  __attribute__((aligned(16))) float kadd[2][TC];
  __attribute__((aligned(16))) float kbnd[2][TC];
};

// BOUND_ONLY (causal calls with one slot per sequence: the walk starts from nothing and needs the key shift only):
// no projections, no values, no state; the shift goes where the reduction would have put it and the call's counter of
// flushed rows back to zero.  grid (1, B*H, 1).
template <bool BOUND_ONLY>
__global__ void __launch_bounds__(512) k_wide_state(WideArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  SmemWState& sm = *reinterpret_cast<SmemWState*>(smem_raw);
  const int slot = blockIdx.x, bh = blockIdx.y, fh = blockIdx.z, b = bh / a.H, h = bh % a.H;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, g = lane >> 4, c = lane & 15;
  const int pg = group_of(a.pgroups, b, h, a.H);
  const float* th = a.theta + (size_t)group_of(a.groups, b, h, a.H) * (FS_THETA_HEADER_ + (size_t)DW + 4 * (size_t)DW * DW);
  const bool isoC = ((int)th[2]) & 1;
  const float wmax = max512(a.wnorm + ((size_t)pg * 2 + 1) * MW);
  const uint16_t* Kb = (const uint16_t*)a.K.ptr + b * a.K.sb + h * a.K.sh;
  const uint16_t* Vb = (const uint16_t*)a.V.ptr + b * a.V.sb + h * a.V.sh;
  const int row_beg = min(a.L, slot * a.rows_per_slot), row_end = min(a.L, row_beg + a.rows_per_slot);

  // projection slice as B operand: column = feature 256 fh + 32 w + 16 mt + c, k = 32 ks + 8g + e
  bf16x8 wk[2][KSW];
  if (!BOUND_ONLY) {
    const uint16_t* Wg = a.Wbf + ((size_t)pg * 2 + 1) * MW * DW;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int ks = 0; ks < KSW; ++ks)
        wk[mt][ks] = *(const bf16x8*)(Wg + (size_t)(256 * fh + 32 * w + 16 * mt + c) * DW + 32 * ks + 8 * g);
  }
  for (int idx = tid; !BOUND_ONLY && idx < 2 * (TLD - DW - 1) * LDJ; idx += 512) {
    const int bb = idx / ((TLD - DW - 1) * LDJ), rem = idx - bb * (TLD - DW - 1) * LDJ;
    sm.vt[bb][DW + 1 + rem / LDJ][rem % LDJ] = 0;
  }
  f32x4 T[2][NVW];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int vt = 0; vt < NVW; ++vt) T[mt][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
  float dk = -INFINITY;

  // staging: two row pieces (rows tid/16 and tid/16 + 32) and two value pieces (token tid%64, pieces tid/64 and + 8)
  u32x4 kr[2], vr[2];
  float rkr[2] = {0.f, 0.f};
  auto load = [&](int row0) {
    const int nv = max(0, min(TC, row_end - row0));
    const __amdgpu_buffer_rsrc_t rk_ = chunk_rsrc(Kb + (long long)row0 * a.K.sl, 2 * (int)a.K.sl, nv, 2 * DW);
    const __amdgpu_buffer_rsrc_t rv_ = chunk_rsrc(Vb + (long long)row0 * a.V.sl, 2 * (int)a.V.sl, nv, 2 * DW);
    const __amdgpu_buffer_rsrc_t rr_ = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.rk + (size_t)bh * a.L + row0), 0,
                                                                         isoC ? 0 : 4 * nv, 0x00020000);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int row = (tid >> 4) + 32 * i;
      kr[i] = __builtin_amdgcn_raw_buffer_load_b128(rk_, 2 * (row * (int)a.K.sl + (tid & 15) * 8), 0, 0);
      rkr[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rr_, 4 * row, 0, 0));
      if (!BOUND_ONLY) vr[i] = __builtin_amdgcn_raw_buffer_load_b128(rv_, 2 * ((tid & 63) * (int)a.V.sl + ((tid >> 6) + 8 * i) * 8), 0, 0);
    }
  };
  auto store = [&](int buf, int row0) {
    const int nv = max(0, min(TC, row_end - row0));
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int row = (tid >> 4) + 32 * i;
      const float n2 = store_row_piece_w(kr[i], sm.k[buf], row, tid & 15);
      const float rt = isoC ? -0.5f * kLog2e * a.scale * a.scale * n2 : rkr[i];
      // rows past the end get -inf: their features are exactly zero whatever the key shift is
      sm.kadd[buf][row] = row < nv ? rt : -INFINITY;
      sm.kbnd[buf][row] = row < nv ? row_shift(n2, wmax) + rt : -INFINITY;
      if (!BOUND_ONLY) store_val_piece(vr[i], sm.vt[buf], tid & 63, (tid >> 6) + 8 * i);
    }
    if (!BOUND_ONLY && tid < 32) {
      const int t0 = 2 * tid;
      *(uint32_t*)(&sm.vt[buf][DW][t0]) = (t0 < nv ? 0x3f80u : 0u) | (t0 + 1 < nv ? 0x3f80u << 16 : 0u);
    }
  };
  load(row_beg);
  store(0, row_beg);
  __syncthreads();

  int buf = 0;
  for (int row0 = row_beg; row0 < row_end; row0 += TC, buf ^= 1) {
    const bool more = row0 + TC < row_end;
    if (more) load(row0 + TC);
    {
      const f32x4 b4 = *(const f32x4*)(&sm.kbnd[buf][4 * c]);
      const float dnew = max16(fmaxf(fmaxf(b4[0], b4[1]), fmaxf(b4[2], b4[3])));
      if (BOUND_ONLY) dk = fmaxf(dk, dnew);
      else if (dnew > dk) {
        const float f = fast_exp2(dk - dnew);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int vt = 0; vt < NVW; ++vt) T[mt][vt] *= f;
        dk = dnew;
      }
    }
#pragma unroll
    for (int jp = 0; !BOUND_ONLY && jp < 2; ++jp) {
      bf16x8 st[2];
      {
        bf16x8 x[2][KSW];
        f32x4 addv[2];
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
          const int jt = 2 * jp + jj;
#pragma unroll
          for (int ks = 0; ks < KSW; ++ks) x[jj][ks] = *(const bf16x8*)(&sm.k[buf][16 * jt + c][32 * ks + 8 * g]);
          addv[jj] = *(const f32x4*)(&sm.kadd[buf][16 * jt + 4 * g]) - dk;
        }
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
          f32x4 acc[2];
#pragma unroll
          for (int jj = 0; jj < 2; ++jj) {
            acc[jj] = mfma(x[jj][0], wk[mt][0], addv[jj]);
#pragma unroll
            for (int ks = 1; ks < KSW; ++ks) acc[jj] = mfma(x[jj][ks], wk[mt][ks], acc[jj]);
          }
          st[mt] = pack8(exp2v(acc[0]), exp2v(acc[1]));
        }
      }
#pragma unroll
      for (int vt = 0; vt < NVW; ++vt) {
        const bf16x8 vop = load_vop_l(sm.vt[buf], jp, vt, lane);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) T[mt][vt] = mfma(st[mt], vop, T[mt][vt]);
      }
    }
    if (more) store(buf ^ 1, row0 + TC);
    __syncthreads();
  }
  if (BOUND_ONLY) {
    if (tid == 0) {
      a.cstar[bh] = dk;
      a.cstar[gridDim.y + bh] = dk;        // the key shift of the sequence's only slot
      if (bh == 0 && a.flushed != nullptr) *a.flushed = 0u;
    }
    return;
  }
  float* out = a.Tpart + (((size_t)bh * 2 + fh) * a.nslot + slot) * 256 * TLD;
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int vt = 0; vt < NVW; ++vt)
#pragma unroll
      for (int r = 0; r < 4; ++r) out[(size_t)(32 * w + 16 * mt + 4 * g + r) * TLD + 16 * vt + c] = T[mt][vt][r];
  if (tid == 0 && fh == 0) a.cpart[(size_t)bh * a.nslot + slot] = dk;
}

// Exclusive prefix over the slots of one (b,h, feature half) on running shifts: the prefix of slot s is scaled by
// the largest shift of the slots up to and including s, which is also the key shift of the slot's walk (written to
// cstar[B*H + bh * nslot + s]; cstar[bh] = the sequence's largest).  Keys late in the sequence thus cannot push the
// states that earlier rows need out of the fp32 range.  Four consecutive numbers per thread.
// grid (ceil(256*144/1024), B*H*2).
// `total` (non-causal calls): no prefixes; the sum of all slots, on the largest shift, goes to slot 0.
__global__ void k_wide_reduce(float* Tpart, const float* cpart, float* cstar, int nslot, int total, unsigned* flushed) {
  const int bh2 = blockIdx.y, bh = bh2 >> 1;
  // the walk of the call counts into this word: it starts every call at zero
  if (flushed != nullptr && (blockIdx.x | blockIdx.y | threadIdx.x) == 0) *flushed = 0u;
  constexpr size_t per = (size_t)256 * TLD;
  const size_t e = 4 * ((size_t)blockIdx.x * blockDim.x + threadIdx.x);
  const bool writer = e == 0 && (bh2 & 1) == 0;
  float* cpre = cstar + (gridDim.y >> 1) + (size_t)bh * nslot;
  float* p = Tpart + (size_t)bh2 * nslot * per + e;
  f32x4 run = {0.f, 0.f, 0.f, 0.f};
  float cr = -INFINITY;
  // eight slots at a time: a batch's loads are all requested before the first number is used (with one or two
  // sequences the kernel is a chain of memory latencies otherwise), and a slot is overwritten only after its batch
  // was read
  constexpr int NB = 8;
  for (int s0 = 0; s0 < nslot; s0 += NB) {
    f32x4 v[NB];
    float cb[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int s = s0 + i;
      v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      cb[i] = -INFINITY;
      if (s < nslot) {
        cb[i] = cpart[(size_t)bh * nslot + s];
        if (e < per) v[i] = *(const f32x4*)(p + (size_t)s * per);
      }
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int s = s0 + i;
      if (s < nslot) {
        const float c = cb[i];
        if (c > cr) { run *= fast_exp2(cr - c); cr = c; }
        if (writer) cpre[s] = cr;
        if (e < per) {
          if (!total) *(f32x4*)(p + (size_t)s * per) = run;
          run += v[i] * fast_exp2(c - cr);
        }
      }
    }
  }
  if (total && e < per) *(f32x4*)p = run;
  if (writer) cstar[bh] = cr;
}

// ---------------------------------------------------------------------------------------------------
// The causal walk of one slot for one column half and the launch's feature half.  grid (nslot, B*H, 2), block 512: four producer
// and four consumer waves; the consumer side is the one of the 64 / 256 kernels (fast_pc.h), the producer side has
// projections of depth 128 and stages rows of 128 numbers.  LDS lifetimes as in kernels_bf16_bwd_pc.hip (walks).
// ---------------------------------------------------------------------------------------------------
struct SmemWWalk {
  __attribute__((aligned(16))) uint16_t xoth[TC][LDRW];       // key rows
  __attribute__((aligned(16))) uint16_t xown[TC][LDRW];       // query rows
  __attribute__((aligned(16))) uint16_t uothT[DVP][LDJ];      // value columns of this half, transposed (+ ones row)
  __attribute__((aligned(16))) float add_oth[TC];
  __attribute__((aligned(16))) float add_own[TC];
  __attribute__((aligned(16))) uint16_t feat[2][4][4][64][8];
  __attribute__((aligned(16))) uint16_t xch[4][4][16][LDXB];
};

struct WCtx {
  const uint16_t *Qb, *Kb, *Vb;
  int bh, pg, fh, ch, row_beg, row_end, nchunk;
  bool isoC, sameB;
  float cs;
};
__device__ __forceinline__ int wrow(const WCtx& cx, int ci) { return cx.row_beg + min(ci, cx.nchunk) * TC; }
__device__ __forceinline__ int wrows(const WCtx& cx, int ci) { return ci < cx.nchunk ? min(TC, cx.row_end - wrow(cx, ci)) : 0; }

struct WStage { u32x4 xo[4], xw[4], v[2]; float rk[4]; };
struct XOpW { bf16x8 b[KSW]; };

// CAUSAL = false: the query pass of a non-causal call: no key rows, no values, no key feature tiles (steps 0 and 1
// only stage and finish); the projection slice is the query side's throughout.
template <bool CAUSAL>
__device__ __forceinline__ void wide_producer(const WideArgs& a, SmemWWalk& sm, const WCtx& cx, int j) {
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 4, c = lane & 15;
  const int b = cx.bh / a.H, h = cx.bh % a.H;
  const float wmaxq = max512(a.wnorm + ((size_t)cx.pg * 2) * MW), amax = max512(a.bias + ((size_t)cx.pg * 2) * MW);
  const int f0 = 256 * cx.fh + 64 * j;

  // projection slice of the side in work as A operands: row = feature f0 + 16 mt + c, k = 32 ks + 8g + e.  One set
  // of registers: the key side's slice for steps 0 and 1, the query side's for steps 2 and 3, each reloaded (from L2)
  // right after the other's last use, a step and a barrier before its first.
  bf16x8 wx[4][KSW];
  auto load_w = [&](int side) {
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int ks = 0; ks < KSW; ++ks)
        wx[mt][ks] = *(const bf16x8*)(a.Wbf + (((size_t)cx.pg * 2 + side) * MW + f0 + 16 * mt + c) * DW + 32 * ks + 8 * g);
  };
  load_w(CAUSAL ? 1 : 0);
  f32x4 qb[4];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int r = 0; r < 4; ++r) qb[mt][r] = 2.f * (a.bias[((size_t)cx.pg * 2) * MW + f0 + 16 * mt + 4 * g + r] - amax);

  WStage stg;
  auto load_x = [&](u32x4 (&p)[4], const uint16_t* base, long long sl, int ci, bool with_rk) {
    const int r0 = wrow(cx, ci), nv = wrows(cx, ci);
    const __amdgpu_buffer_rsrc_t rs = chunk_rsrc(base + (long long)r0 * sl, 2 * (int)sl, nv, 2 * DW);
    const __amdgpu_buffer_rsrc_t rr = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.rk + (size_t)cx.bh * a.L + r0), 0,
                                                                        (with_rk && !cx.isoC) ? 4 * nv : 0, 0x00020000);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = (tid >> 4) + 16 * i;
      p[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, 2 * (row * (int)sl + (tid & 15) * 8), 0, 0);
      if (with_rk) stg.rk[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rr, 4 * row, 0, 0));
    }
  };
  auto store_x = [&](const u32x4 (&p)[4], bool key_side, uint16_t (*tile)[LDRW], float* add, int nv) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = (tid >> 4) + 16 * i;
      const float n2 = store_row_piece_w(p[i], tile, row, tid & 15);
      float t;
      if (key_side) t = (cx.isoC ? -0.5f * kLog2e * a.scale * a.scale * n2 : stg.rk[i]) - cx.cs;
      else t = -row_shift(n2, wmaxq);
      add[row] = row < nv ? t : -INFINITY;
    }
  };
  auto load_v = [&](int ci) {
    const int r0 = wrow(cx, ci), nv = wrows(cx, ci);
    const __amdgpu_buffer_rsrc_t rv = chunk_rsrc(cx.Vb + (long long)r0 * a.V.sl, 2 * (int)a.V.sl, nv, 2 * DW);
#pragma unroll
    for (int i = 0; i < 2; ++i)
      stg.v[i] = __builtin_amdgcn_raw_buffer_load_b128(rv, 2 * ((tid & 63) * (int)a.V.sl + 64 * cx.ch + ((tid >> 6) + 4 * i) * 8), 0, 0);
  };
  auto store_v = [&](int nv) {
#pragma unroll
    for (int i = 0; i < 2; ++i) store_val_piece(stg.v[i], sm.uothT, tid & 63, (tid >> 6) + 4 * i);
    if (tid < 32) {
      const int t0 = 2 * tid;
      const uint32_t one = 0x3f80u;                            // the ones row: both column halves carry the normaliser
      *(uint32_t*)(&sm.uothT[D][t0]) = (t0 < nv ? one : 0u) | (t0 + 1 < nv ? one << 16 : 0u);
    }
  };
  auto load_xop = [&](XOpW& x, const uint16_t (*tile)[LDRW], int jt) {
#pragma unroll
    for (int ks = 0; ks < KSW; ++ks) x.b[ks] = *(const bf16x8*)(&tile[16 * jt + c][32 * ks + 8 * g]);
  };

#pragma unroll
  for (int i = 0; i < 4; ++i) stg.rk[i] = 0.f;
  if (CAUSAL) {
    load_x(stg.xo, cx.Kb, a.K.sl, 0, true);
    load_v(0);
    store_x(stg.xo, true, sm.xoth, sm.add_oth, wrows(cx, 0));
    store_v(wrows(cx, 0));
    load_x(stg.xo, cx.Kb, a.K.sl, 1, true);
    load_v(1);
  }
  load_x(stg.xw, cx.Qb, a.Q.sl, 0, false);
  __syncthreads();                 // barrier 0

  // rows of token tile j of a finished chunk.  Feature half 0: unnormalised sums over this workgroup's 256 features
  // and their partial normaliser, to the partial buffer.  Feature half 1: the other half's partial rows are added,
  // the row is divided by the sum of the two partial normalisers and stored.
  auto finish = [&](int ci_done) {
    f32x4 fsum[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) fsum[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    finish_tiles(fsum, sm, j, 0, lane);
    finish_tiles(fsum, sm, j, 2, lane);
    float den = finish_col64(sm, j, lane);
    const int r0 = wrow(cx, ci_done), nv = wrows(cx, ci_done);
    float* yp = a.Ypart + ((size_t)cx.bh * a.Lq + r0) * YLD;
    const __amdgpu_buffer_rsrc_t ry = chunk_rsrc(yp, 4 * YLD, nv, 4 * YLD);
    const int off = 4 * ((16 * j + c) * YLD + 64 * cx.ch + 4 * g), doff = 4 * ((16 * j + c) * YLD + DW + cx.ch);
    if (cx.fh == 0) {
#pragma unroll
      for (int vt = 0; vt < 4; ++vt) __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, fsum[vt]), ry, off + 64 * vt, 0, 0);
      if (g == 0) __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, den), ry, doff, 0, 0);
    } else {
#pragma unroll
      for (int vt = 0; vt < 4; ++vt) fsum[vt] += __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(ry, off + 64 * vt, 0, 0));
      den += __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ry, doff, 0, 0));
      const float inv = den > 0.f ? __builtin_amdgcn_rcpf(den) : 0.f;
      // a row is finished once per column half: the first half counts it
      if (a.flushed != nullptr && cx.ch == 0 && __builtin_expect(!(den > 0.f) && g == 0 && 16 * j + c < nv, 0))
        atomicAdd(a.flushed, 1u);
#pragma unroll
      for (int vt = 0; vt < 4; ++vt) fsum[vt] *= inv;
      const int esz = a.Y.dtype == 1 ? 2 : 4;
      const char* gp = (const char*)a.Y.ptr + (b * a.Y.sb + h * a.Y.sh + (long long)r0 * a.Y.sl + 64 * cx.ch) * esz;
      finish_store(fsum, a.Y, gp, nv, j, lane);
    }
  };

  for (int ci = 0; ci < cx.nchunk; ++ci) {
    const int nv = wrows(cx, ci);
#pragma unroll
    for (int S = 0; S < 4; ++S) {
      if (CAUSAL || S >= 2) {
      XOpW xs[2];                  // both tiles of the step are requested before the first is used
#pragma unroll
      for (int u = 0; u < 2; ++u) load_xop(xs[u], S < 2 ? sm.xoth : sm.xown, 2 * (S & 1) + u);
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const XOpW& x = xs[u];
        const float add = S < 2 ? sm.add_oth[16 * (2 * S + u) + c] : sm.add_own[16 * (2 * (S - 2) + u) + c];
        const f32x4 add4 = {add, add, add, add};
        f32x4 acc[4];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
          acc[mt] = mfma(wx[mt][0], x.b[0], S < 2 ? add4 : qb[mt]);
#pragma unroll
          for (int ks = 1; ks < KSW; ++ks) acc[mt] = mfma(wx[mt][ks], x.b[ks], acc[mt]);
        }
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
          const bf16x8 img = S < 2 ? pack8(exp2v(acc[2 * blk]), exp2v(acc[2 * blk + 1]))
                                   : pack8(exp2v(acc[2 * blk] + add), exp2v(acc[2 * blk + 1] + add));
          *(bf16x8*)(&sm.feat[S & 1][2 * u + blk][j][lane][0]) = img;
        }
      }
      }
      if (CAUSAL && !cx.sameB) {   // (with B1 = B2 the two slices are the same numbers and stay where they are)
        if (S == 1) load_w(0);
        if (S == 3) load_w(1);
      }

      if (S == 0) {
        store_x(stg.xw, false, sm.xown, sm.add_own, nv);
        load_x(stg.xw, cx.Qb, a.Q.sl, ci + 1, false);
      } else if (S == 1) {
        if (ci > 0) finish(ci - 1);
      } else if (S == 2) {
        if (CAUSAL) {
          store_x(stg.xo, true, sm.xoth, sm.add_oth, wrows(cx, ci + 1));
          load_x(stg.xo, cx.Kb, a.K.sl, ci + 2, true);
        }
      } else if (CAUSAL) {
        store_v(wrows(cx, ci + 1));
        load_v(ci + 2);
      }
      __syncthreads();
    }
  }
  __syncthreads();                 // the consumers' last step
  if (cx.nchunk > 0) finish(cx.nchunk - 1);
}

template <bool CAUSAL>
__global__ void __launch_bounds__(NT8) k_wide_walk(WideArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  SmemWWalk& sm = *reinterpret_cast<SmemWWalk*>(smem_raw);
  const int slot = blockIdx.x, bh = blockIdx.y, b = bh / a.H, h = bh % a.H;
  const float* th = a.theta + (size_t)group_of(a.groups, b, h, a.H) * (FS_THETA_HEADER_ + (size_t)DW + 4 * (size_t)DW * DW);
  WCtx cx;
  cx.isoC = ((int)th[2]) & 1;
  cx.sameB = (((int)th[2]) & 2) != 0;
  cx.bh = bh;
  cx.fh = a.fh;
  cx.ch = blockIdx.z;
  cx.pg = group_of(a.pgroups, b, h, a.H);
  cx.cs = CAUSAL ? a.cstar[gridDim.y + (size_t)bh * a.nslot + slot] : 0.f;     // the slot's key shift (k_wide_reduce)
  cx.Qb = (const uint16_t*)a.Q.ptr + b * a.Q.sb + h * a.Q.sh;
  cx.Kb = (const uint16_t*)a.K.ptr + b * a.K.sb + h * a.K.sh;
  cx.Vb = (const uint16_t*)a.V.ptr + b * a.V.sb + h * a.V.sh;
  cx.row_beg = min(a.Lq, slot * a.rows_per_slot_q);
  cx.row_end = min(a.Lq, cx.row_beg + a.rows_per_slot_q);
  cx.nchunk = (cx.row_end - cx.row_beg + TC - 1) / TC;
  for (int idx = threadIdx.x; idx < DVP * LDJ / 2; idx += NT8) ((uint32_t*)&sm.uothT[0][0])[idx] = 0u;
  __syncthreads();
  const int w = threadIdx.x >> 6;
  if (w < 4) {
    wide_producer<CAUSAL>(a, sm, cx, w);
  } else {
    const int j = w - 4, lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
    // state slice: 64 features of this half x the 64 columns of this column half and the normaliser column (tile 4)
    f32x4 T[4][NVT];
    // (non-causal: the sum over all slots, which the reduction left in slot 0)
    const float* Tg = a.zero_state != nullptr ? a.zero_state
                                              : a.Tpart + (((size_t)bh * 2 + cx.fh) * a.nslot + (CAUSAL ? slot : 0)) * 256 * TLD;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int col = vt < 4 ? 64 * cx.ch + 16 * vt + c : DW + c;
          T[mt][vt][r] = Tg[(size_t)(64 * j + 16 * mt + 4 * g + r) * TLD + col];
        }
    walk_consume<CAUSAL ? 0 : 2>(sm, T, cx.nchunk, j);
  }
}

// ---------------------------------------------------------------------------------------------------
// Statistics scan of the fits for bf16 rows of 128 numbers (Section 4: mu4, mu5, M1, M2 are means of x, y, x x^T,
// y y^T): per (b,h), tensor and row chunk, sum x and sum x x^T on bf16 MFMA tiles.  The rows of a 64-token tile stay
// row-major in LDS; both operands of X^T X (lane <-> number, contraction index <-> tokens) are transposing reads,
// and the column sums come from a constant operand of ones.  Rows of 72 dwords: the four rows that a transposing
// read touches per group of 16 lanes start 8 banks apart, the next group's 32 banks further.  Wave w owns the Gram
// tiles (2w .. 2w+1, 0 .. 7) and the column sums of those two blocks.  Rows past the end are staged as zeros.
// Output layout as the general kernel's: part[which][bh][chunk][d*d + d], with qk_scale applied (squared on the
// Gram part).  grid (nchunks, B*H, 2), block 256.
// ---------------------------------------------------------------------------------------------------
constexpr int LDSW = DW + 16;
struct SmemWStats { __attribute__((aligned(16))) uint16_t x[2][TC][LDSW]; };

// lane <-> number 16 ct + c, contraction index <-> tokens {32 jp + 4g + r, 32 jp + 16 + 4g + r}
__device__ __forceinline__ bf16x8 load_cop_tr(const uint16_t (*x)[LDSW], int jp, int ct, int lane) {
  const int g = lane >> 4, c = lane & 15;
  const uint16_t* p = &x[32 * jp + 4 * g + (c >> 2)][16 * ct + 4 * (c & 3)];
  return join8(lds_read_tr(p), lds_read_tr(p + 16 * LDSW));
}

__global__ void __launch_bounds__(NT) k_stats_wide(TensorDev X, TensorDev Yt, int Lx, int Ly, int H, float scale,
                                                   int rows_per_chunk, int nchunks, float* part) {
  __shared__ SmemWStats sm;
  const int which = blockIdx.z, bh = blockIdx.y, b = bh / H, h = bh % H, chunk = blockIdx.x;
  const TensorDev& T = which ? Yt : X;
  const int L = which ? Ly : Lx;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, g = lane >> 4, c = lane & 15;
  const uint16_t* base = (const uint16_t*)T.ptr + b * T.sb + h * T.sh;
  const int row_beg = chunk * rows_per_chunk, row_end = min(L, row_beg + rows_per_chunk);
  f32x4 acc[2][8], sums[2];
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    sums[a] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int bt = 0; bt < 8; ++bt) acc[a][bt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  const u32x4 ones_bits = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
  const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_bits);
  // sixteen consecutive threads fetch one row (256 bytes); four rows of the tile per thread
  u32x4 r[4];
  auto fetch = [&](int row0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = row0 + (tid >> 4) + 16 * i;
      r[i] = u32x4{0u, 0u, 0u, 0u};
      if (row < row_end) r[i] = *(const u32x4*)(base + (long long)row * T.sl + (tid & 15) * 8);
    }
  };
  auto stage = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) *(u32x4*)(&sm.x[buf][(tid >> 4) + 16 * i][(tid & 15) * 8]) = r[i];
  };
  fetch(row_beg);
  stage(0);
  __syncthreads();
  int buf = 0;
  for (int row0 = row_beg; row0 < row_end; row0 += TC, buf ^= 1) {
    const bool more = row0 + TC < row_end;
    if (more) fetch(row0 + TC);
#pragma unroll
    for (int jp = 0; jp < 2; ++jp) {
      bf16x8 cop[8];
#pragma unroll
      for (int bt = 0; bt < 8; ++bt) cop[bt] = load_cop_tr(sm.x[buf], jp, bt, lane);
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        const bf16x8 mine = w == 0 ? cop[a] : w == 1 ? cop[2 + a] : w == 2 ? cop[4 + a] : cop[6 + a];
#pragma unroll
        for (int bt = 0; bt < 8; ++bt) acc[a][bt] = mfma(mine, cop[bt], acc[a][bt]);
        sums[a] = mfma(ones, mine, sums[a]);
      }
    }
    if (more) stage(buf ^ 1);
    __syncthreads();
  }
  float* out = part + (((size_t)which * gridDim.y + bh) * nchunks + chunk) * ((size_t)DW * DW + DW);
  const float s2 = scale * scale;
#pragma unroll
  for (int a = 0; a < 2; ++a) {
#pragma unroll
    for (int bt = 0; bt < 8; ++bt)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) out[(size_t)(16 * (2 * w + a) + 4 * g + rr) * DW + 16 * bt + c] = s2 * acc[a][bt][rr];
    if (g == 0) out[(size_t)DW * DW + 16 * (2 * w + a) + c] = scale * sums[a][0];
  }
}

}  // namespace wide

using namespace wide;

bool stats_wide_supported(const TensorDev& X, const TensorDev& Y, int d) {
  return X.dtype == 1 && Y.dtype == 1 && d == DW;
}

int launch_stats_wide(const TensorDev& X, const TensorDev& Y, int BH, int H, int Lx, int Ly, float scale,
                      int rows_per_chunk, int nchunks, float* part, hipStream_t st) {
  hipLaunchKernelGGL(k_stats_wide, dim3(nchunks, BH, 2), dim3(NT), 0, st, X, Y, Lx, Ly, H, scale, rows_per_chunk, nchunks,
                     part);
  if (hipGetLastError() != hipSuccess) return 5;
  return 0;
}

bool wide_supported(int dtype, int d, int dv, int M_, int causal) {
  return dtype == 1 && d == DW && dv == DW && M_ == MW && (causal == 0 || causal == 1);
}

size_t wide_lds_bytes() { return std::max(sizeof(SmemWState), sizeof(SmemWWalk)); }

void wide_plan(int BH, int L, int* nslot, int* rows_per_slot) {
  // two workgroups per (sequence, slot) and launch of the walk: about 256 of them, whole chunks each
  const int want = std::max(1, std::min((128 + BH - 1) / BH, (L + TC - 1) / TC));
  *rows_per_slot = (((L + want - 1) / want) + TC - 1) / TC * TC;
  *nslot = (L + *rows_per_slot - 1) / *rows_per_slot;
}

#define FS_LAUNCH_CHECK() do { if (hipGetLastError() != hipSuccess) return 5; } while (0)

int launch_wide_prepare(const float* theta, int groups, const float* Omega, int omega_groups, int pgroups, int B, int H,
                        float scale, uint16_t* Wbf, float* bias, float* wnorm, int* dense_flag, hipStream_t st) {
  WideArgs a = {};
  a.theta = theta; a.Omega = Omega; a.Wbf = Wbf; a.bias = bias; a.wnorm = wnorm;
  a.groups = groups; a.omega_groups = omega_groups; a.pgroups = pgroups; a.B = B; a.H = H; a.scale = scale;
  hipLaunchKernelGGL(k_wide_pre, dim3((MW / (4 * PREF)) * 2 * pgroups), dim3(256), 0, st, a, dense_flag);
  FS_LAUNCH_CHECK();
  return 0;
}

int launch_wide_attention(const WideLaunch& f, hipStream_t st, hipEvent_t ev_begin, hipEvent_t ev_end) {
  WideArgs a;
  a.Q = f.Q; a.K = f.K; a.V = f.V; a.Y = f.Y;
  a.theta = f.theta; a.Omega = f.Omega;
  a.Wbf = f.Wbf; a.bias = f.bias; a.wnorm = f.wnorm; a.rk = f.rk; a.Tpart = f.Tpart; a.cpart = f.cpart; a.cstar = f.cstar;
  a.Ypart = f.Ypart;
  a.groups = f.groups; a.omega_groups = f.omega_groups; a.pgroups = f.pgroups; a.B = f.B; a.H = f.H; a.L = f.L;
  a.nslot = f.nslot; a.rows_per_slot = f.rows_per_slot; a.scale = f.scale;
  a.Lq = f.causal ? f.L : f.Lq;
  a.rows_per_slot_q = f.causal ? f.rows_per_slot : f.rows_per_slot_q;
  const int nslot_q = f.causal ? f.nslot : f.nslot_q;
  a.flushed = f.flushed;
  a.zero_state = nullptr;
  const int BH = f.B * f.H;
  const void* walk = f.causal ? (const void*)k_wide_walk<true> : (const void*)k_wide_walk<false>;
  const bool one_slot = f.causal && f.nslot == 1;
  const void* state = one_slot ? (const void*)k_wide_state<true> : (const void*)k_wide_state<false>;
  if (hipFuncSetAttribute(state, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(SmemWState)) != hipSuccess ||
      hipFuncSetAttribute(walk, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(SmemWWalk)) != hipSuccess) {
    (void)hipGetLastError();
    return 2;
  }
  if (f.pre_mode == 0) {
    hipLaunchKernelGGL(k_wide_pre, dim3((MW / (4 * PREF)) * 2 * f.pgroups), dim3(256), 0, st, a, (int*)nullptr);
    FS_LAUNCH_CHECK();
  }
  // the key row terms of parameter sets with a dense C2 (the host knows that there are none only in mode 2)
  if (f.pre_mode != 2)
    if (int rc = launch_key_row_terms(f.theta, f.groups, f.K, f.B, f.H, f.L, DW, f.scale, f.rk, st)) return rc;
  if (one_slot) {
    // one slot per sequence (128 sequences or more): the walks start from nothing, so no state is computed or
    // scanned; the first state of the (unused) buffer becomes the block of zeros that every workgroup reads
    if (int rc = launch_fill_u32((uint32_t*)f.Tpart, 0u, (size_t)256 * TLD, st)) return rc;
    a.zero_state = f.Tpart;
    hipLaunchKernelGGL(k_wide_state<true>, dim3(1, BH, 1), dim3(512), sizeof(SmemWState), st, a);
    FS_LAUNCH_CHECK();
  } else {
    hipLaunchKernelGGL(k_wide_state<false>, dim3(f.nslot, BH, 2), dim3(512), sizeof(SmemWState), st, a);
    FS_LAUNCH_CHECK();
    if (!f.causal && f.nslot == 1) {
      // the sum over one slot is that slot (its shift cancels in the normalised rows): only the counter is reset
      if (f.flushed != nullptr)
        if (int rc = launch_fill_u32((uint32_t*)f.flushed, 0u, 1, st)) return rc;
    } else {
      hipLaunchKernelGGL(k_wide_reduce, dim3((256 * TLD / 4 + 255) / 256, BH * 2), dim3(256), 0, st, f.Tpart, f.cpart, f.cstar, f.nslot,
                         f.causal ? 0 : 1, f.flushed);
      FS_LAUNCH_CHECK();
    }
  }
  // the optional events are attached to the dispatches of the two walks: begin of the first, end of the second
  for (int fh = 0; fh < 2; ++fh) {
    a.fh = fh;
    hipEvent_t e0 = fh == 0 ? ev_begin : nullptr, e1 = fh == 1 ? ev_end : nullptr;
    if (f.causal) {
      if (e0 || e1) hipExtLaunchKernelGGL(k_wide_walk<true>, dim3(nslot_q, BH, 2), dim3(NT8), sizeof(SmemWWalk), st, e0, e1, 0, a);
      else hipLaunchKernelGGL(k_wide_walk<true>, dim3(nslot_q, BH, 2), dim3(NT8), sizeof(SmemWWalk), st, a);
    } else {
      if (e0 || e1) hipExtLaunchKernelGGL(k_wide_walk<false>, dim3(nslot_q, BH, 2), dim3(NT8), sizeof(SmemWWalk), st, e0, e1, 0, a);
      else hipLaunchKernelGGL(k_wide_walk<false>, dim3(nslot_q, BH, 2), dim3(NT8), sizeof(SmemWWalk), st, a);
    }
    FS_LAUNCH_CHECK();
  }
  return 0;
}

}  // namespace fs
