// Backward pass of causal attention on the bf16 path (d = dv = 64, M = 256); see kernels_bf16_bwd.hip for the
// non-causal variant and the notation.  The kernels of this file need more than 256 registers per lane (state,
// both projection slices, the transposed projection and a chunk's feature tiles all live in registers), so one
// workgroup of four waves runs per CU and MFMA results may live in accumulation registers.
#include "fast_bwd.h"

namespace fs {

using namespace fast;

namespace bwd {

// ===============================================================================================================
// Causal variant.  With T_i the prefix state (keys j <= i) and R_j the suffix sum  sum_{i >= j} P_i^T G1_i, per chunk
// c of 64 tokens (A = tril(G1_c V1_c^T), B = tril(P_c S_c^T), both 64 x 64 with the diagonal):
//   dP_c  = G1_c T_{c-1}^T + A S_c               dV1_c = S_c R_{c+1} + B^T G1_c
//   dS_c  = V1_c R_{c+1}^T + A^T P_c
// Every kernel walks one slot (a run of whole chunks) of one sequence with the running state (T forwards, R
// backwards) in registers; the key features use ONE shift per sequence (the largest bound over all its tokens) so
// that the states of different slots, G1 and the gradients all live on one scale.
//   k_bwd_cfwd      forward walk: Yhat, normaliser, Y, G1 rows                 (T from the exclusive prefix per slot)
//   k_bwd_rstate    (kernels_bf16_bwd.hip) per-slot sums of P^T G1;  k_bwd_suffix  their exclusive suffix per slot
//   k_bwd_cdv       backward walk: dV
//   k_bwd_cgrad_pc  (kernels_bf16_bwd_cgrad.hip) dQ (forward walk) and dK (backward walk)
// ===============================================================================================================
struct SmemCB {
  __attribute__((aligned(16))) uint16_t q[TC][LDR];       // query rows
  __attribute__((aligned(16))) uint16_t k[TC][LDR];       // key rows
  __attribute__((aligned(16))) uint16_t vt[DVP][LDJ];     // [V 1] transposed: [column][token]
  __attribute__((aligned(16))) uint16_t gt[DVP][LDJ];     // G1 transposed
  float qadd[TC];                                         // - row_shift of the query rows
  float kadd[TC];                                         // row term - sequence shift of the key rows (-inf past the end)
  __attribute__((aligned(16))) uint16_t xch[NW][NW][16][LDXB];
};

// Everything a chunk needs in LDS, staged through registers one chunk ahead.
struct ChunkRegs {
  RowRegs q, k, vcol;
  RowRegs3 gcol;
};

template <bool WITH_G>
__device__ __forceinline__ void chunk_load(ChunkRegs& r, const BwdArgs& ba, const uint16_t* Qb, const uint16_t* Kb,
                                           const uint16_t* Vb, const uint16_t* Gb, int row0, int row_end) {
  const FastArgs& a = ba.f;
  load_rows_g(r.q, Qb, a.Q.sl, row0, row_end);
  load_rows_g(r.k, Kb, a.K.sl, row0, row_end);
  load_vals_g(r.vcol, Vb, a.V.sl, row0, row_end);
  if (WITH_G) load_g80_g(r.gcol, Gb, row0, row_end);
}

template <bool WITH_G>
__device__ __forceinline__ void chunk_store(const ChunkRegs& r, SmemCB& sm, const BwdArgs& ba, bool isoC, int bh, float cs,
                                            float wmax1, int row0, int row_end) {
  const FastArgs& a = ba.f;
  float n2[2];
  store_rows_s(r.q, sm.q, n2);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int q = threadIdx.x + NT * i;
    if ((q & 7) == 0) sm.qadd[q >> 3] = -row_shift(n2[i], wmax1);
  }
  store_rows_s(r.k, sm.k, n2);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int q = threadIdx.x + NT * i, row = q >> 3;
    if ((q & 7) == 0) {
      const bool valid = row0 + row < row_end;
      float rt = -0.5f * kLog2e * a.scale * a.scale * n2[i];
      if (!isoC) rt = valid ? a.rk[(size_t)bh * a.L + row0 + row] : 0.f;
      sm.kadd[row] = valid ? rt - cs : -INFINITY;
    }
  }
  store_vals_s(r.vcol, sm.vt, row0, row_end);
  if (WITH_G) store_g80_s(r.gcol, sm.gt);
}

// Zero padding the staging never writes: vt rows 65..
__device__ __forceinline__ void chunk_zero_pad(SmemCB& sm) {
  for (int idx = threadIdx.x; idx < (DVP - D - 1) * LDJ; idx += NT) sm.vt[D + 1 + idx / LDJ][idx % LDJ] = 0;
}

struct SlotCtx {
  const uint16_t *Qb, *Kb, *Vb, *Gb;
  int bh, b, h, pg, row_beg, row_end;
  bool isoC;
  float cs, wmax1, amax1;
};

__device__ __forceinline__ SlotCtx slot_ctx(const BwdArgs& ba, int slot, int bh) {
  const FastArgs& a = ba.f;
  SlotCtx x;
  x.bh = bh; x.b = bh / a.H; x.h = bh % a.H;
  x.pg = group_of(a.pgroups, x.b, x.h, a.H);
  const float* th = a.theta + (size_t)group_of(a.groups, x.b, x.h, a.H) * (FS_THETA_HEADER_ + (size_t)D + 4 * (size_t)D * D);
  x.isoC = ((int)th[2]) & 1;
  x.cs = a.cstar[bh];
  x.wmax1 = max256(a.wnorm + ((size_t)x.pg * 2) * M);
  x.amax1 = max256(a.bias + ((size_t)x.pg * 2) * M);
  x.Qb = (const uint16_t*)a.Q.ptr + x.b * a.Q.sb + x.h * a.Q.sh;
  x.Kb = (const uint16_t*)a.K.ptr + x.b * a.K.sb + x.h * a.K.sh;
  x.Vb = (const uint16_t*)a.V.ptr + x.b * a.V.sb + x.h * a.V.sh;
  x.Gb = ba.gh + (size_t)bh * ba.Lq * DVP;
  x.row_beg = slot * ba.rows_per_rslot;
  x.row_end = min(ba.Lq, x.row_beg + ba.rows_per_rslot);
  return x;
}

// Key feature tiles of a chunk: images s[jt][blk] and their transposes st[mt][jp] (lane <-> feature).
__device__ __forceinline__ void key_tiles(const WSlice& wk, const SmemCB& sm, const bf16x8 (&sel)[2], bf16x8 (&s)[4][2],
                                          bf16x8 (&st)[4][2]) {
  const int c = threadIdx.x & 15;
#pragma unroll
  for (int jp = 0; jp < 2; ++jp) {
    f32x4 tr[2][4];
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
      const int jt = 2 * jp + jj;
      feature_tile<false>(wk, nullptr, sm.k, jt, sm.kadd[16 * jt + c], s[jt]);
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) tr[jj][2 * mb + hh] = mfma(s[jt][mb], sel[hh], f32x4{0.f, 0.f, 0.f, 0.f});
    }
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) st[mt][jp] = pack8(tr[0][mt], tr[1][mt]);
  }
}

// Forward walk of one slot: G1 rows.  grid (nslot, B*H), block 256, one workgroup per CU.
__global__ void __launch_bounds__(NT) k_bwd_cfwd(BwdArgs ba) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  SmemCB& sm = *reinterpret_cast<SmemCB*>(smem_raw);
  const FastArgs& a = ba.f;
  const int slot = blockIdx.x, bh = blockIdx.y;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  const SlotCtx x = slot_ctx(ba, slot, bh);

  WSlice wq, wk;
  load_wslice(wq, a.Wbf + ((size_t)x.pg * 2) * M * D);
  load_wslice(wk, a.Wbf + ((size_t)x.pg * 2 + 1) * M * D);
  QBias qb;
  load_qbias(qb, a.bias + ((size_t)x.pg * 2) * M, x.amax1);
  bf16x8 sel[2];
  make_sel(sel);
  f32x4 T[4][NVT];
  {
    const float* Tg = a.Tpart + ((size_t)bh * a.nslot + slot) * M * DVP;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
        for (int r = 0; r < 4; ++r) T[mt][vt][r] = Tg[(size_t)(64 * w + 16 * mt + 4 * g + r) * DVP + 16 * vt + c];
  }
  chunk_zero_pad(sm);
  ChunkRegs cr;
  chunk_load<false>(cr, ba, x.Qb, x.Kb, x.Vb, x.Gb, x.row_beg, x.row_end);
  __syncthreads();
  chunk_store<false>(cr, sm, ba, x.isoC, bh, x.cs, x.wmax1, x.row_beg, x.row_end);
  __syncthreads();
  for (int row0 = x.row_beg; row0 < x.row_end; row0 += TC) {
    const bool more = row0 + TC < x.row_end;
    if (more) chunk_load<false>(cr, ba, x.Qb, x.Kb, x.Vb, x.Gb, row0 + TC, x.row_end);
    bf16x8 s[4][2], st[4][2];
    key_tiles(wk, sm, sel, s, st);
    bf16x8 tb[NVT][2];
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) tb[vt][mb] = pack8(T[2 * mb][vt], T[2 * mb + 1][vt]);
    bf16x8 vop[2][NVT];
#pragma unroll
    for (int jp = 0; jp < 2; ++jp)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) vop[jp][vt] = load_vop(sm.vt, jp, vt);
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      bf16x8 p[2];
      feature_tile<true>(wq, &qb, sm.q, it, sm.qadd[16 * it + c], p);
      f32x4 y[NVT];
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) {
        y[vt] = mfma(tb[vt][0], p[0], f32x4{0.f, 0.f, 0.f, 0.f});
        y[vt] = mfma(tb[vt][1], p[1], y[vt]);
      }
      // scores^T tiles (rows = keys 16 jt + 4g + r, column = query 16 it + c); keys of later tiles are masked out
#pragma unroll
      for (int jp = 0; jp < 2; ++jp) {
        if (2 * jp <= it) {
          f32x4 sc[2];
#pragma unroll
          for (int jj = 0; jj < 2; ++jj) {
            const int jt = 2 * jp + jj;
            sc[jj] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (jt <= it) {
              sc[jj] = mfma(s[jt][0], p[0], sc[jj]);
              sc[jj] = mfma(s[jt][1], p[1], sc[jj]);
              if (jt == it) {
#pragma unroll
                for (int r = 0; r < 4; ++r) sc[jj][r] = (4 * g + r <= c) ? sc[jj][r] : 0.f;
              }
            }
          }
          const bf16x8 sb = pack8(sc[0], sc[1]);
#pragma unroll
          for (int vt = 0; vt < NVT; ++vt) y[vt] = mfma(vop[jp][vt], sb, y[vt]);
        }
      }
      exchange_put_bf16(sm, y, it, w, lane);
    }
#pragma unroll
    for (int jp = 0; jp < 2; ++jp)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) T[mt][vt] = mfma(st[mt][jp], vop[jp][vt], T[mt][vt]);
    __syncthreads();
    {
      f32x4 fs[4] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
      finish_tiles(fs, sm, w, 0, lane);
      finish_tiles(fs, sm, w, 2, lane);
      const float inv = finish_norm(fs, sm, w, lane);
      const int token = row0 + 16 * w + c;
      const bool valid = token < x.row_end;
      const uint16_t* gy = (const uint16_t*)ba.dY.ptr + x.b * ba.dY.sb + x.h * ba.dY.sh + (long long)token * ba.dY.sl + 4 * g;
      f32x4 gv[4];
      float dot = 0.f;
#pragma unroll
      for (int vt = 0; vt < 4; ++vt) {
        bf16x4 t = {0, 0, 0, 0};
        if (valid) t = *(const bf16x4*)(gy + 16 * vt);
        gv[vt] = __builtin_convertvector(t, f32x4);
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
    }
    __syncthreads();
    if (more) chunk_store<false>(cr, sm, ba, x.isoC, bh, x.cs, x.wmax1, row0 + TC, x.row_end);
    __syncthreads();
  }
}

// Exclusive suffix over the slots of one (b,h), in place.  grid (ceil(M*DVP/256), B*H).
__global__ void k_bwd_suffix(float* Rpart, int nslot) {
  const size_t per = (size_t)M * DVP;
  const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= per) return;
  float* p = Rpart + (size_t)blockIdx.y * nslot * per + e;
  float run = 0.f;
  for (int s = nslot - 1; s >= 0; --s) {
    const float v = p[(size_t)s * per];
    p[(size_t)s * per] = run;
    run += v;
  }
}

// dV of the causal variant: backward walk of one slot with the suffix sum R in registers,
//   dV1_c = S_c R_{c+1} + tril(P_c S_c^T)^T G1_c,   R_c = R_{c+1} + P_c^T G1_c.
// grid (nslot, B*H), block 256, one workgroup per CU.
__global__ void __launch_bounds__(NT) k_bwd_cdv(BwdArgs ba) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  SmemCB& sm = *reinterpret_cast<SmemCB*>(smem_raw);
  const FastArgs& a = ba.f;
  const int slot = blockIdx.x, bh = blockIdx.y;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  const SlotCtx x = slot_ctx(ba, slot, bh);

  WSlice wq, wk;
  load_wslice(wq, a.Wbf + ((size_t)x.pg * 2) * M * D);
  load_wslice(wk, a.Wbf + ((size_t)x.pg * 2 + 1) * M * D);
  QBias qb;
  load_qbias(qb, a.bias + ((size_t)x.pg * 2) * M, x.amax1);
  bf16x8 sel[2];
  make_sel(sel);
  f32x4 T[4][NVT];     // suffix of P^T G1
  {
    const float* Tg = ba.Rpart + ((size_t)bh * a.nslot + slot) * M * DVP;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
        for (int r = 0; r < 4; ++r) T[mt][vt][r] = Tg[(size_t)(64 * w + 16 * mt + 4 * g + r) * DVP + 16 * vt + c];
  }
  chunk_zero_pad(sm);
  const int nchunk = (x.row_end - x.row_beg + TC - 1) / TC;
  auto chunk_row = [&](int i) { return x.row_beg + (nchunk - 1 - i) * TC; };
  ChunkRegs cr;
  if (nchunk > 0) chunk_load<true>(cr, ba, x.Qb, x.Kb, x.Vb, x.Gb, chunk_row(0), x.row_end);
  __syncthreads();
  if (nchunk > 0) chunk_store<true>(cr, sm, ba, x.isoC, bh, x.cs, x.wmax1, chunk_row(0), x.row_end);
  __syncthreads();
  for (int ci = 0; ci < nchunk; ++ci) {
    const int row0 = chunk_row(ci);
    const bool more = ci + 1 < nchunk;
    if (more) chunk_load<true>(cr, ba, x.Qb, x.Kb, x.Vb, x.Gb, chunk_row(ci + 1), x.row_end);

    // query tiles and their transposes
    bf16x8 p[4][2], pt[4][2];
#pragma unroll
    for (int ip = 0; ip < 2; ++ip) {
      f32x4 tr[2][4];
#pragma unroll
      for (int ii = 0; ii < 2; ++ii) {
        const int it = 2 * ip + ii;
        feature_tile<true>(wq, &qb, sm.q, it, sm.qadd[16 * it + c], p[it]);
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int hh = 0; hh < 2; ++hh) tr[ii][2 * mb + hh] = mfma(p[it][mb], sel[hh], f32x4{0.f, 0.f, 0.f, 0.f});
      }
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) pt[mt][ip] = pack8(tr[0][mt], tr[1][mt]);
    }
    bf16x8 rb[NVT][2];
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt) {
      rb[vt][0] = pack8(T[0][vt], T[1][vt]);
      rb[vt][1] = pack8(T[2][vt], T[3][vt]);
    }
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) {
      bf16x8 s[2];
      feature_tile<false>(wk, nullptr, sm.k, jt, sm.kadd[16 * jt + c], s);
      // dV1 tile = R_next^T x S  +  G1^T x B  (B[i][j] = P_i . S_j over this wave's features, i >= j)
      f32x4 y[NVT];
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) {
        y[vt] = mfma(rb[vt][0], s[0], f32x4{0.f, 0.f, 0.f, 0.f});
        y[vt] = mfma(rb[vt][1], s[1], y[vt]);
      }
#pragma unroll
      for (int ip = 0; ip < 2; ++ip) {
        if (2 * ip + 1 >= jt) {
          f32x4 bc[2];
#pragma unroll
          for (int ii = 0; ii < 2; ++ii) {
            const int it = 2 * ip + ii;
            bc[ii] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (it >= jt) {
              bc[ii] = mfma(p[it][0], s[0], bc[ii]);
              bc[ii] = mfma(p[it][1], s[1], bc[ii]);
              if (it == jt) {
#pragma unroll
                for (int r = 0; r < 4; ++r) bc[ii][r] = (4 * g + r >= c) ? bc[ii][r] : 0.f;
              }
            }
          }
          const bf16x8 bb = pack8(bc[0], bc[1]);
#pragma unroll
          for (int vt = 0; vt < NVT; ++vt) y[vt] = mfma(load_vop(sm.gt, ip, vt), bb, y[vt]);
        }
      }
      exchange_put_bf16(sm, y, jt, w, lane);
    }
    // the suffix sum takes this chunk's queries
#pragma unroll
    for (int ip = 0; ip < 2; ++ip)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) {
        const bf16x8 gop = load_vop(sm.gt, ip, vt);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) T[mt][vt] = mfma(pt[mt][ip], gop, T[mt][vt]);
      }
    __syncthreads();
    {
      const int token = row0 + 16 * w + c;
      f32x4 fv[4] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
      finish_tiles(fv, sm, w, 0, lane);
      finish_tiles(fv, sm, w, 2, lane);
      if (token < x.row_end) {
        if (ba.dV.dtype == 1) {
          uint16_t* yp = (uint16_t*)ba.dV.ptr + x.b * ba.dV.sb + x.h * ba.dV.sh + (long long)token * ba.dV.sl + 4 * g;
#pragma unroll
          for (int vt = 0; vt < 4; ++vt) *(bf16x4*)(yp + 16 * vt) = __builtin_convertvector(fv[vt], bf16x4);
        } else {
          float* yp = (float*)ba.dV.ptr + x.b * ba.dV.sb + x.h * ba.dV.sh + (long long)token * ba.dV.sl + 4 * g;
#pragma unroll
          for (int vt = 0; vt < 4; ++vt) *(f32x4*)(yp + 16 * vt) = fv[vt];
        }
      }
    }
    __syncthreads();
    if (more) chunk_store<true>(cr, sm, ba, x.isoC, bh, x.cs, x.wmax1, chunk_row(ci + 1), x.row_end);
    __syncthreads();
  }
}

}  // namespace bwd

using namespace bwd;

#define FS_LAUNCH_CHECK() do { if (hipGetLastError() != hipSuccess) return 5; } while (0)

// One causal backward call after the forward state pass over every slot (f.Tpart = exclusive prefix per slot on the
// sequence's common shift f.cstar).
int launch_fast_backward_causal(const FastLaunch& f, const FastArgs& a, const TensorDev& dY, const TensorDev& dQ,
                                const TensorDev& dK, const TensorDev& dV, uint16_t* gh, float* Rpart, float* rcpart,
                                hipStream_t st) {
  BwdArgs ba;
  ba.f = a;
  ba.dY = dY; ba.dQ = dQ; ba.dK = dK; ba.dV = dV;
  ba.gh = gh; ba.Rpart = Rpart; ba.rcpart = rcpart;
  ba.Lq = f.Lq; ba.Lk = f.Lk; ba.rslots = a.nslot; ba.rows_per_rslot = a.rows_per_seg / a.sub;
  const int BH = f.B * f.H;
  if (int rc = launch_bwd_walk_pc(ba, 0, a.nslot, BH, st)) return rc;
  if (int rc = launch_bwd_rstate(ba, BH, st)) return rc;
  hipLaunchKernelGGL(k_bwd_suffix, dim3((M * DVP + 255) / 256, BH), dim3(256), 0, st, Rpart, a.nslot);
  FS_LAUNCH_CHECK();
  if (int rc = launch_bwd_walk_pc(ba, 1, a.nslot, BH, st)) return rc;
  return launch_bwd_cgrad_pc(ba, a.nslot, BH, st);
}

size_t fast_bwd_causal_lds_bytes() { return bwd_pc_lds_bytes(); }

}  // namespace fs
