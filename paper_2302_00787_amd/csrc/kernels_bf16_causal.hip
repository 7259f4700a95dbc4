// Causal segment kernel of the bf16 attention path (d = dv = 64, M = 256).
//
// One workgroup (8 waves = two per SIMD of one CU) walks one segment of one sequence in 64-token chunks, its state
// seeded with the exclusive prefix of the segment states:
//   Y_c = (tril(P_c S_c^T) [V_c 1] + P_c T_{c-1}) normalised by its last column;  T_c = T_{c-1} + S_c^T [V_c 1].
//
// Wave w owns the 32 random features [32w, 32w+32): its slices of the projection matrix W~ (bf16) and of the state T
// (fp32, 32 x 80) stay in registers, so every wave needs at most 256 registers, two waves share a SIMD and one wave's
// exp2 / convert work overlaps the other's MFMAs and LDS waits.  Register-level dataflow, operand layouts and shifts
// are those described in fast_common.h (with one 32-feature block per wave instead of two).  The partial outputs
// of the eight waves are exchanged through LDS as bf16; wave w finishes token tile w/2, value columns 32 (w%2) .. +31.
//
// Two instantiations: SYM (B1 = B2, the query and key projections share one W~ slice: PosRF, GERF, SDERF; fewer live
// registers, measurably faster) and the general one; each workgroup looks at the flag of its own parameter set and the
// instantiation that does not match returns at once.
#include "fast_common.h"

namespace fs {

using namespace fast;

namespace c8 {

constexpr int NW8 = 8;             // waves per workgroup, 32 features each
constexpr int NT8 = NW8 * 64;
constexpr int LDXB = DVP + 4;      // row stride (bf16 elements) of the exchange buffer: 42 dwords, conflict-free b64 access

struct Smem8 {
  uint16_t k[2][TC][LDR];          // key rows, bf16 bits
  uint16_t q[2][TC][LDR];          // query rows
  uint16_t vt[2][DVP][LDJ];        // values transposed: [column][token]; row 64 = ones, rows 65.. = 0
  float kadd[2][TC];               // per key token: row term log2e y^T C2 y
  __attribute__((aligned(16))) float kbnd[2][TC];   // per key token: row_shift + row term (-inf past the end)
  float qadd[2][TC];               // per query token: - row_shift
  __attribute__((aligned(16))) uint16_t xch[4][NW8][16][LDXB];   // partial outputs (bf16): [token tile][source wave][token][column]
};

struct W32 { bf16x8 w[2][KS]; };   // rows = features 32w + 16mt + c, k = 32ks + 8g + e
struct B32 { f32x4 b[2]; };        // 2 (bias - largest bias) of features 32w + 16mt + 4g + r

__device__ __forceinline__ void load_w32(W32& ws, const uint16_t* Wbf) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      ws.w[mt][ks] = *(const bf16x8*)(Wbf + (size_t)(32 * w + 16 * mt + c) * D + 32 * ks + 8 * g);
}

// One 16-byte piece per thread of a 64 x 64 bf16 tile: row tid/8, bytes 16 (tid%8).
__device__ __forceinline__ u32x4 load_row_piece(const uint16_t* base, long long sl, int row0, int row_end) {
  const int row = threadIdx.x >> 3, pc = threadIdx.x & 7;
  u32x4 p = {0u, 0u, 0u, 0u};
  if (row0 + row < row_end) p = *(const u32x4*)(base + (long long)(row0 + row) * sl + pc * 8);
  return p;
}
__device__ __forceinline__ float store_row_piece(u32x4 p, uint16_t (*tile)[LDR]) {
  const int row = threadIdx.x >> 3, pc = threadIdx.x & 7;
  *(u32x4*)(&tile[row][pc * 8]) = p;
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float lo = __uint_as_float(p[e] << 16), hi = __uint_as_float(p[e] & 0xffff0000u);
    s += lo * lo + hi * hi;
  }
  return sum8(s);
}
// Values: token tid%64, piece tid/64; lane pairs swap halves so that every lane writes whole dwords.
__device__ __forceinline__ u32x4 load_val_piece(const uint16_t* base, long long sl, int row0, int row_end) {
  const int j = threadIdx.x & 63, pc = threadIdx.x >> 6;
  u32x4 p = {0u, 0u, 0u, 0u};
  if (row0 + j < row_end) p = *(const u32x4*)(base + (long long)(row0 + j) * sl + pc * 8);
  return p;
}
__device__ __forceinline__ void store_val_piece(u32x4 p, uint16_t (*vt)[LDJ], int row0, int row_end) {
  const int j = threadIdx.x & 63, pc = threadIdx.x >> 6, odd = j & 1;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const uint32_t mine = p[e], other = dpp_u<0xB1>(mine);
    const uint32_t w = odd ? ((other >> 16) | (mine & 0xffff0000u)) : ((mine & 0xffffu) | (other << 16));
    *(uint32_t*)(&vt[pc * 8 + 2 * e + odd][j & ~1]) = w;
  }
  if (threadIdx.x < 32) {
    const int t0 = 2 * threadIdx.x;
    const uint32_t one = 0x3f80u;     // bf16(1)
    *(uint32_t*)(&vt[D][t0]) = (row0 + t0 < row_end ? one : 0u) | (row0 + t0 + 1 < row_end ? one << 16 : 0u);
  }
}

struct Stage { u32x4 q, k, v; };

__device__ __forceinline__ void stage_load(Stage& s, const uint16_t* Qb, const uint16_t* Kb, const uint16_t* Vb,
                                           const FastArgs& a, int row0, int row_end) {
  s.q = load_row_piece(Qb, a.Q.sl, row0, row_end);
  s.k = load_row_piece(Kb, a.K.sl, row0, row_end);
  s.v = load_val_piece(Vb, a.V.sl, row0, row_end);
}

__device__ __forceinline__ void stage_store(const Stage& s, Smem8& sm, int buf, const FastArgs& a, bool isoC, int bh,
                                            int row0, int row_end, float wmax1, float wmax2) {
  const int row = threadIdx.x >> 3;
  const float nq2 = store_row_piece(s.q, sm.q[buf]);
  const float nk2 = store_row_piece(s.k, sm.k[buf]);
  if ((threadIdx.x & 7) == 0) {
    const bool valid = row0 + row < row_end;
    float rt = -0.5f * kLog2e * a.scale * a.scale * nk2;
    if (!isoC) rt = valid ? a.rk[(size_t)bh * a.L + row0 + row] : 0.f;
    sm.qadd[buf][row] = -row_shift(nq2, wmax1);
    sm.kadd[buf][row] = rt;
    sm.kbnd[buf][row] = valid ? row_shift(nk2, wmax2) + rt : -INFINITY;
  }
  store_val_piece(s.v, sm.vt[buf], row0, row_end);
}

// Feature tile of 16 tokens and this wave's 32 features, packed as an MFMA operand (lane <-> token 16 jt + c,
// k = 8g + e <-> feature 16 (e/4) + 4g + e%4 of the wave's block).
template <bool WITH_BIAS>
__device__ __forceinline__ bf16x8 feature_tile32(const W32& ws, const B32* qb, const uint16_t (*tile)[LDR], int jt, float add) {
  const int lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
  bf16x8 b[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) b[ks] = *(const bf16x8*)(&tile[16 * jt + c][32 * ks + 8 * g]);
  f32x4 acc[2];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt) {
    acc[mt] = WITH_BIAS ? qb->b[mt] : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) acc[mt] = mfma(ws.w[mt][ks], b[ks], acc[mt]);
  }
  return pack8(exp2v(acc[0] + add), exp2v(acc[1] + add));
}

}  // namespace c8

using namespace c8;

// grid (nseg, B*H), block 512.
template <bool SYM>
__global__ void __launch_bounds__(NT8) k_fast_causal(FastArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  Smem8& sm = *reinterpret_cast<Smem8*>(smem_raw);
  const int seg = blockIdx.x, bh = blockIdx.y, b = bh / a.H, h = bh % a.H;
  const float* th = a.theta + (size_t)group_of(a.groups, b, h, a.H) * (FS_THETA_HEADER_ + (size_t)D + 4 * (size_t)D * D);
  const int flags = (int)th[2];
  if (((flags >> 1) & 1) != (SYM ? 1 : 0)) return;
  const bool isoC = flags & 1;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  const int pg = group_of(a.pgroups, b, h, a.H);
  const float wmax1 = a.bounds[((size_t)pg * 2) * 2], amax1 = a.bounds[((size_t)pg * 2) * 2 + 1];
  const float wmax2 = a.bounds[((size_t)pg * 2 + 1) * 2];
  const uint16_t* Qb = (const uint16_t*)a.Q.ptr + b * a.Q.sb + h * a.Q.sh;
  const uint16_t* Kb = (const uint16_t*)a.K.ptr + b * a.K.sb + h * a.K.sh;
  const uint16_t* Vb = (const uint16_t*)a.V.ptr + b * a.V.sb + h * a.V.sh;
  const long long ybase = b * a.Y.sb + h * a.Y.sh;

  W32 wq, wk2;
  load_w32(wq, a.Wbf + ((size_t)pg * 2) * M * D);
  if (!SYM) load_w32(wk2, a.Wbf + ((size_t)pg * 2 + 1) * M * D);
  const W32& wk = SYM ? wq : wk2;
  B32 qb;
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int r = 0; r < 4; ++r) qb.b[mt][r] = 2.f * (a.bias[((size_t)pg * 2) * M + 32 * w + 16 * mt + 4 * g + r] - amax1);
  bf16x8 sel[2];
  make_sel(sel);
  for (int idx = threadIdx.x; idx < 2 * (DVP - D - 1) * LDJ; idx += NT8) {
    const int bb = idx / ((DVP - D - 1) * LDJ), rem = idx - bb * (DVP - D - 1) * LDJ;
    sm.vt[bb][D + 1 + rem / LDJ][rem % LDJ] = 0;
  }
  f32x4 T[2][NVT];
  {
    const float* Tg = a.Tpart + ((size_t)bh * a.nslot + (size_t)seg * a.sub) * M * DVP;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
        for (int r = 0; r < 4; ++r) T[mt][vt][r] = Tg[(size_t)(32 * w + 16 * mt + 4 * g + r) * DVP + 16 * vt + c];
  }
  float dk = a.cstar[bh];          // shift of the prefix state (-inf when there is none)

  const int row_beg = seg * a.rows_per_seg, row_end = min(a.L, row_beg + a.rows_per_seg);
  Stage stg;
  stage_load(stg, Qb, Kb, Vb, a, row_beg, row_end);
  stage_store(stg, sm, 0, a, isoC, bh, row_beg, row_end, wmax1, wmax2);
  __syncthreads();

  // this wave finishes token tile w/2, value tiles 2 (w%2) and 2 (w%2) + 1
  const int oit = w >> 1, ovt = 2 * (w & 1);

  int buf = 0;
  for (int row0 = row_beg; row0 < row_end; row0 += TC, buf ^= 1) {
    const bool more = row0 + TC < row_end;
    if (more) stage_load(stg, Qb, Kb, Vb, a, row0 + TC, row_end);

    // running key shift (every wave computes the same numbers); the state is rebased when it grows
    {
      const f32x4 b4 = *(const f32x4*)(&sm.kbnd[buf][4 * c]);
      const float dnew = max16(fmaxf(fmaxf(b4[0], b4[1]), fmaxf(b4[2], b4[3])));
      if (dnew > dk) {
        const float f = fast_exp2(dk - dnew);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int vt = 0; vt < NVT; ++vt) T[mt][vt] *= f;
        dk = dnew;
      }
    }

    // state before this chunk as A operand (T^T: row v = 16 vt + c, k <-> feature)
    bf16x8 tb[NVT];
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt) tb[vt] = pack8(T[0][vt], T[1][vt]);

    // key side: S (lane <-> token) for the scores, S^T (lane <-> feature) for the state update, pair by pair
    bf16x8 s[4];
#pragma unroll
    for (int jp = 0; jp < 2; ++jp) {
      f32x4 tr[2][2];
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const int jt = 2 * jp + jj;
        s[jt] = feature_tile32<false>(wk, nullptr, sm.k[buf], jt, sm.kadd[buf][16 * jt + c] - dk);
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) tr[jj][hh] = mfma(s[jt], sel[hh], f32x4{0.f, 0.f, 0.f, 0.f});
      }
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        const bf16x8 st = pack8(tr[0][mt], tr[1][mt]);
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt) T[mt][vt] = mfma(st, load_vop(sm.vt[buf], jp, vt), T[mt][vt]);
      }
    }

    // query side, one token tile at a time
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const bf16x8 p = feature_tile32<true>(wq, &qb, sm.q[buf], it, sm.qadd[buf][16 * it + c]);
      f32x4 y[NVT];
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) y[vt] = mfma(tb[vt], p, f32x4{0.f, 0.f, 0.f, 0.f});
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
              sc[jj] = mfma(s[jt], p, sc[jj]);
              if (jt == it) {
#pragma unroll
                for (int r = 0; r < 4; ++r) sc[jj][r] = (4 * g + r <= c) ? sc[jj][r] : 0.f;
              }
            }
          }
          const bf16x8 sb = pack8(sc[0], sc[1]);
#pragma unroll
          for (int vt = 0; vt < NVT; ++vt) y[vt] = mfma(load_vop(sm.vt[buf], jp, vt), sb, y[vt]);
        }
      }
      // hand the partial tile over (bf16): rows v = 16 vt + 4g + r of token column c
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt)
        *(bf16x4*)(&sm.xch[it][w][c][16 * vt + 4 * g]) = __builtin_convertvector(y[vt], bf16x4);
    }
    __syncthreads();

    // finish: sum the eight parts of (token tile oit, value tiles ovt, ovt + 1) and of the normaliser row v = 64.
    // The sum over the source waves is itself a contraction, done on the MFMA pipe: B[k = (source, row-in-group)][n =
    // token] straight from the exchange buffer, A = a 0/1 matrix that routes group q's four rows to accumulator rows
    // 4q .. 4q+3 (so four MFMAs fill one 16 x 16 tile), and for the normaliser a matrix that copies its row everywhere.
    {
      const uint32_t base0 = (c & 3) == 0 ? 0x3f80u : ((c & 3) == 1 ? 0x3f800000u : 0u);
      const uint32_t base1 = (c & 3) == 2 ? 0x3f80u : ((c & 3) == 3 ? 0x3f800000u : 0u);
      f32x4 sum[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const u32x2 lo = *(const u32x2*)(&sm.xch[oit][2 * g][c][16 * (ovt + u) + 4 * q]);
          const u32x2 hi = *(const u32x2*)(&sm.xch[oit][2 * g + 1][c][16 * (ovt + u) + 4 * q]);
          const u32x4 bq = {lo[0], lo[1], hi[0], hi[1]};
          const uint32_t a0 = (c >> 2) == q ? base0 : 0u, a1 = (c >> 2) == q ? base1 : 0u;
          const u32x4 aq = {a0, a1, a0, a1};
          sum[u] = mfma(__builtin_bit_cast(bf16x8, aq), __builtin_bit_cast(bf16x8, bq), sum[u]);
        }
      const u32x2 dlo = *(const u32x2*)(&sm.xch[oit][2 * g][c][D]);
      const u32x2 dhi = *(const u32x2*)(&sm.xch[oit][2 * g + 1][c][D]);
      const u32x4 bd = {dlo[0], dlo[1], dhi[0], dhi[1]};
      const u32x4 ad = {0x3f80u, 0u, 0x3f80u, 0u};
      const f32x4 dn = mfma(__builtin_bit_cast(bf16x8, ad), __builtin_bit_cast(bf16x8, bd), f32x4{0.f, 0.f, 0.f, 0.f});
      const float den = dn[0];
      const float inv = den > 0.f ? 1.f / den : 0.f;
      const int token = row0 + 16 * oit + c;
      if (token < row_end) {
        if (a.Y.dtype == 1) {
          uint16_t* yp = (uint16_t*)a.Y.ptr + ybase + (long long)token * a.Y.sl + 16 * ovt + 4 * g;
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            const f32x4 v = sum[u] * inv;
            *(bf16x4*)(yp + 16 * u) = __builtin_convertvector(v, bf16x4);
          }
        } else {
          float* yp = (float*)a.Y.ptr + ybase + (long long)token * a.Y.sl + 16 * ovt + 4 * g;
#pragma unroll
          for (int u = 0; u < 2; ++u) *(f32x4*)(yp + 16 * u) = sum[u] * inv;
        }
      }
    }
    if (more) stage_store(stg, sm, buf ^ 1, a, isoC, bh, row0 + TC, row_end, wmax1, wmax2);
    __syncthreads();
  }
}

int launch_fast_causal_kernel(const FastArgs& a, int BH, hipStream_t st) {
  const void* fns[2] = {(const void*)k_fast_causal<true>, (const void*)k_fast_causal<false>};
  for (const void* fn : fns)
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(Smem8)) != hipSuccess) {
      (void)hipGetLastError();
      return 2;
    }
  hipLaunchKernelGGL(k_fast_causal<true>, dim3(a.nseg, BH), dim3(NT8), sizeof(Smem8), st, a);
  if (hipGetLastError() != hipSuccess) return 5;
  hipLaunchKernelGGL(k_fast_causal<false>, dim3(a.nseg, BH), dim3(NT8), sizeof(Smem8), st, a);
  if (hipGetLastError() != hipSuccess) return 5;
  return 0;
}

}  // namespace fs
