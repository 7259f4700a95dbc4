// Causal segment kernel of the bf16 attention path (d = dv = 64, M = 256).
//
// One workgroup (8 waves = two per SIMD of one CU) walks one segment of one sequence in 64-token chunks, its state
// seeded with the exclusive prefix of the segment states:
//   Y_c = (tril(P_c S_c^T) [V_c 1] + P_c T_{c-1}) normalised by its last column;  T_c = T_{c-1} + S_c^T [V_c 1].
//
// Wave w owns the 32 random features [32w, 32w+32): its slices of the projection matrix W~ (bf16) and of the state T
// (fp32, 32 x 80) stay in registers, so every wave needs at most 256 registers, two waves share a SIMD and one wave's
// exp2 / convert work overlaps the other's MFMAs and LDS waits.  Register-level dataflow, operand layouts and shifts
// are those described in fast_common.h (with one 32-feature block per wave instead of two).
//
// The partial outputs of the eight waves (each a sum over that wave's features) are exchanged through LDS as bf16 and
// summed on the MFMA pipe, one chunk behind: barrier X | key side of chunk c, and the finish of chunk c-1 (wave w:
// token tile w/2, value columns 32 (w%2) .. +31) | barrier Y | query side of chunk c (writes the exchange buffer),
// and the next chunk's rows go to LDS.  So no wave ever sits in a phase of its own.
//
// Two instantiations: SYM (B1 = B2, the query and key projections share one W~ slice: PosRF, GERF, SDERF; fewer live
// registers) and the general one; each workgroup looks at the flag of its own parameter set and the instantiation
// that does not match returns at once.  (One kernel holding both loops allocates registers worse for both.)
#include "fast_common.h"

namespace fs {

using namespace fast;

namespace c8 {

constexpr int NW8 = 8;             // waves per workgroup, 32 features each
constexpr int NT8 = NW8 * 64;
constexpr int LDXB = DVP + 8;      // row stride (bf16 elements) of the exchange buffer: 176 bytes = 44 dwords: 16-byte accesses of 8 consecutive rows hit 32 different banks

struct Smem8 {
  uint16_t k[2][TC][LDR];          // key rows, bf16 bits
  uint16_t q[2][TC][LDR];          // query rows
  uint16_t vt[2][DVP][LDJ];        // values transposed: [column][token]; row 64 = ones, rows 65.. = 0
  __attribute__((aligned(16))) float kadd[2][TC];   // per key token t, at index 4 (t%16) + t/16: row term log2e y^T C2 y
  __attribute__((aligned(16))) float kbnd[2][TC];   // per key token: row_shift + row term (-inf past the end)
  __attribute__((aligned(16))) float qadd[2][TC];   // per query token t, at index 4 (t%16) + t/16: - row_shift
  // partial outputs (bf16): [token tile][source wave][token][position]; value column 16 vt + 4 g + r sits at position
  // 32 (vt/2) + 8 g + 4 (vt%2) + r (a lane writes two value tiles with one 16-byte store), the normaliser tile
  // (vt = 4) at 64 + 4 g + r
  __attribute__((aligned(16))) uint16_t xch[4][NW8][16][LDXB];
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

// Staging, one chunk ahead: every thread carries one 16-byte piece of the query tile, of the key tile (row tid/8,
// bytes 16 (tid%8)) and of the value tile (token tid%64, bytes 16 (tid/64)).  Addresses are a uniform chunk base plus
// a 32-bit byte offset per thread that does not change from chunk to chunk.
struct Stage { u32x4 q, k, v; float rk; };

// Global memory of a chunk is addressed through buffer descriptors: a uniform base (the chunk's first row), a 32-bit
// byte offset per thread, and a byte count that ends with the last valid row, so that reads past the end of the
// segment return zero and writes there are dropped, without branches or 64-bit address registers.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t chunk_rsrc(const void* base, long long sl_bytes, int rows_valid, int row_bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0,
                                           rows_valid > 0 ? (int)((rows_valid - 1) * sl_bytes + row_bytes) : 0, 0x00020000);
}

__device__ __forceinline__ void stage_load(Stage& s, const uint16_t* Qb, const uint16_t* Kb, const uint16_t* Vb,
                                           const FastArgs& a, bool isoC, int bh, int row0, int nv, int tid) {
  const int row = tid >> 3, pc = tid & 7, j = tid & 63, pv = tid >> 6;
  const __amdgpu_buffer_rsrc_t rq = chunk_rsrc(Qb + (long long)row0 * a.Q.sl, 2 * a.Q.sl, nv, 2 * D);
  const __amdgpu_buffer_rsrc_t rk = chunk_rsrc(Kb + (long long)row0 * a.K.sl, 2 * a.K.sl, nv, 2 * D);
  const __amdgpu_buffer_rsrc_t rv = chunk_rsrc(Vb + (long long)row0 * a.V.sl, 2 * a.V.sl, nv, 2 * D);
  s.q = __builtin_amdgcn_raw_buffer_load_b128(rq, 2 * (row * (int)a.Q.sl + pc * 8), 0, 0);
  s.k = __builtin_amdgcn_raw_buffer_load_b128(rk, 2 * (row * (int)a.K.sl + pc * 8), 0, 0);
  s.v = __builtin_amdgcn_raw_buffer_load_b128(rv, 2 * (j * (int)a.V.sl + pv * 8), 0, 0);
  // key row terms of a dense C2 (an empty range, hence zeros, when the closed form -|k|^2/2 applies)
  const __amdgpu_buffer_rsrc_t rr = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.rk + (size_t)bh * a.L + row0), 0,
                                                                      isoC ? 0 : 4 * max(nv, 0), 0x00020000);
  s.rk = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rr, 4 * row, 0, 0));
}

__device__ __forceinline__ float store_row_piece(u32x4 p, uint16_t (*tile)[LDR], int tid) {
  const int row = tid >> 3, pc = tid & 7;
  *(u32x4*)(&tile[row][pc * 8]) = p;
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float lo = __uint_as_float(p[e] << 16), hi = __uint_as_float(p[e] & 0xffff0000u);
    s += lo * lo + hi * hi;
  }
  return sum8(s);
}
// Values: lane pairs swap halves so that every lane writes whole dwords {token 2t, token 2t+1} of one column.
__device__ __forceinline__ void store_val_piece(u32x4 p, uint16_t (*vt)[LDJ], int row0, int row_end, int tid) {
  const int j = tid & 63, pc = tid >> 6, odd = j & 1;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const uint32_t mine = p[e], other = dpp_u<0xB1>(mine);
    const uint32_t w = odd ? ((other >> 16) | (mine & 0xffff0000u)) : ((mine & 0xffffu) | (other << 16));
    *(uint32_t*)(&vt[pc * 8 + 2 * e + odd][j & ~1]) = w;
  }
  if (tid < 32) {                  // the row of ones (zero past the end of the sequence)
    const int t0 = 2 * tid;
    const uint32_t one = 0x3f80u;  // bf16(1)
    *(uint32_t*)(&vt[D][t0]) = (row0 + t0 < row_end ? one : 0u) | (row0 + t0 + 1 < row_end ? one << 16 : 0u);
  }
}

__device__ __forceinline__ void stage_store(const Stage& s, Smem8& sm, int buf, const FastArgs& a, bool isoC,
                                            int row0, int row_end, float wmax1, float wmax2, int tid) {
  const int row = tid >> 3;
  const float nq2 = store_row_piece(s.q, sm.q[buf], tid);
  const float nk2 = store_row_piece(s.k, sm.k[buf], tid);
  if ((tid & 7) == 0) {
    const bool valid = row0 + row < row_end;
    const float rt = isoC ? -0.5f * kLog2e * a.scale * a.scale * nk2 : s.rk;
    const int pos = 4 * (row & 15) + (row >> 4);
    sm.qadd[buf][pos] = -row_shift(nq2, wmax1);
    sm.kadd[buf][pos] = rt;
    sm.kbnd[buf][row] = valid ? row_shift(nk2, wmax2) + rt : -INFINITY;
  }
  store_val_piece(s.v, sm.vt[buf], row0, row_end, tid);
}

// Selection matrices (B operands) that turn an A operand (lane <-> token, k <-> feature) into an accumulator with
// lane <-> feature: sel[hh] has a one at (k, n) iff k addresses feature 16 hh + n of the 32-feature block.
__device__ __forceinline__ void make_sel32(bf16x8 sel[2], int lane) {
  const int g = lane >> 4, c = lane & 15;
  // the only one of lane (g, c) sits in sel[(c >> 2) == g ? .. ]: element e with e/4 = hh and 4g + e%4 = c
  const uint32_t one = (c & 1) ? 0x3f800000u : 0x3f80u;
  const bool mine = (c >> 2) == g;
#pragma unroll
  for (int hh = 0; hh < 2; ++hh) {
    u32x4 v = {0u, 0u, 0u, 0u};
    v[2 * hh] = (mine && (c & 2) == 0) ? one : 0u;
    v[2 * hh + 1] = (mine && (c & 2) != 0) ? one : 0u;
    sel[hh] = __builtin_bit_cast(bf16x8, v);
  }
}

// 16 token rows as MFMA operand: lane <-> token 16 jt + c, k = 32 ks + 8g + e
struct XOp { bf16x8 b[KS]; };
__device__ __forceinline__ void load_xop(XOp& x, const uint16_t (*tile)[LDR], int jt) {
  const int lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) x.b[ks] = *(const bf16x8*)(&tile[16 * jt + c][32 * ks + 8 * g]);
}

// Feature tile of 16 tokens and this wave's 32 features in two steps, so that the exp2 / convert work of one tile can
// be interleaved with the MFMAs that consume the previous one: the projection (accumulators: rows = features
// 16 mt + 4g + r, column = token c), then the packed MFMA operand (lane <-> token 16 jt + c, k = 8g + e <-> feature
// 16 (e/4) + 4g + e%4 of the wave's block).
struct Proj { f32x4 acc[2]; };
template <bool WITH_BIAS>
__device__ __forceinline__ void project(Proj& pr, const W32& ws, const B32* qb, const XOp& x) {
#pragma unroll
  for (int mt = 0; mt < 2; ++mt) {
    pr.acc[mt] = WITH_BIAS ? qb->b[mt] : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) pr.acc[mt] = mfma(ws.w[mt][ks], x.b[ks], pr.acc[mt]);
  }
}
__device__ __forceinline__ bf16x8 expack(const Proj& pr, float add) {
  return pack8(exp2v(pr.acc[0] + add), exp2v(pr.acc[1] + add));
}

// Finish of one 16 x 32 piece of the output: token tile `it` of a chunk, value tiles 2 cp and 2 cp + 1.  The sum
// over the eight source waves is itself a contraction, done on the MFMA pipe: B[k = (source, row-in-group)][n = token]
// straight from the exchange buffer (lanes of group g read sources g and g + 4; one 16-byte read holds four rows of
// each of the two value tiles), A = a 0/1 matrix that routes column group q's four rows to accumulator rows 4q .. 4q+3
// (four MFMAs fill a tile), and for the normaliser (column 64) a matrix that copies its row everywhere.  Done in
// steps (two column groups at a time) so that the LDS reads can be issued well before their use.
struct FinPart { u32x4 lo[2], hi[2]; };
struct FinSum { f32x4 even, odd; };

__device__ __forceinline__ void finish_read(FinPart& f, const Smem8& sm, int it, int cp, int qh, int lane) {
  const int g = lane >> 4, c = lane & 15;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    f.lo[i] = *(const u32x4*)(&sm.xch[it][g][c][32 * cp + 8 * (2 * qh + i)]);
    f.hi[i] = *(const u32x4*)(&sm.xch[it][g + 4][c][32 * cp + 8 * (2 * qh + i)]);
  }
}
__device__ __forceinline__ void finish_add(FinSum& acc, const FinPart& f, int qh, int lane) {
  const int c = lane & 15;
  const uint32_t base0 = (c & 3) == 0 ? 0x3f80u : ((c & 3) == 1 ? 0x3f800000u : 0u);
  const uint32_t base1 = (c & 3) == 2 ? 0x3f80u : ((c & 3) == 3 ? 0x3f800000u : 0u);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int q = 2 * qh + i;
    const uint32_t a0 = (c >> 2) == q ? base0 : 0u, a1 = (c >> 2) == q ? base1 : 0u;
    const u32x4 aq = {a0, a1, a0, a1};
    const u32x4 be = {f.lo[i][0], f.lo[i][1], f.hi[i][0], f.hi[i][1]};
    const u32x4 bo = {f.lo[i][2], f.lo[i][3], f.hi[i][2], f.hi[i][3]};
    acc.even = mfma(__builtin_bit_cast(bf16x8, aq), __builtin_bit_cast(bf16x8, be), acc.even);
    acc.odd = mfma(__builtin_bit_cast(bf16x8, aq), __builtin_bit_cast(bf16x8, bo), acc.odd);
  }
}
// `chunk_row`: first row of the chunk; `nv`: its number of valid rows (0: nothing is stored).
__device__ __forceinline__ void finish_store(const FinSum& acc, const Smem8& sm, const TensorDev& Y, long long chunk_row,
                                             long long ybase, int nv, int it, int cp, int lane) {
  const int g = lane >> 4, c = lane & 15;
  const u32x2 dlo = *(const u32x2*)(&sm.xch[it][g][c][D]);
  const u32x2 dhi = *(const u32x2*)(&sm.xch[it][g + 4][c][D]);
  const u32x4 bd = {dlo[0], dlo[1], dhi[0], dhi[1]};
  const u32x4 ad = {0x3f80u, 0u, 0x3f80u, 0u};
  const f32x4 dn = mfma(__builtin_bit_cast(bf16x8, ad), __builtin_bit_cast(bf16x8, bd), f32x4{0.f, 0.f, 0.f, 0.f});
  const float den = dn[0];
  const float inv = den > 0.f ? __builtin_amdgcn_rcpf(den) : 0.f;
  const f32x4 ve = acc.even * inv, vo = acc.odd * inv;
  if (Y.dtype == 1) {
    const __amdgpu_buffer_rsrc_t ry = chunk_rsrc((const uint16_t*)Y.ptr + ybase + chunk_row * Y.sl, 2 * Y.sl, nv, 2 * D);
    const int off = 2 * ((16 * it + c) * (int)Y.sl + 32 * cp + 4 * g);
    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, __builtin_convertvector(ve, bf16x4)), ry, off, 0, 0);
    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, __builtin_convertvector(vo, bf16x4)), ry, off + 32, 0, 0);
  } else {
    const __amdgpu_buffer_rsrc_t ry = chunk_rsrc((const float*)Y.ptr + ybase + chunk_row * Y.sl, 4 * Y.sl, nv, 4 * D);
    const int off = 4 * ((16 * it + c) * (int)Y.sl + 32 * cp + 4 * g);
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, ve), ry, off, 0, 0);
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, vo), ry, off + 64, 0, 0);
  }
}

}  // namespace c8

using namespace c8;

#ifdef FS_PROFILE
__device__ unsigned long long fs_prof[8 * 64 * 16];
#define FS_TICK(slot) do { if (prof_on && lane == 0) { __builtin_amdgcn_sched_barrier(0); fs_prof[(w * 64 + ci) * 16 + (slot)] = __builtin_readcyclecounter(); __builtin_amdgcn_sched_barrier(0);} } while (0)
#else
#define FS_TICK(slot)
#endif

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
  const float wmax1 = max256(a.wnorm + ((size_t)pg * 2) * M), amax1 = max256(a.bias + ((size_t)pg * 2) * M);
  const float wmax2 = max256(a.wnorm + ((size_t)pg * 2 + 1) * M);
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
  // padding rows of the transposed value tiles (the staging writes rows 0 .. 64 only)
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
  stage_load(stg, Qb, Kb, Vb, a, isoC, bh, row_beg, min(TC, row_end - row_beg), threadIdx.x);
  stage_store(stg, sm, 0, a, isoC, row_beg, row_end, wmax1, wmax2, threadIdx.x);

  // the piece of every chunk this wave finishes: token tile fit, value tiles 2 fcp and 2 fcp + 1
  const int fit = w >> 1, fcp = w & 1;

  int buf = 0;
#ifdef FS_PROFILE
  const bool prof_on = seg == 3 && bh == 5;
  int ci = -1;
#endif
  for (int row0 = row_beg; row0 < row_end; row0 += TC, buf ^= 1) {
    __syncthreads();               // barrier X: the staged rows of this chunk and the partial outputs of the previous one are complete
#ifdef FS_PROFILE
    ++ci;
    if (prof_on && lane == 0) fs_prof[(w * 64 + ci) * 16 + 15] = wall_clock64();
#endif
    FS_TICK(0);
    // Addresses that are used once per chunk are rebuilt from an opaque copy of the thread number instead of living
    // in registers through the whole loop.
    int tid_here = threadIdx.x;
    asm volatile("" : "+v"(tid_here));
    const int lane_here = tid_here & 63, fit_here = tid_here >> 7, fcp_here = (tid_here >> 6) & 1;
    // next chunk's rows (an empty range, hence zeros that nobody reads, after the last chunk)
    stage_load(stg, Qb, Kb, Vb, a, isoC, bh, row0 + TC, min(TC, row_end - row0 - TC), tid_here);

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

    // Operands are fetched from LDS one tile ahead of their use; the fences keep that order in the schedule.
    const f32x4 kadd4 = *(const f32x4*)(&sm.kadd[buf][4 * c]);
    const f32x4 qadd4 = *(const f32x4*)(&sm.qadd[buf][4 * c]);
    XOp xo[2];
    load_xop(xo[0], sm.k[buf], 0);
    // the previous chunk leaves during the key side (on the first pass there is none: nothing is stored)
    FinPart fp0;
    FinSum fsum = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
    finish_read(fp0, sm, fit_here, fcp_here, 0, lane_here);

    // The selection matrices of the key side are rebuilt every chunk (a dozen instructions) instead of occupying
    // eight registers through the query side; the opaque copy of the lane number keeps them from being hoisted.
    bf16x8 sel[2];
    {
      int lane_here = lane;
      asm volatile("" : "+v"(lane_here));
      make_sel32(sel, lane_here);
    }

    // state before this chunk as A operand (T^T: row v = 16 vt + c, k <-> feature)
    bf16x8 tb[NVT];
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt) tb[vt] = pack8(T[0][vt], T[1][vt]);

    // Software pipeline over the eight feature tiles of the chunk (keys 0..3, queries 0..3): the projection of tile
    // n+1 is issued ahead of the MFMAs that consume tile n, and its exp2 / convert work follows them in program order,
    // so that the two kinds of work are independent neighbours which the hardware can run side by side.
    bf16x8 s[4];
    bf16x8 vop0[NVT];
    Proj pr;
    project<false>(pr, wk, nullptr, xo[0]);
    load_xop(xo[1], sm.k[buf], 1);
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt) vop0[vt] = load_vop(sm.vt[buf], 0, vt);
    s[0] = expack(pr, kadd4[0] - dk);
    bf16x8 p;
#pragma unroll
    for (int jp = 0; jp < 2; ++jp) {
      f32x4 tr[2][2];
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const int jt = 2 * jp + jj;
        // operands two tiles ahead
        if (jt < 2) load_xop(xo[jt & 1], sm.k[buf], jt + 2);
        else load_xop(xo[jt & 1], sm.q[buf], jt - 2);
        __builtin_amdgcn_sched_barrier(0);
        // projection of the next tile
        if (jt < 3) project<false>(pr, wk, nullptr, xo[(jt + 1) & 1]);
        else project<true>(pr, wq, &qb, xo[(jt + 1) & 1]);
        // consumers of this tile
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) tr[jj][hh] = mfma(s[jt], sel[hh], f32x4{0.f, 0.f, 0.f, 0.f});
        if (jt == 0) { finish_add(fsum, fp0, 0, lane_here); finish_read(fp0, sm, fit_here, fcp_here, 1, lane_here); }
        if (jt == 1) finish_add(fsum, fp0, 1, lane_here);
        if (jt == 2) finish_store(fsum, sm, a.Y, row0 - TC, ybase, row0 > row_beg ? TC : 0, fit_here, fcp_here, lane_here);
        if (jj == 1) {
#pragma unroll
          for (int mt = 0; mt < 2; ++mt) {
            const bf16x8 st = pack8(tr[0][mt], tr[1][mt]);
#pragma unroll
            for (int vt = 0; vt < NVT; ++vt)
              T[mt][vt] = mfma(st, jp == 0 ? vop0[vt] : load_vop(sm.vt[buf], 1, vt), T[mt][vt]);
          }
        }
        // exp2 / convert of the next tile
        if (jt < 3) s[jt + 1] = expack(pr, kadd4[jt + 1] - dk);
        else p = expack(pr, qadd4[0]);
      }
    }
    FS_TICK(1);
    __syncthreads();               // barrier Y: every wave has read what it needs of the previous chunk's partial outputs
    FS_TICK(3);

    // query side, one token tile at a time
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      if (it < 2) load_xop(xo[it & 1], sm.q[buf], it + 2);
      __builtin_amdgcn_sched_barrier(0);
      if (it < 3) project<true>(pr, wq, &qb, xo[(it + 1) & 1]);
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
          for (int vt = 0; vt < NVT; ++vt) y[vt] = mfma(jp == 0 ? vop0[vt] : load_vop(sm.vt[buf], 1, vt), sb, y[vt]);
        }
      }
      if (it < 3) p = expack(pr, qadd4[it + 1]);
      // hand the partial tile over (bf16): rows v = 16 vt + 4g + r of token column c, two value tiles per store
#pragma unroll
      for (int vp = 0; vp < 2; ++vp)
        *(bf16x8*)(&sm.xch[it][w][c][32 * vp + 8 * g]) = pack8(y[2 * vp], y[2 * vp + 1]);
      *(bf16x4*)(&sm.xch[it][w][c][D + 4 * g]) = __builtin_convertvector(y[NVT - 1], bf16x4);
      // the staged rows of the next chunk go to LDS while nobody reads that buffer
      if (it == 1) stage_store(stg, sm, buf ^ 1, a, isoC, row0 + TC, row_end, wmax1, wmax2, tid_here);
    }
    FS_TICK(4);
  }
  // the last chunk
  __syncthreads();
  if (row_end > row_beg) {
    const int last0 = row_beg + ((row_end - row_beg - 1) / TC) * TC;
    FinPart fp0;
    FinSum fsum = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
    for (int qh = 0; qh < 2; ++qh) {
      finish_read(fp0, sm, fit, fcp, qh, lane);
      finish_add(fsum, fp0, qh, lane);
    }
    finish_store(fsum, sm, a.Y, last0, ybase, row_end - last0, fit, fcp, lane);
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

#ifdef FS_PROFILE
extern "C" int favorsharp_prof_read(unsigned long long* host) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(fs::fs_prof), sizeof(unsigned long long) * 8 * 64 * 16);
}
#endif
