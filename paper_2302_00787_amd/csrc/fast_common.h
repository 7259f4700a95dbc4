// Device-side building blocks of the bf16 attention kernels (d = dv = 64, M = 256) for gfx950.
//
// Key-side state kernel and non-causal query-side kernel: one workgroup = 4 waves; wave w owns the 64 random
// features [64w, 64w+64): its slice of the projection matrix W~ (bf16) and of the M x (d+1) state T (fp32 MFMA
// accumulators) stay in registers for the whole kernel, so the feature matrices P, S are produced, used and
// discarded in registers.  (The causal kernel splits the same dataflow over producer and consumer waves, see
// kernels_bf16_causal.hip; operand layouts, exponents and shifts are the ones described here.)
//
//   E^T tile   = W~ (A operand) x tokens (B operand)      -> accumulator: lane <-> token, registers <-> feature
//   S, P       = exp2(E^T)  (bias preloaded in the accumulator, per-token shift added before the exp2)
//   scores^T   = S (A operand, straight from the accumulator layout) x P^T (B operand, ditto)
//   Y^T        = T^T (A operand = converted accumulators) x P^T  +  V'^T (A operand) x scores^T (B operand)
//   T         += S^T x V'   where S^T (lane <-> feature) is obtained from S by an MFMA against a selection matrix
//
// All MFMAs are v_mfma_f32_16x16x32_bf16: lane l supplies A[l%16][8(l/16)..+7], B[8(l/16)..+7][l%16] and owns
// D[4(l/16)..+3][l%16].  Stacking two 16-row accumulator tiles gives, per lane, the 8 values of one operand row;
// the induced order of the contraction index is k = 8g+e  <->  16(e/4) + 4g + e%4, the same for every operand
// built that way, so products stay consistent.
//
// Exponents live in the log2 domain; W~ carries log2(e) and qk_scale.  Shifts: every query row has its own (it
// cancels in the normalisation, Section 2.2); the key side needs a common one, kept as a running maximum of a
// per-token bound with the state rescaled whenever it grows.  Both come from the Cauchy-Schwarz bound on the
// projection (see row_shift), so nothing can overflow; rows whose bound exceeds about 2^250 may flush to zero.
#pragma once
#include "fs_common.h"
#include "kernels.h"

namespace fs {
namespace fast {

constexpr int D = 64;            // head dimension (= value dimension)
constexpr int M = 256;           // random features
constexpr int NW = 4;            // waves per workgroup, 64 features each
constexpr int NT = NW * 64;
constexpr int TC = 64;           // tokens per chunk
constexpr int KS = D / 32;       // MFMA k-steps of a projection
constexpr int NVT = 5;           // value tiles of 16 columns: 64 values + normaliser column + padding
constexpr int DVP = NVT * 16;    // 80
constexpr int LDR = D + 8;       // row stride (bf16 elements) of a token tile in LDS: 36 dwords, conflict-free b128 reads
constexpr int LDJ = TC + 4;      // row stride of the transposed value tile in LDS: 34 dwords, conflict-free b64 reads
constexpr float kBeta = 0.5f;

typedef __attribute__((ext_vector_type(8))) float f32x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;

__device__ __forceinline__ f32x4 mfma(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ bf16x8 pack8(f32x4 a, f32x4 b) {
  f32x8 t = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_convertvector(t, bf16x8);
}
__device__ __forceinline__ f32x4 exp2v(f32x4 x) {
  return f32x4{fast_exp2(x[0]), fast_exp2(x[1]), fast_exp2(x[2]), fast_exp2(x[3])};
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int s = 1; s < 64; s <<= 1) v = fmaxf(v, __shfl_xor(v, s));
  return v;
}

// Data-parallel-primitive moves inside a row of 16 lanes (no LDS round trip).  CTRL: 0xB1 = swap lanes within pairs,
// 0x4E = swap pairs within quads, 0x141 = mirror within 8 lanes, 0x124 / 0x128 = rotate the row by 4 / 8 lanes.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
// Sum over the aligned group of 8 lanes the lane belongs to; every lane of the group gets the total.
__device__ __forceinline__ float sum8(float v) {
  v += dpp_f<0xB1>(v);
  v += dpp_f<0x4E>(v);
  v += dpp_f<0x141>(v);
  return v;
}
// Maximum over the row of 16 lanes the lane belongs to; every lane of the row gets it.
__device__ __forceinline__ float max16(float v) {
  v = fmaxf(v, dpp_f<0xB1>(v));
  v = fmaxf(v, dpp_f<0x4E>(v));
  v = fmaxf(v, dpp_f<0x124>(v));
  v = fmaxf(v, dpp_f<0x128>(v));
  return v;
}

// Largest of 256 floats (16-byte aligned), as a wave-uniform value.
__device__ __forceinline__ float max256(const float* p) {
  const f32x4 v = *(const f32x4*)(p + 4 * (threadIdx.x & 63));
  const float m = wave_max(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])));
  return __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, m)));
}

// Per-token shift of the projection part W~_m . x of the exponent.  With cs = max_m |W~_m| |x| (Cauchy-Schwarz)
// the projection never exceeds cs; random directions reach about 0.4 cs.  max(cs/2, cs - 120) keeps the largest
// shifted exponent below 2^120 for every input and near zero for ordinary ones.
__device__ __forceinline__ float row_shift(float n2, float wmax) {
  const float cs = wmax * __builtin_amdgcn_sqrtf(n2);     // the hardware square root: any bound of this size will do
  return fmaxf(kBeta * cs, cs - 120.f);
}

// LDS of a key-side state kernel in the layout with transposed values (the query-side state kernel of the
// backward pass): double-buffered rows, values transposed, one constant per token.
struct Smem {
  uint16_t k[2][TC][LDR];       // rows, bf16 bits
  uint16_t vt[2][DVP][LDJ];     // values transposed: [column][token]
  __attribute__((aligned(16))) float kadd[2][TC];   // per token: the constant added to its exponents
};

// Everything the kernels of one attention call share.
struct FastArgs {
  TensorDev Q, K, V, Y;
  const uint16_t* Wbf;     // [pg][2][M][D]
  const float* bias;       // [pg][2][M]
  const float* wnorm;      // [pg][2][M]: |Wbf_m|
  const float* theta;
  const float* rk;         // [BH][L] key row terms for parameter sets with a dense C2, else unused
  float* Tpart;            // [BH][nslot][M][DVP], nslot = nseg * sub: one state per sub-segment
  float* cpart;            // [BH][nslot]
  float* cstar;            // [BH] largest shift of each sequence, then [BH][nslot] the shift of each slot's prefix state
  int groups, pgroups, H, L, rows_per_seg, nseg;
  int sub, nslot;          // sub-segments per segment (key-side kernel granularity) and total state slots
  int timg;                // layout of a state in Tpart: 0 = [M][DVP] row-major; 1 = accumulator images, the four
                           // numbers of lane l for tile (mt, vt) of wave w at ((w*4 + mt)*NVT + vt)*256 + 4 l
                           // (16-byte accesses; the forward kernels, whose waves all hold a state that way)
  float scale;
  unsigned* flushed;       // counter of output rows with a zero normaliser (nullptr: not counted)
};

// ---- transposing LDS reads ----------------------------------------------------------------------------------------
// ds_read_b64_tr_b16: every lane supplies the address of an 8-byte piece (four bf16 numbers); inside each row of 16
// lanes the lane (a, b) = (c / 4, c % 4) receives element b of the pieces addressed by lanes a, 4 + a, 8 + a, 12 + a.
// With lane c pointing at row c / 4 and 8-byte column group c % 4 of a row-major 4 x 16 block, lane c therefore
// receives column c of rows 0 .. 3: the block read column-wise, which is what an MFMA operand needs when its
// contraction index runs along the rows of the tile in memory.
typedef __attribute__((ext_vector_type(4))) short s16x4;

__device__ __forceinline__ u32x2 lds_read_tr(const uint16_t* p) {
  const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
  return __builtin_bit_cast(u32x2, v);
}
__device__ __forceinline__ bf16x8 join8(u32x2 lo, u32x2 hi) {
  const u32x4 v = {lo[0], lo[1], hi[0], hi[1]};
  return __builtin_bit_cast(bf16x8, v);
}

// Float maximum into an LDS word (every active lane takes part; the file is compiled with the compiler's wave-level
// pre-reduction of atomics switched off: a handful of lanes hit one address, which the LDS serialises cheaply).
__device__ __forceinline__ void lds_fmax(float* p, float v) {
  __builtin_amdgcn_ds_fmaxf((__attribute__((address_space(3))) float*)p, v, 0, 0, false);
}

// Value rows kept row-major in LDS ([token][column]): 160-byte rows = 64 values, a one (the normaliser column) and
// 15 zeros; 40 dwords per row, so that the four rows a transposing read touches per column group start 8 banks apart.
constexpr int LDV = DVP;

// Value operand of token pair jp and column tile vt: lane <-> column 16 vt + c, contraction index <-> tokens
// {32 jp + 4g + r, 32 jp + 16 + 4g + r} (lane c addresses row 4g + c/4 of the pair's first / second tile, column
// group c%4 of the tile, and receives column 4 (c/4) + c%4 = c of rows 4g .. 4g+3).
__device__ __forceinline__ bf16x8 load_vop_tr(const uint16_t (*v)[LDV], int jp, int vt, int lane) {
  const int g = lane >> 4, c = lane & 15;
  const uint16_t* p = &v[32 * jp + 4 * g + (c >> 2)][16 * vt + 4 * (c & 3)];
  return join8(lds_read_tr(p), lds_read_tr(p + 16 * LDV));
}

// The constant columns 64 .. 79 of `rows` value rows: a one, then zeros (the staging writes columns 0 .. 63 only).
__device__ __forceinline__ void init_value_pad(uint16_t (*v)[LDV], int rows, int nthreads) {
  for (int idx = threadIdx.x; idx < rows * (LDV - D); idx += nthreads) {
    const int row = idx / (LDV - D), col = idx % (LDV - D);
    v[row][D + col] = col == 0 ? 0x3f80 : 0;
  }
}

// Squared norms of the 16 rows of a token tile as the diagonal of X X^T on the MFMA pipe (products of bf16 numbers
// are exact in fp32; the sum is an fp32 sum).  `x0`, `x1`: the tile as MFMA operand (lane <-> row c, contraction
// index 32 ks + 8g + e), which serves as both operands.  The entry of row c sits in lane (g, c) = (c / 4, c),
// register c % 4: the returned value is the squared norm of row c in those 16 lanes (garbage in the others).
__device__ __forceinline__ float tile_row_norms(bf16x8 x0, bf16x8 x1, int lane) {
  f32x4 gm = mfma(x0, x0, f32x4{0.f, 0.f, 0.f, 0.f});
  gm = mfma(x1, x1, gm);
  const int r = lane & 3;
  return r == 0 ? gm[0] : r == 1 ? gm[1] : r == 2 ? gm[2] : gm[3];
}

// ---- staging: global -> registers (one chunk ahead) -> LDS -------------------------------------------------------
// Rows: each thread carries two 16-byte pieces of a 64 x 64 bf16 tile: piece q = tid + 256 i -> row q/8, bytes 16 (q%8).
struct RowRegs { u32x4 p[2]; };

__device__ __forceinline__ void load_rows_g(RowRegs& r, const uint16_t* base, long long sl, int row0, int row_end) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int q = threadIdx.x + NT * i, row = q >> 3, pc = q & 7;
    r.p[i] = u32x4{0u, 0u, 0u, 0u};
    if (row0 + row < row_end) r.p[i] = *(const u32x4*)(base + (long long)(row0 + row) * sl + pc * 8);
  }
}

// Writes the pieces and returns, in every lane of the 8 that share a row, the squared norm of that row.
__device__ __forceinline__ void store_rows_s(const RowRegs& r, uint16_t (*tile)[LDR], float (&n2)[2]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int q = threadIdx.x + NT * i, row = q >> 3, pc = q & 7;
    *(u32x4*)(&tile[row][pc * 8]) = r.p[i];
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float lo = __uint_as_float(r.p[i][e] << 16), hi = __uint_as_float(r.p[i][e] & 0xffff0000u);
      s += lo * lo + hi * hi;
    }
    n2[i] = sum8(s);
  }
}

template <class S>
__device__ __forceinline__ void store_query_rows(const RowRegs& r, S& sm, int buf, float wmax) {
  float n2[2];
  store_rows_s(r, sm.q[buf], n2);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int q = threadIdx.x + NT * i;
    if ((q & 7) == 0) sm.qadd[buf][q >> 3] = -row_shift(n2[i], wmax);
  }
}


// Values: lane pairs (2t, 2t+1) exchange halves so that each lane writes whole dwords {token 2t, token 2t+1} of one
// column: thread -> token tid%64, 16-byte pieces tid/64 and tid/64 + 4 of that token's row.
__device__ __forceinline__ void load_vals_g(RowRegs& r, const uint16_t* base, long long sl, int row0, int row_end) {
  const int j = threadIdx.x & 63;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int pc = (threadIdx.x >> 6) + 4 * i;
    r.p[i] = u32x4{0u, 0u, 0u, 0u};
    if (row0 + j < row_end) r.p[i] = *(const u32x4*)(base + (long long)(row0 + j) * sl + pc * 8);
  }
}

__device__ __forceinline__ void store_vals_s(const RowRegs& r, uint16_t (*vt)[LDJ], int row0, int row_end) {
  const int j = threadIdx.x & 63, odd = j & 1;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int pc = (threadIdx.x >> 6) + 4 * i;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t mine = r.p[i][e], other = dpp_u<0xB1>(mine);
      // even lane: column 2e of tokens (j, j+1); odd lane: column 2e+1 of tokens (j-1, j)
      const uint32_t w = odd ? ((other >> 16) | (mine & 0xffff0000u)) : ((mine & 0xffffu) | (other << 16));
      *(uint32_t*)(&vt[pc * 8 + 2 * e + odd][j & ~1]) = w;
    }
  }
  if (threadIdx.x < 32) {
    const int t0 = 2 * threadIdx.x;
    const uint32_t one = 0x3f80u;     // bf16(1)
    *(uint32_t*)(&vt[D][t0]) = (row0 + t0 < row_end ? one : 0u) | (row0 + t0 + 1 < row_end ? one << 16 : 0u);
  }
}


// ---- per-wave constants ----------------------------------------------------------------------------------------
// The bias_m = log2e (w_m^T A w_m + log D - 1/2 log M) is the same for both sides (A and D are shared by f1 and f2,
// Section 4).  It is applied once, doubled, on the query side; key features and the state carry none:
//   S'[j,m] = exp2(W~2_m . k_j + rowterm_j - shift),   P'[i,m] = exp2(W~1_m . q_i - rowshift_i + 2 (bias_m - amax)),
// so that sum_m P' S' equals sum_m P S up to factors that cancel in the normalisation.
struct WSlice {
  bf16x8 w[4][KS];     // W~ slice as A operand: row = feature 64w + 16mt + c, k = 32ks + 8g + e
};
struct QBias {
  f32x4 b[4];          // 2 (bias - largest bias) of features 64w + 16mt + 4g + r
};

__device__ __forceinline__ void load_wslice(WSlice& ws, const uint16_t* Wbf) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      ws.w[mt][ks] = *(const bf16x8*)(Wbf + (size_t)(64 * w + 16 * mt + c) * D + 32 * ks + 8 * g);
}

__device__ __forceinline__ void load_qbias(QBias& qb, const float* bias, float amax) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int r = 0; r < 4; ++r) qb.b[mt][r] = 2.f * (bias[64 * w + 16 * mt + 4 * g + r] - amax);
}


// Feature tile of 16 tokens: for each 32-feature block mb the packed exp2 values (A / B operand layout:
// lane <-> token 16 jt + c, k <-> feature).  `add` is the per-token part of the exponent (lane c's token).
template <bool WITH_BIAS>
__device__ __forceinline__ void feature_tile(const WSlice& ws, const QBias* qb, const uint16_t (*tile)[LDR], int jt,
                                             float add, bf16x8 out[2]) {
  const int lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
  bf16x8 b[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) b[ks] = *(const bf16x8*)(&tile[16 * jt + c][32 * ks + 8 * g]);
  // without a bias the token's part of the exponent is the accumulator's initial value: nothing is left to add
  const f32x4 add4 = {add, add, add, add};
  f32x4 acc[4];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
    acc[mt] = mfma(ws.w[mt][0], b[0], WITH_BIAS ? qb->b[mt] : add4);
#pragma unroll
    for (int ks = 1; ks < KS; ++ks) acc[mt] = mfma(ws.w[mt][ks], b[ks], acc[mt]);
  }
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) acc[mt] = exp2v(WITH_BIAS ? acc[mt] + add : acc[mt]);
  out[0] = pack8(acc[0], acc[1]);
  out[1] = pack8(acc[2], acc[3]);
}

// Features of one pair of token tiles, feature-major: st[mt] has lane <-> feature 64w + 16 mt + c and contraction
// index <-> the pair's tokens {32 jp + 4g + r, 32 jp + 16 + 4g + r}: the projection MFMA with its operands swapped
// (rows = tokens, columns = features), so the state update S^T [V 1] needs no transpose.  add[t] - sub is the
// per-token part of the exponent; bcol[mt] the bias term of lane c's feature (WITH_BIAS).
template <bool WITH_BIAS>
__device__ __forceinline__ void feature_pair_major(const WSlice& ws, const float (&bcol)[4], const uint16_t (*tile)[LDR],
                                                   const float* add, int jp, float sub, bf16x8 (&st)[4]) {
  const int lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
  bf16x8 x[2][KS];
  f32x4 addv[2];
#pragma unroll
  for (int jj = 0; jj < 2; ++jj) {
    const int jt = 2 * jp + jj;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) x[jj][ks] = *(const bf16x8*)(&tile[16 * jt + c][32 * ks + 8 * g]);
    addv[jj] = *(const f32x4*)(add + 16 * jt + 4 * g) - sub;
  }
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
    f32x4 acc[2];
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
      acc[jj] = mfma(x[jj][0], ws.w[mt][0], WITH_BIAS ? addv[jj] + bcol[mt] : addv[jj]);
#pragma unroll
      for (int ks = 1; ks < KS; ++ks) acc[jj] = mfma(x[jj][ks], ws.w[mt][ks], acc[jj]);
    }
    st[mt] = pack8(exp2v(acc[0]), exp2v(acc[1]));
  }
}


// B operand / A operand of the value tile: lane <-> column 16 vt + c, k <-> tokens {32 jp + 4g + r, 32 jp + 16 + 4g + r}.
__device__ __forceinline__ bf16x8 load_vop(const uint16_t (*vt)[LDJ], int jp, int vtile) {
  const int lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
  const u32x2 lo = *(const u32x2*)(&vt[16 * vtile + c][32 * jp + 4 * g]);
  const u32x2 hi = *(const u32x2*)(&vt[16 * vtile + c][32 * jp + 16 + 4 * g]);
  const u32x4 v = {lo[0], lo[1], hi[0], hi[1]};
  return __builtin_bit_cast(bf16x8, v);
}




// ---- bf16 exchange of partial output tiles and their sum on the MFMA pipe -----------------------------------------
constexpr int LDXB = DVP + 8;      // row stride (bf16 elements) of the bf16 exchange buffer: 176 bytes = 44 dwords: 16-byte accesses of 8 consecutive rows hit 32 different banks

// Partial tile of token tile `it` from source `src` (rows v = 16 vt + 4g + r of token column c), as bf16.
template <class S>
__device__ __forceinline__ void exchange_put_bf16(S& sm, const f32x4 (&y)[NVT], int it, int src, int lane) {
  const int g = lane >> 4, c = lane & 15;
#pragma unroll
  for (int vt = 0; vt < NVT; ++vt) *(bf16x4*)(&sm.xch[it][src][c][16 * vt + 4 * g]) = __builtin_convertvector(y[vt], bf16x4);
}

// Finish of token tile `it` of a chunk (value tiles vt0, vt0 + 1): the sum over the four sources' partial tiles is a
// contraction on the MFMA pipe.  B[k = 8g + e][n = token] = partial of source g, column 16 vt + 8 h + e: one 16-byte
// read straight from the exchange buffer; A_h[i][8g + e] = 1 iff e = i - 8h routes it to accumulator row i (two
// MFMAs, h = 0, 1, fill a 16 x 16 tile).
template <class S>
__device__ __forceinline__ void finish_tiles(f32x4 (&fs)[4], const S& sm, int it, int vt0, int lane) {
  const int g = lane >> 4, c = lane & 15;
  const uint32_t one = (c & 1) ? 0x3f800000u : 0x3f80u;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    u32x4 av = {0u, 0u, 0u, 0u};
    const bool mine = (c >> 3) == h;
#pragma unroll
    for (int i = 0; i < 4; ++i) av[i] = (mine && ((c & 7) >> 1) == i) ? one : 0u;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const bf16x8 bv = *(const bf16x8*)(&sm.xch[it][g][c][16 * (vt0 + u) + 8 * h]);
      fs[vt0 + u] = mfma(__builtin_bit_cast(bf16x8, av), bv, fs[vt0 + u]);
    }
  }
}
// Column 64 of the four partial tiles of token tile `it`, summed and copied to every row by an MFMA: every lane
// (g, c) gets the sum for token c.
template <class S>
__device__ __forceinline__ float finish_col64(const S& sm, int it, int lane) {
  const int g = lane >> 4, c = lane & 15;
  const bf16x8 bd = *(const bf16x8*)(&sm.xch[it][g][c][D]);
  const u32x4 ad = {0x3f80u, 0u, 0u, 0u};
  const f32x4 dn = mfma(__builtin_bit_cast(bf16x8, ad), bd, f32x4{0.f, 0.f, 0.f, 0.f});
  return dn[0];
}
// Normaliser of token tile `it` (column 64); the sums are scaled in place.  Returns 1 / normaliser (0 if it is 0).
// `zero_tokens` (optional) receives the tile's tokens whose normaliser is not positive as a bit mask (bit c = token
// 16 it + c; wave-uniform): all of such a row's features, or all of the state it meets, flushed to zero, and the row
// is written as zeros.
template <class S>
__device__ __forceinline__ float finish_norm(f32x4 (&fs)[4], const S& sm, int it, int lane,
                                             unsigned* zero_tokens = nullptr) {
  const float den = finish_col64(sm, it, lane);
  const float inv = den > 0.f ? __builtin_amdgcn_rcpf(den) : 0.f;
  if (zero_tokens != nullptr) *zero_tokens = (unsigned)__ballot(!(den > 0.f)) & 0xffffu;     // lanes 0..15: g = 0, c = lane
#pragma unroll
  for (int vt = 0; vt < 4; ++vt) fs[vt] *= inv;
  return inv;
}
// How many of the tokens in `zero_tokens` are among the first `nv` tokens of the chunk (wave-uniform arithmetic).
__device__ __forceinline__ int count_zero_tokens(unsigned zero_tokens, int it, int nv) {
  const int left = nv - 16 * it;
  const unsigned valid = left >= 16 ? 0xffffu : (left > 0 ? (1u << left) - 1u : 0u);
  return __builtin_popcount(zero_tokens & valid);
}
// One wave's count goes to the call's counter of rows with a zero normaliser (nothing to do in the usual case).
__device__ __forceinline__ void report_zero_rows(unsigned* flushed, int n, int lane) {
  if (flushed != nullptr && n > 0 && lane == 0) atomicAdd(flushed, (unsigned)n);
}

// Shared memory of the query-side kernels that keep their state in registers (64 kB: two workgroups per CU).
struct SmemApply {
  __attribute__((aligned(16))) uint16_t q[2][TC][LDR];            // rows (queries, or keys in the backward pass)
  float qadd[2][TC];                                              // per token: what is added to its exponents
  __attribute__((aligned(16))) uint16_t xch[NW][NW][16][LDXB];    // partial outputs (bf16): [token tile][source wave][token][column]
};

}  // namespace fast

// Launcher of the causal segment kernel (its own translation unit: it is compiled with different code-generation
// options than the other kernels of the path).
int launch_fast_causal_kernel(const fast::FastArgs& a, int BH, hipStream_t st, hipEvent_t ev_begin = nullptr,
                              hipEvent_t ev_end = nullptr);
size_t fast_causal_lds_bytes();
// Backward pass (kernels_bf16_bwd.hip) and the reduction it borrows from the forward pass (kernels_bf16.hip).
void launch_fast_reduce_sum(float* part, const float* cpart, float* cstar, int nslot, int BH, hipStream_t st);
// Key-side row terms of parameter sets with a dense C2 for bf16 rows of d = 64 or 128 numbers (kernels_bf16.hip).
int launch_key_row_terms(const float* theta, int groups, const TensorDev& K, int B, int H, int L, int d, float scale,
                         float* rk, hipStream_t st);
int launch_fast_backward(const FastLaunch& f, const fast::FastArgs& a, const TensorDev& dY, const TensorDev& dQ,
                         const TensorDev& dK, const TensorDev& dV, uint16_t* gh, float* Rpart, float* rcpart,
                         float* rcstar, int rslots, int rows_per_rslot, hipStream_t st);
int launch_fast_backward_whole(const FastLaunch& f, const fast::FastArgs& a, const TensorDev& dY, const TensorDev& dQ,
                               const TensorDev& dK, const TensorDev& dV, uint16_t* gh, hipStream_t st);
size_t fast_bwd_lds_bytes();
int launch_fast_backward_causal(const FastLaunch& f, const fast::FastArgs& a, const TensorDev& dY, const TensorDev& dQ,
                                const TensorDev& dK, const TensorDev& dV, uint16_t* gh, float* Rpart, float* rcpart,
                                hipStream_t st);
size_t fast_bwd_causal_lds_bytes();

}  // namespace fs
