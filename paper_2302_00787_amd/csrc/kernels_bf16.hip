// bf16 fast path of FAVOR# attention for gfx950: d = dv = 64, M = 256, bf16 Q/K/V, fp32 accumulation.
//
// One workgroup = 4 waves = one CU.  Wave w owns the 64 random features [64w, 64w+64): its slice of the
// projection matrix W~ (bf16) and of the M x (d+1) state T (fp32 MFMA accumulators) stay in registers for the
// whole kernel, so the feature matrices P, S are produced, used and discarded in registers:
//
//   E^T tile   = W~ (A operand) x tokens (B operand)      -> accumulator: lane <-> token, registers <-> feature
//   S, P       = exp2(E^T)  (bias and shift pre-loaded in the accumulator)
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
#include <algorithm>

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
constexpr int LDR = D + 8;       // row stride (bf16 elements) of a token tile in LDS
constexpr int LDJ = TC + 8;      // row stride of the transposed value tile in LDS
constexpr int LDX = DVP + 4;     // row stride (floats) of the exchange buffer
constexpr float kBeta = 0.5f;

typedef __attribute__((ext_vector_type(8))) float f32x8;

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

struct Smem {
  uint16_t q[2][TC][LDR];       // query rows, bf16 bits
  uint16_t k[2][TC][LDR];       // key rows
  uint16_t vt[2][DVP][LDJ];     // values transposed: [column][token]; row 64 = ones, rows 65.. = 0
  float nq2[2][TC];             // squared norms of the raw rows
  float nk2[2][TC];
  float xch[NW][NW - 1][16][LDX];   // partial outputs: [owner token tile][slot][token][column]
};

// ---- staging -----------------------------------------------------------------------------------------
// Each thread carries two 16-byte pieces of a 64 x 64 bf16 tile: piece q = tid + 256 i -> row q/8, bytes 16 (q%8).
struct RowRegs { u32x4 p[2]; };

__device__ __forceinline__ void load_rows_g(RowRegs& r, const uint16_t* base, long long sl, int row0, int row_end) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int q = threadIdx.x + NT * i, row = q >> 3, pc = q & 7;
    r.p[i] = u32x4{0u, 0u, 0u, 0u};
    if (row0 + row < row_end) r.p[i] = *(const u32x4*)(base + (long long)(row0 + row) * sl + pc * 8);
  }
}

__device__ __forceinline__ void store_rows_s(const RowRegs& r, uint16_t (*tile)[LDR], float* n2) {
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
    s += __shfl_xor(s, 1);
    s += __shfl_xor(s, 2);
    s += __shfl_xor(s, 4);
    if (pc == 0) n2[row] = s;
  }
}

// Values: thread -> token tid%64, pieces tid/64 and tid/64 + 4, written transposed.
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
  const int j = threadIdx.x & 63;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int pc = (threadIdx.x >> 6) + 4 * i;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      vt[pc * 8 + 2 * e][j] = (uint16_t)(r.p[i][e] & 0xffffu);
      vt[pc * 8 + 2 * e + 1][j] = (uint16_t)(r.p[i][e] >> 16);
    }
  }
  if (threadIdx.x < 64) vt[D][j] = (row0 + j < row_end) ? (uint16_t)0x3f80 : (uint16_t)0;   // bf16(1)
}

__device__ __forceinline__ void zero_pad_rows(Smem& sm) {
  for (int idx = threadIdx.x; idx < 2 * (DVP - D - 1) * LDJ; idx += NT) {
    const int b = idx / ((DVP - D - 1) * LDJ), rem = idx - b * (DVP - D - 1) * LDJ;
    sm.vt[b][D + 1 + rem / LDJ][rem % LDJ] = 0;
  }
}

// ---- per-wave constants --------------------------------------------------------------------------------
struct WaveConst {
  bf16x8 w[4][KS];     // W~ slice as A operand: row = feature 64w + 16mt + c, k = 32ks + 8g + e
  f32x4 bias[4];       // bias of features 64w + 16mt + 4g + r, shift subtracted
  const float* bias_src;   // unshifted biases of all features (global memory)
};

__device__ __forceinline__ void load_wave_const(WaveConst& wc, const uint16_t* Wbf, const float* bias) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      wc.w[mt][ks] = *(const bf16x8*)(Wbf + (size_t)(64 * w + 16 * mt + c) * D + 32 * ks + 8 * g);
#pragma unroll
    for (int r = 0; r < 4; ++r) wc.bias[mt][r] = bias[64 * w + 16 * mt + 4 * g + r];
  }
  wc.bias_src = bias;
}

__device__ __forceinline__ void set_shift(WaveConst& wc, float shift) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int r = 0; r < 4; ++r) wc.bias[mt][r] = wc.bias_src[64 * w + 16 * mt + 4 * g + r] - shift;
}

// Selection matrices (B operands) that turn an A operand (lane <-> token, k <-> feature) into an accumulator with
// lane <-> feature: sel[hh] has a one at (k, n) iff k addresses feature 16 hh + n of the 32-feature block.
__device__ __forceinline__ void make_sel(bf16x8 sel[2]) {
  const int lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
#pragma unroll
  for (int hh = 0; hh < 2; ++hh) {
    f32x8 t;
#pragma unroll
    for (int e = 0; e < 8; ++e) t[e] = ((e >> 2) == hh && 4 * g + (e & 3) == c) ? 1.f : 0.f;
    sel[hh] = __builtin_convertvector(t, bf16x8);
  }
}

// Feature tile of 16 tokens: returns for each 32-feature block mb the packed exp2 values (A / B operand layout:
// lane <-> token 16 jt + c, k <-> feature).  `add` is a per-token exponent (lane c's token), 0 for queries.
__device__ __forceinline__ void feature_tile(const WaveConst& wc, const uint16_t (*tile)[LDR], int jt, float add,
                                             bf16x8 out[2]) {
  const int lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
  bf16x8 b[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) b[ks] = *(const bf16x8*)(&tile[16 * jt + c][32 * ks + 8 * g]);
  f32x4 acc[4];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
    acc[mt] = wc.bias[mt];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) acc[mt] = mfma(wc.w[mt][ks], b[ks], acc[mt]);
  }
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) acc[mt] = exp2v(acc[mt] + add);
  out[0] = pack8(acc[0], acc[1]);
  out[1] = pack8(acc[2], acc[3]);
}

// B operand / A operand of the value tile: lane <-> column 16 vt + c, k <-> tokens {32 jp + 4g + r, 32 jp + 16 + 4g + r}.
__device__ __forceinline__ bf16x8 load_vop(const uint16_t (*vt)[LDJ], int jp, int vtile) {
  const int lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
  const u32x2 lo = *(const u32x2*)(&vt[16 * vtile + c][32 * jp + 4 * g]);
  const u32x2 hi = *(const u32x2*)(&vt[16 * vtile + c][32 * jp + 16 + 4 * g]);
  const u32x4 v = {lo[0], lo[1], hi[0], hi[1]};
  return __builtin_bit_cast(bf16x8, v);
}

// Per-token shift of the projection part W~_m . x of the exponent.  With cs = max_m |W~_m| |x| (Cauchy-Schwarz)
// the projection never exceeds cs; random directions reach about 0.4 cs.  max(cs/2, cs - 120) keeps the largest
// shifted exponent below 2^120 for every input and near zero for ordinary ones.
__device__ __forceinline__ float row_shift(float n2, float wmax) {
  const float cs = wmax * sqrtf(n2);
  return fmaxf(kBeta * cs, cs - 120.f);
}

}  // namespace fast

using namespace fast;

// ---------------------------------------------------------------------------------------------------
// Projection constants of the fast path: Wbf[pg][side][m][:] = bf16(qk_scale log2e omega_m^T B),
// bias[pg][side][m] = log2e (omega_m^T A omega_m + log D - 1/2 log M), bounds[pg][side] = {max_m |Wbf_m|, max_m bias}.
// grid (2, pgroups), block 256 (= M).
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_fast_prep(const float* theta, int groups, const float* Omega,
                                                   int omega_groups, int pgroups, int B, int H, float scale,
                                                   uint16_t* Wbf, float* bias, float* bounds) {
  __shared__ float red[2][4];
  const int side = blockIdx.x, pg = blockIdx.y, m = threadIdx.x;
  int b = 0, h = 0;
  if (pgroups == H && pgroups != 1) h = pg;
  else if (pgroups != 1) { b = pg / H; h = pg % H; }
  const size_t tf = FS_THETA_HEADER_ + (size_t)D + 4 * (size_t)D * D;
  const float* th = theta + (size_t)group_of(groups, b, h, H) * tf;
  const float* om = Omega + ((size_t)group_of(omega_groups, b, h, H) * M + m) * D;
  const float* Bm = th + FS_THETA_HEADER_ + D + (side ? (size_t)D * D : 0);
  const float* A = th + FS_THETA_HEADER_;
  const size_t o = ((size_t)pg * 2 + side) * M + m;
  float n2 = 0.f, q = 0.f;
  for (int c = 0; c < D; ++c) {
    float acc = 0.f;
    for (int l = 0; l < D; ++l) acc += om[l] * Bm[l * D + c];
    const uint16_t bits = f32_to_bf16_bits(acc * kLog2e * scale);
    Wbf[o * D + c] = bits;
    const float r = bf16_bits_to_f32(bits);
    n2 += r * r;
  }
  for (int l = 0; l < D; ++l) q += A[l] * om[l] * om[l];
  const float bv = kLog2e * (q + th[0] - 0.5f * logf((float)M));
  bias[o] = bv;
  const float wn = wave_max(sqrtf(n2)), bm = wave_max(bv);
  if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = wn; red[1][threadIdx.x >> 6] = bm; }
  __syncthreads();
  if (threadIdx.x == 0) {
    bounds[((size_t)pg * 2 + side) * 2 + 0] = fmaxf(fmaxf(red[0][0], red[0][1]), fmaxf(red[0][2], red[0][3]));
    bounds[((size_t)pg * 2 + side) * 2 + 1] = fmaxf(fmaxf(red[1][0], red[1][1]), fmaxf(red[1][2], red[1][3]));
  }
}

// Key-side row term log2e * y^T C2 y for parameter sets whose C2 is not -I/2 (ADERF, SADERF); rows of sets with
// the -I/2 flag are skipped (the kernels use -|y|^2/2 directly).  grid (ceil(L/256), B*H), block 256.
__global__ void k_fast_rowterm(TensorDev K, int L, int H, const float* theta, int groups, float scale, float* rk) {
  const int bh = blockIdx.y, b = bh / H, h = bh % H;
  const size_t tf = FS_THETA_HEADER_ + (size_t)D + 4 * (size_t)D * D;
  const float* th = theta + (size_t)group_of(groups, b, h, H) * tf;
  if (((int)th[2]) & 1) return;
  const float* C2 = th + FS_THETA_HEADER_ + D + 3 * (size_t)D * D;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= L) return;
  const uint16_t* row = (const uint16_t*)K.ptr + b * K.sb + h * K.sh + (long long)j * K.sl;
  float y[D];
#pragma unroll
  for (int a = 0; a < D; ++a) y[a] = scale * bf16_bits_to_f32(row[a]);
  float acc = 0.f;
  for (int a = 0; a < D; ++a) {
    float t = 0.f;
#pragma unroll
    for (int c = 0; c < D; ++c) t += C2[a * D + c] * y[c];
    acc += y[a] * t;
  }
  rk[(size_t)bh * L + j] = kLog2e * acc;
}

// ---------------------------------------------------------------------------------------------------
// Key-side state of one segment: Tpart[bh][seg] = sum_{j in seg} S_j [V_j 1]^T / 2^cpart[bh][seg]
// (Section 2.1, S^T C with C = [V 1]).  grid (nseg, B*H), block 256.
// ---------------------------------------------------------------------------------------------------
struct FastArgs {
  TensorDev Q, K, V, Y;
  const uint16_t* Wbf;     // [pg][2][M][D]
  const float* bias;       // [pg][2][M]
  const float* bounds;     // [pg][2][2]
  const float* theta;
  const float* rk;         // key row terms for parameter sets with a dense C2, else unused
  float* Tpart;            // [BH][nseg][M][DVP]
  float* cpart;            // [BH][nseg]
  float* cstar;            // [BH]
  int groups, pgroups, H, L, rows_per_seg, nseg;
  float scale;
};

__device__ __forceinline__ float key_rowterm(const FastArgs& a, bool isoC, int bh, int token, float n2, bool valid) {
  if (isoC) return -0.5f * kLog2e * a.scale * a.scale * n2;
  return valid ? a.rk[(size_t)bh * a.L + token] : 0.f;
}

// Largest possible key exponent of the chunk: max over its tokens of row_shift + row term, plus the largest bias.
// Every wave computes the same value (same inputs, same operations).
__device__ __forceinline__ float key_chunk_bound(const FastArgs& a, bool isoC, int bh, int row0, int row_end,
                                                 const float* n2, float wmax, float amax) {
  const int lane = threadIdx.x & 63, tok = row0 + lane;
  float v = -INFINITY;
  if (tok < row_end) v = row_shift(n2[lane], wmax) + key_rowterm(a, isoC, bh, tok, n2[lane], true);
  return wave_max(v) + amax;
}

__global__ void __launch_bounds__(NT) k_fast_state(FastArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  Smem& sm = *reinterpret_cast<Smem*>(smem_raw);
  const int seg = blockIdx.x, bh = blockIdx.y, b = bh / a.H, h = bh % a.H;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  const int pg = group_of(a.pgroups, b, h, a.H);
  const float* th = a.theta + (size_t)group_of(a.groups, b, h, a.H) * (FS_THETA_HEADER_ + (size_t)D + 4 * (size_t)D * D);
  const bool isoC = ((int)th[2]) & 1;
  const float wmax = a.bounds[((size_t)pg * 2 + 1) * 2], amax = a.bounds[((size_t)pg * 2 + 1) * 2 + 1];
  const uint16_t* Kb = (const uint16_t*)a.K.ptr + b * a.K.sb + h * a.K.sh;
  const uint16_t* Vb = (const uint16_t*)a.V.ptr + b * a.V.sb + h * a.V.sh;

  WaveConst wc;
  load_wave_const(wc, a.Wbf + ((size_t)pg * 2 + 1) * M * D, a.bias + ((size_t)pg * 2 + 1) * M);
  bf16x8 sel[2];
  make_sel(sel);
  zero_pad_rows(sm);
  f32x4 T[4][NVT];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt) T[mt][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
  float crun = -INFINITY;

  const int row_beg = seg * a.rows_per_seg, row_end = min(a.L, row_beg + a.rows_per_seg);
  RowRegs kr, vr;
  load_rows_g(kr, Kb, a.K.sl, row_beg, row_end);
  load_vals_g(vr, Vb, a.V.sl, row_beg, row_end);
  store_rows_s(kr, sm.k[0], sm.nk2[0]);
  store_vals_s(vr, sm.vt[0], row_beg, row_end);
  __syncthreads();

  int buf = 0;
  for (int row0 = row_beg; row0 < row_end; row0 += TC, buf ^= 1) {
    const bool more = row0 + TC < row_end;
    if (more) {
      load_rows_g(kr, Kb, a.K.sl, row0 + TC, row_end);
      load_vals_g(vr, Vb, a.V.sl, row0 + TC, row_end);
    }
    // running shift (identical in every wave: same inputs, same operations)
    const float cnew = key_chunk_bound(a, isoC, bh, row0, row_end, sm.nk2[buf], wmax, amax);
    if (cnew > crun) {
      const float f = fast_exp2(crun - cnew);
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt) T[mt][vt] *= f;
      crun = cnew;
      set_shift(wc, crun);
    }
    bf16x8 st[4][2];       // S^T as A operand: [feature tile][token pair block]
#pragma unroll
    for (int jp = 0; jp < 2; ++jp) {
      f32x4 tr[2][4];      // [token tile within the pair][feature tile]
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const int jt = 2 * jp + jj, tok = row0 + 16 * jt + c;
        const float add = key_rowterm(a, isoC, bh, tok, sm.nk2[buf][16 * jt + c], tok < row_end);
        bf16x8 s[2];
        feature_tile(wc, sm.k[buf], jt, add, s);
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int hh = 0; hh < 2; ++hh)
            tr[jj][2 * mb + hh] = mfma(s[mb], sel[hh], f32x4{0.f, 0.f, 0.f, 0.f});
      }
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) st[mt][jp] = pack8(tr[0][mt], tr[1][mt]);
    }
#pragma unroll
    for (int jp = 0; jp < 2; ++jp)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) {
        const bf16x8 vop = load_vop(sm.vt[buf], jp, vt);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) T[mt][vt] = mfma(st[mt][jp], vop, T[mt][vt]);
      }
    if (more) {
      store_rows_s(kr, sm.k[buf ^ 1], sm.nk2[buf ^ 1]);
      store_vals_s(vr, sm.vt[buf ^ 1], row0 + TC, row_end);
    }
    __syncthreads();
  }
  float* out = a.Tpart + ((size_t)bh * a.nseg + seg) * M * DVP;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
      for (int r = 0; r < 4; ++r) out[(size_t)(64 * w + 16 * mt + 4 * g + r) * DVP + 16 * vt + c] = T[mt][vt][r];
  if (threadIdx.x == 0) a.cpart[(size_t)bh * a.nseg + seg] = crun;
}

// Brings the segment states of one (b,h) to the common shift c* = max_seg cpart and sums them (prefix = 0: total
// in slot 0) or replaces them by their exclusive prefix sums (prefix = 1).  grid (ceil(M*DVP/256), B*H).
__global__ void k_fast_reduce(float* Tpart, const float* cpart, float* cstar, int nseg, int nseg_valid, int prefix) {
  const int bh = blockIdx.y;
  const size_t per = (size_t)M * DVP;
  const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  float cs = -INFINITY;
  for (int s = 0; s < nseg_valid; ++s) cs = fmaxf(cs, cpart[(size_t)bh * nseg + s]);
  if (e == 0) cstar[bh] = cs;
  if (e >= per) return;
  float* p = Tpart + (size_t)bh * nseg * per + e;
  float run = 0.f;
  for (int s = 0; s < nseg; ++s) {
    float v = 0.f;
    if (s < nseg_valid) v = p[(size_t)s * per] * fast_exp2(cpart[(size_t)bh * nseg + s] - cs);
    if (prefix) p[(size_t)s * per] = run;
    run += v;
  }
  if (!prefix) p[0] = run;
}

// ---------------------------------------------------------------------------------------------------
// Shared tail of the query-side kernels: exchange the partial Y^T tiles between the waves, normalise, store.
// y[it][vt] holds, for this wave's features, rows v = 16 vt + 4g + r and column token 16 it + c.
// ---------------------------------------------------------------------------------------------------
// Token tile `it` (compile-time) of this wave's partial result: kept if the wave owns the tile, else handed over.
__device__ __forceinline__ void exchange_put(Smem& sm, const f32x4 (&y)[NVT], int it, f32x4 (&own)[NVT]) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  if (it == w) {
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt) own[vt] = y[vt];
  } else {
    const int slot = w - (w > it ? 1 : 0);
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt) *(f32x4*)(&sm.xch[it][slot][c][16 * vt + 4 * g]) = y[vt];
  }
}

// After every tile has been put: add the other waves' parts of the owned tile, normalise by row v = 64, store.
__device__ __forceinline__ void exchange_finish(Smem& sm, f32x4 (&own)[NVT], const TensorDev& Y, long long ybase,
                                                int row0, int row_end) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  __syncthreads();
#pragma unroll
  for (int vt = 0; vt < NVT; ++vt) {
#pragma unroll
    for (int slot = 0; slot < NW - 1; ++slot) own[vt] += *(const f32x4*)(&sm.xch[w][slot][c][16 * vt + 4 * g]);
  }
  const float den = __shfl(own[NVT - 1][0], c);          // row v = 64 lives in lane (g = 0, c), register 0
  const float inv = den > 0.f ? 1.f / den : 0.f;
  const int token = row0 + 16 * w + c;
  if (token < row_end) {
    if (Y.dtype == 1) {
      uint16_t* yp = (uint16_t*)Y.ptr + ybase + (long long)token * Y.sl + 4 * g;
#pragma unroll
      for (int vt = 0; vt < 4; ++vt) {
        const f32x4 v = own[vt] * inv;
        typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
        *(bf16x4*)(yp + 16 * vt) = __builtin_convertvector(v, bf16x4);
      }
    } else {
      float* yp = (float*)Y.ptr + ybase + (long long)token * Y.sl + 4 * g;
#pragma unroll
      for (int vt = 0; vt < 4; ++vt) *(f32x4*)(yp + 16 * vt) = own[vt] * inv;
    }
  }
}

// ---------------------------------------------------------------------------------------------------
// Query side of the non-causal contraction: Y = (P T) normalised by its last column (Sections 2.1, 2.2) for a block
// of query rows; T = total state of the (b,h) (slot 0 of Tpart).  grid (nblk, B*H), block 256.
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(NT) k_fast_apply(FastArgs a, int Lq, int rows_per_blk) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  Smem& sm = *reinterpret_cast<Smem*>(smem_raw);
  const int blk = blockIdx.x, bh = blockIdx.y, b = bh / a.H, h = bh % a.H;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  const int pg = group_of(a.pgroups, b, h, a.H);
  const float wmax = a.bounds[((size_t)pg * 2) * 2], amax = a.bounds[((size_t)pg * 2) * 2 + 1];
  const uint16_t* Qb = (const uint16_t*)a.Q.ptr + b * a.Q.sb + h * a.Q.sh;
  const long long ybase = b * a.Y.sb + h * a.Y.sh;

  WaveConst wc;
  load_wave_const(wc, a.Wbf + ((size_t)pg * 2) * M * D, a.bias + ((size_t)pg * 2) * M);
  // T^T as A operand: row v = 16 vt + c, k <-> features 64w + 32 mb + 16 (e/4) + 4g + e%4
  bf16x8 tb[NVT][2];
  const float* Tg = a.Tpart + (size_t)bh * a.nseg * M * DVP;
#pragma unroll
  for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      f32x8 t;
#pragma unroll
      for (int e = 0; e < 8; ++e) t[e] = Tg[(size_t)(64 * w + 32 * mb + 16 * (e >> 2) + 4 * g + (e & 3)) * DVP + 16 * vt + c];
      tb[vt][mb] = __builtin_convertvector(t, bf16x8);
    }
  set_shift(wc, amax);
  const int row_beg = blk * rows_per_blk, row_end = min(Lq, row_beg + rows_per_blk);
  RowRegs qr;
  load_rows_g(qr, Qb, a.Q.sl, row_beg, row_end);
  store_rows_s(qr, sm.q[0], sm.nq2[0]);
  __syncthreads();
  int buf = 0;
  for (int row0 = row_beg; row0 < row_end; row0 += TC, buf ^= 1) {
    const bool more = row0 + TC < row_end;
    if (more) load_rows_g(qr, Qb, a.Q.sl, row0 + TC, row_end);
    f32x4 own[NVT];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      bf16x8 p[2];
      feature_tile(wc, sm.q[buf], it, -row_shift(sm.nq2[buf][16 * it + c], wmax), p);
      f32x4 y[NVT];
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) {
        y[vt] = mfma(tb[vt][0], p[0], f32x4{0.f, 0.f, 0.f, 0.f});
        y[vt] = mfma(tb[vt][1], p[1], y[vt]);
      }
      exchange_put(sm, y, it, own);
    }
    exchange_finish(sm, own, a.Y, ybase, row0, row_end);
    if (more) store_rows_s(qr, sm.q[buf ^ 1], sm.nq2[buf ^ 1]);
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------------------
// Causal contraction over one segment (64-token chunks), state seeded with the exclusive prefix of the segment
// states at the common shift c*:
//   Y_c = (tril(P_c S_c^T) [V_c 1] + P_c T_{c-1}) normalised by its last column;  T_c = T_{c-1} + S_c^T [V_c 1].
// grid (nseg, B*H), block 256.
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(NT) k_fast_causal(FastArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  Smem& sm = *reinterpret_cast<Smem*>(smem_raw);
  const int seg = blockIdx.x, bh = blockIdx.y, b = bh / a.H, h = bh % a.H;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  const int pg = group_of(a.pgroups, b, h, a.H);
  const float* th = a.theta + (size_t)group_of(a.groups, b, h, a.H) * (FS_THETA_HEADER_ + (size_t)D + 4 * (size_t)D * D);
  const bool isoC = ((int)th[2]) & 1;
  const float wmax1 = a.bounds[((size_t)pg * 2) * 2], amax1 = a.bounds[((size_t)pg * 2) * 2 + 1];
  const float wmax2 = a.bounds[((size_t)pg * 2 + 1) * 2], amax2 = a.bounds[((size_t)pg * 2 + 1) * 2 + 1];
  const uint16_t* Qb = (const uint16_t*)a.Q.ptr + b * a.Q.sb + h * a.Q.sh;
  const uint16_t* Kb = (const uint16_t*)a.K.ptr + b * a.K.sb + h * a.K.sh;
  const uint16_t* Vb = (const uint16_t*)a.V.ptr + b * a.V.sb + h * a.V.sh;
  const long long ybase = b * a.Y.sb + h * a.Y.sh;

  WaveConst wq, wk;
  load_wave_const(wq, a.Wbf + ((size_t)pg * 2) * M * D, a.bias + ((size_t)pg * 2) * M);
  load_wave_const(wk, a.Wbf + ((size_t)pg * 2 + 1) * M * D, a.bias + ((size_t)pg * 2 + 1) * M);
  float ck = a.cstar[bh];          // shift of the prefix state (-inf when there is none)
  set_shift(wk, ck);
  bf16x8 sel[2];
  make_sel(sel);
  zero_pad_rows(sm);
  f32x4 T[4][NVT];
  {
    const float* Tg = a.Tpart + ((size_t)bh * a.nseg + seg) * M * DVP;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
        for (int r = 0; r < 4; ++r) T[mt][vt][r] = Tg[(size_t)(64 * w + 16 * mt + 4 * g + r) * DVP + 16 * vt + c];
  }
  set_shift(wq, amax1);

  const int row_beg = seg * a.rows_per_seg, row_end = min(a.L, row_beg + a.rows_per_seg);
  RowRegs qr, kr, vr;
  load_rows_g(qr, Qb, a.Q.sl, row_beg, row_end);
  load_rows_g(kr, Kb, a.K.sl, row_beg, row_end);
  load_vals_g(vr, Vb, a.V.sl, row_beg, row_end);
  store_rows_s(qr, sm.q[0], sm.nq2[0]);
  store_rows_s(kr, sm.k[0], sm.nk2[0]);
  store_vals_s(vr, sm.vt[0], row_beg, row_end);
  __syncthreads();

  int buf = 0;
  for (int row0 = row_beg; row0 < row_end; row0 += TC, buf ^= 1) {
    const bool more = row0 + TC < row_end;
    if (more) {
      load_rows_g(qr, Qb, a.Q.sl, row0 + TC, row_end);
      load_rows_g(kr, Kb, a.K.sl, row0 + TC, row_end);
      load_vals_g(vr, Vb, a.V.sl, row0 + TC, row_end);
    }
    const float cknew = key_chunk_bound(a, isoC, bh, row0, row_end, sm.nk2[buf], wmax2, amax2);
    if (cknew > ck) {              // keys of this chunk may exceed the running shift: rebase the state
      const float f = fast_exp2(ck - cknew);
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt) T[mt][vt] *= f;
      ck = cknew;
      set_shift(wk, ck);
    }

    // key side: S (operand layout for the scores) and S^T (operand layout for the state update)
    bf16x8 s[4][2], st[4][2];
#pragma unroll
    for (int jp = 0; jp < 2; ++jp) {
      f32x4 tr[2][4];
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const int jt = 2 * jp + jj, tok = row0 + 16 * jt + c;
        const float add = key_rowterm(a, isoC, bh, tok, sm.nk2[buf][16 * jt + c], tok < row_end);
        feature_tile(wk, sm.k[buf], jt, add, s[jt]);
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int hh = 0; hh < 2; ++hh)
            tr[jj][2 * mb + hh] = mfma(s[jt][mb], sel[hh], f32x4{0.f, 0.f, 0.f, 0.f});
      }
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) st[mt][jp] = pack8(tr[0][mt], tr[1][mt]);
    }
    // state before this chunk as A operand (T^T: row v, k <-> feature)
    bf16x8 tb[NVT][2];
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) tb[vt][mb] = pack8(T[2 * mb][vt], T[2 * mb + 1][vt]);
    bf16x8 vop[2][NVT];
#pragma unroll
    for (int jp = 0; jp < 2; ++jp)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) vop[jp][vt] = load_vop(sm.vt[buf], jp, vt);

    f32x4 own[NVT];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      bf16x8 p[2];
      feature_tile(wq, sm.q[buf], it, -row_shift(sm.nq2[buf][16 * it + c], wmax1), p);
      f32x4 y[NVT];
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) {
        y[vt] = mfma(tb[vt][0], p[0], f32x4{0.f, 0.f, 0.f, 0.f});
        y[vt] = mfma(tb[vt][1], p[1], y[vt]);
      }
      // scores^T tiles (rows = keys 16 jt + 4g + r, column = query 16 it + c), keys of later tiles are masked out
      f32x4 sc[4];
#pragma unroll
      for (int jt = 0; jt < 4; ++jt) {
        sc[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (jt <= it) {
          sc[jt] = mfma(s[jt][0], p[0], sc[jt]);
          sc[jt] = mfma(s[jt][1], p[1], sc[jt]);
          if (jt == it) {
#pragma unroll
            for (int r = 0; r < 4; ++r) sc[jt][r] = (4 * g + r <= c) ? sc[jt][r] : 0.f;
          }
        }
      }
#pragma unroll
      for (int jp = 0; jp < 2; ++jp) {
        if (2 * jp <= it) {
          const bf16x8 sb = pack8(sc[2 * jp], sc[2 * jp + 1]);
#pragma unroll
          for (int vt = 0; vt < NVT; ++vt) y[vt] = mfma(vop[jp][vt], sb, y[vt]);
        }
      }
      exchange_put(sm, y, it, own);
    }
    // state update
#pragma unroll
    for (int jp = 0; jp < 2; ++jp)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) T[mt][vt] = mfma(st[mt][jp], vop[jp][vt], T[mt][vt]);

    exchange_finish(sm, own, a.Y, ybase, row0, row_end);
    if (more) {
      store_rows_s(qr, sm.q[buf ^ 1], sm.nq2[buf ^ 1]);
      store_rows_s(kr, sm.k[buf ^ 1], sm.nk2[buf ^ 1]);
      store_vals_s(vr, sm.vt[buf ^ 1], row0 + TC, row_end);
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------------
#define FS_LAUNCH_CHECK() do { if (hipGetLastError() != hipSuccess) return 5; } while (0)

size_t fast_lds_bytes() { return sizeof(Smem); }

bool fast_supported(int dtype, int d, int dv, int M_) { return dtype == 1 && d == D && dv == D && M_ == M; }

void fast_plan(int BH, int L, int* nseg, int* rows_per_seg) {
  int want = std::max(1, std::min((256 + BH - 1) / BH, (L + TC - 1) / TC));
  *rows_per_seg = (((L + want - 1) / want) + TC - 1) / TC * TC;
  *nseg = (L + *rows_per_seg - 1) / *rows_per_seg;
}

static int set_fast_lds(const void* fn) {
  if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(Smem)) != hipSuccess) {
    (void)hipGetLastError();
    return 2;
  }
  return 0;
}

int launch_fast_attention(const FastLaunch& f, hipStream_t st, hipEvent_t ev_begin, hipEvent_t ev_end) {
  FastArgs a;
  a.Q = f.Q; a.K = f.K; a.V = f.V; a.Y = f.Y;
  a.Wbf = f.Wbf; a.bias = f.bias; a.bounds = f.bounds; a.theta = f.theta; a.rk = f.rk;
  a.Tpart = f.Tpart; a.cpart = f.cpart; a.cstar = f.cstar;
  a.groups = f.groups; a.pgroups = f.pgroups; a.H = f.H; a.L = f.Lk; a.rows_per_seg = f.rows_per_seg; a.nseg = f.nseg;
  a.scale = f.scale;
  const int BH = f.B * f.H;
  hipLaunchKernelGGL(k_fast_prep, dim3(2, f.pgroups), dim3(256), 0, st, f.theta, f.groups, f.Omega, f.omega_groups,
                     f.pgroups, f.B, f.H, f.scale, f.Wbf, f.bias, f.bounds);
  FS_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_fast_rowterm, dim3((f.Lk + 255) / 256, BH), dim3(256), 0, st, f.K, f.Lk, f.H, f.theta, f.groups,
                     f.scale, f.rk);
  FS_LAUNCH_CHECK();
  if (int rc = set_fast_lds((const void*)k_fast_state)) return rc;
  if (int rc = set_fast_lds((const void*)k_fast_apply)) return rc;
  if (int rc = set_fast_lds((const void*)k_fast_causal)) return rc;
  // the last segment's state is never needed by the causal pass
  const int nstate = f.causal ? f.nseg - 1 : f.nseg;
  if (nstate > 0) {
    hipLaunchKernelGGL(k_fast_state, dim3(nstate, BH), dim3(NT), sizeof(Smem), st, a);
    FS_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(k_fast_reduce, dim3((M * DVP + 255) / 256, BH), dim3(256), 0, st, f.Tpart, f.cpart, f.cstar,
                     f.nseg, nstate, f.causal);
  FS_LAUNCH_CHECK();
  if (ev_begin && hipEventRecord(ev_begin, st) != hipSuccess) return 5;
  if (f.causal) {
    hipLaunchKernelGGL(k_fast_causal, dim3(f.nseg, BH), dim3(NT), sizeof(Smem), st, a);
  } else {
    int nblk, rows_per_blk;
    fast_plan(BH, f.Lq, &nblk, &rows_per_blk);
    hipLaunchKernelGGL(k_fast_apply, dim3(nblk, BH), dim3(NT), sizeof(Smem), st, a, f.Lq, rows_per_blk);
  }
  FS_LAUNCH_CHECK();
  if (ev_end && hipEventRecord(ev_end, st) != hipSuccess) return 5;
  return 0;
}

}  // namespace fs
