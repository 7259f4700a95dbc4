// Backward pass of causal attention on the bf16 path (d = dv = 64, M = 256); see kernels_bf16_bwd.hip for the
// non-causal variant and the notation.  With T_i the prefix state (keys j <= i) and R_j the suffix sum
// sum_{i >= j} P_i^T G1_i, per chunk c of 64 tokens (A = tril(G1_c V1_c^T), B = tril(P_c S_c^T)):
//   dP_c  = G1_c T_{c-1}^T + A S_c               dV1_c = S_c R_{c+1} + B^T G1_c
//   dS_c  = V1_c R_{c+1}^T + A^T P_c
// Every kernel walks one slot (a run of whole chunks) of one sequence; the key features use ONE shift per sequence
// (the largest bound over all its tokens) so that the states of different slots, G1 and the gradients all live on
// one scale.  One call:
//   k_bwd_walk_pc<0>   forward walk: Yhat, normaliser, Y, G1 rows             (T from the exclusive prefix per slot)
//   k_bwd_rstate       (kernels_bf16_bwd.hip) per-slot sums of P^T G1;  k_bwd_suffix  their exclusive suffix
//   k_bwd_walk_pc<1>   backward walk: dV
//   k_bwd_cgrad_pc<0>  forward walk: dQ;   k_bwd_cgrad_pc<1>  backward walk: dK
//
// ---- gradient rows dQ and dK: one kernel template, the two sides being mirror images of each other ----------------
//
// Per chunk of 64 tokens, with F the feature matrix of a side (P for queries, S for keys), U the 80-column rows that
// go with it (G1 = [dY / den, -(dY . Y) / den] for queries, V1 = [V 1] for keys) and Z the running state built from
// the OTHER side (KEY = 0, forward walk: Z = sum over earlier keys of S^T V1; KEY = 1, backward walk: Z = sum over
// later queries of P^T G1):
//   dF_own = U_own Z^T + mask(U_own U_oth^T) F_oth        (mask: other token not after / not before the own token)
//   grad   = ln2 (F_own * dF_own) W~_own  (+ the key row term)
//   Z     += F_oth^T U_oth
// Z is kept TRANSPOSED in the accumulators (rows = U columns, lane <-> feature), so that its bf16 image is directly
// the MFMA operand of U_own Z^T and no register transposes are needed anywhere.
//
// Eight waves: producers 0..3 and consumers 4..7; producer j and consumer j share a SIMD and the features
// [64j, 64j + 64).  A chunk is four steps with one workgroup barrier each; the consumers run one step behind.
//   producer, step 0/1: feature tiles of the other side for token tiles (0,1) / (2,3), feature-major (lane <->
//             feature, contraction index <-> tokens; the projection MFMA with the operands swapped);
//             step 2/3: feature tiles of the own side, token-major.  Beside that: staging of the rows (global ->
//             registers a chunk ahead -> LDS), the masked 64 x 64 products U_oth U_own^T as operand images, and one
//             chunk later the sum of the consumers' partial gradient tiles (MFMA against a routing matrix), the key
//             row term and the store.
//   consumer, step 0/1: state update with the previous chunk's tiles, then the new feature-major tiles into registers;
//             step 2/3: dF tiles, the product with the own features, the contraction with W~^T and the partial
//             tiles to LDS.
// LDS lifetimes (interval t = 4 (chunk index) + step; the consumer's step s runs in interval 4c + s + 1):
//   xoth (rows of the other side)   written in step 2 for the next chunk, read in steps 3 and 0
//   xown (two buffers)              written in step 0, read in steps 1 and 2 and, for the keys' row term, in step 1
//                                   of the next chunk
//   uown, uoth (U rows)             written in step 1, read by the producers in step 2 and by the consumers in their
//                                   steps 2 and 3 (intervals 4c+3, 4c+4; the next write is in 4c+5)
//   uothT (U_oth transposed)        written in step 3, read by the consumers' state update in intervals 4c+5, 4c+6
//   ab (mask products)              written in step 2, read in intervals 4c+3 and 4c+4
//   xch (partial tiles)             written in intervals 4c+3 and 4c+4, summed in step 1 of the next chunk (4c+5)
#include <type_traits>

#include "fast_bwd.h"
#include "fast_pc.h"

namespace fs {

using namespace fast;

namespace cg {

using namespace pc;
using bwd::BwdArgs;

constexpr int LDU = 96 + 8;        // row stride (bf16) of the U rows: 52 dwords, conflict-free 16-byte reads

struct SmemCG {
  __attribute__((aligned(16))) uint16_t xoth[TC][LDR];
  __attribute__((aligned(16))) uint16_t xown[2][TC][LDR];     // by chunk parity: the keys' row term needs them a chunk later
  // U rows, 96 columns (80.. are zero) in the order of two stacked accumulator tiles: column v sits at
  // 32 (v/32) + 8 ((v%16)/4) + 4 ((v%32)/16) + v%4, so that 16 bytes at [32 kk + 8g] are one MFMA operand that pairs
  // with the bf16 image of the state
  __attribute__((aligned(16))) uint16_t uown[TC][LDU];
  __attribute__((aligned(16))) uint16_t uoth[TC][LDU];
  __attribute__((aligned(16))) uint16_t uothT[DVP][LDJ];      // [column][token]
  __attribute__((aligned(16))) float add_oth[TC];             // what is added to the exponents of a token (-inf past the end)
  __attribute__((aligned(16))) float add_own[TC];
  __attribute__((aligned(16))) uint16_t feat[2][4][4][64][8]; // register images: [slot][image of the step][pair][lane]
  __attribute__((aligned(16))) uint16_t ab[6][64][8];         // mask products as operand images
  __attribute__((aligned(16))) uint16_t xch[4][4][16][LDXB];  // partial gradient tiles: [token tile][pair][token][column]
  // C2 + C2^T as A operands of the keys' row term when C2 is dense: [16-row tile][k-step][lane] (rows = gradient columns)
  __attribute__((aligned(16))) uint16_t csym[4][KS][64][8];
};

__device__ __forceinline__ int upos(int v) { return 32 * (v / 32) + 8 * ((v % 16) / 4) + 4 * ((v % 32) / 16) + v % 4; }

struct Ctx {
  const uint16_t *Qb, *Kb, *Vb, *Gb;
  int bh, pg, row_beg, row_end, nchunk;
  bool isoC;
  float cs;
};

template <int KEY>
__device__ __forceinline__ int chunk_row(const Ctx& cx, int ci) {
  if (ci >= cx.nchunk) return cx.row_beg;
  return cx.row_beg + (KEY ? cx.nchunk - 1 - ci : ci) * TC;
}
template <int KEY>
__device__ __forceinline__ int chunk_rows(const Ctx& cx, int ci) {
  if (ci < 0 || ci >= cx.nchunk) return 0;
  return min(TC, cx.row_end - chunk_row<KEY>(cx, ci));
}

// Staging registers of the 256 producer threads: two 16-byte pieces of the rows of each side (rows tid/8 and
// tid/8 + 32, bytes 16 (tid%8)), two of the value rows and three of the G1 rows (token tid%64, pieces tid/64 + 4i).
struct StageG { u32x4 xo[2], xw[2], v[2], g[3]; float rko[2], rkw[2]; };   // rk: row terms of the key rows (dense C2)

template <int KEY>
__device__ __forceinline__ void load_x(u32x4 (&p)[2], float (&rk)[2], bool with_rk, const uint16_t* base, long long sl,
                                       const FastArgs& a, const Ctx& cx, int ci, int tid) {
  const int r0 = chunk_row<KEY>(cx, ci), nv = chunk_rows<KEY>(cx, ci);
  const __amdgpu_buffer_rsrc_t rs = chunk_rsrc(base + (long long)r0 * sl, 2 * (int)sl, nv, 2 * D);
  const __amdgpu_buffer_rsrc_t rr = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.rk + (size_t)cx.bh * a.L + r0), 0,
                                                                      (with_rk && !cx.isoC) ? 4 * nv : 0, 0x00020000);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int row = (tid >> 3) + 32 * i;
    p[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, 2 * (row * (int)sl + (tid & 7) * 8), 0, 0);
    if (with_rk) rk[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rr, 4 * row, 0, 0));
  }
}

template <int KEY>
__device__ __forceinline__ void load_u(StageG& s, const FastArgs& a, const Ctx& cx, int ci, int tid) {
  const int r0 = chunk_row<KEY>(cx, ci), nv = chunk_rows<KEY>(cx, ci);
  const __amdgpu_buffer_rsrc_t rv = chunk_rsrc(cx.Vb + (long long)r0 * a.V.sl, 2 * (int)a.V.sl, nv, 2 * D);
  const __amdgpu_buffer_rsrc_t rg = chunk_rsrc(cx.Gb + (long long)r0 * DVP, 2 * DVP, nv, 2 * DVP);
  const int j = tid & 63, pv = tid >> 6;
#pragma unroll
  for (int i = 0; i < 2; ++i) s.v[i] = __builtin_amdgcn_raw_buffer_load_b128(rv, 2 * (j * (int)a.V.sl + (pv + 4 * i) * 8), 0, 0);
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    s.g[i] = u32x4{0u, 0u, 0u, 0u};
    if (pv + 4 * i < DVP / 8) s.g[i] = __builtin_amdgcn_raw_buffer_load_b128(rg, 2 * (j * DVP + (pv + 4 * i) * 8), 0, 0);
  }
}

// Rows of one side to LDS with the per-token exponent term.  `key_side`: row term - sequence shift, else - row shift.
__device__ __forceinline__ void store_x(const u32x4 (&p)[2], const float (&rk)[2], bool key_side, uint16_t (*tile)[LDR],
                                        float* add, const FastArgs& a, const Ctx& cx, int nv, float wmax, int tid) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int row = (tid >> 3) + 32 * i;
    const float n2 = store_row_piece(p[i], tile, row, tid & 7);
    float t;
    if (key_side) t = (cx.isoC ? -0.5f * kLog2e * a.scale * a.scale * n2 : rk[i]) - cx.cs;
    else t = -row_shift(n2, wmax);
    add[row] = row < nv ? t : -INFINITY;      // the eight lanes of a row write the same word
  }
}

// One 16-byte piece (columns 8 pc ..) of a U row in the stacked order.
__device__ __forceinline__ void store_u_piece(u32x4 p, uint16_t (*rows)[LDU], int j, int pc) {
  *(u32x2*)(&rows[j][upos(8 * pc)]) = u32x2{p[0], p[1]};
  *(u32x2*)(&rows[j][upos(8 * pc + 4)]) = u32x2{p[2], p[3]};
}

template <int KEY>
__device__ __forceinline__ void store_u_rows(const StageG& s, SmemCG& sm, int nv, int tid) {
  uint16_t (*vrows)[LDU] = KEY ? sm.uown : sm.uoth;
  uint16_t (*grows)[LDU] = KEY ? sm.uoth : sm.uown;
  const int j = tid & 63, pv = tid >> 6;
#pragma unroll
  for (int i = 0; i < 2; ++i) store_u_piece(s.v[i], vrows, j, pv + 4 * i);
  if (pv == 0) *(u32x2*)(&vrows[j][upos(D)]) = u32x2{j < nv ? 0x3f80u : 0u, 0u};     // the ones column
#pragma unroll
  for (int i = 0; i < 3; ++i)
    if (pv + 4 * i < DVP / 8) store_u_piece(s.g[i], grows, j, pv + 4 * i);
}

template <int KEY, class SM>
__device__ __forceinline__ void store_u_transposed(const StageG& s, SM& sm, int nv, int tid) {
  const int j = tid & 63, pv = tid >> 6;
  if (KEY) {
#pragma unroll
    for (int i = 0; i < 3; ++i)
      if (pv + 4 * i < DVP / 8) store_val_piece(s.g[i], sm.uothT, j, pv + 4 * i);
  } else {
#pragma unroll
    for (int i = 0; i < 2; ++i) store_val_piece(s.v[i], sm.uothT, j, pv + 4 * i);
    if (tid < 32) {
      const int t0 = 2 * tid;
      *(uint32_t*)(&sm.uothT[D][t0]) = (t0 < nv ? 0x3f80u : 0u) | (t0 + 1 < nv ? 0x3f80u << 16 : 0u);
    }
  }
}

__device__ __forceinline__ bf16x8 urow_op(const uint16_t (*rows)[LDU], int tile, int kk, int lane) {
  return *(const bf16x8*)(&rows[16 * tile + (lane & 15)][32 * kk + 8 * (lane >> 4)]);
}

// Index of the mask-product image of own token tile t and other-side tile pair `pair`.
template <int KEY>
__device__ __forceinline__ constexpr int ab_index(int t, int pair) {
  return KEY ? (t < 2 ? 2 * t + pair : 2 + t) : (t < 2 ? t : 2 + 2 * (t - 2) + pair);
}

// Mask product of own token tile t with the pair of other-side tiles (2 pair, 2 pair + 1): accumulator rows = other
// tokens, column = own token, entries outside the causal mask zeroed, as B operand of the contraction over the
// pair's 32 tokens.
template <int KEY>
__device__ __forceinline__ void mask_image(SmemCG& sm, int t, int pair, int lane) {
  const int g = lane >> 4, c = lane & 15;
  f32x4 ac[2];
#pragma unroll
  for (int uu = 0; uu < 2; ++uu) {
    const int ot = 2 * pair + uu;
    ac[uu] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (KEY ? ot >= t : ot <= t) {
#pragma unroll
      for (int kk = 0; kk < 3; ++kk) ac[uu] = mfma(urow_op(sm.uoth, ot, kk, lane), urow_op(sm.uown, t, kk, lane), ac[uu]);
      if (ot == t) {
#pragma unroll
        for (int r = 0; r < 4; ++r) ac[uu][r] = (KEY ? 4 * g + r >= c : 4 * g + r <= c) ? ac[uu][r] : 0.f;
      }
    }
  }
  *(bf16x8*)(&sm.ab[ab_index<KEY>(t, pair)][lane][0]) = pack8(ac[0], ac[1]);
}

// Feature-major images of a pair of token tiles: img[mt] has lane <-> feature 64j + 16mt + c and contraction index
// <-> the pair's tokens {4g + r, 16 + 4g + r}.  addv[u][r]: exponent term of token 16 (tile u) + 4g + r.
template <bool WITH_BIAS>
__device__ __forceinline__ void feature_pair_t(const W64& ws, const float (&bq)[4], const XOp (&x)[2], const f32x4 (&addv)[2],
                                               bf16x8 (&img)[4]) {
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
    f32x4 acc[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      acc[u] = mfma(x[u].b[0], ws.w[mt][0], WITH_BIAS ? addv[u] + bq[mt] : addv[u]);
#pragma unroll
      for (int ks = 1; ks < KS; ++ks) acc[u] = mfma(x[u].b[ks], ws.w[mt][ks], acc[u]);
    }
    img[mt] = pack8(exp2v(acc[0]), exp2v(acc[1]));
  }
}

template <int KEY>
__device__ __forceinline__ void producer(const BwdArgs& ba, SmemCG& sm, const Ctx& cx, int j) {
  const FastArgs& a = ba.f;
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 4, c = lane & 15;
  const TensorDev& G = KEY ? ba.dK : ba.dQ;
  const uint16_t* Xown = KEY ? cx.Kb : cx.Qb;
  const uint16_t* Xoth = KEY ? cx.Qb : cx.Kb;
  const long long sl_own = KEY ? a.K.sl : a.Q.sl, sl_oth = KEY ? a.Q.sl : a.K.sl;
  const float wmaxq = max256(a.wnorm + ((size_t)cx.pg * 2) * M), amax = max256(a.bias + ((size_t)cx.pg * 2) * M);

  W64 wq, wk;
  load_w64(wq, a.Wbf + ((size_t)cx.pg * 2) * M * D, j, lane);
  load_w64(wk, a.Wbf + ((size_t)cx.pg * 2 + 1) * M * D, j, lane);
  const W64& wown = KEY ? wk : wq;
  const W64& woth = KEY ? wq : wk;
  B64 qb;            // bias of the query features, token-major tiles (KEY = 0)
  float bq[4];       // ditto, feature-major tiles (KEY = 1)
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
    for (int r = 0; r < 4; ++r) qb.b[mt][r] = 2.f * (a.bias[((size_t)cx.pg * 2) * M + 64 * j + 16 * mt + 4 * g + r] - amax);
    bq[mt] = 2.f * (a.bias[((size_t)cx.pg * 2) * M + 64 * j + 16 * mt + c] - amax);
  }

  // first chunk: rows of the other side to LDS; the rest of it waits in the staging registers
  StageG stg;
  stg.rko[0] = stg.rko[1] = stg.rkw[0] = stg.rkw[1] = 0.f;
  load_x<KEY>(stg.xo, stg.rko, !KEY, Xoth, sl_oth, a, cx, 0, tid);
  store_x(stg.xo, stg.rko, !KEY, sm.xoth, sm.add_oth, a, cx, chunk_rows<KEY>(cx, 0), wmaxq, tid);
  load_x<KEY>(stg.xo, stg.rko, !KEY, Xoth, sl_oth, a, cx, 1, tid);
  load_x<KEY>(stg.xw, stg.rkw, KEY, Xown, sl_own, a, cx, 0, tid);
  load_u<KEY>(stg, a, cx, 0, tid);
  __syncthreads();                 // barrier 0

  XOp xo[2][2];                    // [step parity][tile of the step]
  load_xop(xo[0][0], sm.xoth, 0, lane);
  load_xop(xo[0][1], sm.xoth, 1, lane);

  // sum of the four partial tiles of token tile j of a finished chunk, row term, store
  auto finish = [&](int ci_done) {
    f32x4 fsum[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) fsum[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    finish_tiles(fsum, sm, j, 0, lane);
    finish_tiles(fsum, sm, j, 2, lane);
    if (KEY) {
      const float rs = finish_col64(sm, j, lane) * a.scale * a.scale;
      // row term rs (C2 + C2^T) k from the chunk's key rows (still in their LDS buffer)
      const uint16_t (*krows)[LDR] = sm.xown[ci_done & 1];
      if (cx.isoC) {
        // C2 + C2^T = -identity (the factor is in rs)
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const bf16x4 kb = *(const bf16x4*)(&krows[16 * j + c][16 * dt + 4 * g]);
          fsum[dt] = kLn2 * fsum[dt] - rs * __builtin_convertvector(kb, f32x4);
        }
      } else {
        // dense: the matrix as A operand (rows = gradient columns), the key rows as B operand
        XOp kop;
        load_xop(kop, krows, j, lane);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          f32x4 u = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) u = mfma(*(const bf16x8*)(&sm.csym[dt][ks][lane][0]), kop.b[ks], u);
          fsum[dt] = kLn2 * fsum[dt] + rs * u;
        }
      }
    } else {
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) fsum[dt] *= kLn2;
    }
    const int esz = G.dtype == 1 ? 2 : 4;
    const char* gp = (const char*)G.ptr + ((cx.bh / a.H) * G.sb + (cx.bh % a.H) * G.sh + (long long)chunk_row<KEY>(cx, ci_done) * G.sl) * esz;
    finish_store(fsum, G, gp, chunk_rows<KEY>(cx, ci_done), j, lane);
  };

  for (int ci = 0; ci < cx.nchunk; ++ci) {
    const int nv = chunk_rows<KEY>(cx, ci);
#pragma unroll
    for (int S = 0; S < 4; ++S) {
      // operands of the next step
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        if (S == 0) load_xop(xo[1][u], sm.xoth, 2 + u, lane);
        else if (S == 1) load_xop(xo[0][u], sm.xown[ci & 1], u, lane);
        else if (S == 2) load_xop(xo[1][u], sm.xown[ci & 1], 2 + u, lane);
        else load_xop(xo[0][u], sm.xoth, u, lane);
      }
      __builtin_amdgcn_sched_barrier(0);

      if (S < 2) {
        bf16x8 img[4];
        const f32x4 addv[2] = {*(const f32x4*)(&sm.add_oth[16 * (2 * S) + 4 * g]), *(const f32x4*)(&sm.add_oth[16 * (2 * S + 1) + 4 * g])};
        feature_pair_t<KEY != 0>(woth, bq, xo[S & 1], addv, img);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) *(bf16x8*)(&sm.feat[S & 1][mt][j][lane][0]) = img[mt];
      } else {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          bf16x8 img[2];
          feature_tile64<KEY == 0>(wown, &qb, xo[S & 1][u], sm.add_own[16 * (2 * (S - 2) + u) + c], img);
#pragma unroll
          for (int blk = 0; blk < 2; ++blk) *(bf16x8*)(&sm.feat[S & 1][2 * u + blk][j][lane][0]) = img[blk];
        }
      }

      if (S == 0) {
        store_x(stg.xw, stg.rkw, KEY, sm.xown[ci & 1], sm.add_own, a, cx, nv, wmaxq, tid);
        load_x<KEY>(stg.xw, stg.rkw, KEY, Xown, sl_own, a, cx, ci + 1, tid);
      } else if (S == 1) {
        store_u_rows<KEY>(stg, sm, nv, tid);
        if (ci > 0) finish(ci - 1);
      } else if (S == 2) {
        store_x(stg.xo, stg.rko, !KEY, sm.xoth, sm.add_oth, a, cx, chunk_rows<KEY>(cx, ci + 1), wmaxq, tid);
        load_x<KEY>(stg.xo, stg.rko, !KEY, Xoth, sl_oth, a, cx, ci + 2, tid);
        // mask products, spread over the four producers
        if (KEY) {
          if (j == 0) mask_image<KEY>(sm, 0, 0, lane);
          else if (j == 1) mask_image<KEY>(sm, 0, 1, lane);
          else if (j == 2) { mask_image<KEY>(sm, 1, 0, lane); mask_image<KEY>(sm, 2, 1, lane); }
          else { mask_image<KEY>(sm, 1, 1, lane); mask_image<KEY>(sm, 3, 1, lane); }
        } else {
          if (j == 0) { mask_image<KEY>(sm, 0, 0, lane); mask_image<KEY>(sm, 3, 1, lane); }
          else if (j == 1) mask_image<KEY>(sm, 1, 0, lane);
          else if (j == 2) { mask_image<KEY>(sm, 2, 0, lane); mask_image<KEY>(sm, 2, 1, lane); }
          else mask_image<KEY>(sm, 3, 0, lane);
        }
      } else {
        store_u_transposed<KEY>(stg, sm, nv, tid);
        load_u<KEY>(stg, a, cx, ci + 1, tid);
      }
      __syncthreads();
    }
  }
  __syncthreads();                 // the consumers' last step
  if (cx.nchunk > 0) finish(cx.nchunk - 1);
}

template <int KEY>
__device__ __forceinline__ void consumer(const BwdArgs& ba, SmemCG& sm, const Ctx& cx, int slot, int j) {
  const FastArgs& a = ba.f;
  const int lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
  // state, transposed: Zt[vt][mt] has rows = U columns 16 vt + 4g + r, lane <-> feature 64j + 16 mt + c
  f32x4 Zt[NVT][4];
  {
    // (single slot per sequence: neither a prefix nor a suffix was computed; every workgroup reads one block of zeros)
    const float* Zg = ba.zero_state != nullptr ? ba.zero_state
                                               : (KEY ? ba.Rpart : a.Tpart) + ((size_t)cx.bh * a.nslot + slot) * M * DVP;
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) Zt[vt][mt] = *(const f32x4*)(Zg + (size_t)(64 * j + 16 * mt + c) * DVP + 16 * vt + 4 * g);
  }
  // W~^T of the own side as A operand of the gradient tile (rows = the 64 columns; for the keys a row of ones is
  // appended: the row sum of the feature gradient)
  const uint16_t* Wg = a.Wbf + ((size_t)cx.pg * 2 + KEY) * M * D;
  bf16x8 wt[NVT][2];
#pragma unroll
  for (int dt = 0; dt < NVT; ++dt)
#pragma unroll
    for (int bk = 0; bk < 2; ++bk) {
      u32x4 v = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int f = 64 * j + 32 * bk + 16 * (e >> 2) + 4 * g + (e & 3);
        uint32_t bits;
        if (dt < 4) bits = Wg[(size_t)f * D + 16 * dt + c];
        else bits = c == 0 ? 0x3f80u : 0u;
        v[e >> 1] |= bits << (16 * (e & 1));
      }
      wt[dt][bk] = __builtin_bit_cast(bf16x8, v);
    }
  __syncthreads();                 // barrier 0
  __syncthreads();                 // the producers' first step

  bf16x8 st[4][2];                 // feature-major tiles of the other side: [feature tile][token pair]
  for (int ci = 0; ci < cx.nchunk; ++ci) {
#pragma unroll
    for (int S = 0; S < 4; ++S) {
      if (S < 2) {
        if (ci > 0) {
          // the state takes the previous chunk's tokens, one pair of token tiles per step (the pair whose registers
          // are refilled next)
#pragma unroll
          for (int vt = 0; vt < NVT; ++vt) {
            const bf16x8 uop = load_vop_l(sm.uothT, S, vt, lane);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) Zt[vt][mt] = mfma(uop, st[mt][S], Zt[vt][mt]);
          }
        }
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) st[mt][S] = *(const bf16x8*)(&sm.feat[S & 1][mt][j][lane][0]);
      } else {
        // state as A operand: rows = features 16 mt + c, contraction index <-> U columns in the stacked order
        bf16x8 sa[4][3];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
          sa[mt][0] = pack8(Zt[0][mt], Zt[1][mt]);
          sa[mt][1] = pack8(Zt[2][mt], Zt[3][mt]);
          sa[mt][2] = pack8(Zt[4][mt], f32x4{0.f, 0.f, 0.f, 0.f});
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int t = 2 * (S - 2) + u;
          bf16x8 p[2];
#pragma unroll
          for (int blk = 0; blk < 2; ++blk) p[blk] = *(const bf16x8*)(&sm.feat[S & 1][2 * u + blk][j][lane][0]);
          f32x4 df[4] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
          for (int kk = 0; kk < 3; ++kk) {
            const bf16x8 uop = urow_op(sm.uown, t, kk, lane);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) df[mt] = mfma(sa[mt][kk], uop, df[mt]);
          }
#pragma unroll
          for (int pair = 0; pair < 2; ++pair) {
            if (KEY ? 2 * pair + 1 >= t : 2 * pair <= t) {
              const bf16x8 ab = *(const bf16x8*)(&sm.ab[ab_index<KEY>(t, pair)][lane][0]);
#pragma unroll
              for (int mt = 0; mt < 4; ++mt) df[mt] = mfma(st[mt][pair], ab, df[mt]);
            }
          }
          bf16x8 eimg[2];
#pragma unroll
          for (int bk = 0; bk < 2; ++bk) {
            const f32x8 fv = __builtin_convertvector(p[bk], f32x8);
            const f32x4 lo = {fv[0] * df[2 * bk][0], fv[1] * df[2 * bk][1], fv[2] * df[2 * bk][2], fv[3] * df[2 * bk][3]};
            const f32x4 hi = {fv[4] * df[2 * bk + 1][0], fv[5] * df[2 * bk + 1][1], fv[6] * df[2 * bk + 1][2], fv[7] * df[2 * bk + 1][3]};
            eimg[bk] = pack8(lo, hi);
          }
          f32x4 gtile[NVT];
#pragma unroll
          for (int dt = 0; dt < NVT; ++dt) {
            if (dt < 4 || KEY) {
              gtile[dt] = mfma(wt[dt][0], eimg[0], f32x4{0.f, 0.f, 0.f, 0.f});
              gtile[dt] = mfma(wt[dt][1], eimg[1], gtile[dt]);
            } else {
              gtile[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
          }
          exchange_put_bf16(sm, gtile, t, j, lane);
        }
      }
      __syncthreads();
    }
  }
}

// grid (nslot, B*H), block 512.
template <int KEY>
__global__ void __launch_bounds__(NT8) k_bwd_cgrad_pc(BwdArgs ba) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  SmemCG& sm = *reinterpret_cast<SmemCG*>(smem_raw);
  const FastArgs& a = ba.f;
  const int slot = blockIdx.x, bh = blockIdx.y, b = bh / a.H, h = bh % a.H;
  const float* th = a.theta + (size_t)group_of(a.groups, b, h, a.H) * (FS_THETA_HEADER_ + (size_t)D + 4 * (size_t)D * D);
  Ctx cx;
  cx.isoC = ((int)th[2]) & 1;
  cx.bh = bh;
  cx.pg = group_of(a.pgroups, b, h, a.H);
  cx.cs = a.cstar[bh];
  cx.Qb = (const uint16_t*)a.Q.ptr + b * a.Q.sb + h * a.Q.sh;
  cx.Kb = (const uint16_t*)a.K.ptr + b * a.K.sb + h * a.K.sh;
  cx.Vb = (const uint16_t*)a.V.ptr + b * a.V.sb + h * a.V.sh;
  cx.Gb = ba.gh + (size_t)bh * ba.Lq * DVP;
  cx.row_beg = min(ba.Lq, slot * ba.rows_per_rslot);
  cx.row_end = min(ba.Lq, cx.row_beg + ba.rows_per_rslot);
  cx.nchunk = (cx.row_end - cx.row_beg + TC - 1) / TC;
  // the staging writes columns 0..79 of the U rows and, of the value columns, rows 0..64 of the transposed tile
  for (int idx = threadIdx.x; idx < TC * LDU / 2; idx += NT8) {
    ((uint32_t*)&sm.uown[0][0])[idx] = 0u;
    ((uint32_t*)&sm.uoth[0][0])[idx] = 0u;
  }
  for (int idx = threadIdx.x; idx < DVP * LDJ / 2; idx += NT8) ((uint32_t*)&sm.uothT[0][0])[idx] = 0u;
  if (KEY && !cx.isoC) {
    // one operand piece per thread
    const float* C2 = th + FS_THETA_HEADER_ + D + 3 * (size_t)D * D;
    const int lane = threadIdx.x & 63, ks = (threadIdx.x >> 6) & 1, dt = threadIdx.x >> 7;
    const int dd = 16 * dt + (lane & 15), e0 = 32 * ks + 8 * (lane >> 4);
    f32x8 cv;
#pragma unroll
    for (int e = 0; e < 8; ++e) cv[e] = C2[dd * D + e0 + e] + C2[(e0 + e) * D + dd];
    *(bf16x8*)(&sm.csym[dt][ks][lane][0]) = __builtin_convertvector(cv, bf16x8);
  }
  __syncthreads();
  const int w = threadIdx.x >> 6;
  if (w < 4) producer<KEY>(ba, sm, cx, w);
  else consumer<KEY>(ba, sm, cx, slot, w - 4);
}


// ===============================================================================================================
// The two walks that have the shape of the forward pass, on the same producer/consumer split:
//   MODE 0  forward walk:  Yhat_c = tril(P_c S_c^T) V1_c + P_c T_{c-1},  T_c = T_{c-1} + S_c^T V1_c;  the producers
//           normalise, read dY and write the G1 rows [dY / den, -(dY . Y) / den].
//   MODE 1  backward walk: dV1_c = tril(P_c S_c^T)^T G1_c + S_c R_{c+1},  R_c = R_{c+1} + P_c^T G1_c  (the same
//           dataflow with queries and keys exchanged, G1 in the place of V1 and the mask mirrored); the producers
//           write dV.
// The FIRST side (keys in MODE 0, queries in MODE 1) builds the state and is produced in steps 0 and 1, the SECOND
// side in steps 2 and 3; all feature tiles are token-major, the consumer gets the first side's transposes from an
// MFMA against a selection matrix, as in the forward pass.  LDS: xoth / xown = rows of the first / second side,
// uothT = transposed value rows of the first side (written in step 3 for the next chunk, read by the consumers in
// intervals 4c+1 and 4c+2).
// ===============================================================================================================
struct SmemWalk {
  __attribute__((aligned(16))) uint16_t xoth[TC][LDR];
  __attribute__((aligned(16))) uint16_t xown[TC][LDR];
  __attribute__((aligned(16))) uint16_t uothT[DVP][LDJ];
  __attribute__((aligned(16))) float add_oth[TC];
  __attribute__((aligned(16))) float add_own[TC];
  __attribute__((aligned(16))) uint16_t feat[2][4][4][64][8]; // [slot][2 (tile of the step) + block][pair][lane]
  __attribute__((aligned(16))) uint16_t xch[4][4][16][LDXB];
};

// DYF32: the rows of dY are fp32 (MODE 0 reads them; they stay fp32 until the G1 row is rounded)
template <int MODE, bool DYF32>
__device__ __forceinline__ void walk_producer(const BwdArgs& ba, SmemWalk& sm, const Ctx& cx, int j) {
  const FastArgs& a = ba.f;
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 4, c = lane & 15;
  const uint16_t* Xown = MODE ? cx.Kb : cx.Qb;
  const uint16_t* Xoth = MODE ? cx.Qb : cx.Kb;
  const long long sl_own = MODE ? a.K.sl : a.Q.sl, sl_oth = MODE ? a.Q.sl : a.K.sl;
  const float wmaxq = max256(a.wnorm + ((size_t)cx.pg * 2) * M), amax = max256(a.bias + ((size_t)cx.pg * 2) * M);
  const int b = cx.bh / a.H, h = cx.bh % a.H;

  W64 wq, wk;
  load_w64(wq, a.Wbf + ((size_t)cx.pg * 2) * M * D, j, lane);
  load_w64(wk, a.Wbf + ((size_t)cx.pg * 2 + 1) * M * D, j, lane);
  const W64& wown = MODE ? wk : wq;
  const W64& woth = MODE ? wq : wk;
  B64 qb;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int r = 0; r < 4; ++r) qb.b[mt][r] = 2.f * (a.bias[((size_t)cx.pg * 2) * M + 64 * j + 16 * mt + 4 * g + r] - amax);

  StageG stg;
  stg.rko[0] = stg.rko[1] = stg.rkw[0] = stg.rkw[1] = 0.f;
  load_x<MODE>(stg.xo, stg.rko, !MODE, Xoth, sl_oth, a, cx, 0, tid);
  load_u<MODE>(stg, a, cx, 0, tid);
  store_x(stg.xo, stg.rko, !MODE, sm.xoth, sm.add_oth, a, cx, chunk_rows<MODE>(cx, 0), wmaxq, tid);
  store_u_transposed<MODE>(stg, sm, chunk_rows<MODE>(cx, 0), tid);
  load_x<MODE>(stg.xo, stg.rko, !MODE, Xoth, sl_oth, a, cx, 1, tid);
  load_u<MODE>(stg, a, cx, 1, tid);
  load_x<MODE>(stg.xw, stg.rkw, MODE, Xown, sl_own, a, cx, 0, tid);
  __syncthreads();                 // barrier 0

  XOp xo[2][2];
  load_xop(xo[0][0], sm.xoth, 0, lane);
  load_xop(xo[0][1], sm.xoth, 1, lane);
  // dY pieces of token tile j of the chunk that is finished next (MODE 0): four bf16 or four fp32 numbers per tile
  typedef typename std::conditional<DYF32, u32x4, u32x2>::type GyPiece;
  GyPiece gy[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) gy[i] = GyPiece{};

  auto load_dy = [&](int ci_done) {
    const int r0 = chunk_row<MODE>(cx, ci_done);
    constexpr int esz = DYF32 ? 4 : 2;
    const __amdgpu_buffer_rsrc_t rd = chunk_rsrc((const char*)ba.dY.ptr + (b * ba.dY.sb + h * ba.dY.sh + (long long)r0 * ba.dY.sl) * esz,
                                                 esz * (int)ba.dY.sl, chunk_rows<MODE>(cx, ci_done), esz * D);
#pragma unroll
    for (int vt = 0; vt < 4; ++vt) {
      const int off = esz * ((16 * j + c) * (int)ba.dY.sl + 16 * vt + 4 * g);
      if constexpr (DYF32) gy[vt] = __builtin_amdgcn_raw_buffer_load_b128(rd, off, 0, 0);
      else gy[vt] = __builtin_amdgcn_raw_buffer_load_b64(rd, off, 0, 0);
    }
  };
  int nzero = 0;                   // (forward walk) rows this wave finished with a zero normaliser
  auto finish = [&](int ci_done) {
    f32x4 fsum[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) fsum[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    finish_tiles(fsum, sm, j, 0, lane);
    finish_tiles(fsum, sm, j, 2, lane);
    const int r0 = chunk_row<MODE>(cx, ci_done), nv = chunk_rows<MODE>(cx, ci_done);
    if (MODE) {
      const int esz = ba.dV.dtype == 1 ? 2 : 4;
      const char* gp = (const char*)ba.dV.ptr + (b * ba.dV.sb + h * ba.dV.sh + (long long)r0 * ba.dV.sl) * esz;
      finish_store(fsum, ba.dV, gp, nv, j, lane);
    } else {
      unsigned zt;
      const float inv = finish_norm(fsum, sm, j, lane, &zt);   // fsum = Y rows now
      nzero += count_zero_tokens(zt, j, nv);
      f32x4 gv[4];
      float dot = 0.f;
#pragma unroll
      for (int vt = 0; vt < 4; ++vt) {
        if constexpr (DYF32) gv[vt] = __builtin_bit_cast(f32x4, gy[vt]);
        else gv[vt] = __builtin_convertvector(__builtin_bit_cast(bf16x4, gy[vt]), f32x4);
#pragma unroll
        for (int r = 0; r < 4; ++r) dot += gv[vt][r] * fsum[vt][r];
      }
      dot += __shfl_xor(dot, 16);
      dot += __shfl_xor(dot, 32);
      const __amdgpu_buffer_rsrc_t rg = chunk_rsrc(cx.Gb + (long long)r0 * DVP, 2 * DVP, nv, 2 * DVP);
      const int off = 2 * ((16 * j + c) * DVP + 4 * g);
#pragma unroll
      for (int vt = 0; vt < 4; ++vt)
        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, __builtin_convertvector(gv[vt] * inv, bf16x4)), rg, off + 32 * vt, 0, 0);
      const f32x4 last = {g == 0 ? -dot * inv : 0.f, 0.f, 0.f, 0.f};
      __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, __builtin_convertvector(last, bf16x4)), rg, off + 2 * D, 0, 0);
    }
  };

  for (int ci = 0; ci < cx.nchunk; ++ci) {
    const int nv = chunk_rows<MODE>(cx, ci);
#pragma unroll
    for (int S = 0; S < 4; ++S) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        if (S == 0) load_xop(xo[1][u], sm.xoth, 2 + u, lane);
        else if (S == 1) load_xop(xo[0][u], sm.xown, u, lane);
        else if (S == 2) load_xop(xo[1][u], sm.xown, 2 + u, lane);
        else load_xop(xo[0][u], sm.xoth, u, lane);
      }
      __builtin_amdgcn_sched_barrier(0);

#pragma unroll
      for (int u = 0; u < 2; ++u) {
        bf16x8 img[2];
        if (S < 2) feature_tile64<MODE != 0>(woth, &qb, xo[S & 1][u], sm.add_oth[16 * (2 * S + u) + c], img);
        else feature_tile64<MODE == 0>(wown, &qb, xo[S & 1][u], sm.add_own[16 * (2 * (S - 2) + u) + c], img);
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) *(bf16x8*)(&sm.feat[S & 1][2 * u + blk][j][lane][0]) = img[blk];
      }

      if (S == 0) {
        store_x(stg.xw, stg.rkw, MODE, sm.xown, sm.add_own, a, cx, nv, wmaxq, tid);
        load_x<MODE>(stg.xw, stg.rkw, MODE, Xown, sl_own, a, cx, ci + 1, tid);
        if (!MODE && ci > 0) load_dy(ci - 1);
      } else if (S == 1) {
        if (ci > 0) finish(ci - 1);
      } else if (S == 2) {
        store_x(stg.xo, stg.rko, !MODE, sm.xoth, sm.add_oth, a, cx, chunk_rows<MODE>(cx, ci + 1), wmaxq, tid);
        load_x<MODE>(stg.xo, stg.rko, !MODE, Xoth, sl_oth, a, cx, ci + 2, tid);
      } else {
        store_u_transposed<MODE>(stg, sm, chunk_rows<MODE>(cx, ci + 1), tid);
        load_u<MODE>(stg, a, cx, ci + 2, tid);
      }
      __syncthreads();
    }
  }
  if (!MODE && cx.nchunk > 0) load_dy(cx.nchunk - 1);
  __syncthreads();                 // the consumers' last step
  if (cx.nchunk > 0) finish(cx.nchunk - 1);
  if (!MODE) report_zero_rows(a.flushed, nzero, lane);
}

template <int MODE>
__device__ __forceinline__ void walk_consumer(const BwdArgs& ba, SmemWalk& sm, const Ctx& cx, int slot, int j) {
  const FastArgs& a = ba.f;
  const int lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
  f32x4 T[4][NVT];
  {
    // (single slot per sequence: neither a prefix nor a suffix was computed; every workgroup reads one block of zeros)
    const float* Tg = ba.zero_state != nullptr ? ba.zero_state
                                               : (MODE ? ba.Rpart : a.Tpart) + ((size_t)cx.bh * a.nslot + slot) * M * DVP;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
        for (int r = 0; r < 4; ++r) T[mt][vt][r] = Tg[(size_t)(64 * j + 16 * mt + 4 * g + r) * DVP + 16 * vt + c];
  }
  walk_consume<MODE>(sm, T, cx.nchunk, j);
}

// grid (nslot, B*H), block 512.
template <int MODE, bool DYF32>
__global__ void __launch_bounds__(NT8) k_bwd_walk_pc(BwdArgs ba) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  SmemWalk& sm = *reinterpret_cast<SmemWalk*>(smem_raw);
  const FastArgs& a = ba.f;
  const int slot = blockIdx.x, bh = blockIdx.y, b = bh / a.H, h = bh % a.H;
  const float* th = a.theta + (size_t)group_of(a.groups, b, h, a.H) * (FS_THETA_HEADER_ + (size_t)D + 4 * (size_t)D * D);
  Ctx cx;
  cx.isoC = ((int)th[2]) & 1;
  cx.bh = bh;
  cx.pg = group_of(a.pgroups, b, h, a.H);
  cx.cs = a.cstar[bh];
  cx.Qb = (const uint16_t*)a.Q.ptr + b * a.Q.sb + h * a.Q.sh;
  cx.Kb = (const uint16_t*)a.K.ptr + b * a.K.sb + h * a.K.sh;
  cx.Vb = (const uint16_t*)a.V.ptr + b * a.V.sb + h * a.V.sh;
  cx.Gb = ba.gh + (size_t)bh * ba.Lq * DVP;
  cx.row_beg = min(ba.Lq, slot * ba.rows_per_rslot);
  cx.row_end = min(ba.Lq, cx.row_beg + ba.rows_per_rslot);
  cx.nchunk = (cx.row_end - cx.row_beg + TC - 1) / TC;
  // the value columns fill rows 0..64 of the transposed tile only
  for (int idx = threadIdx.x; idx < DVP * LDJ / 2; idx += NT8) ((uint32_t*)&sm.uothT[0][0])[idx] = 0u;
  __syncthreads();
  const int w = threadIdx.x >> 6;
  if (w < 4) walk_producer<MODE, DYF32>(ba, sm, cx, w);
  else walk_consumer<MODE>(ba, sm, cx, slot, w - 4);
}

}  // namespace cg

namespace bwd {

// Exclusive suffix over the slots of one (b,h), in place; four consecutive numbers per thread.
// grid (ceil(M*DVP/1024), B*H).
__global__ void k_bwd_suffix(float* Rpart, int nslot) {
  constexpr size_t per = (size_t)M * DVP;
  const size_t e = 4 * ((size_t)blockIdx.x * blockDim.x + threadIdx.x);
  if (e >= per) return;
  float* p = Rpart + (size_t)blockIdx.y * nslot * per + e;
  f32x4 run = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
  for (int s = nslot - 1; s >= 0; --s) {
    const f32x4 v = *(const f32x4*)(p + (size_t)s * per);
    *(f32x4*)(p + (size_t)s * per) = run;
    run += v;
  }
}

}  // namespace bwd

int launch_bwd_cgrad_pc(const bwd::BwdArgs& ba, int nslot, int BH, hipStream_t st) {
  const void* fns[2] = {(const void*)cg::k_bwd_cgrad_pc<0>, (const void*)cg::k_bwd_cgrad_pc<1>};
  for (const void* fn : fns)
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(cg::SmemCG)) != hipSuccess) {
      (void)hipGetLastError();
      return 2;
    }
  hipLaunchKernelGGL(cg::k_bwd_cgrad_pc<0>, dim3(nslot, BH), dim3(pc::NT8), sizeof(cg::SmemCG), st, ba);
  if (hipGetLastError() != hipSuccess) return 5;
  hipLaunchKernelGGL(cg::k_bwd_cgrad_pc<1>, dim3(nslot, BH), dim3(pc::NT8), sizeof(cg::SmemCG), st, ba);
  if (hipGetLastError() != hipSuccess) return 5;
  return 0;
}

int launch_bwd_walk_pc(const bwd::BwdArgs& ba, int mode, int nslot, int BH, hipStream_t st) {
  const bool f32dy = ba.dY.dtype == 0;
  const void* fn = mode ? (const void*)cg::k_bwd_walk_pc<1, false>
                        : (f32dy ? (const void*)cg::k_bwd_walk_pc<0, true> : (const void*)cg::k_bwd_walk_pc<0, false>);
  if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(cg::SmemWalk)) != hipSuccess) {
    (void)hipGetLastError();
    return 2;
  }
  if (mode) hipLaunchKernelGGL((cg::k_bwd_walk_pc<1, false>), dim3(nslot, BH), dim3(pc::NT8), sizeof(cg::SmemWalk), st, ba);
  else if (f32dy) hipLaunchKernelGGL((cg::k_bwd_walk_pc<0, true>), dim3(nslot, BH), dim3(pc::NT8), sizeof(cg::SmemWalk), st, ba);
  else hipLaunchKernelGGL((cg::k_bwd_walk_pc<0, false>), dim3(nslot, BH), dim3(pc::NT8), sizeof(cg::SmemWalk), st, ba);
  if (hipGetLastError() != hipSuccess) return 5;
  return 0;
}

#define FS_LAUNCH_CHECK() do { if (hipGetLastError() != hipSuccess) return 5; } while (0)

// One causal backward call after the forward state pass over every slot (f.Tpart = exclusive prefix per slot on the
// sequence's common shift f.cstar).
int launch_fast_backward_causal(const FastLaunch& f, const FastArgs& a, const TensorDev& dY, const TensorDev& dQ,
                                const TensorDev& dK, const TensorDev& dV, uint16_t* gh, float* Rpart, float* rcpart,
                                hipStream_t st) {
  bwd::BwdArgs ba;
  ba.f = a;
  ba.dY = dY; ba.dQ = dQ; ba.dK = dK; ba.dV = dV;
  ba.gh = gh; ba.Rpart = Rpart; ba.rcpart = rcpart;
  ba.Lq = f.Lq; ba.Lk = f.Lk; ba.rslots = a.nslot; ba.rows_per_rslot = a.rows_per_seg / a.sub;
  const int BH = f.B * f.H;
  if (a.nslot == 1) {
    // a single slot per sequence: no prefix and no suffix states; the first state of the (unused) suffix buffer is
    // the block of zeros that every workgroup starts from
    if (int rc = launch_fill_u32((uint32_t*)Rpart, 0u, (size_t)M * DVP, st)) return rc;
    ba.zero_state = Rpart;
  }
  if (int rc = launch_bwd_walk_pc(ba, 0, a.nslot, BH, st)) return rc;
  if (a.nslot > 1) {
    if (int rc = launch_bwd_rstate(ba, BH, st)) return rc;
    hipLaunchKernelGGL(bwd::k_bwd_suffix, dim3((M * DVP / 4 + 255) / 256, BH), dim3(256), 0, st, Rpart, a.nslot);
    FS_LAUNCH_CHECK();
  }
  if (int rc = launch_bwd_walk_pc(ba, 1, a.nslot, BH, st)) return rc;
  return launch_bwd_cgrad_pc(ba, a.nslot, BH, st);
}

size_t fast_bwd_causal_lds_bytes() { return bwd_pc_lds_bytes(); }

size_t bwd_pc_lds_bytes() { return sizeof(cg::SmemCG) > sizeof(cg::SmemWalk) ? sizeof(cg::SmemCG) : sizeof(cg::SmemWalk); }

}  // namespace fs
