// Building blocks shared by the kernels whose waves are split into producers (staging, feature tiles, finishing)
// and consumers (contractions with the state in registers): the causal segment kernel of the forward pass
// (kernels_bf16_causal.hip), the causal gradient kernels (kernels_bf16_bwd_pc.hip) and the kernels for d = dv = 128,
// M = 512 (kernels_bf16_wide.hip).
#pragma once
#include "fast_common.h"

namespace fs {
namespace pc {

using namespace fast;

constexpr int NT8 = 512;           // threads per workgroup: four producer and four consumer waves

// Global memory of a chunk is addressed through buffer descriptors: a uniform base (the chunk's first row), a 32-bit
// byte offset per thread, and a byte count that ends with the last valid row, so that reads past the end of the
// segment return zero and writes there are dropped, without branches or 64-bit address registers.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t chunk_rsrc(const void* base, int sl_bytes, int rows_valid, int row_bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0,
                                           rows_valid > 0 ? (int)((rows_valid - 1) * sl_bytes + row_bytes) : 0, 0x00020000);
}

// Writes one piece of a row; returns, in every lane of the 8 that share the row, its squared norm.
__device__ __forceinline__ float store_row_piece(u32x4 p, uint16_t (*tile)[LDR], int row, int pc) {
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
__device__ __forceinline__ void store_val_piece(u32x4 p, uint16_t (*vt)[LDJ], int j, int pc) {
  const int odd = j & 1;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const uint32_t mine = p[e], other = dpp_u<0xB1>(mine);
    const uint32_t w = odd ? ((other >> 16) | (mine & 0xffff0000u)) : ((mine & 0xffffu) | (other << 16));
    *(uint32_t*)(&vt[pc * 8 + 2 * e + odd][j & ~1]) = w;
  }
}

// ---- producer pieces -----------------------------------------------------------------------------------------------
struct W64 { bf16x8 w[4][KS]; };   // rows = features 64j + 16mt + c, k = 32ks + 8g + e
struct B64 { f32x4 b[4]; };        // 2 (bias - largest bias) of features 64j + 16mt + 4g + r

__device__ __forceinline__ void load_w64(W64& ws, const uint16_t* Wbf, int j, int lane) {
  const int g = lane >> 4, c = lane & 15;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      ws.w[mt][ks] = *(const bf16x8*)(Wbf + (size_t)(64 * j + 16 * mt + c) * D + 32 * ks + 8 * g);
}

// Selection matrices (B operands) that turn an A operand (lane <-> token, k <-> feature) into an accumulator with
// lane <-> feature: sel[hh] has a one at (k, n) iff k addresses feature 16 hh + n of the 32-feature block.
__device__ __forceinline__ void make_sel32(bf16x8 sel[2], int lane) {
  const int g = lane >> 4, c = lane & 15;
  // lane (g, c) holds at most one 1: element e with e/4 = hh and 4g + e%4 = c
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
__device__ __forceinline__ void load_xop(XOp& x, const uint16_t (*tile)[LDR], int jt, int lane) {
  const int g = lane >> 4, c = lane & 15;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) x.b[ks] = *(const bf16x8*)(&tile[16 * jt + c][32 * ks + 8 * g]);
}

// Feature tile of 16 tokens and the pair's 64 features: img[blk] is the packed MFMA operand of the 32-feature block
// blk (lane <-> token 16 jt + c, k = 8g + e <-> feature 32 blk + 16 (e/4) + 4g + e%4).
template <bool WITH_BIAS>
__device__ __forceinline__ void feature_tile64(const W64& ws, const B64* qb, const XOp& x, float add, bf16x8 img[2]) {
  // without a bias the token's shift is the accumulator's initial value: nothing is left to add afterwards
  const f32x4 add4 = {add, add, add, add};
  f32x4 acc[4];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
    acc[mt] = mfma(ws.w[mt][0], x.b[0], WITH_BIAS ? qb->b[mt] : add4);
#pragma unroll
    for (int ks = 1; ks < KS; ++ks) acc[mt] = mfma(ws.w[mt][ks], x.b[ks], acc[mt]);
  }
#pragma unroll
  for (int blk = 0; blk < 2; ++blk)
    img[blk] = WITH_BIAS ? pack8(exp2v(acc[2 * blk] + add), exp2v(acc[2 * blk + 1] + add)) : pack8(exp2v(acc[2 * blk]), exp2v(acc[2 * blk + 1]));
}

// `ychunk`: first output row of the chunk (bytes); `nv`: its number of valid rows (0: nothing is stored).
__device__ __forceinline__ void finish_store(const f32x4 (&fs)[4], const TensorDev& Y, const char* ychunk, int nv, int it, int lane) {
  const int g = lane >> 4, c = lane & 15;
  if (Y.dtype == 1) {
    const __amdgpu_buffer_rsrc_t ry = chunk_rsrc(ychunk, 2 * (int)Y.sl, nv, 2 * D);
    const int off = 2 * ((16 * it + c) * (int)Y.sl + 4 * g);
#pragma unroll
    for (int vt = 0; vt < 4; ++vt)
      __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, __builtin_convertvector(fs[vt], bf16x4)), ry, off + 32 * vt, 0, 0);
  } else {
    const __amdgpu_buffer_rsrc_t ry = chunk_rsrc(ychunk, 4 * (int)Y.sl, nv, 4 * D);
    const int off = 4 * ((16 * it + c) * (int)Y.sl + 4 * g);
#pragma unroll
    for (int vt = 0; vt < 4; ++vt)
      __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, fs[vt]), ry, off + 64 * vt, 0, 0);
  }
}

// B operand / A operand of the value tile: lane <-> column 16 vt + c, k <-> tokens {32 jp + 4g + r, 32 jp + 16 + 4g + r}.
__device__ __forceinline__ bf16x8 load_vop_l(const uint16_t (*vt)[LDJ], int jp, int vtile, int lane) {
  const int g = lane >> 4, c = lane & 15;
  const u32x2 lo = *(const u32x2*)(&vt[16 * vtile + c][32 * jp + 4 * g]);
  const u32x2 hi = *(const u32x2*)(&vt[16 * vtile + c][32 * jp + 16 + 4 * g]);
  const u32x4 v = {lo[0], lo[1], hi[0], hi[1]};
  return __builtin_bit_cast(bf16x8, v);
}

// Consumer side of a walk that has the shape of the forward pass (state T of 64 features x 80 columns in registers,
// first-side tiles in steps 0 and 1 with the state update, second-side tiles in steps 2 and 3 with the output tiles),
// for producers that hand over token-major register images of both sides and values transposed in LDS: the walks of
// the causal gradient kernels and of the d = dv = 128 shape.  (The forward kernel for d = dv = 64 has a consumer of
// its own, built on row-major tiles and transposing reads, with a running key shift: kernels_bf16_causal.hip.)
//   MODE 0: second-side token i sees first-side tokens j <= i;  MODE 1: j >= i;  MODE 2: no first side at all (the
//   state is the whole sum and stays as it is: the query pass of a non-causal call; steps 0 and 1 are empty).
// `sm` needs feat[2][4][4][64][8], uothT[DVP][LDJ] and xch[4][4][16][LDXB].  Executes 2 + 4 nchunk barriers.
template <int MODE, class SM>
__device__ __forceinline__ void walk_consume(SM& sm, f32x4 (&T)[4][NVT], int nchunk, int j) {
  const int lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
  __syncthreads();                 // barrier 0
  __syncthreads();                 // the producers' first step

  // state as A operand (rows = value columns, contraction index <-> feature): before every chunk, or once
  bf16x8 tb[2][NVT];
  if (MODE == 2) {
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) tb[blk][vt] = pack8(T[2 * blk][vt], T[2 * blk + 1][vt]);
  }
  for (int ci = 0; ci < nchunk; ++ci) {
    if (MODE != 2) {
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt) tb[blk][vt] = pack8(T[2 * blk][vt], T[2 * blk + 1][vt]);
    }
    bf16x8 sk[4][2];               // first-side feature tiles of the chunk
    bf16x8 vop[2][NVT];            // value operands of the chunk
#pragma unroll
    for (int S = 0; S < 4; ++S) {
      if (S < 2 && MODE == 2) {
        // nothing: the barrier below keeps the step structure of the producers
      } else if (S < 2) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int blk = 0; blk < 2; ++blk) sk[2 * S + u][blk] = *(const bf16x8*)(&sm.feat[S & 1][2 * u + blk][j][lane][0]);
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt) vop[S][vt] = load_vop_l(sm.uothT, S, vt, lane);
        bf16x8 sel[2];
        {
          int lane_here = lane;
          asm volatile("" : "+v"(lane_here));
          make_sel32(sel, lane_here);
        }
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
          const f32x4 tr0 = mfma(sk[2 * S][mt >> 1], sel[mt & 1], f32x4{0.f, 0.f, 0.f, 0.f});
          const f32x4 tr1 = mfma(sk[2 * S + 1][mt >> 1], sel[mt & 1], f32x4{0.f, 0.f, 0.f, 0.f});
          const bf16x8 stv = pack8(tr0, tr1);
#pragma unroll
          for (int vt = 0; vt < NVT; ++vt) T[mt][vt] = mfma(stv, vop[S][vt], T[mt][vt]);
        }
      } else {
        bf16x8 pq[2][2];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int blk = 0; blk < 2; ++blk) pq[u][blk] = *(const bf16x8*)(&sm.feat[S & 1][2 * u + blk][j][lane][0]);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int it = 2 * (S - 2) + u;
          const bf16x8* p = pq[u];
          f32x4 y[NVT];
#pragma unroll
          for (int vt = 0; vt < NVT; ++vt) {
            y[vt] = mfma(tb[0][vt], p[0], f32x4{0.f, 0.f, 0.f, 0.f});
            y[vt] = mfma(tb[1][vt], p[1], y[vt]);
          }
          // scores^T tiles (rows = first-side tokens 16 jt + 4g + r, column = second-side token 16 it + c), masked
#pragma unroll
          for (int jp = 0; jp < 2; ++jp) {
            if (MODE != 2 && (MODE ? 2 * jp + 1 >= it : 2 * jp <= it)) {
              f32x4 sc[2];
#pragma unroll
              for (int jj = 0; jj < 2; ++jj) {
                const int jt = 2 * jp + jj;
                sc[jj] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (MODE ? jt >= it : jt <= it) {
                  sc[jj] = mfma(sk[jt][0], p[0], sc[jj]);
                  sc[jj] = mfma(sk[jt][1], p[1], sc[jj]);
                  if (jt == it) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) sc[jj][r] = (MODE ? 4 * g + r >= c : 4 * g + r <= c) ? sc[jj][r] : 0.f;
                  }
                }
              }
              const bf16x8 sb = pack8(sc[0], sc[1]);
#pragma unroll
              for (int vt = 0; vt < NVT; ++vt) y[vt] = mfma(vop[jp][vt], sb, y[vt]);
            }
          }
          exchange_put_bf16(sm, y, it, j, lane);
        }
      }
      __syncthreads();
    }
  }
}

}  // namespace pc
}  // namespace fs
