// Causal segment kernel of the bf16 attention path (d = dv = 64, M = 256).
//
// One workgroup (8 waves = two per SIMD of one CU) walks one segment of one sequence in 64-token chunks, its state
// seeded with the exclusive prefix of the segment states:
//   Y_c = (tril(P_c S_c^T) [V_c 1] + P_c T_{c-1}) normalised by its last column;  T_c = T_{c-1} + S_c^T [V_c 1].
//
// The waves are specialised.  Waves 0..3 are PRODUCERS, waves 4..7 CONSUMERS; producer j and consumer j share a SIMD
// and the 64 random features [64j, 64j+64):
//   producer j  stages the next chunk's Q, K, V rows (global -> registers -> LDS, all three row-major as they are in
//               memory), computes the row norms of its token tile on the MFMA pipe (the diagonal of X X^T), computes
//               the feature tiles of its 64 features (projection MFMA, exp2, convert) and hands them to its
//               consumer through LDS; one chunk later it sums the four consumers' partial tiles of token tile j (an
//               MFMA against a 0/1 routing matrix), normalises and stores them.
//   consumer j  holds the state slice T (64 features x 80 columns, fp32) in registers and does the contractions:
//               state update S^T [V 1], inter-chunk term P T, scores S P^T (masked on the diagonal tiles) and
//               scores x [V 1]; it writes its partial output tiles (a sum over its 64 features) to LDS as bf16.
// One wave's exp2 / convert stream thus runs beside the other's MFMA stream on every SIMD by construction.
//
// Operand layouts.  Every MFMA is v_mfma_f32_16x16x32_bf16 (lane (g, c) = (lane / 16, lane % 16) supplies A[c][8g..8g+7],
// B[8g..8g+7][c] and owns D[4g..4g+3][c]).
//   key features are computed FEATURE-MAJOR (A = token rows, B = W~: the accumulator has lane <-> feature, registers
//   <-> four consecutive tokens): the per-token part of the exponent (row term - key shift) is the accumulator's
//   initial value, read from LDS as one 16-byte vector, so nothing is added afterwards, and the converted tiles are
//   directly the A operands S^T of the state update.  They go to LDS as 8-byte units (one feature, four tokens).
//   The scores need the same numbers token-major (lane <-> token, contraction index <-> feature): the consumer gets
//   them from the same units with the transposing LDS read (ds_read_b64_tr_b16: the lane (a, b) = (c / 4, c % 4) of
//   a row of 16 lanes receives element b of the 8-byte pieces addressed by lanes a, 4 + a, 8 + a, 12 + a).
//   query features are computed token-major (A = W~, B = token rows; bias preloaded in the accumulator) and travel as
//   register images (lane-linear 16-byte pieces).
//   values stay row-major in LDS ([token][column], 160-byte rows: 64 values, a one, 15 zeros); the operand
//   (lane <-> column, contraction index <-> tokens) of the state update and of scores x [V 1] is again a transposing
//   read.
// Unit u of a (token tile, feature tile) block sits at 8 sigma(u) bytes, sigma(g, c) = 16 (c/4) + 4 (c%4) + (g + c/4)%4:
// the plain accesses (16 consecutive lanes = one g) and the transposing ones (one row of 16 lanes reads features
// 4g' .. 4g'+3 of token quads 0..3) both touch 16 different 8-byte bank pairs.
//
// Shifts.  Keys: running maximum of a per-token bound, the state rebased when it grows (fast_common.h).  Queries:
// when every row of the chunk has a Cauchy-Schwarz bound below 2^80 no shift is needed at all (the common case: the
// per-row factor cancels in the normalisation) and the per-element addition is skipped; otherwise every row gets
// its own shift as in the other kernels.
//
// The chunk is four steps of two token tiles (key tiles 0-1, 2-3, query tiles 0-1, 2-3), one workgroup barrier after
// each; the producer works one step ahead of the consumer.  Both roles execute exactly the same number of barriers
// (3 + 4 per chunk).  With t = 4 (chunk index) + step: the feature tiles of step t are written in interval t and
// read in interval t+1 (two slots); the partial outputs of chunk c are written in intervals 4c+3 and 4c+4 and summed
// by the producers in interval 4c+6 (their third step of the next chunk, before the consumers overwrite them in
// 4c+7); the rows of chunk c+1 go to the other LDS buffer part by part in the four steps of chunk c (after every
// reader of chunk c-1: the producers' tile reads end in interval 4c-1, the consumers' value reads in 4c) and are
// first read in interval 4c+3 (row norms, and the prefetch of the next chunk's first key tiles; the key and query
// rows were stored in steps 0 and 1); each part's registers are refilled at once with the same part of chunk c+2.
// The per-token constants of chunk c+1 (row terms, query shifts) and the chunk's two maxima (largest key bound,
// largest query shift: LDS float-maximum atomics from the lanes that hold a row norm) are written in interval 4c+3
// and first read in interval 4c+4; the maxima of that parity were last read in interval 4c+1 and are reset in 4c+2.
#include <hip/hip_ext.h>

#include "fast_pc.h"

namespace fs {

using namespace fast;

namespace pc {

struct SmemPC {
  uint16_t k[2][TC][LDR];          // key rows, bf16 bits
  uint16_t q[2][TC][LDR];          // query rows
  __attribute__((aligned(16))) uint16_t v[2][TC][LDV];   // value rows: columns 0..63, column 64 = 1, columns 65.. = 0
  __attribute__((aligned(16))) float kadd[2][TC];   // per key token t, at index t: row term log2e y^T C2 y (-inf past the end)
  float kmax[2], qmax[2];                           // per chunk parity: largest key bound (row_shift + row term), largest query row_shift
  __attribute__((aligned(16))) float qadd[2][TC];   // per query token t, at index 4 (t%16) + t/16: - row_shift
  // feature tiles of one step, two slots of 16 kB.  Key steps: [tile of the pair][producer][feature tile] blocks of
  // 64 units of 8 bytes (unit (g, c) at 8 sigma(g, c): feature c, tokens 4g .. 4g+3).  Query steps: [tile of the
  // step][producer][32-feature block][lane] register images of 16 bytes.
  __attribute__((aligned(16))) uint16_t feat[2][8192];
  // partial outputs (bf16): [token tile][source pair][token][column]
  __attribute__((aligned(16))) uint16_t xch[4][4][16][LDXB];
};

// Unit slots of a lane: its own unit (plain accesses) and the unit it addresses in a transposing read.
__device__ __forceinline__ int sigma_own(int lane) {
  const int g = lane >> 4, c = lane & 15;
  return 16 * (c >> 2) + 4 * (c & 3) + ((g + (c >> 2)) & 3);
}
__device__ __forceinline__ int sigma_tr(int lane) {
  const int g = lane >> 4, c = lane & 15;      // addresses unit (g' = c % 4, c' = 4 g + c / 4)
  return 16 * g + 4 * (c >> 2) + (((c & 3) + g) & 3);
}

// ---- staging by the 256 producer threads, one chunk ahead --------------------------------------------------------
// Every thread carries two 16-byte pieces of the query, key and value tiles (rows tid/8 and tid/8 + 32, bytes
// 16 (tid%8)) and, for parameter sets with a dense C2, the key row terms of those two rows.
struct Stage { u32x4 q[2], k[2], v[2]; float rk[2]; };

// The staged rows go to LDS in four parts (0: query rows, 1: key rows, 2 and 3: value rows).
__device__ __forceinline__ void stage_store(const Stage& s, SmemPC& sm, int buf, bool isoC, int row0, int row_end, int tid, int part) {
  const int row = tid >> 3, pc = tid & 7;
  if (part == 0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) *(u32x4*)(&sm.q[buf][row + 32 * i][pc * 8]) = s.q[i];
  } else if (part == 1) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      *(u32x4*)(&sm.k[buf][row + 32 * i][pc * 8]) = s.k[i];
      // dense C2: the row term comes from the table (the eight lanes of a row write the same word)
      if (!isoC) sm.kadd[buf][row + 32 * i] = row0 + row + 32 * i < row_end ? s.rk[i] : -INFINITY;
    }
  } else {
    const int i = part - 2;
    *(u32x4*)(&sm.v[buf][row + 32 * i][pc * 8]) = s.v[i];
  }
}

struct SegCtx {
  const uint16_t *Qb, *Kb, *Vb;
  long long ybase;
  int bh, pg, row_beg, row_end;
  bool isoC;
};

// Every barrier of the kernel goes through this macro; the two roles must execute the same number of them.
#define FS_STEP_BARRIER() __syncthreads()

struct ChunkPtr { const uint16_t *q, *k, *v; const float* rk; };   // first row of a chunk in each tensor (uniform)

__device__ __forceinline__ void stage_load_part(Stage& s, const ChunkPtr& cp, const SegCtx& cx, const FastArgs& a, int nv, int tid, int part) {
  const int row = tid >> 3, pc = tid & 7;
  if (part == 0) {
    const __amdgpu_buffer_rsrc_t rq = chunk_rsrc(cp.q, 2 * (int)a.Q.sl, nv, 2 * D);
#pragma unroll
    for (int i = 0; i < 2; ++i) s.q[i] = __builtin_amdgcn_raw_buffer_load_b128(rq, 2 * ((row + 32 * i) * (int)a.Q.sl + pc * 8), 0, 0);
  } else if (part == 1) {
    const __amdgpu_buffer_rsrc_t rk = chunk_rsrc(cp.k, 2 * (int)a.K.sl, nv, 2 * D);
    // key row terms of a dense C2 (an empty range, hence zeros, when the closed form -|k|^2/2 applies)
    const __amdgpu_buffer_rsrc_t rr = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(cp.rk), 0,
                                                                        cx.isoC ? 0 : 4 * max(nv, 0), 0x00020000);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      s.k[i] = __builtin_amdgcn_raw_buffer_load_b128(rk, 2 * ((row + 32 * i) * (int)a.K.sl + pc * 8), 0, 0);
      s.rk[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rr, 4 * (row + 32 * i), 0, 0));
    }
  } else {
    const int i = part - 2;
    const __amdgpu_buffer_rsrc_t rv = chunk_rsrc(cp.v, 2 * (int)a.V.sl, nv, 2 * D);
    s.v[i] = __builtin_amdgcn_raw_buffer_load_b128(rv, 2 * ((row + 32 * i) * (int)a.V.sl + pc * 8), 0, 0);
  }
}

// Per-token constants of token tile j of the rows in buffer `buf` (whose first row is `row0`): squared row norms as
// the diagonal of X X^T on the MFMA pipe (bf16 products are exact in fp32), then the key row term and bound and the
// query shift.  The diagonal entry of token c sits in lane (g, c) = (c / 4, c), register c % 4.
__device__ __forceinline__ void row_constants(SmemPC& sm, int buf, const FastArgs& a, bool isoC, int row0, int row_end,
                                              float wmax1, float wmax2, int j, int lane) {
  const int g = lane >> 4, c = lane & 15;
  XOp xk, xq;
  load_xop(xk, sm.k[buf], j, lane);
  load_xop(xq, sm.q[buf], j, lane);
  const float nk2 = tile_row_norms(xk.b[0], xk.b[1], lane), nq2 = tile_row_norms(xq.b[0], xq.b[1], lane);
  if (g == (c >> 2)) {
    const int t = 16 * j + c;
    const bool valid = row0 + t < row_end;
    // rows past the end get -inf: their features are exactly zero whatever the key shift is
    const float rt = isoC ? (valid ? -0.5f * kLog2e * a.scale * a.scale * nk2 : -INFINITY) : sm.kadd[buf][t];
    if (isoC) sm.kadd[buf][t] = rt;
    if (valid) lds_fmax(&sm.kmax[buf], row_shift(nk2, wmax2) + rt);
    const float qs = row_shift(nq2, wmax1);
    sm.qadd[buf][4 * c + j] = -qs;
    lds_fmax(&sm.qmax[buf], qs);
  }
}

// Query feature tile without a row shift (every bound of the chunk is small: the per-row factor cancels later).
__device__ __forceinline__ void feature_tile64_noshift(const W64& ws, const B64& qb, const XOp& x, bf16x8 img[2]) {
  f32x4 acc[4];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
    acc[mt] = mfma(ws.w[mt][0], x.b[0], qb.b[mt]);
#pragma unroll
    for (int ks = 1; ks < KS; ++ks) acc[mt] = mfma(ws.w[mt][ks], x.b[ks], acc[mt]);
  }
#pragma unroll
  for (int blk = 0; blk < 2; ++blk) img[blk] = pack8(exp2v(acc[2 * blk]), exp2v(acc[2 * blk + 1]));
}

// Key features of one token tile and the pair's 64 features, feature-major, straight to LDS: for each feature tile
// mt one unit per lane (feature 16 mt + c, tokens 4g .. 4g+3 of the tile).  `init` = row term - key shift of the
// lane's four tokens.
__device__ __forceinline__ void key_tile_major(const W64& wk, const XOp& x, f32x4 init, uint16_t* block, int sig) {
  f32x4 acc[4];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
    acc[mt] = mfma(x.b[0], wk.w[mt][0], init);
#pragma unroll
    for (int ks = 1; ks < KS; ++ks) acc[mt] = mfma(x.b[ks], wk.w[mt][ks], acc[mt]);
  }
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
    *(bf16x4*)(block + mt * 256 + 4 * sig) = __builtin_convertvector(exp2v(acc[mt]), bf16x4);
}

__device__ __forceinline__ void producer(const FastArgs& a, SmemPC& sm, const SegCtx& cx, int j) {
  const int tid = threadIdx.x, lane = tid & 63;
  int nzero = 0;                   // rows this wave finished with a zero normaliser
  const float wmax1 = max256(a.wnorm + ((size_t)cx.pg * 2) * M), amax1 = max256(a.bias + ((size_t)cx.pg * 2) * M);
  const float wmax2 = max256(a.wnorm + ((size_t)cx.pg * 2 + 1) * M);
  // both projection slices stay in registers (they are the same numbers when B1 = B2; the producers have room)
  W64 wq, wk;
  load_w64(wq, a.Wbf + ((size_t)cx.pg * 2) * M * D, j, lane);
  load_w64(wk, a.Wbf + ((size_t)cx.pg * 2 + 1) * M * D, j, lane);
  B64 qb;
  {
    const int g = lane >> 4;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int r = 0; r < 4; ++r) qb.b[mt][r] = 2.f * (a.bias[((size_t)cx.pg * 2) * M + 64 * j + 16 * mt + 4 * g + r] - amax1);
  }
  // shift of the prefix state (the first segment has none: a zero state on the shift -inf, nothing read)
  float dk = blockIdx.x > 0 ? a.cstar[gridDim.y + (size_t)cx.bh * a.nslot + (size_t)blockIdx.x * a.sub] : -INFINITY;

  // first chunk to LDS, second chunk into the staging registers
  Stage stg;
  ChunkPtr cp = {cx.Qb + (long long)cx.row_beg * a.Q.sl, cx.Kb + (long long)cx.row_beg * a.K.sl,
                 cx.Vb + (long long)cx.row_beg * a.V.sl, a.rk + (size_t)cx.bh * a.L + cx.row_beg};
  const long long qstep = TC * a.Q.sl, kstep = TC * a.K.sl, vstep = TC * a.V.sl;
#pragma unroll
  for (int part = 0; part < 4; ++part) stage_load_part(stg, cp, cx, a, min(TC, cx.row_end - cx.row_beg), tid, part);
  cp.q += qstep; cp.k += kstep; cp.v += vstep; cp.rk += TC;
#pragma unroll
  for (int part = 0; part < 4; ++part) {
    stage_store(stg, sm, 0, cx.isoC, cx.row_beg, cx.row_end, tid, part);
    stage_load_part(stg, cp, cx, a, min(TC, cx.row_end - cx.row_beg - TC), tid, part);
  }
  // output rows of the previous chunk (finished by the producers one chunk later)
  const long long ystep = (long long)TC * a.Y.sl * (a.Y.dtype == 1 ? 2 : 4);
  const char* yprev = (const char*)a.Y.ptr + (cx.ybase + (long long)cx.row_beg * a.Y.sl) * (a.Y.dtype == 1 ? 2 : 4) - ystep;
  if (tid < 2) { sm.kmax[tid] = -INFINITY; sm.qmax[tid] = -INFINITY; }
  FS_STEP_BARRIER();               // barrier 0: the first chunk's rows are in LDS
  row_constants(sm, 0, a, cx.isoC, cx.row_beg, cx.row_end, wmax1, wmax2, j, lane);
  FS_STEP_BARRIER();               // barrier 1: and their per-token constants

  XOp xo[2][2];                    // [step parity][tile of the step]
  load_xop(xo[0][0], sm.k[0], 0, lane);
  load_xop(xo[0][1], sm.k[0], 1, lane);
  int buf = 0;
  for (int row0 = cx.row_beg; row0 < cx.row_end; row0 += TC, buf ^= 1) {
    // Addresses that are used once per chunk are rebuilt from an opaque copy of the thread number instead of living
    // in registers through the whole loop.
    int tid_here = threadIdx.x;
    asm volatile("" : "+v"(tid_here));
    const int lane_here = tid_here & 63, c_here = tid_here & 15, g_here = lane_here >> 4;

    // running key shift (every wave reads the same number)
    dk = fmaxf(dk, sm.kmax[buf]);
    const f32x4 qadd4 = *(const f32x4*)(&sm.qadd[buf][4 * c_here]);
    // no query shift at all when every row's shift is below 40 (Cauchy-Schwarz bound below 2^80)
    const bool noshift = __builtin_amdgcn_readfirstlane((int)(sm.qmax[buf] < 40.f)) != 0;
    cp.q += qstep; cp.k += kstep; cp.v += vstep; cp.rk += TC;     // now the chunk after the next
    // running pointers stay loop-carried scalars (the compiler would otherwise rebuild each of them from the chunk
    // counter with a 64-bit multiplication per chunk)
    asm volatile("" : "+s"(cp.q), "+s"(cp.k), "+s"(cp.v), "+s"(cp.rk));
    const int nv2 = min(TC, cx.row_end - row0 - 2 * TC);
    f32x4 fsum[4] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
    const int sig = sigma_own(lane_here);

#pragma unroll
    for (int S = 0; S < 4; ++S) {
      // operands of the next step's two tiles (after the last step: the first two key tiles of the next chunk, whose
      // key rows went to the other buffer in step 1)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        if (S < 1) load_xop(xo[(S + 1) & 1][u], sm.k[buf], 2 * (S + 1) + u, lane_here);
        else if (S < 3) load_xop(xo[(S + 1) & 1][u], sm.q[buf], 2 * (S - 1) + u, lane_here);
        else load_xop(xo[(S + 1) & 1][u], sm.k[buf ^ 1], u, lane_here);
      }
      __builtin_amdgcn_sched_barrier(0);

      // the two feature tiles of the step, independent of each other
      if (S < 2) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const f32x4 init = *(const f32x4*)(&sm.kadd[buf][16 * (2 * S + u) + 4 * g_here]) - dk;
          key_tile_major(wk, xo[S & 1][u], init, &sm.feat[S & 1][(u * 4 + j) * 1024], sig);
        }
      } else {
        bf16x8 img[2][2];
        if (noshift) {
#pragma unroll
          for (int u = 0; u < 2; ++u) feature_tile64_noshift(wq, qb, xo[S & 1][u], img[u]);
        } else {
#pragma unroll
          for (int u = 0; u < 2; ++u) feature_tile64<true>(wq, &qb, xo[S & 1][u], qadd4[2 * (S - 2) + u], img[u]);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int blk = 0; blk < 2; ++blk) *(bf16x8*)(&sm.feat[S & 1][((u * 4 + j) * 2 + blk) * 512 + lane_here * 8]) = img[u][blk];
      }

      // staging: part S of the next chunk goes to LDS, part S of the chunk after it is requested
      stage_store(stg, sm, buf ^ 1, cx.isoC, row0 + TC, cx.row_end, tid_here, S);
      stage_load_part(stg, cp, cx, a, nv2, tid_here, S);
      // the previous chunk leaves: its partial tiles are summed in step 2 (before the consumers start to overwrite
      // them in interval 4c+3) and stored in step 3 (nothing is stored on the first pass: there is no previous chunk)
      if (S == 2) {
        // the other parity's maxima were last read in interval 4c+1 and are gathered again in the next step
        if (tid_here < 2) { if (tid_here == 0) sm.kmax[buf ^ 1] = -INFINITY; else sm.qmax[buf ^ 1] = -INFINITY; }
        finish_tiles(fsum, sm, j, 0, lane_here);
        finish_tiles(fsum, sm, j, 2, lane_here);
        unsigned zt;
        finish_norm(fsum, sm, j, lane_here, &zt);
        nzero += row0 > cx.row_beg ? __builtin_popcount(zt) : 0;      // (the previous chunk is a whole one)
      }
      if (S == 3) {
        finish_store(fsum, a.Y, yprev, row0 > cx.row_beg ? TC : 0, j, lane_here);
        // per-token constants of the next chunk (its query and key rows are in the other buffer since steps 0, 1)
        row_constants(sm, buf ^ 1, a, cx.isoC, row0 + TC, cx.row_end, wmax1, wmax2, j, lane_here);
      }
      FS_STEP_BARRIER();
    }
    yprev += ystep;
    asm volatile("" : "+s"(yprev));
  }
  FS_STEP_BARRIER();               // the consumers' last step: every partial tile of the last chunk is written
  if (cx.row_end > cx.row_beg) {
    const int last0 = cx.row_beg + ((cx.row_end - cx.row_beg - 1) / TC) * TC;
    f32x4 fsum[4] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
    finish_tiles(fsum, sm, j, 0, lane);
    finish_tiles(fsum, sm, j, 2, lane);
    unsigned zt;
    finish_norm(fsum, sm, j, lane, &zt);
    nzero += count_zero_tokens(zt, j, cx.row_end - last0);
    finish_store(fsum, a.Y, yprev, cx.row_end - last0, j, lane);
  }
  report_zero_rows(a.flushed, nzero, lane);
}

__device__ __forceinline__ void consumer(const FastArgs& a, SmemPC& sm, const SegCtx& cx, int seg, int j) {
  const int lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
  f32x4 T[4][NVT];
  {
    // the prefix state as the state pass left it: accumulator images, 16 bytes per lane and tile
    // (the first segment starts from nothing: with many short sequences every segment is a first one, and a state is
    // more bytes than 128 rows of Q, K, V and Y)
    const float* Tg = a.Tpart + ((size_t)cx.bh * a.nslot + (size_t)seg * a.sub) * M * DVP;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) {
        T[mt][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (seg > 0) T[mt][vt] = *(const f32x4*)(Tg + (size_t)((j * 4 + mt) * NVT + vt) * 256 + 4 * lane);
      }
  }
  float dk = seg > 0 ? a.cstar[gridDim.y + (size_t)cx.bh * a.nslot + (size_t)seg * a.sub] : -INFINITY;   // shift of the prefix state
  FS_STEP_BARRIER();               // barrier 0
  bf16x8 vop[2][NVT];              // value operands of the chunk; the first pair's are requested one step early
#pragma unroll
  for (int vt = 0; vt < NVT; ++vt) vop[0][vt] = load_vop_tr(sm.v[0], 0, vt, lane);
  FS_STEP_BARRIER();               // barrier 1
  FS_STEP_BARRIER();               // the producers' first step

  int buf = 0;
  for (int row0 = cx.row_beg; row0 < cx.row_end; row0 += TC, buf ^= 1) {
    // running key shift (every wave computes the same numbers); the state is rebased when it grows
    {
      const float dnew = sm.kmax[buf];
      if (dnew > dk) {
        const float f = fast_exp2(dk - dnew);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
          for (int vt = 0; vt < NVT; ++vt) T[mt][vt] *= f;
        dk = dnew;
      }
    }
    // state before this chunk as A operand (T^T: row v = 16 vt + c, k <-> feature), one per 32-feature block
    bf16x8 tb[2][NVT];
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) tb[blk][vt] = pack8(T[2 * blk][vt], T[2 * blk + 1][vt]);

    bf16x8 sk[4][2];               // key feature tiles of the chunk, token-major
#pragma unroll
    for (int S = 0; S < 4; ++S) {
      if (S < 2) {
        // key side: a pair of token tiles
        int lane_here = lane;      // unit slots are rebuilt instead of living in registers through the query steps
        asm volatile("" : "+v"(lane_here));
        const uint16_t* blk0 = &sm.feat[S & 1][(0 * 4 + j) * 1024];
        const uint16_t* blk1 = &sm.feat[S & 1][(1 * 4 + j) * 1024];
        const int so = 4 * sigma_own(lane_here), st = 4 * sigma_tr(lane_here);
        // S^T of the pair (lane <-> feature 16 mt + c, contraction index <-> the pair's tokens): two units per tile
        bf16x8 stv[4];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
          stv[mt] = join8(*(const u32x2*)(blk0 + mt * 256 + so), *(const u32x2*)(blk1 + mt * 256 + so));
        // the same numbers token-major for the scores: lane <-> token, contraction index <-> features of a 32-block
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
          sk[2 * S][blk] = join8(lds_read_tr(blk0 + (2 * blk) * 256 + st), lds_read_tr(blk0 + (2 * blk + 1) * 256 + st));
          sk[2 * S + 1][blk] = join8(lds_read_tr(blk1 + (2 * blk) * 256 + st), lds_read_tr(blk1 + (2 * blk + 1) * 256 + st));
        }
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
          for (int vt = 0; vt < NVT; ++vt) T[mt][vt] = mfma(stv[mt], vop[S][vt], T[mt][vt]);
        // the value rows do not wait for the producers' current step: the second pair's operands are requested ahead
        // of the barrier, so that they have arrived behind it
        if (S == 0) {
#pragma unroll
          for (int vt = 0; vt < NVT; ++vt) vop[1][vt] = load_vop_tr(sm.v[buf], 1, vt, lane_here);
        }
      } else {
        // both tiles' query images are requested before the first one is used
        bf16x8 pq[2][2];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int blk = 0; blk < 2; ++blk) pq[u][blk] = *(const bf16x8*)(&sm.feat[S & 1][((u * 4 + j) * 2 + blk) * 512 + lane * 8]);
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
                  sc[jj] = mfma(sk[jt][0], p[0], sc[jj]);
                  sc[jj] = mfma(sk[jt][1], p[1], sc[jj]);
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
          // hand the partial tile over (bf16): rows v = 16 vt + 4g + r of token column c
#pragma unroll
          for (int vt = 0; vt < NVT; ++vt)
            *(bf16x4*)(&sm.xch[it][j][c][16 * vt + 4 * g]) = __builtin_convertvector(y[vt], bf16x4);
        }
        // the next chunk's value rows are in the other buffer since the producers' step 3 of this chunk (one interval
        // ago): its first pair's operands, ahead of the barrier
        if (S == 3) {
#pragma unroll
          for (int vt = 0; vt < NVT; ++vt) vop[0][vt] = load_vop_tr(sm.v[buf ^ 1], 0, vt, lane);
        }
      }
      FS_STEP_BARRIER();
    }
  }
}

}  // namespace pc

using namespace pc;

// grid (nseg, B*H), block 512.
__global__ void __launch_bounds__(NT8) k_fast_causal(FastArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  SmemPC& sm = *reinterpret_cast<SmemPC*>(smem_raw);
  const int seg = blockIdx.x, bh = blockIdx.y, b = bh / a.H, h = bh % a.H;
  const float* th = a.theta + (size_t)group_of(a.groups, b, h, a.H) * (FS_THETA_HEADER_ + (size_t)D + 4 * (size_t)D * D);
  const int flags = (int)th[2];
  SegCtx cx;
  cx.isoC = flags & 1;
  cx.bh = bh;
  cx.pg = group_of(a.pgroups, b, h, a.H);
  cx.Qb = (const uint16_t*)a.Q.ptr + b * a.Q.sb + h * a.Q.sh;
  cx.Kb = (const uint16_t*)a.K.ptr + b * a.K.sb + h * a.K.sh;
  cx.Vb = (const uint16_t*)a.V.ptr + b * a.V.sb + h * a.V.sh;
  cx.ybase = b * a.Y.sb + h * a.Y.sh;
  cx.row_beg = seg * a.rows_per_seg;
  cx.row_end = min(a.L, cx.row_beg + a.rows_per_seg);
  init_value_pad(sm.v[0], 2 * TC, NT8);
  const int w = threadIdx.x >> 6;
  if (w < 4) producer(a, sm, cx, w);
  else consumer(a, sm, cx, seg, w - 4);
}

size_t fast_causal_lds_bytes() { return sizeof(SmemPC); }

int launch_fast_causal_kernel(const FastArgs& a, int BH, hipStream_t st, hipEvent_t ev_begin, hipEvent_t ev_end) {
  if (hipFuncSetAttribute((const void*)k_fast_causal, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(SmemPC)) !=
      hipSuccess) {
    (void)hipGetLastError();
    return 2;
  }
  // with events: they are attached to the dispatch itself and carry the kernel's own begin and end times (events
  // recorded before and after it on the stream would add the gaps of two more queue packets)
  if (ev_begin || ev_end) hipExtLaunchKernelGGL(k_fast_causal, dim3(a.nseg, BH), dim3(NT8), sizeof(SmemPC), st, ev_begin, ev_end, 0, a);
  else hipLaunchKernelGGL(k_fast_causal, dim3(a.nseg, BH), dim3(NT8), sizeof(SmemPC), st, a);
  if (hipGetLastError() != hipSuccess) return 5;
  return 0;
}

}  // namespace fs
