// bf16 path of FAVOR# attention (d = dv = 64, M = 256): projection constants, key row terms, key-side segment
// states (the loop itself: fast_state.h), their reduction / prefix, the non-causal query-side kernel, the kernel that
// takes a whole non-causal sequence per workgroup, and the host-side launchers of the forward and backward calls.
// The design is described in fast_common.h; the causal segment kernel lives in kernels_bf16_causal.hip.
#include <hip/hip_ext.h>

#include <algorithm>
#include <cstddef>

#include "fast_pc.h"
#include "fast_state.h"

namespace fs {

using namespace fast;

// ---------------------------------------------------------------------------------------------------
// Projection constants (Section 4, evaluation recipe), one launch of 128 * pgroups workgroups of 256 threads, one
// wave per feature, one lane per column: Wbf[pg][side][m][:] = bf16(qk_scale log2e omega_m^T B), bias[pg][side][m] =
// log2e (omega_m^T A omega_m + log D - 1/2 log M), wnorm[pg][side][m] = |Wbf_m|.
// dense_flag (optional) is or-ed with 1 when a visited parameter set has a dense C2.
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_fast_pre(const float* theta, int groups, const float* Omega, int omega_groups,
                                                  int pgroups, int B, int H, float scale, uint16_t* Wbf, float* bias,
                                                  float* wnorm, int* dense_flag) {
  const size_t tf = FS_THETA_HEADER_ + (size_t)D + 4 * (size_t)D * D;
  const int block = blockIdx.x;
  {
    const int pg = block / ((M / 4) * 2), rem = block % ((M / 4) * 2), side = rem / (M / 4);
    const int m = (rem % (M / 4)) * 4 + (threadIdx.x >> 6), c = threadIdx.x & 63;
    int b = 0, h = 0;
    if (pgroups == H && pgroups != 1) h = pg;
    else if (pgroups != 1) { b = pg / H; h = pg % H; }
    const float* th = theta + (size_t)group_of(groups, b, h, H) * tf;
    if (dense_flag != nullptr && rem == 0 && threadIdx.x == 0 && !(((int)th[2]) & 1)) atomicOr(dense_flag, 1);
    const float* om = Omega + ((size_t)group_of(omega_groups, b, h, H) * M + m) * D;
    const float* Bm = th + FS_THETA_HEADER_ + D + (side ? (size_t)D * D : 0);
    const float* A = th + FS_THETA_HEADER_;
    const size_t o = ((size_t)pg * 2 + side) * M + m;
    // omega_m^T B, column c: the lane's column of B is requested whole (64 loads in flight, one memory latency),
    // omega_m sits one number per lane and is read across the wave
    float bcol[D];
#pragma unroll
    for (int l = 0; l < D; ++l) bcol[l] = Bm[l * D + c];
    const float om_c = om[c];
    float acc = 0.f;
#pragma unroll
    for (int l = 0; l < D; ++l) acc += __shfl(om_c, l) * bcol[l];
    const uint16_t bits = f32_to_bf16_bits(acc * kLog2e * scale);
    Wbf[o * D + c] = bits;
    const float r = bf16_bits_to_f32(bits);
    float n2 = r * r, q = A[c] * om_c * om_c;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) { n2 += __shfl_xor(n2, s); q += __shfl_xor(q, s); }
    if (c == 0) {
      bias[o] = kLog2e * (q + th[0] - 0.5f * logf((float)M));
      wnorm[o] = sqrtf(n2);
    }
  }
}

// ---------------------------------------------------------------------------------------------------
// Key-side row terms rk[bh][j] = log2e * y_j^T C2 y_j, y_j = qk_scale K_j (the quadratic form of the DERF exponent,
// Section 4), for parameter sets whose C2 is not -I/2 (ADERF, SADERF; workgroups of sets with the -I/2 flag return at
// once: the kernels then use -|y|^2/2), for bf16 rows of DD = 64 or 128 numbers.
//
// C2 y runs on the MFMA pipe.  The rows are bf16 as they come; C2 is split into two bf16 parts, C2 = hi + lo with
// |C2 - hi - lo| <= 2^-17 |C2|, so the fp32 sums carry the accuracy of an fp32 product (the term is an exponent:
// bf16 entries of C2 alone would shift it by tenths).  Both parts lie in LDS as operand images (rows a of C2 as
// the A operand: lane (g, c) <-> row 16 mt + c, contraction index 32 ks + 8 g + e); a wave takes 64 tokens at a
// time, its rows straight from memory as B operands (lane <-> token, the same contraction index), and for every
// block of 16 rows of C2 gets (C2 y)[a] for a = 16 mt + 4 g + r of token c in its accumulators, multiplies by y[a]
// (an 8-byte read of the row) and sums over the lane's numbers; two cross-lane steps finish the token.
// grid (blocks per sequence, B*H), block 256 (DD = 64) or 512 (DD = 128: the images take 64 kB, so two workgroups
// share a CU and eight waves each keep four waves per SIMD); the waves of a sequence stride over its groups of 64
// tokens.
// ---------------------------------------------------------------------------------------------------
template <int DD>
__global__ void __launch_bounds__(4 * DD, 2) k_key_row_terms(const float* theta, int groups, TensorDev K, int L, int H,
                                                       float scale, float* rk) {
  constexpr int NMT = DD / 16, NKS = DD / 32, NTH = 4 * DD, NWV = NTH / 64;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  typedef uint16_t OpImage[NMT][NKS][64][8];
  OpImage* c2op = reinterpret_cast<OpImage*>(smem_raw);        // [hi / lo]
  const int bh = blockIdx.y, b = bh / H, h = bh % H;
  const float* th = theta + (size_t)group_of(groups, b, h, H) * (FS_THETA_HEADER_ + (size_t)DD + 4 * (size_t)DD * DD);
  if (((int)th[2]) & 1) return;
  const float* C2 = th + FS_THETA_HEADER_ + DD + 3 * (size_t)DD * DD;
  for (int idx = threadIdx.x; idx < NMT * NKS * 64; idx += NTH) {
    const int l = idx & 63, ks = (idx >> 6) % NKS, mt = idx / (64 * NKS);
    const float* src = C2 + (size_t)(16 * mt + (l & 15)) * DD + 32 * ks + 8 * (l >> 4);
    u32x4 hi4 = {0u, 0u, 0u, 0u}, lo4 = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float v = src[e];
      const uint16_t hi = f32_to_bf16_bits(v);
      hi4[e >> 1] |= (uint32_t)hi << (16 * (e & 1));
      lo4[e >> 1] |= (uint32_t)f32_to_bf16_bits(v - bf16_bits_to_f32(hi)) << (16 * (e & 1));
    }
    *(u32x4*)(&c2op[0][mt][ks][l][0]) = hi4;
    *(u32x4*)(&c2op[1][mt][ks][l][0]) = lo4;
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  const uint16_t* Kb = (const uint16_t*)K.ptr + b * K.sb + h * K.sh;
  for (int t0 = (blockIdx.x * NWV + w) * 64; t0 < L; t0 += gridDim.x * NWV * 64) {
    // the rows of the group as B operands (a buffer descriptor that ends with the last row: rows past it read as zero)
    u32x4 yb[4][NKS];
    const __amdgpu_buffer_rsrc_t rs = pc::chunk_rsrc(Kb + (long long)t0 * K.sl, 2 * (int)K.sl, min(64, L - t0), 2 * DD);
#pragma unroll
    for (int tile = 0; tile < 4; ++tile)
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks)
        yb[tile][ks] = __builtin_amdgcn_raw_buffer_load_b128(rs, 2 * ((16 * tile + c) * (int)K.sl + 32 * ks + 8 * g), 0, 0);
    float part[4] = {0.f, 0.f, 0.f, 0.f};
    // (an opaque copy of the lane number: the images do not depend on the group, and reading all of them once,
    // ahead of the loop, would not fit in the registers)
    int lane_here = lane;
    asm volatile("" : "+v"(lane_here));
#pragma unroll
    for (int mt = 0; mt < NMT; ++mt) {
      __builtin_amdgcn_sched_barrier(0);     // block by block: not every block's LDS reads at the top
      f32x4 acc[4];
#pragma unroll
      for (int tile = 0; tile < 4; ++tile) acc[tile] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        const bf16x8 hi = *(const bf16x8*)(&c2op[0][mt][ks][lane_here][0]), lo = *(const bf16x8*)(&c2op[1][mt][ks][lane_here][0]);
#pragma unroll
        for (int tile = 0; tile < 4; ++tile) {
          acc[tile] = mfma(hi, __builtin_bit_cast(bf16x8, yb[tile][ks]), acc[tile]);
          acc[tile] = mfma(lo, __builtin_bit_cast(bf16x8, yb[tile][ks]), acc[tile]);
        }
      }
      // y[a] for a = 16 mt + 4 g + r of the lane's token: the numbers are in the operand registers of the lane with
      // the same token and lane group 2 (mt % 2) + g / 2 (k-step mt / 2, its dwords 2 (g % 2) and 2 (g % 2) + 1)
      const int src = 4 * (16 * (2 * (mt & 1) + (g >> 1)) + c);
#pragma unroll
      for (int tile = 0; tile < 4; ++tile) {
        const u32x4 v = yb[tile][mt >> 1];
        const uint32_t d0 = __builtin_amdgcn_ds_bpermute(src, v[0]), d1 = __builtin_amdgcn_ds_bpermute(src, v[1]);
        const uint32_t d2 = __builtin_amdgcn_ds_bpermute(src, v[2]), d3 = __builtin_amdgcn_ds_bpermute(src, v[3]);
        const u32x2 pr = {(g & 1) ? d2 : d0, (g & 1) ? d3 : d1};
        const f32x4 yf = __builtin_convertvector(__builtin_bit_cast(bf16x4, pr), f32x4);
#pragma unroll
        for (int r = 0; r < 4; ++r) part[tile] += acc[tile][r] * yf[r];
      }
    }
#pragma unroll
    for (int tile = 0; tile < 4; ++tile) {
      float p = part[tile];
      p += __shfl_xor(p, 16);
      p += __shfl_xor(p, 32);
      const int token = t0 + 16 * tile + c;
      if (g == 0 && token < L) rk[(size_t)bh * L + token] = kLog2e * scale * scale * p;
    }
  }
}

int launch_key_row_terms(const float* theta, int groups, const TensorDev& K, int B, int H, int L, int d, float scale,
                         float* rk, hipStream_t st) {
  // every wave of a sequence gets about four groups of 64 tokens, so that the operand images are built rarely
  const int BH = B * H, waves = d / 16, per_block = 4 * 64 * waves;
  const int blocks = std::max(1, std::min((L + per_block - 1) / per_block, std::max(1, 2048 / BH)));
  const size_t lds = (size_t)2 * d * d * sizeof(uint16_t);
  if (d == 64) {
    hipLaunchKernelGGL(k_key_row_terms<64>, dim3(blocks, BH), dim3(256), lds, st, theta, groups, K, L, H, scale, rk);
  } else if (d == 128) {
    if (hipFuncSetAttribute((const void*)k_key_row_terms<128>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
      (void)hipGetLastError();
      return 2;
    }
    hipLaunchKernelGGL(k_key_row_terms<128>, dim3(blocks, BH), dim3(512), lds, st, theta, groups, K, L, H, scale, rk);
  } else {
    return 2;
  }
  if (hipGetLastError() != hipSuccess) return 5;
  return 0;
}

// Key-side state of one slot (fast_state.h: state_rows), written to Tpart with its shift in cpart.  grid (nslot, B*H),
// block 256, two workgroups per CU.
__global__ void __launch_bounds__(NT, 2) k_fast_state(FastArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int slot = blockIdx.x, bh = blockIdx.y;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  const int rows_per_slot = a.rows_per_seg / a.sub;
  const int row_beg = slot * rows_per_slot;
  f32x4 T[4][NVT];
  float dk;
  state_rows(a, *reinterpret_cast<SmemState*>(smem_raw), bh, row_beg, min(a.L, row_beg + rows_per_slot), T, dk);
  float* out = a.Tpart + ((size_t)bh * a.nslot + slot) * M * DVP;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt) {
      if (a.timg) {
        *(f32x4*)(out + (size_t)((w * 4 + mt) * NVT + vt) * 256 + 4 * lane) = T[mt][vt];
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) out[(size_t)(64 * w + 16 * mt + 4 * g + r) * DVP + 16 * vt + c] = T[mt][vt][r];
      }
    }
  if (threadIdx.x == 0) a.cpart[(size_t)bh * a.nslot + slot] = dk;
}

// The key shift of every sequence without the states (causal backward pass with one slot per sequence: its kernels
// start from nothing and need the shift only): cstar[bh] = the largest bound of the sequence's keys, as the state
// kernel would have left it.  Also puts the call's counter of flushed rows back to zero.  grid (B*H), block 256.
__global__ void __launch_bounds__(NT, 2) k_fast_bound(FastArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int bh = blockIdx.x;
  f32x4 T[4][NVT];
  float dk;
  state_rows<true>(a, *reinterpret_cast<SmemState*>(smem_raw), bh, 0, a.L, T, dk);
  if (threadIdx.x == 0) {
    a.cstar[bh] = dk;
    if (bh == 0 && a.flushed != nullptr) *a.flushed = 0u;
  }
}

// Brings the segment states of one (b,h) to the common shift c* = max_seg cpart and sums them (prefix = 0: total
// in slot 0) or replaces them by their exclusive prefix sums (prefix = 1).  prefix = 2: exclusive prefix sums on
// running shifts: the prefix of slot s is scaled by the largest shift of the slots before it (written behind the
// per-sequence shifts, at cstar[B*H + bh * nseg + s]; -inf and a zero state for slot 0), so that keys late in the
// sequence cannot push the states the earlier rows need out of the fp32 range.  grid (ceil(M*DVP/1024), B*H).
__global__ void k_fast_reduce(float* Tpart, const float* cpart, float* cstar, int nseg, int nseg_valid, int prefix,
                              int sub, unsigned* flushed) {
  const int bh = blockIdx.y;
  // the query-side kernel of the call counts into this word: it starts every call at zero
  if (flushed != nullptr && (blockIdx.x | blockIdx.y | threadIdx.x) == 0) *flushed = 0u;
  constexpr size_t per = (size_t)M * DVP;
  const size_t e = 4 * ((size_t)blockIdx.x * blockDim.x + threadIdx.x);      // four consecutive numbers per thread
  float* p = Tpart + (size_t)bh * nseg * per + e;
  f32x4 run = {0.f, 0.f, 0.f, 0.f};
  // The slots are taken eight at a time: all of a batch's loads are requested before the first number is used (one
  // memory latency per batch instead of one per slot: with few sequences and hundreds of slots the kernel is a chain
  // of latencies), and a slot is overwritten only after its batch was read.
  constexpr int NB = 8;
  if (prefix == 2) {
    float* cpre = cstar + gridDim.y + (size_t)bh * nseg;
    float cr = -INFINITY;
    for (int s0 = 0; s0 < nseg; s0 += NB) {
      f32x4 v[NB];
      float c[NB];
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int s = s0 + i;
        v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        c[i] = -INFINITY;
        if (s < nseg_valid) {
          c[i] = cpart[(size_t)bh * nseg + s];
          if (e < per) v[i] = *(const f32x4*)(p + (size_t)s * per);
        }
      }
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int s = s0 + i;
        if (s < nseg && s % sub == 0) {            // only the slots that open a segment are read back
          if (e == 0) cpre[s] = cr;
          if (e < per) *(f32x4*)(p + (size_t)s * per) = run;
        }
        if (s < nseg_valid) {
          if (c[i] > cr) { run *= fast_exp2(cr - c[i]); cr = c[i]; }
          run += v[i] * fast_exp2(c[i] - cr);
        }
      }
    }
    if (e == 0) cstar[bh] = cr;
    return;
  }
  float cs = -INFINITY;
  for (int s = 0; s < nseg_valid; ++s) cs = fmaxf(cs, cpart[(size_t)bh * nseg + s]);
  if (e == 0) cstar[bh] = cs;
  if (e >= per) return;
  for (int s0 = 0; s0 < nseg; s0 += NB) {
    f32x4 v[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int s = s0 + i;
      v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (s < nseg_valid) v[i] = *(const f32x4*)(p + (size_t)s * per) * fast_exp2(cpart[(size_t)bh * nseg + s] - cs);
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int s = s0 + i;
      if (prefix && s < nseg && s % sub == 0) *(f32x4*)(p + (size_t)s * per) = run;    // only the slots that open a segment are read back
      run += v[i];
    }
  }
  if (!prefix) *(f32x4*)p = run;
}

// The same reduction for few sequences with many slots (one sequence of 262144 rows has 512 of them, and twenty
// workgroups walking them one after the other take longer than the two kernels around them): the slots are cut into
// ranges of R, one workgroup row per range.
//   k_fast_reduce_totals  range z: sum of its slots on the range's own largest shift -> scr[bh][z], cscr[bh][z]
//   k_fast_reduce         over the Z totals (sum, or exclusive prefixes on running shifts), in place in scr
//   k_fast_reduce_walk    (causal) range z: the exclusive prefixes of its slots as k_fast_reduce (prefix = 2) writes
//                         them, starting from the prefix and the shift of the range
// Sums are taken in another order than by the one-kernel form: the results agree to rounding, not bit for bit.
// grid (ceil(M*DVP/1024), B*H, Z).
__global__ void k_fast_reduce_totals(const float* Tpart, const float* cpart, float* scr, float* cscr, int nseg,
                                     int nseg_valid, int R) {
  const int bh = blockIdx.y, z = blockIdx.z, Z = gridDim.z;
  constexpr size_t per = (size_t)M * DVP;
  const size_t e = 4 * ((size_t)blockIdx.x * blockDim.x + threadIdx.x);
  const int s_beg = z * R, s_end = min(nseg_valid, s_beg + R);
  float m = -INFINITY;
  for (int s = s_beg; s < s_end; ++s) m = fmaxf(m, cpart[(size_t)bh * nseg + s]);
  if (e == 0) cscr[(size_t)bh * Z + z] = m;
  if (e >= per) return;
  const float* p = Tpart + (size_t)bh * nseg * per + e;
  f32x4 run = {0.f, 0.f, 0.f, 0.f};
  constexpr int NB = 8;
  for (int s0 = s_beg; s0 < s_end; s0 += NB) {
    f32x4 v[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int s = s0 + i;
      v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (s < s_end) v[i] = *(const f32x4*)(p + (size_t)s * per) * fast_exp2(cpart[(size_t)bh * nseg + s] - m);
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) run += v[i];
  }
  *(f32x4*)(scr + ((size_t)bh * Z + z) * per + e) = run;
}

// `base` = scr after the scan (exclusive prefix of range z), `cbase` = the scan's shifts (largest shift of the ranges
// before z at cbase[B*H + bh * Z + z]).
__global__ void k_fast_reduce_walk(float* Tpart, const float* cpart, float* cstar, const float* base, const float* cbase,
                                   int nseg, int nseg_valid, int sub, int R, unsigned* flushed) {
  const int bh = blockIdx.y, z = blockIdx.z, Z = gridDim.z;
  if (flushed != nullptr && (blockIdx.x | blockIdx.y | blockIdx.z | threadIdx.x) == 0) *flushed = 0u;
  constexpr size_t per = (size_t)M * DVP;
  const size_t e = 4 * ((size_t)blockIdx.x * blockDim.x + threadIdx.x);
  float* p = Tpart + (size_t)bh * nseg * per + e;
  float* cpre = cstar + gridDim.y + (size_t)bh * nseg;
  const int s_beg = z * R, s_end = min(nseg, s_beg + R);
  f32x4 run = {0.f, 0.f, 0.f, 0.f};
  if (e < per) run = *(const f32x4*)(base + ((size_t)bh * Z + z) * per + e);
  float cr = cbase[gridDim.y + (size_t)bh * Z + z];
  constexpr int NB = 8;
  for (int s0 = s_beg; s0 < s_end; s0 += NB) {
    f32x4 v[NB];
    float c[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int s = s0 + i;
      v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      c[i] = -INFINITY;
      if (s < s_end && s < nseg_valid) {
        c[i] = cpart[(size_t)bh * nseg + s];
        if (e < per) v[i] = *(const f32x4*)(p + (size_t)s * per);
      }
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int s = s0 + i;
      if (s < s_end && s % sub == 0) {
        if (e == 0) cpre[s] = cr;
        if (e < per) *(f32x4*)(p + (size_t)s * per) = run;
      }
      if (s < s_end && s < nseg_valid) {
        if (c[i] > cr) { run *= fast_exp2(cr - c[i]); cr = c[i]; }
        run += v[i] * fast_exp2(c[i] - cr);
      }
    }
  }
  if (e == 0 && z == Z - 1) cstar[bh] = cr;
}

// ---------------------------------------------------------------------------------------------------
// Query side of the non-causal contraction: Y = (P T) normalised by its last column (Sections 2.1, 2.2) for a block
// of query rows; T = total state of the (b,h) (slot 0 of Tpart).  Four waves of 64 features; the partial output
// tiles cross the waves as bf16 and are summed on the MFMA pipe.  The kernel needs a third of the LDS of the
// key-side kernels and at most 256 registers, so two workgroups share a CU (two waves per SIMD: one's exp2 and
// convert work beside the other's MFMAs and memory waits).  grid (nblk, B*H), block 256.
// ---------------------------------------------------------------------------------------------------
// Rows [row_beg, row_end) of the queries of one (b,h) against the state image tb (T^T as A operand: row v = 16 vt + c,
// k <-> features 64w + 32 mb + 16 (e/4) + 4g + e%4).  Returns the number of rows this wave finished with a zero
// normaliser.
__device__ __forceinline__ int apply_rows(const FastArgs& a, SmemApply& sm, int bh, const bf16x8 (&tb)[NVT][2], int row_beg,
                                          int row_end) {
  const int b = bh / a.H, h = bh % a.H;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  const int pg = group_of(a.pgroups, b, h, a.H);
  const float wmax = max256(a.wnorm + ((size_t)pg * 2) * M), amax = max256(a.bias + ((size_t)pg * 2) * M);
  const uint16_t* Qb = (const uint16_t*)a.Q.ptr + b * a.Q.sb + h * a.Q.sh;
  const long long ybase = b * a.Y.sb + h * a.Y.sh;
  WSlice wq;
  load_wslice(wq, a.Wbf + ((size_t)pg * 2) * M * D);
  QBias qb;
  load_qbias(qb, a.bias + ((size_t)pg * 2) * M, amax);
  RowRegs qr;
  load_rows_g(qr, Qb, a.Q.sl, row_beg, row_end);
  store_query_rows(qr, sm, 0, wmax);
  __syncthreads();
  int buf = 0, nzero = 0;
  for (int row0 = row_beg; row0 < row_end; row0 += TC, buf ^= 1) {
    const bool more = row0 + TC < row_end;
    if (more) load_rows_g(qr, Qb, a.Q.sl, row0 + TC, row_end);
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      bf16x8 p[2];
      feature_tile<true>(wq, &qb, sm.q[buf], it, sm.qadd[buf][16 * it + c], p);
      f32x4 y[NVT];
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) {
        y[vt] = mfma(tb[vt][0], p[0], f32x4{0.f, 0.f, 0.f, 0.f});
        y[vt] = mfma(tb[vt][1], p[1], y[vt]);
      }
      exchange_put_bf16(sm, y, it, w, lane);
    }
    __syncthreads();
    // wave w sums the four partial tiles of token tile w, normalises and stores
    {
      f32x4 fs[4] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
      finish_tiles(fs, sm, w, 0, lane);
      finish_tiles(fs, sm, w, 2, lane);
      unsigned zt;
      finish_norm(fs, sm, w, lane, &zt);
      nzero += count_zero_tokens(zt, w, row_end - row0);
      const int token = row0 + 16 * w + c;
      if (token < row_end) {
        if (a.Y.dtype == 1) {
          uint16_t* yp = (uint16_t*)a.Y.ptr + ybase + (long long)token * a.Y.sl + 4 * g;
#pragma unroll
          for (int vt = 0; vt < 4; ++vt) *(bf16x4*)(yp + 16 * vt) = __builtin_convertvector(fs[vt], bf16x4);
        } else {
          float* yp = (float*)a.Y.ptr + ybase + (long long)token * a.Y.sl + 4 * g;
#pragma unroll
          for (int vt = 0; vt < 4; ++vt) *(f32x4*)(yp + 16 * vt) = fs[vt];
        }
      }
    }
    if (more) store_query_rows(qr, sm, buf ^ 1, wmax);
    __syncthreads();
  }
  return nzero;
}

__global__ void __launch_bounds__(NT, 2) k_fast_apply(FastArgs a, int Lq, int rows_per_blk) {
  __shared__ SmemApply sm;
  const int blk = blockIdx.x, bh = blockIdx.y;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  bf16x8 tb[NVT][2];
  const float* Tg = a.Tpart + (size_t)bh * a.nslot * M * DVP;
#pragma unroll
  for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      // accumulator images of tiles (2 mb, vt) and (2 mb + 1, vt) of wave w (the forward state pass writes images)
      const f32x4 lo = *(const f32x4*)(Tg + (size_t)((w * 4 + 2 * mb) * NVT + vt) * 256 + 4 * lane);
      const f32x4 hi = *(const f32x4*)(Tg + (size_t)((w * 4 + 2 * mb + 1) * NVT + vt) * 256 + 4 * lane);
      tb[vt][mb] = pack8(lo, hi);
    }
  const int row_beg = blk * rows_per_blk;
  const int nzero = apply_rows(a, sm, bh, tb, row_beg, min(Lq, row_beg + rows_per_blk));
  report_zero_rows(a.flushed, nzero, lane);
}

// ---------------------------------------------------------------------------------------------------
// Non-causal call, one workgroup per (b,h): the state of all keys, then all query rows against it, the state never
// leaving the registers (with many short sequences the states' way through memory, 80 kB each written and read
// again, outweighs the rows themselves: a sequence of 128 tokens is 64 kB of Q, K, V, Y).  The shift of the state
// cancels in the normalised rows.  grid (B*H), block 256, two workgroups per CU.
// ---------------------------------------------------------------------------------------------------
union SmemWhole {
  SmemState s;
  SmemApply q;
};

__global__ void __launch_bounds__(NT, 2) k_fast_whole(FastArgs a, int Lq) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int bh = blockIdx.x, lane = threadIdx.x & 63;
  bf16x8 tb[NVT][2];
  {
    f32x4 T[4][NVT];
    float dk;
    state_rows(a, *reinterpret_cast<SmemState*>(smem_raw), bh, 0, a.L, T, dk);
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) tb[vt][mb] = pack8(T[2 * mb][vt], T[2 * mb + 1][vt]);
  }
  const int nzero = apply_rows(a, *reinterpret_cast<SmemApply*>(smem_raw), bh, tb, 0, Lq);
  report_zero_rows(a.flushed, nzero, lane);
}

// ---------------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------------
#define FS_LAUNCH_CHECK() do { if (hipGetLastError() != hipSuccess) return 5; } while (0)

// Largest dynamic / static LDS request of the forward kernels of this path (the causal kernel's is the largest).
size_t fast_lds_bytes() { return std::max({sizeof(SmemState), sizeof(SmemApply), fast_causal_lds_bytes()}); }

bool fast_supported(int dtype, int d, int dv, int M_) { return dtype == 1 && d == D && dv == D && M_ == M; }

void fast_reduce_ranges(int BH, int nslot, int* Z, int* R) {
  *Z = 1;
  *R = nslot;
  if (BH <= 8 && nslot >= 64) {
    *R = 16;
    *Z = (nslot + 15) / 16;
  }
}

void fast_plan(int BH, int L, int* nseg, int* rows_per_seg, int* sub) {
  int want = std::max(1, std::min((256 + BH - 1) / BH, (L + TC - 1) / TC));
  *rows_per_seg = (((L + want - 1) / want) + TC - 1) / TC * TC;
  *nseg = (L + *rows_per_seg - 1) / *rows_per_seg;
  // the key-side kernel runs two workgroups per CU: give it half-segments when they are whole chunks
  *sub = (*rows_per_seg % (2 * TC) == 0) ? 2 : 1;
}

// ---------------------------------------------------------------------------------------------------
// Statistics scan of the fits for bf16 rows of 64 numbers (Section 4: mu4, mu5, M1, M2 are means of x, y, x x^T,
// y y^T): per (b,h), tensor and row chunk, sum x and sum x x^T on bf16 MFMA tiles.  The rows of a 64-token tile are
// staged transposed ([number][token], a row of ones appended), so that one operand layout (lane <-> number, k <->
// tokens) serves both sides of X^T X and the ones row yields the column sums.  Wave w owns the Gram tiles (w, 0..3)
// and the 16 column sums of block w.  Output layout as the general kernel's: part[which][bh][chunk][d*d + d], with
// qk_scale applied (squared on the Gram part).  grid (nchunks, B*H, 2), block 256.
// ---------------------------------------------------------------------------------------------------
struct SmemStats { uint16_t vt[2][DVP][LDJ]; };

__global__ void __launch_bounds__(NT) k_stats_bf16(TensorDev X, TensorDev Yt, int Lx, int Ly, int H, float scale,
                                                   int rows_per_chunk, int nchunks, float* part) {
  __shared__ SmemStats sm;
  const int which = blockIdx.z, bh = blockIdx.y, b = bh / H, h = bh % H, chunk = blockIdx.x;
  const TensorDev& T = which ? Yt : X;
  const int L = which ? Ly : Lx;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
  const uint16_t* base = (const uint16_t*)T.ptr + b * T.sb + h * T.sh;
  for (int idx = threadIdx.x; idx < 2 * (DVP - D - 1) * LDJ; idx += NT) {
    const int bb = idx / ((DVP - D - 1) * LDJ), rem = idx - bb * (DVP - D - 1) * LDJ;
    sm.vt[bb][D + 1 + rem / LDJ][rem % LDJ] = 0;
  }
  f32x4 acc[4], sums = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int bt = 0; bt < 4; ++bt) acc[bt] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int row_beg = chunk * rows_per_chunk, row_end = min(L, row_beg + rows_per_chunk);
  RowRegs r;
  load_vals_g(r, base, T.sl, row_beg, row_end);
  store_vals_s(r, sm.vt[0], row_beg, row_end);
  __syncthreads();
  int buf = 0;
  for (int row0 = row_beg; row0 < row_end; row0 += TC, buf ^= 1) {
    const bool more = row0 + TC < row_end;
    if (more) load_vals_g(r, base, T.sl, row0 + TC, row_end);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const bf16x8 mine = load_vop(sm.vt[buf], ks, w);
      const bf16x8 ones = load_vop(sm.vt[buf], ks, 4);
#pragma unroll
      for (int bt = 0; bt < 4; ++bt) acc[bt] = mfma(mine, load_vop(sm.vt[buf], ks, bt), acc[bt]);
      sums = mfma(ones, mine, sums);
    }
    if (more) store_vals_s(r, sm.vt[buf ^ 1], row0 + TC, row_end);
    __syncthreads();
  }
  float* out = part + (((size_t)which * gridDim.y + bh) * nchunks + chunk) * ((size_t)D * D + D);
  const float s2 = scale * scale;
#pragma unroll
  for (int bt = 0; bt < 4; ++bt)
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) out[(size_t)(16 * w + 4 * g + rr) * D + 16 * bt + c] = s2 * acc[bt][rr];
  if (g == 0) out[(size_t)D * D + 16 * w + c] = scale * sums[0];
}

bool stats_bf16_supported(const TensorDev& X, const TensorDev& Y, int d) {
  return X.dtype == 1 && Y.dtype == 1 && d == D;
}

int launch_stats_bf16(const TensorDev& X, const TensorDev& Y, int BH, int H, int Lx, int Ly, float scale,
                      int rows_per_chunk, int nchunks, float* part, hipStream_t st) {
  hipLaunchKernelGGL(k_stats_bf16, dim3(nchunks, BH, 2), dim3(NT), 0, st, X, Y, Lx, Ly, H, scale, rows_per_chunk, nchunks,
                     part);
  FS_LAUNCH_CHECK();
  return 0;
}

// Kernel arguments of a call, its projection constants and, for parameter sets with a dense C2, the key row terms.
static int launch_fast_constants(const FastLaunch& f, FastArgs& a, hipStream_t st, bool images) {
  a.Q = f.Q; a.K = f.K; a.V = f.V; a.Y = f.Y;
  a.Wbf = f.Wbf; a.bias = f.bias; a.wnorm = f.wnorm; a.theta = f.theta; a.rk = f.rk;
  a.Tpart = f.Tpart; a.cpart = f.cpart; a.cstar = f.cstar;
  a.groups = f.groups; a.pgroups = f.pgroups; a.H = f.H; a.L = f.Lk; a.rows_per_seg = f.rows_per_seg; a.nseg = f.nseg;
  a.sub = f.sub; a.nslot = f.nseg * f.sub;
  a.timg = images ? 1 : 0;
  a.scale = f.scale;
  a.flushed = f.flushed;
  if (f.pre_mode == 0) {
    hipLaunchKernelGGL(k_fast_pre, dim3((M / 4) * 2 * f.pgroups), dim3(256), 0, st, f.theta, f.groups, f.Omega,
                       f.omega_groups, f.pgroups, f.B, f.H, f.scale, f.Wbf, f.bias, f.wnorm, (int*)nullptr);
    FS_LAUNCH_CHECK();
  }
  // the key row terms of parameter sets with a dense C2 (the host knows that there are none only in mode 2)
  if (f.pre_mode != 2)
    if (int rc = launch_key_row_terms(f.theta, f.groups, f.K, f.B, f.H, f.Lk, D, f.scale, f.rk, st)) return rc;
  return 0;
}

// Constants, key-side segment states and their reduction (sum, or exclusive prefix when causal).
// `every_slot`: states of all slots (the last segment's too) and, when causal, the exclusive prefix of every slot.
static int launch_fast_state_pass(const FastLaunch& f, FastArgs& a, hipStream_t st, bool every_slot = false, bool images = false) {
  if (int rc = launch_fast_constants(f, a, st, images)) return rc;
  const int BH = f.B * f.H;
  // the last segment's states are never needed by the causal pass
  const int nstate = (f.causal && !every_slot ? f.nseg - 1 : f.nseg) * f.sub;
  if (nstate > 0) {
    hipLaunchKernelGGL(k_fast_state, dim3(nstate, BH), dim3(NT), sizeof(SmemState), st, a);
    FS_LAUNCH_CHECK();
  }
  const int prefix = f.causal ? (every_slot ? 1 : 2) : 0, nblk = (M * DVP / 4 + 255) / 256;
  if (prefix == 2 && nstate == 0) {
    // one segment per sequence: the causal kernel starts it from nothing and reads no prefix; only the counter of
    // the call has to start at zero
    if (f.flushed != nullptr) return launch_fill_u32((uint32_t*)f.flushed, 0u, 1, st);
    return 0;
  }
  int Z = 1, R = a.nslot;
  if (f.rscr != nullptr && prefix != 1) fast_reduce_ranges(BH, a.nslot, &Z, &R);
  const int Zvalid = (nstate + R - 1) / R;
  if (Z > 1 && Zvalid >= 1) {
    // few sequences, many slots: range totals, the reduction over them, and (causal) the walk over every range
    float* cscan = f.cscr + (size_t)BH * Z;
    hipLaunchKernelGGL(k_fast_reduce_totals, dim3(nblk, BH, Z), dim3(256), 0, st, f.Tpart, f.cpart, f.rscr, f.cscr, a.nslot,
                       nstate, R);
    FS_LAUNCH_CHECK();
    if (prefix == 0) {
      // the sum of everything ends in range 0 of the scratch buffer: the query-side kernel reads it there
      hipLaunchKernelGGL(k_fast_reduce, dim3(nblk, BH), dim3(256), 0, st, f.rscr, f.cscr, f.cstar, Z, Zvalid, 0, 1, f.flushed);
      FS_LAUNCH_CHECK();
      a.Tpart = f.rscr;
      a.nslot = Z;
    } else {
      hipLaunchKernelGGL(k_fast_reduce, dim3(nblk, BH), dim3(256), 0, st, f.rscr, f.cscr, cscan, Z, Zvalid, 2, 1,
                         (unsigned*)nullptr);
      FS_LAUNCH_CHECK();
      hipLaunchKernelGGL(k_fast_reduce_walk, dim3(nblk, BH, Z), dim3(256), 0, st, f.Tpart, f.cpart, f.cstar, f.rscr, cscan,
                         a.nslot, nstate, every_slot ? 1 : f.sub, R, f.flushed);
      FS_LAUNCH_CHECK();
    }
    return 0;
  }
  hipLaunchKernelGGL(k_fast_reduce, dim3(nblk, BH), dim3(256), 0, st, f.Tpart, f.cpart, f.cstar, a.nslot, nstate, prefix,
                     every_slot ? 1 : f.sub, f.flushed);
  FS_LAUNCH_CHECK();
  return 0;
}

int launch_fast_prepare(const float* theta, int groups, const float* Omega, int omega_groups, int pgroups, int B, int H,
                        float scale, uint16_t* Wbf, float* bias, float* wnorm, int* dense_flag, hipStream_t st) {
  hipLaunchKernelGGL(k_fast_pre, dim3((M / 4) * 2 * pgroups), dim3(256), 0, st, theta, groups, Omega, omega_groups, pgroups,
                     B, H, scale, Wbf, bias, wnorm, dense_flag);
  FS_LAUNCH_CHECK();
  return 0;
}

// Sum of `nslot` segment states per (b,h) into slot 0 (the reduction kernel of the forward pass on another buffer).
void launch_fast_reduce_sum(float* part, const float* cpart, float* cstar, int nslot, int BH, hipStream_t st) {
  hipLaunchKernelGGL(k_fast_reduce, dim3((M * DVP / 4 + 255) / 256, BH), dim3(256), 0, st, part, cpart, cstar, nslot, nslot, 0, 1,
                     (unsigned*)nullptr);
}

// Non-causal calls that run one workgroup per sequence (k_fast_whole): enough sequences to fill most of the chip's
// 512 workgroup places, or sequences so short that their chunks in a row cost less than the two further launches
// and the states' way through memory (measured: the three-kernel form wins from about B*H / 8 chunks of keys and
// queries together; with 384 sequences or more it never does).
static bool fast_whole_sequences(int BH, int Lq, int Lk) {
  const int chunks = (Lq + TC - 1) / TC + (Lk + TC - 1) / TC;
  return BH >= 384 || chunks <= std::min(32, std::max(4, BH / 8));
}

// The same choice for the backward pass of a non-causal call (k_bwd_whole): six loops over the sequence in a row, so
// the short-sequence bound is half the forward one (measured: B*H / 16 chunks, 4 .. 16).
static bool fast_whole_sequences_backward(int BH, int Lq, int Lk) {
  const int chunks = (Lq + TC - 1) / TC + (Lk + TC - 1) / TC;
  return BH >= 384 || chunks <= std::min(16, std::max(4, BH / 16));
}

int launch_fast_attention(const FastLaunch& f, hipStream_t st, hipEvent_t ev_begin, hipEvent_t ev_end) {
  FastArgs a;
  const int BH = f.B * f.H;
  if (!f.causal && fast_whole_sequences(BH, f.Lq, f.Lk)) {
    static_assert(sizeof(SmemWhole) <= 65536, "k_fast_whole: two workgroups per CU");
    if (int rc = launch_fast_constants(f, a, st, false)) return rc;
    if (f.flushed != nullptr)
      if (int rc = launch_fill_u32((uint32_t*)f.flushed, 0u, 1, st)) return rc;
    if (ev_begin || ev_end) hipExtLaunchKernelGGL(k_fast_whole, dim3(BH), dim3(NT), sizeof(SmemWhole), st, ev_begin, ev_end, 0, a, f.Lq);
    else hipLaunchKernelGGL(k_fast_whole, dim3(BH), dim3(NT), sizeof(SmemWhole), st, a, f.Lq);
    FS_LAUNCH_CHECK();
    return 0;
  }
  if (int rc = launch_fast_state_pass(f, a, st, false, true)) return rc;
  // the optional events are attached to the main kernel's dispatch: they carry its own begin and end times
  if (f.causal) {
    if (int rc = launch_fast_causal_kernel(a, BH, st, ev_begin, ev_end)) return rc;
  } else {
    // two workgroups per CU: about 512 blocks in all, whole chunks each
    const int want = std::max(1, std::min((512 + BH - 1) / BH, (f.Lq + TC - 1) / TC));
    const int rows_per_blk = (((f.Lq + want - 1) / want) + TC - 1) / TC * TC;
    const int nblk = (f.Lq + rows_per_blk - 1) / rows_per_blk;
    if (ev_begin || ev_end) hipExtLaunchKernelGGL(k_fast_apply, dim3(nblk, BH), dim3(NT), 0, st, ev_begin, ev_end, 0, a, f.Lq, rows_per_blk);
    else hipLaunchKernelGGL(k_fast_apply, dim3(nblk, BH), dim3(NT), 0, st, a, f.Lq, rows_per_blk);
    FS_LAUNCH_CHECK();
  }
  return 0;
}

// Backward pass of a non-causal call: the forward state pass, then the kernels of kernels_bf16_bwd.hip.
int launch_fast_attention_backward(const FastLaunch& f, const TensorDev& dY, const TensorDev& dQ, const TensorDev& dK,
                                   const TensorDev& dV, uint16_t* gh, float* Rpart, float* rcpart, float* rcstar,
                                   int rslots, int rows_per_rslot, hipStream_t st) {
  FastArgs a;
  if (f.causal) {
    if (f.nseg == 1) {
      // one slot per sequence (256 sequences or more, or a single chunk): the walks start from nothing, so there are
      // no states to compute, to scan or to read; only the sequence's key shift
      FastLaunch f1 = f;
      f1.sub = 1;
      if (int rc = launch_fast_constants(f1, a, st, false)) return rc;
      hipLaunchKernelGGL(k_fast_bound, dim3(f.B * f.H), dim3(NT), sizeof(SmemState), st, a);
      FS_LAUNCH_CHECK();
      return launch_fast_backward_causal(f1, a, dY, dQ, dK, dV, gh, Rpart, rcpart, st);
    }
    if (int rc = launch_fast_state_pass(f, a, st, true)) return rc;
    return launch_fast_backward_causal(f, a, dY, dQ, dK, dV, gh, Rpart, rcpart, st);
  }
  if (fast_whole_sequences_backward(f.B * f.H, f.Lq, f.Lk)) {
    if (int rc = launch_fast_constants(f, a, st, false)) return rc;
    if (f.flushed != nullptr)
      if (int rc = launch_fill_u32((uint32_t*)f.flushed, 0u, 1, st)) return rc;
    return launch_fast_backward_whole(f, a, dY, dQ, dK, dV, gh, st);
  }
  if (int rc = launch_fast_state_pass(f, a, st)) return rc;
  return launch_fast_backward(f, a, dY, dQ, dK, dV, gh, Rpart, rcpart, rcstar, rslots, rows_per_rslot, st);
}

}  // namespace fs
