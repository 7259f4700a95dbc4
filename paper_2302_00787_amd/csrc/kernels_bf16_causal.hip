// Causal segment kernel of the bf16 attention path (see fast_common.h for the register-level design).
//
// One workgroup walks one segment of one sequence in 64-token chunks, its state seeded with the exclusive prefix
// of the segment states:
//   Y_c = (tril(P_c S_c^T) [V_c 1] + P_c T_{c-1}) normalised by its last column;  T_c = T_{c-1} + S_c^T [V_c 1].
//
// Register plan.  This translation unit is compiled so that MFMA results land in ordinary vector registers (they
// feed exp2 / convert / mask steps).  The state T (80 registers per lane) would not fit next to everything else, so
// it is pinned to the accumulation registers: the only MFMAs that touch it are issued through mfma_state() below,
// whose accumulator operand is constrained to that register class.  Two instantiations: SYM (B1 = B2, the query and
// key projections share one W~ slice: PosRF, GERF, SDERF) and the general one; each workgroup looks at the flag of its
// own parameter set and the instantiation that does not match returns at once.
#include "fast_common.h"

namespace fs {

using namespace fast;

// T += A x B with T held in accumulation registers.  The leading s_nop covers the issue-to-read spacing the
// compiler would otherwise provide for an MFMA it knows about.
__device__ __forceinline__ void mfma_state(f32x4& t, bf16x8 a, bf16x8 b) {
  asm volatile("s_nop 1\n\tv_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(t) : "v"(a), "v"(b));
}

// grid (nseg, B*H), block 256.
template <bool SYM>
__global__ void __launch_bounds__(NT) k_fast_causal(FastArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  Smem& sm = *reinterpret_cast<Smem*>(smem_raw);
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

  WSlice wq, wk2;
  load_wslice(wq, a.Wbf + ((size_t)pg * 2) * M * D);
  if (!SYM) load_wslice(wk2, a.Wbf + ((size_t)pg * 2 + 1) * M * D);
  const WSlice& wk = SYM ? wq : wk2;
  QBias qb;
  load_qbias(qb, a.bias + ((size_t)pg * 2) * M, amax1);
  bf16x8 sel[2];
  make_sel(sel);
  zero_pad_rows(sm);
  f32x4 T[4][NVT];
  {
    const float* Tg = a.Tpart + ((size_t)bh * a.nslot + (size_t)seg * a.sub) * M * DVP;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
        for (int r = 0; r < 4; ++r) T[mt][vt][r] = Tg[(size_t)(64 * w + 16 * mt + 4 * g + r) * DVP + 16 * vt + c];
  }
  float dk = a.cstar[bh];          // shift of the prefix state (-inf when there is none)

  const int row_beg = seg * a.rows_per_seg, row_end = min(a.L, row_beg + a.rows_per_seg);
  RowRegs qr, kr, vr;
  load_rows_g(qr, Qb, a.Q.sl, row_beg, row_end);
  load_rows_g(kr, Kb, a.K.sl, row_beg, row_end);
  load_vals_g(vr, Vb, a.V.sl, row_beg, row_end);
  store_query_rows(qr, sm, 0, wmax1);
  store_key_rows(kr, sm, 0, a, isoC, bh, row_beg, row_end, wmax2);
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
    dk = key_shift_update(sm, buf, dk, T);

    // state before this chunk as A operand (T^T: row v, k <-> feature)
    bf16x8 tb[NVT][2];
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) tb[vt][mb] = pack8(T[2 * mb][vt], T[2 * mb + 1][vt]);

    // key side, one pair of token tiles at a time: S for the scores, S^T for the state update (done at once)
    bf16x8 s[4][2];
#pragma unroll
    for (int jp = 0; jp < 2; ++jp) {
      bf16x8 sp[2][2], st[4];
      key_pair(wk, sm, buf, jp, dk, sel, sp, st);
      s[2 * jp][0] = sp[0][0]; s[2 * jp][1] = sp[0][1];
      s[2 * jp + 1][0] = sp[1][0]; s[2 * jp + 1][1] = sp[1][1];
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) {
        const bf16x8 vop = load_vop(sm.vt[buf], jp, vt);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) mfma_state(T[mt][vt], st[mt], vop);
      }
    }

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
          for (int vt = 0; vt < NVT; ++vt) y[vt] = mfma(load_vop(sm.vt[buf], jp, vt), sb, y[vt]);
        }
      }
      exchange_put(sm, y, it);
    }
    exchange_finish(sm, a.Y, ybase, row0, row_end);
    if (more) {
      store_query_rows(qr, sm, buf ^ 1, wmax1);
      store_key_rows(kr, sm, buf ^ 1, a, isoC, bh, row0 + TC, row_end, wmax2);
      store_vals_s(vr, sm.vt[buf ^ 1], row0 + TC, row_end);
    }
    __syncthreads();
  }
}

int launch_fast_causal_kernel(const FastArgs& a, int BH, hipStream_t st) {
  const void* fns[2] = {(const void*)k_fast_causal<true>, (const void*)k_fast_causal<false>};
  for (const void* fn : fns)
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(Smem)) != hipSuccess) {
      (void)hipGetLastError();
      return 2;
    }
  hipLaunchKernelGGL(k_fast_causal<true>, dim3(a.nseg, BH), dim3(NT), sizeof(Smem), st, a);
  if (hipGetLastError() != hipSuccess) return 5;
  hipLaunchKernelGGL(k_fast_causal<false>, dim3(a.nseg, BH), dim3(NT), sizeof(Smem), st, a);
  if (hipGetLastError() != hipSuccess) return 5;
  return 0;
}

}  // namespace fs
