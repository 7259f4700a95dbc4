// Shared declarations of the bf16 backward kernels (kernels_bf16_bwd.hip: non-causal; kernels_bf16_bwd_pc.hip:
// causal).
#pragma once
#include "fast_common.h"

namespace fs {
namespace bwd {

using namespace fast;

struct BwdArgs {
  FastArgs f;                // forward arguments; Tpart slot 0 holds the total state, cstar the key shifts
  TensorDev dY, dQ, dK, dV;
  uint16_t* gh;              // [BH][Lq][80] bf16: G1 rows (columns 65.. are zero)
  float* Rpart;              // [BH][rslots][256][80]
  float* rcpart;             // [BH][rslots] zeros (shifts of the R segments: none)
  int Lq, Lk, rslots, rows_per_rslot;
  const float* zero_state = nullptr;   // causal kernels, one slot per sequence: a state of zeros in place of prefix and suffix
};

// Three 16-byte pieces per thread for tiles of up to 768 pieces.
struct RowRegs3 { u32x4 p[3]; };

__device__ __forceinline__ void load_g80_g(RowRegs3& r, const uint16_t* base, int row0, int row_end) {
  const int j = threadIdx.x & 63;
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const int pc = (threadIdx.x >> 6) + 4 * i;
    r.p[i] = u32x4{0u, 0u, 0u, 0u};
    if (pc < DVP / 8 && row0 + j < row_end) r.p[i] = *(const u32x4*)(base + (size_t)(row0 + j) * DVP + pc * 8);
  }
}
// Transposed into vt[column][token]; lane pairs swap halves so that every lane writes whole dwords.
__device__ __forceinline__ void store_g80_s(const RowRegs3& r, uint16_t (*vt)[LDJ]) {
  const int j = threadIdx.x & 63, odd = j & 1;
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const int pc = (threadIdx.x >> 6) + 4 * i;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t mine = r.p[i][e], other = dpp_u<0xB1>(mine);
      const uint32_t wv = odd ? ((other >> 16) | (mine & 0xffff0000u)) : ((mine & 0xffffu) | (other << 16));
      if (pc < DVP / 8) *(uint32_t*)(&vt[pc * 8 + 2 * e + odd][j & ~1]) = wv;
    }
  }
}

constexpr int KL = 96;             // contraction length of dF: 80 columns padded to three MFMA steps
constexpr int LDL = KL + 8;        // row stride (bf16) of the left-rows tile: 52 dwords, conflict-free 16-byte reads

// Per-slot sums of P^T G1 (kernel in kernels_bf16_bwd.hip).  grid (rslots, B*H).
int launch_bwd_rstate(const BwdArgs& ba, int BH, hipStream_t st);

}  // namespace bwd

// Kernels of the causal variant with producer and consumer waves (kernels_bf16_bwd_pc.hip), grid (nslot, B*H) each:
// gradient rows dQ and dK; forward walk that leaves the G1 rows (mode 0) and backward walk for dV (mode 1).
int launch_bwd_cgrad_pc(const bwd::BwdArgs& ba, int nslot, int BH, hipStream_t st);
int launch_bwd_walk_pc(const bwd::BwdArgs& ba, int mode, int nslot, int BH, hipStream_t st);
size_t bwd_pc_lds_bytes();

}  // namespace fs
