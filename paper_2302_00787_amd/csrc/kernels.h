// Host-callable launchers of the FAVOR# kernels.  Every launcher enqueues on `st`, returns an fs_status
// value (0 ok, 2 unsupported, 5 HIP error) and allocates nothing.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "fs_common.h"

namespace fs {

constexpr int FS_THETA_HEADER_ = 8;

// One side (queries or keys) of a feature map as the general-shape kernels see it.
struct GenSide {
  TensorDev X;          // rows to map
  float scale;          // qk_scale
  float alpha;          // coefficient of |x|^2 added to the exponent (Section 2.3), 0 for attention
  const float* W;       // [pgroups][2][M][d] projection matrices times log2(e)
  const float* bias;    // [pgroups][2][M]    biases times log2(e)
  const float* theta;   // parameter sets
  int groups;           // number of parameter sets
  int pgroups;          // number of projection-constant sets
  long long theta_stride;
  long long c_offset;   // offset of this side's C matrix inside a parameter set
  float* rk = nullptr;  // [B*H][rows] row terms of this side's rows (written by k_gen_kmax, read by the kernels after
                        // it instead of evaluating the quadratic form once per feature block); nullptr: none
};

size_t gen_lds_features(int d);
size_t gen_lds_state(int d, int ldt);
size_t gen_lds_apply(int d, int ldt);
size_t gen_lds_causal(int d, int ldt);
size_t gen_lds_stats(int d);

int launch_prep(const float* theta, int groups, const float* Omega, int omega_groups, int pgroups, int B, int H,
                int M, int d, float* W, uint16_t* Wbf, float* bias, hipStream_t st);
int launch_fill_u32(uint32_t* p, uint32_t v, size_t n, hipStream_t st);
int launch_gen_features(const TensorDev& X, int n, int d, float scale, float alpha, const float* W, const float* bias,
                        const float* theta, long long c_offset, int M, float* out, float* row_logscale,
                        hipStream_t st);
int launch_gen_kmax(const GenSide& ks, int Lk, int BH, int H, int M, int d, uint32_t* kmax_u, hipStream_t st);
int launch_gen_state(const GenSide& ks, const TensorDev& V, int Lk, int BH, int H, int M, int d, int nv,
                     int append_ones, int ldt, int rows_per_seg, int nseg, const uint32_t* kmax_u,
                     const float* row_shift, float* Tpart, hipStream_t st);
int launch_gen_reduce(float* Tpart, int BH, int nseg, size_t per_state, int prefix, hipStream_t st);
int launch_gen_apply(const GenSide& qs, int Lq, int BH, int H, int M, int d, int nv, int ldt, const float* T,
                     size_t state_stride, const uint32_t* kmax_u, int matvec, const TensorDev& Y, float* den_out,
                     float* shift_out, hipStream_t st, unsigned* flushed = nullptr);
// Backward pass of non-causal attention (general-shape kernels).
size_t gen_lds_bwd_side(int d, int ldt);
int launch_bwd_ghat(const TensorDev& dY, float* buf, const float* den, int L, int BH, int H, int nv, int ldt,
                    hipStream_t st);
int launch_gen_bwd_side(const GenSide& sd, int side, const TensorDev& A, int a_cols, int append_ones, int L, int BH,
                        int H, int M, int d, int nv, int ldt, const float* St, size_t state_stride,
                        const uint32_t* kmax_u, const float* row_shift, const TensorDev& out1, int want_out1,
                        const TensorDev& grad, hipStream_t st);
int launch_gen_causal(const GenSide& qs, const GenSide& ks, const TensorDev& V, int L, int BH, int H, int M, int d,
                      int nv, int ldt, int rows_per_seg, int nseg, const uint32_t* kmax_u, float* Tstate,
                      const TensorDev& Y, float* den_out, float* shift_out, hipStream_t st, unsigned* flushed = nullptr);
size_t gen_lds_bwd_causal(int d, int ldt);
int launch_gen_bwd_causal(const GenSide& qs, const GenSide& ks, const TensorDev& V, const float* ghat, int L, int BH, int H,
                          int M, int d, int nv, int ldt, int rows_per_seg, int nseg, const uint32_t* kmax_u,
                          const float* row_shift, float* Tstate, float* Rstate, const TensorDev& dQ, const TensorDev& dK,
                          const TensorDev& dV, hipStream_t st);
bool stats_bf16_supported(const TensorDev& X, const TensorDev& Y, int d);
int launch_stats_bf16(const TensorDev& X, const TensorDev& Y, int BH, int H, int Lx, int Ly, float scale,
                      int rows_per_chunk, int nchunks, float* part, hipStream_t st);
// The same for bf16 rows of 128 numbers (kernels_bf16_wide.hip).
bool stats_wide_supported(const TensorDev& X, const TensorDev& Y, int d);
int launch_stats_wide(const TensorDev& X, const TensorDev& Y, int BH, int H, int Lx, int Ly, float scale,
                      int rows_per_chunk, int nchunks, float* part, hipStream_t st);
// Device-resident closed-form fit (kernels_fit.hip): one workgroup per group; ws holds fit_device_workspace_doubles
// doubles; status[g] receives an fs_status value.
size_t fit_device_workspace_doubles(int d, int groups);
int launch_fit_device(int variant, int d, int groups, const double* stats, double ridge, double* ws, float* theta,
                      int* status, size_t theta_floats, hipStream_t st);
int launch_stats(const TensorDev& X, const TensorDev& Y, int B, int H, int Lx, int Ly, int d, float scale, int groups,
                 int rows_per_chunk, int nchunks, float* part, double* stats, hipStream_t st);

}  // namespace fs

namespace fs {

// bf16 fast path (d = dv = 64, M = 256): everything one attention call needs.
struct FastLaunch {
  TensorDev Q, K, V, Y;
  const float* theta;
  const float* Omega;
  int groups, omega_groups, pgroups;
  int B, H, Lq, Lk, causal;
  int nseg, rows_per_seg, sub;
  float scale;
  uint16_t* Wbf;    // [pgroups][2][256][64]
  float* bias;      // [pgroups][2][256]
  float* wnorm;     // [pgroups][2][256]
  float* rk;        // [B*H][Lk]
  float* Tpart;     // [B*H][nseg*sub][256][80]
  float* cpart;     // [B*H][nseg*sub]
  float* cstar;     // [B*H]
  unsigned* flushed = nullptr;   // counter of output rows whose normaliser came out as zero (nullptr: not counted)
  float* rscr = nullptr;         // [B*H][Z][256][80] range totals of the slot reduction (nullptr: one-kernel reduction)
  float* cscr = nullptr;         // [B*H][Z] their shifts, then [B*H] + [B*H][Z] the shifts of the scan over them
  // 0: compute the projection constants and the key row terms; 1: the constants are already in Wbf / bias / wnorm
  // (prepared by an earlier call), only the row terms of parameter sets with a dense C2 are computed; 2: the
  // constants are there and no parameter set has a dense C2: nothing to do
  int pre_mode = 0;
};

// bf16 path for d = dv = 128, M = 512, causal and non-causal (kernels_bf16_wide.hip).
struct WideLaunch {
  TensorDev Q, K, V, Y;
  const float* theta;
  const float* Omega;
  int groups, omega_groups, pgroups;
  int B, H, L;                       // L keys (causal calls: and as many queries)
  int nslot, rows_per_slot;          // wide_plan of the keys
  int causal = 1;
  int Lq = 0, nslot_q = 0, rows_per_slot_q = 0;   // non-causal calls: the queries and their wide_plan
  float scale;
  uint16_t* Wbf;    // [pgroups][2][512][128]
  float* bias;      // [pgroups][2][512]
  float* wnorm;     // [pgroups][2][512]
  float* rk;        // [B*H][L]
  float* Tpart;     // [B*H][2][nslot][256][144]
  float* cpart;     // [B*H][nslot]
  float* cstar;     // [B*H]
  float* Ypart;     // [B*H][queries][132]
  unsigned* flushed = nullptr;   // as in FastLaunch
  int pre_mode = 0; // as in FastLaunch
};
bool wide_supported(int dtype, int d, int dv, int M, int causal);
// Projection constants only (for a later call with pre_mode 1 or 2); *dense_flag (device) is or-ed with 1 if any of
// the parameter sets the kernel visits has a dense C2.
int launch_wide_prepare(const float* theta, int groups, const float* Omega, int omega_groups, int pgroups, int B, int H,
                        float scale, uint16_t* Wbf, float* bias, float* wnorm, int* dense_flag, hipStream_t st);
int launch_fast_prepare(const float* theta, int groups, const float* Omega, int omega_groups, int pgroups, int B, int H,
                        float scale, uint16_t* Wbf, float* bias, float* wnorm, int* dense_flag, hipStream_t st);
size_t wide_lds_bytes();
void wide_plan(int BH, int L, int* nslot, int* rows_per_slot);
int launch_wide_attention(const WideLaunch& f, hipStream_t st, hipEvent_t ev_begin, hipEvent_t ev_end);

// fp32 kernel operator for a few right-hand sides (kernels_op.hip).
bool op_supported(int dtype_x, int dtype_y, int d, int M, int n);
size_t op_workspace_floats(int Ny, int d, int M);
int launch_op_matvec(const float* theta, const TensorDev& X, const TensorDev& Y, int Nx, int Ny, int d, float scale,
                     float alpha, const float* Omega, int M, const float* C, int n, float* out, float* ws, hipStream_t st);

size_t fast_lds_bytes();
bool fast_supported(int dtype, int d, int dv, int M);
void fast_plan(int BH, int L, int* nseg, int* rows_per_seg, int* sub);
// Ranges of the slot reduction: Z > 1 (ranges of R slots, reduced side by side) for few sequences with many slots.
void fast_reduce_ranges(int BH, int nslot, int* Z, int* R);
int launch_fast_attention(const FastLaunch& f, hipStream_t st, hipEvent_t ev_begin, hipEvent_t ev_end);
int launch_fast_attention_backward(const FastLaunch& f, const TensorDev& dY, const TensorDev& dQ, const TensorDev& dK,
                                   const TensorDev& dV, uint16_t* gh, float* Rpart, float* rcpart, float* rcstar,
                                   int rslots, int rows_per_rslot, hipStream_t st);
size_t fast_bwd_lds_bytes();
size_t fast_bwd_causal_lds_bytes();

}  // namespace fs
