// C ABI of the FAVOR# library: argument validation, workspace planning and kernel dispatch.
// Nothing here allocates device memory; everything runs on the caller's stream.
#include "../../include/favorsharp.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <mutex>
#include <thread>
#include <vector>

#include "host_fit.h"
#include "kernels.h"

using namespace fs;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

bool tensor_ok(const fs_tensor* t, int d, bool need_ptr = true) {
  if (t == nullptr) return false;
  if (need_ptr && t->ptr == nullptr) return false;
  if (t->dtype != FS_F32 && t->dtype != FS_BF16) return false;
  if (t->stride_l < d) return false;
  const int q = t->dtype == FS_BF16 ? 8 : 4;
  if (t->stride_l % q || t->stride_b % q || t->stride_h % q) return false;
  if (((uintptr_t)t->ptr) % 16) return false;
  return true;
}

TensorDev dev(const fs_tensor* t) { return TensorDev{t->ptr, t->dtype, t->stride_b, t->stride_h, t->stride_l}; }

// B*H is a grid dimension of most kernels (at most 65535 workgroups there)
constexpr long long kMaxSequences = 65535;
bool sequences_ok(int B, int H) { return (long long)B * H <= kMaxSequences; }

bool groups_ok(int g, int B, int H) { return g == 1 || g == H || g == B * H; }

struct AttnPlan {
  int pgroups, ldt, nseg, rows_per_seg;
  size_t off_W, off_Wbf, off_bias, off_kmax, off_rk, off_state, total;
};

// Every attention workspace starts with one 32-bit word (in a block of kAlign bytes): the number of output rows of the
// last call whose normaliser came out as zero (favorsharp_attention_flushed_rows reads it).
//
// Shared by the workspace query and the call so that both agree.
void plan_contraction(int BH, int pgroups, int Lk, int d, int M, int nv1, int causal, AttnPlan* p) {
  p->pgroups = pgroups;
  p->ldt = ceil_div(nv1, 16) * 16;
  const int nmb = ceil_div(M, 32);
  int want;
  if (causal) want = std::max(1, std::min(ceil_div(1024, BH), ceil_div(Lk, 128)));
  else want = std::max(1, std::min(ceil_div(2048, BH * nmb), ceil_div(Lk, 32)));
  p->rows_per_seg = ceil_div(ceil_div(Lk, want), 32) * 32;
  p->nseg = ceil_div(Lk, p->rows_per_seg);
  size_t off = kAlign;       // the counter word; the key maxima follow it so that one fill clears both
  p->off_kmax = off; off = align_up(off + (size_t)BH * sizeof(uint32_t));
  p->off_W = off;    off = align_up(off + (size_t)pgroups * 2 * M * d * sizeof(float));
  p->off_Wbf = off;  off = align_up(off + (size_t)pgroups * 2 * M * d * sizeof(uint16_t));
  p->off_bias = off; off = align_up(off + (size_t)pgroups * 2 * M * sizeof(float));
  p->off_rk = off;   off = align_up(off + (size_t)BH * Lk * sizeof(float));       // key row terms (general attention kernels)
  p->off_state = off; off = align_up(off + (size_t)BH * p->nseg * M * p->ldt * sizeof(float));
  p->total = off;
}

struct FitPlan {
  int nchunks, rows_per_chunk;
  size_t off_part, off_stats, total;
};

void plan_fit(int B, int H, int Lx, int Ly, int d, int groups, FitPlan* p) {
  const int L = std::max(Lx, Ly);
  // about two workgroups of the scan per CU and tensor; every chunk is one more partial sum for the final kernel
  const int want = std::max(1, std::min(ceil_div(512, B * H), ceil_div(L, 32)));
  p->rows_per_chunk = ceil_div(ceil_div(L, want), 32) * 32;
  p->nchunks = ceil_div(L, p->rows_per_chunk);
  const size_t per = (size_t)d * d + d;
  size_t off = 0;
  p->off_part = off;  off = align_up(off + (size_t)2 * B * H * p->nchunks * per * sizeof(float));
  p->off_stats = off; off = align_up(off + (size_t)groups * 2 * per * sizeof(double));
  p->total = off;
}

struct FastPlan {
  int pgroups, nseg, rows_per_seg, sub;
  size_t off_Wbf, off_bias, off_wnorm, off_rk, off_state, off_cpart, off_cstar, off_rscr, off_cscr, total;
  int Z;
};

void plan_fast(int BH, int pgroups, int Lk, FastPlan* p) {
  p->pgroups = pgroups;
  fast_plan(BH, Lk, &p->nseg, &p->rows_per_seg, &p->sub);
  size_t off = kAlign;       // the counter word
  p->off_Wbf = off;    off = align_up(off + (size_t)pgroups * 2 * 256 * 64 * sizeof(uint16_t));
  p->off_bias = off;   off = align_up(off + (size_t)pgroups * 2 * 256 * sizeof(float));
  p->off_wnorm = off;  off = align_up(off + (size_t)pgroups * 2 * 256 * sizeof(float));
  p->off_rk = off;     off = align_up(off + (size_t)BH * Lk * sizeof(float));
  p->off_state = off;  off = align_up(off + (size_t)BH * p->nseg * p->sub * 256 * 80 * sizeof(float));
  p->off_cpart = off;  off = align_up(off + (size_t)BH * p->nseg * p->sub * sizeof(float));
  p->off_cstar = off;  off = align_up(off + (size_t)BH * (1 + (size_t)p->nseg * p->sub) * sizeof(float));
  // (few sequences with many slots: the range totals of the slot reduction and their shifts)
  int R;
  fast_reduce_ranges(BH, p->nseg * p->sub, &p->Z, &R);
  p->off_rscr = off;   off = align_up(off + (p->Z > 1 ? (size_t)BH * p->Z * 256 * 80 * sizeof(float) : 0));
  p->off_cscr = off;   off = align_up(off + (p->Z > 1 ? (size_t)BH * (1 + 2 * (size_t)p->Z) * sizeof(float) : 0));
  p->total = off;
}

struct WidePlan {
  int nslot, rows_per_slot;         // slots of the keys
  int nslot_q, rows_per_slot_q;     // slots of the queries (the walk)
  size_t off_Wbf, off_bias, off_wnorm, off_rk, off_state, off_cpart, off_cstar, off_ypart, total;
};

void plan_wide(int BH, int pgroups, int Lq, int L, WidePlan* p) {
  wide_plan(BH, L, &p->nslot, &p->rows_per_slot);
  wide_plan(BH, Lq, &p->nslot_q, &p->rows_per_slot_q);
  size_t off = kAlign;       // the counter word
  p->off_Wbf = off;    off = align_up(off + (size_t)pgroups * 2 * 512 * 128 * sizeof(uint16_t));
  p->off_bias = off;   off = align_up(off + (size_t)pgroups * 2 * 512 * sizeof(float));
  p->off_wnorm = off;  off = align_up(off + (size_t)pgroups * 2 * 512 * sizeof(float));
  p->off_rk = off;     off = align_up(off + (size_t)BH * L * sizeof(float));
  p->off_state = off;  off = align_up(off + (size_t)BH * 2 * p->nslot * 256 * 144 * sizeof(float));
  p->off_cpart = off;  off = align_up(off + (size_t)BH * p->nslot * sizeof(float));
  p->off_cstar = off;  off = align_up(off + (size_t)BH * (1 + (size_t)p->nslot) * sizeof(float));
  p->off_ypart = off;  off = align_up(off + (size_t)BH * Lq * 132 * sizeof(float));
  p->total = off;
}

// Scratch memory of favorsharp_attention_noalloc: one array per GPU, owned by the library for the life of the
// process.  In host code the array's name is only a handle for hipGetSymbolAddress; every use of its memory (kernel
// arguments) goes through the per-device pointer obtained below.
static __device__ __align__(256) unsigned char scratch[FS_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_ptr[kMaxDevices] = {};

// Address of the current device's copy of `scratch` (looked up once per device, with that device current).
int scratch_for_current_device(void** out) {
  int dev_id = 0;
  if (hipGetDevice(&dev_id) != hipSuccess) return FS_ERR_DEVICE;
  if (dev_id < 0 || dev_id >= kMaxDevices) return FS_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (scratch_ptr[dev_id] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return FS_ERR_DEVICE;
    }
    scratch_ptr[dev_id] = p;
  }
  *out = scratch_ptr[dev_id];
  return FS_OK;
}

// Layout of the buffer favorsharp_attention_prepare fills: a header word (bit 0: some parameter set has a dense C2),
// then the projection constants of the bf16 kernels.
struct PreparedPlan {
  int Mk, dk;            // the kernels' M and d (0: no bf16 kernels for this shape)
  size_t off_flag, off_Wbf, off_bias, off_wnorm, total;
};

void plan_prepared(int d, int M, int pgroups, PreparedPlan* p) {
  p->Mk = p->dk = 0;
  p->total = 0;
  if (fast_supported(FS_BF16, d, d, M)) { p->Mk = 256; p->dk = 64; }
  else if (wide_supported(FS_BF16, d, d, M, 1)) { p->Mk = 512; p->dk = 128; }
  else return;
  size_t off = 0;
  p->off_flag = off;  off = align_up(off + sizeof(int));
  p->off_Wbf = off;   off = align_up(off + (size_t)pgroups * 2 * p->Mk * p->dk * sizeof(uint16_t));
  p->off_bias = off;  off = align_up(off + (size_t)pgroups * 2 * p->Mk * sizeof(float));
  p->off_wnorm = off; off = align_up(off + (size_t)pgroups * 2 * p->Mk * sizeof(float));
  p->total = off;
}

int attention_impl(const float* theta, int groups, const fs_tensor* Q, const fs_tensor* K, const fs_tensor* V, int B,
                   int H, int Lq, int Lk, int d, int dv, float qk_scale, const float* Omega, int omega_groups, int M,
                   int causal, int chunk, const fs_tensor* Y, void* workspace, size_t workspace_bytes, void* stream,
                   void* event_main_begin, void* event_main_end, const void* prepared, int dense_c2);

int device_lds_limit() {
  int dev_id = 0, v = 0;
  if (hipGetDevice(&dev_id) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev_id) != hipSuccess) return 0;
  return v;
}

}  // namespace

extern "C" {

size_t favorsharp_theta_floats(int d) { return d > 0 ? (size_t)FS_THETA_HEADER + (size_t)d + 4 * (size_t)d * d : 0; }

const char* favorsharp_status_string(int status) {
  switch (status) {
    case FS_OK: return "ok";
    case FS_ERR_INVALID_ARG: return "invalid argument";
    case FS_ERR_UNSUPPORTED: return "unsupported shape or option";
    case FS_ERR_NOT_PD: return "statistics are singular";
    case FS_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case FS_ERR_DEVICE: return "device error";
    case FS_ERR_SCRATCH_LIMIT: return "problem needs more scratch memory than the library's fixed buffer holds";
    default: return "unknown status";
  }
}

const char* favorsharp_version(void) { return "favorsharp 0.1 (gfx950)"; }

// ------------------------------------------------------------------------------------------ orthogonal omega (host)
int favorsharp_orthogonal_omega(const float* host_gauss_dir, const float* host_gauss_len, int groups, int M, int d,
                                float* host_omega) {
  if (host_gauss_dir == nullptr || host_gauss_len == nullptr || host_omega == nullptr) return FS_ERR_INVALID_ARG;
  if (groups < 1 || M < 1 || d < 1) return FS_ERR_INVALID_ARG;
  std::vector<double> g((size_t)d * d), len(d), out((size_t)d * d);
  for (int grp = 0; grp < groups; ++grp)
    for (int r0 = 0; r0 < M; r0 += d) {
      const int n = std::min(d, M - r0);
      const size_t base = ((size_t)grp * M + r0) * d;
      for (int i = 0; i < n; ++i) {
        double l2 = 0.0;
        for (int c = 0; c < d; ++c) {
          g[(size_t)i * d + c] = host_gauss_dir[base + (size_t)i * d + c];
          const double v = host_gauss_len[base + (size_t)i * d + c];
          l2 += v * v;
        }
        len[i] = std::sqrt(l2);
      }
      if (!orthogonal_rows(n, d, g.data(), len.data(), out.data())) return FS_ERR_NOT_PD;
      for (size_t e = 0; e < (size_t)n * d; ++e) host_omega[base + e] = (float)out[e];
    }
  return FS_OK;
}

// ------------------------------------------------------------------------------------------ fit
size_t favorsharp_fit_workspace_bytes(int B, int H, int Lx, int Ly, int d, int groups) {
  if (B < 1 || H < 1 || Lx < 1 || Ly < 1 || d < 1 || d > 128 || !sequences_ok(B, H) || !groups_ok(groups, B, H)) return 0;
  FitPlan p;
  plan_fit(B, H, Lx, Ly, d, groups, &p);
  return p.total;
}

int favorsharp_fit_params(int variant, const fs_tensor* X, const fs_tensor* Y, int B, int H, int Lx, int Ly, int d,
                          float qk_scale, int groups, float eig_ridge, float* theta, void* workspace,
                          size_t workspace_bytes, void* stream) {
  if (variant < FS_POSRF || variant > FS_SDERF) return FS_ERR_INVALID_ARG;
  if (B < 1 || H < 1 || Lx < 1 || Ly < 1 || d < 1 || !groups_ok(groups, B, H)) return FS_ERR_INVALID_ARG;
  if (d > 128 || !sequences_ok(B, H)) return FS_ERR_UNSUPPORTED;
  if (!tensor_ok(X, d) || !tensor_ok(Y, d) || X->dtype != Y->dtype) return FS_ERR_INVALID_ARG;
  if (theta == nullptr || workspace == nullptr || !(eig_ridge >= 0.f) || !(qk_scale > 0.f)) return FS_ERR_INVALID_ARG;
  FitPlan p;
  plan_fit(B, H, Lx, Ly, d, groups, &p);
  if (workspace_bytes < p.total) return FS_ERR_WORKSPACE_TOO_SMALL;
  if ((int)gen_lds_stats(d) > device_lds_limit()) return FS_ERR_UNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  float* part = (float*)(ws + p.off_part);
  double* stats = (double*)(ws + p.off_stats);
  if (int rc = launch_stats(dev(X), dev(Y), B, H, Lx, Ly, d, qk_scale, groups, p.rows_per_chunk, p.nchunks, part,
                            stats, st))
    return rc;
  const size_t per = (size_t)d * d + d;
  std::vector<double> host_stats((size_t)groups * 2 * per);
  if (hipMemcpyAsync(host_stats.data(), stats, host_stats.size() * sizeof(double), hipMemcpyDeviceToHost, st) != hipSuccess)
    return FS_ERR_DEVICE;
  if (hipStreamSynchronize(st) != hipSuccess) return FS_ERR_DEVICE;
  const size_t tf = favorsharp_theta_floats(d);
  std::vector<float> host_theta((size_t)groups * tf);
  // the groups are independent d x d problems: one host thread each (at most 16)
  std::vector<int> status_of(groups, FS_OK);
  auto fit_range = [&](int g0, int g1) {
    for (int g = g0; g < g1; ++g) {
      const double* sx = host_stats.data() + ((size_t)g * 2) * per;
      const double* sy = sx + per;
      status_of[g] = fit_group(variant, d, sx, sy, sx + (size_t)d * d, sy + (size_t)d * d, (double)eig_ridge,
                               host_theta.data() + (size_t)g * tf);
    }
  };
  const int nthreads = std::max(1, std::min({groups, 16, (int)std::thread::hardware_concurrency()}));
  if (nthreads == 1) {
    fit_range(0, groups);
  } else {
    std::vector<std::thread> pool;
    for (int t = 0; t < nthreads; ++t) pool.emplace_back(fit_range, groups * t / nthreads, groups * (t + 1) / nthreads);
    for (auto& th : pool) th.join();
  }
  for (int g = 0; g < groups; ++g)
    if (status_of[g] != FS_OK) return status_of[g];
  if (hipMemcpyAsync(theta, host_theta.data(), host_theta.size() * sizeof(float), hipMemcpyHostToDevice, st) != hipSuccess)
    return FS_ERR_DEVICE;
  if (hipStreamSynchronize(st) != hipSuccess) return FS_ERR_DEVICE;
  return FS_OK;
}

size_t favorsharp_fit_device_workspace_bytes(int B, int H, int Lx, int Ly, int d, int groups) {
  const size_t base = favorsharp_fit_workspace_bytes(B, H, Lx, Ly, d, groups);
  if (base == 0) return 0;
  return base + align_up(fit_device_workspace_doubles(d, groups) * sizeof(double));
}

int favorsharp_fit_params_device(int variant, const fs_tensor* X, const fs_tensor* Y, int B, int H, int Lx, int Ly, int d,
                                 float qk_scale, int groups, float eig_ridge, float* theta, int32_t* status,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  if (variant < FS_POSRF || variant > FS_SDERF) return FS_ERR_INVALID_ARG;
  if (B < 1 || H < 1 || Lx < 1 || Ly < 1 || d < 1 || !groups_ok(groups, B, H)) return FS_ERR_INVALID_ARG;
  if (d > 128 || !sequences_ok(B, H)) return FS_ERR_UNSUPPORTED;
  if (!tensor_ok(X, d) || !tensor_ok(Y, d) || X->dtype != Y->dtype) return FS_ERR_INVALID_ARG;
  if (theta == nullptr || status == nullptr || workspace == nullptr || !(eig_ridge >= 0.f) || !(qk_scale > 0.f))
    return FS_ERR_INVALID_ARG;
  FitPlan p;
  plan_fit(B, H, Lx, Ly, d, groups, &p);
  if (workspace_bytes < favorsharp_fit_device_workspace_bytes(B, H, Lx, Ly, d, groups)) return FS_ERR_WORKSPACE_TOO_SMALL;
  if ((int)gen_lds_stats(d) > device_lds_limit()) return FS_ERR_UNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  float* part = (float*)(ws + p.off_part);
  double* stats = (double*)(ws + p.off_stats);
  double* fitws = (double*)(ws + p.total);
  if (int rc = launch_stats(dev(X), dev(Y), B, H, Lx, Ly, d, qk_scale, groups, p.rows_per_chunk, p.nchunks, part,
                            stats, st))
    return rc;
  return launch_fit_device(variant, d, groups, stats, (double)eig_ridge, fitws, theta, status,
                           favorsharp_theta_floats(d), st);
}

// ------------------------------------------------------------------------------------------ features
size_t favorsharp_features_workspace_bytes(int n, int d, int M) {
  if (n < 0 || d < 1 || d > 128 || M < 1) return 0;
  AttnPlan p;
  plan_contraction(1, 1, 32, d, M, 1, 0, &p);
  return p.off_rk;         // everything in front of the row terms: the projection constants are the part used here
}

int favorsharp_features(const float* theta, int side, const fs_tensor* X, int n, int d, float qk_scale, float alpha,
                        const float* Omega, int M, float* out, float* row_logscale, void* workspace,
                        size_t workspace_bytes, void* stream) {
  if (n < 0 || d < 1 || M < 1 || (side != 1 && side != 2)) return FS_ERR_INVALID_ARG;
  if (d > 128) return FS_ERR_UNSUPPORTED;
  if (theta == nullptr || Omega == nullptr || workspace == nullptr || !tensor_ok(X, d, n > 0)) return FS_ERR_INVALID_ARG;
  if (n > 0 && out == nullptr) return FS_ERR_INVALID_ARG;
  if (workspace_bytes < favorsharp_features_workspace_bytes(n, d, M)) return FS_ERR_WORKSPACE_TOO_SMALL;
  if (n == 0) return FS_OK;
  if ((int)gen_lds_features(d) > device_lds_limit()) return FS_ERR_UNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  AttnPlan p;
  plan_contraction(1, 1, 32, d, M, 1, 0, &p);
  char* ws = (char*)workspace;
  float* W = (float*)(ws + p.off_W);
  uint16_t* Wbf = (uint16_t*)(ws + p.off_Wbf);
  float* bias = (float*)(ws + p.off_bias);
  if (int rc = launch_prep(theta, 1, Omega, 1, 1, 1, 1, M, d, W, Wbf, bias, st)) return rc;
  const size_t dd = (size_t)d * d;
  const long long c_off = FS_THETA_HEADER + d + 2 * dd + (side == 2 ? dd : 0);
  return launch_gen_features(dev(X), n, d, qk_scale, alpha, W + (side == 2 ? (size_t)M * d : 0),
                             bias + (side == 2 ? M : 0), theta, c_off, M, out, row_logscale, st);
}

// ------------------------------------------------------------------------------------------ attention
size_t favorsharp_attention_workspace_bytes(int B, int H, int Lq, int Lk, int d, int dv, int M, int causal,
                                            int groups, int omega_groups) {
  if (B < 1 || H < 1 || Lq < 0 || Lk < 1 || d < 1 || d > 128 || dv < 1 || dv > 128 || M < 1 || !sequences_ok(B, H)) return 0;
  if (!groups_ok(groups, B, H) || !groups_ok(omega_groups, B, H)) return 0;
  AttnPlan p;
  plan_contraction(B * H, std::max(groups, omega_groups), Lk, d, M, dv + 1, causal, &p);
  size_t total = p.total;
  if (fast_supported(FS_BF16, d, dv, M)) {      // the query does not know the dtype: cover both paths
    FastPlan fp;
    plan_fast(B * H, std::max(groups, omega_groups), Lk, &fp);
    total = std::max(total, fp.total);
  }
  if (wide_supported(FS_BF16, d, dv, M, causal) && (Lq == Lk || !causal)) {
    WidePlan wp;
    plan_wide(B * H, std::max(groups, omega_groups), Lq, Lk, &wp);
    total = std::max(total, wp.total);
  }
  return total;
}

int favorsharp_attention(const float* theta, int groups, const fs_tensor* Q, const fs_tensor* K, const fs_tensor* V,
                         int B, int H, int Lq, int Lk, int d, int dv, float qk_scale, const float* Omega,
                         int omega_groups, int M, int causal, int chunk, const fs_tensor* Y, void* workspace,
                         size_t workspace_bytes, void* stream) {
  return favorsharp_attention_timed(theta, groups, Q, K, V, B, H, Lq, Lk, d, dv, qk_scale, Omega, omega_groups, M,
                                    causal, chunk, Y, workspace, workspace_bytes, stream, nullptr, nullptr);
}

int favorsharp_attention_timed(const float* theta, int groups, const fs_tensor* Q, const fs_tensor* K,
                               const fs_tensor* V, int B, int H, int Lq, int Lk, int d, int dv, float qk_scale,
                               const float* Omega, int omega_groups, int M, int causal, int chunk,
                               const fs_tensor* Y, void* workspace, size_t workspace_bytes, void* stream,
                               void* event_main_begin, void* event_main_end) {
  return attention_impl(theta, groups, Q, K, V, B, H, Lq, Lk, d, dv, qk_scale, Omega, omega_groups, M, causal, chunk, Y,
                        workspace, workspace_bytes, stream, event_main_begin, event_main_end, nullptr, 0);
}

size_t favorsharp_prepared_bytes(int B, int H, int d, int M, int groups, int omega_groups) {
  if (B < 1 || H < 1 || d < 1 || M < 1 || !groups_ok(groups, B, H) || !groups_ok(omega_groups, B, H)) return 0;
  PreparedPlan pp;
  plan_prepared(d, M, std::max(groups, omega_groups), &pp);
  return pp.total;
}

int favorsharp_attention_prepare(const float* theta, int groups, const float* Omega, int omega_groups, int B, int H,
                                 int d, int M, float qk_scale, void* prepared, size_t prepared_bytes,
                                 int* host_dense_c2, void* stream) {
  if (B < 1 || H < 1 || d < 1 || M < 1 || !groups_ok(groups, B, H) || !groups_ok(omega_groups, B, H))
    return FS_ERR_INVALID_ARG;
  if (theta == nullptr || Omega == nullptr || prepared == nullptr || host_dense_c2 == nullptr || !(qk_scale > 0.f))
    return FS_ERR_INVALID_ARG;
  const int pgroups = std::max(groups, omega_groups);
  PreparedPlan pp;
  plan_prepared(d, M, pgroups, &pp);
  if (pp.total == 0) return FS_ERR_UNSUPPORTED;
  if (prepared_bytes < pp.total) return FS_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t st = (hipStream_t)stream;
  char* p8 = (char*)prepared;
  int* flag = (int*)(p8 + pp.off_flag);
  if (int rc = launch_fill_u32((uint32_t*)flag, 0u, 1, st)) return rc;
  const int rc = pp.dk == 64
      ? launch_fast_prepare(theta, groups, Omega, omega_groups, pgroups, B, H, qk_scale, (uint16_t*)(p8 + pp.off_Wbf),
                            (float*)(p8 + pp.off_bias), (float*)(p8 + pp.off_wnorm), flag, st)
      : launch_wide_prepare(theta, groups, Omega, omega_groups, pgroups, B, H, qk_scale, (uint16_t*)(p8 + pp.off_Wbf),
                            (float*)(p8 + pp.off_bias), (float*)(p8 + pp.off_wnorm), flag, st);
  if (rc) return rc;
  int host_flag = 0;
  if (hipMemcpyAsync(&host_flag, flag, sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess) return FS_ERR_DEVICE;
  if (hipStreamSynchronize(st) != hipSuccess) return FS_ERR_DEVICE;
  *host_dense_c2 = host_flag & 1;
  return FS_OK;
}

int favorsharp_attention_prepared(const void* prepared, size_t prepared_bytes, int dense_c2, const float* theta,
                                  int groups, const fs_tensor* Q, const fs_tensor* K, const fs_tensor* V, int B, int H,
                                  int Lq, int Lk, int d, int dv, float qk_scale, const float* Omega, int omega_groups,
                                  int M, int causal, int chunk, const fs_tensor* Y, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  if (prepared == nullptr || (dense_c2 != 0 && dense_c2 != 1)) return FS_ERR_INVALID_ARG;
  if (B < 1 || H < 1 || d < 1 || M < 1 || !groups_ok(groups, B, H) || !groups_ok(omega_groups, B, H))
    return FS_ERR_INVALID_ARG;
  PreparedPlan pp;
  plan_prepared(d, M, std::max(groups, omega_groups), &pp);
  if (pp.total == 0 || dv != d) return FS_ERR_UNSUPPORTED;
  if (prepared_bytes < pp.total) return FS_ERR_WORKSPACE_TOO_SMALL;
  return attention_impl(theta, groups, Q, K, V, B, H, Lq, Lk, d, dv, qk_scale, Omega, omega_groups, M, causal, chunk, Y,
                        workspace, workspace_bytes, stream, nullptr, nullptr, prepared, dense_c2);
}

}  // extern "C"

namespace {
int attention_impl(const float* theta, int groups, const fs_tensor* Q, const fs_tensor* K, const fs_tensor* V, int B,
                   int H, int Lq, int Lk, int d, int dv, float qk_scale, const float* Omega, int omega_groups, int M,
                   int causal, int chunk, const fs_tensor* Y, void* workspace, size_t workspace_bytes, void* stream,
                   void* event_main_begin, void* event_main_end, const void* prepared, int dense_c2) {
  if (B < 1 || H < 1 || Lq < 0 || Lk < 1 || d < 1 || dv < 1 || M < 1) return FS_ERR_INVALID_ARG;
  if (!groups_ok(groups, B, H) || !groups_ok(omega_groups, B, H)) return FS_ERR_INVALID_ARG;
  if (causal != 0 && causal != 1) return FS_ERR_INVALID_ARG;
  if (chunk != 0 && chunk != 32 && chunk != 64) return chunk < 0 ? FS_ERR_INVALID_ARG : FS_ERR_UNSUPPORTED;
  if (d > 128 || dv > 128 || !sequences_ok(B, H)) return FS_ERR_UNSUPPORTED;
  if (causal && Lq != Lk) return FS_ERR_UNSUPPORTED;
  if (theta == nullptr || Omega == nullptr || workspace == nullptr || !(qk_scale > 0.f)) return FS_ERR_INVALID_ARG;
  if (!tensor_ok(Q, d, Lq > 0) || !tensor_ok(K, d) || !tensor_ok(V, dv) || !tensor_ok(Y, dv, Lq > 0))
    return FS_ERR_INVALID_ARG;
  if (Q->dtype != K->dtype || Q->dtype != V->dtype) return FS_ERR_INVALID_ARG;
  const int BH = B * H, pgroups = std::max(groups, omega_groups);
  if (workspace_bytes < favorsharp_attention_workspace_bytes(B, H, Lq, Lk, d, dv, M, causal, groups, omega_groups))
    return FS_ERR_WORKSPACE_TOO_SMALL;
  if (Lq == 0) return launch_fill_u32((uint32_t*)workspace, 0u, 1, (hipStream_t)stream);     // no rows: the counter reads 0
  const int lds_limit = device_lds_limit();
  // the bf16 kernels address the rows of a chunk with 32-bit offsets
  const long long max_sl = 1ll << 23;
  const bool small_strides = Q->stride_l < max_sl && K->stride_l < max_sl && V->stride_l < max_sl && Y->stride_l < max_sl;
  if (fast_supported(Q->dtype, d, dv, M) && small_strides && (int)fast_lds_bytes() <= lds_limit) {
    FastPlan fp;
    plan_fast(BH, pgroups, Lk, &fp);
    char* w8 = (char*)workspace;
    FastLaunch f;
    f.Q = dev(Q); f.K = dev(K); f.V = dev(V); f.Y = dev(Y);
    f.theta = theta; f.Omega = Omega;
    f.groups = groups; f.omega_groups = omega_groups; f.pgroups = pgroups;
    f.B = B; f.H = H; f.Lq = Lq; f.Lk = Lk; f.causal = causal;
    f.nseg = fp.nseg; f.rows_per_seg = fp.rows_per_seg; f.sub = fp.sub; f.scale = qk_scale;
    f.Wbf = (uint16_t*)(w8 + fp.off_Wbf); f.bias = (float*)(w8 + fp.off_bias); f.wnorm = (float*)(w8 + fp.off_wnorm);
    f.rk = (float*)(w8 + fp.off_rk); f.Tpart = (float*)(w8 + fp.off_state); f.cpart = (float*)(w8 + fp.off_cpart);
    f.cstar = (float*)(w8 + fp.off_cstar);
    f.flushed = (unsigned*)w8;
    if (fp.Z > 1) { f.rscr = (float*)(w8 + fp.off_rscr); f.cscr = (float*)(w8 + fp.off_cscr); }
    if (prepared != nullptr) {
      PreparedPlan pp;
      plan_prepared(d, M, pgroups, &pp);
      char* p8 = (char*)const_cast<void*>(prepared);
      f.Wbf = (uint16_t*)(p8 + pp.off_Wbf); f.bias = (float*)(p8 + pp.off_bias); f.wnorm = (float*)(p8 + pp.off_wnorm);
      f.pre_mode = dense_c2 ? 1 : 2;
    }
    return launch_fast_attention(f, (hipStream_t)stream, (hipEvent_t)event_main_begin, (hipEvent_t)event_main_end);
  }
  if (wide_supported(Q->dtype, d, dv, M, causal) && (Lq == Lk || !causal) && small_strides &&
      (int)wide_lds_bytes() <= lds_limit) {
    WidePlan wp;
    plan_wide(BH, pgroups, Lq, Lk, &wp);
    char* w8 = (char*)workspace;
    WideLaunch f;
    f.Q = dev(Q); f.K = dev(K); f.V = dev(V); f.Y = dev(Y);
    f.theta = theta; f.Omega = Omega;
    f.groups = groups; f.omega_groups = omega_groups; f.pgroups = pgroups;
    f.B = B; f.H = H; f.L = Lk; f.nslot = wp.nslot; f.rows_per_slot = wp.rows_per_slot; f.scale = qk_scale;
    f.causal = causal;
    f.Lq = Lq; f.nslot_q = wp.nslot_q; f.rows_per_slot_q = wp.rows_per_slot_q;
    f.Wbf = (uint16_t*)(w8 + wp.off_Wbf); f.bias = (float*)(w8 + wp.off_bias); f.wnorm = (float*)(w8 + wp.off_wnorm);
    f.rk = (float*)(w8 + wp.off_rk); f.Tpart = (float*)(w8 + wp.off_state); f.cpart = (float*)(w8 + wp.off_cpart);
    f.cstar = (float*)(w8 + wp.off_cstar); f.Ypart = (float*)(w8 + wp.off_ypart);
    f.flushed = (unsigned*)w8;
    if (prepared != nullptr) {
      PreparedPlan pp;
      plan_prepared(d, M, pgroups, &pp);
      char* p8 = (char*)const_cast<void*>(prepared);
      f.Wbf = (uint16_t*)(p8 + pp.off_Wbf); f.bias = (float*)(p8 + pp.off_bias); f.wnorm = (float*)(p8 + pp.off_wnorm);
      f.pre_mode = dense_c2 ? 1 : 2;
    }
    return launch_wide_attention(f, (hipStream_t)stream, (hipEvent_t)event_main_begin, (hipEvent_t)event_main_end);
  }
  // the general-shape kernels keep no constants across calls: a prepared call of such a shape (other dtype, strides
  // beyond 32-bit offsets) recomputes them like favorsharp_attention
  AttnPlan p;
  plan_contraction(BH, pgroups, Lk, d, M, dv + 1, causal, &p);
  const size_t lds_need = causal ? gen_lds_causal(d, p.ldt) : std::max(gen_lds_state(d, p.ldt), gen_lds_apply(d, p.ldt));
  if ((int)lds_need > lds_limit) return FS_ERR_UNSUPPORTED;

  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  float* W = (float*)(ws + p.off_W);
  uint16_t* Wbf = (uint16_t*)(ws + p.off_Wbf);
  float* bias = (float*)(ws + p.off_bias);
  uint32_t* kmax = (uint32_t*)(ws + p.off_kmax);
  float* state = (float*)(ws + p.off_state);
  const size_t dd = (size_t)d * d;
  const long long tf = (long long)favorsharp_theta_floats(d);

  if (int rc = launch_prep(theta, groups, Omega, omega_groups, pgroups, B, H, M, d, W, Wbf, bias, st)) return rc;
  // the counter word and the key maxima behind it
  unsigned* flushed = (unsigned*)ws;
  if (int rc = launch_fill_u32((uint32_t*)ws, 0u, p.off_kmax / sizeof(uint32_t) + BH, st)) return rc;
  GenSide qs{dev(Q), qk_scale, 0.f, W, bias, theta, groups, pgroups, tf, (long long)(FS_THETA_HEADER + d + 2 * dd)};
  GenSide ks{dev(K), qk_scale, 0.f, W, bias, theta, groups, pgroups, tf, (long long)(FS_THETA_HEADER + d + 3 * dd)};
  ks.rk = (float*)(ws + p.off_rk);      // the key row terms are evaluated once (k_gen_kmax) and read by the kernels after it
  if (int rc = launch_gen_kmax(ks, Lk, BH, H, M, d, kmax, st)) return rc;
  if (int rc = launch_gen_state(ks, dev(V), Lk, BH, H, M, d, dv, 1, p.ldt, p.rows_per_seg, p.nseg, kmax, nullptr, state, st))
    return rc;
  const size_t per_state = (size_t)M * p.ldt;
  if (int rc = launch_gen_reduce(state, BH, p.nseg, per_state, causal, st)) return rc;
  if (event_main_begin && hipEventRecord((hipEvent_t)event_main_begin, st) != hipSuccess) return FS_ERR_DEVICE;
  int rc;
  if (causal)
    rc = launch_gen_causal(qs, ks, dev(V), Lk, BH, H, M, d, dv, p.ldt, p.rows_per_seg, p.nseg, kmax, state, dev(Y), nullptr, nullptr, st, flushed);
  else
    rc = launch_gen_apply(qs, Lq, BH, H, M, d, dv, p.ldt, state, (size_t)p.nseg * per_state, kmax, 0, dev(Y), nullptr, nullptr, st, flushed);
  if (rc) return rc;
  if (event_main_end && hipEventRecord((hipEvent_t)event_main_end, st) != hipSuccess) return FS_ERR_DEVICE;
  return FS_OK;
}
}  // namespace

extern "C" {

int favorsharp_attention_noalloc(const float* theta, int groups, const fs_tensor* Q, const fs_tensor* K,
                                 const fs_tensor* V, int B, int H, int Lq, int Lk, int d, int dv, float qk_scale,
                                 const float* Omega, int omega_groups, int M, int causal, int chunk, const fs_tensor* Y,
                                 void* stream) {
  const size_t need = favorsharp_attention_workspace_bytes(B, H, Lq, Lk, d, dv, M, causal, groups, omega_groups);
  if (need > (size_t)FS_NOALLOC_SCRATCH_BYTES) return FS_ERR_SCRATCH_LIMIT;
  void* ws = nullptr;
  if (need > 0)      // (0: the shapes are invalid or unsupported, and the call below says which)
    if (int rc = scratch_for_current_device(&ws)) return rc;
  // every kernel of the call writes the part of the workspace it later reads: nothing has to start at zero
  return favorsharp_attention_timed(theta, groups, Q, K, V, B, H, Lq, Lk, d, dv, qk_scale, Omega, omega_groups, M,
                                    causal, chunk, Y, ws, FS_NOALLOC_SCRATCH_BYTES, stream, nullptr, nullptr);
}

int favorsharp_attention_flushed_rows(const void* workspace, int* host_count, void* stream) {
  if (host_count == nullptr) return FS_ERR_INVALID_ARG;
  if (workspace == nullptr) {
    void* ws = nullptr;
    if (int rc = scratch_for_current_device(&ws)) return rc;
    workspace = ws;
  }
  hipStream_t st = (hipStream_t)stream;
  unsigned v = 0;
  if (hipMemcpyAsync(&v, workspace, sizeof(unsigned), hipMemcpyDeviceToHost, st) != hipSuccess) return FS_ERR_DEVICE;
  if (hipStreamSynchronize(st) != hipSuccess) return FS_ERR_DEVICE;
  *host_count = (int)std::min(v, 0x7fffffffu);
  return FS_OK;
}

// ------------------------------------------------------------------------------------------ attention, backward
namespace {
struct BwdPlan {
  AttnPlan k, q;           // key-side and query-side segmentations (the projection constants live in `k`)
  size_t off_ghat, off_den, off_shift, off_rstate, off_state2, total;
};

void plan_backward(int BH, int pgroups, int Lq, int Lk, int d, int dv, int M, int causal, BwdPlan* p) {
  plan_contraction(BH, pgroups, Lk, d, M, dv + 1, causal, &p->k);
  plan_contraction(BH, pgroups, Lq, d, M, dv + 1, causal, &p->q);
  size_t off = p->k.total;
  p->off_ghat = off;   off = align_up(off + (size_t)BH * Lq * p->k.ldt * sizeof(float));
  p->off_den = off;    off = align_up(off + (size_t)BH * Lq * sizeof(float));
  p->off_shift = off;  off = align_up(off + (size_t)BH * Lq * sizeof(float));
  p->off_rstate = off; off = align_up(off + (size_t)BH * p->q.nseg * M * p->k.ldt * sizeof(float));
  p->off_state2 = off; off = align_up(off + (causal ? (size_t)BH * p->k.nseg * M * p->k.ldt * sizeof(float) : 0));
  p->total = off;
}
}  // namespace

namespace {
// bf16 path of the non-causal backward pass: the forward plan plus G1 rows and the query-side segment sums.
struct FastBwdPlan {
  FastPlan f;
  int rslots, rows_per_rslot;
  size_t off_gh, off_rpart, off_rcpart, off_rcstar, total;
};

void plan_fast_backward(int BH, int pgroups, int Lq, int Lk, FastBwdPlan* p) {
  plan_fast(BH, pgroups, Lk, &p->f);
  int nseg, rows_per_seg, sub;
  fast_plan(BH, Lq, &nseg, &rows_per_seg, &sub);
  p->rslots = nseg * sub;
  p->rows_per_rslot = rows_per_seg / sub;
  size_t off = p->f.total;
  p->off_gh = off;     off = align_up(off + (size_t)BH * Lq * 80 * sizeof(uint16_t));
  p->off_rpart = off;  off = align_up(off + (size_t)BH * p->rslots * 256 * 80 * sizeof(float));
  p->off_rcpart = off; off = align_up(off + (size_t)BH * p->rslots * sizeof(float));
  p->off_rcstar = off; off = align_up(off + (size_t)BH * sizeof(float));
  p->total = off;
}
}  // namespace

size_t favorsharp_attention_backward_workspace_bytes(int B, int H, int Lq, int Lk, int d, int dv, int M, int causal,
                                                     int groups, int omega_groups) {
  if (B < 1 || H < 1 || Lq < 1 || Lk < 1 || d < 1 || d > 128 || dv < 1 || dv > 128 || M < 1 || !sequences_ok(B, H)) return 0;
  if ((causal != 0 && causal != 1) || (causal && Lq != Lk)) return 0;
  if (!groups_ok(groups, B, H) || !groups_ok(omega_groups, B, H)) return 0;
  BwdPlan p;
  plan_backward(B * H, std::max(groups, omega_groups), Lq, Lk, d, dv, M, causal, &p);
  size_t total = p.total;
  if (fast_supported(FS_BF16, d, dv, M)) {      // the query does not know the dtype: cover both paths
    FastBwdPlan fp;
    plan_fast_backward(B * H, std::max(groups, omega_groups), Lq, Lk, &fp);
    total = std::max(total, fp.total);
  }
  return total;
}

}  // extern "C"

namespace {
int attention_backward_impl(const float* theta, int groups, const fs_tensor* Q, const fs_tensor* K, const fs_tensor* V,
                            const fs_tensor* dY, int B, int H, int Lq, int Lk, int d, int dv, float qk_scale,
                            const float* Omega, int omega_groups, int M, int causal, const fs_tensor* dQ,
                            const fs_tensor* dK, const fs_tensor* dV, void* workspace, size_t workspace_bytes, void* stream,
                            const void* prepared, int dense_c2) {
  if (B < 1 || H < 1 || Lq < 1 || Lk < 1 || d < 1 || dv < 1 || M < 1) return FS_ERR_INVALID_ARG;
  if (!groups_ok(groups, B, H) || !groups_ok(omega_groups, B, H)) return FS_ERR_INVALID_ARG;
  if (causal != 0 && causal != 1) return FS_ERR_INVALID_ARG;
  if (d > 128 || dv > 128 || (causal && Lq != Lk) || !sequences_ok(B, H)) return FS_ERR_UNSUPPORTED;
  if (theta == nullptr || Omega == nullptr || workspace == nullptr || !(qk_scale > 0.f)) return FS_ERR_INVALID_ARG;
  if (!tensor_ok(Q, d) || !tensor_ok(K, d) || !tensor_ok(V, dv) || !tensor_ok(dY, dv)) return FS_ERR_INVALID_ARG;
  if (!tensor_ok(dQ, d) || !tensor_ok(dK, d) || !tensor_ok(dV, dv)) return FS_ERR_INVALID_ARG;
  if (Q->dtype != K->dtype || Q->dtype != V->dtype) return FS_ERR_INVALID_ARG;
  const int BH = B * H, pgroups = std::max(groups, omega_groups);
  if (workspace_bytes < favorsharp_attention_backward_workspace_bytes(B, H, Lq, Lk, d, dv, M, causal, groups, omega_groups))
    return FS_ERR_WORKSPACE_TOO_SMALL;
  // bf16 kernels: d = dv = 64, M = 256, bf16 inputs (dY and the gradients: bf16 or fp32), rows addressable with 32 bits
  const long long max_sl = 1ll << 23;
  if (fast_supported(Q->dtype, d, dv, M) && Q->stride_l < max_sl && K->stride_l < max_sl &&
      V->stride_l < max_sl && dY->stride_l < max_sl && dQ->stride_l < max_sl && dK->stride_l < max_sl &&
      dV->stride_l < max_sl &&
      (int)std::max({fast_lds_bytes(), fast_bwd_lds_bytes(), fast_bwd_causal_lds_bytes()}) <= device_lds_limit()) {
    FastBwdPlan fp;
    plan_fast_backward(BH, pgroups, Lq, Lk, &fp);
    char* w8 = (char*)workspace;
    FastLaunch f;
    f.Q = dev(Q); f.K = dev(K); f.V = dev(V); f.Y = dev(dV);     // no forward output is written on this path
    f.theta = theta; f.Omega = Omega;
    f.groups = groups; f.omega_groups = omega_groups; f.pgroups = pgroups;
    f.B = B; f.H = H; f.Lq = Lq; f.Lk = Lk; f.causal = causal;
    f.nseg = fp.f.nseg; f.rows_per_seg = fp.f.rows_per_seg; f.sub = fp.f.sub; f.scale = qk_scale;
    f.Wbf = (uint16_t*)(w8 + fp.f.off_Wbf); f.bias = (float*)(w8 + fp.f.off_bias); f.wnorm = (float*)(w8 + fp.f.off_wnorm);
    f.rk = (float*)(w8 + fp.f.off_rk); f.Tpart = (float*)(w8 + fp.f.off_state); f.cpart = (float*)(w8 + fp.f.off_cpart);
    f.cstar = (float*)(w8 + fp.f.off_cstar);
    f.flushed = (unsigned*)w8;      // counted by the kernel that recomputes the normalisers
    if (prepared != nullptr) {
      PreparedPlan pp;
      plan_prepared(d, M, pgroups, &pp);
      char* p8 = (char*)const_cast<void*>(prepared);
      f.Wbf = (uint16_t*)(p8 + pp.off_Wbf); f.bias = (float*)(p8 + pp.off_bias); f.wnorm = (float*)(p8 + pp.off_wnorm);
      f.pre_mode = dense_c2 ? 1 : 2;
    }
    return launch_fast_attention_backward(f, dev(dY), dev(dQ), dev(dK), dev(dV), (uint16_t*)(w8 + fp.off_gh),
                                          (float*)(w8 + fp.off_rpart), (float*)(w8 + fp.off_rcpart),
                                          (float*)(w8 + fp.off_rcstar), fp.rslots, fp.rows_per_rslot, (hipStream_t)stream);
  }
  BwdPlan p;
  plan_backward(BH, pgroups, Lq, Lk, d, dv, M, causal, &p);
  const int ldt = p.k.ldt;
  const size_t lds_need = causal ? std::max({gen_lds_state(d, ldt), gen_lds_causal(d, ldt), gen_lds_bwd_causal(d, ldt)})
                                 : std::max({gen_lds_state(d, ldt), gen_lds_apply(d, ldt), gen_lds_bwd_side(d, ldt)});
  if ((int)lds_need > device_lds_limit()) return FS_ERR_UNSUPPORTED;

  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  float* W = (float*)(ws + p.k.off_W);
  uint16_t* Wbf = (uint16_t*)(ws + p.k.off_Wbf);
  float* bias = (float*)(ws + p.k.off_bias);
  uint32_t* kmax = (uint32_t*)(ws + p.k.off_kmax);
  float* state = (float*)(ws + p.k.off_state);
  float* ghat = (float*)(ws + p.off_ghat);
  float* den = (float*)(ws + p.off_den);
  float* shift = (float*)(ws + p.off_shift);
  float* rstate = (float*)(ws + p.off_rstate);
  float* state2 = (float*)(ws + p.off_state2);
  const size_t dd = (size_t)d * d, per_state = (size_t)M * ldt;
  const long long tf = (long long)favorsharp_theta_floats(d);

  // forward quantities: segment states of S^T [V 1] (summed, or their exclusive prefix when causal), then Y, the
  // denominators and the query shifts
  if (int rc = launch_prep(theta, groups, Omega, omega_groups, pgroups, B, H, M, d, W, Wbf, bias, st)) return rc;
  // the counter word and the key maxima behind it
  unsigned* flushed = (unsigned*)ws;
  if (int rc = launch_fill_u32((uint32_t*)ws, 0u, p.k.off_kmax / sizeof(uint32_t) + BH, st)) return rc;
  GenSide qs{dev(Q), qk_scale, 0.f, W, bias, theta, groups, pgroups, tf, (long long)(FS_THETA_HEADER + d + 2 * dd)};
  GenSide ks{dev(K), qk_scale, 0.f, W, bias, theta, groups, pgroups, tf, (long long)(FS_THETA_HEADER + d + 3 * dd)};
  ks.rk = (float*)(ws + p.k.off_rk);      // the key row terms are evaluated once (k_gen_kmax) and read by the kernels after it
  if (int rc = launch_gen_kmax(ks, Lk, BH, H, M, d, kmax, st)) return rc;
  if (int rc = launch_gen_state(ks, dev(V), Lk, BH, H, M, d, dv, 1, ldt, p.k.rows_per_seg, p.k.nseg, kmax, nullptr, state, st))
    return rc;
  if (int rc = launch_gen_reduce(state, BH, p.k.nseg, per_state, causal, st)) return rc;
  const TensorDev gbuf{ghat, 0, (long long)H * Lq * ldt, (long long)Lq * ldt, (long long)ldt};
  if (causal) {
    // the forward kernel advances its copy of the prefix states; the backward query kernel needs them afresh
    if (hipMemcpyAsync(state2, state, (size_t)BH * p.k.nseg * per_state * sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess)
      return FS_ERR_DEVICE;
    if (int rc = launch_gen_causal(qs, ks, dev(V), Lk, BH, H, M, d, dv, ldt, p.k.rows_per_seg, p.k.nseg, kmax, state, gbuf, den,
                                   shift, st, flushed))
      return rc;
  } else {
    if (int rc = launch_gen_apply(qs, Lq, BH, H, M, d, dv, ldt, state, (size_t)p.k.nseg * per_state, kmax, 0, gbuf, den, shift, st,
                                  flushed))
      return rc;
  }
  // G1 in place of Y, then the segment sums of P^T G1 (the query-side twin of the state pass)
  if (int rc = launch_bwd_ghat(dev(dY), ghat, den, Lq, BH, H, dv, ldt, st)) return rc;
  if (int rc = launch_gen_state(qs, gbuf, Lq, BH, H, M, d, ldt, 0, ldt, p.q.rows_per_seg, p.q.nseg, kmax, shift, rstate, st))
    return rc;
  if (int rc = launch_gen_reduce(rstate, BH, p.q.nseg, per_state, causal ? 2 : 0, st)) return rc;
  if (causal)
    return launch_gen_bwd_causal(qs, ks, dev(V), ghat, Lk, BH, H, M, d, dv, ldt, p.k.rows_per_seg, p.k.nseg, kmax, shift,
                                 state2, rstate, dev(dQ), dev(dK), dev(dV), st);
  // query side: dP = G1 T^T -> dQ;  key side: dV = S R, dS = [V 1] R^T -> dK
  if (int rc = launch_gen_bwd_side(qs, 0, gbuf, ldt, 0, Lq, BH, H, M, d, dv, ldt, state, (size_t)p.k.nseg * per_state, kmax,
                                   shift, dev(dV), 0, dev(dQ), st))
    return rc;
  return launch_gen_bwd_side(ks, 1, dev(V), dv, 1, Lk, BH, H, M, d, dv, ldt, rstate, (size_t)p.q.nseg * per_state, kmax,
                             nullptr, dev(dV), 1, dev(dK), st);
}
}  // namespace

extern "C" {

int favorsharp_attention_backward(const float* theta, int groups, const fs_tensor* Q, const fs_tensor* K,
                                  const fs_tensor* V, const fs_tensor* dY, int B, int H, int Lq, int Lk, int d, int dv,
                                  float qk_scale, const float* Omega, int omega_groups, int M, int causal,
                                  const fs_tensor* dQ, const fs_tensor* dK, const fs_tensor* dV, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  return attention_backward_impl(theta, groups, Q, K, V, dY, B, H, Lq, Lk, d, dv, qk_scale, Omega, omega_groups, M, causal,
                                 dQ, dK, dV, workspace, workspace_bytes, stream, nullptr, 0);
}

int favorsharp_attention_backward_prepared(const void* prepared, size_t prepared_bytes, int dense_c2, const float* theta,
                                           int groups, const fs_tensor* Q, const fs_tensor* K, const fs_tensor* V,
                                           const fs_tensor* dY, int B, int H, int Lq, int Lk, int d, int dv,
                                           float qk_scale, const float* Omega, int omega_groups, int M, int causal,
                                           const fs_tensor* dQ, const fs_tensor* dK, const fs_tensor* dV, void* workspace,
                                           size_t workspace_bytes, void* stream) {
  if (prepared == nullptr || (dense_c2 != 0 && dense_c2 != 1)) return FS_ERR_INVALID_ARG;
  if (B < 1 || H < 1 || d < 1 || M < 1 || !groups_ok(groups, B, H) || !groups_ok(omega_groups, B, H))
    return FS_ERR_INVALID_ARG;
  PreparedPlan pp;
  plan_prepared(d, M, std::max(groups, omega_groups), &pp);
  if (pp.total == 0 || dv != d) return FS_ERR_UNSUPPORTED;
  if (prepared_bytes < pp.total) return FS_ERR_WORKSPACE_TOO_SMALL;
  return attention_backward_impl(theta, groups, Q, K, V, dY, B, H, Lq, Lk, d, dv, qk_scale, Omega, omega_groups, M, causal,
                                 dQ, dK, dV, workspace, workspace_bytes, stream, prepared, dense_c2);
}

// ------------------------------------------------------------------------------------------ operator
size_t favorsharp_kernel_matvec_workspace_bytes(int Nx, int Ny, int d, int M, int n) {
  if (Nx < 0 || Ny < 1 || d < 1 || d > 128 || M < 1 || n < 1 || n > 128) return 0;
  AttnPlan p;
  plan_contraction(1, 1, Ny, d, M, n, 0, &p);
  size_t total = p.total;
  if (op_supported(FS_F32, FS_F32, d, M, n)) total = std::max(total, align_up(op_workspace_floats(Ny, d, M) * sizeof(float)));
  return total;
}

int favorsharp_kernel_matvec(const float* theta, const fs_tensor* X, const fs_tensor* Y, int Nx, int Ny, int d,
                             float qk_scale, float alpha, const float* Omega, int M, const float* C, int n, float* out,
                             void* workspace, size_t workspace_bytes, void* stream) {
  if (Nx < 0 || Ny < 1 || d < 1 || M < 1 || n < 1) return FS_ERR_INVALID_ARG;
  if (d > 128 || n > 128) return FS_ERR_UNSUPPORTED;
  if (theta == nullptr || Omega == nullptr || C == nullptr || workspace == nullptr || !(qk_scale > 0.f))
    return FS_ERR_INVALID_ARG;
  if (!tensor_ok(X, d, Nx > 0) || !tensor_ok(Y, d) || X->dtype != Y->dtype) return FS_ERR_INVALID_ARG;
  if (Nx > 0 && out == nullptr) return FS_ERR_INVALID_ARG;
  AttnPlan p;
  plan_contraction(1, 1, Ny, d, M, n, 0, &p);
  if (workspace_bytes < favorsharp_kernel_matvec_workspace_bytes(Nx, Ny, d, M, n)) return FS_ERR_WORKSPACE_TOO_SMALL;
  if (Nx == 0) return FS_OK;
  // fp32 rows, a few right-hand sides: the dedicated kernels (contiguous columns, rows addressed by stride_l)
  if (op_supported(X->dtype, Y->dtype, d, M, n))
    return launch_op_matvec(theta, dev(X), dev(Y), Nx, Ny, d, qk_scale, alpha, Omega, M, C, n, out, (float*)workspace,
                            (hipStream_t)stream);
  if ((int)std::max(gen_lds_state(d, p.ldt), gen_lds_apply(d, p.ldt)) > device_lds_limit()) return FS_ERR_UNSUPPORTED;

  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  float* W = (float*)(ws + p.off_W);
  uint16_t* Wbf = (uint16_t*)(ws + p.off_Wbf);
  float* bias = (float*)(ws + p.off_bias);
  uint32_t* kmax = (uint32_t*)(ws + p.off_kmax);
  float* state = (float*)(ws + p.off_state);
  const size_t dd = (size_t)d * d;
  const long long tf = (long long)favorsharp_theta_floats(d);
  if (int rc = launch_prep(theta, 1, Omega, 1, 1, 1, 1, M, d, W, Wbf, bias, st)) return rc;
  if (int rc = launch_fill_u32(kmax, 0u, 1, st)) return rc;
  GenSide qs{dev(X), qk_scale, alpha, W, bias, theta, 1, 1, tf, (long long)(FS_THETA_HEADER + d + 2 * dd)};
  GenSide ks{dev(Y), qk_scale, alpha, W, bias, theta, 1, 1, tf, (long long)(FS_THETA_HEADER + d + 3 * dd)};
  qs.X.sb = qs.X.sh = ks.X.sb = ks.X.sh = 0;
  TensorDev Cv{C, FS_F32, 0, 0, n};
  TensorDev Ov{out, FS_F32, 0, 0, n};
  if (int rc = launch_gen_kmax(ks, Ny, 1, 1, M, d, kmax, st)) return rc;
  if (int rc = launch_gen_state(ks, Cv, Ny, 1, 1, M, d, n, 0, p.ldt, p.rows_per_seg, p.nseg, kmax, nullptr, state, st)) return rc;
  const size_t per_state = (size_t)M * p.ldt;
  if (int rc = launch_gen_reduce(state, 1, p.nseg, per_state, 0, st)) return rc;
  return launch_gen_apply(qs, Nx, 1, 1, M, d, n, p.ldt, state, (size_t)p.nseg * per_state, kmax, 1, Ov, nullptr, nullptr, st);
}

}  // extern "C"
