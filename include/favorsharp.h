/*
 * favorsharp.h -- C ABI of the FAVOR# hot path for AMD MI355X (gfx950).
 *
 * FAVOR# approximates the softmax / Gaussian kernel operator with positive
 * "dense-exponential" random features (DERFs):
 *
 *     f^(k)(omega, x) = D exp(omega^T A omega + omega^T B^(k) x + x^T C^(k) x),   k = 1 (queries), 2 (keys)
 *
 * (paper Section 4, DERF definition), with parameters theta = {A, B1, B2, C1, C2, D}
 * fitted in closed form to statistics of the query / key sets (Theorems on
 * ADERF and SDERF, Section 4.3 for SADERF, Section 2.3 for GERF / PosRF).
 * With P[i,m] = M^-1/2 f1(omega_m, x_i), S[j,m] = M^-1/2 f2(omega_m, y_j)
 * (Section 2.1) the kernel matrix is estimated by K_hat = P S^T and every
 * product K_hat C costs O(L M n).
 *
 * Conventions for every entry point
 *   - returns an fs_status; never throws, never aborts, never allocates device
 *     memory: the caller owns every buffer, including the workspace, whose
 *     size comes from the matching *_workspace_bytes query (same shapes)
 *     (favorsharp_attention_noalloc alone uses a buffer the library owns);
 *   - pointers are DEVICE pointers unless the name starts with host_;
 *   - work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream).  favorsharp_fit_params additionally waits for the
 *     stream (its d x d closed form runs on the host in fp64); the others
 *     return as soon as their kernels are enqueued;
 *   - outputs are fully overwritten, inputs are never modified; the workspace
 *     content is undefined afterwards; calls that share a workspace must be
 *     ordered by the caller; there is no global mutable state apart from
 *     favorsharp_attention_noalloc's scratch array;
 *   - tensors are row-major; an fs_tensor carries element strides for the
 *     batch, head and row axes, the innermost (feature) axis has stride 1 and
 *     row starts must be 16-byte aligned (stride_l a multiple of 8 for bf16, of 4 for f32);
 *   - x = qk_scale * Q_i and y = qk_scale * K_j are the vectors the paper's
 *     formulas see (attention: qk_scale = d^-1/4, Section 2.2).
 */
#ifndef FAVORSHARP_H
#define FAVORSHARP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FS_OK = 0,
  FS_ERR_INVALID_ARG = 1,        /* null pointer, bad shape / stride / dtype / enum */
  FS_ERR_UNSUPPORTED = 2,        /* valid but outside what the kernels cover (d > 128, causal with Lq != Lk,
                                    B * H > 65535: the sequences are a grid dimension, ...) */
  FS_ERR_NOT_PD = 3,             /* fit: statistics are singular where the theorem needs them nonsingular */
  FS_ERR_WORKSPACE_TOO_SMALL = 4,
  FS_ERR_DEVICE = 5,             /* a HIP call failed */
  FS_ERR_SCRATCH_LIMIT = 6       /* favorsharp_attention_noalloc: the call needs more than FS_NOALLOC_SCRATCH_BYTES */
} fs_status;

typedef enum { FS_F32 = 0, FS_BF16 = 1 } fs_dtype;

/* Which closed-form family favorsharp_fit_params fits. */
typedef enum {
  FS_POSRF = 0,   /* A = 0: exp(omega.x - |x|^2/2)                         (Section 2.3) */
  FS_GERF = 1,    /* scalar A, homogeneity heuristic                        (Sections 2.3, 3.1) */
  FS_SADERF = 2,  /* GERF on (Psi x, Psi^-1 y), diagonal Psi                (Section 4.3) */
  FS_ADERF = 3,   /* A = a I, B1 != B2, via eig(M1), eig(M2) and one SVD    (Theorem on ADERF) */
  FS_SDERF = 4    /* B1 = B2, diagonal A, via one eigendecomposition        (Theorem on SDERF) */
} fs_variant;

/* A [B, H, L, d] tensor (or [L, d] with B = H = 1): element strides, innermost stride 1. */
typedef struct {
  const void* ptr;     /* device */
  int32_t dtype;       /* fs_dtype */
  int64_t stride_b;
  int64_t stride_h;
  int64_t stride_l;
} fs_tensor;

/*
 * Layout of one parameter set theta (float32, `favorsharp_theta_floats(d)` values):
 *   [0] log D   [1] fitted value of the shifted log-variance objective (Section 3.1; NaN if none)
 *   [2] flags (as a float; bit 0 set: C1 = C2 = -I/2 exactly, bit 1 set: B1 = B2)   [3] fs_variant   [4..7] reserved
 *   then diag(A)[d], B1[d*d], B2[d*d], C1[d*d], C2[d*d], all row-major.
 * The flags are promises the kernels rely on (a set bit lets them skip the dense quadratic form, or use one
 * projection matrix for both sides); the fits set them, and a caller who builds theta by hand sets a bit only when
 * the arrays satisfy it exactly (0 is always safe).
 * A parameter buffer holds `groups` such sets back to back; the set used for
 * batch b, head h is 0 (groups = 1), h (groups = H) or b*H + h (groups = B*H).
 */
#define FS_THETA_HEADER 8
size_t favorsharp_theta_floats(int d);

const char* favorsharp_status_string(int status);
const char* favorsharp_version(void);

/*
 * Fit theta from data statistics (Theorems on ADERF / SDERF, Sections 2.3, 3.1, 4.3).
 * Per group: mu4 = mean x, mu5 = mean y, M1 = mean x x^T, M2 = mean y y^T over all rows of
 * all (b, h) that map to the group (one scan of X and Y on the GPU), then the variant's closed form
 * (eigendecompositions / SVD of d x d matrices in fp64 on the host), written to `theta`.
 *   X: [B, H, Lx, d], Y: [B, H, Ly, d] (f32 or bf16, same dtype); d <= 128; groups in {1, H, B*H}.
 *   eig_ridge >= 0 is added to the diagonals of M1 and M2 before the ADERF decompositions (0 = exact theorem).
 *   theta: device, groups * favorsharp_theta_floats(d) floats, overwritten.
 * Synchronous with respect to `stream`.  FS_ERR_NOT_PD when ADERF / SADERF meet a singular statistic.
 */
size_t favorsharp_fit_workspace_bytes(int B, int H, int Lx, int Ly, int d, int groups);
int favorsharp_fit_params(int variant, const fs_tensor* X, const fs_tensor* Y,
                          int B, int H, int Lx, int Ly, int d, float qk_scale, int groups,
                          float eig_ridge, float* theta, void* workspace, size_t workspace_bytes,
                          void* stream);

/*
 * The same fit without a host round trip (the paper names the eigendecomposition on accelerators as the
 * practical obstacle of the dense families, Section 4.3 and the discussion of limitations): the statistics scan and
 * the closed forms of the Theorems on ADERF / SDERF and of Sections 2.3, 3.1, 4.3 all run on the device, the
 * d x d decompositions as one-sided Jacobi iterations in fp64, one workgroup per group.
 * Arguments as favorsharp_fit_params, plus
 *   status: device, `groups` int32 values, overwritten: FS_OK, or FS_ERR_NOT_PD for a group whose statistics are
 *           singular where ADERF / SADERF need them nonsingular (that group's theta is then left unwritten).
 * Asynchronous: returns once the kernels are enqueued on `stream`; theta and status are valid after the stream
 * reaches that point.  The returned value covers argument and launch errors only.
 * Eigenvectors are unique only up to sign and up to rotations inside equal-eigenvalue blocks, so theta may differ
 * from favorsharp_fit_params' in exactly those freedoms; log D, diag(A), the objective value, B^T B and the kernel
 * estimate's distribution are the same.
 */
size_t favorsharp_fit_device_workspace_bytes(int B, int H, int Lx, int Ly, int d, int groups);
int favorsharp_fit_params_device(int variant, const fs_tensor* X, const fs_tensor* Y,
                                 int B, int H, int Lx, int Ly, int d, float qk_scale, int groups,
                                 float eig_ridge, float* theta, int32_t* status,
                                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * Materialise one side of the feature matrix (Section 2.1: rows of P for side = 1, of S for side = 2):
 *   out[i, m] = M^-1/2 exp(alpha |x_i|^2) f^(side)(omega_m, x_i),  x_i = qk_scale * X[i, :]
 * (Section 2.3 for the exp(alpha |x|^2) factor that turns softmax-kernel features into K^(alpha) features).
 *   X: [n, d] (stride_l used; B = H = 1), theta: one parameter set, Omega: [M, d] float32 rows omega_m,
 *   out: [n, M] float32.  If row_logscale != NULL (n floats) the row is stabilised:
 *   row_logscale[i] = max_m log out[i, m] and out[i, m] is divided by exp(row_logscale[i]).
 */
size_t favorsharp_features_workspace_bytes(int n, int d, int M);
int favorsharp_features(const float* theta, int side, const fs_tensor* X, int n, int d,
                        float qk_scale, float alpha, const float* Omega, int M,
                        float* out, float* row_logscale,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Attention with K_hat in place of the softmax kernel matrix (Section 2.2, the attention equation):
 *   Y[b,h,i,:] = sum_j K_hat[i,j] V[b,h,j,:] / sum_j K_hat[i,j],   K_hat = P S^T,
 * over all j (causal = 0) or over j <= i (causal = 1, requires Lq == Lk).  P and S are never written to memory.
 *   Q: [B,H,Lq,d], K: [B,H,Lk,d], V: [B,H,Lk,dv], Y: [B,H,Lq,dv] (Y->ptr is written; dtypes f32 or bf16,
 *   Q, K, V share one dtype, Y may differ); d <= 128, dv <= 128.
 *   theta: `groups` parameter sets, Omega: [omega_groups, M, d] float32, groups and omega_groups in {1, H, B*H}.
 *   chunk: rows per step of the causal prefix-state recurrence; it changes the schedule, not the result
 *   (0 = library default; supported: 32 or 64).
 */
size_t favorsharp_attention_workspace_bytes(int B, int H, int Lq, int Lk, int d, int dv, int M,
                                            int causal, int groups, int omega_groups);
int favorsharp_attention(const float* theta, int groups, const fs_tensor* Q, const fs_tensor* K,
                         const fs_tensor* V, int B, int H, int Lq, int Lk, int d, int dv,
                         float qk_scale, const float* Omega, int omega_groups, int M,
                         int causal, int chunk, const fs_tensor* Y,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward pass of favorsharp_attention: gradients of  sum(Y * dY)  with respect to Q, K and V (the chain rule on
 * the attention equation of Section 2.2 with K_hat = P S^T; theta and omega are constants of the feature map, as
 * in the paper's training experiments where theta is fitted from the data's statistics, Sections 3.1 and 4.3).
 * Nothing from the forward call is needed: the state, the outputs and the denominators are recomputed.
 *   Q, K, V as in favorsharp_attention; dY: [B,H,Lq,dv] (f32 or bf16); dQ: [B,H,Lq,d], dK: [B,H,Lk,d],
 *   dV: [B,H,Lk,dv] are written (->ptr; f32 or bf16 each).
 *   causal = 1 differentiates the causal variant (sum over j <= i; requires Lq == Lk): a forward sweep with the
 *   prefix states and a backward sweep with the suffix sums of P^T G1.  Asynchronous on `stream`.
 */
size_t favorsharp_attention_backward_workspace_bytes(int B, int H, int Lq, int Lk, int d, int dv, int M,
                                                     int causal, int groups, int omega_groups);
int favorsharp_attention_backward(const float* theta, int groups, const fs_tensor* Q, const fs_tensor* K,
                                  const fs_tensor* V, const fs_tensor* dY, int B, int H, int Lq, int Lk, int d, int dv,
                                  float qk_scale, const float* Omega, int omega_groups, int M, int causal,
                                  const fs_tensor* dQ, const fs_tensor* dK, const fs_tensor* dV,
                                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * Unbiased estimate of the kernel operator K^(alpha)(X, Y) C (Section 2.1, the problem statement):
 *   out = P (S^T C),  P, S built from x_i = qk_scale * X[i,:], y_j = qk_scale * Y[j,:] with the
 *   exp(alpha |.|^2) factors of Section 2.3, D and M^-1/2 all kept (alpha = -1/2: Gaussian kernel).
 *   X: [Nx, d], Y: [Ny, d] (same dtype), C: [Ny, n] float32 contiguous, out: [Nx, n] float32, n <= 128.
 */
size_t favorsharp_kernel_matvec_workspace_bytes(int Nx, int Ny, int d, int M, int n);
int favorsharp_kernel_matvec(const float* theta, const fs_tensor* X, const fs_tensor* Y,
                             int Nx, int Ny, int d, float qk_scale, float alpha,
                             const float* Omega, int M, const float* C, int n, float* out,
                             void* workspace, size_t workspace_bytes, void* stream);

/*
 * favorsharp_attention with two optional hipEvent_t handles (NULL to skip) around the kernel that performs the
 * contraction of Section 2.1 / 2.2 for most of the rows (the causal segment pass, or the query-side pass when
 * causal = 0): on the bf16 paths the events are attached to that kernel's dispatch and carry its own begin and end
 * times (for d = dv = 128: begin of the first, end of the second launch of the walk); on the general path
 * event_main_begin is recorded on `stream` right before the kernel and event_main_end right after it.  For measuring
 * that kernel alone from outside; the result is identical to favorsharp_attention.
 */
int favorsharp_attention_timed(const float* theta, int groups, const fs_tensor* Q, const fs_tensor* K,
                               const fs_tensor* V, int B, int H, int Lq, int Lk, int d, int dv,
                               float qk_scale, const float* Omega, int omega_groups, int M,
                               int causal, int chunk, const fs_tensor* Y,
                               void* workspace, size_t workspace_bytes, void* stream,
                               void* event_main_begin, void* event_main_end);

/*
 * Attention with the projection constants kept across calls.  The evaluation recipe of Section 4 precomputes
 * B^T omega once per parameter set; favorsharp_attention does so on every call because theta and Omega may have
 * changed.  When they have not, favorsharp_attention_prepare computes the constants (W~ = log2e qk_scale Omega B of
 * both sides as bf16, the per-feature terms log2e (omega^T A omega + log D - 1/2 log M) and the row norms of W~)
 * into a caller-owned buffer once, and favorsharp_attention_prepared runs the rest of favorsharp_attention from
 * it.  Results are bit-identical to favorsharp_attention with the same theta, Omega and qk_scale.
 *   favorsharp_prepared_bytes: size of that buffer; 0 for shapes without constants to keep (the kernels that keep
 *     them are the bf16 ones: d = dv = 64 with M = 256, and d = dv = 128 with M = 512).
 *   favorsharp_attention_prepare: theta, Omega, groups as in favorsharp_attention; prepared: device, overwritten;
 *     host_dense_c2 (HOST pointer, out): 1 if some parameter set has a C2 other than -I/2 (ADERF, SADERF: the key
 *     row terms y^T C2 y then still have to be recomputed from K on every call), else 0.  SYNCHRONOUS with respect to
 *     `stream`.  FS_ERR_UNSUPPORTED for shapes with favorsharp_prepared_bytes = 0.
 *   favorsharp_attention_prepared: `prepared`, `dense_c2` as left / reported by favorsharp_attention_prepare for the
 *     same theta, Omega, groups, omega_groups, B, H, d, M and qk_scale (the caller vouches for that: the buffer is
 *     not checked); all other arguments, the workspace and the statuses as favorsharp_attention.  Asynchronous.
 */
size_t favorsharp_prepared_bytes(int B, int H, int d, int M, int groups, int omega_groups);
int favorsharp_attention_prepare(const float* theta, int groups, const float* Omega, int omega_groups,
                                 int B, int H, int d, int M, float qk_scale,
                                 void* prepared, size_t prepared_bytes, int* host_dense_c2, void* stream);
int favorsharp_attention_prepared(const void* prepared, size_t prepared_bytes, int dense_c2,
                                  const float* theta, int groups, const fs_tensor* Q, const fs_tensor* K,
                                  const fs_tensor* V, int B, int H, int Lq, int Lk, int d, int dv,
                                  float qk_scale, const float* Omega, int omega_groups, int M,
                                  int causal, int chunk, const fs_tensor* Y,
                                  void* workspace, size_t workspace_bytes, void* stream);
/*
 * favorsharp_attention_backward on the same kept constants (Section 4, evaluation recipe: B^T omega is computed once per
 * parameter set, here for the forward and the backward call of a training step alike): `prepared`, `dense_c2` as for
 * favorsharp_attention_prepared, every other argument, the workspace and the statuses as
 * favorsharp_attention_backward.  Gradients are bit-identical to favorsharp_attention_backward's.  Shapes whose
 * gradient kernels keep no constants (everything but bf16 rows with d = dv = 64, M = 256) recompute them.
 * Asynchronous.
 */
int favorsharp_attention_backward_prepared(const void* prepared, size_t prepared_bytes, int dense_c2,
                                           const float* theta, int groups, const fs_tensor* Q, const fs_tensor* K,
                                           const fs_tensor* V, const fs_tensor* dY, int B, int H, int Lq, int Lk,
                                           int d, int dv, float qk_scale, const float* Omega, int omega_groups, int M,
                                           int causal, const fs_tensor* dQ, const fs_tensor* dK, const fs_tensor* dV,
                                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * favorsharp_attention for callers that cannot allocate or pass device memory of their own: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and result as favorsharp_attention
 * minus the workspace: the scratch memory is a fixed array of FS_NOALLOC_SCRATCH_BYTES that the library holds on
 * every GPU it runs on until the process ends.  The call allocates nothing (no hipMalloc / hipFree, no allocating
 * library routine); its first call on a device looks the array's address up once.
 *   FS_ERR_SCRATCH_LIMIT when favorsharp_attention_workspace_bytes(same shapes) exceeds FS_NOALLOC_SCRATCH_BYTES
 *   (nothing is enqueued then); the other statuses as favorsharp_attention.
 * All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (different streams,
 * different host threads) race and must be ordered by the caller.  The array keeps the last call's contents; the
 * kernels write every part of it before they read it.
 */
#define FS_NOALLOC_SCRATCH_BYTES (64u << 20)
int favorsharp_attention_noalloc(const float* theta, int groups, const fs_tensor* Q, const fs_tensor* K,
                                 const fs_tensor* V, int B, int H, int Lq, int Lk, int d, int dv,
                                 float qk_scale, const float* Omega, int omega_groups, int M,
                                 int causal, int chunk, const fs_tensor* Y, void* stream);

/*
 * Denominator guard of the attention equation (Section 2.2: the row sums of K_hat divide the output).  With positive
 * features the row sum is positive mathematically; in fp32 a query row whose largest feature exponent lies more than
 * about 2^126 below the row's own shift, or that meets only key features flushed the same way, can still give a row
 * sum of exactly 0.  Every attention entry point above then writes that output row as zeros instead of dividing, and
 * counts it: the first 32-bit word of the call's workspace holds, once the call's kernels have finished, the number
 * of such rows of that call (all (b, h) together; every call starts it at 0).  favorsharp_attention_backward
 * recomputes the normalisers and counts the same rows in the first word of ITS workspace: such a row gets a zero
 * dQ row and contributes nothing to dK and dV.  A caller that wants no host synchronisation reads that word from
 * the workspace itself; this function does it for them:
 *   workspace:  the workspace of the attention (or backward) call in question (device), or NULL for the scratch
 *               array of favorsharp_attention_noalloc on the current device;
 *   host_count: (out, host) the counter.
 * SYNCHRONOUS with respect to `stream` (pass the attention call's stream).  FS_ERR_INVALID_ARG on a null
 * host_count, FS_ERR_DEVICE when the copy fails.
 */
int favorsharp_attention_flushed_rows(const void* workspace, int* host_count, void* stream);

/*
 * Block-orthogonal random features (the appendix on the classification experiments says the omegas there are
 * orthogonal; the construction is not printed in the paper: this is the textbook one).  HOST function, host pointers:
 *   host_gauss_dir, host_gauss_len: [groups][M][d] float32, independent N(0,1) draws supplied by the caller;
 *   host_omega (out):               [groups][M][d] float32.
 * The M rows of a group are taken in blocks of d (the last block may be shorter); inside a block the rows of
 * host_gauss_dir are orthonormalised in order (Gram-Schmidt, double precision), and row i is then given the length
 * |host_gauss_len[i,:]|, so that every omega_i is marginally N(0, I_d) while the directions of a block are exactly
 * orthogonal.  FS_ERR_NOT_PD if a block is numerically rank deficient, FS_ERR_INVALID_ARG on null pointers or
 * non-positive sizes.  No device work, no stream.
 */
int favorsharp_orthogonal_omega(const float* host_gauss_dir, const float* host_gauss_len, int groups, int M, int d,
                                float* host_omega);

#ifdef __cplusplus
}
#endif
#endif /* FAVORSHARP_H */
