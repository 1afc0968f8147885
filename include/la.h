/*
 * la.h - C ABI of the MI355X (gfx950) batched Cholesky operator library.
 *
 * Operators follow "Auto-Differentiating Linear Algebra" (arXiv 1710.08717),
 * section 4 (operator table) and section 4.2 ("Cholesky Decomposition. Related
 * Operators"), with the backward expressions of the appendix.
 *
 * Common conventions
 * ------------------
 *  - Every pointer except where stated is a DEVICE pointer owned by the caller.
 *  - Matrices are full rectangles in ROW-MAJOR order (section 4.1, "BLAS and
 *    LAPACK": flat storage, no packed triangles).  A batched operand of shape
 *    [batch, r, c] is contiguous: item i starts at base + i*r*c elements
 *    ("batch mode", section 4.1; the caller flattens all leading axes into batch).
 *  - dt selects the element type of every matrix argument (LA_F32 / LA_F64).
 *  - lower != 0: the triangular factor is lower triangular L (A = L L^T).
 *    lower == 0: it is upper triangular R (A = R^T R; appendix, last paragraph
 *    of "potrf", and the R variants of trsm / trmm).  Entries on the other side
 *    of the diagonal of a triangular INPUT are never read.
 *  - trans != 0 applies t(L) = L^T, rightside != 0 multiplies / solves from the
 *    right (operator table and section 4.2).
 *  - stream is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *    only enqueue work on that stream and return; results are ready when the
 *    stream reaches that point.
 *  - batch == 0 or a zero matrix dimension is valid: LA_OK, nothing is launched.
 *  - Return value: LA_OK, or LA_ERR_INVALID_ARG (null pointer with non-empty
 *    work, negative size, bad enum, forbidden aliasing), LA_ERR_UNSUPPORTED,
 *    LA_ERR_RUNTIME (a HIP call failed; see la_last_error()).
 *    LA_ERR_WORKSPACE: the call needs more scratch memory than it was given.
 *  - The library allocates nothing and keeps no device memory or other state between
 *    calls; it is re-entrant, and calls on different streams may overlap as long as
 *    their workspaces differ.  Small problems (potrf and potri with n <= 128, backward with
 *    n <= 128 in fp32 and <= 96 in fp64, trsm with n <= 128 and at most 48 right-hand
 *    sides and with n <= 512 and at most 512 of them, every operator with n <= 32 on operands of at
 *    most 16 vectors / an inner dimension of at most 32, sumlogdiag, gp_glue, gp_criterion up to the
 *    same n as backward, kalman_filter) need no scratch memory; la_workspace_bytes() is the authority.  The blocked paths for larger
 *    n do (explicit inverses of the factor or of its diagonal blocks, a working copy of
 *    the triangle being factored or one work panel, partial results of products split
 *    along a long inner dimension): la_workspace_bytes() says how many bytes a call
 *    takes, and the caller passes that much device memory to the entry point's _ws form.
 *    The plain form of an entry point is its _ws form without a workspace: it returns
 *    LA_ERR_WORKSPACE (and launches nothing) when the call needs one.
 *    A workspace is device memory, 256-byte aligned, disjoint from every operand; its
 *    contents are undefined after the call; it may be reused by the next call on the
 *    same stream and must not be shared by calls that may run at the same time.
 */
#ifndef LA_MI355X_H
#define LA_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LA_OK = 0,
    LA_ERR_INVALID_ARG = 1,
    LA_ERR_UNSUPPORTED = 2,
    LA_ERR_RUNTIME = 3,
    LA_ERR_WORKSPACE = 4
} la_status;
typedef enum { LA_F32 = 0, LA_F64 = 1 } la_dtype;
typedef enum {
    LA_OP_POTRF = 0,
    LA_OP_POTRF_BACKWARD = 1,
    LA_OP_TRSM = 2,
    LA_OP_TRMM = 3,
    LA_OP_SYRK = 4,
    LA_OP_GEMM2 = 5,
    LA_OP_TRSM_BACKWARD = 6,
    LA_OP_TRMM_BACKWARD = 7,
    LA_OP_SYRK_BACKWARD = 8,
    LA_OP_GEMM2_BACKWARD = 9,
    LA_OP_POTRI = 10,
    LA_OP_POTRI_BACKWARD = 11
} la_op;

/* Scratch memory, in bytes, that one call of operator `op` takes for these sizes (0: none).  The
 * sizes carry the names they have in the operator's own signature: n for potrf, its backward,
 * potri and its backward; n and m for trsm / trmm and their backward rules; n and k for syrk and
 * its backward; m, n and k for gemm2 and its backward; the others are ignored.  The answer holds
 * for every value of the operator's flags and alpha and for every aliasing it permits (the
 * section 4.2 operators "need no extra memory" when built on vendor solvers; here the blocked
 * paths trade scratch for work that runs on the matrix cores).  Host-only: no GPU call is made.
 * Bad arguments give 0. */
size_t la_workspace_bytes(la_op op, la_dtype dt, int64_t batch, int n, int m, int k);

/* potrf forward (operator table row "potrf"; section 4.2): for each item,
 * L lower triangular with positive diagonal and A = L L^T (lower != 0), or R upper
 * with A = R^T R (lower == 0).  A, L: [batch, n, n].  Only the named triangle of A
 * is read; the other triangle of the output is written as exact zeros.  L may be
 * the same buffer as A (the paper's "L can overwrite A"); partial overlap is
 * forbidden.  info: NULL, or int32 [batch] on the device: 0, or the 1-based index
 * of the first pivot that is not > 0 (that item's factor is then unspecified from
 * that column on; the call still returns LA_OK). */
la_status la_potrf_batched(la_dtype dt, int lower, int64_t batch, int n, const void *A, void *L,
                           int32_t *info, void *stream);
la_status la_potrf_batched_ws(la_dtype dt, int lower, int64_t batch, int n, const void *A, void *L,
                           int32_t *info, void *workspace,
        size_t workspace_bytes, void *stream);

/* la_potrf_batched for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results
 * and errors as la_potrf_batched; the scratch of the blocked path (n > 128) is a static array of
 * LA_NOALLOC_SCRATCH_BYTES in device memory that every GPU the library is loaded on holds until the
 * process ends.  No hipMalloc / hipFree, no allocating library call.  A problem whose
 * la_workspace_bytes(LA_OP_POTRF, ...) exceeds that size is refused with LA_ERR_WORKSPACE (text in
 * la_last_error()) before anything is launched: in fp64 one matrix up to n = 1672, or any batch with
 * batch * n * n <= 2.79e6; twice that in fp32 (above 23e6 elements per batch or n >= 4096 the
 * limit is a third lower).  All calls on one GPU share that array: calls that may run at the same time on
 * one GPU (different streams or threads) race and must be serialised by the caller; successive
 * calls on one stream are fine, the array needs no clearing between them.  The first call on a
 * device looks up the array's address and should therefore be made outside graph capture. */
#define LA_NOALLOC_SCRATCH_BYTES (64u << 20)
la_status la_potrf_batched_noalloc(la_dtype dt, int lower, int64_t batch, int n, const void *A, void *L,
                                   int32_t *info, void *stream);

/* potrf backward (section 4.2, backward of potrf; appendix "potrf"):
 *   Abar = 1/2 L^{-T} copyltu(L^T Lbar) L^{-1}                      (lower != 0)
 *   Abar = 1/2 R^{-1} copyutl(Rbar R^T) R^{-T}                      (lower == 0)
 * evaluated as sym(L^{-T} Phi(L^T Lbar) L^{-1}) with Phi = lower triangle with
 * halved diagonal, which is the same matrix (copyltu X = Phi X + (Phi X)^T).
 * L, Lbar, Abar: [batch, n, n].  Only the named triangles of L and Lbar are read.
 * Abar is written in full and is exactly symmetric.  Abar may be the same buffer
 * as Lbar ("Abar can overwrite Lbar"); it must not overlap L. */
la_status la_potrf_backward(la_dtype dt, int lower, int64_t batch, int n, const void *L,
                            const void *Lbar, void *Abar, void *stream);
la_status la_potrf_backward_ws(la_dtype dt, int lower, int64_t batch, int n, const void *L,
                            const void *Lbar, void *Abar, void *workspace,
        size_t workspace_bytes, void *stream);

/* trsm (section 4.2 "trsm"): B = alpha * t(L)^{-1} A   (rightside == 0, A,B: [batch, n, m])
 *                            B = alpha * A t(L)^{-1}   (rightside != 0, A,B: [batch, m, n])
 * L: [batch, n, n] triangular (see lower).  alpha = 1 is the paper's operator.
 * B may be the same buffer as A; neither may overlap L. */
la_status la_trsm_batched(la_dtype dt, int lower, int trans, int rightside, double alpha,
                          int64_t batch, int n, int m, const void *L, const void *A, void *B,
                          void *stream);
la_status la_trsm_batched_ws(la_dtype dt, int lower, int trans, int rightside, double alpha,
                          int64_t batch, int n, int m, const void *L, const void *A, void *B,
                          void *workspace,
        size_t workspace_bytes, void *stream);

/* trmm (section 4.2 "trmm"): B = alpha * t(L) A   (rightside == 0, A,B: [batch, n, m])
 *                            B = alpha * A t(L)   (rightside != 0, A,B: [batch, m, n])
 * Same shapes and aliasing rules as la_trsm_batched. */
la_status la_trmm_batched(la_dtype dt, int lower, int trans, int rightside, double alpha,
                          int64_t batch, int n, int m, const void *L, const void *A, void *B,
                          void *stream);
la_status la_trmm_batched_ws(la_dtype dt, int lower, int trans, int rightside, double alpha,
                          int64_t batch, int n, int m, const void *L, const void *A, void *B,
                          void *workspace,
        size_t workspace_bytes, void *stream);

/* trsm backward (section 4.2 "trsm", backward; appendix "trsm", also for an upper factor).
 * For the forward B = alpha t(L)^{-1} A (or alpha A t(L)^{-1}), with Y = t(L)^{-T} Bbar (or
 * Bbar t(L)^{-T}):
 *   Abar = alpha Y,
 *   Lbar = -tri(Y B^T), -tri(B Y^T), -tri(B^T Y), -tri(Y^T B)   for (left, t = no), (left, t = yes),
 *          (right, t = no), (right, t = yes); tri = tril for lower != 0, triu for lower == 0.
 * With alpha = 1 these are the paper's four cases with Abar in place of Y.
 * L, Lbar: [batch, n, n]; B (the forward OUTPUT), Bbar, Abar: [batch, n, m] or [batch, m, n] as
 * in la_trsm_batched.  Lbar is written in full (zeros in the other triangle).  Abar may be the
 * same buffer as Bbar and Lbar the same buffer as L ("Abar can overwrite Bbar", "Lbar can
 * overwrite L"); any other overlap is an error. */
la_status la_trsm_backward(la_dtype dt, int lower, int trans, int rightside, double alpha, int64_t batch,
                           int n, int m, const void *L, const void *B, const void *Bbar, void *Abar,
                           void *Lbar, void *stream);
la_status la_trsm_backward_ws(la_dtype dt, int lower, int trans, int rightside, double alpha, int64_t batch,
                           int n, int m, const void *L, const void *B, const void *Bbar, void *Abar,
                           void *Lbar, void *workspace,
        size_t workspace_bytes, void *stream);

/* trmm backward (section 4.2 "trmm", backward; appendix "trmm"): for the forward
 * B = alpha t(L) A (or alpha A t(L)):
 *   Abar = alpha t(L)^T Bbar  (or alpha Bbar t(L)^T),
 *   Lbar = alpha tri(Bbar A^T), tri(A Bbar^T), tri(A^T Bbar), tri(Bbar^T A)   (same four cases).
 * A is the forward INPUT.  Shapes as above.  Lbar is computed first, so Abar may be the same
 * buffer as Bbar; Lbar must not overlap L or anything else. */
la_status la_trmm_backward(la_dtype dt, int lower, int trans, int rightside, double alpha, int64_t batch,
                           int n, int m, const void *L, const void *A, const void *Bbar, void *Abar,
                           void *Lbar, void *stream);
la_status la_trmm_backward_ws(la_dtype dt, int lower, int trans, int rightside, double alpha, int64_t batch,
                           int n, int m, const void *L, const void *A, const void *Bbar, void *Abar,
                           void *Lbar, void *workspace,
        size_t workspace_bytes, void *stream);

/* syrk backward (section 4.2 "syrk", backward; Bbar need not be symmetric):
 *   B = alpha A A^T (trans == 0):  Abar = 2 alpha sym(Bbar) A = alpha (Bbar + Bbar^T) A
 *   B = alpha A^T A (trans != 0):  Abar = alpha A (Bbar + Bbar^T)
 * A, Abar: [batch, n, k] (trans == 0) or [batch, k, n]; Bbar: [batch, n, n].  Abar must not
 * overlap A or Bbar. */
la_status la_syrk_backward(la_dtype dt, int trans, double alpha, int64_t batch, int n, int k, const void *A,
                           const void *Bbar, void *Abar, void *stream);
la_status la_syrk_backward_ws(la_dtype dt, int trans, double alpha, int64_t batch, int n, int k, const void *A,
                           const void *Bbar, void *Abar, void *workspace,
        size_t workspace_bytes, void *stream);

/* syrk (section 4.2 "syrk"): B = alpha * A A^T  (trans == 0, A: [batch, n, k])
 *                            B = alpha * A^T A  (trans != 0, A: [batch, k, n])
 * B: [batch, n, n], both triangles written, exactly symmetric.  B must not
 * overlap A. */
la_status la_syrk_batched(la_dtype dt, int trans, double alpha, int64_t batch, int n, int k,
                          const void *A, void *B, void *stream);
la_status la_syrk_batched_ws(la_dtype dt, int trans, double alpha, int64_t batch, int n, int k,
                          const void *A, void *B, void *workspace,
        size_t workspace_bytes, void *stream);

/* gemm2 (section 4.2 "gemm2"): C = alpha * t_a(A) t_b(B), t_a(A): m x k, t_b(B): k x n.
 * A: [batch, m, k] (ta == 0) or [batch, k, m] (ta != 0); B: [batch, k, n] (tb == 0) or
 * [batch, n, k] (tb != 0); C: [batch, m, n].  C must not overlap A or B ("does not allow
 * in-place computation"). */
la_status la_gemm2_batched(la_dtype dt, int ta, int tb, double alpha, int64_t batch, int m, int n, int k,
                           const void *A, const void *B, void *C, void *stream);
la_status la_gemm2_batched_ws(la_dtype dt, int ta, int tb, double alpha, int64_t batch, int m, int n, int k,
                           const void *A, const void *B, void *C, void *workspace,
        size_t workspace_bytes, void *stream);

/* gemm2 backward (section 4.2 "gemm2", backward): for C = alpha t_a(A) t_b(B),
 *   Abar = alpha Cbar t_b(B)^T  (ta == 0)  or  alpha t_b(B) Cbar^T  (ta != 0),
 *   Bbar = alpha t_a(A)^T Cbar  (tb == 0)  or  alpha Cbar^T t_a(A)  (tb != 0),
 * each in the storage shape of its operand (see la_gemm2_batched); Cbar: [batch, m, n].
 * Abar and Bbar must not overlap each other or any input. */
la_status la_gemm2_backward(la_dtype dt, int ta, int tb, double alpha, int64_t batch, int m, int n, int k,
                            const void *A, const void *B, const void *Cbar, void *Abar, void *Bbar,
                            void *stream);
la_status la_gemm2_backward_ws(la_dtype dt, int ta, int tb, double alpha, int64_t batch, int m, int n, int k,
                            const void *A, const void *B, const void *Cbar, void *Abar, void *Bbar,
                            void *workspace,
        size_t workspace_bytes, void *stream);

/* potri (section 4.2 "potri"): B = A^{-1} from the Cholesky factor of A,
 *   A = L L^T (lower != 0)  or  A = R^T R (lower == 0).
 * L, B: [batch, n, n]; only the named triangle of the factor is read; B is written in full and is
 * exactly symmetric.  B may be the same buffer as L ("B can overwrite L"). */
la_status la_potri(la_dtype dt, int lower, int64_t batch, int n, const void *L, void *B, void *stream);
la_status la_potri_ws(la_dtype dt, int lower, int64_t batch, int n, const void *L, void *B, void *workspace,
        size_t workspace_bytes, void *stream);

/* potri backward (section 4.2 "potri", backward; appendix "potri"; Bbar need not be symmetric):
 *   Lbar = -2 tril(B sym(Bbar) L^{-T})   (lower != 0)
 *   Rbar = -2 triu(R^{-T} sym(Bbar) B)   (lower == 0)
 * B is the forward output A^{-1}.  All operands [batch, n, n]; Lbar is written in full (zeros in the
 * other triangle) and must not overlap any input. */
la_status la_potri_backward(la_dtype dt, int lower, int64_t batch, int n, const void *L, const void *B,
                            const void *Bbar, void *Lbar, void *stream);
la_status la_potri_backward_ws(la_dtype dt, int lower, int64_t batch, int n, const void *L, const void *B,
                            const void *Bbar, void *Lbar, void *workspace,
        size_t workspace_bytes, void *stream);

/* log|L| = sum_i log l_ii (section 3.1, identity below the GP criterion code).
 * L: [batch, n, n]; out: [batch] of dt.  Plain log, no abs: a non-positive
 * diagonal gives NaN / -inf. n == 0 gives 0. */
la_status la_sumlogdiag(la_dtype dt, int64_t batch, int n, const void *L, void *out, void *stream);

/* Gaussian-process criterion glue (section 3.1; trsm backward, first case, of
 * section 4.2).  Given the factor L of the noisy kernel matrix, targets y,
 * z = L^{-1} y and alpha = L^{-T} z (two la_trsm_batched calls):
 *   loss[b] = 1/2 y^T alpha + sum_i log l_ii      (the criterion minus n/2 log 2 pi)
 *   Lbar    = -tril(alpha z^T) + diag(1 / l_ii)   (gradient of loss w.r.t. L)
 * L, Lbar: [batch, n, n]; y, z, alpha: [batch, n]; loss: [batch].  Lbar is written
 * in full (zeros above the diagonal) and must not overlap L.  Lower factor only. */
la_status la_gp_glue(la_dtype dt, int64_t batch, int n, const void *L, const void *y, const void *z,
                     const void *alpha, void *loss, void *Lbar, void *stream);

/* Gaussian-process criterion and its gradient in one call (section 3.1; backward rules of section
 * 4.2): for each item, with A the kernel matrix plus noise (symmetric positive definite; its lower
 * triangle is read) and targets y,
 *   L = potrf(A),  z = L^{-1} y,  alpha = L^{-T} z,
 *   loss = 1/2 y^T alpha + sum_i log l_ii           (the criterion minus n/2 log 2 pi),
 *   Abar = d loss / d A = 1/2 (A^{-1} - alpha alpha^T), obtained as the potrf backward of
 *          Lbar = -tril(alpha z^T) + diag(1 / l_ii); written in full, exactly symmetric.
 * A, Abar: [batch, n, n]; y: [batch, n]; loss: [batch]; info: NULL or int32 [batch] as for potrf.
 * Abar may be the same buffer as A.  Up to n = 128 (fp32) / 96 (fp64) this is ONE kernel per call
 * and needs no workspace; beyond that it is the sequence la_potrf_batched, two la_trsm_batched,
 * la_gp_glue, la_potrf_backward on `workspace` (device memory, 256-byte aligned, at least
 * la_gp_workspace_bytes(dt, batch, n) bytes, not overlapping the other arguments). */
size_t la_gp_workspace_bytes(la_dtype dt, int64_t batch, int n);
la_status la_gp_criterion(la_dtype dt, int64_t batch, int n, const void *A, const void *y, void *loss, void *Abar,
                          int32_t *info, void *workspace, size_t workspace_bytes, void *stream);

/* Variational sparse Gaussian-process criterion and its gradient (section 3.2: the criterion is
 * -log N(y | 0, Q + lam I) + tr(Kff - Q) / (2 lam) with Q = Kuf^T Kuu^-1 Kuf, evaluated through two
 * Cholesky factors of U x U matrices; the gradient is the reverse sweep over that evaluation with the
 * backward rules of section 4.2).  One problem per call:
 *   Lu = potrf(Kuu);  B = Lu^{-1} Kuf;  A = B B^T / lam + I;  La = potrf(A);  w = La^{-1} (B y);
 *   phi = (log 2 pi + log lam) n / 2 + sum_i log La_ii + |y|^2 / (2 lam) - |w|^2 / (2 lam^2)
 *         - (|B|_F^2 - sum Kff_diag) / (2 lam),            lam = noise_var > 0.
 * Device inputs: Kuu [U, U] (lower triangle read), Kuf [U, n], Kff_diag [n], y [n].  Device outputs:
 * phi [1], Kuu_bar [U, U] (symmetric: d phi = <Kuu_bar, dKuu> for symmetric dKuu), Kuf_bar [U, n],
 * Kff_diag_bar [n], y_bar [n], noise_bar [1].  workspace: device memory, at least
 * la_sgp_workspace_bytes(dt, U, n) bytes (intermediate results plus the scratch of the blocked
 * operators inside), 256-byte aligned; outputs and workspace must not overlap the inputs or each
 * other. */
size_t la_sgp_workspace_bytes(la_dtype dt, int U, int n);
la_status la_sgp_criterion(la_dtype dt, int U, int n, const void *Kuu, const void *Kuf, const void *Kff_diag,
                           const void *y, double noise_var, void *phi, void *Kuu_bar, void *Kuf_bar,
                           void *Kff_diag_bar, void *y_bar, void *noise_bar, void *workspace,
                           size_t workspace_bytes, void *stream);

/* Kalman filter over a batch of sequences (section 3.4): Gaussian linear dynamical system
 *   h_t ~ N(A h_{t-1}, S_h),  v_t ~ N(B h_t, S_v),  h_0 ~ N(mu_0, S_0),   h in R^dh, v in R^dv.
 * For every sequence and t = 0 .. T-1, in the order of the section's equations:
 *   mu_h = A f_{t-1}, S_hh = A F_{t-1} A^T + S_h   (t = 0: mu_h = mu_0, S_hh = S_0);
 *   mu_v = B mu_h;  S_vv = B S_hh B^T + S_v = L L^T;  K = (S_hh B^T) L^{-T} L^{-1};
 *   f_t = mu_h + K (v_t - mu_v);  F_t = (I - K B) S_hh (I - K B)^T + K S_v K^T;
 * and the negative log likelihood the section trains on,
 *   nll = sum_t [ dv/2 log 2 pi + sum_i log L_ii + 1/2 |L^{-1} (v_t - mu_v)|^2 ].
 * 1 <= dh, dv <= 16 (anything else: LA_ERR_UNSUPPORTED).  All pointers are device memory, row-major.
 * Parameters A [dh,dh], B [dv,dh], S_h [dh,dh], S_v [dv,dv], mu_0 [dh], S_0 [dh,dh]: one set for every
 * sequence (shared_params != 0) or one per sequence with a leading [batch] axis.  v: [batch, T, dv].
 * Outputs: nll [batch]; f [batch, T, dh] or NULL; F [batch, T, dh, dh] or NULL; info: NULL or int32
 * [batch]: 0, or 1 + the first step whose S_vv has a pivot that is not > 0 (that sequence's outputs
 * are then unspecified from that step on; the call still returns LA_OK).  No scratch memory. */
la_status la_kalman_filter(la_dtype dt, int64_t batch, int T, int dh, int dv, int shared_params, const void *A,
                           const void *B, const void *Sh, const void *Sv, const void *mu0, const void *S0,
                           const void *v, void *f, void *F, void *nll, int32_t *info, void *stream);

/* Text of the last HIP error seen by this thread's calls (host pointer, never NULL). */
const char *la_last_error(void);

/* Library version as major*10000 + minor*100 + patch. */
int la_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LA_MI355X_H */
