// C ABI of the library (see include/la.h) and the host-side blocked algorithms.
//
// Everything is phrased on a LOGICAL lower-triangular factor Lam: a lower factor is the
// row-major view of the caller's buffer, an upper factor R = Lam^T (appendix of arXiv
// 1710.08717, "potrf", last paragraph, and the R variants of trsm / trmm) is the transposed
// view of the same memory, so no data is ever transposed or copied for it.
//
// potrf / backward of small matrices are single register-resident kernels.  Everything else is
// split recursively in halves (multiples of 64) down to 64 x 64 diagonal blocks; all the work
// is GEMMs on the matrix cores: off-diagonal updates, products with (masked) diagonal blocks,
// and solves as products with the diagonal blocks' inverses, which one kernel launch computes
// for the whole batch up front.
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "common.hpp"

namespace la {

static thread_local char g_err[256] = "no error";

void set_error(hipError_t e, const char *where)
{
    snprintf(g_err, sizeof(g_err), "%s: %s", where, hipGetErrorString(e));
}

// ---------------------------------------------------------------------------------
// Scratch memory of the blocked paths: the dense inverses of the 64 x 64 diagonal blocks of the
// triangular factor (batch * ceil(n/64) * 64 * 64 elements).  One buffer per device, grown on
// demand with hipMalloc and kept until the process ends; a buffer that is outgrown is parked,
// not freed, because work queued on a stream may still be using it.  Calls that use it
// (n > 64) must therefore not run concurrently on several streams of one device.
// ---------------------------------------------------------------------------------
struct Scratch {
    void *p = nullptr;
    size_t bytes = 0;
};
static std::mutex g_ws_mutex;
static std::vector<Scratch> g_ws(64);
static std::vector<void *> g_parked;

static la_status scratch_get(size_t bytes, void **out)
{
    int dev = 0;
    LA_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    if (dev < 0 || dev >= (int)g_ws.size())
        return LA_ERR_UNSUPPORTED;
    Scratch &s = g_ws[dev];
    if (s.bytes < bytes) {
        size_t want = bytes + bytes / 4;
        void *np = nullptr;
        LA_HIP(hipMalloc(&np, want));
        if (s.p)
            g_parked.push_back(s.p);
        s.p = np;
        s.bytes = want;
    }
    *out = s.p;
    return LA_OK;
}

// Inverses of the diagonal blocks of one factor: block j of item b at p + b*bs + j*64*64.
template <typename T>
struct InvBlocks {
    T *p = nullptr;
    int64_t bs = 0;
    View<const T> block(int j) const { return {p + (int64_t)j * NB * NB, bs, NB, 1}; }
};

template <typename T>
static la_status inv_alloc(int64_t batch, int n, InvBlocks<T> &inv)
{
    const int nblk = (n + NB - 1) / NB;
    void *p = nullptr;
    LA_TRY(scratch_get((size_t)batch * nblk * NB * NB * sizeof(T), &p));
    inv.p = (T *)p;
    inv.bs = (int64_t)nblk * NB * NB;
    return LA_OK;
}

static inline int split_point(int n)
{
    // first part: a multiple of the tile edge, about half of n, always < n for n > NB
    int h = (n / 2 + NB - 1) / NB * NB;
    return h;
}

template <typename T>
static inline View<const T> cv(View<T> v)
{
    return {v.p, v.bs, v.rs, v.cs};
}

// ---------------------------------------------------------------------------------
// Triangular solve / multiply with a logical lower-triangular Lam (n x n) applied to nvec
// vectors held in X: element e of vector v at X(e, v).
//   solve fwd: X <- Lam^-1 X      solve !fwd: X <- Lam^-T X
//   mult  fwd: X <- Lam X         mult  !fwd: X <- Lam^T X
// ---------------------------------------------------------------------------------
// Leaves (n <= 64) are in-place GEMMs: a solve multiplies by the precomputed inverse of the
// diagonal block (inv, block index blk), a product multiplies by the masked block itself.
// In place is safe there because one workgroup tile covers all n <= 64 rows of its vectors.
template <typename T>
static la_status solve_rec(View<const T> Lam, View<T> X, int64_t batch, int n, int64_t nvec, bool fwd,
                           const InvBlocks<T> &inv, int blk, hipStream_t st)
{
    GemmOpts o;
    if (n <= NB) {
        View<const T> Ib = inv.block(blk);
        return launch_gemm<T>(fwd ? Ib : Ib.t(), cv(X), X, batch, n, (int)nvec, n, T(1), T(0), o, st);
    }
    const int n1 = split_point(n), n2 = n - n1;
    View<const T> L11 = Lam, L21 = Lam.sub(n1, 0), L22 = Lam.sub(n1, n1);
    View<T> X1 = X, X2 = X.sub(n1, 0);
    if (fwd) {
        LA_TRY(solve_rec<T>(L11, X1, batch, n1, nvec, true, inv, blk, st));
        LA_TRY(launch_gemm<T>(L21, cv(X1), X2, batch, n2, (int)nvec, n1, T(-1), T(1), o, st));
        return solve_rec<T>(L22, X2, batch, n2, nvec, true, inv, blk + n1 / NB, st);
    }
    LA_TRY(solve_rec<T>(L22, X2, batch, n2, nvec, false, inv, blk + n1 / NB, st));
    LA_TRY(launch_gemm<T>(L21.t(), cv(X2), X1, batch, n1, (int)nvec, n2, T(-1), T(1), o, st));
    return solve_rec<T>(L11, X1, batch, n1, nvec, false, inv, blk, st);
}

template <typename T>
static la_status mult_rec(View<const T> Lam, View<T> X, int64_t batch, int n, int64_t nvec, bool fwd, hipStream_t st)
{
    GemmOpts o;
    if (n <= NB) {
        o.triA = fwd ? 1 : 2;  // Lam keeps i >= k, Lam^T keeps i <= k
        return launch_gemm<T>(fwd ? Lam : Lam.t(), cv(X), X, batch, n, (int)nvec, n, T(1), T(0), o, st);
    }
    const int n1 = split_point(n), n2 = n - n1;
    View<const T> L11 = Lam, L21 = Lam.sub(n1, 0), L22 = Lam.sub(n1, n1);
    View<T> X1 = X, X2 = X.sub(n1, 0);
    if (fwd) {  // y2 = Lam21 x1 + Lam22 x2 first (needs the old x1), then y1 = Lam11 x1
        LA_TRY(mult_rec<T>(L22, X2, batch, n2, nvec, true, st));
        LA_TRY(launch_gemm<T>(L21, cv(X1), X2, batch, n2, (int)nvec, n1, T(1), T(1), o, st));
        return mult_rec<T>(L11, X1, batch, n1, nvec, true, st);
    }
    // y1 = Lam11^T x1 + Lam21^T x2 first (needs the old x2), then y2 = Lam22^T x2
    LA_TRY(mult_rec<T>(L11, X1, batch, n1, nvec, false, st));
    LA_TRY(launch_gemm<T>(L21.t(), cv(X2), X1, batch, n1, (int)nvec, n2, T(1), T(1), o, st));
    return mult_rec<T>(L22, X2, batch, n2, nvec, false, st);
}

// ---------------------------------------------------------------------------------
// Right-looking blocked potrf on the logical lower triangle held in W (section 4.2:
// A = L L^T).  W already holds tril(A).  off is the index of W's first row in the whole matrix.
// ---------------------------------------------------------------------------------
template <typename T>
static la_status potrf_rec(View<T> W, int32_t *info, int off, int64_t batch, int n, const InvBlocks<T> &inv,
                           hipStream_t st)
{
    if (n <= NB) {
        LA_TRY(launch_potrf_tiny<T>(cv(W), W, info, off, batch, n, st));
        // the inverse of the fresh diagonal block serves every later panel solve against it
        return launch_tile_inverse<T>(cv(W), inv.p, inv.bs, batch, n, off / NB, st);
    }
    const int n1 = split_point(n), n2 = n - n1;
    View<T> W21 = W.sub(n1, 0), W22 = W.sub(n1, n1);
    LA_TRY(potrf_rec<T>(W, info, off, batch, n1, inv, st));
    // panel: L21 = A21 L11^-T, i.e. every row x of the panel solves L11 x^T = a^T
    LA_TRY(solve_rec<T>(cv(W), W21.t(), batch, n1, n2, true, inv, off / NB, st));
    // trailing update of the lower triangle: A22 -= L21 L21^T
    GemmOpts o;
    o.maskC = 1;
    LA_TRY(launch_gemm<T>(cv(W21), cv(W21).t(), W22, batch, n2, n2, n1, T(-1), T(1), o, st));
    return potrf_rec<T>(W22, info, off + n1, batch, n2, inv, st);
}

// ---------------------------------------------------------------------------------
// Pieces of the potrf backward expression (section 4.2; appendix "potrf"):
//   Abar = sym( Lam^-T Phi(Lam^T Lbar) Lam^-1 ),  Phi = lower triangle, halved diagonal.
// ---------------------------------------------------------------------------------

// W (lower triangular, zeros above) <- Phi(tril(Lam^T W)), in place.
template <typename T>
static la_status phi_ltw_rec(View<const T> Lam, View<T> W, int64_t batch, int n, hipStream_t st)
{
    GemmOpts o;
    if (n <= NB) {
        // Lam^T (keeps i <= k) times the lower-triangular block (keeps k >= j); lower part kept, diagonal halved
        o.triA = 2;
        o.triB = 1;
        o.maskC = 1;
        o.halfDiag = 1;
        return launch_gemm<T>(Lam.t(), cv(W), W, batch, n, n, n, T(1), T(0), o, st);
    }
    const int n1 = split_point(n), n2 = n - n1;
    View<const T> L21 = Lam.sub(n1, 0), L22 = Lam.sub(n1, n1);
    View<T> W21 = W.sub(n1, 0), W22 = W.sub(n1, n1);
    LA_TRY(phi_ltw_rec<T>(Lam, W, batch, n1, st));
    o.maskC = 1;
    o.halfDiag = 1;
    LA_TRY(launch_gemm<T>(L21.t(), cv(W21), W, batch, n1, n1, n2, T(1), T(1), o, st));
    LA_TRY(mult_rec<T>(L22, W21, batch, n2, n1, false, st));
    return phi_ltw_rec<T>(L22, W22, batch, n2, st);
}

// W (lower triangular) <- W Lam^-1, which stays lower triangular.
template <typename T>
static la_status rsolve_tri_rec(View<const T> Lam, View<T> W, int64_t batch, int n, const InvBlocks<T> &inv, int blk,
                                hipStream_t st)
{
    if (n <= NB)  // rows of W are the vectors: x Lam = b  <=>  Lam^T x^T = b^T
        return solve_rec<T>(Lam, W.t(), batch, n, n, false, inv, blk, st);
    const int n1 = split_point(n), n2 = n - n1;
    View<const T> L21 = Lam.sub(n1, 0), L22 = Lam.sub(n1, n1);
    View<T> W21 = W.sub(n1, 0), W22 = W.sub(n1, n1);
    LA_TRY(rsolve_tri_rec<T>(Lam, W, batch, n1, inv, blk, st));
    LA_TRY(rsolve_tri_rec<T>(L22, W22, batch, n2, inv, blk + n1 / NB, st));
    // X21 = (W21 - X22 Lam21) Lam11^-1
    GemmOpts o;
    o.triA = 1;
    LA_TRY(launch_gemm<T>(cv(W22), L21, W21, batch, n2, n1, n2, T(-1), T(1), o, st));
    return solve_rec<T>(Lam, W21.t(), batch, n1, n2, false, inv, blk, st);
}

template <typename T>
static la_status backward_impl(View<const T> Lam, View<const T> G, View<T> W, int64_t batch, int n, hipStream_t st)
{
    if (n <= 32)
        return launch_backward_tiny<T>(Lam, G, W, batch, n, st);
    InvBlocks<T> inv;
    LA_TRY(inv_alloc<T>(batch, n, inv));
    LA_TRY(launch_tile_inverse<T>(Lam, inv.p, inv.bs, batch, n, 0, st));
    LA_TRY(launch_copy<T>(G, W, batch, n, n, T(1), 1, st));          // W = tril(Lbar)
    LA_TRY(phi_ltw_rec<T>(Lam, W, batch, n, st));                    // W = Phi(Lam^T Lbar)
    LA_TRY(rsolve_tri_rec<T>(Lam, W, batch, n, inv, 0, st));         // W = Phi(.) Lam^-1   (still lower)
    LA_TRY(solve_rec<T>(Lam, W, batch, n, n, false, inv, 0, st));    // W = Lam^-T Phi(.) Lam^-1
    return launch_symmetrize<T>(W, batch, n, T(0.5), st);            // Abar = 1/2 (W + W^T)
}

// ---------------------------------------------------------------------------------
// argument checking helpers
// ---------------------------------------------------------------------------------
static inline bool overlap(const void *a, size_t na, const void *b, size_t nb)
{
    const char *pa = (const char *)a, *pb = (const char *)b;
    return pa < pb + nb && pb < pa + na;
}
static inline size_t esize(la_dtype dt) { return dt == LA_F32 ? 4 : 8; }
static inline bool bad_dtype(la_dtype dt) { return dt != LA_F32 && dt != LA_F64; }
constexpr int MAX_N = 1 << 20;

template <typename T>
static inline View<T> tri_view(T *p, int n, int lower)
{
    const int64_t nn = (int64_t)n * n;
    return lower ? View<T>{p, nn, n, 1} : View<T>{p, nn, 1, n};
}

template <typename T>
static la_status potrf_t(int lower, int64_t batch, int n, const void *A, void *L, int32_t *info, hipStream_t st)
{
    View<const T> Av = tri_view<const T>((const T *)A, n, lower);
    View<T> Lv = tri_view<T>((T *)L, n, lower);
    if (info)
        LA_TRY(launch_fill_i32(info, batch, 0, st));
    if (n <= NB)
        return launch_potrf_tiny<T>(Av, Lv, info, 0, batch, n, st);
    InvBlocks<T> inv;
    LA_TRY(inv_alloc<T>(batch, n, inv));
    LA_TRY(launch_copy<T>(Av, Lv, batch, n, n, T(1), 1, st));  // L = tril(A), zeros above
    return potrf_rec<T>(Lv, info, 0, batch, n, inv, st);
}

template <typename T>
static la_status tri_apply_t(bool solve, int lower, int trans, int rightside, double alpha, int64_t batch, int n, int m,
                             const void *L, const void *A, void *B, hipStream_t st)
{
    View<const T> Lam = tri_view<const T>((const T *)L, n, lower);
    const int64_t nm = (int64_t)n * m;
    // data laid out as the caller gave it; alpha is applied while copying (or in place)
    View<const T> Ain = rightside ? View<const T>{(const T *)A, nm, n, 1} : View<const T>{(const T *)A, nm, m, 1};
    View<T> Bout = rightside ? View<T>{(T *)B, nm, n, 1} : View<T>{(T *)B, nm, m, 1};
    if (A != B || alpha != 1.0)
        LA_TRY(launch_copy<T>(Ain, Bout, batch, rightside ? m : n, rightside ? n : m, (T)alpha, 0, st));
    // vectors: columns of B (left) or rows of B (right); X(e, v) = element e of vector v
    View<T> X = rightside ? View<T>{(T *)B, nm, 1, n} : View<T>{(T *)B, nm, m, 1};
    const bool use_lt = (trans != 0) != (lower == 0);  // t(L) equals Lam^T
    const bool fwd = (use_lt == (rightside != 0));
    if (!solve)
        return mult_rec<T>(Lam, X, batch, n, m, fwd, st);
    InvBlocks<T> inv;
    LA_TRY(inv_alloc<T>(batch, n, inv));
    LA_TRY(launch_tile_inverse<T>(Lam, inv.p, inv.bs, batch, n, 0, st));
    return solve_rec<T>(Lam, X, batch, n, m, fwd, inv, 0, st);
}

template <typename T>
static la_status syrk_t(int trans, double alpha, int64_t batch, int n, int k, const void *A, void *B, hipStream_t st)
{
    const int64_t nk = (int64_t)n * k, nn = (int64_t)n * n;
    View<const T> Ank = trans ? View<const T>{(const T *)A, nk, 1, n} : View<const T>{(const T *)A, nk, k, 1};  // n x k
    View<T> C{(T *)B, nn, n, 1};
    GemmOpts o;
    o.maskC = 1;
    LA_TRY(launch_gemm<T>(Ank, Ank.t(), C, batch, n, n, k, (T)alpha, T(0), o, st));
    return launch_mirror_lower<T>(C, batch, n, st);
}

}  // namespace la

using namespace la;

extern "C" {

la_status la_potrf_batched(la_dtype dt, int lower, int64_t batch, int n, const void *A, void *L, int32_t *info,
                           void *stream)
{
    if (bad_dtype(dt) || batch < 0 || n < 0 || n > MAX_N)
        return LA_ERR_INVALID_ARG;
    if (batch == 0 || n == 0)
        return LA_OK;
    if (!A || !L)
        return LA_ERR_INVALID_ARG;
    const size_t bytes = (size_t)batch * n * n * esize(dt);
    if (A != L && overlap(A, bytes, L, bytes))
        return LA_ERR_INVALID_ARG;
    if (info && (overlap(info, (size_t)batch * 4, L, bytes) || overlap(info, (size_t)batch * 4, A, bytes)))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    return dt == LA_F32 ? potrf_t<float>(lower, batch, n, A, L, info, st)
                        : potrf_t<double>(lower, batch, n, A, L, info, st);
}

la_status la_potrf_backward(la_dtype dt, int lower, int64_t batch, int n, const void *L, const void *Lbar, void *Abar,
                            void *stream)
{
    if (bad_dtype(dt) || batch < 0 || n < 0 || n > MAX_N)
        return LA_ERR_INVALID_ARG;
    if (batch == 0 || n == 0)
        return LA_OK;
    if (!L || !Lbar || !Abar)
        return LA_ERR_INVALID_ARG;
    const size_t bytes = (size_t)batch * n * n * esize(dt);
    if (overlap(L, bytes, Abar, bytes) || (Lbar != Abar && overlap(Lbar, bytes, Abar, bytes)))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (dt == LA_F32)
        return backward_impl<float>(tri_view<const float>((const float *)L, n, lower),
                                    tri_view<const float>((const float *)Lbar, n, lower),
                                    tri_view<float>((float *)Abar, n, lower), batch, n, st);
    return backward_impl<double>(tri_view<const double>((const double *)L, n, lower),
                                 tri_view<const double>((const double *)Lbar, n, lower),
                                 tri_view<double>((double *)Abar, n, lower), batch, n, st);
}

static la_status tri_apply(bool solve, la_dtype dt, int lower, int trans, int rightside, double alpha, int64_t batch,
                           int n, int m, const void *L, const void *A, void *B, void *stream)
{
    if (bad_dtype(dt) || batch < 0 || n < 0 || m < 0 || n > MAX_N || m > MAX_N)
        return LA_ERR_INVALID_ARG;
    if (batch == 0 || n == 0 || m == 0)
        return LA_OK;
    if (!L || !A || !B)
        return LA_ERR_INVALID_ARG;
    const size_t lb = (size_t)batch * n * n * esize(dt), ab = (size_t)batch * n * m * esize(dt);
    if (overlap(L, lb, B, ab) || (A != B && overlap(A, ab, B, ab)))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    return dt == LA_F32 ? tri_apply_t<float>(solve, lower, trans, rightside, alpha, batch, n, m, L, A, B, st)
                        : tri_apply_t<double>(solve, lower, trans, rightside, alpha, batch, n, m, L, A, B, st);
}

la_status la_trsm_batched(la_dtype dt, int lower, int trans, int rightside, double alpha, int64_t batch, int n, int m,
                          const void *L, const void *A, void *B, void *stream)
{
    return tri_apply(true, dt, lower, trans, rightside, alpha, batch, n, m, L, A, B, stream);
}

la_status la_trmm_batched(la_dtype dt, int lower, int trans, int rightside, double alpha, int64_t batch, int n, int m,
                          const void *L, const void *A, void *B, void *stream)
{
    return tri_apply(false, dt, lower, trans, rightside, alpha, batch, n, m, L, A, B, stream);
}

la_status la_syrk_batched(la_dtype dt, int trans, double alpha, int64_t batch, int n, int k, const void *A, void *B,
                          void *stream)
{
    if (bad_dtype(dt) || batch < 0 || n < 0 || k < 0 || n > MAX_N || k > MAX_N)
        return LA_ERR_INVALID_ARG;
    if (batch == 0 || n == 0)
        return LA_OK;
    if (!B || (k > 0 && !A))
        return LA_ERR_INVALID_ARG;
    const size_t ab = (size_t)batch * n * k * esize(dt), bb = (size_t)batch * n * n * esize(dt);
    if (k > 0 && overlap(A, ab, B, bb))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    return dt == LA_F32 ? syrk_t<float>(trans, alpha, batch, n, k, A, B, st)
                        : syrk_t<double>(trans, alpha, batch, n, k, A, B, st);
}

la_status la_sumlogdiag(la_dtype dt, int64_t batch, int n, const void *L, void *out, void *stream)
{
    if (bad_dtype(dt) || batch < 0 || n < 0 || n > MAX_N)
        return LA_ERR_INVALID_ARG;
    if (batch == 0)
        return LA_OK;
    if (!out || (n > 0 && !L))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    return dt == LA_F32 ? launch_sumlogdiag<float>((const float *)L, (float *)out, batch, n, st)
                        : launch_sumlogdiag<double>((const double *)L, (double *)out, batch, n, st);
}

la_status la_gp_glue(la_dtype dt, int64_t batch, int n, const void *L, const void *y, const void *z, const void *alpha,
                     void *loss, void *Lbar, void *stream)
{
    if (bad_dtype(dt) || batch < 0 || n < 0 || n > MAX_N)
        return LA_ERR_INVALID_ARG;
    if (batch == 0)
        return LA_OK;
    if (!loss || (n > 0 && (!L || !y || !z || !alpha || !Lbar)))
        return LA_ERR_INVALID_ARG;
    const size_t bytes = (size_t)batch * n * n * esize(dt);
    if (n > 0 && overlap(L, bytes, Lbar, bytes))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    return dt == LA_F32 ? launch_gp_glue<float>((const float *)L, (const float *)y, (const float *)z,
                                                (const float *)alpha, (float *)loss, (float *)Lbar, batch, n, st)
                        : launch_gp_glue<double>((const double *)L, (const double *)y, (const double *)z,
                                                 (const double *)alpha, (double *)loss, (double *)Lbar, batch, n, st);
}

const char *la_last_error(void) { return g_err; }

int la_version(void) { return 100; }

}  // extern "C"
