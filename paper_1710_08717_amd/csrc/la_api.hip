// C ABI of the library (see include/la.h) and the host-side blocked algorithms.
//
// Everything is phrased on a LOGICAL lower-triangular factor Lam: a lower factor is the
// row-major view of the caller's buffer, an upper factor R = Lam^T (appendix of arXiv
// 1710.08717, "potrf", last paragraph, and the R variants of trsm / trmm) is the transposed
// view of the same memory, so no data is ever transposed or copied for it.
//
// potrf / backward of small matrices are single register-resident kernels, blocks of up to 128
// rows one-workgroup kernels that keep the block in LDS.  Everything larger is host code over
// those and GEMMs on the matrix cores: off-diagonal updates, products with (masked) triangular
// blocks, and solves as products with explicit inverses of diagonal blocks (128 x 128 blocks by
// one launch for the whole batch, merged level by level where larger ones are wanted).
// The library owns no device memory: scratch comes out of the workspace the caller passes to the
// _ws form of an entry point (la_workspace_bytes says how much a call takes).
#include <cstdio>
#include <cstring>
#include <mutex>

#include "common.hpp"

namespace la {

static thread_local char g_err[256] = "no error";

void set_error(hipError_t e, const char *where)
{
    snprintf(g_err, sizeof(g_err), "%s: %s", where, hipGetErrorString(e));
}

// ---------------------------------------------------------------------------------
// Scratch memory (see common.hpp): the arena of the call that is running on this thread.
// ---------------------------------------------------------------------------------
Arena *&current_arena()
{
    static thread_local Arena *a = nullptr;
    return a;
}

la_status arena_take(size_t bytes, void **out)
{
    Arena *a = current_arena();
    const size_t need = (bytes + 255) & ~(size_t)255;
    if (!a || (!a->dry && a->used + need > a->cap)) {
        snprintf(g_err, sizeof(g_err), "workspace too small: %zu more bytes wanted at offset %zu of %zu", need,
                 a ? a->used : (size_t)0, a ? a->cap : (size_t)0);
        return LA_ERR_WORKSPACE;
    }
    *out = a->base + a->used;
    a->used += need;
    if (a->used > a->peak)
        a->peak = a->used;
    return LA_OK;
}

template <typename T>
static la_status scratch_views(int64_t batch, int n, int count, View<T> *out)
{
    // `count` row-major n x n matrices per batch item, each batch-contiguous
    const int64_t nn = (int64_t)n * n;
    void *p = nullptr;
    LA_TRY(arena_take((size_t)count * batch * nn * sizeof(T), &p));
    for (int c = 0; c < count; ++c)
        out[c] = View<T>{(T *)p + (int64_t)c * batch * nn, nn, n, 1};
    return LA_OK;
}

// Rough time, per unit of K, of the lower-triangle update C -= P P^T on n2 rows: the product
// kernel runs two workgroups per compute unit (512 slots), with 128 x 128 tiles from 2048 rows on
// and 64 x 64 tiles below, and a launch costs whole rounds of tiles: 528 tiles take twice as long
// as 496.  (Relative figures measured on this kernel: a full round, a round that leaves half of
// the compute units with a single workgroup.)
static double lower_update_cost(int n2)
{
    const bool big = n2 >= 2048;
    const int e = big ? 128 : 64;
    const int64_t t = (n2 + e - 1) / e, c = t * (t + 1) / 2;
    const double full = big ? 0.30 : 0.11, half = big ? 0.18 : 0.06;
    const int64_t rounds = c / 512, rem = c % 512;
    return rounds * full + (rem > 256 ? full : (rem > 0 ? half : 0.0));
}

static inline int split_point(int n)
{
    // first part: a multiple of the tile edge (of 128 for larger n), about half of n, always < n
    // for n > NB; moved up by at most n / 8 if that lets the trailing update run in full rounds
    const int step = n >= 512 ? 2 * NB : NB;
    const int h = (n / 2 + step - 1) / step * step;
    if (n < 2048)
        return h;
    int best = h;
    double best_score = lower_update_cost(n - h) / ((double)(n - h) * (n - h));
    for (int n1 = h + step; n1 <= h + n / 8 && n1 < n; n1 += step) {
        const double score = lower_update_cost(n - n1) / ((double)(n - n1) * (n - n1));
        if (score < 0.95 * best_score) {
            best = n1;
            best_score = score;
        }
    }
    return best;
}

template <typename T>
static inline View<const T> cv(View<T> v)
{
    return {v.p, v.bs, v.rs, v.cs, v.bs2, v.nb2};
}

// ---------------------------------------------------------------------------------
// Explicit inverse of a lower-triangular Lam (n x n) into Inv (n x n, lower triangle; what lies
// above the diagonal is never written and never read).  First the 128 x 128 diagonal blocks (one
// launch for the whole batch), then level by level
//     inv [A 0; C D] = [A^-1 0; -D^-1 C A^-1, D^-1]
// with all pairs of one level in one batched GEMM pair.  Stops when blocks of `upto` are
// inverted (upto >= n: the whole matrix).  Tmp: scratch of at least n*n/2 per item.
// ---------------------------------------------------------------------------------
template <typename T>
static la_status inverse_merge(View<const T> Lam, View<T> Inv, View<T> Tmp, int64_t batch, int n, int upto,
                               hipStream_t st);

template <typename T>
static la_status inverse_build(View<const T> Lam, View<T> Inv, View<T> Tmp, int64_t batch, int n, int upto,
                               hipStream_t st)
{
    LA_TRY(launch_tri_inverse128<T>(Lam, Inv, batch, n, st));
    return inverse_merge<T>(Lam, Inv, Tmp, batch, n, upto, st);
}

// The merge levels of inverse_build alone: Inv already holds the inverses of the 128 x 128 diagonal blocks.
template <typename T>
static la_status inverse_merge(View<const T> Lam, View<T> Inv, View<T> Tmp, int64_t batch, int n, int upto,
                               hipStream_t st)
{
    for (int64_t h = 2 * NB; h < upto && h < n; h *= 2) {
        const int nfull = (int)(n / (2 * h));                       // pairs whose right block is a full h
        const int r = (int)(n - (int64_t)nfull * 2 * h - h);        // rows of a ragged right block (if > 0)
        for (int pass = 0; pass < 2; ++pass) {
            const int cnt = pass == 0 ? nfull : (r > 0 ? 1 : 0);
            if (cnt == 0)
                continue;
            const int64_t o0 = pass == 0 ? 0 : (int64_t)nfull * 2 * h;  // first row of the first pair
            const int mr = pass == 0 ? (int)h : r;
            View<const T> A = cv(Inv).sub(o0, o0).level2(2 * h * (Inv.rs + Inv.cs), cnt);
            View<const T> D = cv(Inv).sub(o0 + h, o0 + h).level2(2 * h * (Inv.rs + Inv.cs), cnt);
            View<const T> C = Lam.sub(o0 + h, o0).level2(2 * h * (Lam.rs + Lam.cs), cnt);
            View<T> O = Inv.sub(o0 + h, o0).level2(2 * h * (Inv.rs + Inv.cs), cnt);
            View<T> Tv{Tmp.p + (pass == 0 ? 0 : (int64_t)nfull * h * h), Tmp.bs, h, 1, h * h, cnt};
            GemmOpts o1, o2;
            o1.triA = 1;     // D^-1 is lower triangular: the K range grows with the tile row,
            o1.reverse = 1;  //   so the last rows go first
            o2.triB = 1;     // A^-1 is lower triangular: the K range shrinks with the tile column
                             //   (the launcher enumerates such tiles column by column)
            LA_TRY(launch_gemm<T>(D, C, Tv, batch * cnt, mr, (int)h, mr, T(1), T(0), o1, st));
            LA_TRY(launch_gemm<T>(cv(Tv), A, O, batch * cnt, mr, (int)h, (int)h, T(-1), T(0), o2, st));
        }
    }
    return LA_OK;
}

// ---------------------------------------------------------------------------------
// Right-looking blocked potrf with panels of 128 columns: per panel one leaf launch (factor and
// inverse of the diagonal block), one product for the rows below (L21 = A21 Li11^T) and one for
// the trailing lower triangle.  No merged inverses, so fewer launches than the recursion for a
// stand-alone problem of a few panels; every update has K = 128 only, which is why large
// matrices take the recursion.
// ---------------------------------------------------------------------------------
template <typename T>
static la_status potrf_right_looking(View<T> Wk, View<T> L, int32_t *info, int off, int64_t batch, int n, View<T> Inv,
                                     hipStream_t st)
{
    constexpr int P = 2 * NB;
    for (int o = 0; o < n; o += P) {
        const int nb = n - o < P ? n - o : P, r = n - o - nb;
        LA_TRY(launch_potrf_leaf16<T>(cv(Wk).sub(o, o), L.sub(o, o), Inv.sub(o, o), info, off + o, batch, nb, false, st));
        if (r == 0)
            break;
        View<T> L21 = L.sub(o + nb, o);
        GemmOpts op;
        op.triB = 2;  // Li11^T is upper triangular
        LA_TRY(launch_gemm<T>(cv(Wk).sub(o + nb, o), cv(Inv).sub(o, o).t(), L21, batch, r, nb, nb, T(1), T(0), op, st));
        GemmOpts ou;
        ou.maskC = 1;
        LA_TRY(launch_gemm<T>(cv(L21), cv(L21).t(), Wk.sub(o + nb, o + nb), batch, r, r, nb, T(-1), T(1), ou, st));
    }
    return LA_OK;
}

// ---------------------------------------------------------------------------------
// Blocked potrf by recursive halving (section 4.2: A = L L^T).  Wk holds the lower triangle of
// the block still to be factored (a working copy, updated in place), L receives the factor, Inv
// the inverses of the factors of the diagonal sub-blocks; off is the index of the block's first
// row in the whole matrix.
//   [A11 . ; A21 A22]:  L11, Li11 = rec(A11);  L21 = A21 Li11^T;  A22 -= L21 L21^T;  L22 = rec(A22)
// Every panel solve is ONE product with the explicit inverse of the left factor, so a left
// child always returns its complete inverse, merged from its own children's by
//   Li21 = -Li22 (L21 Li11)
// (need_inv; a right child needs it only if its parent does).  The extra products add one sixth
// to the n^3 / 3 of the factorisation and remove every recursive solve.  The temporary
// L21 Li11 lives in the unused upper-right block of the node's part of Inv.
// The halving stops at blocks of about 2000 rows, which are factored panel by panel
// (potrf_right_looking) and, where the parent needs it, inverted level by level with all pairs
// of a level in one launch (inverse_merge, temporary in Tmp): the long dependent chain of small
// launches at the bottom of the recursion is what a large factorisation waits for.
// ---------------------------------------------------------------------------------
template <typename T>
static la_status potrf_rec(View<T> Wk, View<T> L, int32_t *info, int off, int64_t batch, int n, View<T> Inv,
                           View<T> Tmp, bool need_inv, hipStream_t st)
{
    if (n <= 2 * NB)  // factor and inverse in one launch
        return launch_potrf_leaf16<T>(cv(Wk), L, Inv, info, off, batch, n, false, st);
    // Blocks of up to 2304 rows: panel by panel.  Measured against halving all the way down: one matrix
    // of n = 2048 0.95 -> 0.77 ms, 3000 1.78 -> 1.38, 4096 2.58 -> 2.19, 8192 8.62 -> 7.89 (fp64); with many
    // matrices in the batch the short products of the panels stop paying (32 x 1024: 0.91 -> 0.93).
    if (n <= 2304 && (double)batch * n * n < 24e6) {
        LA_TRY(potrf_right_looking<T>(Wk, L, info, off, batch, n, Inv, st));
        return need_inv ? inverse_merge<T>(cv(L), Inv, Tmp, batch, n, n, st) : LA_OK;
    }
    const int n1 = split_point(n), n2 = n - n1;
    View<T> L21 = L.sub(n1, 0), Wk22 = Wk.sub(n1, n1);
    LA_TRY(potrf_rec<T>(Wk, L, info, off, batch, n1, Inv, Tmp, true, st));
    GemmOpts op;
    op.triB = 2;  // Li11^T is upper triangular
    LA_TRY(launch_gemm<T>(cv(Wk).sub(n1, 0), cv(Inv).t(), L21, batch, n2, n1, n1, T(1), T(0), op, st));
    GemmOpts ou;
    ou.maskC = 1;  // trailing update of the lower triangle: A22 -= L21 L21^T
    LA_TRY(launch_gemm<T>(cv(L21), cv(L21).t(), Wk22, batch, n2, n2, n1, T(-1), T(1), ou, st));
    LA_TRY(potrf_rec<T>(Wk22, L.sub(n1, n1), info, off + n1, batch, n2, Inv.sub(n1, n1), Tmp, need_inv, st));
    if (!need_inv)
        return LA_OK;
    View<T> T1 = Inv.sub(0, n1).t();  // n2 x n1 temporary in the upper-right block
    GemmOpts o1, o2;
    o1.triB = 1;  // Li11 is lower triangular: the K range shrinks with the tile column
    LA_TRY(launch_gemm<T>(cv(L21), cv(Inv), T1, batch, n2, n1, n1, T(1), T(0), o1, st));
    o2.triA = 1;  // Li22 is lower triangular: the K range grows with the tile row
    o2.reverse = 1;
    return launch_gemm<T>(cv(Inv).sub(n1, n1), cv(T1), Inv.sub(n1, 0), batch, n2, n1, n2, T(-1), T(0), o2, st);
}

// ---------------------------------------------------------------------------------
// Pieces of the potrf backward expression (section 4.2; appendix "potrf"):
//   Abar = sym( Lam^-T Phi(Lam^T Lbar) Lam^-1 ),  Phi = lower triangle, halved diagonal.
// ---------------------------------------------------------------------------------

// With the explicit inverse Li of the factor the whole expression is three masked GEMMs whose
// K ranges skip every structural zero (5 n^3 / 3 flops in all, inverse included):
//   P = Phi(tril(Lam^T Lbar))      lower x lower, lower part kept, diagonal halved
//   Z = P Li                       lower x lower = lower
//   Abar = 1/2 (W + W^T), W = Li^T Z (upper x lower = full): the lower tiles of Li^T Z + Z^T Li, mirrored
template <typename T>
static la_status backward_blocked(View<const T> Lam, View<const T> G, View<T> W, int64_t batch, int n, bool aliased,
                                  hipStream_t st);

// Largest block the inverse-based expression is used on.  Its 5 n^3 / 3 flops run in a few large
// products; the blocked sweep needs 2 n^3 / 3 but in many smaller, dependent ones, so it pays once
// the products of a block fill the chip: from about 8 M (fp64; 16 M fp32) matrix elements per
// level over the whole batch (measured: 2048 for one matrix, 1024 for 4 to 8, 256 for 256).
static int bwd_base(int64_t batch, size_t elem)
{
    const double budget = (elem == 4 ? 16.0 : 8.0) * 1048576.0;
    int b = 2048;
    while (b > 256 && (double)b * b * (double)batch > budget)
        b /= 2;
    return b;
}

template <typename T>
static la_status backward_impl(View<const T> Lam, View<const T> G, View<T> W, int64_t batch, int n, bool aliased,
                               hipStream_t st)
{
    if (n > bwd_base(batch, sizeof(T)))
        return backward_blocked<T>(Lam, G, W, batch, n, aliased, st);
    // n <= 16: 16 lanes per matrix, HBM bound.  16 < n <= 32: the register kernel has the higher
    // throughput (11 against 16 ns per fp32 matrix), the one-workgroup kernel the shorter latency
    // (25 against 37 us), so the batch size decides.
    if (n <= 16 || (n <= 32 && batch > 2048))
        return launch_backward_tiny<T>(Lam, G, W, batch, n, st);
    if (n <= backward_leaf16_max_n<T>())  // one workgroup per matrix, everything in LDS, no scratch
        return launch_backward_leaf16<T>(Lam, G, W, batch, n, st);
    ArenaFrame frame;
    View<T> sc[2];
    LA_TRY(scratch_views<T>(batch, n, 2, sc));
    View<T> Li = sc[0], X = sc[1];
    LA_TRY(inverse_build<T>(Lam, Li, X, batch, n, n, st));
    View<const T> Gs = G;
    if (aliased) {  // Abar overwrites Lbar: keep a copy of its lower triangle
        LA_TRY(launch_copy<T>(G, X, batch, n, n, T(1), 1, st));
        Gs = cv(X);
    }
    GemmOpts o;
    o.triA = 2;  // Lam^T
    o.triB = 1;
    o.maskC = 1;
    o.halfDiag = 1;
    LA_TRY(launch_gemm<T>(Lam.t(), Gs, W, batch, n, n, n, T(1), T(0), o, st));
    GemmOpts oz;
    oz.triA = 1;
    oz.triB = 1;
    oz.maskC = 1;
    oz.reverse = 1;  // K range of tile (i, j) grows with i - j: bottom rows first
    LA_TRY(launch_gemm<T>(cv(W), cv(Li), X, batch, n, n, n, T(1), T(0), oz, st));
    // Abar = 1/2 (Li^T Z + Z^T Li) in one launch: the tiles on and below the diagonal accumulate both
    // products (K range from the tile's first row on) and write every entry with its mirror image
    GemmOpts ow;
    ow.triA = 2;
    ow.triB = 1;
    ow.symsum = 1;
    return launch_gemm<T>(cv(Li).t(), cv(X), W, batch, n, n, n, T(0.5), T(0), ow, st);
}

template <typename T>
static la_status tri_apply_v(bool solve, bool fwd, T alpha, int64_t batch, int n, int m, View<const T> Lam,
                             View<const T> Xin, View<T> X, bool inplace, hipStream_t st);

// ---------------------------------------------------------------------------------
// Large n: reverse sweep over the blocked factorisation (section 4.2 names differentiating the
// blocked algorithm itself as the cheaper route).  For the split
//   L11 = chol(A11),  L21 = A21 L11^-T,  S = A22 - L21 L21^T,  L22 = chol(S)
// the adjoints follow in reverse order (W holds Lbar's lower triangle on entry and the symmetric
// Abar on return, block by block, in place):
//   W22 <- backward(L22, W22)                       symmetric, both triangles
//   W21 <- W21 - 2 W22 L21                          adjoint of the update S
//   W21 <- 1/2 W21 L11^-1                           adjoint of the panel solve, halved because A21
//                                                   enters the symmetric A twice
//   W11 <- W11 - 2 tril(W21^T L21)                  the panel solve's effect on L11
//   W11 <- backward(L11, W11)
//   W12 <- W21^T
// 2 n^3 / 3 flops at the blocked levels instead of 5 n^3 / 3 with the full inverse; blocks of at
// most bwd_base(batch) rows take the inverse-based path.
// ---------------------------------------------------------------------------------
template <typename T>
static la_status backward_rec(View<const T> Lam, View<T> W, int64_t batch, int n, hipStream_t st)
{
    if (n <= bwd_base(batch, sizeof(T)))
        return backward_impl<T>(Lam, cv(W), W, batch, n, true, st);
    // Halving (to the multiple of 128 next to n / 2) when that lands on whole base blocks all the way
    // down, i.e. n = 2048 * 2^k; any other n > 4096 peels a first block of 2048 columns instead, which
    // keeps the solve with L11 small and the blocks at the bottom at the full base size
    // (n = 6144: 5.5 -> 4.8 ms, 12288: 27.9 -> 25.5 ms; 8192: no difference).
    const int q = n / 2048;
    const bool halves_fit = n % 2048 == 0 && (q & (q - 1)) == 0;
    const int n1 = (n > 4096 && !halves_fit) ? 2048 : (n / 2 + 127) / 128 * 128, n2 = n - n1;
    View<T> W21 = W.sub(n1, 0), W22 = W.sub(n1, n1);
    View<const T> L21 = Lam.sub(n1, 0);
    LA_TRY(backward_rec<T>(Lam.sub(n1, n1), W22, batch, n2, st));
    GemmOpts plain;
    LA_TRY(launch_gemm<T>(cv(W22), L21, W21, batch, n2, n1, n2, T(-2), T(1), plain, st));
    // rows of W21 are the vectors; x <- x L11^-1 is L11^-T applied to x^T
    LA_TRY(tri_apply_v<T>(true, false, T(0.5), batch, n1, n2, Lam, cv(W21).t(), W21.t(), true, st));
    GemmOpts om;
    om.maskC = 1;
    LA_TRY(launch_gemm<T>(cv(W21).t(), L21, W, batch, n1, n1, n2, T(-2), T(1), om, st));
    LA_TRY(backward_rec<T>(Lam, W, batch, n1, st));
    return launch_copy<T>(cv(W21).t(), W.sub(0, n1), batch, n1, n2, T(1), 0, st);
}

template <typename T>
static la_status backward_blocked(View<const T> Lam, View<const T> G, View<T> W, int64_t batch, int n, bool aliased,
                                  hipStream_t st)
{
    if (!aliased)  // lower triangle of Lbar into the output, which is then updated in place; what lies above the
                   // diagonal is never read and is all written by the sweep (base blocks and mirror copies)
        LA_TRY(launch_copy<T>(G, W, batch, n, n, T(1), 2, st));
    return backward_rec<T>(Lam, W, batch, n, st);
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
    // Many matrices of up to four tile rows: four wavefronts per matrix, tiles in LDS.  Measured against the lane-group
    // kernels at equal data volume, n = 33 ... 64 (us, fp32: 146 -> 111, 113 -> 84 at 38, 146 -> 71 at 41, 57 -> 42 at 48,
    // 90 -> 59 at 56, 56 -> 38 at 64; fp64: 334 -> 180, 161 -> 73 at 48, 123 -> 64 at 64); only fp32 at n = 40, whose rows fill
    // the three-rows-per-lane kernel exactly, is faster there (54 against 75).
    if (n > 32 && n <= NB && batch > 1024 && !(sizeof(T) == 4 && n == 40))
        return launch_potrf_small16<T>(Av, Lv, info, batch, n, st);
    if (n <= NB)
        return launch_potrf_tiny<T>(Av, Lv, info, 0, batch, n, st);
    if (n <= 2 * NB)  // one leaf: it reads A and writes L directly; nobody wants the inverse
        return launch_potrf_leaf16<T>(Av, Lv, View<T>{nullptr, 0, 0, 0}, info, 0, batch, n, true, st);
    ArenaFrame frame;
    // inverses of the diagonal blocks; working copy of the lower triangle of A; temporary of the inverse merges
    // (not needed where the whole matrix is factored panel by panel without merged inverses)
    const bool outer_panels = (batch == 1 && n >= 4096) || n >= 8192;
    const bool merges = outer_panels || !(n <= 2304 && (double)batch * n * n < 24e6);
    View<T> sc[3];
    LA_TRY(scratch_views<T>(batch, n, merges ? 3 : 2, sc));
    if (!merges)
        sc[2] = sc[1];  // never used
    LA_TRY(launch_tril_split<T>(Av, sc[1], Lv, batch, n, st));  // zeros above the diagonal of L
    // Large matrices: right-looking over panels of 2048 columns -- the panel's diagonal block by the
    // recursion below (which factors it 128 columns at a time and merges its inverse), one product
    // for the rows under it, one for the trailing triangle (K = 2048).  Against halving all the way
    // from the top this drops the merges of the large inverses: n = 8192 7.6 -> 7.2 ms, 12288
    // 19.7 -> 17.3, 6144 4.5 -> 4.1 (fp64; other panel widths from 1024 to 4096 are slower).  Below
    // n = 4096, and for several matrices of that size, the halving is faster (3000: 1.36 against 1.39 ms).
    constexpr int outer = 2048;
    if (outer_panels) {
        View<T> Wk = sc[1], Inv = sc[0];
        for (int o = 0; o < n; o += outer) {
            const int w = n - o < outer ? n - o : outer, r = n - o - w;
            LA_TRY(potrf_rec<T>(Wk.sub(o, o), Lv.sub(o, o), info, o, batch, w, Inv.sub(o, o), sc[2], r > 0, st));
            if (r == 0)
                break;
            View<T> L21 = Lv.sub(o + w, o);
            GemmOpts op;
            op.triB = 2;  // Li^T is upper triangular
            LA_TRY(launch_gemm<T>(cv(Wk).sub(o + w, o), cv(Inv).sub(o, o).t(), L21, batch, r, w, w, T(1), T(0), op, st));
            GemmOpts ou;
            ou.maskC = 1;
            LA_TRY(launch_gemm<T>(cv(L21), cv(L21).t(), Wk.sub(o + w, o + w), batch, r, r, w, T(-1), T(1), ou, st));
        }
        return LA_OK;
    }
    return potrf_rec<T>(sc[1], Lv, info, 0, batch, n, sc[0], sc[2], false, st);
}

// trsm / trmm (section 4.2).  vectors: columns of A/B (left) or rows (right); X(e, v) = element e
// of vector v, so that every case is "apply Lam, Lam^T or one of their inverses to vectors".
//   trmm: one GEMM with the triangular operand masked.
//   trsm / trmm, n <= 64 and at most 16 vectors, many items: lane groups (two rows per lane for 16 < n <= 32).
//   trsm, n <= 128 and at most 48 vectors: one block-substitution kernel.
//   trsm, 128 < n <= 512: one launch per call, one workgroup per item and slab of 16 vectors, the
//     factor streamed from memory (launch_trsm_stream), unless many vectors meet few items.
//   trsm, n <= 128 otherwise: product (in place) with the inverse of the single diagonal block.
//   trsm, otherwise: explicit inverses of the diagonal blocks of 256 to 1024 rows (the more vectors,
//     the larger; see inverse_build); n within one block: one masked GEMM with the whole inverse,
//     else block substitution with two GEMMs per block (the block's solution goes through a scratch
//     panel because a product cannot overwrite its own operand across several tiles).
template <typename T>
static la_status tri_apply_v(bool solve, bool fwd, T alpha, int64_t batch, int n, int m, View<const T> Lam,
                             View<const T> Xin, View<T> X, bool inplace, hipStream_t st)
{
    const int64_t nm = (int64_t)n * m, nn = (int64_t)n * n;
    GemmOpts o;
    o.triA = fwd ? 1 : 2;  // Lam keeps e >= k, Lam^T keeps e <= k; the same holds for their inverses
    o.reverse = fwd ? 1 : 0;  // heavy tile rows first: the last ones for a lower operand

    // n <= 64 with at most 16 vectors stored as whole items back to back: G lanes per matrix.  (A solve
    // with 16 < n over a small batch is quicker in the one-workgroup kernel below: 16 matrices of n = 32,
    // fp64: 6.5 against 10.9 us; up to n = 32 the lane-group kernel wins once there are more matrices than
    // workgroup slots, above that the one-workgroup kernel with four wavefronts per item does: 7281
    // solves of 48 x 48 with 16 vectors 136 -> 35 us in fp32, 285 -> 46 in fp64.)
    // A multiply on many small items: one workgroup per item, Lam's lower tiles and the vectors in LDS, no scratch.
    // Up to n = 32 with at most 16 vectors the lane-group kernels below are faster; above that this one is
    // (7281 x 48 x 48 times 16 vectors, fp32 / fp64: 64 lanes per matrix 91 / 183 us).
    const bool leaf_mul = !solve && trmm_leaf_takes<T>(batch, n, m) && Lam.nb2 == 1 && Xin.nb2 == 1 && X.nb2 == 1;
    if (leaf_mul && (n > 32 || m > 16))
        return launch_trmm_leaf<T>(Lam, Xin, X, batch, n, m, alpha, fwd, st);

    if (n <= 64 && m <= 16 && (!solve || n <= 16 || (batch > 1024 && n <= 32)) && X.bs == nm && Xin.bs == nm && Xin.rs == X.rs && Xin.cs == X.cs && X.nb2 == 1 &&
        Xin.nb2 == 1 && Lam.nb2 == 1) {
        const bool rowmajor = (X.rs == m && X.cs == 1), colmajor = (X.rs == 1 && X.cs == n);
        if ((rowmajor || colmajor) && n > 16 && n <= 32)  // 16 lanes per matrix, two rows per lane
            return launch_tri_rows<T>(solve, fwd, alpha, batch, n, m, Lam, Xin.p, X.p, !rowmajor, st);
        if (rowmajor || colmajor)
            return launch_tri_tiny<T>(solve, fwd, alpha, batch, n, m, Lam, Xin.p, X.p, !rowmajor, st);
    }

    if (leaf_mul)  // (operands the lane-group kernels do not take: other strides)
        return launch_trmm_leaf<T>(Lam, Xin, X, batch, n, m, alpha, fwd, st);

    if (solve && n <= 128 && m <= 48)  // small: one workgroup per item does the whole substitution, no scratch
        return launch_trsm_leaf16<T>(Lam, Xin, X, batch, n, m, alpha, fwd, st);

    if (solve && trsm_stream_takes<T>(batch, n, m)) {  // one launch, no scratch
        const la_status s = launch_trsm_stream<T>(Lam, Xin, X, batch, n, m, alpha, fwd, st);
        if (s != LA_ERR_UNSUPPORTED)  // (strides beyond its 32-bit offsets, two-level batches: the blocked path below)
            return s;
    }

    ArenaFrame frame;
    if (solve && n <= NB) {  // inverse of the single block, then one product in place
        if (!inplace || alpha != T(1))
            LA_TRY(launch_copy<T>(Xin, X, batch, n, m, alpha, 0, st));
        View<T> Inv;
        LA_TRY(scratch_views<T>(batch, n, 1, &Inv));
        LA_TRY(launch_tri_inverse128<T>(Lam, Inv, batch, n, st));
        GemmOpts oi;
        oi.triA = fwd ? 1 : 2;
        oi.min_tile64 = 1;  // in place is safe because one 64 x 64 workgroup tile covers all n rows of its vectors
        return launch_gemm<T>(fwd ? cv(Inv) : cv(Inv).t(), cv(X), X, batch, n, m, n, T(1), T(0), oi, st);
    }

    // scratch: [inverse n*n] [merge temporary n*n] (solve only), then a panel shaped like X
    void *sp = nullptr;
    const size_t per_item = (solve ? 2 * (size_t)nn : 0) + (size_t)nm;
    LA_TRY(arena_take(per_item * batch * sizeof(T), &sp));
    T *base = (T *)sp;
    View<T> Inv{base, nn, n, 1}, Tmp{base + (solve ? batch * nn : 0), nn, n, 1};
    // a compact panel whose fast index is the one X has
    View<T> S = X.rs <= X.cs ? View<T>{base + (solve ? 2 * batch * nn : 0), nm, 1, n}
                             : View<T>{base + (solve ? 2 * batch * nn : 0), nm, m, 1};

    // Edge of the diagonal blocks that get an explicit inverse; block substitution above it.  A merge
    // level of the inverse costs n b^2 multiply-adds per matrix whatever the number of vectors, a
    // substitution step three short launches: with few vectors the merges stop paying early.
    // Measured (fp64, us; edge 256 / 512 / 1024): 32 x 512, 64 vectors 93 / 118 / 118; 8 x 1024, 64:
    // 112 / 118 / 166; 4 x 2048, 128: 223 / 196 / 234; 1 x 4096, 512: 548 / 431 / 396.
    int NBI = 256;
    while (NBI < 1024 && NBI < 4 * m)
        NBI *= 2;
    if (!solve || n <= NBI) {
        View<const T> M = Lam;
        if (solve) {
            LA_TRY(inverse_build<T>(Lam, Inv, Tmp, batch, n, n, st));
            M = cv(Inv);
        }
        View<const T> src = Xin;
        if (inplace) {
            LA_TRY(launch_copy<T>(Xin, S, batch, n, m, T(1), 0, st));
            src = cv(S);
        }
        return launch_gemm<T>(fwd ? M : M.t(), src, X, batch, n, m, n, alpha, T(0), o, st);
    }

    LA_TRY(inverse_build<T>(Lam, Inv, Tmp, batch, n, NBI, st));
    if (!inplace || alpha != T(1))
        LA_TRY(launch_copy<T>(Xin, X, batch, n, m, alpha, 0, st));
    const int nblk = (n + NBI - 1) / NBI;
    GemmOpts plain;
    for (int step = 0; step < nblk; ++step) {
        const int j = fwd ? step : nblk - 1 - step;
        const int64_t o0 = (int64_t)j * NBI;
        const int nbj = (int)((n - o0) < NBI ? (n - o0) : NBI);
        View<const T> Ij = cv(Inv).sub(o0, o0);
        View<T> Xj = X.sub(o0, 0);
        LA_TRY(launch_gemm<T>(fwd ? Ij : Ij.t(), cv(Xj), S, batch, nbj, m, nbj, T(1), T(0), o, st));
        if (fwd && o0 + nbj < n) {  // rows below: X -= Lam[below, j] S
            const int rest = (int)(n - o0 - nbj);
            LA_TRY(launch_gemm<T>(Lam.sub(o0 + nbj, o0), cv(S), X.sub(o0 + nbj, 0), batch, rest, m, nbj, T(-1), T(1),
                                  plain, st));
        } else if (!fwd && o0 > 0) {  // rows above: X -= Lam[j, above]^T S
            LA_TRY(launch_gemm<T>(Lam.sub(o0, 0).t(), cv(S), X, batch, (int)o0, m, nbj, T(-1), T(1), plain, st));
        }
        LA_TRY(launch_copy<T>(cv(S), Xj, batch, nbj, m, T(1), 0, st));
    }
    return LA_OK;
}

template <typename T>
static la_status tri_apply_t(bool solve, int lower, int trans, int rightside, double alpha, int64_t batch, int n, int m,
                             const void *L, const void *A, void *B, hipStream_t st)
{
    View<const T> Lam = tri_view<const T>((const T *)L, n, lower);
    const int64_t nm = (int64_t)n * m;
    View<const T> Xin = rightside ? View<const T>{(const T *)A, nm, 1, n} : View<const T>{(const T *)A, nm, m, 1};
    View<T> X = rightside ? View<T>{(T *)B, nm, 1, n} : View<T>{(T *)B, nm, m, 1};
    const bool use_lt = (trans != 0) != (lower == 0);  // t(L) equals Lam^T
    const bool fwd = (use_lt == (rightside != 0));
    return tri_apply_v<T>(solve, fwd, (T)alpha, batch, n, m, Lam, Xin, X, A == B, st);
}

template <typename T>
static la_status syrk_t(int trans, double alpha, int64_t batch, int n, int k, const void *A, void *B, hipStream_t st)
{
    const int64_t nk = (int64_t)n * k, nn = (int64_t)n * n;
    View<const T> Ank = trans ? View<const T>{(const T *)A, nk, 1, n} : View<const T>{(const T *)A, nk, k, 1};  // n x k
    View<T> C{(T *)B, nn, n, 1};
    if (n <= 16 && k >= 1 && k <= 32)  // G lanes per matrix, HBM bound
        return launch_syrk_tiny<T>(trans != 0, (T)alpha, batch, n, k, (const T *)A, C, st);
    if (outer_rows_takes<T>(n, k, false))  // 16 < n <= 32: 16 lanes per matrix, two rows per lane
        return launch_outer_rows<T>(trans != 0, 0, (T)alpha, batch, n, k, (const T *)A, (const T *)A, C, st);
    if (outer_leaf_takes<T>(batch, n, k, false))  // one workgroup per matrix, operands in LDS
        return launch_outer_leaf<T>(0, (T)alpha, batch, n, k, Ank, Ank, C, st);
    GemmOpts o;
    o.maskC = 1;
    LA_TRY(launch_gemm<T>(Ank, Ank.t(), C, batch, n, n, k, (T)alpha, T(0), o, st));
    return launch_mirror_lower<T>(C, batch, n, st);
}

template <typename T>
static la_status gemm2_t(int ta, int tb, double alpha, int64_t batch, int m, int n, int k, const void *A, const void *B,
                         void *C, hipStream_t st)
{
    const int64_t sa = (int64_t)m * k, sb = (int64_t)k * n, sc = (int64_t)m * n;
    View<const T> Av = ta ? View<const T>{(const T *)A, sa, 1, m} : View<const T>{(const T *)A, sa, k, 1};  // m x k
    View<const T> Bv = tb ? View<const T>{(const T *)B, sb, 1, k} : View<const T>{(const T *)B, sb, n, 1};  // k x n
    View<T> Cv{(T *)C, sc, n, 1};
    if (m <= 16 && n <= 16 && k >= 1 && k <= 16)  // lane groups of 4, 8 or 16 per item, HBM bound
        return launch_gemm2_tiny<T>(ta, tb, (T)alpha, batch, m, n, k, (const T *)A, (const T *)B, (T *)C, st);
    if (gemm2_rows_takes<T>(m, n, k))  // up to 32 each: 16 lanes per item, two rows per lane
        return launch_gemm2_rows<T>(ta, tb, (T)alpha, batch, m, n, k, (const T *)A, (const T *)B, (T *)C, st);
    GemmOpts o;
    return launch_gemm<T>(Av, Bv, Cv, batch, m, n, k, (T)alpha, T(0), o, st);
}

}  // namespace la

using namespace la;

// ---------------------------------------------------------------------------------
// Backward rules of trmm and trsm (section 4.2; appendix "trmm", "trsm", both for a lower and an
// upper factor).  The gradient of the triangular operand is the factor's triangle of an outer
// product of two matrices P, Q of the shape of A: with (X1, X2) = (P, Q), or (Q, P) when the
// operator transposes L,
//   left:  G = X1 X2^T,     right:  G = X2^T X1.
// ---------------------------------------------------------------------------------
template <typename T>
static la_status tri_outer_t(int lower, int trans, int rightside, T scale, int64_t batch, int n, int m, const T *P,
                             const T *Q, T *out, hipStream_t st)
{
    const int64_t nn = (int64_t)n * n, nm = (int64_t)n * m;
    View<T> G{out, nn, n, 1};
    if ((n <= 16 && m >= 1 && m <= 32) || outer_rows_takes<T>(n, m, true)) {  // lane groups: product, mask and zeros in one launch
        const T *U = rightside ? (trans ? P : Q) : (trans ? Q : P), *V = rightside ? (trans ? Q : P) : (trans ? P : Q);
        if (n <= 16)
            return launch_outer_tiny<T>(rightside != 0, lower ? 1 : 2, scale, batch, n, m, U, V, G, st);
        return launch_outer_rows<T>(rightside != 0, lower ? 1 : 2, scale, batch, n, m, U, V, G, st);
    }
    if (outer_leaf_takes<T>(batch, n, m, true)) {  // one workgroup per matrix: product, mask and zeros in one launch
        const T *X1 = trans ? Q : P, *X2 = trans ? P : Q;
        if (!rightside)
            return launch_outer_leaf<T>(lower ? 1 : 2, scale, batch, n, m, View<const T>{X1, nm, m, 1},
                                        View<const T>{X2, nm, m, 1}, G, st);
        return launch_outer_leaf<T>(lower ? 1 : 2, scale, batch, n, m, View<const T>{X2, nm, 1, n},
                                    View<const T>{X1, nm, 1, n}, G, st);
    }
    LA_TRY(launch_zero_strict_upper<T>(lower ? G : G.t(), batch, n, st));  // the other triangle of the result
    GemmOpts o;
    o.maskC = lower ? 1 : 2;
    if (m == 0)  // empty product: the kept triangle is zero too (written without reading what the buffer held)
        return launch_fill_i32((int32_t *)out, batch * nn * (int64_t)(sizeof(T) / 4), 0, st);
    const T *X1 = trans ? Q : P, *X2 = trans ? P : Q;
    if (!rightside)
        return launch_gemm<T>(View<const T>{X1, nm, m, 1}, View<const T>{X2, nm, 1, m}, G, batch, n, n, m, scale, T(0), o,
                              st);
    return launch_gemm<T>(View<const T>{X2, nm, 1, n}, View<const T>{X1, nm, n, 1}, G, batch, n, n, m, scale, T(0), o,
                          st);
}

template <typename T>
static la_status trmm_backward_t(int lower, int trans, int rightside, double alpha, int64_t batch, int n, int m,
                                 const void *L, const void *A, const void *Bbar, void *Abar, void *Lbar, hipStream_t st)
{
    // Lbar = alpha tri(outer(Bbar, A)) first, then Abar = alpha t(L)^T Bbar (which may overwrite Bbar)
    LA_TRY(tri_outer_t<T>(lower, trans, rightside, (T)alpha, batch, n, m, (const T *)Bbar, (const T *)A, (T *)Lbar, st));
    if (m == 0)
        return LA_OK;
    return tri_apply_t<T>(false, lower, !trans, rightside, alpha, batch, n, m, L, Bbar, Abar, st);
}

template <typename T>
static la_status trsm_backward_t(int lower, int trans, int rightside, double alpha, int64_t batch, int n, int m,
                                 const void *L, const void *B, const void *Bbar, void *Abar, void *Lbar, hipStream_t st)
{
    // Y = t(L)^-T Bbar into Abar (which may overwrite Bbar), Lbar = -tri(outer(Y, B)) (which may
    // overwrite L: L is not needed any more), Abar = alpha Y
    if (m > 0)
        LA_TRY(tri_apply_t<T>(true, lower, !trans, rightside, 1.0, batch, n, m, L, Bbar, Abar, st));
    LA_TRY(tri_outer_t<T>(lower, trans, rightside, T(-1), batch, n, m, (const T *)Abar, (const T *)B, (T *)Lbar, st));
    if (m > 0 && alpha != 1.0) {
        View<T> Y{(T *)Abar, (int64_t)n * m, rightside ? n : m, 1};
        LA_TRY(launch_copy<T>(cv(Y), Y, batch, rightside ? m : n, rightside ? n : m, (T)alpha, 0, st));
    }
    return LA_OK;
}

// syrk backward (section 4.2 "syrk"): Abar = alpha (Bbar + Bbar^T) A  resp.  alpha A (Bbar + Bbar^T),
// two products accumulated in Abar.
template <typename T>
static la_status syrk_backward_t(int trans, double alpha, int64_t batch, int n, int k, const void *A, const void *Bbar,
                                 void *Abar, hipStream_t st)
{
    const int64_t nk = (int64_t)n * k, nn = (int64_t)n * n;
    View<const T> G{(const T *)Bbar, nn, n, 1};
    if (n <= 16 && k >= 1 && k <= 32)  // lane groups of 4, 8 or 16 per matrix, one launch
        return launch_symm_tiny<T>(trans != 0, (T)alpha, batch, n, k, G, (const T *)A, (T *)Abar, st);
    if (symm_rows_takes<T>(n, k))  // 16 < n <= 32: 16 lanes per matrix, two rows per lane
        return launch_symm_rows<T>(trans != 0, (T)alpha, batch, n, k, G, (const T *)A, (T *)Abar, st);
    if (symm_leaf_takes<T>(batch, n, k)) {  // one workgroup per matrix, operands in LDS; A and Abar as n x k views
        if (!trans)
            return launch_symm_leaf<T>((T)alpha, batch, n, k, G, View<const T>{(const T *)A, nk, k, 1},
                                       View<T>{(T *)Abar, nk, k, 1}, st);
        return launch_symm_leaf<T>((T)alpha, batch, n, k, G, View<const T>{(const T *)A, nk, 1, n},
                                   View<T>{(T *)Abar, nk, 1, n}, st);
    }
    GemmOpts o;
    if (!trans) {
        View<const T> Av{(const T *)A, nk, k, 1};
        View<T> Ov{(T *)Abar, nk, k, 1};
        LA_TRY(launch_gemm<T>(G, Av, Ov, batch, n, k, n, (T)alpha, T(0), o, st));
        return launch_gemm<T>(G.t(), Av, Ov, batch, n, k, n, (T)alpha, T(1), o, st);
    }
    View<const T> Av{(const T *)A, nk, n, 1};
    View<T> Ov{(T *)Abar, nk, n, 1};
    LA_TRY(launch_gemm<T>(Av, G, Ov, batch, k, n, n, (T)alpha, T(0), o, st));
    return launch_gemm<T>(Av, G.t(), Ov, batch, k, n, n, (T)alpha, T(1), o, st);
}

// potri (section 4.2 "potri"): A^-1 = Lam^-T Lam^-1 for A = Lam Lam^T (Lam = L, or R^T for an upper
// factor: the same symmetric matrix either way).  Explicit inverse of the factor, then the lower
// tiles of Li^T Li (K range from max(i, j) on), mirrored.
template <typename T>
static la_status potri_t(int lower, int64_t batch, int n, const void *L, void *B, hipStream_t st)
{
    View<const T> Lam = tri_view<const T>((const T *)L, n, lower);
    if (n <= 32)  // both solves on the identity in registers, G lanes per matrix (two rows per lane above 16)
        return launch_potri_tiny<T>(Lam, View<T>{(T *)B, (int64_t)n * n, n, 1}, batch, n, st);
    if (n <= 2 * NB)  // one workgroup per matrix, everything in LDS, no scratch
        return launch_potri_leaf16<T>(Lam, View<T>{(T *)B, (int64_t)n * n, n, 1}, batch, n, st);
    ArenaFrame frame;
    View<T> sc[2];
    LA_TRY(scratch_views<T>(batch, n, 2, sc));
    LA_TRY(inverse_build<T>(Lam, sc[0], sc[1], batch, n, n, st));
    View<T> Bv{(T *)B, (int64_t)n * n, n, 1};
    GemmOpts o;
    o.triA = 2;
    o.triB = 1;
    o.maskC = 1;
    LA_TRY(launch_gemm<T>(cv(sc[0]).t(), cv(sc[0]), Bv, batch, n, n, n, T(1), T(0), o, st));
    return launch_mirror_lower<T>(Bv, batch, n, st);
}

// potri backward (section 4.2 "potri"; appendix "potri"):
//   Lbar = -2 tril(B sym(Bbar) L^-T) = -tril((B Bbar + B Bbar^T) L^-T)      (lower factor)
//   Rbar = -2 triu(R^-T sym(Bbar) B) = -triu(R^-T (Bbar B + Bbar^T B))      (upper factor)
// The two products accumulate in Lbar, the solve runs in place there, the other triangle is cleared.
template <typename T>
static la_status potri_backward_t(int lower, int64_t batch, int n, const void *L, const void *B, const void *Bbar,
                                  void *Lbar, hipStream_t st)
{
    const int64_t nn = (int64_t)n * n;
    View<const T> Bv{(const T *)B, nn, n, 1}, G{(const T *)Bbar, nn, n, 1};
    View<T> X{(T *)Lbar, nn, n, 1};
    GemmOpts o;
    if (lower) {
        LA_TRY(launch_gemm<T>(Bv, G, X, batch, n, n, n, T(1), T(0), o, st));
        LA_TRY(launch_gemm<T>(Bv, G.t(), X, batch, n, n, n, T(1), T(1), o, st));
        LA_TRY(tri_apply_t<T>(true, 1, 1, 1, -1.0, batch, n, n, L, Lbar, Lbar, st));
        return launch_zero_strict_upper<T>(X, batch, n, st);
    }
    LA_TRY(launch_gemm<T>(G, Bv, X, batch, n, n, n, T(1), T(0), o, st));
    LA_TRY(launch_gemm<T>(G.t(), Bv, X, batch, n, n, n, T(1), T(1), o, st));
    LA_TRY(tri_apply_t<T>(true, 0, 1, 0, -1.0, batch, n, n, L, Lbar, Lbar, st));
    return launch_zero_strict_upper<T>(X.t(), batch, n, st);
}

// gemm2 backward (section 4.2 "gemm2"): each gradient is a gemm2 of Cbar with the other operand.
template <typename T>
static la_status gemm2_backward_t(int ta, int tb, double alpha, int64_t batch, int m, int n, int k, const void *A,
                                  const void *B, const void *Cbar, void *Abar, void *Bbar, hipStream_t st)
{
    if (!ta)  // Abar (m x k) = alpha Cbar t_b(B)^T
        LA_TRY(gemm2_t<T>(0, !tb, alpha, batch, m, k, n, Cbar, B, Abar, st));
    else  // Abar (k x m) = alpha t_b(B) Cbar^T
        LA_TRY(gemm2_t<T>(tb, 1, alpha, batch, k, m, n, B, Cbar, Abar, st));
    if (!tb)  // Bbar (k x n) = alpha t_a(A)^T Cbar
        return gemm2_t<T>(!ta, 0, alpha, batch, k, n, m, A, Cbar, Bbar, st);
    return gemm2_t<T>(1, ta, alpha, batch, n, k, m, Cbar, A, Bbar, st);  // Bbar (n x k) = alpha Cbar^T t_a(A)
}

// ---------------------------------------------------------------------------------
// Variational sparse Gaussian-process criterion (section 3.2) and its gradient through two Cholesky
// factors of U x U matrices -- the evaluation that makes the criterion cost O(n U^2) -- as a chain of
// the operators above; the gradient is the reverse sweep over that chain with the operators' backward
// rules (section 4.2), the two places where gradients meet written out.  One problem per call.  The
// caller's workspace holds
//   Lu (U^2), B (U n), A (U^2), La (U^2), La_bar -> A_bar (U^2), v, w, v_bar (U each), one scalar,
// then 7 x SGP_PARTIALS fp64 partial sums.
// ---------------------------------------------------------------------------------
template <typename T>
static size_t sgp_workspace_elems(int U, int n)
{
    return 4 * (size_t)U * U + (size_t)U * n + 3 * (size_t)U + 16;
}

template <typename T>
static la_status sgp_t(int U, int n, const void *Kuu_, const void *Kuf_, const void *Kff_, const void *y_, double lam,
                       void *phi_, void *Kuu_bar_, void *Kuf_bar_, void *Kff_bar_, void *y_bar_, void *lam_bar_,
                       void *ws, hipStream_t st)
{
    const int64_t uu = (int64_t)U * U, un = (int64_t)U * n;
    T *Lu = (T *)ws, *B = Lu + uu, *A = B + un, *La = A + uu, *Ab = La + uu, *v = Ab + uu, *w = v + U, *vb = w + U,
      *dummy = vb + U;
    double *sums = reinterpret_cast<double *>(((uintptr_t)(dummy + 16) + 7) & ~(uintptr_t)7);
    const T *Kuf = (const T *)Kuf_, *y = (const T *)y_, *Kff = (const T *)Kff_;
    T *Kuf_bar = (T *)Kuf_bar_, *Kuu_bar = (T *)Kuu_bar_, *y_bar = (T *)y_bar_;
    auto S = [&](int q) { return sums + q * SGP_PARTIALS; };

    // ---- forward ----------------------------------------------------------------------------
    LA_TRY(potrf_t<T>(1, 1, U, Kuu_, Lu, nullptr, st));                                        // Lu
    LA_TRY(tri_apply_t<T>(true, 1, 0, 0, 1.0, 1, U, n, Lu, Kuf, B, st));                       // B = Lu^-1 Kuf
    LA_TRY(syrk_t<T>(0, 1.0 / lam, 1, U, n, B, A, st));                                        // A = B B^T / lam ...
    LA_TRY(launch_add_diag<T>(A, U, T(1), st));                                                //     ... + I
    LA_TRY(potrf_t<T>(1, 1, U, A, La, nullptr, st));                                           // La
    LA_TRY(gemm2_t<T>(0, 0, 1.0, 1, U, 1, n, B, y, v, st));                                    // v = B y
    LA_TRY(tri_apply_t<T>(true, 1, 0, 0, 1.0, 1, U, 1, La, v, w, st));                         // w = La^-1 v
    LA_TRY(launch_partial_sums<T>(0, y, nullptr, n, 0, S(0), st));
    LA_TRY(launch_partial_sums<T>(0, w, nullptr, U, 0, S(1), st));
    LA_TRY(launch_partial_sums<T>(0, B, nullptr, un, 0, S(2), st));
    LA_TRY(launch_partial_sums<T>(1, Kff, nullptr, n, 0, S(3), st));
    LA_TRY(launch_partial_sums<T>(4, La, nullptr, U, U, S(4), st));
    LA_TRY(launch_partial_sums<T>(1, Kff, nullptr, 0, 0, S(5), st));  // zero until the backward sweep fills them
    LA_TRY(launch_partial_sums<T>(1, Kff, nullptr, 0, 0, S(6), st));
    LA_TRY(launch_sgp_scalars<T>(0, sums, lam, n, (T *)phi_, (T *)nullptr, (T *)nullptr, 0, st));

    // ---- backward ---------------------------------------------------------------------------
    // w = La^-1 v with w_bar = -w / lam^2:  v_bar = La^-T w_bar;  La_bar = -tril(v_bar w^T) + diag(1 / La_ii)
    LA_TRY(tri_apply_t<T>(true, 1, 1, 0, -1.0 / (lam * lam), 1, U, 1, La, w, vb, st));
    LA_TRY(launch_gp_glue<T>(La, w, w, vb, dummy, Ab, 1, U, st));
    LA_TRY(backward_impl<T>(View<const T>{La, uu, U, 1}, View<const T>{Ab, uu, U, 1}, View<T>{Ab, uu, U, 1}, 1, U, true,
                            st));                                                              // A_bar (symmetric)
    LA_TRY(launch_partial_sums<T>(2, Ab, A, uu, 0, S(5), st));
    LA_TRY(launch_partial_sums<T>(3, Ab, nullptr, U, U, S(6), st));
    LA_TRY(launch_sgp_scalars<T>(1, sums, lam, n, (T *)nullptr, (T *)lam_bar_, (T *)Kff_bar_, n, st));
    // B_bar = (2 / lam) A_bar B - B / lam + v_bar y^T   (into Kuf_bar's buffer)
    View<T> Gb{Kuf_bar, un, n, 1};
    LA_TRY(launch_copy<T>(View<const T>{B, un, n, 1}, Gb, 1, U, n, (T)(-1.0 / lam), 0, st));
    GemmOpts o;
    LA_TRY(launch_gemm<T>(View<const T>{Ab, uu, U, 1}, View<const T>{B, un, n, 1}, Gb, 1, U, n, U, (T)(2.0 / lam), T(1), o,
                          st));
    LA_TRY(launch_rank1_add<T>(Kuf_bar, vb, y, U, n, st));
    // y_bar = B^T v_bar + y / lam
    View<T> yb{y_bar, n, 1, 1};
    LA_TRY(launch_copy<T>(View<const T>{y, n, 1, 1}, yb, 1, n, 1, (T)(1.0 / lam), 0, st));
    LA_TRY(launch_gemm<T>(View<const T>{B, un, 1, n}, View<const T>{vb, U, 1, 1}, yb, 1, n, 1, U, T(1), T(1), o, st));
    // B = Lu^-1 Kuf:  Kuf_bar = Lu^-T B_bar (in place),  Lu_bar = -tril(Kuf_bar B^T);  then Kuu_bar
    LA_TRY(tri_apply_t<T>(true, 1, 1, 0, 1.0, 1, U, n, Lu, Kuf_bar, Kuf_bar, st));
    LA_TRY(tri_outer_t<T>(1, 0, 0, T(-1), 1, U, n, Kuf_bar, B, Kuu_bar, st));
    return backward_impl<T>(View<const T>{Lu, uu, U, 1}, View<const T>{Kuu_bar, uu, U, 1}, View<T>{Kuu_bar, uu, U, 1}, 1, U,
                            true, st);
}

template <typename T>
static la_status gp_t(int64_t batch, int n, const void *A, const void *y, void *loss, void *Abar, int32_t *info,
                      void *workspace, hipStream_t st)
{
    if (n <= backward_leaf16_max_n<T>()) {
        if (info)
            LA_TRY(launch_fill_i32(info, batch, 0, st));
        return launch_gp_leaf16<T>(tri_view<const T>((const T *)A, n, 1), (const T *)y, (T *)loss,
                                   tri_view<T>((T *)Abar, n, 1), info, batch, n, st);
    }
    const int64_t nn = (int64_t)n * n;
    T *Lw = (T *)workspace, *Gw = Lw + batch * nn, *z = Gw + batch * nn, *al = z + batch * n;
    LA_TRY(potrf_t<T>(1, batch, n, A, Lw, info, st));
    LA_TRY(tri_apply_t<T>(true, 1, 0, 0, 1.0, batch, n, 1, Lw, y, z, st));
    LA_TRY(tri_apply_t<T>(true, 1, 1, 0, 1.0, batch, n, 1, Lw, z, al, st));
    LA_TRY(launch_gp_glue<T>(Lw, (const T *)y, z, al, (T *)loss, Gw, batch, n, st));
    return backward_impl<T>(tri_view<const T>(Lw, n, 1), tri_view<const T>(Gw, n, 1), tri_view<T>((T *)Abar, n, 1), batch,
                            n, false, st);
}

// ---------------------------------------------------------------------------------
// Workspace handling of the entry points.  An operator body `op` (host code that enqueues the
// kernels) runs twice: a sizing pass that launches nothing and records how much scratch the body
// takes, then, if the caller's workspace holds that much, for real on that workspace.
// ---------------------------------------------------------------------------------
template <class F>
static la_status sizing_pass(F &&op, size_t *peak)
{
    Arena a;
    a.dry = true;
    a.base = reinterpret_cast<char *>((uintptr_t)1 << 46);  // never dereferenced
    Arena *prev = current_arena();
    current_arena() = &a;
    const la_status s = op();
    current_arena() = prev;
    *peak = a.peak;
    return s;
}

template <class F>
static la_status with_workspace(void *ws, size_t ws_bytes, F &&op)
{
    size_t need = 0;
    LA_TRY(sizing_pass(op, &need));
    if (need > 0) {
        if (!ws || need > ws_bytes) {
            snprintf(g_err, sizeof(g_err), "this call needs a workspace of %zu bytes (la_workspace_bytes), %zu given", need,
                     ws ? ws_bytes : (size_t)0);
            return LA_ERR_WORKSPACE;
        }
        if ((uintptr_t)ws & 255) {
            snprintf(g_err, sizeof(g_err), "the workspace must be 256-byte aligned");
            return LA_ERR_INVALID_ARG;
        }
    }
    Arena a;
    a.base = (char *)ws;
    a.cap = need > 0 ? ws_bytes : 0;
    Arena *prev = current_arena();
    current_arena() = &a;
    const la_status s = op();
    current_arena() = prev;
    return s;
}

// does the part of the workspace a call may use overlap an operand?
static inline bool ws_hits(const void *ws, size_t ws_bytes, const void *p, size_t bytes)
{
    return ws && ws_bytes && p && bytes && overlap(ws, ws_bytes, p, bytes);
}

// ---- operator bodies: validated arguments in, kernels enqueued, scratch from the current arena ----
static la_status potrf_body(la_dtype dt, int lower, int64_t batch, int n, const void *A, void *L, int32_t *info,
                            hipStream_t st)
{
    return dt == LA_F32 ? potrf_t<float>(lower, batch, n, A, L, info, st)
                        : potrf_t<double>(lower, batch, n, A, L, info, st);
}

static la_status backward_body(la_dtype dt, int lower, int64_t batch, int n, const void *L, const void *Lbar, void *Abar,
                               hipStream_t st)
{
    if (dt == LA_F32)
        return backward_impl<float>(tri_view<const float>((const float *)L, n, lower),
                                    tri_view<const float>((const float *)Lbar, n, lower),
                                    tri_view<float>((float *)Abar, n, lower), batch, n, Lbar == Abar, st);
    return backward_impl<double>(tri_view<const double>((const double *)L, n, lower),
                                 tri_view<const double>((const double *)Lbar, n, lower),
                                 tri_view<double>((double *)Abar, n, lower), batch, n, Lbar == Abar, st);
}

static la_status tri_body(bool solve, la_dtype dt, int lower, int trans, int rightside, double alpha, int64_t batch, int n,
                          int m, const void *L, const void *A, void *B, hipStream_t st)
{
    return dt == LA_F32 ? tri_apply_t<float>(solve, lower, trans, rightside, alpha, batch, n, m, L, A, B, st)
                        : tri_apply_t<double>(solve, lower, trans, rightside, alpha, batch, n, m, L, A, B, st);
}

static la_status tri_backward_body(bool solve, la_dtype dt, int lower, int trans, int rightside, double alpha,
                                   int64_t batch, int n, int m, const void *L, const void *X, const void *Bbar, void *Abar,
                                   void *Lbar, hipStream_t st)
{
    if (solve)
        return dt == LA_F32 ? trsm_backward_t<float>(lower, trans, rightside, alpha, batch, n, m, L, X, Bbar, Abar, Lbar, st)
                            : trsm_backward_t<double>(lower, trans, rightside, alpha, batch, n, m, L, X, Bbar, Abar, Lbar, st);
    return dt == LA_F32 ? trmm_backward_t<float>(lower, trans, rightside, alpha, batch, n, m, L, X, Bbar, Abar, Lbar, st)
                        : trmm_backward_t<double>(lower, trans, rightside, alpha, batch, n, m, L, X, Bbar, Abar, Lbar, st);
}

static la_status syrk_body(la_dtype dt, int trans, double alpha, int64_t batch, int n, int k, const void *A, void *B,
                           hipStream_t st)
{
    return dt == LA_F32 ? syrk_t<float>(trans, alpha, batch, n, k, A, B, st)
                        : syrk_t<double>(trans, alpha, batch, n, k, A, B, st);
}

static la_status syrk_backward_body(la_dtype dt, int trans, double alpha, int64_t batch, int n, int k, const void *A,
                                    const void *Bbar, void *Abar, hipStream_t st)
{
    return dt == LA_F32 ? syrk_backward_t<float>(trans, alpha, batch, n, k, A, Bbar, Abar, st)
                        : syrk_backward_t<double>(trans, alpha, batch, n, k, A, Bbar, Abar, st);
}

static la_status gemm2_body(la_dtype dt, int ta, int tb, double alpha, int64_t batch, int m, int n, int k, const void *A,
                            const void *B, void *C, hipStream_t st)
{
    return dt == LA_F32 ? gemm2_t<float>(ta, tb, alpha, batch, m, n, k, A, B, C, st)
                        : gemm2_t<double>(ta, tb, alpha, batch, m, n, k, A, B, C, st);
}

static la_status gemm2_backward_body(la_dtype dt, int ta, int tb, double alpha, int64_t batch, int m, int n, int k,
                                     const void *A, const void *B, const void *Cbar, void *Abar, void *Bbar, hipStream_t st)
{
    return dt == LA_F32 ? gemm2_backward_t<float>(ta, tb, alpha, batch, m, n, k, A, B, Cbar, Abar, Bbar, st)
                        : gemm2_backward_t<double>(ta, tb, alpha, batch, m, n, k, A, B, Cbar, Abar, Bbar, st);
}

static la_status potri_body(la_dtype dt, int lower, int64_t batch, int n, const void *L, void *B, hipStream_t st)
{
    return dt == LA_F32 ? potri_t<float>(lower, batch, n, L, B, st) : potri_t<double>(lower, batch, n, L, B, st);
}

static la_status potri_backward_body(la_dtype dt, int lower, int64_t batch, int n, const void *L, const void *B,
                                     const void *Bbar, void *Lbar, hipStream_t st)
{
    return dt == LA_F32 ? potri_backward_t<float>(lower, batch, n, L, B, Bbar, Lbar, st)
                        : potri_backward_t<double>(lower, batch, n, L, B, Bbar, Lbar, st);
}

// ---- argument checks + workspace + body, shared by the plain and the _ws entry points ------------
static la_status potrf_call(la_dtype dt, int lower, int64_t batch, int n, const void *A, void *L, int32_t *info, void *ws,
                            size_t ws_bytes, void *stream)
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
    if (ws_hits(ws, ws_bytes, A, bytes) || ws_hits(ws, ws_bytes, L, bytes) || ws_hits(ws, ws_bytes, info, (size_t)batch * 4))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    return with_workspace(ws, ws_bytes, [&] { return potrf_body(dt, lower, batch, n, A, L, info, st); });
}

static la_status backward_call(la_dtype dt, int lower, int64_t batch, int n, const void *L, const void *Lbar, void *Abar,
                               void *ws, size_t ws_bytes, void *stream)
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
    if (ws_hits(ws, ws_bytes, L, bytes) || ws_hits(ws, ws_bytes, Lbar, bytes) || ws_hits(ws, ws_bytes, Abar, bytes))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    return with_workspace(ws, ws_bytes, [&] { return backward_body(dt, lower, batch, n, L, Lbar, Abar, st); });
}

static la_status tri_call(bool solve, la_dtype dt, int lower, int trans, int rightside, double alpha, int64_t batch, int n,
                          int m, const void *L, const void *A, void *B, void *ws, size_t ws_bytes, void *stream)
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
    if (ws_hits(ws, ws_bytes, L, lb) || ws_hits(ws, ws_bytes, A, ab) || ws_hits(ws, ws_bytes, B, ab))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    return with_workspace(ws, ws_bytes,
                          [&] { return tri_body(solve, dt, lower, trans, rightside, alpha, batch, n, m, L, A, B, st); });
}

static la_status tri_backward_call(bool solve, la_dtype dt, int lower, int trans, int rightside, double alpha,
                                   int64_t batch, int n, int m, const void *L, const void *X, const void *Bbar, void *Abar,
                                   void *Lbar, void *ws, size_t ws_bytes, void *stream)
{
    if (bad_dtype(dt) || batch < 0 || n < 0 || m < 0 || n > MAX_N || m > MAX_N)
        return LA_ERR_INVALID_ARG;
    if (batch == 0 || n == 0)
        return LA_OK;
    if (!L || !Lbar || (m > 0 && (!X || !Bbar || !Abar)))
        return LA_ERR_INVALID_ARG;
    const size_t lb = (size_t)batch * n * n * esize(dt), ab = (size_t)batch * n * m * esize(dt);
    // Abar may be Bbar itself; Lbar may be L itself for trsm (L is consumed first).  Everything else
    // must be disjoint.
    if (m > 0) {
        if (overlap(Abar, ab, L, lb) || overlap(Abar, ab, X, ab) || (Abar != Bbar && overlap(Abar, ab, Bbar, ab)) ||
            overlap(Lbar, lb, X, ab) || overlap(Lbar, lb, Bbar, ab) || overlap(Lbar, lb, Abar, ab))
            return LA_ERR_INVALID_ARG;
    }
    if (overlap(Lbar, lb, L, lb) && !(solve && Lbar == L))
        return LA_ERR_INVALID_ARG;
    if (ws_hits(ws, ws_bytes, L, lb) || ws_hits(ws, ws_bytes, Lbar, lb) || ws_hits(ws, ws_bytes, X, ab) ||
        ws_hits(ws, ws_bytes, Bbar, ab) || ws_hits(ws, ws_bytes, Abar, ab))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    return with_workspace(ws, ws_bytes, [&] {
        return tri_backward_body(solve, dt, lower, trans, rightside, alpha, batch, n, m, L, X, Bbar, Abar, Lbar, st);
    });
}

static la_status syrk_call(la_dtype dt, int trans, double alpha, int64_t batch, int n, int k, const void *A, void *B,
                           void *ws, size_t ws_bytes, void *stream)
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
    if (ws_hits(ws, ws_bytes, A, ab) || ws_hits(ws, ws_bytes, B, bb))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    return with_workspace(ws, ws_bytes, [&] { return syrk_body(dt, trans, alpha, batch, n, k, A, B, st); });
}

static la_status syrk_backward_call(la_dtype dt, int trans, double alpha, int64_t batch, int n, int k, const void *A,
                                    const void *Bbar, void *Abar, void *ws, size_t ws_bytes, void *stream)
{
    if (bad_dtype(dt) || batch < 0 || n < 0 || k < 0 || n > MAX_N || k > MAX_N)
        return LA_ERR_INVALID_ARG;
    if (batch == 0 || n == 0 || k == 0)
        return LA_OK;
    if (!A || !Bbar || !Abar)
        return LA_ERR_INVALID_ARG;
    const size_t ab = (size_t)batch * n * k * esize(dt), bb = (size_t)batch * n * n * esize(dt);
    if (overlap(Abar, ab, A, ab) || overlap(Abar, ab, Bbar, bb))
        return LA_ERR_INVALID_ARG;
    if (ws_hits(ws, ws_bytes, A, ab) || ws_hits(ws, ws_bytes, Bbar, bb) || ws_hits(ws, ws_bytes, Abar, ab))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    return with_workspace(ws, ws_bytes, [&] { return syrk_backward_body(dt, trans, alpha, batch, n, k, A, Bbar, Abar, st); });
}

static la_status gemm2_call(la_dtype dt, int ta, int tb, double alpha, int64_t batch, int m, int n, int k, const void *A,
                            const void *B, void *C, void *ws, size_t ws_bytes, void *stream)
{
    if (bad_dtype(dt) || batch < 0 || m < 0 || n < 0 || k < 0 || m > MAX_N || n > MAX_N || k > MAX_N)
        return LA_ERR_INVALID_ARG;
    if (batch == 0 || m == 0 || n == 0)
        return LA_OK;
    if (!C || (k > 0 && (!A || !B)))
        return LA_ERR_INVALID_ARG;
    const size_t ab = (size_t)batch * m * k * esize(dt), bb = (size_t)batch * k * n * esize(dt),
                 cb = (size_t)batch * m * n * esize(dt);
    if (k > 0 && (overlap(A, ab, C, cb) || overlap(B, bb, C, cb)))
        return LA_ERR_INVALID_ARG;
    if (ws_hits(ws, ws_bytes, A, ab) || ws_hits(ws, ws_bytes, B, bb) || ws_hits(ws, ws_bytes, C, cb))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    return with_workspace(ws, ws_bytes, [&] { return gemm2_body(dt, ta, tb, alpha, batch, m, n, k, A, B, C, st); });
}

static la_status gemm2_backward_call(la_dtype dt, int ta, int tb, double alpha, int64_t batch, int m, int n, int k,
                                     const void *A, const void *B, const void *Cbar, void *Abar, void *Bbar, void *ws,
                                     size_t ws_bytes, void *stream)
{
    if (bad_dtype(dt) || batch < 0 || m < 0 || n < 0 || k < 0 || m > MAX_N || n > MAX_N || k > MAX_N)
        return LA_ERR_INVALID_ARG;
    if (batch == 0)
        return LA_OK;
    const size_t sa = (size_t)batch * m * k * esize(dt), sb = (size_t)batch * k * n * esize(dt),
                 sc = (size_t)batch * m * n * esize(dt);
    if ((sa && (!A || !Abar)) || (sb && (!B || !Bbar)) || (sc && !Cbar))
        return LA_ERR_INVALID_ARG;
    if (overlap(Abar, sa, A, sa) || overlap(Abar, sa, B, sb) || overlap(Abar, sa, Cbar, sc) || overlap(Bbar, sb, A, sa) ||
        overlap(Bbar, sb, B, sb) || overlap(Bbar, sb, Cbar, sc) || overlap(Abar, sa, Bbar, sb))
        return LA_ERR_INVALID_ARG;
    if (ws_hits(ws, ws_bytes, A, sa) || ws_hits(ws, ws_bytes, B, sb) || ws_hits(ws, ws_bytes, Cbar, sc) ||
        ws_hits(ws, ws_bytes, Abar, sa) || ws_hits(ws, ws_bytes, Bbar, sb))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (m == 0 || n == 0 || k == 0) {  // empty products: the gradients that exist are zero
        if (sa)
            LA_TRY(launch_fill_i32((int32_t *)Abar, (int64_t)(sa / 4), 0, st));
        if (sb)
            LA_TRY(launch_fill_i32((int32_t *)Bbar, (int64_t)(sb / 4), 0, st));
        return LA_OK;
    }
    return with_workspace(ws, ws_bytes,
                          [&] { return gemm2_backward_body(dt, ta, tb, alpha, batch, m, n, k, A, B, Cbar, Abar, Bbar, st); });
}

static la_status potri_call(la_dtype dt, int lower, int64_t batch, int n, const void *L, void *B, void *ws, size_t ws_bytes,
                            void *stream)
{
    if (bad_dtype(dt) || batch < 0 || n < 0 || n > MAX_N)
        return LA_ERR_INVALID_ARG;
    if (batch == 0 || n == 0)
        return LA_OK;
    if (!L || !B)
        return LA_ERR_INVALID_ARG;
    const size_t nb = (size_t)batch * n * n * esize(dt);
    if (L != B && overlap(L, nb, B, nb))
        return LA_ERR_INVALID_ARG;
    if (ws_hits(ws, ws_bytes, L, nb) || ws_hits(ws, ws_bytes, B, nb))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    return with_workspace(ws, ws_bytes, [&] { return potri_body(dt, lower, batch, n, L, B, st); });
}

static la_status potri_backward_call(la_dtype dt, int lower, int64_t batch, int n, const void *L, const void *B,
                                     const void *Bbar, void *Lbar, void *ws, size_t ws_bytes, void *stream)
{
    if (bad_dtype(dt) || batch < 0 || n < 0 || n > MAX_N)
        return LA_ERR_INVALID_ARG;
    if (batch == 0 || n == 0)
        return LA_OK;
    if (!L || !B || !Bbar || !Lbar)
        return LA_ERR_INVALID_ARG;
    const size_t nb = (size_t)batch * n * n * esize(dt);
    if (overlap(Lbar, nb, L, nb) || overlap(Lbar, nb, B, nb) || overlap(Lbar, nb, Bbar, nb))
        return LA_ERR_INVALID_ARG;
    if (ws_hits(ws, ws_bytes, L, nb) || ws_hits(ws, ws_bytes, B, nb) || ws_hits(ws, ws_bytes, Bbar, nb) ||
        ws_hits(ws, ws_bytes, Lbar, nb))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    return with_workspace(ws, ws_bytes, [&] { return potri_backward_body(dt, lower, batch, n, L, B, Bbar, Lbar, st); });
}

// Operand addresses for the sizing passes of la_workspace_bytes: far apart, 256-byte aligned, never dereferenced.
static inline void *fake_operand(int i) { return reinterpret_cast<void *>(((uintptr_t)1 << 45) + ((uintptr_t)i << 41)); }

static inline size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

extern "C" {

size_t la_workspace_bytes(la_op op, la_dtype dt, int64_t batch, int n, int m, int k)
{
    if (bad_dtype(dt) || batch <= 0 || n < 0 || m < 0 || k < 0 || n > MAX_N || m > MAX_N || k > MAX_N)
        return 0;
    void *p0 = fake_operand(0), *p1 = fake_operand(1), *p2 = fake_operand(2), *p3 = fake_operand(3), *p4 = fake_operand(4);
    size_t most = 0;
    auto take = [&](auto &&body) {
        size_t peak = 0;
        if (sizing_pass(body, &peak) == LA_OK && peak > most)
            most = peak;
    };
    // every flag combination and every permitted aliasing: the answer holds for all of them
    for (int f = 0; f < 8; ++f) {
        const int lower = f & 1, trans = (f >> 1) & 1, right = (f >> 2) & 1;
        switch (op) {
        case LA_OP_POTRF:
            if (n > 0 && f < 2) {
                take([&] { return potrf_body(dt, lower, batch, n, p0, p1, nullptr, nullptr); });
                take([&] { return potrf_body(dt, lower, batch, n, p0, p0, nullptr, nullptr); });
            }
            break;
        case LA_OP_POTRF_BACKWARD:
            if (n > 0 && f < 2) {
                take([&] { return backward_body(dt, lower, batch, n, p0, p1, p2, nullptr); });
                take([&] { return backward_body(dt, lower, batch, n, p0, p1, p1, nullptr); });
            }
            break;
        case LA_OP_TRSM:
        case LA_OP_TRMM:
            if (n > 0 && m > 0) {
                take([&] { return tri_body(op == LA_OP_TRSM, dt, lower, trans, right, 1.0, batch, n, m, p0, p1, p2, nullptr); });
                take([&] { return tri_body(op == LA_OP_TRSM, dt, lower, trans, right, 0.5, batch, n, m, p0, p1, p1, nullptr); });
            }
            break;
        case LA_OP_TRSM_BACKWARD:
        case LA_OP_TRMM_BACKWARD:
            if (n > 0) {
                const bool solve = op == LA_OP_TRSM_BACKWARD;
                take([&] { return tri_backward_body(solve, dt, lower, trans, right, 0.5, batch, n, m, p0, p1, p2, p3, p4, nullptr); });
                take([&] { return tri_backward_body(solve, dt, lower, trans, right, 1.0, batch, n, m, p0, p1, p2, p2, p4, nullptr); });
            }
            break;
        case LA_OP_SYRK:
            if (n > 0 && f < 2)
                take([&] { return syrk_body(dt, f, 1.0, batch, n, k, p0, p1, nullptr); });
            break;
        case LA_OP_SYRK_BACKWARD:
            if (n > 0 && k > 0 && f < 2)
                take([&] { return syrk_backward_body(dt, f, 1.0, batch, n, k, p0, p1, p2, nullptr); });
            break;
        case LA_OP_GEMM2:
            if (m > 0 && n > 0 && f < 4)
                take([&] { return gemm2_body(dt, f & 1, f >> 1, 1.0, batch, m, n, k, p0, p1, p2, nullptr); });
            break;
        case LA_OP_GEMM2_BACKWARD:
            if (m > 0 && n > 0 && k > 0 && f < 4)
                take([&] { return gemm2_backward_body(dt, f & 1, f >> 1, 1.0, batch, m, n, k, p0, p1, p2, p3, p4, nullptr); });
            break;
        case LA_OP_POTRI:
            if (n > 0 && f < 2) {
                take([&] { return potri_body(dt, lower, batch, n, p0, p1, nullptr); });
                take([&] { return potri_body(dt, lower, batch, n, p0, p0, nullptr); });
            }
            break;
        case LA_OP_POTRI_BACKWARD:
            if (n > 0 && f < 2)
                take([&] { return potri_backward_body(dt, lower, batch, n, p0, p1, p2, p3, nullptr); });
            break;
        default:
            return 0;
        }
    }
    return most;
}

la_status la_potrf_batched(la_dtype dt, int lower, int64_t batch, int n, const void *A, void *L, int32_t *info,
                           void *stream)
{
    return potrf_call(dt, lower, batch, n, A, L, info, nullptr, 0, stream);
}
la_status la_potrf_batched_ws(la_dtype dt, int lower, int64_t batch, int n, const void *A, void *L, int32_t *info,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    return potrf_call(dt, lower, batch, n, A, L, info, workspace, workspace_bytes, stream);
}

// ---------------------------------------------------------------------------------
// potrf for callers that cannot allocate: the scratch of the blocked path is a static array in
// device memory, one copy per GPU, held from the moment the library is loaded on that GPU.
// Its device address is looked up once per device (first call on that device) and passed to the
// kernels like any workspace; the host-side name of the array is not an address and is never
// handed to a kernel or a copy.
// ---------------------------------------------------------------------------------
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[LA_NOALLOC_SCRATCH_BYTES];
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[64] = {};

la_status la_potrf_batched_noalloc(la_dtype dt, int lower, int64_t batch, int n, const void *A, void *L, int32_t *info,
                                   void *stream)
{
    if (bad_dtype(dt) || batch < 0 || n < 0 || n > MAX_N)
        return LA_ERR_INVALID_ARG;
    if (batch == 0 || n == 0)
        return LA_OK;
    int dev = 0;
    LA_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64)
        return LA_ERR_UNSUPPORTED;
    void *ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void *p = nullptr;
            LA_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            if (!p) {
                snprintf(g_err, sizeof(g_err), "hipGetSymbolAddress returned no address for the static scratch array");
                return LA_ERR_RUNTIME;
            }
            g_scratch_ptr[dev] = p;
        }
        ptr = g_scratch_ptr[dev];
    }
    const la_status s = potrf_call(dt, lower, batch, n, A, L, info, ptr, (size_t)LA_NOALLOC_SCRATCH_BYTES, stream);
    if (s == LA_ERR_WORKSPACE) {
        const size_t need = la_workspace_bytes(LA_OP_POTRF, dt, batch, n, 0, 0);
        snprintf(g_err, sizeof(g_err),
                 "la_potrf_batched_noalloc: batch %lld of n = %d needs %zu bytes of scratch, the static buffer holds %zu",
                 (long long)batch, n, need, (size_t)LA_NOALLOC_SCRATCH_BYTES);
    }
    return s;
}

la_status la_potrf_backward(la_dtype dt, int lower, int64_t batch, int n, const void *L, const void *Lbar, void *Abar,
                            void *stream)
{
    return backward_call(dt, lower, batch, n, L, Lbar, Abar, nullptr, 0, stream);
}
la_status la_potrf_backward_ws(la_dtype dt, int lower, int64_t batch, int n, const void *L, const void *Lbar, void *Abar,
                               void *workspace, size_t workspace_bytes, void *stream)
{
    return backward_call(dt, lower, batch, n, L, Lbar, Abar, workspace, workspace_bytes, stream);
}

la_status la_trsm_batched(la_dtype dt, int lower, int trans, int rightside, double alpha, int64_t batch, int n, int m,
                          const void *L, const void *A, void *B, void *stream)
{
    return tri_call(true, dt, lower, trans, rightside, alpha, batch, n, m, L, A, B, nullptr, 0, stream);
}
la_status la_trsm_batched_ws(la_dtype dt, int lower, int trans, int rightside, double alpha, int64_t batch, int n, int m,
                             const void *L, const void *A, void *B, void *workspace, size_t workspace_bytes, void *stream)
{
    return tri_call(true, dt, lower, trans, rightside, alpha, batch, n, m, L, A, B, workspace, workspace_bytes, stream);
}

la_status la_trmm_batched(la_dtype dt, int lower, int trans, int rightside, double alpha, int64_t batch, int n, int m,
                          const void *L, const void *A, void *B, void *stream)
{
    return tri_call(false, dt, lower, trans, rightside, alpha, batch, n, m, L, A, B, nullptr, 0, stream);
}
la_status la_trmm_batched_ws(la_dtype dt, int lower, int trans, int rightside, double alpha, int64_t batch, int n, int m,
                             const void *L, const void *A, void *B, void *workspace, size_t workspace_bytes, void *stream)
{
    return tri_call(false, dt, lower, trans, rightside, alpha, batch, n, m, L, A, B, workspace, workspace_bytes, stream);
}

la_status la_trsm_backward(la_dtype dt, int lower, int trans, int rightside, double alpha, int64_t batch, int n, int m,
                           const void *L, const void *B, const void *Bbar, void *Abar, void *Lbar, void *stream)
{
    return tri_backward_call(true, dt, lower, trans, rightside, alpha, batch, n, m, L, B, Bbar, Abar, Lbar, nullptr, 0, stream);
}
la_status la_trsm_backward_ws(la_dtype dt, int lower, int trans, int rightside, double alpha, int64_t batch, int n, int m,
                              const void *L, const void *B, const void *Bbar, void *Abar, void *Lbar, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    return tri_backward_call(true, dt, lower, trans, rightside, alpha, batch, n, m, L, B, Bbar, Abar, Lbar, workspace,
                             workspace_bytes, stream);
}

la_status la_trmm_backward(la_dtype dt, int lower, int trans, int rightside, double alpha, int64_t batch, int n, int m,
                           const void *L, const void *A, const void *Bbar, void *Abar, void *Lbar, void *stream)
{
    return tri_backward_call(false, dt, lower, trans, rightside, alpha, batch, n, m, L, A, Bbar, Abar, Lbar, nullptr, 0, stream);
}
la_status la_trmm_backward_ws(la_dtype dt, int lower, int trans, int rightside, double alpha, int64_t batch, int n, int m,
                              const void *L, const void *A, const void *Bbar, void *Abar, void *Lbar, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    return tri_backward_call(false, dt, lower, trans, rightside, alpha, batch, n, m, L, A, Bbar, Abar, Lbar, workspace,
                             workspace_bytes, stream);
}

la_status la_gemm2_backward(la_dtype dt, int ta, int tb, double alpha, int64_t batch, int m, int n, int k,
                            const void *A, const void *B, const void *Cbar, void *Abar, void *Bbar, void *stream)
{
    return gemm2_backward_call(dt, ta, tb, alpha, batch, m, n, k, A, B, Cbar, Abar, Bbar, nullptr, 0, stream);
}
la_status la_gemm2_backward_ws(la_dtype dt, int ta, int tb, double alpha, int64_t batch, int m, int n, int k,
                               const void *A, const void *B, const void *Cbar, void *Abar, void *Bbar, void *workspace,
                               size_t workspace_bytes, void *stream)
{
    return gemm2_backward_call(dt, ta, tb, alpha, batch, m, n, k, A, B, Cbar, Abar, Bbar, workspace, workspace_bytes, stream);
}

la_status la_potri(la_dtype dt, int lower, int64_t batch, int n, const void *L, void *B, void *stream)
{
    return potri_call(dt, lower, batch, n, L, B, nullptr, 0, stream);
}
la_status la_potri_ws(la_dtype dt, int lower, int64_t batch, int n, const void *L, void *B, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    return potri_call(dt, lower, batch, n, L, B, workspace, workspace_bytes, stream);
}

la_status la_potri_backward(la_dtype dt, int lower, int64_t batch, int n, const void *L, const void *B,
                            const void *Bbar, void *Lbar, void *stream)
{
    return potri_backward_call(dt, lower, batch, n, L, B, Bbar, Lbar, nullptr, 0, stream);
}
la_status la_potri_backward_ws(la_dtype dt, int lower, int64_t batch, int n, const void *L, const void *B,
                               const void *Bbar, void *Lbar, void *workspace, size_t workspace_bytes, void *stream)
{
    return potri_backward_call(dt, lower, batch, n, L, B, Bbar, Lbar, workspace, workspace_bytes, stream);
}

la_status la_syrk_backward(la_dtype dt, int trans, double alpha, int64_t batch, int n, int k, const void *A,
                           const void *Bbar, void *Abar, void *stream)
{
    return syrk_backward_call(dt, trans, alpha, batch, n, k, A, Bbar, Abar, nullptr, 0, stream);
}
la_status la_syrk_backward_ws(la_dtype dt, int trans, double alpha, int64_t batch, int n, int k, const void *A,
                              const void *Bbar, void *Abar, void *workspace, size_t workspace_bytes, void *stream)
{
    return syrk_backward_call(dt, trans, alpha, batch, n, k, A, Bbar, Abar, workspace, workspace_bytes, stream);
}

la_status la_syrk_batched(la_dtype dt, int trans, double alpha, int64_t batch, int n, int k, const void *A, void *B,
                          void *stream)
{
    return syrk_call(dt, trans, alpha, batch, n, k, A, B, nullptr, 0, stream);
}
la_status la_syrk_batched_ws(la_dtype dt, int trans, double alpha, int64_t batch, int n, int k, const void *A, void *B,
                             void *workspace, size_t workspace_bytes, void *stream)
{
    return syrk_call(dt, trans, alpha, batch, n, k, A, B, workspace, workspace_bytes, stream);
}

la_status la_gemm2_batched(la_dtype dt, int ta, int tb, double alpha, int64_t batch, int m, int n, int k, const void *A,
                           const void *B, void *C, void *stream)
{
    return gemm2_call(dt, ta, tb, alpha, batch, m, n, k, A, B, C, nullptr, 0, stream);
}
la_status la_gemm2_batched_ws(la_dtype dt, int ta, int tb, double alpha, int64_t batch, int m, int n, int k, const void *A,
                              const void *B, void *C, void *workspace, size_t workspace_bytes, void *stream)
{
    return gemm2_call(dt, ta, tb, alpha, batch, m, n, k, A, B, C, workspace, workspace_bytes, stream);
}

size_t la_sgp_workspace_bytes(la_dtype dt, int U, int n)
{
    if (bad_dtype(dt) || U <= 0 || n <= 0 || U > MAX_N || n > MAX_N)
        return 0;
    const size_t e = dt == LA_F32 ? sgp_workspace_elems<float>(U, n) : sgp_workspace_elems<double>(U, n);
    const size_t fixed = align256(e * esize(dt) + 8 + 7 * SGP_PARTIALS * sizeof(double));
    void *p[10];
    for (int i = 0; i < 10; ++i)
        p[i] = fake_operand(i);
    size_t peak = 0;
    const la_status s = sizing_pass(
        [&] {
            return dt == LA_F32 ? sgp_t<float>(U, n, p[0], p[1], p[2], p[3], 1.0, p[4], p[5], p[6], p[7], p[8], p[9],
                                               fake_operand(10), nullptr)
                                : sgp_t<double>(U, n, p[0], p[1], p[2], p[3], 1.0, p[4], p[5], p[6], p[7], p[8], p[9],
                                                fake_operand(10), nullptr);
        },
        &peak);
    return s == LA_OK ? fixed + peak : 0;
}

la_status la_sgp_criterion(la_dtype dt, int U, int n, const void *Kuu, const void *Kuf, const void *Kff_diag,
                           const void *y, double noise_var, void *phi, void *Kuu_bar, void *Kuf_bar, void *Kff_diag_bar,
                           void *y_bar, void *noise_bar, void *workspace, size_t workspace_bytes, void *stream)
{
    if (bad_dtype(dt) || U <= 0 || n <= 0 || U > MAX_N || n > MAX_N || !(noise_var > 0.0))
        return LA_ERR_INVALID_ARG;
    if (!Kuu || !Kuf || !Kff_diag || !y || !phi || !Kuu_bar || !Kuf_bar || !Kff_diag_bar || !y_bar || !noise_bar ||
        !workspace || ((uintptr_t)workspace & 255))
        return LA_ERR_INVALID_ARG;
    const size_t e = dt == LA_F32 ? sgp_workspace_elems<float>(U, n) : sgp_workspace_elems<double>(U, n);
    const size_t fixed = align256(e * esize(dt) + 8 + 7 * SGP_PARTIALS * sizeof(double));
    if (workspace_bytes < fixed) {
        snprintf(g_err, sizeof(g_err), "this call needs a workspace of la_sgp_workspace_bytes bytes, %zu given",
                 workspace_bytes);
        return LA_ERR_WORKSPACE;
    }
    const size_t uu = (size_t)U * U * esize(dt), un = (size_t)U * n * esize(dt);
    if (overlap(Kuu_bar, uu, Kuu, uu) || overlap(Kuf_bar, un, Kuf, un) || overlap(Kuu_bar, uu, Kuf_bar, un) ||
        overlap(workspace, workspace_bytes, Kuu_bar, uu) || overlap(workspace, workspace_bytes, Kuf_bar, un) ||
        overlap(workspace, workspace_bytes, Kuu, uu) || overlap(workspace, workspace_bytes, Kuf, un))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    return with_workspace((char *)workspace + fixed, workspace_bytes - fixed, [&] {
        return dt == LA_F32 ? sgp_t<float>(U, n, Kuu, Kuf, Kff_diag, y, noise_var, phi, Kuu_bar, Kuf_bar, Kff_diag_bar, y_bar,
                                           noise_bar, workspace, st)
                            : sgp_t<double>(U, n, Kuu, Kuf, Kff_diag, y, noise_var, phi, Kuu_bar, Kuf_bar, Kff_diag_bar, y_bar,
                                            noise_bar, workspace, st);
    });
}

la_status la_kalman_filter(la_dtype dt, int64_t batch, int T, int dh, int dv, int shared_params, const void *A,
                           const void *B, const void *Sh, const void *Sv, const void *mu0, const void *S0,
                           const void *v, void *f, void *F, void *nll, int32_t *info, void *stream)
{
    if (bad_dtype(dt) || batch < 0 || T < 0 || dh < 1 || dv < 1)
        return LA_ERR_INVALID_ARG;
    if (dh > 16 || dv > 16)
        return LA_ERR_UNSUPPORTED;
    if (batch == 0)
        return LA_OK;
    if (!A || !B || !Sh || !Sv || !mu0 || !S0 || !nll || (T > 0 && !v))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (dt == LA_F32)
        return launch_kalman<float>((const float *)A, (const float *)B, (const float *)Sh, (const float *)Sv,
                                    (const float *)mu0, (const float *)S0, (const float *)v, (float *)f, (float *)F,
                                    (float *)nll, info, batch, T, dh, dv, shared_params != 0, st);
    return launch_kalman<double>((const double *)A, (const double *)B, (const double *)Sh, (const double *)Sv,
                                 (const double *)mu0, (const double *)S0, (const double *)v, (double *)f, (double *)F,
                                 (double *)nll, info, batch, T, dh, dv, shared_params != 0, st);
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

// fixed part of the GP criterion's workspace above the one-launch sizes: L, Lbar, z, alpha
static size_t gp_fixed_bytes(la_dtype dt, int64_t batch, int n)
{
    return align256(((size_t)batch * n * n * 2 + (size_t)batch * n * 2) * esize(dt));
}

size_t la_gp_workspace_bytes(la_dtype dt, int64_t batch, int n)
{
    if (bad_dtype(dt) || batch <= 0 || n <= 0 || n > MAX_N)
        return 0;
    const int fused = dt == LA_F32 ? backward_leaf16_max_n<float>() : backward_leaf16_max_n<double>();
    if (n <= fused)
        return 0;
    size_t peak = 0;
    const la_status s = sizing_pass(
        [&] {
            return dt == LA_F32 ? gp_t<float>(batch, n, fake_operand(0), fake_operand(1), fake_operand(2), fake_operand(3),
                                              nullptr, fake_operand(4), nullptr)
                                : gp_t<double>(batch, n, fake_operand(0), fake_operand(1), fake_operand(2), fake_operand(3),
                                               nullptr, fake_operand(4), nullptr);
        },
        &peak);
    return s == LA_OK ? gp_fixed_bytes(dt, batch, n) + peak : 0;
}

la_status la_gp_criterion(la_dtype dt, int64_t batch, int n, const void *A, const void *y, void *loss, void *Abar,
                          int32_t *info, void *workspace, size_t workspace_bytes, void *stream)
{
    if (bad_dtype(dt) || batch < 0 || n < 0 || n > MAX_N)
        return LA_ERR_INVALID_ARG;
    if (batch == 0)
        return LA_OK;
    if (!loss || (n > 0 && (!A || !y || !Abar)))
        return LA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (n == 0)  // empty sums
        return dt == LA_F32 ? launch_gp_glue<float>(nullptr, nullptr, nullptr, nullptr, (float *)loss, nullptr, batch, 0, st)
                            : launch_gp_glue<double>(nullptr, nullptr, nullptr, nullptr, (double *)loss, nullptr, batch, 0,
                                                     st);
    const int fused = dt == LA_F32 ? backward_leaf16_max_n<float>() : backward_leaf16_max_n<double>();
    const size_t fixed = n <= fused ? 0 : gp_fixed_bytes(dt, batch, n);
    const size_t bytes = (size_t)batch * n * n * esize(dt);
    if (fixed > 0) {
        if (!workspace || workspace_bytes < fixed) {
            snprintf(g_err, sizeof(g_err), "this call needs a workspace of la_gp_workspace_bytes bytes, %zu given",
                     workspace ? workspace_bytes : (size_t)0);
            return LA_ERR_WORKSPACE;
        }
        if (((uintptr_t)workspace & 255) || overlap(workspace, workspace_bytes, A, bytes) ||
            overlap(workspace, workspace_bytes, Abar, bytes))
            return LA_ERR_INVALID_ARG;
    }
    if (A != Abar && overlap(A, bytes, Abar, bytes))
        return LA_ERR_INVALID_ARG;
    return with_workspace(fixed ? (char *)workspace + fixed : nullptr, fixed ? workspace_bytes - fixed : 0, [&] {
        return dt == LA_F32 ? gp_t<float>(batch, n, A, y, loss, Abar, info, workspace, st)
                            : gp_t<double>(batch, n, A, y, loss, Abar, info, workspace, st);
    });
}

const char *la_last_error(void) { return g_err; }

int la_version(void) { return 200; }

}  // extern "C"
