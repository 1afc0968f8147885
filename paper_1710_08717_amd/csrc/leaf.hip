// Diagonal-block leaf of the blocked potrf (section 4.2 of arXiv 1710.08717: A = L L^T):
// factors one block of edge nb <= 64 per workgroup AND inverts the factor in the same pass,
// because every panel solve against this block later multiplies by that inverse.
//
// 512 threads; thread (r, g) keeps the CW = 8 columns CW*g .. CW*g+CW-1 of row r of the block,
// and of the inverse under construction, in registers (two wavefronts per SIMD: the 64 pivots
// are strictly sequential, so the time of a step is what counts, and that is the instructions
// a SIMD has to issue per step plus one barrier).  Both the right-looking factorisation and the
// right-looking triangular inversion need, at step k, one column (of A) and one row (of X)
// broadcast to everybody: the owners drop them RAW into LDS, one barrier, and every thread
// applies the pivot scaling itself:
//     a_rc -= a_rk a_ck / a_kk        (rank-1 update of the trailing block)
//     x_rc -= a_rk x_kc / a_kk        (row k of L^-1 times column k of L)
// so a step costs one barrier.  Double-buffered broadcast slots make that single barrier enough.
#include "common.hpp"

namespace la {

constexpr int LEAF_CW = 8;                    // columns per thread
constexpr int LEAF_GR = NB / LEAF_CW;         // column groups (threads per row)
constexpr int LEAF_THREADS = NB * LEAF_GR;    // 512
constexpr int LEAF_TPW = 16 / (LEAF_THREADS / 64);  // 16 x 16 output tiles per wavefront in the block products

// The 64 pivot steps on the calling workgroup's registers: a[] (row r, columns CW*g ..) holds the
// lower triangle of the block on entry and the factor on exit, x[] the identity on entry and
// the inverse of the factor on exit.  fail becomes fail_base + (failing column + 1) at the first
// pivot that is not > 0 (kept in a register of every thread: no shared-memory traffic).
template <typename T>
__device__ __forceinline__ void leaf_factor(T (&a)[LEAF_CW], T (&x)[LEAF_CW], T (*colbuf)[NB], T (*rowbuf)[NB],
                                            T (*piv)[2], int &fail, int fail_base)
{
    constexpr int CW = LEAF_CW, GR = LEAF_GR;
    const int tid = threadIdx.x;
    const int r = tid / GR, g = tid % GR;
    T lf[CW];
    T myrs = T(1);
#pragma unroll
    for (int c = 0; c < CW; ++c)
        lf[c] = T(0);
    // Only clean values are ever broadcast: the column slot gets zeros for rows above the pivot,
    // and rows of the inverse are zero beyond their diagonal by construction.  The updates
    // below therefore need no masks: what they do to register entries above the diagonal, or to
    // entries of columns that are already finished (saved in lf[]), is never looked at again.
#pragma unroll 1
    for (int kg = 0; kg < GR; ++kg) {
#pragma unroll
        for (int kk = 0; kk < CW; ++kk) {
            const int k = kg * CW + kk;
            const int slot = k & 1;
            if (g == kg)
                colbuf[slot][r] = (r >= k) ? a[kk] : T(0);  // raw column k, rows >= k
            if (r == k) {
#pragma unroll
                for (int c = 0; c < CW; ++c)
                    rowbuf[slot][g * CW + c] = x[c];  // raw row k of the inverse
                if (g == kg) {  // the owner of the pivot works out 1 / sqrt(a_kk) for everybody
                    piv[slot][0] = a[kk];
                    piv[slot][1] = rsqrt_acc(a[kk]);
                }
            }
            __syncthreads();
            const T akk = piv[slot][0];
            const T rs = piv[slot][1];
            const T ark = colbuf[slot][r];
            fail = (!(akk > T(0)) && fail == 0) ? fail_base + k + 1 : fail;  // every thread keeps its own copy
            const T t = (r > k) ? ark * (rs * rs) : T(0);  // a_rk / a_kk
            T cb[CW], rb[CW];
#pragma unroll
            for (int c = 0; c < CW; ++c) {
                cb[c] = colbuf[slot][g * CW + c];
                rb[c] = rowbuf[slot][g * CW + c];
            }
#pragma unroll
            for (int c = 0; c < CW; ++c) {
                a[c] = fma(-t, cb[c], a[c]);  // a_rc -= a_rk a_ck / a_kk
                x[c] = fma(-t, rb[c], x[c]);  // x_rc -= a_rk x_kc / a_kk
            }
            // keep the compiler from postponing these updates over several steps (which would hold
            // every step's broadcast values in registers at once)
#pragma unroll
            for (int c = 0; c < CW; ++c) {
                asm volatile("" : "+v"(a[c]));
                asm volatile("" : "+v"(x[c]));
            }
            lf[kk] = (g == kg) ? ark * rs : lf[kk];  // column k of L: a_rk / sqrt(a_kk), zero above the pivot
            myrs = (r == k) ? rs : myrs;             // row r of L^-1 is its raw row times 1 / l_rr
        }
    }
#pragma unroll
    for (int c = 0; c < CW; ++c) {
        a[c] = lf[c];
        x[c] *= myrs;
    }
    __syncthreads();  // the broadcast slots may be reused by the caller
}

template <typename T>
__global__ __launch_bounds__(LEAF_THREADS) void k_potrf_leaf(View<const T> A, View<T> L, View<T> Inv, int32_t *info,
                                                             int info_off, int64_t batch, int nb)
{
    __shared__ T colbuf[2][NB];
    __shared__ T rowbuf[2][NB];
    __shared__ __align__(16) T piv[2][2];
    constexpr int CW = LEAF_CW, GR = LEAF_GR;
    const int tid = threadIdx.x;
    const int r = tid / GR, g = tid % GR;
    const int64_t b = blockIdx.x;
    const T *ap = A.p + b * A.bs;
    int fail = 0;

    // my CW entries of row r (lower triangle only; identity outside nb x nb)
    T a[CW], x[CW];
#pragma unroll
    for (int c = 0; c < CW; ++c) {
        const int col = g * CW + c;
        T v = (col == r) ? T(1) : T(0);
        if (r < nb && col <= r)
            v = ap[(int64_t)r * A.rs + (int64_t)col * A.cs];
        a[c] = v;
        x[c] = (col == r) ? T(1) : T(0);
    }
    leaf_factor<T>(a, x, colbuf, rowbuf, piv, fail, 0);

    T *lp = L.p + b * L.bs;
    T *ip = Inv.p + b * Inv.bs;
#pragma unroll
    for (int c = 0; c < CW; ++c) {
        const int col = g * CW + c;
        if (r < nb && col < nb) {
            lp[(int64_t)r * L.rs + (int64_t)col * L.cs] = (col <= r) ? a[c] : T(0);
            ip[(int64_t)r * Inv.rs + (int64_t)col * Inv.cs] = (col <= r) ? x[c] : T(0);
        }
    }
    if (info != nullptr && tid == 0 && fail != 0 && fail <= nb) {
        if (info[b] == 0)
            info[b] = info_off + fail;
    }
}

// ---------------------------------------------------------------------------------------
// Blocks of edge 64 < nb <= 128 in one launch: [A00 0; A10 A11] with 64 x 64 sub-blocks,
//   L00, Li00 = factor(A00);  L10 = A10 Li00^T;  L11, Li11 = factor(A11 - L10 L10^T);
//   Li10 = -Li11 (L10 Li00)
// The four 64 x 64 x 64 products run on the matrix cores, a row of four 16 x 16 output tiles
// per wavefront, operands in LDS.
// ---------------------------------------------------------------------------------------
constexpr int LEAF_LD = NB + 1;

// Tiles (ti, tj0 .. tj0 + TPW - 1), 16 x 16 each, of  sum_k A(i,k) B(k,j)  with
// A(i,k) = sA[i*a_si + k*a_sk] and B(k,j) = sB[k*b_sk + j*b_sj].
template <typename T>
__device__ __forceinline__ void leaf_product(typename Mfma<T>::acc_t (&acc)[LEAF_TPW], const T *sA, int a_si, int a_sk,
                                             const T *sB, int b_sk, int b_sj, int ti, int tj0, int lane)
{
    using MF = Mfma<T>;
    const int l16 = lane & 15, lk = lane >> 4;
#pragma unroll
    for (int q = 0; q < LEAF_TPW; ++q)
        acc[q] = typename MF::acc_t{0, 0, 0, 0};
#pragma unroll 4
    for (int kk = 0; kk < NB; kk += 4) {
        const T av = sA[(ti * 16 + l16) * a_si + (kk + lk) * a_sk];
#pragma unroll
        for (int q = 0; q < LEAF_TPW; ++q) {
            const T bv = sB[(kk + lk) * b_sk + ((tj0 + q) * 16 + l16) * b_sj];
            acc[q] = MF::run(av, bv, acc[q]);
        }
    }
}

template <typename T>
__global__ __launch_bounds__(LEAF_THREADS) void k_potrf_leaf128(View<const T> A, View<T> L, View<T> Inv, int32_t *info,
                                                                int info_off, int64_t batch, int nb)
{
    using MF = Mfma<T>;
    __shared__ T sLi0[NB * LEAF_LD];
    __shared__ T sLi1[NB * LEAF_LD];
    __shared__ T sB1[NB * LEAF_LD];  // A10, then L10
    __shared__ T sC[NB * LEAF_LD];   // A11 - L10 L10^T, then L10 Li00
    __shared__ T colbuf[2][NB];
    __shared__ T rowbuf[2][NB];
    __shared__ __align__(16) T piv[2][2];
    constexpr int CW = LEAF_CW, GR = LEAF_GR, LD = LEAF_LD;
    const int tid = threadIdx.x;
    const int r = tid / GR, g = tid % GR;
    constexpr int TPW = LEAF_TPW;
    const int lane = tid & 63, w = tid >> 6;
    const int ti = w / (4 / TPW), tj0 = (w % (4 / TPW)) * TPW;  // this wavefront's output tiles
    const int l16 = lane & 15;
    const int n2 = nb - NB;  // rows of the second block (1 .. 64)
    const int64_t b = blockIdx.x;
    const T *ap = A.p + b * A.bs;
    T *lp = L.p + b * L.bs;
    T *ip = Inv.p + b * Inv.bs;
    int fail = 0;

    // ---- block (0,0) --------------------------------------------------------------------
    T a[CW], x[CW];
#pragma unroll
    for (int c = 0; c < CW; ++c) {
        const int col = g * CW + c;
        a[c] = (col <= r) ? ap[(int64_t)r * A.rs + (int64_t)col * A.cs] : T(0);
        x[c] = (col == r) ? T(1) : T(0);
        // A10 for the panel product (rows past the end of the block read as zero)
        sB1[r * LD + col] = (r < n2) ? ap[(int64_t)(NB + r) * A.rs + (int64_t)col * A.cs] : T(0);
    }
    leaf_factor<T>(a, x, colbuf, rowbuf, piv, fail, 0);
#pragma unroll
    for (int c = 0; c < CW; ++c) {
        const int col = g * CW + c;
        const T lv = (col <= r) ? a[c] : T(0), iv = (col <= r) ? x[c] : T(0);
        lp[(int64_t)r * L.rs + (int64_t)col * L.cs] = lv;
        ip[(int64_t)r * Inv.rs + (int64_t)col * Inv.cs] = iv;
        sLi0[r * LD + col] = iv;
    }
    __syncthreads();

    // ---- panel: L10 = A10 Li00^T ------------------------------------------------------------
    typename MF::acc_t acc[TPW];
    leaf_product<T>(acc, sB1, LD, 1, sLi0, 1, LD, ti, tj0, lane);
    __syncthreads();  // everybody is done reading A10
#pragma unroll
    for (int q = 0; q < TPW; ++q)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int tj = tj0 + q;
            const int i = ti * 16 + MF::row(lane, v), j = tj * 16 + l16;
            sB1[i * LD + j] = acc[q][v];
            if (i < n2)
                lp[(int64_t)(NB + i) * L.rs + (int64_t)j * L.cs] = acc[q][v];
        }
    __syncthreads();

    // ---- trailing block: A11 - L10 L10^T (lower triangle, identity padding) -------------------
    leaf_product<T>(acc, sB1, LD, 1, sB1, 1, LD, ti, tj0, lane);
#pragma unroll
    for (int q = 0; q < TPW; ++q)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int tj = tj0 + q;
            const int i = ti * 16 + MF::row(lane, v), j = tj * 16 + l16;
            T val = (i == j) ? T(1) : T(0);
            if (i < n2 && j <= i)
                val = ap[(int64_t)(NB + i) * A.rs + (int64_t)(NB + j) * A.cs] - acc[q][v];
            sC[i * LD + j] = val;
        }
    __syncthreads();

    // ---- block (1,1) --------------------------------------------------------------------
#pragma unroll
    for (int c = 0; c < CW; ++c) {
        const int col = g * CW + c;
        a[c] = (col <= r) ? sC[r * LD + col] : T(0);
        x[c] = (col == r) ? T(1) : T(0);
    }
    leaf_factor<T>(a, x, colbuf, rowbuf, piv, fail, NB);
#pragma unroll
    for (int c = 0; c < CW; ++c) {
        const int col = g * CW + c;
        const T lv = (col <= r) ? a[c] : T(0), iv = (col <= r) ? x[c] : T(0);
        if (r < n2 && col < n2) {
            lp[(int64_t)(NB + r) * L.rs + (int64_t)(NB + col) * L.cs] = lv;
            ip[(int64_t)(NB + r) * Inv.rs + (int64_t)(NB + col) * Inv.cs] = iv;
        }
        sLi1[r * LD + col] = iv;
    }
    __syncthreads();

    // ---- inverse, block (1,0): -Li11 (L10 Li00) ------------------------------------------------
    leaf_product<T>(acc, sB1, LD, 1, sLi0, LD, 1, ti, tj0, lane);
#pragma unroll
    for (int q = 0; q < TPW; ++q)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            sC[(ti * 16 + MF::row(lane, v)) * LD + (tj0 + q) * 16 + l16] = acc[q][v];
    __syncthreads();
    leaf_product<T>(acc, sLi1, LD, 1, sC, LD, 1, ti, tj0, lane);
#pragma unroll
    for (int q = 0; q < TPW; ++q)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int tj = tj0 + q;
            const int i = ti * 16 + MF::row(lane, v), j = tj * 16 + l16;
            if (i < n2)
                ip[(int64_t)(NB + i) * Inv.rs + (int64_t)j * Inv.cs] = -acc[q][v];
        }
    if (info != nullptr && tid == 0 && fail != 0 && fail <= nb) {
        if (info[b] == 0)
            info[b] = info_off + fail;
    }
}

template <typename T>
la_status launch_potrf_leaf(View<const T> A, View<T> L, View<T> Inv, int32_t *info, int info_off, int64_t batch, int nb,
                            hipStream_t st)
{
    if (batch <= 0 || nb <= 0)
        return LA_OK;
    if (nb > 2 * NB || batch > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    if (nb <= NB)
        hipLaunchKernelGGL((k_potrf_leaf<T>), dim3((unsigned)batch), dim3(LEAF_THREADS), 0, st, A, L, Inv, info,
                           info_off, batch, nb);
    else
        hipLaunchKernelGGL((k_potrf_leaf128<T>), dim3((unsigned)batch), dim3(LEAF_THREADS), 0, st, A, L, Inv, info,
                           info_off, batch, nb);
    return launch_check("potrf_leaf");
}

template la_status launch_potrf_leaf<float>(View<const float>, View<float>, View<float>, int32_t *, int, int64_t, int,
                                            hipStream_t);
template la_status launch_potrf_leaf<double>(View<const double>, View<double>, View<double>, int32_t *, int, int64_t,
                                             int, hipStream_t);

}  // namespace la
