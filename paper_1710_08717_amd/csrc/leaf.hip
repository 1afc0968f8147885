// Diagonal-block leaf of the blocked potrf (section 4.2 of arXiv 1710.08717: A = L L^T):
// factors one block of edge nb <= 64 per workgroup AND inverts the factor in the same pass,
// because every panel solve against this block later multiplies by that inverse.
//
// 1024 threads; thread (r, g) keeps the CW = 4 columns CW*g .. CW*g+CW-1 of row r of the block,
// and of the inverse under construction, in registers (many threads with little work each:
// the 64 pivots are strictly sequential, so the time of a step is what counts).  Both the right-looking factorisation and the
// right-looking triangular inversion need, at step k, one column (of A) and one row (of X)
// broadcast to everybody: the owners drop them RAW into LDS, one barrier, and every thread
// applies the pivot scaling itself:
//     a_rc -= a_rk a_ck / a_kk        (rank-1 update of the trailing block)
//     x_rc -= a_rk x_kc / a_kk        (row k of L^-1 times column k of L)
// so a step costs one barrier.  Double-buffered broadcast slots make that single barrier enough.
#include "common.hpp"

namespace la {

constexpr int LEAF_CW = 4;                    // columns per thread
constexpr int LEAF_GR = NB / LEAF_CW;         // column groups (threads per row)
constexpr int LEAF_THREADS = NB * LEAF_GR;    // 1024

template <typename T>
__global__ __launch_bounds__(LEAF_THREADS) void k_potrf_leaf(View<const T> A, View<T> L, View<T> Inv, int32_t *info,
                                                    int info_off, int64_t batch, int nb)
{
    __shared__ T colbuf[2][NB];
    __shared__ T rowbuf[2][NB];
    __shared__ int s_fail;
    const int tid = threadIdx.x;
    constexpr int CW = LEAF_CW, GR = LEAF_GR;
    const int r = tid / GR, g = tid % GR;
    const int64_t b = blockIdx.x;
    const T *ap = A.p + b * A.bs;
    if (tid == 0)
        s_fail = 0;

    // my CW entries of row r (lower triangle only; identity outside nb x nb).  a[] is the working
    // copy, lf[] receives the finished entries of L, x[] is the inverse under construction.
    T a[CW], lf[CW], x[CW];
    T myrs = T(1);
#pragma unroll
    for (int c = 0; c < CW; ++c) {
        const int col = g * CW + c;
        T v = (col == r) ? T(1) : T(0);
        if (r < nb && col <= r)
            v = ap[(int64_t)r * A.rs + (int64_t)col * A.cs];
        a[c] = v;
        lf[c] = T(0);
        x[c] = (col == r) ? T(1) : T(0);
    }

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
            }
            __syncthreads();
            const T akk = colbuf[slot][k];
            if (tid == 0 && !(akk > T(0)) && s_fail == 0)
                s_fail = k + 1;
            const T rs = rsqrt_acc(akk);
            const T ark = colbuf[slot][r];
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
    if (info != nullptr && tid == 0 && s_fail != 0 && s_fail <= nb) {
        if (info[b] == 0)
            info[b] = info_off + s_fail;
    }
}

template <typename T>
la_status launch_potrf_leaf(View<const T> A, View<T> L, View<T> Inv, int32_t *info, int info_off, int64_t batch, int nb,
                            hipStream_t st)
{
    if (batch <= 0 || nb <= 0)
        return LA_OK;
    if (nb > NB || batch > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((k_potrf_leaf<T>), dim3((unsigned)batch), dim3(LEAF_THREADS), 0, st, A, L, Inv, info, info_off, batch, nb);
    return launch_check("potrf_leaf");
}

template la_status launch_potrf_leaf<float>(View<const float>, View<float>, View<float>, int32_t *, int, int64_t, int,
                                            hipStream_t);
template la_status launch_potrf_leaf<double>(View<const double>, View<double>, View<double>, int32_t *, int, int64_t,
                                             int, hipStream_t);

}  // namespace la
