// Diagonal-block leaf of the blocked potrf (section 4.2 of arXiv 1710.08717: A = L L^T):
// one workgroup factors a block of edge nb <= 128 AND inverts the factor, because every panel
// solve against this block later multiplies by that inverse.
//
// The block is cut into 16 x 16 tiles that live in LDS for the whole kernel.  Step k of the
// right-looking sweep over the K = ceil(nb / 16) tile columns:
//   (a) one wavefront factors the diagonal tile A_kk and inverts the factor in registers
//       (lane = row, registers = columns, column broadcasts are DPP operands of the
//       multiply-adds): L_kk, Li_kk;
//   (b) panel      L_ik = A_ik Li_kk^T  (i > k)   and   X_kj <- Li_kk X_kj  (j < k), which
//       completes row k of the inverse X = L^-1;
//   (c) trailing   A_ij -= L_ik L_jk^T  (k < j <= i)   and   X_ij -= L_ik X_kj  (i > k, j <= k).
// (b) and (c) are 16 x 16 x 16 products on the matrix cores, one tile per wavefront at a
// time.  The 16 * K pivots are strictly sequential, so what counts is the length of (a); the
// matrix-core phases are short and parallel.
#include "common.hpp"

namespace la {

constexpr int LT = 16;              // tile edge
constexpr int LK = 8;               // tiles per block edge (128 / 16)
constexpr int LEAF16_THREADS = 512;
constexpr int LEAF16_WAVES = LEAF16_THREADS / 64;

template <typename T>
struct Leaf16 {
    // row stride of the diagonal tiles (padded so that "lane = row" accesses spread over the
    // banks and stay 16-byte aligned)
    static constexpr int PS = LT + 16 / (int)sizeof(T);
    static constexpr int DT = LT * PS;            // elements of a padded diagonal tile
    static constexpr int OT = LT * LT;            // elements of an off-diagonal tile
    static constexpr int NOFF = LK * (LK - 1) / 2;
    // LDS map (elements): diagonal tiles of A/L, diagonal tiles of X, off-diagonal of A/L, of X
    static constexpr int OFF_D = 0;
    static constexpr int OFF_XD = OFF_D + LK * DT;
    static constexpr int OFF_A = OFF_XD + LK * DT;
    static constexpr int OFF_X = OFF_A + NOFF * OT;
    static constexpr int TOTAL = OFF_X + NOFF * OT;
};

__device__ __forceinline__ int tri_off(int i, int j) { return i * (i - 1) / 2 + j; }  // i > j

// acc -= (value of src in lane K of the 16-lane row) * other, one instruction.  The hardware
// needs two wait states between a VALU write of src and this read of it; callers keep that.
template <int K>
__device__ __forceinline__ void fnmac_row(float &acc, float src, float other)
{
    asm volatile("v_fmac_f32_dpp %0, -%1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
                 : "+v"(acc)
                 : "v"(src), "v"(other), "n"(K));
}
template <int K>
__device__ __forceinline__ void fnmac_row(double &acc, double src, double other)
{
    asm volatile("v_fmac_f64_dpp %0, -%1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
                 : "+v"(acc)
                 : "v"(src), "v"(other), "n"(K));
}
// acc -= (value of acc in lane K of the row) * other
template <int K>
__device__ __forceinline__ void fnmac_row_self(float &acc, float other)
{
    asm volatile("v_fmac_f32_dpp %0, -%0, %1 row_newbcast:%2 row_mask:0xf bank_mask:0xf" : "+v"(acc) : "v"(other), "n"(K));
}
template <int K>
__device__ __forceinline__ void fnmac_row_self(double &acc, double other)
{
    asm volatile("v_fmac_f64_dpp %0, -%0, %1 row_newbcast:%2 row_mask:0xf bank_mask:0xf" : "+v"(acc) : "v"(other), "n"(K));
}
// (value of src in lane K of the row) * other
template <int K>
__device__ __forceinline__ float mul_row(float src, float other)
{
    float d = 0.0f;
    asm volatile("v_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
                 : "+v"(d)
                 : "v"(src), "v"(other), "n"(K));
    return d;
}
template <int K>
__device__ __forceinline__ double mul_row(double src, double other)
{
    double d = 0.0;
    asm volatile("v_fmac_f64_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
                 : "+v"(d)
                 : "v"(src), "v"(other), "n"(K));
    return d;
}
// two wait states, with v routed through the statement so that whatever computes it stays before
template <typename T>
__device__ __forceinline__ void settle(T &v)
{
    asm volatile("s_nop 1" : "+v"(v));
}

__device__ __forceinline__ float rcp_newton(float x) { return __builtin_amdgcn_rcpf(x); }
__device__ __forceinline__ double rcp_newton(double x)
{
    double r = __builtin_amdgcn_rcp(x);
    double e = fma(-x, r, 1.0);
    r = fma(r, e, r);
    e = fma(-x, r, 1.0);
    return fma(r, e, r);
}

// Factor and invert one 16 x 16 tile held one row per lane (all four 16-lane rows of the
// wavefront work on copies of the same tile).  In: a[c] = A(r, c) for c <= r (what lies above
// the diagonal is never looked at).  Out: a[c] = L(r, c), x[c] = L^-1(r, c) for c <= r (entries
// above the diagonal hold leftovers) and the return value is the 1-based index of the first pivot
// that is not > 0, or 0.
//
// The pivots run on the unscaled matrix,   a_rc -= a_rk a_ck / a_kk,   x_rc -= a_rk x_kc / a_kk,
// which needs only a reciprocal on the critical path; the square roots are taken for all 16
// pivots at once afterwards:  L = A_raw diag(d)^-1/2,  L^-1 = diag(d)^-1/2 X_raw.
template <typename T>
__device__ __forceinline__ int diag_factor_invert(T (&a)[LT], T (&x)[LT], int r)
{
    T d = T(1);
#pragma unroll
    for (int c = 0; c < LT; ++c)
        x[c] = (c == r) ? T(1) : T(0);
    static_for<0, LT>([&](auto kc) {
        constexpr int k = decltype(kc)::value;
        T rinv = rcp_newton(a[k]);  // meaningful in lane k only
        const T am = (r > k) ? a[k] : T(0);
        d = (r == k) ? a[k] : d;
        settle(rinv);
        const T t = mul_row<k>(rinv, am);  // a_rk / a_kk below the pivot, zero elsewhere
        static_for<k + 1, LT>([&](auto cc) {
            constexpr int c = decltype(cc)::value;
            fnmac_row<c>(a[c], a[k], t);  // a_rc -= a_ck t_r
        });
        static_for<0, k + 1>([&](auto cc) {
            constexpr int c = decltype(cc)::value;
            fnmac_row_self<k>(x[c], t);  // x_rc -= x_kc t_r
        });
    });
    const unsigned long long bad = __ballot(!(d > T(0)));
    T rs = rsqrt_acc(d);
    settle(rs);
    static_for<0, LT>([&](auto cc) {
        constexpr int c = decltype(cc)::value;
        a[c] = mul_row<c>(rs, a[c]);  // column c times d_c^-1/2
        x[c] *= rs;                   // row r times d_r^-1/2
    });
    const unsigned first = (unsigned)(bad & 0xffffu);
    return first ? __builtin_ctz(first) + 1 : 0;
}

// four consecutive elements starting at p (16-byte aligned for the strides used here)
template <typename T>
__device__ __forceinline__ void load4(const T *p, T (&v)[4])
{
    using V = typename Mfma<T>::vec_t;
    constexpr int VW = Mfma<T>::VW;
    const V *q = reinterpret_cast<const V *>(p);
#pragma unroll
    for (int i = 0; i < 4 / VW; ++i) {
        const V w = q[i];
        if constexpr (VW == 2) {
            v[2 * i] = w.x;
            v[2 * i + 1] = w.y;
        } else {
            v[0] = w.x;
            v[1] = w.y;
            v[2] = w.z;
            v[3] = w.w;
        }
    }
}

// One 16 x 16 x 16 product step on a tile.  Operand element k of the contraction is dealt to
// lane group q = lane / 16 and register s as k = 4 q + s, the same for both operands, so that an
// operand stored with k contiguous is read as four consecutive elements per lane.
//   rowA / rowB: operand(i, k) = p[i * ld + k]        (this wavefront's lane supplies i = lane % 16)
//   natB:        operand(k, j) = p[k * ld + j]
template <typename T>
__device__ __forceinline__ void op_rows(const T *p, int ld, int lane, T (&v)[4])
{
    load4<T>(p + (lane & 15) * ld + 4 * (lane >> 4), v);
}
template <typename T>
__device__ __forceinline__ void op_nat(const T *p, int ld, int lane, T (&v)[4])
{
#pragma unroll
    for (int s = 0; s < 4; ++s)
        v[s] = p[(4 * (lane >> 4) + s) * ld + (lane & 15)];
}
template <typename T>
__device__ __forceinline__ typename Mfma<T>::acc_t acc_load(const T *p, int ld, int lane)
{
    typename Mfma<T>::acc_t c;
#pragma unroll
    for (int v = 0; v < 4; ++v)
        c[v] = p[Mfma<T>::row(lane, v) * ld + (lane & 15)];
    return c;
}
template <typename T>
__device__ __forceinline__ void acc_store(T *p, int ld, int lane, typename Mfma<T>::acc_t c)
{
#pragma unroll
    for (int v = 0; v < 4; ++v)
        p[Mfma<T>::row(lane, v) * ld + (lane & 15)] = c[v];
}
template <typename T>
__device__ __forceinline__ typename Mfma<T>::acc_t mma4(const T (&a)[4], const T (&b)[4], typename Mfma<T>::acc_t c,
                                                        bool neg)
{
#pragma unroll
    for (int s = 0; s < 4; ++s)
        c = Mfma<T>::run(neg ? -a[s] : a[s], b[s], c);
    return c;
}

template <typename T>
__global__ __launch_bounds__(LEAF16_THREADS) void k_potrf_leaf16(View<const T> A, View<T> L, View<T> Inv, int32_t *info,
                                                                 int info_off, int64_t batch, int nb, int zero_upper)
{
    using C = Leaf16<T>;
    using MF = Mfma<T>;
    extern __shared__ __align__(16) unsigned char leaf16_lds[];
    T *lds = reinterpret_cast<T *>(leaf16_lds);
    T *sD = lds + C::OFF_D, *sXD = lds + C::OFF_XD, *sA = lds + C::OFF_A, *sX = lds + C::OFF_X;
    constexpr int PS = C::PS, DT = C::DT, OT = C::OT;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int K = (nb + LT - 1) / LT;  // tile columns in use
    const int ne = K * LT;
    const int64_t b = blockIdx.x;
    const T *ap = A.p + b * A.bs;

    // ---- lower triangle of the block into tiles (identity outside nb x nb) ------------------
    {
        const bool colfast = (A.cs == 1) || (A.rs != 1);
        for (int e = tid; e < ne * ne; e += LEAF16_THREADS) {
            const int u = e / ne, w = e % ne;
            const int r = colfast ? u : w, c = colfast ? w : u;
            const int ti = r / LT, tj = c / LT;
            if (tj > ti)
                continue;
            T v = (r == c) ? T(1) : T(0);
            if (r < nb && c <= r)
                v = ap[(int64_t)r * A.rs + (int64_t)c * A.cs];
            if (ti == tj)
                sD[ti * DT + (r % LT) * PS + (c % LT)] = v;
            else
                sA[tri_off(ti, tj) * OT + (r % LT) * LT + (c % LT)] = v;
        }
    }
    __syncthreads();

    int fail = 0;
    for (int k = 0; k < K; ++k) {
        // ---- (a) diagonal tile ------------------------------------------------------------
        if (wave == 0) {
            const int r = lane & 15;
            T a[LT], x[LT];
            T *dk = sD + k * DT + r * PS, *xk = sXD + k * DT + r * PS;
#pragma unroll
            for (int c = 0; c < LT; c += 4) {
                T v[4];
                load4<T>(dk + c, v);
                a[c] = v[0];
                a[c + 1] = v[1];
                a[c + 2] = v[2];
                a[c + 3] = v[3];
            }
            const int f = diag_factor_invert<T>(a, x, r);
            if (fail == 0 && f != 0)
                fail = k * LT + f;
            if (lane < LT) {
#pragma unroll
                for (int c = 0; c < LT; ++c) {
                    dk[c] = (c <= r) ? a[c] : T(0);
                    xk[c] = (c <= r) ? x[c] : T(0);
                }
            }
        }
        __syncthreads();

        // ---- (b) panel below the diagonal tile, and row k of the inverse ------------------------
        const T *lik = sXD + k * DT;  // Li_kk, row stride PS
        for (int it = wave; it < K - 1; it += LEAF16_WAVES) {
            T av[4], bv[4];
            typename MF::acc_t acc = {0, 0, 0, 0};
            if (it < K - 1 - k) {  // L_ik = A_ik Li_kk^T
                const int i = k + 1 + it;
                T *t = sA + tri_off(i, k) * OT;
                op_rows<T>(t, LT, lane, av);
                op_rows<T>(lik, PS, lane, bv);
                acc = mma4<T>(av, bv, acc, false);
                acc_store<T>(t, LT, lane, acc);
            } else {  // X_kj <- Li_kk X_kj
                const int j = it - (K - 1 - k);
                T *t = sX + tri_off(k, j) * OT;
                op_rows<T>(lik, PS, lane, av);
                op_nat<T>(t, LT, lane, bv);
                acc = mma4<T>(av, bv, acc, false);
                acc_store<T>(t, LT, lane, acc);
            }
        }
        __syncthreads();

        // ---- (c) trailing updates --------------------------------------------------------------
        const int m = K - 1 - k;         // tile rows below the pivot row
        const int nx = m * (k + 1);      // tiles of X to update
        const int na = m * (m + 1) / 2;  // tiles of A to update
        for (int it = wave; it < nx + na; it += LEAF16_WAVES) {
            T av[4], bv[4];
            if (it < nx) {  // X_ij -= L_ik X_kj, j <= k
                const int i = k + 1 + it / (k + 1), j = it % (k + 1);
                T *t = sX + tri_off(i, j) * OT;
                op_rows<T>(sA + tri_off(i, k) * OT, LT, lane, av);
                typename MF::acc_t acc = {0, 0, 0, 0};
                if (j == k) {
                    op_nat<T>(lik, PS, lane, bv);
                } else {
                    op_nat<T>(sX + tri_off(k, j) * OT, LT, lane, bv);
                    acc = acc_load<T>(t, LT, lane);
                }
                acc = mma4<T>(av, bv, acc, true);
                acc_store<T>(t, LT, lane, acc);
            } else {  // A_ij -= L_ik L_jk^T, k < j <= i
                int e = it - nx, ii = 0;
                while (e > ii) {  // row ii of the triangle has ii + 1 tiles
                    e -= ii + 1;
                    ++ii;
                }
                const int i = k + 1 + ii, j = k + 1 + e;
                T *t = (i == j) ? sD + i * DT : sA + tri_off(i, j) * OT;
                const int ld = (i == j) ? PS : LT;
                op_rows<T>(sA + tri_off(i, k) * OT, LT, lane, av);
                op_rows<T>(sA + tri_off(j, k) * OT, LT, lane, bv);
                typename MF::acc_t acc = acc_load<T>(t, ld, lane);
                acc = mma4<T>(av, bv, acc, true);
                acc_store<T>(t, ld, lane, acc);
            }
        }
        __syncthreads();
    }

    // ---- factor and inverse back to memory (lower tiles; zeros above the diagonal of the
    //      diagonal tiles) ----------------------------------------------------------------------
    {
        T *lp = L.p + b * L.bs;
        T *ip = Inv.p + b * Inv.bs;
        const bool colfast = (L.cs == 1) || (L.rs != 1);
        for (int e = tid; e < ne * ne; e += LEAF16_THREADS) {
            const int u = e / ne, w = e % ne;
            const int r = colfast ? u : w, c = colfast ? w : u;
            const int ti = r / LT, tj = c / LT;
            if (r >= nb || c >= nb)
                continue;
            if (tj > ti) {
                if (zero_upper)
                    lp[(int64_t)r * L.rs + (int64_t)c * L.cs] = T(0);
                continue;
            }
            T lv, xv;
            if (ti == tj) {
                lv = sD[ti * DT + (r % LT) * PS + (c % LT)];
                xv = sXD[ti * DT + (r % LT) * PS + (c % LT)];
            } else {
                lv = sA[tri_off(ti, tj) * OT + (r % LT) * LT + (c % LT)];
                xv = sX[tri_off(ti, tj) * OT + (r % LT) * LT + (c % LT)];
            }
            lp[(int64_t)r * L.rs + (int64_t)c * L.cs] = lv;
            ip[(int64_t)r * Inv.rs + (int64_t)c * Inv.cs] = xv;
        }
    }
    if (info != nullptr && tid == 0 && fail != 0 && fail <= nb) {
        if (info[b] == 0)
            info[b] = info_off + fail;
    }
}

template <typename T>
la_status launch_potrf_leaf16(View<const T> A, View<T> L, View<T> Inv, int32_t *info, int info_off, int64_t batch,
                              int nb, bool zero_upper, hipStream_t st)
{
    if (batch <= 0 || nb <= 0)
        return LA_OK;
    if (nb > LT * LK || batch > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    constexpr size_t lds_bytes = (size_t)Leaf16<T>::TOTAL * sizeof(T);
    static bool configured[64] = {};
    int dev = 0;
    LA_HIP(hipGetDevice(&dev));
    if (dev >= 0 && dev < 64 && !configured[dev]) {
        LA_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_potrf_leaf16<T>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
        configured[dev] = true;
    }
    hipLaunchKernelGGL((k_potrf_leaf16<T>), dim3((unsigned)batch), dim3(LEAF16_THREADS), lds_bytes, st, A, L, Inv, info,
                       info_off, batch, nb, zero_upper ? 1 : 0);
    return launch_check("potrf_leaf16");
}

template la_status launch_potrf_leaf16<float>(View<const float>, View<float>, View<float>, int32_t *, int, int64_t, int,
                                              bool, hipStream_t);
template la_status launch_potrf_leaf16<double>(View<const double>, View<double>, View<double>, int32_t *, int, int64_t,
                                               int, bool, hipStream_t);

}  // namespace la
