// Operators on many small matrices in lane groups (G = 4 .. 64 lanes of a wavefront per matrix, as in
// tiny.hip): trsm / trmm, syrk and the outer products of the trmm / trsm backward rules, gemm2, the syrk
// backward rule and potri (section 4.2 of arXiv 1710.08717 and its appendix).  Operands that are not
// square travel as flat memory images of whole items through LDS.  (Their forms with two rows per lane
// for 16 < n <= 32 are in tiny_rows.hip; potri's is here.)
#include "tiny_stage.hpp"

namespace la {

// ---------------------------------------------------------------------------------
// trsm / trmm for n <= 64 and at most 16 vectors (section 4.2 "trsm", "trmm"), G lanes per matrix:
// lane i holds row i of M (M = Lam or Lam^T, whichever the operator applies) and row i of the
// n x m operand, registers = its m columns.  The operand travels as its flat memory image (n x m
// or, for right-side operators, m x n per item, items back to back): 16-byte loads into LDS,
// rows or columns picked out of LDS by the lanes, the result back the same way.
//   solve: with D = diag(M), M x = b  <=>  (D^-1 M) x = D^-1 b, unit diagonal; for k in solve order
//          b_i -= (m_ik / m_ii) b_k (i != k): ONE broadcast multiply-add per column and step, row k is
//          final when it is broadcast.  multiply: x_i = sum_k m_ik b_k.
// LDS index of image element e is e + e / 16, so that 16 lanes reading a column of a 16-wide image
// (stride 16) fall into different banks.
// ---------------------------------------------------------------------------------
constexpr int TRI_MC = 16;  // vectors per matrix, at most


template <typename T, int G, bool SOLVE>
__global__ __launch_bounds__(WAVE) void k_tri_tiny(View<const T> Lam, const T *Bin, T *Bout, int64_t batch, int n, int m,
                                                    int fwd, int img_tr, T alpha)
{
    using S = Stage<T, G>;
    using V4 = typename VecOf<T>::type;
    constexpr int VN = VecOf<T>::N;
    constexpr int MPW = S::MPW;
    constexpr int IMG = MPW * G * TRI_MC;  // image elements of one wavefront, at most
    __shared__ __align__(16) T sm[S::ELEMS];
    __shared__ __align__(16) T img[IMG + IMG / 16 + 4];
    const int lane = threadIdx.x;
    const int q = lane / G, i = lane % G;
    const int64_t b0 = (int64_t)blockIdx.x * MPW;
    const int cnt = (int)((batch - b0) < MPW ? (batch - b0) : MPW);  // items of this wavefront
    const int nm = n * m, tot = cnt * nm;

    // ---- the operand's image: vector loads when the wavefront has all its items ----
    const T *src = Bin + b0 * nm;
    // (every wavefront's chunk must start on a 16-byte boundary and hold whole vectors)
    const bool vec = (cnt == MPW) && ((MPW * nm) % VN == 0) && ((reinterpret_cast<uintptr_t>(Bin) & 15) == 0);
    if (vec) {
        constexpr int ITV = (IMG / VN + WAVE - 1) / WAVE;
        const int nvec = tot / VN;
        V4 v[ITV];
#pragma unroll
        for (int t = 0; t < ITV; ++t)
            if (t * WAVE + lane < nvec)
                v[t] = __builtin_nontemporal_load(reinterpret_cast<const V4 *>(src) + t * WAVE + lane);
#pragma unroll
        for (int t = 0; t < ITV; ++t)
            if (t * WAVE + lane < nvec) {
                const int e = (t * WAVE + lane) * VN;
                img[img_idx(e)] = v[t].x;
                img[img_idx(e + 1)] = v[t].y;
                if constexpr (VN == 4) {
                    img[img_idx(e + 2)] = v[t].z;
                    img[img_idx(e + 3)] = v[t].w;
                }
            }
    } else {
        for (int e = lane; e < tot; e += WAVE)
            img[img_idx(e)] = src[e];
    }
    const Mem<const T> Lm = mem_of(Lam);
    stage_load<T, G>(sm, Lm, b0, batch, n);
    __syncthreads();

    // ---- row i of M and of the operand ----
    T mr[G];
    if (fwd)
        read_lrow<T, G>(sm + q * S::MS, i, Lm.tr, mr);  // M = Lam: entries k <= i
    else
        read_lcol<T, G>(sm + q * S::MS, i, Lm.tr, mr);  // M = Lam^T: entries k >= i
    T dii = T(1);
#pragma unroll
    for (int k = 0; k < G; ++k) {
        if (k == i)
            dii = mr[k];
        if (fwd ? (k > i) : (k < i))
            mr[k] = T(0);  // the other triangle is never used
    }
    T b[TRI_MC];
    const bool live = (i < n) && (q < cnt);
    const int ebase = q * nm + (img_tr ? i : i * m), estep = img_tr ? n : 1;
#pragma unroll
    for (int c = 0; c < TRI_MC; ++c)
        b[c] = (live && c < m) ? img[img_idx(ebase + c * estep)] : T(0);

    if constexpr (SOLVE) {
        const T rinv = rcp_acc(dii);
#pragma unroll
        for (int k = 0; k < G; ++k)
            mr[k] = (k == i) ? T(0) : mr[k] * rinv;
        const T sc = rinv * alpha;
#pragma unroll
        for (int c = 0; c < TRI_MC; ++c)
            b[c] *= sc;
        dpp_settle<G>(b);
        static_for<0, TRI_MC / 4>([&](auto CB) {
            constexpr int c0 = 4 * decltype(CB)::value;
            if (c0 < m) {
                static_for<0, G>([&](auto Kk) {
                    constexpr int kk = decltype(Kk)::value;
                    // forward: k = 0, 1, ...; backward: k = G-1, G-2, ... (rows >= n are identity padding)
                    if (fwd) {
                        static_for<0, 4>([&](auto J) { fma_bcast_self<G, kk>(b[c0 + decltype(J)::value], mr[kk], true); });
                    } else {
                        static_for<0, 4>([&](auto J) {
                            fma_bcast_self<G, G - 1 - kk>(b[c0 + decltype(J)::value], mr[G - 1 - kk], true);
                        });
                    }
                });
            }
        });
    } else {
        T x[TRI_MC];
#pragma unroll
        for (int c = 0; c < TRI_MC; ++c)
            x[c] = T(0);
        dpp_settle<G>(b);
        static_for<0, TRI_MC / 4>([&](auto CB) {
            constexpr int c0 = 4 * decltype(CB)::value;
            if (c0 < m) {
                static_for<0, G>([&](auto Kk) {
                    constexpr int kk = decltype(Kk)::value;
                    static_for<0, 4>([&](auto J) {
                        constexpr int c = c0 + decltype(J)::value;
                        fma_bcast<G, kk>(x[c], b[c], mr[kk], false);
                    });
                });
            }
        });
#pragma unroll
        for (int c = 0; c < TRI_MC; ++c)
            b[c] = alpha * x[c];
    }

    // ---- result into the image, image back to memory ----
    __syncthreads();
#pragma unroll
    for (int c = 0; c < TRI_MC; ++c)
        if (live && c < m)
            img[img_idx(ebase + c * estep)] = b[c];
    __syncthreads();
    T *dst = Bout + b0 * nm;
    if (vec && (reinterpret_cast<uintptr_t>(Bout) & 15) == 0) {
        constexpr int ITV = (IMG / VN + WAVE - 1) / WAVE;
        const int nvec = tot / VN;
#pragma unroll
        for (int t = 0; t < ITV; ++t)
            if (t * WAVE + lane < nvec) {
                const int e = (t * WAVE + lane) * VN;
                V4 v;
                v.x = img[img_idx(e)];
                v.y = img[img_idx(e + 1)];
                if constexpr (VN == 4) {
                    v.z = img[img_idx(e + 2)];
                    v.w = img[img_idx(e + 3)];
                }
                __builtin_nontemporal_store(v, reinterpret_cast<V4 *>(dst) + t * WAVE + lane);
            }
    } else {
        for (int e = lane; e < tot; e += WAVE)
            dst[e] = img[img_idx(e)];
    }
}

template <typename T, int G>
static la_status launch_tri_tiny_g(bool solve, View<const T> Lam, const T *Bin, T *Bout, int64_t batch, int n, int m,
                                   bool fwd, bool img_tr, T alpha, hipStream_t st)
{
    constexpr int MPW = Stage<T, G>::MPW;
    const dim3 grid((unsigned)((batch + MPW - 1) / MPW));
    if (solve)
        LA_LAUNCH((k_tri_tiny<T, G, true>), grid, dim3(WAVE), 0, st, Lam, Bin, Bout, batch, n, m, fwd ? 1 : 0,
                           img_tr ? 1 : 0, alpha);
    else
        LA_LAUNCH((k_tri_tiny<T, G, false>), grid, dim3(WAVE), 0, st, Lam, Bin, Bout, batch, n, m, fwd ? 1 : 0,
                           img_tr ? 1 : 0, alpha);
    return launch_check("tri_tiny");
}

// Bin / Bout: items of n * m elements back to back; img_tr says an item is stored m x n (the
// right-side operators) instead of n x m.
template <typename T>
la_status launch_tri_tiny(bool solve, bool fwd, T alpha, int64_t batch, int n, int m, View<const T> Lam, const T *Bin,
                          T *Bout, bool img_tr, hipStream_t st)
{
    if (batch <= 0 || n <= 0 || m <= 0)
        return LA_OK;
    if (n > 64 || m > TRI_MC || batch > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    if (n <= 4)
        return launch_tri_tiny_g<T, 4>(solve, Lam, Bin, Bout, batch, n, m, fwd, img_tr, alpha, st);
    if (n <= 8)
        return launch_tri_tiny_g<T, 8>(solve, Lam, Bin, Bout, batch, n, m, fwd, img_tr, alpha, st);
    if (n <= 16)
        return launch_tri_tiny_g<T, 16>(solve, Lam, Bin, Bout, batch, n, m, fwd, img_tr, alpha, st);
    if (n <= 32)  // broadcasts through ds_bpermute
        return launch_tri_tiny_g<T, 32>(solve, Lam, Bin, Bout, batch, n, m, fwd, img_tr, alpha, st);
    return launch_tri_tiny_g<T, 64>(solve, Lam, Bin, Bout, batch, n, m, fwd, img_tr, alpha, st);  // v_readlane
}

template la_status launch_tri_tiny<float>(bool, bool, float, int64_t, int, int, View<const float>, const float *, float *,
                                          bool, hipStream_t);
template la_status launch_tri_tiny<double>(bool, bool, double, int64_t, int, int, View<const double>, const double *,
                                           double *, bool, hipStream_t);

// ---------------------------------------------------------------------------------
// syrk for n <= 16 and inner dimension <= 32 (section 4.2 "syrk"), G lanes per matrix: lane i holds
// row i of the n x k operand (column i of the k x n one when trans), b_ij = sum_c a_ic a_jc with
// a_jc broadcast from lane j.  Lane i and lane j form the same products in the same order, so the
// result is exactly symmetric.  Operand in as its flat image (as in k_tri_tiny), result out through
// the padded stage.
// ---------------------------------------------------------------------------------
constexpr int SYRK_KC = 32;

// C = alpha U V^T for n x k operands U, V (V == U: syrk); tri = 0 writes the whole square, 1 / 2 keep
// the lower / upper triangle and write zeros to the other one (the gradient of a triangular
// operand in the trmm / trsm backward rules, section 4.2).
template <typename T, int G, bool TWO>
__global__ __launch_bounds__(WAVE) void k_syrk_tiny(const T *Uin, const T *Vin, View<T> C, int64_t batch, int n, int k,
                                                     int img_tr, int tri, T alpha)
{
    using S = Stage<T, G>;
    constexpr int MPW = S::MPW;
    constexpr int IMG = MPW * G * SYRK_KC;
    const int imgp = (MPW * n * k * 17 / 16 + 4 + 3) / 4 * 4;  // image of this n, k with its padding, a multiple of 16 bytes
    extern __shared__ __align__(16) unsigned char tiny_lds[];
    // the result's stage overlays the images: they are dead (in registers) by the time it is written
    T *sm = reinterpret_cast<T *>(tiny_lds), *img = sm, *img2 = img + imgp;  // img2 only when V != U
    const int lane = threadIdx.x;
    const int q = lane / G, i = lane % G;
    const int64_t b0 = (int64_t)blockIdx.x * MPW;
    const int cnt = (int)((batch - b0) < MPW ? (batch - b0) : MPW);
    const int nk = n * k;
    image_load<T, IMG, MPW>(img, Uin, b0, cnt, nk, lane);
    if constexpr (TWO)
        image_load<T, IMG, MPW>(img2, Vin, b0, cnt, nk, lane);
    __syncthreads();

    T a[SYRK_KC], v[TWO ? SYRK_KC : 1];
    const bool live = (i < n) && (q < cnt);
    const int ebase = q * nk + (img_tr ? i : i * k), estep = img_tr ? n : 1;
#pragma unroll
    for (int c = 0; c < SYRK_KC; ++c)
        a[c] = (live && c < k) ? img[img_idx(ebase + c * estep)] : T(0);
    if constexpr (TWO) {
#pragma unroll
        for (int c = 0; c < SYRK_KC; ++c)
            v[c] = (live && c < k) ? img2[img_idx(ebase + c * estep)] : T(0);
        dpp_settle<G>(v);
    } else {
        dpp_settle<G>(a);
    }
    T out[G];
#pragma unroll
    for (int j = 0; j < G; ++j)
        out[j] = T(0);
    static_for<0, G>([&](auto Jj) {
        constexpr int j = decltype(Jj)::value;
        if (j < n) {
            static_for<0, SYRK_KC / 4>([&](auto CB) {
                constexpr int c0 = 4 * decltype(CB)::value;
                if (c0 < k) {
                    static_for<0, 4>([&](auto U) {
                        constexpr int c = c0 + decltype(U)::value;
                        if constexpr (TWO)
                            fma_bcast<G, j>(out[j], v[c], a[c], false);  // u_ic v_jc
                        else
                            fma_bcast<G, j>(out[j], a[c], a[c], false);
                    });
                }
            });
        }
    });
#pragma unroll
    for (int j = 0; j < G; ++j) {
        const bool keep = tri == 0 || (tri == 1 ? j <= i : j >= i);
        out[j] = keep ? out[j] * alpha : T(0);
    }
    __syncthreads();
    write_row<T, G>(sm + q * S::MS, i, out);
    __syncthreads();
    stage_store<T, G>(sm, Mem<T>{C.p, C.bs, C.rs, false}, b0, batch, n);
}

template <typename T>
la_status launch_outer_tiny(bool img_tr, int tri, T alpha, int64_t batch, int n, int k, const T *U, const T *V, View<T> C,
                            hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    if (n > 16 || k > SYRK_KC || k < 1 || (batch + 3) / 4 > 0x7fffffffll || C.cs != 1)
        return LA_ERR_UNSUPPORTED;
    const int images = (U == V) ? 1 : 2;
    auto lds = [&](int g, int elems) {  // stage + images, as laid out in the kernel
        const int imgp = ((64 / g) * n * k * 17 / 16 + 4 + 3) / 4 * 4, smp = (elems + 3) / 4 * 4;
        return (size_t)(smp > images * imgp ? smp : images * imgp) * sizeof(T);
    };
    const dim3 blk(WAVE);
    const int itr = img_tr ? 1 : 0;
#define LA_SYRK_TINY(GG)                                                                                                  \
    do {                                                                                                                  \
        constexpr int MPW = Stage<T, GG>::MPW;                                                                            \
        const dim3 grid((unsigned)((batch + MPW - 1) / MPW));                                                             \
        if (images == 2)                                                                                                  \
            LA_LAUNCH((k_syrk_tiny<T, GG, true>), grid, blk, lds(GG, Stage<T, GG>::ELEMS), st, U, V, C, batch, n, \
                               k, itr, tri, alpha);                                                                       \
        else                                                                                                              \
            LA_LAUNCH((k_syrk_tiny<T, GG, false>), grid, blk, lds(GG, Stage<T, GG>::ELEMS), st, U, V, C, batch,   \
                               n, k, itr, tri, alpha);                                                                    \
    } while (0)
    if (n <= 4)
        LA_SYRK_TINY(4);
    else if (n <= 8)
        LA_SYRK_TINY(8);
    else
        LA_SYRK_TINY(16);
#undef LA_SYRK_TINY
    return launch_check("syrk_tiny");
}

template <typename T>
la_status launch_syrk_tiny(bool img_tr, T alpha, int64_t batch, int n, int k, const T *A, View<T> C, hipStream_t st)
{
    return launch_outer_tiny<T>(img_tr, 0, alpha, batch, n, k, A, A, C, st);
}

template la_status launch_outer_tiny<float>(bool, int, float, int64_t, int, int, const float *, const float *, View<float>,
                                            hipStream_t);
template la_status launch_outer_tiny<double>(bool, int, double, int64_t, int, int, const double *, const double *,
                                             View<double>, hipStream_t);
template la_status launch_syrk_tiny<float>(bool, float, int64_t, int, int, const float *, View<float>, hipStream_t);
template la_status launch_syrk_tiny<double>(bool, double, int64_t, int, int, const double *, View<double>, hipStream_t);

// ---------------------------------------------------------------------------------
// gemm2 for m, n, k <= 16 (section 4.2 "gemm2"): C = alpha op(A) op(B), G >= max(m, k) lanes per
// item.  Lane i holds row i of op(A) (k registers) and row i of op(B) (n registers);
// c_ij = sum_c a_ic b_cj with b_cj broadcast from lane c.  All three operands travel as flat images.
// ---------------------------------------------------------------------------------
constexpr int GEMM2_MC = 16;

template <typename T, int G>
__global__ __launch_bounds__(WAVE) void k_gemm2_tiny(const T *A, const T *B, T *C, int64_t batch, int m, int n, int k,
                                                      int ta, int tb, T alpha)
{
    constexpr int MPW = WAVE / G;
    constexpr int IMG = MPW * G * GEMM2_MC;
    __shared__ __align__(16) T imga[IMG + IMG / 16 + 4];
    __shared__ __align__(16) T imgb[IMG + IMG / 16 + 4];
    const int lane = threadIdx.x;
    const int q = lane / G, i = lane % G;
    const int64_t b0 = (int64_t)blockIdx.x * MPW;
    const int cnt = (int)((batch - b0) < MPW ? (batch - b0) : MPW);
    image_load<T, IMG, MPW>(imga, A, b0, cnt, m * k, lane);
    image_load<T, IMG, MPW>(imgb, B, b0, cnt, k * n, lane);
    __syncthreads();
    T a[G], br[GEMM2_MC], out[GEMM2_MC];
    const bool la_ = (q < cnt) && (i < m), lb = (q < cnt) && (i < k);
    const int ea = q * m * k + (ta ? i : i * k), sa = ta ? m : 1;  // op(A)(i, c)
    const int eb = q * k * n + (tb ? i : i * n), sb = tb ? k : 1;  // op(B)(i, j)
#pragma unroll
    for (int c = 0; c < G; ++c)
        a[c] = (la_ && c < k) ? imga[img_idx(ea + c * sa)] : T(0);
#pragma unroll
    for (int j = 0; j < GEMM2_MC; ++j) {
        br[j] = (lb && j < n) ? imgb[img_idx(eb + j * sb)] : T(0);
        out[j] = T(0);
    }
    dpp_settle<G>(br);
    static_for<0, G>([&](auto Cc) {
        constexpr int c = decltype(Cc)::value;
        if (c < k) {
            static_for<0, GEMM2_MC / 4>([&](auto JB) {
                constexpr int j0 = 4 * decltype(JB)::value;
                if (j0 < n) {
                    static_for<0, 4>([&](auto U) {
                        constexpr int j = j0 + decltype(U)::value;
                        fma_bcast<G, c>(out[j], br[j], a[c], false);
                    });
                }
            });
        }
    });
    __syncthreads();
    const int ec = q * m * n + i * n;
#pragma unroll
    for (int j = 0; j < GEMM2_MC; ++j)
        if (la_ && j < n)
            imga[img_idx(ec + j)] = alpha * out[j];
    __syncthreads();
    image_store<T, IMG, MPW>(imga, C, b0, cnt, m * n, lane);
}

template <typename T>
la_status launch_gemm2_tiny(int ta, int tb, T alpha, int64_t batch, int m, int n, int k, const T *A, const T *B, T *C,
                            hipStream_t st)
{
    if (batch <= 0 || m <= 0 || n <= 0)
        return LA_OK;
    if (m > 16 || n > GEMM2_MC || k > 16 || k < 1 || (batch + 3) / 4 > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    const int d = m > k ? m : k;
    if (d <= 4)
        LA_LAUNCH((k_gemm2_tiny<T, 4>), dim3((unsigned)((batch + 15) / 16)), dim3(WAVE), 0, st, A, B, C, batch, m, n,
                           k, ta, tb, alpha);
    else if (d <= 8)
        LA_LAUNCH((k_gemm2_tiny<T, 8>), dim3((unsigned)((batch + 7) / 8)), dim3(WAVE), 0, st, A, B, C, batch, m, n, k,
                           ta, tb, alpha);
    else
        LA_LAUNCH((k_gemm2_tiny<T, 16>), dim3((unsigned)((batch + 3) / 4)), dim3(WAVE), 0, st, A, B, C, batch, m, n,
                           k, ta, tb, alpha);
    return launch_check("gemm2_tiny");
}

template la_status launch_gemm2_tiny<float>(int, int, float, int64_t, int, int, int, const float *, const float *, float *,
                                            hipStream_t);
template la_status launch_gemm2_tiny<double>(int, int, double, int64_t, int, int, int, const double *, const double *,
                                             double *, hipStream_t);

// ---------------------------------------------------------------------------------
// syrk backward for n <= 16 and inner dimension <= 32 (section 4.2 "syrk"):
//   Abar = alpha (Bbar + Bbar^T) A   (A n x k; for the k x n operand of the transposed form the same
//   on its transposed image).  Lane i holds row i of S = Bbar + Bbar^T (row + column i of the staged
// Bbar) and row i of A; abar_ic = alpha sum_j s_ij a_jc with a_jc broadcast from lane j.
// ---------------------------------------------------------------------------------
template <typename T, int G>
__global__ __launch_bounds__(WAVE) void k_symm_tiny(View<const T> Gb, const T *Ain, T *Out, int64_t batch, int n, int k,
                                                     int img_tr, T alpha)
{
    using S = Stage<T, G>;
    constexpr int MPW = S::MPW;
    constexpr int IMG = MPW * G * SYRK_KC;
    __shared__ __align__(16) T sm[S::ELEMS];
    __shared__ __align__(16) T img[IMG + IMG / 16 + 4];
    const int lane = threadIdx.x;
    const int q = lane / G, i = lane % G;
    const int64_t b0 = (int64_t)blockIdx.x * MPW;
    const int cnt = (int)((batch - b0) < MPW ? (batch - b0) : MPW);
    const int nk = n * k;
    image_load<T, IMG, MPW>(img, Ain, b0, cnt, nk, lane);
    stage_load<T, G>(sm, mem_of(Gb), b0, batch, n);
    __syncthreads();
    T sr[G], sc[G];
    read_row<T, G>(sm + q * S::MS, i, sr);
    read_col<T, G>(sm + q * S::MS, i, sc);
#pragma unroll
    for (int j = 0; j < G; ++j)
        sr[j] += sc[j];
    T a[SYRK_KC], out[SYRK_KC];
    const bool live = (i < n) && (q < cnt);
    const int ebase = q * nk + (img_tr ? i : i * k), estep = img_tr ? n : 1;
#pragma unroll
    for (int c = 0; c < SYRK_KC; ++c) {
        a[c] = (live && c < k) ? img[img_idx(ebase + c * estep)] : T(0);
        out[c] = T(0);
    }
    dpp_settle<G>(a);
    static_for<0, G>([&](auto Jj) {
        constexpr int j = decltype(Jj)::value;
        if (j < n) {
            static_for<0, SYRK_KC / 4>([&](auto CB) {
                constexpr int c0 = 4 * decltype(CB)::value;
                if (c0 < k) {
                    static_for<0, 4>([&](auto U) {
                        constexpr int c = c0 + decltype(U)::value;
                        fma_bcast<G, j>(out[c], a[c], sr[j], false);
                    });
                }
            });
        }
    });
    __syncthreads();
#pragma unroll
    for (int c = 0; c < SYRK_KC; ++c)
        if (live && c < k)
            img[img_idx(ebase + c * estep)] = alpha * out[c];
    __syncthreads();
    image_store<T, IMG, MPW>(img, Out, b0, cnt, nk, lane);
}

template <typename T>
la_status launch_symm_tiny(bool img_tr, T alpha, int64_t batch, int n, int k, View<const T> Gb, const T *A, T *Out,
                           hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    if (n > 16 || k > SYRK_KC || k < 1 || (batch + 3) / 4 > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    const int itr = img_tr ? 1 : 0;
    if (n <= 4)
        LA_LAUNCH((k_symm_tiny<T, 4>), dim3((unsigned)((batch + 15) / 16)), dim3(WAVE), 0, st, Gb, A, Out, batch, n, k,
                           itr, alpha);
    else if (n <= 8)
        LA_LAUNCH((k_symm_tiny<T, 8>), dim3((unsigned)((batch + 7) / 8)), dim3(WAVE), 0, st, Gb, A, Out, batch, n, k,
                           itr, alpha);
    else
        LA_LAUNCH((k_symm_tiny<T, 16>), dim3((unsigned)((batch + 3) / 4)), dim3(WAVE), 0, st, Gb, A, Out, batch, n, k,
                           itr, alpha);
    return launch_check("symm_tiny");
}

template la_status launch_symm_tiny<float>(bool, float, int64_t, int, int, View<const float>, const float *, float *,
                                           hipStream_t);
template la_status launch_symm_tiny<double>(bool, double, int64_t, int, int, View<const double>, const double *, double *,
                                            hipStream_t);

// ---------------------------------------------------------------------------------
// potri for n <= 16 (section 4.2 "potri": A^-1 from the factor by two triangular solves), G lanes
// per matrix, both solves of k_tri_tiny on the identity in registers:
//   X = Lam^-1,  B = Lam^-T X;  the upper triangle of B is then taken from the lower one through
// the stage (exactly symmetric result).
// ---------------------------------------------------------------------------------
template <typename T, int G>
__global__ __launch_bounds__(WAVE) void k_potri_tiny(View<const T> Lam, View<T> B, int64_t batch, int n)
{
    using S = Stage<T, G>;
    __shared__ __align__(16) T sm[S::ELEMS];
    const int lane = threadIdx.x;
    const int q = lane / G, i = lane % G;
    const int64_t b0 = (int64_t)blockIdx.x * S::MPW;
    T *smq = sm + q * S::MS;
    const Mem<const T> Lm = mem_of(Lam);
    stage_load<T, G>(sm, Lm, b0, batch, n);
    __syncthreads();
    T m1[G], m2[G];  // row i of Lam, row i of Lam^T
    read_lrow<T, G>(smq, i, Lm.tr, m1);
    read_lcol<T, G>(smq, i, Lm.tr, m2);
    T dii = T(1);
#pragma unroll
    for (int k = 0; k < G; ++k)
        if (k == i)
            dii = m1[k];
    const T rinv = rcp_acc(dii);
#pragma unroll
    for (int k = 0; k < G; ++k) {
        m1[k] = (k < i) ? m1[k] * rinv : T(0);
        m2[k] = (k > i) ? m2[k] * rinv : T(0);
    }
    T b[G];
#pragma unroll
    for (int c = 0; c < G; ++c)
        b[c] = (c == i) ? rinv : T(0);
    dpp_settle<G>(b);
    static_for<0, G / 4>([&](auto CB) {
        constexpr int c0 = 4 * decltype(CB)::value;
        static_for<0, G>([&](auto Kk) {
            constexpr int kk = decltype(Kk)::value;
            static_for<0, 4>([&](auto J) { fma_bcast_self<G, kk>(b[c0 + decltype(J)::value], m1[kk], true); });
        });
    });
#pragma unroll
    for (int c = 0; c < G; ++c)
        b[c] *= rinv;
    dpp_settle<G>(b);
    static_for<0, G / 4>([&](auto CB) {
        constexpr int c0 = 4 * decltype(CB)::value;
        static_for<0, G>([&](auto Kk) {
            constexpr int kk = G - 1 - decltype(Kk)::value;
            static_for<0, 4>([&](auto J) { fma_bcast_self<G, kk>(b[c0 + decltype(J)::value], m2[kk], true); });
        });
    });
    __syncthreads();
    write_row<T, G>(smq, i, b);
    __syncthreads();
    T bt[G];
    read_col<T, G>(smq, i, bt);
#pragma unroll
    for (int c = 0; c < G; ++c)
        b[c] = (c <= i) ? b[c] : bt[c];
    __syncthreads();
    write_row<T, G>(smq, i, b);
    __syncthreads();
    stage_store<T, G>(sm, mem_of(B), b0, batch, n);  // symmetric: orientation is immaterial
}

// ---------------------------------------------------------------------------------
// potri for 16 < n <= 32 in 16 lanes per matrix: lane i owns the rows i and i + 16 (slot h = 0, 1) of the
// factor and of the result, so every broadcast is a DPP row broadcast; row k = 16 kh + kl lives in slot kh
// of lane kl.  Same two substitutions as k_potri_tiny, restricted to the columns that can be non-zero
// (Lam^-1 is lower triangular) or that are kept (the lower triangle of the symmetric result): row k takes
// part with its columns 0 .. k, in blocks of four.  N: the column count kept (24 or 32).
// ---------------------------------------------------------------------------------
template <typename T, int N>
__global__ __launch_bounds__(WAVE) void k_potri_tiny2(View<const T> Lam, View<T> B, int64_t batch, int n)
{
    constexpr int G = 16, MPW = WAVE / G;
    static_assert(N > G && N <= 2 * G && N % 4 == 0, "column count does not fit two row slots");
    using S = Stage<T, N, MPW>;
    __shared__ __align__(16) T sm[S::ELEMS];
    const int lane = threadIdx.x;
    const int q = lane / G, i = lane % G;
    const int64_t b0 = (int64_t)blockIdx.x * MPW;
    T *smq = sm + q * S::MS;
    const bool own1 = (N == 2 * G) || i + G < N;  // does row i + 16 exist among the N kept?
    const int i1 = own1 ? i + G : N - 1;
    const Mem<const T> Lm = mem_of(Lam);
    stage_load<T, N, MPW>(sm, Lm, b0, batch, n);  // identity outside n x n
    __syncthreads();

    // X = Lam^-1, rows r: x_r = (e_r - sum_{k < r} l_rk x_k) / l_rr
    T m0[N], m1[N];
    read_lrow<T, N>(smq, i, Lm.tr, m0);
    read_lrow<T, N>(smq, i1, Lm.tr, m1);
    T d0 = T(1), d1 = T(1);
#pragma unroll
    for (int k = 0; k < N; ++k) {
        if (k == i)
            d0 = m0[k];
        if (own1 && k == i + G)
            d1 = m1[k];
    }
    const T r0 = rcp_acc(d0), r1 = rcp_acc(d1);
    T x0[N], x1[N];
#pragma unroll
    for (int k = 0; k < N; ++k) {
        m0[k] = (k < i) ? m0[k] * r0 : T(0);
        m1[k] = (own1 && k < i + G) ? m1[k] * r1 : T(0);
        x0[k] = (k == i) ? r0 : T(0);
        x1[k] = (own1 && k == i + G) ? r1 : T(0);
    }
    dpp_settle<G>(x0);
    dpp_settle<G>(x1);
    static_for<0, N>([&](auto Kk) {
        constexpr int kk = decltype(Kk)::value;
        constexpr int kl = kk % G, kh = kk / G;
        static_for<0, kk / 4 + 1>([&](auto CB) {
            constexpr int c0 = 4 * decltype(CB)::value;
            if constexpr (kh == 0) {  // row kk < 16 reaches the later rows of both slots
                static_for<0, 4>([&](auto J) {
                    constexpr int c = c0 + decltype(J)::value;
                    fma_bcast<G, kl>(x1[c], x0[c], m1[kk], true);
                });
                static_for<0, 4>([&](auto J) {
                    constexpr int c = c0 + decltype(J)::value;
                    fma_bcast<G, kl>(x0[c], x0[c], m0[kk], true);
                });
            } else {  // the rows 0 .. 15 have nothing in column kk >= 16
                static_for<0, 4>([&](auto J) {
                    constexpr int c = c0 + decltype(J)::value;
                    fma_bcast<G, kl>(x1[c], x1[c], m1[kk], true);
                });
            }
        });
    });

    // B = Lam^-T X, rows from the bottom: b_r = (x_r - sum_{k > r} l_kr b_k) / l_rr
    read_lcol<T, N>(smq, i, Lm.tr, m0);
    read_lcol<T, N>(smq, i1, Lm.tr, m1);
#pragma unroll
    for (int k = 0; k < N; ++k) {
        m0[k] = (k > i) ? m0[k] * r0 : T(0);
        m1[k] = (own1 && k > i + G) ? m1[k] * r1 : T(0);
        x0[k] *= r0;
        x1[k] *= r1;
    }
    dpp_settle<G>(x0);
    dpp_settle<G>(x1);
    static_for<0, N>([&](auto Kk) {
        constexpr int kk = N - 1 - decltype(Kk)::value;
        constexpr int kl = kk % G, kh = kk / G;
        static_for<0, kk / 4 + 1>([&](auto CB) {
            constexpr int c0 = 4 * decltype(CB)::value;
            if constexpr (kh == 1) {  // row kk >= 16 reaches the earlier rows of both slots
                static_for<0, 4>([&](auto J) {
                    constexpr int c = c0 + decltype(J)::value;
                    fma_bcast<G, kl>(x0[c], x1[c], m0[kk], true);
                });
                static_for<0, 4>([&](auto J) {
                    constexpr int c = c0 + decltype(J)::value;
                    fma_bcast<G, kl>(x1[c], x1[c], m1[kk], true);
                });
            } else {
                static_for<0, 4>([&](auto J) {
                    constexpr int c = c0 + decltype(J)::value;
                    fma_bcast<G, kl>(x0[c], x0[c], m0[kk], true);
                });
            }
        });
    });

    // the upper triangle from the lower one through the stage (exactly symmetric result)
    __syncthreads();
    write_row<T, N>(smq, i, x0);
    if (own1)
        write_row<T, N>(smq, i + G, x1);
    __syncthreads();
    read_col<T, N>(smq, i, m0);
    read_col<T, N>(smq, i1, m1);
#pragma unroll
    for (int c = 0; c < N; ++c) {
        x0[c] = (c <= i) ? x0[c] : m0[c];
        x1[c] = (c <= i + G) ? x1[c] : m1[c];
    }
    __syncthreads();
    write_row<T, N>(smq, i, x0);
    if (own1)
        write_row<T, N>(smq, i + G, x1);
    __syncthreads();
    stage_store<T, N, MPW>(sm, mem_of(B), b0, batch, n);  // symmetric: orientation is immaterial
}

template <typename T>
la_status launch_potri_tiny(View<const T> Lam, View<T> B, int64_t batch, int n, hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    if (n > 32 || (batch + 3) / 4 > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    if (n > 24) {
        LA_LAUNCH((k_potri_tiny2<T, 32>), dim3((unsigned)((batch + 3) / 4)), dim3(WAVE), 0, st, Lam, B, batch, n);
    } else if (n > 16) {
        LA_LAUNCH((k_potri_tiny2<T, 24>), dim3((unsigned)((batch + 3) / 4)), dim3(WAVE), 0, st, Lam, B, batch, n);
    } else if (n <= 4) {
        constexpr int MPW = Stage<T, 4>::MPW;
        LA_LAUNCH((k_potri_tiny<T, 4>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, Lam, B, batch, n);
    } else if (n <= 8) {
        constexpr int MPW = Stage<T, 8>::MPW;
        LA_LAUNCH((k_potri_tiny<T, 8>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, Lam, B, batch, n);
    } else {
        constexpr int MPW = Stage<T, 16>::MPW;
        LA_LAUNCH((k_potri_tiny<T, 16>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, Lam, B, batch, n);
    }
    return launch_check("potri_tiny");
}

template la_status launch_potri_tiny<float>(View<const float>, View<float>, int64_t, int, hipStream_t);
template la_status launch_potri_tiny<double>(View<const double>, View<double>, int64_t, int, hipStream_t);

}  // namespace la
