// Operators on many small matrices with 16 < n <= 32 in 16 lanes per matrix: lane i holds the rows i and
// i + 16 (row slot h = 0, 1) of every operand, so that all broadcasts are DPP row broadcasts fused into
// the multiply-adds (as in the kernels of tiny.hip with two rows per lane); four matrices per
// wavefront.  Row j = 16 jh + jl lives in slot jh of lane jl.  syrk and the outer products of the
// trmm / trsm backward rules, the syrk backward rule, gemm2, trsm / trmm (section 4.2 of arXiv 1710.08717
// and its appendix).  Operands that are not square travel as flat memory images through LDS; the long dimension
// is taken in passes of CH columns to bound the registers.
#include "tiny_stage.hpp"

namespace la {

constexpr int ROWS_G = 16, ROWS_MPW = WAVE / ROWS_G;
constexpr int ROWS_KMAX = 32;  // inner dimension (syrk, outer products, syrk backward), at most
constexpr int ROWS_CH = 8;     // columns per pass

// elements of the padded LDS image of ROWS_MPW items of `per` elements, a multiple of 16 bytes
static inline __host__ __device__ int rows_image_elems(int per) { return (ROWS_MPW * per * 17 / 16 + 4 + 3) / 4 * 4; }

// ---------------------------------------------------------------------------------
// C = alpha U V^T for n x k operands U, V (V == U: syrk), 16 < n <= N, k <= 32.  tri = 0 writes the whole
// square, 1 / 2 keep the lower / upper triangle and write zeros to the other one.  In the syrk case lane
// pairs form the same products in the same order, so the result is exactly symmetric.
// ---------------------------------------------------------------------------------
template <typename T, int N, bool TWO>
__global__ __launch_bounds__(WAVE) void k_syrk_rows(const T *Uin, const T *Vin, View<T> C, int64_t batch, int n, int k,
                                                    int img_tr, int tri, T alpha)
{
    constexpr int G = ROWS_G, MPW = ROWS_MPW, CH = ROWS_CH;
    constexpr int IMG = MPW * N * ROWS_KMAX;
    using S = Stage<T, N, MPW>;
    extern __shared__ __align__(16) unsigned char tiny_lds[];
    // the result's stage overlays the images: they are dead by the time it is written
    T *sm = reinterpret_cast<T *>(tiny_lds), *img = sm, *img2 = img + rows_image_elems(n * k);
    const int lane = threadIdx.x;
    const int q = lane / G, i = lane % G;
    const int64_t b0 = (int64_t)blockIdx.x * MPW;
    const int cnt = (int)((batch - b0) < MPW ? (batch - b0) : MPW);
    const int nk = n * k;
    image_load<T, IMG, MPW>(img, Uin, b0, cnt, nk, lane);
    if constexpr (TWO)
        image_load<T, IMG, MPW>(img2, Vin, b0, cnt, nk, lane);
    __syncthreads();

    const bool live0 = (i < n) && (q < cnt), live1 = (i + G < n) && (q < cnt);
    const int e0 = q * nk + (img_tr ? i : i * k), e1 = q * nk + (img_tr ? i + G : (i + G) * k), estep = img_tr ? n : 1;
    T o0[N], o1[N];
#pragma unroll
    for (int j = 0; j < N; ++j) {
        o0[j] = T(0);
        o1[j] = T(0);
    }
    static_for<0, ROWS_KMAX / CH>([&](auto CB) {
        constexpr int c0 = CH * decltype(CB)::value;
        if (c0 < k) {  // the same for all lanes
            T a0[CH], a1[CH], v0[TWO ? CH : 1], v1[TWO ? CH : 1];
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                a0[u] = (live0 && c0 + u < k) ? img[img_idx(e0 + (c0 + u) * estep)] : T(0);
                a1[u] = (live1 && c0 + u < k) ? img[img_idx(e1 + (c0 + u) * estep)] : T(0);
            }
            if constexpr (TWO) {
#pragma unroll
                for (int u = 0; u < CH; ++u) {
                    v0[u] = (live0 && c0 + u < k) ? img2[img_idx(e0 + (c0 + u) * estep)] : T(0);
                    v1[u] = (live1 && c0 + u < k) ? img2[img_idx(e1 + (c0 + u) * estep)] : T(0);
                }
                dpp_settle<G>(v0);
                dpp_settle<G>(v1);
            } else {
                dpp_settle<G>(a0);
                dpp_settle<G>(a1);
            }
            static_for<0, N>([&](auto Jj) {
                constexpr int j = decltype(Jj)::value;
                constexpr int jl = j % G, jh = j / G;
                if (j < n) {
                    static_for<0, CH>([&](auto U) {
                        constexpr int u = decltype(U)::value;
                        // c_rj += u_rc v_jc, v_jc from slot jh of lane jl
                        // (the broadcast operand is named register by register: a copy made for the asm
                        // statement would be written right before its DPP read)
                        if constexpr (TWO && jh == 0) {
                            fma_bcast<G, jl>(o0[j], v0[u], a0[u], false);
                            fma_bcast<G, jl>(o1[j], v0[u], a1[u], false);
                        } else if constexpr (TWO) {
                            fma_bcast<G, jl>(o0[j], v1[u], a0[u], false);
                            fma_bcast<G, jl>(o1[j], v1[u], a1[u], false);
                        } else if constexpr (jh == 0) {
                            fma_bcast<G, jl>(o0[j], a0[u], a0[u], false);
                            fma_bcast<G, jl>(o1[j], a0[u], a1[u], false);
                        } else {
                            fma_bcast<G, jl>(o0[j], a1[u], a0[u], false);
                            fma_bcast<G, jl>(o1[j], a1[u], a1[u], false);
                        }
                    });
                }
            });
        }
    });
#pragma unroll
    for (int j = 0; j < N; ++j) {
        const bool keep0 = tri == 0 || (tri == 1 ? j <= i : j >= i);
        const bool keep1 = tri == 0 || (tri == 1 ? j <= i + G : j >= i + G);
        o0[j] = keep0 ? o0[j] * alpha : T(0);
        o1[j] = keep1 ? o1[j] * alpha : T(0);
    }
    __syncthreads();
    write_row<T, N>(sm + q * S::MS, i, o0);
    if (N == 2 * G || i + G < N)
        write_row<T, N>(sm + q * S::MS, i + G, o1);
    __syncthreads();
    stage_store<T, N, MPW>(sm, Mem<T>{C.p, C.bs, C.rs, false}, b0, batch, n);
}

template <typename T>
static size_t syrk_rows_lds(int N, int n, int k, int images)
{
    const size_t stage = (size_t)(N == 24 ? Stage<T, 24, ROWS_MPW>::ELEMS : Stage<T, 32, ROWS_MPW>::ELEMS);
    const size_t imgs = (size_t)images * rows_image_elems(n * k);
    return (stage > imgs ? stage : imgs) * sizeof(T);
}

template <typename T>
bool outer_rows_takes(int n, int k, bool two)
{
    return n > 16 && n <= 32 && k >= 1 && k <= ROWS_KMAX && syrk_rows_lds<T>(n <= 24 ? 24 : 32, n, k, two ? 2 : 1) <= 64 * 1024;
}
template bool outer_rows_takes<float>(int, int, bool);
template bool outer_rows_takes<double>(int, int, bool);

template <typename T>
la_status launch_outer_rows(bool img_tr, int tri, T alpha, int64_t batch, int n, int k, const T *U, const T *V, View<T> C,
                            hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    if (!outer_rows_takes<T>(n, k, U != V) || (batch + 3) / 4 > 0x7fffffffll || C.cs != 1)
        return LA_ERR_UNSUPPORTED;
    const bool two = (U != V);
    const dim3 grid((unsigned)((batch + ROWS_MPW - 1) / ROWS_MPW)), blk(WAVE);
    const int itr = img_tr ? 1 : 0;
#define LA_SYRK_ROWS(NN, TW)                                                                                         \
    LA_LAUNCH((k_syrk_rows<T, NN, TW>), grid, blk, syrk_rows_lds<T>(NN, n, k, TW ? 2 : 1), st, U, V, C, batch, n, k, \
              itr, tri, alpha)
    if (n <= 24) {
        if (two)
            LA_SYRK_ROWS(24, true);
        else
            LA_SYRK_ROWS(24, false);
    } else {
        if (two)
            LA_SYRK_ROWS(32, true);
        else
            LA_SYRK_ROWS(32, false);
    }
#undef LA_SYRK_ROWS
    return launch_check("syrk_rows");
}

template la_status launch_outer_rows<float>(bool, int, float, int64_t, int, int, const float *, const float *, View<float>,
                                            hipStream_t);
template la_status launch_outer_rows<double>(bool, int, double, int64_t, int, int, const double *, const double *,
                                             View<double>, hipStream_t);


// raise the dynamic LDS limit of a kernel once per device (two images of fp64 operands exceed 64 KB)
template <class K>
static la_status rows_lds_limit(K kernel, size_t bytes, bool (&done)[64])
{
    int dev = 0;
    LA_HIP(hipGetDevice(&dev));
    if (dev >= 0 && dev < 64 && !done[dev]) {
        LA_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)bytes));
        done[dev] = true;
    }
    return LA_OK;
}

// ---------------------------------------------------------------------------------
// syrk backward for 16 < n <= N and inner dimension <= 32 (section 4.2 "syrk"):
//   Abar = alpha (Bbar + Bbar^T) A   (A n x k; for the k x n operand of the transposed form the same on
//   its transposed image).  Lane i holds the rows i, i + 16 of S = Bbar + Bbar^T (row + column of the
// staged Bbar); abar_rc = alpha sum_j s_rj a_jc with a_jc broadcast from slot jh of lane jl, CH columns c
// per pass, written back over the image of A.
// ---------------------------------------------------------------------------------
template <typename T, int N>
__global__ __launch_bounds__(WAVE) void k_symm_rows(View<const T> Gb, const T *Ain, T *Out, int64_t batch, int n, int k,
                                                    int img_tr, T alpha)
{
    constexpr int G = ROWS_G, MPW = ROWS_MPW, CH = ROWS_CH;
    constexpr int IMG = MPW * N * ROWS_KMAX;
    using S = Stage<T, N, MPW>;
    extern __shared__ __align__(16) unsigned char tiny_lds[];
    T *sm = reinterpret_cast<T *>(tiny_lds), *img = sm + (S::ELEMS + 3) / 4 * 4;
    const int lane = threadIdx.x;
    const int q = lane / G, i = lane % G;
    const int64_t b0 = (int64_t)blockIdx.x * MPW;
    const int cnt = (int)((batch - b0) < MPW ? (batch - b0) : MPW);
    const int nk = n * k;
    const bool own1 = (N == 2 * G) || i + G < N;
    const int i1 = own1 ? i + G : N - 1;
    image_load<T, IMG, MPW>(img, Ain, b0, cnt, nk, lane);
    stage_load<T, N, MPW>(sm, mem_of(Gb), b0, batch, n);
    __syncthreads();
    T s0[N], s1[N];
    {
        T t0[N], t1[N];
        read_row<T, N>(sm + q * S::MS, i, s0);
        read_col<T, N>(sm + q * S::MS, i, t0);
        read_row<T, N>(sm + q * S::MS, i1, s1);
        read_col<T, N>(sm + q * S::MS, i1, t1);
#pragma unroll
        for (int j = 0; j < N; ++j) {
            s0[j] += t0[j];
            s1[j] += t1[j];
        }
    }
    const bool live0 = (i < n) && (q < cnt), live1 = (i + G < n) && (q < cnt);
    const int e0 = q * nk + (img_tr ? i : i * k), e1 = q * nk + (img_tr ? i + G : (i + G) * k), estep = img_tr ? n : 1;
    static_for<0, ROWS_KMAX / CH>([&](auto CB) {
        constexpr int c0 = CH * decltype(CB)::value;
        if (c0 < k) {  // the same for all lanes
            T a0[CH], a1[CH], o0[CH], o1[CH];
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                a0[u] = (live0 && c0 + u < k) ? img[img_idx(e0 + (c0 + u) * estep)] : T(0);
                a1[u] = (live1 && c0 + u < k) ? img[img_idx(e1 + (c0 + u) * estep)] : T(0);
                o0[u] = T(0);
                o1[u] = T(0);
            }
            dpp_settle<G>(a0);
            dpp_settle<G>(a1);
            static_for<0, N>([&](auto Jj) {
                constexpr int j = decltype(Jj)::value;
                constexpr int jl = j % G, jh = j / G;
                if (j < n) {
                    static_for<0, CH>([&](auto U) {
                        constexpr int u = decltype(U)::value;
                        if constexpr (jh == 0) {
                            fma_bcast<G, jl>(o0[u], a0[u], s0[j], false);
                            fma_bcast<G, jl>(o1[u], a0[u], s1[j], false);
                        } else {
                            fma_bcast<G, jl>(o0[u], a1[u], s0[j], false);
                            fma_bcast<G, jl>(o1[u], a1[u], s1[j], false);
                        }
                    });
                }
            });
            // every lane holds its entries of these columns in registers: the image can take the result
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                if (live0 && c0 + u < k)
                    img[img_idx(e0 + (c0 + u) * estep)] = alpha * o0[u];
                if (live1 && c0 + u < k)
                    img[img_idx(e1 + (c0 + u) * estep)] = alpha * o1[u];
            }
        }
    });
    __syncthreads();
    image_store<T, IMG, MPW>(img, Out, b0, cnt, nk, lane);
}

template <typename T>
bool symm_rows_takes(int n, int k)
{
    return n > 16 && n <= 32 && k >= 1 && k <= ROWS_KMAX;
}
template bool symm_rows_takes<float>(int, int);
template bool symm_rows_takes<double>(int, int);

template <typename T>
la_status launch_symm_rows(bool img_tr, T alpha, int64_t batch, int n, int k, View<const T> Gb, const T *A, T *Out,
                           hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    if (!symm_rows_takes<T>(n, k) || (batch + 3) / 4 > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    if (dry_run())
        return LA_OK;
    const dim3 grid((unsigned)((batch + ROWS_MPW - 1) / ROWS_MPW)), blk(WAVE);
    const int itr = img_tr ? 1 : 0;
    auto bytes = [&](int stage_elems) { return ((size_t)(stage_elems + 3) / 4 * 4 + rows_image_elems(n * k)) * sizeof(T); };
    if (n <= 24) {
        constexpr int SE = Stage<T, 24, ROWS_MPW>::ELEMS;
        static bool done[64] = {};
        LA_TRY(rows_lds_limit(&k_symm_rows<T, 24>, ((size_t)(SE + 3) / 4 * 4 + rows_image_elems(24 * ROWS_KMAX)) * sizeof(T), done));
        LA_LAUNCH((k_symm_rows<T, 24>), grid, blk, bytes(SE), st, Gb, A, Out, batch, n, k, itr, alpha);
    } else {
        constexpr int SE = Stage<T, 32, ROWS_MPW>::ELEMS;
        static bool done[64] = {};
        LA_TRY(rows_lds_limit(&k_symm_rows<T, 32>, ((size_t)(SE + 3) / 4 * 4 + rows_image_elems(32 * ROWS_KMAX)) * sizeof(T), done));
        LA_LAUNCH((k_symm_rows<T, 32>), grid, blk, bytes(SE), st, Gb, A, Out, batch, n, k, itr, alpha);
    }
    return launch_check("symm_rows");
}

template la_status launch_symm_rows<float>(bool, float, int64_t, int, int, View<const float>, const float *, float *,
                                           hipStream_t);
template la_status launch_symm_rows<double>(bool, double, int64_t, int, int, View<const double>, const double *, double *,
                                            hipStream_t);

// ---------------------------------------------------------------------------------
// gemm2 with m, n, k <= 32 and one of them above 16 (section 4.2 "gemm2"): C = alpha op(A) op(B).  Lane i
// holds the rows i, i + 16 of op(A) (k registers each); c_rj = sum_c a_rc b_cj with b_cj broadcast from
// slot ch of lane cl, CH columns j of op(B) and C per pass.  All three operands travel as flat images;
// the image of C takes the place of that of A, which is in registers by then.
// ---------------------------------------------------------------------------------
constexpr int GEMM2R_MAX = 32;

template <typename T>
__global__ __launch_bounds__(WAVE) void k_gemm2_rows(const T *A, const T *B, T *C, int64_t batch, int m, int n, int k, int ta,
                                                     int tb, T alpha)
{
    constexpr int G = ROWS_G, MPW = ROWS_MPW, CH = ROWS_CH, MX = GEMM2R_MAX;
    constexpr int IMG = MPW * MX * MX;
    extern __shared__ __align__(16) unsigned char tiny_lds[];
    const int mk = m * k, kn = k * n, mn = m * n;
    T *imga = reinterpret_cast<T *>(tiny_lds), *imgb = imga + rows_image_elems(mk > mn ? mk : mn);
    const int lane = threadIdx.x;
    const int q = lane / G, i = lane % G;
    const int64_t b0 = (int64_t)blockIdx.x * MPW;
    const int cnt = (int)((batch - b0) < MPW ? (batch - b0) : MPW);
    image_load<T, IMG, MPW>(imga, A, b0, cnt, mk, lane);
    image_load<T, IMG, MPW>(imgb, B, b0, cnt, kn, lane);
    __syncthreads();
    const bool la0 = (q < cnt) && (i < m), la1 = (q < cnt) && (i + G < m);  // rows of op(A) and of C
    const bool lb0 = (q < cnt) && (i < k), lb1 = (q < cnt) && (i + G < k);  // rows of op(B)
    const int sa = ta ? m : 1, sb = tb ? k : 1;
    const int ea0 = q * mk + (ta ? i : i * k), ea1 = q * mk + (ta ? i + G : (i + G) * k);  // op(A)(r, c)
    const int eb0 = q * kn + (tb ? i : i * n), eb1 = q * kn + (tb ? i + G : (i + G) * n);  // op(B)(r, j)
    T a0[MX], a1[MX];
#pragma unroll
    for (int c = 0; c < MX; ++c) {
        a0[c] = (la0 && c < k) ? imga[img_idx(ea0 + c * sa)] : T(0);
        a1[c] = (la1 && c < k) ? imga[img_idx(ea1 + c * sa)] : T(0);
    }
    __syncthreads();  // the image of A is in registers: C may overwrite it
    const int ec0 = q * mn + i * n, ec1 = q * mn + (i + G) * n;
    static_for<0, MX / CH>([&](auto JB) {
        constexpr int j0 = CH * decltype(JB)::value;
        if (j0 < n) {  // the same for all lanes
            T r0[CH], r1[CH], o0[CH], o1[CH];
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                r0[u] = (lb0 && j0 + u < n) ? imgb[img_idx(eb0 + (j0 + u) * sb)] : T(0);
                r1[u] = (lb1 && j0 + u < n) ? imgb[img_idx(eb1 + (j0 + u) * sb)] : T(0);
                o0[u] = T(0);
                o1[u] = T(0);
            }
            dpp_settle<G>(r0);
            dpp_settle<G>(r1);
            static_for<0, MX>([&](auto Cc) {
                constexpr int c = decltype(Cc)::value;
                constexpr int cl = c % G, ch = c / G;
                if (c < k) {
                    static_for<0, CH>([&](auto U) {
                        constexpr int u = decltype(U)::value;
                        if constexpr (ch == 0) {
                            fma_bcast<G, cl>(o0[u], r0[u], a0[c], false);
                            fma_bcast<G, cl>(o1[u], r0[u], a1[c], false);
                        } else {
                            fma_bcast<G, cl>(o0[u], r1[u], a0[c], false);
                            fma_bcast<G, cl>(o1[u], r1[u], a1[c], false);
                        }
                    });
                }
            });
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                if (la0 && j0 + u < n)
                    imga[img_idx(ec0 + j0 + u)] = alpha * o0[u];
                if (la1 && j0 + u < n)
                    imga[img_idx(ec1 + j0 + u)] = alpha * o1[u];
            }
        }
    });
    __syncthreads();
    image_store<T, IMG, MPW>(imga, C, b0, cnt, mn, lane);
}

template <typename T>
bool gemm2_rows_takes(int m, int n, int k)
{
    return m >= 1 && n >= 1 && k >= 1 && m <= GEMM2R_MAX && n <= GEMM2R_MAX && k <= GEMM2R_MAX && (m > 16 || n > 16 || k > 16);
}
template bool gemm2_rows_takes<float>(int, int, int);
template bool gemm2_rows_takes<double>(int, int, int);

template <typename T>
la_status launch_gemm2_rows(int ta, int tb, T alpha, int64_t batch, int m, int n, int k, const T *A, const T *B, T *C,
                            hipStream_t st)
{
    if (batch <= 0 || m <= 0 || n <= 0)
        return LA_OK;
    if (!gemm2_rows_takes<T>(m, n, k) || (batch + 3) / 4 > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    if (dry_run())
        return LA_OK;
    static bool done[64] = {};
    LA_TRY(rows_lds_limit(&k_gemm2_rows<T>, 2 * (size_t)rows_image_elems(GEMM2R_MAX * GEMM2R_MAX) * sizeof(T), done));
    const int mk = m * k, mn = m * n;
    const size_t lds = ((size_t)rows_image_elems(mk > mn ? mk : mn) + rows_image_elems(k * n)) * sizeof(T);
    LA_LAUNCH((k_gemm2_rows<T>), dim3((unsigned)((batch + ROWS_MPW - 1) / ROWS_MPW)), dim3(WAVE), lds, st, A, B, C, batch, m, n,
              k, ta, tb, alpha);
    return launch_check("gemm2_rows");
}

template la_status launch_gemm2_rows<float>(int, int, float, int64_t, int, int, int, const float *, const float *, float *,
                                            hipStream_t);
template la_status launch_gemm2_rows<double>(int, int, double, int64_t, int, int, int, const double *, const double *,
                                             double *, hipStream_t);


// ---------------------------------------------------------------------------------
// trsm / trmm for 16 < n <= N and at most 16 vectors (section 4.2 "trsm", "trmm"): lane i holds the rows
// i, i + 16 of M (M = Lam or Lam^T, whichever the operator applies) and of the n x m operand, which
// travels as its flat image (n x m or, for the right-side operators, m x n per item).
//   solve: unit-diagonal form (D^-1 M) x = D^-1 b; in solve order b_r -= (m_rk / m_rr) b_k (r != k), one
//          broadcast multiply-add per column, row slot and step; row k is final when it is broadcast.
//   multiply: x_r = sum_k m_rk b_k.
// Steps that only meet structural zeros of the triangle in a row slot are left out.
// ---------------------------------------------------------------------------------
constexpr int TRIR_MC = 16;  // vectors per matrix, at most

template <typename T, int N, bool SOLVE>
__global__ __launch_bounds__(WAVE) void k_tri_rows(View<const T> Lam, const T *Bin, T *Bout, int64_t batch, int n, int m,
                                                   int fwd, int img_tr, T alpha)
{
    constexpr int G = ROWS_G, MPW = ROWS_MPW;
    constexpr int IMG = MPW * N * TRIR_MC;
    using S = Stage<T, N, MPW>;
    __shared__ __align__(16) T sm[S::ELEMS];
    __shared__ __align__(16) T img[IMG + IMG / 16 + 4];
    const int lane = threadIdx.x;
    const int q = lane / G, i = lane % G;
    const int64_t b0 = (int64_t)blockIdx.x * MPW;
    const int cnt = (int)((batch - b0) < MPW ? (batch - b0) : MPW);
    const int nm = n * m;
    const bool own1 = (N == 2 * G) || i + G < N;
    const int i1 = own1 ? i + G : N - 1;
    image_load<T, IMG, MPW>(img, Bin, b0, cnt, nm, lane);
    const Mem<const T> Lm = mem_of(Lam);
    stage_load<T, N, MPW>(sm, Lm, b0, batch, n);  // identity outside n x n
    __syncthreads();

    T m0[N], m1[N];
    if (fwd) {  // M = Lam: entries k <= r
        read_lrow<T, N>(sm + q * S::MS, i, Lm.tr, m0);
        read_lrow<T, N>(sm + q * S::MS, i1, Lm.tr, m1);
    } else {  // M = Lam^T: entries k >= r
        read_lcol<T, N>(sm + q * S::MS, i, Lm.tr, m0);
        read_lcol<T, N>(sm + q * S::MS, i1, Lm.tr, m1);
    }
    T d0 = T(1), d1 = T(1);
#pragma unroll
    for (int k = 0; k < N; ++k) {
        if (k == i)
            d0 = m0[k];
        if (own1 && k == i + G)
            d1 = m1[k];
        if (fwd ? (k > i) : (k < i))
            m0[k] = T(0);  // the other triangle is never used
        if (!own1 || (fwd ? (k > i + G) : (k < i + G)))
            m1[k] = T(0);
    }
    const bool live0 = (i < n) && (q < cnt), live1 = (i + G < n) && (q < cnt);
    const int e0 = q * nm + (img_tr ? i : i * m), e1 = q * nm + (img_tr ? i + G : (i + G) * m), estep = img_tr ? n : 1;
    T x0[TRIR_MC], x1[TRIR_MC];
#pragma unroll
    for (int c = 0; c < TRIR_MC; ++c) {
        x0[c] = (live0 && c < m) ? img[img_idx(e0 + c * estep)] : T(0);
        x1[c] = (live1 && c < m) ? img[img_idx(e1 + c * estep)] : T(0);
    }

    if constexpr (SOLVE) {
        const T r0 = rcp_acc(d0), r1 = rcp_acc(d1);
#pragma unroll
        for (int k = 0; k < N; ++k) {
            m0[k] = (k == i) ? T(0) : m0[k] * r0;
            m1[k] = (k == i + G) ? T(0) : m1[k] * r1;
        }
#pragma unroll
        for (int c = 0; c < TRIR_MC; ++c) {
            x0[c] *= r0 * alpha;
            x1[c] *= r1 * alpha;
        }
        dpp_settle<G>(x0);
        dpp_settle<G>(x1);
        static_for<0, TRIR_MC / 4>([&](auto CB) {
            constexpr int c0 = 4 * decltype(CB)::value;
            if (c0 < m) {
                static_for<0, N>([&](auto Kk) {
                    constexpr int kf = decltype(Kk)::value, kb = N - 1 - kf;  // forward: 0, 1, ...; backward: N-1, N-2, ...
                    if (fwd) {
                        constexpr int kl = kf % G;
                        if constexpr (kf < G) {  // row kf of slot 0 reaches the later rows of both slots
                            static_for<0, 4>([&](auto J) { fma_bcast<G, kl>(x1[c0 + decltype(J)::value], x0[c0 + decltype(J)::value], m1[kf], true); });
                            static_for<0, 4>([&](auto J) { fma_bcast<G, kl>(x0[c0 + decltype(J)::value], x0[c0 + decltype(J)::value], m0[kf], true); });
                        } else {
                            static_for<0, 4>([&](auto J) { fma_bcast<G, kl>(x1[c0 + decltype(J)::value], x1[c0 + decltype(J)::value], m1[kf], true); });
                        }
                    } else {
                        constexpr int kl = kb % G;
                        if constexpr (kb >= G) {  // row kb of slot 1 reaches the earlier rows of both slots
                            static_for<0, 4>([&](auto J) { fma_bcast<G, kl>(x0[c0 + decltype(J)::value], x1[c0 + decltype(J)::value], m0[kb], true); });
                            static_for<0, 4>([&](auto J) { fma_bcast<G, kl>(x1[c0 + decltype(J)::value], x1[c0 + decltype(J)::value], m1[kb], true); });
                        } else {
                            static_for<0, 4>([&](auto J) { fma_bcast<G, kl>(x0[c0 + decltype(J)::value], x0[c0 + decltype(J)::value], m0[kb], true); });
                        }
                    }
                });
            }
        });
    } else {
        dpp_settle<G>(x0);
        dpp_settle<G>(x1);
        static_for<0, TRIR_MC / 4>([&](auto CB) {
            constexpr int c0 = 4 * decltype(CB)::value;
            if (c0 < m) {
                T y0[4] = {T(0), T(0), T(0), T(0)}, y1[4] = {T(0), T(0), T(0), T(0)};
                static_for<0, N>([&](auto Kk) {
                    constexpr int kk = decltype(Kk)::value;
                    constexpr int kl = kk % G;
                    // lower M (forward): the rows 0 .. 15 end at column 15; upper M: the rows 16 .. start at column 16
                    if constexpr (kk < G) {
                        static_for<0, 4>([&](auto J) { fma_bcast<G, kl>(y0[decltype(J)::value], x0[c0 + decltype(J)::value], m0[kk], false); });
                        if (fwd)
                            static_for<0, 4>([&](auto J) { fma_bcast<G, kl>(y1[decltype(J)::value], x0[c0 + decltype(J)::value], m1[kk], false); });
                    } else {
                        if (!fwd)
                            static_for<0, 4>([&](auto J) { fma_bcast<G, kl>(y0[decltype(J)::value], x1[c0 + decltype(J)::value], m0[kk], false); });
                        static_for<0, 4>([&](auto J) { fma_bcast<G, kl>(y1[decltype(J)::value], x1[c0 + decltype(J)::value], m1[kk], false); });
                    }
                });
                // column c of the operand only feeds column c of the product: the block can be replaced now
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    x0[c0 + j] = alpha * y0[j];
                    x1[c0 + j] = alpha * y1[j];
                }
            }
        });
    }

    __syncthreads();
#pragma unroll
    for (int c = 0; c < TRIR_MC; ++c) {
        if (live0 && c < m)
            img[img_idx(e0 + c * estep)] = x0[c];
        if (live1 && c < m)
            img[img_idx(e1 + c * estep)] = x1[c];
    }
    __syncthreads();
    image_store<T, IMG, MPW>(img, Bout, b0, cnt, nm, lane);
}

// Bin / Bout: items of n * m elements back to back; img_tr says an item is stored m x n (the right-side
// operators) instead of n x m.
template <typename T>
la_status launch_tri_rows(bool solve, bool fwd, T alpha, int64_t batch, int n, int m, View<const T> Lam, const T *Bin, T *Bout,
                          bool img_tr, hipStream_t st)
{
    if (batch <= 0 || n <= 0 || m <= 0)
        return LA_OK;
    if (n <= 16 || n > 32 || m > TRIR_MC || (batch + 3) / 4 > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)((batch + ROWS_MPW - 1) / ROWS_MPW)), blk(WAVE);
    const int f = fwd ? 1 : 0, itr = img_tr ? 1 : 0;
#define LA_TRI_ROWS(NN, SV) LA_LAUNCH((k_tri_rows<T, NN, SV>), grid, blk, 0, st, Lam, Bin, Bout, batch, n, m, f, itr, alpha)
    if (n <= 24) {
        if (solve)
            LA_TRI_ROWS(24, true);
        else
            LA_TRI_ROWS(24, false);
    } else {
        if (solve)
            LA_TRI_ROWS(32, true);
        else
            LA_TRI_ROWS(32, false);
    }
#undef LA_TRI_ROWS
    return launch_check("tri_rows");
}

template la_status launch_tri_rows<float>(bool, bool, float, int64_t, int, int, View<const float>, const float *, float *, bool,
                                          hipStream_t);
template la_status launch_tri_rows<double>(bool, bool, double, int64_t, int, int, View<const double>, const double *, double *,
                                           bool, hipStream_t);

}  // namespace la
