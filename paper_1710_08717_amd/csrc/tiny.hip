// Register-resident kernels for small matrices: G lanes of a wavefront own one matrix
// (lane = row, registers = columns), so a wave64 works on 64/G matrices at once and the
// column reductions of the factorisation are lane broadcasts (DPP row broadcast for
// G = 16, LDS crossbar permute for G = 32, v_readlane for G = 64).
//
// potrf forward: section 4.2 of arXiv 1710.08717 (A = L L^T, positive diagonal).
// potrf backward: section 4.2 / appendix "potrf":
//   Abar = 1/2 L^-T copyltu(L^T Lbar) L^-1 = sym(L^-T Phi(L^T Lbar) L^-1),
//   Phi = lower triangle with halved diagonal (copyltu X = Phi X + (Phi X)^T).
//
// Global memory is only touched through coalesced passes that stage whole matrices in
// LDS; the lanes then pick rows or columns out of LDS, which is also how the transposed
// (upper-factor) views are served.
#include "common.hpp"
#include "tiny_stage.hpp"

namespace la {

// ---------------------------------------------------------------------------------
// potrf forward.  View A / L give the LOGICAL lower-triangular problem: A(i,j), i >= j,
// is read; L(i,j) is written for the whole nb x nb block (zeros for i < j).
// ---------------------------------------------------------------------------------
template <typename T, int G, int N = G>
__global__ __launch_bounds__(WAVE) void k_potrf_tiny(View<const T> A, View<T> L, int32_t *info, int info_off,
                                                      int64_t batch, int nb)
{
    // G lanes per matrix, N <= G columns kept: a lane group that the matrix does not fill (n = 12 in
    // 16 lanes) stages and eliminates N columns only; its lanes i >= N follow row N - 1 and write nothing.
    constexpr int MPW = WAVE / G;
    using S = Stage<T, N, MPW>;
    __shared__ __align__(16) T sm[S::ELEMS];
    const int lane = threadIdx.x;
    const int q = lane / G, i = lane % G;
    const int ir = (N < G && i >= N) ? N - 1 : i;
    const int64_t b0 = (int64_t)blockIdx.x * MPW;

    const Mem<const T> Am = mem_of(A);
    const Mem<T> Lm = mem_of(L);
    stage_load<T, N, MPW>(sm, Am, b0, batch, nb);
    __syncthreads();
    T a[N];
    read_lrow<T, N>(sm + q * S::MS, ir, Am.tr, a);
#pragma unroll
    for (int k = 0; k < N; ++k)
        if (k > i)
            a[k] = T(0);  // the other triangle of A is never used

    int fail = 0;
    static_for<0, N>([&](auto J) {
        constexpr int j = decltype(J)::value;
        T piv = group_bcast<G>(a[j], j);  // a_jj after the updates of columns < j
        if (!(piv > T(0)) && fail == 0)
            fail = j + 1;
        T r = rsqrt_acc(piv);
        a[j] = (i >= j) ? a[j] * r : T(0);  // column j of L (lane j gets sqrt(piv))
        dpp_settle1<G>(a[j]);
        static_for<j + 1, N>([&](auto K) {
            constexpr int k = decltype(K)::value;
            fma_bcast<G, k>(a[k], a[j], a[j], true);  // a_ik -= l_ij l_kj
        });
    });
#pragma unroll
    for (int k = 0; k < N; ++k)
        if (k > i)
            a[k] = T(0);

    __syncthreads();
    if (N == G || i < N) {
        if (Lm.tr)
            write_col<T, N>(sm + q * S::MS, i, a);
        else
            write_row<T, N>(sm + q * S::MS, i, a);
    }
    __syncthreads();
    stage_store<T, N, MPW>(sm, Lm, b0, batch, nb);
    if (info != nullptr && i == 0 && b0 + q < batch && fail != 0 && fail <= nb) {
        if (info[b0 + q] == 0)
            info[b0 + q] = info_off + fail;
    }
}

// ---------------------------------------------------------------------------------
// potrf forward for 16 < n <= 16 R in 16 lanes per matrix: lane i holds the R rows i, i + 16, ...
// so that every broadcast stays inside a 16-lane DPP row (one instruction with the multiply-add)
// instead of going through the LDS crossbar or a scalar register as with 32 or 64 lanes per
// matrix; four matrices per wavefront.  Column j = 16 jh + jl: its entries sit in register j of
// row slot jh of lane jl.  R = 2 for n <= 32, R = 3 for n <= 48 (R N registers per lane; in fp64 R = 3 overflows
// into accumulation registers, takes the guarded broadcast multiply-add and is still 1.1 to 1.8 times faster
// than 64 lanes per matrix).
// ---------------------------------------------------------------------------------
template <typename T, int R, int N = 16 * R>
__global__ __launch_bounds__(WAVE) void k_potrf_tiny_rows(View<const T> A, View<T> L, int32_t *info, int info_off,
                                                           int64_t batch, int nb)
{
    // N columns kept, 16 (R - 1) < N <= 16 R: the last row slot is only partly filled when N < 16 R; a
    // lane without a row there follows row N - 1 and writes nothing.
    constexpr int G = 16, MPW = WAVE / G;
    static_assert(N > G * (R - 1) && N <= G * R && N % 4 == 0, "column count does not fit the row slots");
    using S = Stage<T, N, MPW>;
    extern __shared__ __align__(16) unsigned char tiny_lds[];
    T *sm = reinterpret_cast<T *>(tiny_lds);
    const int lane = threadIdx.x;
    const int q = lane / G, i = lane % G;
    const int64_t b0 = (int64_t)blockIdx.x * MPW;

    const Mem<const T> Am = mem_of(A);
    const Mem<T> Lm = mem_of(L);
    stage_load<T, N, MPW>(sm, Am, b0, batch, nb);
    __syncthreads();
    T a[R][N];  // a[h] = row i + 16 h
    static_for<0, R>([&](auto H) {
        constexpr int h = decltype(H)::value;
        const int row = (G * h + G > N && i + G * h >= N) ? N - 1 : i + G * h;
        read_lrow<T, N>(sm + q * S::MS, row, Am.tr, a[h]);
#pragma unroll
        for (int k = 0; k < N; ++k)
            if (k > i + G * h)
                a[h][k] = T(0);  // the other triangle of A is never used
    });

    int fail = 0;
    static_for<0, N>([&](auto J) {
        constexpr int j = decltype(J)::value;
        constexpr int jl = j % G, jh = j / G;
        T piv = group_bcast<G>(a[jh][j], jl);  // a_jj after the updates of columns < j
        if (!(piv > T(0)) && fail == 0)
            fail = j + 1;
        T r = rsqrt_acc(piv);
        static_for<jh, R>([&](auto H) {  // rows above slot jh have nothing in column j
            constexpr int h = decltype(H)::value;
            a[h][j] = (i + G * h >= j) ? a[h][j] * r : T(0);  // column j of L (row j gets sqrt(piv))
            dpp_settle1<G>(a[h][j]);
        });
        static_for<j + 1, N>([&](auto K) {
            constexpr int k = decltype(K)::value;
            constexpr int kl = k % G, kh = k / G;
            static_for<jh, R>([&](auto H) {  // a_rk -= l_rj l_kj, with l_kj in row slot kh of lane kl
                constexpr int h = decltype(H)::value;
                if constexpr (R >= 3)
                    fma_bcast16_guarded<kl>(a[h][k], a[kh][j], a[h][j], true);
                else
                    fma_bcast<G, kl>(a[h][k], a[kh][j], a[h][j], true);
            });
        });
    });

    __syncthreads();
    static_for<0, R>([&](auto H) {
        constexpr int h = decltype(H)::value;
#pragma unroll
        for (int k = 0; k < N; ++k)
            if (k > i + G * h)
                a[h][k] = T(0);
        if (G * h + G <= N || i + G * h < N) {
            if (Lm.tr)
                write_col<T, N>(sm + q * S::MS, i + G * h, a[h]);
            else
                write_row<T, N>(sm + q * S::MS, i + G * h, a[h]);
        }
    });
    __syncthreads();
    stage_store<T, N, MPW>(sm, Lm, b0, batch, nb);
    if (info != nullptr && i == 0 && b0 + q < batch && fail != 0 && fail <= nb) {
        if (info[b0 + q] == 0)
            info[b0 + q] = info_off + fail;
    }
}

// ---------------------------------------------------------------------------------
// potrf backward for n <= G.  Views give the logical lower-triangular L and Lbar.
// ---------------------------------------------------------------------------------
template <typename T, int G, int N = G>
__global__ __launch_bounds__(WAVE) void k_backward_tiny(View<const T> Lv, View<const T> Gv, View<T> Av,
                                                         int64_t batch, int n)
{
    // N <= G columns kept (see k_potrf_tiny); lanes i >= N carry zeros and write nothing
    constexpr int MPW = WAVE / G;
    using S = Stage<T, N, MPW>;
    __shared__ __align__(16) T sm[S::ELEMS];
    const int lane = threadIdx.x;
    const int q = lane / G, i = lane % G;
    const int ir = (N < G && i >= N) ? N - 1 : i;
    const bool own = (N == G) || i < N;
    const int64_t b0 = (int64_t)blockIdx.x * MPW;
    T *smq = sm + q * S::MS;

    // lane i takes column i of L: lc[k] = l_ki (k >= i), and its reciprocal diagonal
    T lc[N];
    const Mem<const T> Lm = mem_of(Lv);
    const Mem<const T> Gm = mem_of(Gv);
    stage_load<T, N, MPW>(sm, Lm, b0, batch, n);
    __syncthreads();
    read_lcol<T, N>(smq, ir, Lm.tr, lc);
    T dii = T(1);
#pragma unroll
    for (int k = 0; k < N; ++k) {
        if (k == i)
            dii = lc[k];
        if (k < i)
            lc[k] = T(0);
    }
    const T rd = rcp_acc(dii);
    __syncthreads();

    // lane k takes row k of Lbar: g[j] = lbar_kj (j <= k)
    T g[N];
    stage_load<T, N, MPW>(sm, Gm, b0, batch, n);
    __syncthreads();
    read_lrow<T, N>(smq, ir, Gm.tr, g);
#pragma unroll
    for (int j = 0; j < N; ++j)
        if (j > i || i >= n)
            g[j] = T(0);  // also drops the identity padding of the stage

    // P = L^T Lbar, row i in lane i: p_ij = sum_k l_ki lbar_kj   (terms with j > k are zero)
    T y[N];
#pragma unroll
    for (int j = 0; j < N; ++j)
        y[j] = T(0);
    dpp_settle<G>(g);
    static_for<0, N>([&](auto K) {
        constexpr int k = decltype(K)::value;
        static_for<0, k + 1>([&](auto J) {
            constexpr int j = decltype(J)::value;
            fma_bcast<G, k>(y[j], g[j], lc[k], false);
        });
    });
    // Phi, then the row scaling D^-1 of L = Lt D (Lt unit lower triangular)
#pragma unroll
    for (int j = 0; j < N; ++j) {
        T v = (j < i) ? y[j] : ((j == i) ? T(0.5) * y[j] : T(0));
        y[j] = v * rd;
    }
    // lt[k] = l_ki / l_ii for k > i, zero otherwise
#pragma unroll
    for (int k = 0; k < N; ++k)
        lc[k] = (k > i) ? lc[k] * rd : T(0);

    // Y = Lt^-T (D^-1 Phi): rows from the bottom; row k is final when it is broadcast
    dpp_settle<G>(y);
    static_for<0, N - 1>([&](auto Tt) {
        constexpr int k = N - 1 - decltype(Tt)::value;
        static_for<0, N>([&](auto C) {
            constexpr int c = decltype(C)::value;
            fma_bcast_self<G, k>(y[c], lc[k], true);  // G instructions lie between two touches of y[c]
        });
    });
    // V = Y D^-1 (column c scaled by 1 / l_cc), then W = V Lt^-1 from the last column back
#pragma unroll
    for (int c = 0; c < N; ++c)
        y[c] *= group_bcast<G>(rd, c);
    dpp_settle<G>(lc);
    static_for<0, N - 1>([&](auto Tt) {
        constexpr int c = N - 2 - decltype(Tt)::value;
        static_for<c + 1, N>([&](auto K) {
            constexpr int k = decltype(K)::value;
            fma_bcast<G, c>(y[c], lc[k], y[k], true);
        });
    });

    // Abar = 1/2 (W + W^T): rows out to LDS, columns back in
    __syncthreads();
    if (own)
        write_row<T, N>(smq, i, y);
    __syncthreads();
    T wt[N];
    read_col<T, N>(smq, ir, wt);
#pragma unroll
    for (int c = 0; c < N; ++c)
        y[c] = T(0.5) * (y[c] + wt[c]);
    __syncthreads();
    if (own)
        write_row<T, N>(smq, i, y);
    __syncthreads();
    stage_store<T, N, MPW>(sm, mem_of(Av), b0, batch, n);  // symmetric: orientation is immaterial
}

// ---------------------------------------------------------------------------------
// potrf backward for 16 < n <= 32 in 16 lanes per matrix: lane i owns rows i and i + 16 of
// P, Y, W and columns i and i + 16 of L (slot h = 0, 1), so all broadcasts are DPP row broadcasts.
// Same steps as k_backward_tiny; row / column k = 16 kh + kl lives in slot kh of lane kl.
// ---------------------------------------------------------------------------------
template <typename T, int N = 32>
__global__ __launch_bounds__(WAVE) void k_backward_tiny2(View<const T> Lv, View<const T> Gv, View<T> Av,
                                                          int64_t batch, int n)
{
    // N columns kept, 16 < N <= 32; a lane whose second row i + 16 does not exist carries zeros there
    constexpr int G = 16, MPW = WAVE / G;
    static_assert(N > G && N <= 2 * G && N % 4 == 0, "column count does not fit two row slots");
    using S = Stage<T, N, MPW>;
    __shared__ __align__(16) T sm[S::ELEMS];
    const int lane = threadIdx.x;
    const int q = lane / G, i = lane % G;
    const int64_t b0 = (int64_t)blockIdx.x * MPW;
    T *smq = sm + q * S::MS;
    const bool own1 = (N == 2 * G) || i + G < N;
    const int i1 = own1 ? i + G : N - 1;
    const Mem<const T> Lm = mem_of(Lv);
    const Mem<const T> Gm = mem_of(Gv);

    // columns i and i + 16 of L: lc_h[k] = l_{k, i + 16 h} (k >= i + 16 h), reciprocal diagonals
    T lc0[N], lc1[N];
    stage_load<T, N, MPW>(sm, Lm, b0, batch, n);
    __syncthreads();
    read_lcol<T, N>(smq, i, Lm.tr, lc0);
    read_lcol<T, N>(smq, i1, Lm.tr, lc1);
    T d0 = T(1), d1 = T(1);
#pragma unroll
    for (int k = 0; k < N; ++k) {
        if (k == i)
            d0 = lc0[k];
        if (k == i + G)
            d1 = lc1[k];
        if (k < i)
            lc0[k] = T(0);
        if (k < i + G)
            lc1[k] = T(0);
    }
    T rd0 = rcp_acc(d0), rd1 = rcp_acc(d1);
    __syncthreads();

    // rows i and i + 16 of Lbar
    T g0[N], g1[N];
    stage_load<T, N, MPW>(sm, Gm, b0, batch, n);
    __syncthreads();
    read_lrow<T, N>(smq, i, Gm.tr, g0);
    read_lrow<T, N>(smq, i1, Gm.tr, g1);
#pragma unroll
    for (int j = 0; j < N; ++j) {
        if (j > i || i >= n)
            g0[j] = T(0);  // also drops the identity padding of the stage
        if (j > i + G || i + G >= n)
            g1[j] = T(0);
    }

    // P = L^T Lbar: p_rj = sum_k l_kr lbar_kj (k >= r, j <= k)
    T y0[N], y1[N];
#pragma unroll
    for (int j = 0; j < N; ++j) {
        y0[j] = T(0);
        y1[j] = T(0);
    }
    dpp_settle<G>(g0);
    dpp_settle<G>(g1);
    static_for<0, N>([&](auto K) {
        constexpr int k = decltype(K)::value;
        constexpr int kl = k % G, kh = k / G;
        static_for<0, k + 1>([&](auto J) {
            constexpr int j = decltype(J)::value;
            if constexpr (kh == 0) {
                fma_bcast16_guarded<kl>(y0[j], g0[j], lc0[k], false);  // rows >= 16 have l_kr = 0 for k < 16
            } else {
                fma_bcast16_guarded<kl>(y0[j], g1[j], lc0[k], false);
                fma_bcast16_guarded<kl>(y1[j], g1[j], lc1[k], false);
            }
        });
    });
    // Phi, then the row scaling D^-1 of L = Lt D (Lt unit lower triangular)
#pragma unroll
    for (int j = 0; j < N; ++j) {
        const T v0 = (j < i) ? y0[j] : ((j == i) ? T(0.5) * y0[j] : T(0));
        const T v1 = (j < i + G) ? y1[j] : ((j == i + G) ? T(0.5) * y1[j] : T(0));
        y0[j] = v0 * rd0;
        y1[j] = v1 * rd1;
    }
    // lt_h[k] = l_kr / l_rr for k > r, zero otherwise
#pragma unroll
    for (int k = 0; k < N; ++k) {
        lc0[k] = (k > i) ? lc0[k] * rd0 : T(0);
        lc1[k] = (k > i + G) ? lc1[k] * rd1 : T(0);
    }

    // Y = Lt^-T (D^-1 Phi): rows from the bottom; row k is final when it is broadcast
    dpp_settle<G>(y0);
    dpp_settle<G>(y1);
    static_for<0, N - 1>([&](auto Tt) {
        constexpr int k = N - 1 - decltype(Tt)::value;
        constexpr int kl = k % G, kh = k / G;
        static_for<0, N>([&](auto C) {
            constexpr int c = decltype(C)::value;
            if constexpr (kh == 0) {
                fma_bcast16_guarded<kl>(y0[c], y0[c], lc0[k], true);  // rows >= 16: lt[k] = 0 for k <= 16
            } else {
                fma_bcast16_guarded<kl>(y0[c], y1[c], lc0[k], true);
                fma_bcast16_guarded<kl>(y1[c], y1[c], lc1[k], true);
            }
        });
    });
    // V = Y D^-1 (column c scaled by 1 / l_cc), then W = V Lt^-1 from the last column back
#pragma unroll
    for (int c = 0; c < N; ++c) {
        const T s = group_bcast<G>(c < G ? rd0 : rd1, c % G);
        y0[c] *= s;
        y1[c] *= s;
    }
    dpp_settle<G>(lc0);
    dpp_settle<G>(lc1);
    static_for<0, N - 1>([&](auto Tt) {
        constexpr int c = N - 2 - decltype(Tt)::value;
        constexpr int cl = c % G, ch = c / G;
        static_for<c + 1, N>([&](auto K) {
            constexpr int k = decltype(K)::value;
            if constexpr (ch == 0) {
                fma_bcast16_guarded<cl>(y0[c], lc0[k], y0[k], true);
                fma_bcast16_guarded<cl>(y1[c], lc0[k], y1[k], true);
            } else {
                fma_bcast16_guarded<cl>(y0[c], lc1[k], y0[k], true);
                fma_bcast16_guarded<cl>(y1[c], lc1[k], y1[k], true);
            }
        });
    });

    // Abar = 1/2 (W + W^T): rows out to LDS, columns back in
    __syncthreads();
    write_row<T, N>(smq, i, y0);
    if (own1)
        write_row<T, N>(smq, i + G, y1);
    __syncthreads();
    read_col<T, N>(smq, i, g0);
    read_col<T, N>(smq, i1, g1);
#pragma unroll
    for (int c = 0; c < N; ++c) {
        y0[c] = T(0.5) * (y0[c] + g0[c]);
        y1[c] = T(0.5) * (y1[c] + g1[c]);
    }
    __syncthreads();
    write_row<T, N>(smq, i, y0);
    if (own1)
        write_row<T, N>(smq, i + G, y1);
    __syncthreads();
    stage_store<T, N, MPW>(sm, mem_of(Av), b0, batch, n);  // symmetric: orientation is immaterial
}

template <typename T>
la_status launch_potrf_tiny(View<const T> A, View<T> L, int32_t *info, int info_off, int64_t batch, int nb,
                            hipStream_t st)
{
    if (batch <= 0 || nb <= 0)
        return LA_OK;
    if (nb > 64)
        return LA_ERR_UNSUPPORTED;
    if (nb <= 4) {
        constexpr int MPW = Stage<T, 4>::MPW;
        LA_LAUNCH((k_potrf_tiny<T, 4>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, A, L,
                           info, info_off, batch, nb);
    } else if (nb <= 8) {  // 8 lanes per matrix: half the pivots and twice the matrices per wavefront of the 16-lane form
        constexpr int MPW = Stage<T, 8>::MPW;
        LA_LAUNCH((k_potrf_tiny<T, 8>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, A, L,
                           info, info_off, batch, nb);
    } else if (nb <= 12) {  // 16 lanes per matrix, 12 columns staged and eliminated
        LA_LAUNCH((k_potrf_tiny<T, 16, 12>), dim3((unsigned)((batch + 3) / 4)), dim3(WAVE), 0, st, A, L, info,
                  info_off, batch, nb);
    } else if (nb <= 16) {
        constexpr int MPW = Stage<T, 16>::MPW;
        LA_LAUNCH((k_potrf_tiny<T, 16>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, A, L,
                           info, info_off, batch, nb);
    } else if (nb <= 48) {
        // 16 lanes per matrix, 2 or 3 rows per lane.  (4 rows per lane for n <= 64 need all 256
        // registers and one wavefront per SIMD: no faster than 64 lanes per matrix at n = 64,
        // slower below.)
        constexpr int MPW = 4;
        const dim3 grid((unsigned)((batch + MPW - 1) / MPW));
        // the column count kept is the next of 24, 32, 40, 48: the eliminations cost its cube
        if (nb <= 24) {
            LA_LAUNCH((k_potrf_tiny_rows<T, 2, 24>), grid, dim3(WAVE), (sizeof(T) * Stage<T, 24, MPW>::ELEMS), st, A, L,
                      info, info_off, batch, nb);
        } else if (nb <= 32) {
            LA_LAUNCH((k_potrf_tiny_rows<T, 2, 32>), grid, dim3(WAVE), (sizeof(T) * Stage<T, 32, MPW>::ELEMS), st, A, L,
                      info, info_off, batch, nb);
        } else if (nb <= 40) {
            LA_LAUNCH((k_potrf_tiny_rows<T, 3, 40>), grid, dim3(WAVE), (sizeof(T) * Stage<T, 40, MPW>::ELEMS), st, A, L,
                      info, info_off, batch, nb);
        } else {
            LA_LAUNCH((k_potrf_tiny_rows<T, 3, 48>), grid, dim3(WAVE), (sizeof(T) * Stage<T, 48, MPW>::ELEMS), st, A, L,
                      info, info_off, batch, nb);
        }
    } else {
        LA_LAUNCH((k_potrf_tiny<T, 64>), dim3((unsigned)batch), dim3(WAVE), 0, st, A, L, info, info_off,
                           batch, nb);
    }
    return launch_check("potrf_tiny");
}

template <typename T>
la_status launch_backward_tiny(View<const T> L, View<const T> G, View<T> Abar, int64_t batch, int n, hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    if (n > 32)
        return LA_ERR_UNSUPPORTED;
    if (n <= 4) {
        constexpr int MPW = Stage<T, 4>::MPW;
        LA_LAUNCH((k_backward_tiny<T, 4>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, L,
                           G, Abar, batch, n);
    } else if (n <= 8) {
        constexpr int MPW = Stage<T, 8>::MPW;
        LA_LAUNCH((k_backward_tiny<T, 8>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, L,
                           G, Abar, batch, n);
    } else if (n <= 12) {
        LA_LAUNCH((k_backward_tiny<T, 16, 12>), dim3((unsigned)((batch + 3) / 4)), dim3(WAVE), 0, st, L, G, Abar,
                  batch, n);
    } else if (n <= 16) {
        constexpr int MPW = Stage<T, 16>::MPW;
        LA_LAUNCH((k_backward_tiny<T, 16>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, L,
                           G, Abar, batch, n);
    } else if (n <= 24) {
        LA_LAUNCH((k_backward_tiny2<T, 24>), dim3((unsigned)((batch + 3) / 4)), dim3(WAVE), 0, st, L, G, Abar,
                  batch, n);
    } else {
        // 16 lanes per matrix, two rows per lane.  In fp64 the kernel needs 294 registers; the overflow lives in
        // accumulation registers (hence the guarded broadcast multiply-adds), which still beats 32 lanes per
        // matrix with ds_bpermute broadcasts by 2.5 times (16384 matrices of n = 32: 357 -> 140 us).
        LA_LAUNCH((k_backward_tiny2<T, 32>), dim3((unsigned)((batch + 3) / 4)), dim3(WAVE), 0, st, L, G, Abar,
                           batch, n);
    }
    return launch_check("backward_tiny");
}

template la_status launch_potrf_tiny<float>(View<const float>, View<float>, int32_t *, int, int64_t, int, hipStream_t);
template la_status launch_potrf_tiny<double>(View<const double>, View<double>, int32_t *, int, int64_t, int,
                                             hipStream_t);
template la_status launch_backward_tiny<float>(View<const float>, View<const float>, View<float>, int64_t, int,
                                               hipStream_t);
template la_status launch_backward_tiny<double>(View<const double>, View<const double>, View<double>, int64_t, int,
                                                hipStream_t);

}  // namespace la
