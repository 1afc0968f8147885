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

namespace la {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef double f64x2 __attribute__((ext_vector_type(2)));

template <typename T>
struct VecOf;
template <>
struct VecOf<float> {
    using type = f32x4;
    static constexpr int N = 4;
};
template <>
struct VecOf<double> {
    using type = f64x2;
    static constexpr int N = 2;
};

// LDS staging area of one wave: MPW matrices of G x G, rows padded by 16 bytes and
// matrices by 64 bytes so row reads, column reads and the flat fill are conflict-poor.
template <typename T, int G, int MPW_ = WAVE / G>
struct Stage {
    static constexpr int MPW = MPW_;
    static constexpr int PAD = 16 / sizeof(T);
    static constexpr int LD = G + PAD;
    static constexpr int MS = G * LD + 64 / sizeof(T);
    static constexpr int ELEMS = MPW * MS;
};

// Memory-order description of a batched block operand: entry (r, c) of item b at
// p + b*bs + r*ld + c.  tr says the LOGICAL matrix is the transpose of what memory holds.
template <typename T>
struct Mem {
    T *p;
    int64_t bs, ld;
    bool tr;
};
template <typename T>
__device__ __forceinline__ Mem<T> mem_of(View<T> V)
{
    const bool tr = (V.cs != 1);
    return {V.p, V.bs, tr ? V.cs : V.rs, tr};
}

template <typename T, int G, int MPW = WAVE / G>
__device__ __forceinline__ bool flat_ok(const T *p, int64_t bs, int64_t ld, int64_t b0, int64_t batch, int nb)
{
    return nb == G && ld == G && bs == G * G && b0 + MPW <= batch &&
           (reinterpret_cast<uintptr_t>(p) & 15) == 0;
}

// Fill the stage from global memory, in memory order.  Matrix q of the wave is item
// (b0 + q); entries outside nb x nb, and whole matrices past the batch end, become identity.
// (Leaving out the 16-byte pieces that lie entirely in the unused triangle was tried: the HBM
// fetch counter did not move -- rows are fetched in units of at least 64 bytes -- and the
// predicated loads made the kernels slower.)
template <typename T, int G, int MPW = WAVE / G>
__device__ __forceinline__ void stage_load(T *sm, Mem<const T> M, int64_t b0, int64_t batch, int nb)
{
    using S = Stage<T, G, MPW>;
    const int lane = threadIdx.x;
    // fast path: full G x G matrices stored back to back -> one flat vectorised copy
    if (flat_ok<T, G, MPW>(M.p, M.bs, M.ld, b0, batch, nb)) {
        using V4 = typename VecOf<T>::type;
        constexpr int VN = VecOf<T>::N;
        const V4 *src = reinterpret_cast<const V4 *>(M.p + b0 * M.bs);
        constexpr int NV = S::MPW * G * G / VN;
#pragma unroll
        for (int t = 0; t < NV / WAVE; ++t) {
            int e = (t * WAVE + lane) * VN;
            int q = e / (G * G), r = (e / G) % G, c = e % G;
            // streamed once: non-temporal, so the lines do not linger in the caches
            *reinterpret_cast<V4 *>(sm + q * S::MS + r * S::LD + c) = __builtin_nontemporal_load(&src[t * WAVE + lane]);
        }
        return;
    }
    // all loads of a batch of 16 first, then the LDS writes: the loads are in flight together
    constexpr int NIT = S::MPW * G * G / WAVE, CH = NIT < 16 ? NIT : 16;
    for (int t0 = 0; t0 < NIT; t0 += CH) {
        T v[CH];
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int e = (t0 + u) * WAVE + lane;
            const int q = e / (G * G), r = (e / G) % G, c = e % G;
            v[u] = (r == c) ? T(1) : T(0);
            if (b0 + q < batch && r < nb && c < nb)
                v[u] = M.p[(b0 + q) * M.bs + r * M.ld + c];
        }
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int e = (t0 + u) * WAVE + lane;
            const int q = e / (G * G), r = (e / G) % G, c = e % G;
            sm[q * S::MS + r * S::LD + c] = v[u];
        }
    }
}

template <typename T, int G, int MPW = WAVE / G>
__device__ __forceinline__ void stage_store(const T *sm, Mem<T> M, int64_t b0, int64_t batch, int nb)
{
    using S = Stage<T, G, MPW>;
    const int lane = threadIdx.x;
    if (flat_ok<T, G, MPW>(M.p, M.bs, M.ld, b0, batch, nb)) {
        using V4 = typename VecOf<T>::type;
        constexpr int VN = VecOf<T>::N;
        V4 *dst = reinterpret_cast<V4 *>(M.p + b0 * M.bs);
        constexpr int NV = S::MPW * G * G / VN;
#pragma unroll
        for (int t = 0; t < NV / WAVE; ++t) {
            int e = (t * WAVE + lane) * VN;
            int q = e / (G * G), r = (e / G) % G, c = e % G;
            __builtin_nontemporal_store(*reinterpret_cast<const V4 *>(sm + q * S::MS + r * S::LD + c),
                                        &dst[t * WAVE + lane]);
        }
        return;
    }
#pragma unroll 4
    for (int t = 0; t < S::MPW * G * G / WAVE; ++t) {
        int e = t * WAVE + lane;
        int q = e / (G * G);
        int r = (e / G) % G, c = e % G;
        if (b0 + q < batch && r < nb && c < nb)
            M.p[(b0 + q) * M.bs + r * M.ld + c] = sm[q * S::MS + r * S::LD + c];
    }
}

// Row i of the staged matrix into registers (row read), or column i (column read).
template <typename T, int G>
__device__ __forceinline__ void read_row(const T *smq, int i, T (&a)[G])
{
    using S = Stage<T, G>;
    using V4 = typename VecOf<T>::type;
    constexpr int VN = VecOf<T>::N;
#pragma unroll
    for (int c = 0; c < G; c += VN) {
        V4 v = *reinterpret_cast<const V4 *>(smq + i * S::LD + c);
        if constexpr (VN == 4) {
            a[c] = v.x; a[c + 1] = v.y; a[c + 2] = v.z; a[c + 3] = v.w;
        } else {
            a[c] = v.x; a[c + 1] = v.y;
        }
    }
}
template <typename T, int G>
__device__ __forceinline__ void write_row(T *smq, int i, const T (&a)[G])
{
    using S = Stage<T, G>;
    using V4 = typename VecOf<T>::type;
    constexpr int VN = VecOf<T>::N;
#pragma unroll
    for (int c = 0; c < G; c += VN) {
        V4 v;
        if constexpr (VN == 4) {
            v.x = a[c]; v.y = a[c + 1]; v.z = a[c + 2]; v.w = a[c + 3];
        } else {
            v.x = a[c]; v.y = a[c + 1];
        }
        *reinterpret_cast<V4 *>(smq + i * S::LD + c) = v;
    }
}
template <typename T, int G>
__device__ __forceinline__ void read_col(const T *smq, int i, T (&a)[G])
{
    using S = Stage<T, G>;
#pragma unroll
    for (int r = 0; r < G; ++r)
        a[r] = smq[r * S::LD + i];
}

template <typename T, int G>
__device__ __forceinline__ void write_col(T *smq, int i, const T (&a)[G])
{
    using S = Stage<T, G>;
#pragma unroll
    for (int r = 0; r < G; ++r)
        smq[r * S::LD + i] = a[r];
}
// Logical row i of a staged matrix whose memory image may be the transpose.
template <typename T, int G>
__device__ __forceinline__ void read_lrow(const T *smq, int i, bool tr, T (&a)[G])
{
    if (tr)
        read_col<T, G>(smq, i, a);
    else
        read_row<T, G>(smq, i, a);
}
template <typename T, int G>
__device__ __forceinline__ void read_lcol(const T *smq, int i, bool tr, T (&a)[G])
{
    if (tr)
        read_row<T, G>(smq, i, a);
    else
        read_col<T, G>(smq, i, a);
}

// ---------------------------------------------------------------------------------
// potrf forward.  View A / L give the LOGICAL lower-triangular problem: A(i,j), i >= j,
// is read; L(i,j) is written for the whole nb x nb block (zeros for i < j).
// ---------------------------------------------------------------------------------
template <typename T, int G>
__global__ __launch_bounds__(WAVE) void k_potrf_tiny(View<const T> A, View<T> L, int32_t *info, int info_off,
                                                      int64_t batch, int nb)
{
    using S = Stage<T, G>;
    __shared__ __align__(16) T sm[S::ELEMS];
    const int lane = threadIdx.x;
    const int q = lane / G, i = lane % G;
    const int64_t b0 = (int64_t)blockIdx.x * S::MPW;

    const Mem<const T> Am = mem_of(A);
    const Mem<T> Lm = mem_of(L);
    stage_load<T, G>(sm, Am, b0, batch, nb);
    __syncthreads();
    T a[G];
    read_lrow<T, G>(sm + q * S::MS, i, Am.tr, a);
#pragma unroll
    for (int k = 0; k < G; ++k)
        if (k > i)
            a[k] = T(0);  // the other triangle of A is never used

    int fail = 0;
    static_for<0, G>([&](auto J) {
        constexpr int j = decltype(J)::value;
        T piv = group_bcast<G>(a[j], j);  // a_jj after the updates of columns < j
        if (!(piv > T(0)) && fail == 0)
            fail = j + 1;
        T r = rsqrt_acc(piv);
        a[j] = (i >= j) ? a[j] * r : T(0);  // column j of L (lane j gets sqrt(piv))
        dpp_settle1<G>(a[j]);
        static_for<j + 1, G>([&](auto K) {
            constexpr int k = decltype(K)::value;
            fma_bcast<G, k>(a[k], a[j], a[j], true);  // a_ik -= l_ij l_kj
        });
    });
#pragma unroll
    for (int k = 0; k < G; ++k)
        if (k > i)
            a[k] = T(0);

    __syncthreads();
    if (Lm.tr)
        write_col<T, G>(sm + q * S::MS, i, a);
    else
        write_row<T, G>(sm + q * S::MS, i, a);
    __syncthreads();
    stage_store<T, G>(sm, Lm, b0, batch, nb);
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
// row slot jh of lane jl.  R = 2 in fp32 and fp64, R = 3 (n <= 48) in fp32 (R N registers per lane).
// ---------------------------------------------------------------------------------
template <typename T, int R>
__global__ __launch_bounds__(WAVE) void k_potrf_tiny_rows(View<const T> A, View<T> L, int32_t *info, int info_off,
                                                           int64_t batch, int nb)
{
    constexpr int G = 16, N = G * R, MPW = WAVE / G;
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
        read_lrow<T, N>(sm + q * S::MS, i + G * h, Am.tr, a[h]);
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
        if (Lm.tr)
            write_col<T, N>(sm + q * S::MS, i + G * h, a[h]);
        else
            write_row<T, N>(sm + q * S::MS, i + G * h, a[h]);
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
template <typename T, int G>
__global__ __launch_bounds__(WAVE) void k_backward_tiny(View<const T> Lv, View<const T> Gv, View<T> Av,
                                                         int64_t batch, int n)
{
    using S = Stage<T, G>;
    __shared__ __align__(16) T sm[S::ELEMS];
    const int lane = threadIdx.x;
    const int q = lane / G, i = lane % G;
    const int64_t b0 = (int64_t)blockIdx.x * S::MPW;
    T *smq = sm + q * S::MS;

    // lane i takes column i of L: lc[k] = l_ki (k >= i), and its reciprocal diagonal
    T lc[G];
    const Mem<const T> Lm = mem_of(Lv);
    const Mem<const T> Gm = mem_of(Gv);
    stage_load<T, G>(sm, Lm, b0, batch, n);
    __syncthreads();
    read_lcol<T, G>(smq, i, Lm.tr, lc);
    T dii = T(1);
#pragma unroll
    for (int k = 0; k < G; ++k) {
        if (k == i)
            dii = lc[k];
        if (k < i)
            lc[k] = T(0);
    }
    const T rd = rcp_acc(dii);
    __syncthreads();

    // lane k takes row k of Lbar: g[j] = lbar_kj (j <= k)
    T g[G];
    stage_load<T, G>(sm, Gm, b0, batch, n);
    __syncthreads();
    read_lrow<T, G>(smq, i, Gm.tr, g);
#pragma unroll
    for (int j = 0; j < G; ++j)
        if (j > i || i >= n)
            g[j] = T(0);  // also drops the identity padding of the stage

    // P = L^T Lbar, row i in lane i: p_ij = sum_k l_ki lbar_kj   (terms with j > k are zero)
    T y[G];
#pragma unroll
    for (int j = 0; j < G; ++j)
        y[j] = T(0);
    dpp_settle<G>(g);
    static_for<0, G>([&](auto K) {
        constexpr int k = decltype(K)::value;
        static_for<0, k + 1>([&](auto J) {
            constexpr int j = decltype(J)::value;
            fma_bcast<G, k>(y[j], g[j], lc[k], false);
        });
    });
    // Phi, then the row scaling D^-1 of L = Lt D (Lt unit lower triangular)
#pragma unroll
    for (int j = 0; j < G; ++j) {
        T v = (j < i) ? y[j] : ((j == i) ? T(0.5) * y[j] : T(0));
        y[j] = v * rd;
    }
    // lt[k] = l_ki / l_ii for k > i, zero otherwise
#pragma unroll
    for (int k = 0; k < G; ++k)
        lc[k] = (k > i) ? lc[k] * rd : T(0);

    // Y = Lt^-T (D^-1 Phi): rows from the bottom; row k is final when it is broadcast
    dpp_settle<G>(y);
    static_for<0, G - 1>([&](auto Tt) {
        constexpr int k = G - 1 - decltype(Tt)::value;
        static_for<0, G>([&](auto C) {
            constexpr int c = decltype(C)::value;
            fma_bcast_self<G, k>(y[c], lc[k], true);  // G instructions lie between two touches of y[c]
        });
    });
    // V = Y D^-1 (column c scaled by 1 / l_cc), then W = V Lt^-1 from the last column back
#pragma unroll
    for (int c = 0; c < G; ++c)
        y[c] *= group_bcast<G>(rd, c);
    dpp_settle<G>(lc);
    static_for<0, G - 1>([&](auto Tt) {
        constexpr int c = G - 2 - decltype(Tt)::value;
        static_for<c + 1, G>([&](auto K) {
            constexpr int k = decltype(K)::value;
            fma_bcast<G, c>(y[c], lc[k], y[k], true);
        });
    });

    // Abar = 1/2 (W + W^T): rows out to LDS, columns back in
    __syncthreads();
    write_row<T, G>(smq, i, y);
    __syncthreads();
    T wt[G];
    read_col<T, G>(smq, i, wt);
#pragma unroll
    for (int c = 0; c < G; ++c)
        y[c] = T(0.5) * (y[c] + wt[c]);
    __syncthreads();
    write_row<T, G>(smq, i, y);
    __syncthreads();
    stage_store<T, G>(sm, mem_of(Av), b0, batch, n);  // symmetric: orientation is immaterial
}

// ---------------------------------------------------------------------------------
// potrf backward for 16 < n <= 32 in 16 lanes per matrix (fp32): lane i owns rows i and i + 16 of
// P, Y, W and columns i and i + 16 of L (slot h = 0, 1), so all broadcasts are DPP row broadcasts.
// Same steps as k_backward_tiny; row / column k = 16 kh + kl lives in slot kh of lane kl.
// ---------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(WAVE) void k_backward_tiny2(View<const T> Lv, View<const T> Gv, View<T> Av,
                                                          int64_t batch, int n)
{
    constexpr int N = 32, G = 16, MPW = WAVE / G;
    using S = Stage<T, N, MPW>;
    __shared__ __align__(16) T sm[S::ELEMS];
    const int lane = threadIdx.x;
    const int q = lane / G, i = lane % G;
    const int64_t b0 = (int64_t)blockIdx.x * MPW;
    T *smq = sm + q * S::MS;
    const Mem<const T> Lm = mem_of(Lv);
    const Mem<const T> Gm = mem_of(Gv);

    // columns i and i + 16 of L: lc_h[k] = l_{k, i + 16 h} (k >= i + 16 h), reciprocal diagonals
    T lc0[N], lc1[N];
    stage_load<T, N, MPW>(sm, Lm, b0, batch, n);
    __syncthreads();
    read_lcol<T, N>(smq, i, Lm.tr, lc0);
    read_lcol<T, N>(smq, i + G, Lm.tr, lc1);
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
    read_lrow<T, N>(smq, i + G, Gm.tr, g1);
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
                fma_bcast<G, kl>(y0[j], g0[j], lc0[k], false);  // rows >= 16 have l_kr = 0 for k < 16
            } else {
                fma_bcast<G, kl>(y0[j], g1[j], lc0[k], false);
                fma_bcast<G, kl>(y1[j], g1[j], lc1[k], false);
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
                fma_bcast<G, kl>(y0[c], y0[c], lc0[k], true);  // rows >= 16: lt[k] = 0 for k <= 16
            } else {
                fma_bcast<G, kl>(y0[c], y1[c], lc0[k], true);
                fma_bcast<G, kl>(y1[c], y1[c], lc1[k], true);
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
                fma_bcast<G, cl>(y0[c], lc0[k], y0[k], true);
                fma_bcast<G, cl>(y1[c], lc0[k], y1[k], true);
            } else {
                fma_bcast<G, cl>(y0[c], lc1[k], y0[k], true);
                fma_bcast<G, cl>(y1[c], lc1[k], y1[k], true);
            }
        });
    });

    // Abar = 1/2 (W + W^T): rows out to LDS, columns back in
    __syncthreads();
    write_row<T, N>(smq, i, y0);
    write_row<T, N>(smq, i + G, y1);
    __syncthreads();
    read_col<T, N>(smq, i, g0);
    read_col<T, N>(smq, i + G, g1);
#pragma unroll
    for (int c = 0; c < N; ++c) {
        y0[c] = T(0.5) * (y0[c] + g0[c]);
        y1[c] = T(0.5) * (y1[c] + g1[c]);
    }
    __syncthreads();
    write_row<T, N>(smq, i, y0);
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
        hipLaunchKernelGGL((k_potrf_tiny<T, 4>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, A, L,
                           info, info_off, batch, nb);
    } else if (nb <= 8) {  // 8 lanes per matrix: half the pivots and twice the matrices per wavefront of the 16-lane form
        constexpr int MPW = Stage<T, 8>::MPW;
        hipLaunchKernelGGL((k_potrf_tiny<T, 8>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, A, L,
                           info, info_off, batch, nb);
    } else if (nb <= 16) {
        constexpr int MPW = Stage<T, 16>::MPW;
        hipLaunchKernelGGL((k_potrf_tiny<T, 16>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, A, L,
                           info, info_off, batch, nb);
    } else if (nb <= 32 || (sizeof(T) == 4 && nb <= 48)) {
        // 16 lanes per matrix, 2 or 3 rows per lane.  (4 rows per lane for n <= 64 need all 256
        // registers and one wavefront per SIMD: no faster than 64 lanes per matrix at n = 64,
        // slower below.)
        constexpr int MPW = 4;
        const dim3 grid((unsigned)((batch + MPW - 1) / MPW));
        constexpr size_t lds2 = sizeof(T) * Stage<T, 32, MPW>::ELEMS, lds3 = sizeof(T) * Stage<T, 48, MPW>::ELEMS;
        if (nb <= 32) {
            hipLaunchKernelGGL((k_potrf_tiny_rows<T, 2>), grid, dim3(WAVE), lds2, st, A, L, info, info_off, batch, nb);
        } else if constexpr (sizeof(T) == 4) {
            hipLaunchKernelGGL((k_potrf_tiny_rows<T, 3>), grid, dim3(WAVE), lds3, st, A, L, info, info_off, batch, nb);
        }
    } else {
        hipLaunchKernelGGL((k_potrf_tiny<T, 64>), dim3((unsigned)batch), dim3(WAVE), 0, st, A, L, info, info_off,
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
        hipLaunchKernelGGL((k_backward_tiny<T, 4>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, L,
                           G, Abar, batch, n);
    } else if (n <= 8) {
        constexpr int MPW = Stage<T, 8>::MPW;
        hipLaunchKernelGGL((k_backward_tiny<T, 8>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, L,
                           G, Abar, batch, n);
    } else if (n <= 16) {
        constexpr int MPW = Stage<T, 16>::MPW;
        hipLaunchKernelGGL((k_backward_tiny<T, 16>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, L,
                           G, Abar, batch, n);
    } else if constexpr (sizeof(T) == 4) {  // 16 lanes per matrix, two rows per lane (its registers do not fit in fp64)
        hipLaunchKernelGGL((k_backward_tiny2<T>), dim3((unsigned)((batch + 3) / 4)), dim3(WAVE), 0, st, L, G, Abar,
                           batch, n);
    } else {
        constexpr int MPW = Stage<T, 32>::MPW;
        hipLaunchKernelGGL((k_backward_tiny<T, 32>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, L,
                           G, Abar, batch, n);
    }
    return launch_check("backward_tiny");
}

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

__device__ __forceinline__ int img_idx(int e) { return e + (e >> 4); }

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
        hipLaunchKernelGGL((k_tri_tiny<T, G, true>), grid, dim3(WAVE), 0, st, Lam, Bin, Bout, batch, n, m, fwd ? 1 : 0,
                           img_tr ? 1 : 0, alpha);
    else
        hipLaunchKernelGGL((k_tri_tiny<T, G, false>), grid, dim3(WAVE), 0, st, Lam, Bin, Bout, batch, n, m, fwd ? 1 : 0,
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

// flat image of cnt items of `per` elements each into LDS (16-byte loads when whole and aligned)
template <typename T, int IMG, int MPW>
__device__ __forceinline__ void image_load(T *img, const T *base, int64_t b0, int cnt, int per, int lane)
{
    using V4 = typename VecOf<T>::type;
    constexpr int VN = VecOf<T>::N;
    const int tot = cnt * per;
    const T *src = base + b0 * per;
    if ((cnt == MPW) && ((MPW * per) % VN == 0) && ((reinterpret_cast<uintptr_t>(base) & 15) == 0)) {
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
}

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
    constexpr int IMGP = (IMG + IMG / 16 + 4 + 3) / 4 * 4;  // padded image, a multiple of 16 bytes
    constexpr int SMP = (S::ELEMS + 3) / 4 * 4;
    extern __shared__ __align__(16) unsigned char tiny_lds[];
    T *sm = reinterpret_cast<T *>(tiny_lds), *img = sm + SMP, *img2 = img + IMGP;  // img2 only when V != U
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
        const int img = (64 / g) * g * SYRK_KC, imgp = (img + img / 16 + 4 + 3) / 4 * 4;
        return (size_t)((elems + 3) / 4 * 4 + images * imgp) * sizeof(T);
    };
    const dim3 blk(WAVE);
    const int itr = img_tr ? 1 : 0;
#define LA_SYRK_TINY(GG)                                                                                                  \
    do {                                                                                                                  \
        constexpr int MPW = Stage<T, GG>::MPW;                                                                            \
        const dim3 grid((unsigned)((batch + MPW - 1) / MPW));                                                             \
        if (images == 2)                                                                                                  \
            hipLaunchKernelGGL((k_syrk_tiny<T, GG, true>), grid, blk, lds(GG, Stage<T, GG>::ELEMS), st, U, V, C, batch, n, \
                               k, itr, tri, alpha);                                                                       \
        else                                                                                                              \
            hipLaunchKernelGGL((k_syrk_tiny<T, GG, false>), grid, blk, lds(GG, Stage<T, GG>::ELEMS), st, U, V, C, batch,   \
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

// flat image back to memory (the mirror of image_load)
template <typename T, int IMG, int MPW>
__device__ __forceinline__ void image_store(const T *img, T *base, int64_t b0, int cnt, int per, int lane)
{
    using V4 = typename VecOf<T>::type;
    constexpr int VN = VecOf<T>::N;
    const int tot = cnt * per;
    T *dst = base + b0 * per;
    if ((cnt == MPW) && ((MPW * per) % VN == 0) && ((reinterpret_cast<uintptr_t>(base) & 15) == 0)) {
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
        hipLaunchKernelGGL((k_gemm2_tiny<T, 4>), dim3((unsigned)((batch + 15) / 16)), dim3(WAVE), 0, st, A, B, C, batch, m, n,
                           k, ta, tb, alpha);
    else if (d <= 8)
        hipLaunchKernelGGL((k_gemm2_tiny<T, 8>), dim3((unsigned)((batch + 7) / 8)), dim3(WAVE), 0, st, A, B, C, batch, m, n, k,
                           ta, tb, alpha);
    else
        hipLaunchKernelGGL((k_gemm2_tiny<T, 16>), dim3((unsigned)((batch + 3) / 4)), dim3(WAVE), 0, st, A, B, C, batch, m, n,
                           k, ta, tb, alpha);
    return launch_check("gemm2_tiny");
}

template la_status launch_gemm2_tiny<float>(int, int, float, int64_t, int, int, int, const float *, const float *, float *,
                                            hipStream_t);
template la_status launch_gemm2_tiny<double>(int, int, double, int64_t, int, int, int, const double *, const double *,
                                             double *, hipStream_t);

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

template <typename T>
la_status launch_potri_tiny(View<const T> Lam, View<T> B, int64_t batch, int n, hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    if (n > 16 || (batch + 3) / 4 > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    if (n <= 4) {
        constexpr int MPW = Stage<T, 4>::MPW;
        hipLaunchKernelGGL((k_potri_tiny<T, 4>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, Lam, B, batch, n);
    } else if (n <= 8) {
        constexpr int MPW = Stage<T, 8>::MPW;
        hipLaunchKernelGGL((k_potri_tiny<T, 8>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, Lam, B, batch, n);
    } else {
        constexpr int MPW = Stage<T, 16>::MPW;
        hipLaunchKernelGGL((k_potri_tiny<T, 16>), dim3((unsigned)((batch + MPW - 1) / MPW)), dim3(WAVE), 0, st, Lam, B, batch, n);
    }
    return launch_check("potri_tiny");
}

template la_status launch_potri_tiny<float>(View<const float>, View<float>, int64_t, int, hipStream_t);
template la_status launch_potri_tiny<double>(View<const double>, View<double>, int64_t, int, hipStream_t);

template la_status launch_potrf_tiny<float>(View<const float>, View<float>, int32_t *, int, int64_t, int, hipStream_t);
template la_status launch_potrf_tiny<double>(View<const double>, View<double>, int32_t *, int, int64_t, int,
                                             hipStream_t);
template la_status launch_backward_tiny<float>(View<const float>, View<const float>, View<float>, int64_t, int,
                                               hipStream_t);
template la_status launch_backward_tiny<double>(View<const double>, View<const double>, View<double>, int64_t, int,
                                                hipStream_t);

}  // namespace la
