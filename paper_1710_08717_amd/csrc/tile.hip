// Triangular base-case tiles of the blocked algorithms (section 4.2 of arXiv 1710.08717:
// trsm "backsubstitution with lower triangular matrix", trmm "multiplication with lower
// triangular matrix"; the same tiles serve the panel solve of the blocked potrf and the
// three triangular phases of the potrf backward expression).
//
// One wavefront takes 64 vectors of length nb <= 64; each lane keeps ITS vector in
// registers and runs the substitution / product by itself, so there is no cross-lane
// traffic at all: the triangular block sits in LDS and is read with wave-uniform
// (broadcast) addresses.  Vectors that are contiguous in memory are transposed through
// LDS so that global accesses stay coalesced.
#include "common.hpp"

namespace la {

template <typename T>
struct TileCfg {
    static constexpr int LDM = NB + 16 / sizeof(T);  // 16-byte aligned rows for wide uniform reads
    static constexpr int LDX = NB + 1;               // odd stride: lane-private rows without conflicts
};

// sM[a][b] = Lam(a,b) (tflag == 0) or Lam(b,a) (tflag == 1), Lam lower triangular nb x nb:
// entries above its diagonal read as zero, padding up to 64 x 64 is the identity.
template <typename T>
__device__ __forceinline__ void load_tri(T *sM, View<const T> Lam, int64_t b, int nb, bool tflag)
{
    constexpr int LDM = TileCfg<T>::LDM;
    const int lane = threadIdx.x;
    const bool tr = (Lam.cs != 1);  // memory holds the transpose of the logical block
    const int64_t ld = tr ? Lam.cs : Lam.rs;
    const T *p = Lam.p + b * Lam.bs;
    for (int r = 0; r < NB; ++r) {
        const int c = lane;  // memory entry (r, c), lanes along the contiguous direction
        const int i = tr ? c : r, k = tr ? r : c;  // logical position
        T v = (i == k) ? T(1) : T(0);
        if (i < nb && k < nb && i >= k)
            v = p[r * ld + c];
        const int a = tflag ? k : i, bb = tflag ? i : k;
        sM[a * LDM + bb] = v;
    }
}

// MODE 0: solve M x = b, M lower (k ascending)      sM[k][i] = M(i,k)
// MODE 1: solve M x = b, M upper (k descending)     sM[k][i] = M(i,k)
// MODE 2: x <- M x, M lower (rows descending)       sM[i][k] = M(i,k)
// MODE 3: x <- M x, M upper (rows ascending)        sM[i][k] = M(i,k)
template <typename T, int MODE>
__global__ __launch_bounds__(WAVE) void k_tile(View<const T> Lam, View<T> X, int64_t batch, int nb, int64_t nvec,
                                               int tflag, int phi)
{
    constexpr int LDM = TileCfg<T>::LDM;
    constexpr int LDX = TileCfg<T>::LDX;
    __shared__ __align__(16) T sM[NB * LDM];
    __shared__ T sX[NB * LDX];
    __shared__ T sD[NB];
    const int lane = threadIdx.x;
    const int64_t ntile = (nvec + NB - 1) / NB;
    const int64_t b = blockIdx.x / ntile;
    const int64_t v0 = (blockIdx.x % ntile) * NB;
    const int64_t myv = v0 + lane;
    const bool active = myv < nvec;

    load_tri<T>(sM, Lam, b, nb, tflag != 0);

    T *xp = X.p + b * X.bs;
    const bool vec_adjacent = (X.cs == 1);  // consecutive vectors are consecutive in memory
    T x[NB];
    if (vec_adjacent) {
#pragma unroll
        for (int e = 0; e < NB; ++e)
            x[e] = (active && e < nb) ? xp[e * X.rs + myv] : T(0);
        __syncthreads();
    } else {
        for (int v = 0; v < NB; ++v) {
            const int e = lane;
            T val = T(0);
            if (v0 + v < nvec && e < nb)
                val = xp[e * X.rs + (v0 + v) * X.cs];
            sX[v * LDX + e] = val;
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < NB; ++e)
            x[e] = sX[lane * LDX + e];
    }

    if constexpr (MODE <= 1) {
        sD[lane] = rcp_acc(sM[lane * LDM + lane]);
        __syncthreads();
    }

    if constexpr (MODE == 0) {
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            x[k] *= sD[k];
#pragma unroll
            for (int i = k + 1; i < NB; ++i)
                x[i] = fma(-sM[k * LDM + i], x[k], x[i]);
        }
    } else if constexpr (MODE == 1) {
#pragma unroll
        for (int k = NB - 1; k >= 0; --k) {
            x[k] *= sD[k];
#pragma unroll
            for (int i = 0; i < k; ++i)
                x[i] = fma(-sM[k * LDM + i], x[k], x[i]);
        }
    } else if constexpr (MODE == 2) {
#pragma unroll
        for (int i = NB - 1; i >= 0; --i) {
            T s = sM[i * LDM + i] * x[i];
#pragma unroll
            for (int k = 0; k < i; ++k)
                s = fma(sM[i * LDM + k], x[k], s);
            x[i] = s;
        }
    } else {
        if (phi) {
            // the vectors are columns of a lower-triangular block: entries above its diagonal are zero
#pragma unroll
            for (int e = 0; e < NB; ++e)
                if (e < lane)
                    x[e] = T(0);
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            T s = sM[i * LDM + i] * x[i];
#pragma unroll
            for (int k = i + 1; k < NB; ++k)
                s = fma(sM[i * LDM + k], x[k], s);
            x[i] = s;
        }
        if (phi) {
            // keep the lower triangle, halve the diagonal (the map Phi of the backward expression)
#pragma unroll
            for (int e = 0; e < NB; ++e)
                x[e] = (e > lane) ? x[e] : ((e == lane) ? T(0.5) * x[e] : T(0));
        }
    }

    if (vec_adjacent) {
#pragma unroll
        for (int e = 0; e < NB; ++e)
            if (active && e < nb)
                xp[e * X.rs + myv] = x[e];
    } else {
        __syncthreads();
#pragma unroll
        for (int e = 0; e < NB; ++e)
            sX[lane * LDX + e] = x[e];
        __syncthreads();
        for (int v = 0; v < NB; ++v) {
            const int e = lane;
            if (v0 + v < nvec && e < nb)
                xp[e * X.rs + (v0 + v) * X.cs] = sX[v * LDX + e];
        }
    }
}

// Inverses of the 64 x 64 diagonal blocks of a lower-triangular Lam (n x n), written onto the
// diagonal blocks of Inv (lower triangle and zeros above it inside each block; a ragged last
// block writes only its nb x nb part).  Lane c solves Lam_jj x = e_c: column c of the inverse.
template <typename T>
__global__ __launch_bounds__(WAVE) void k_tile_inv(View<const T> Lam, View<T> Inv, int64_t batch, int n, int nblk)
{
    constexpr int LDM = TileCfg<T>::LDM;
    constexpr int LDX = TileCfg<T>::LDX;
    __shared__ __align__(16) T sM[NB * LDM];
    __shared__ T sX[NB * LDX];
    __shared__ T sD[NB];
    const int lane = threadIdx.x;
    const int64_t b = blockIdx.x / nblk;
    const int j = (int)(blockIdx.x % nblk);
    const int nb = min(NB, n - j * NB);
    load_tri<T>(sM, Lam.sub((int64_t)j * NB, (int64_t)j * NB), b, nb, true);  // sM[k][i] = Lam_jj(i,k)
    __syncthreads();
    sD[lane] = rcp_acc(sM[lane * LDM + lane]);
    __syncthreads();
    T x[NB];
#pragma unroll
    for (int e = 0; e < NB; ++e)
        x[e] = (e == lane) ? T(1) : T(0);
#pragma unroll
    for (int k = 0; k < NB; ++k) {
        x[k] *= sD[k];
#pragma unroll
        for (int i = k + 1; i < NB; ++i)
            x[i] = fma(-sM[k * LDM + i], x[k], x[i]);
    }
    // x[e] = inverse(e, lane); go through LDS so that the store walks Inv's contiguous direction
    View<T> O = Inv.sub((int64_t)j * NB, (int64_t)j * NB);
    T *op = O.p + b * O.bs;
#pragma unroll
    for (int e = 0; e < NB; ++e)
        sX[e * LDX + lane] = x[e];  // sX[row][col]
    __syncthreads();
    const bool colfast = (O.cs == 1);
    for (int u = 0; u < NB; ++u) {
        const int r = colfast ? u : lane, c = colfast ? lane : u;
        if (r < nb && c < nb)
            op[r * O.rs + c * O.cs] = sX[r * LDX + c];
    }
}

template <typename T>
la_status launch_tile_inverse(View<const T> Lam, View<T> Inv, int64_t batch, int n, hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    const int nblk = (n + NB - 1) / NB;
    const int64_t blocks = (int64_t)nblk * batch;
    if (blocks > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((k_tile_inv<T>), dim3((unsigned)blocks), dim3(WAVE), 0, st, Lam, Inv, batch, n, nblk);
    return launch_check("tile_inverse");
}

template <typename T, int MODE>
static la_status launch_tile(View<const T> Lam, View<T> X, int64_t batch, int nb, int64_t nvec, int tflag, int phi,
                             hipStream_t st)
{
    if (batch <= 0 || nb <= 0 || nvec <= 0)
        return LA_OK;
    if (nb > NB)
        return LA_ERR_UNSUPPORTED;
    const int64_t ntile = (nvec + NB - 1) / NB;
    const int64_t blocks = ntile * batch;
    if (blocks > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((k_tile<T, MODE>), dim3((unsigned)blocks), dim3(WAVE), 0, st, Lam, X, batch, nb, nvec, tflag,
                       phi);
    return launch_check("tile");
}

template <typename T>
la_status launch_tile_solve(View<const T> Lam, View<T> X, int64_t batch, int nb, int64_t nvec, bool fwd, hipStream_t st)
{
    // fwd: M = Lam (lower), sM[k][i] = Lam(i,k) -> transposed load.  !fwd: M = Lam^T (upper), sM[k][i] = Lam(k,i).
    return fwd ? launch_tile<T, 0>(Lam, X, batch, nb, nvec, 1, 0, st) : launch_tile<T, 1>(Lam, X, batch, nb, nvec, 0, 0, st);
}

template <typename T>
la_status launch_tile_mult(View<const T> Lam, View<T> X, int64_t batch, int nb, int64_t nvec, bool fwd, bool phi,
                           hipStream_t st)
{
    // fwd: M = Lam, sM[i][k] = Lam(i,k).  !fwd: M = Lam^T, sM[i][k] = Lam(k,i) -> transposed load.
    if (fwd) {
        if (phi)
            return LA_ERR_UNSUPPORTED;
        return launch_tile<T, 2>(Lam, X, batch, nb, nvec, 0, 0, st);
    }
    if (phi && nvec != nb)
        return LA_ERR_INVALID_ARG;
    return launch_tile<T, 3>(Lam, X, batch, nb, nvec, 1, phi ? 1 : 0, st);
}

template la_status launch_tile_inverse<float>(View<const float>, View<float>, int64_t, int, hipStream_t);
template la_status launch_tile_inverse<double>(View<const double>, View<double>, int64_t, int, hipStream_t);
template la_status launch_tile_solve<float>(View<const float>, View<float>, int64_t, int, int64_t, bool, hipStream_t);
template la_status launch_tile_solve<double>(View<const double>, View<double>, int64_t, int, int64_t, bool, hipStream_t);
template la_status launch_tile_mult<float>(View<const float>, View<float>, int64_t, int, int64_t, bool, bool,
                                           hipStream_t);
template la_status launch_tile_mult<double>(View<const double>, View<double>, int64_t, int, int64_t, bool, bool,
                                            hipStream_t);

}  // namespace la
