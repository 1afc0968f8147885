// Small triangular kernels (section 4.2 of arXiv 1710.08717, "trsm": backsubstitution with a
// lower triangular matrix):
//  * k_tile_inv: inverses of the 64 x 64 diagonal blocks of a factor, one wavefront per block,
//    each lane running the forward substitution for its own column of the identity with the
//    block read from LDS at wave-uniform addresses.  The blocked paths multiply by these.
//  * k_trsm_small: the whole solve for n <= 128 and a handful of right-hand sides, one wavefront
//    per right-hand side with the vector spread over the lanes: at step k the pivot entry is
//    read with v_readlane and every lane updates its rows with column k of the matrix, which
//    sits transposed in LDS.  No barrier inside the substitution.
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

// ---------------------------------------------------------------------------------------
// Whole solve for small n: X <- alpha * M^-1 Xin with M = Lam (fwd) or Lam^T (!fwd), n <= 128,
// vectors X(e, v).  256 threads = 4 wavefronts = 4 vectors per workgroup; all of them first
// stage sMt[k][i] = M(i,k) and the reciprocal diagonal in LDS.
// ---------------------------------------------------------------------------------------
constexpr int SMALL_N = 128;

template <typename T>
__global__ __launch_bounds__(256) void k_trsm_small(View<const T> Lam, View<const T> Xin, View<T> X, int64_t batch, int n,
                                                    int m, T alpha, int fwd, int vchunks)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    T *sMt = reinterpret_cast<T *>(smem_raw);  // n x (n + 1)
    const int LD = n + 1;
    T *sD = sMt + n * LD;  // n reciprocals of the diagonal
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int64_t b = blockIdx.x / vchunks;
    const int v = (int)(blockIdx.x % vchunks) * 4 + w;

    // stage: walk Lam's memory along its contiguous direction
    const bool tr = (Lam.cs != 1);
    const int64_t ld = tr ? Lam.cs : Lam.rs;
    const T *lp = Lam.p + b * Lam.bs;
    for (int idx = tid; idx < n * n; idx += 256) {
        const int r = idx / n, c = idx % n;          // memory entry (r, c)
        const int i = tr ? c : r, k = tr ? r : c;    // logical Lam(i, k)
        if (i >= k) {
            const T val = lp[(int64_t)r * ld + c];
            // M(i', k') with M = Lam: (i, k); with M = Lam^T: (k, i).  Stored as sMt[k'][i'].
            if (fwd)
                sMt[k * LD + i] = val;
            else
                sMt[i * LD + k] = val;
            if (i == k)
                sD[i] = rcp_acc(val);
        }
    }
    __syncthreads();
    if (v >= m)
        return;

    const T *xin = Xin.p + b * Xin.bs + (int64_t)v * Xin.cs;
    T *xout = X.p + b * X.bs + (int64_t)v * X.cs;
    const int r0 = lane, r1 = lane + 64;
    const int c0 = min(r0, n - 1), c1 = min(r1, n - 1);  // in-range LDS columns for the idle lanes
    T x0 = (r0 < n) ? alpha * xin[(int64_t)r0 * Xin.rs] : T(0);
    T x1 = (r1 < n) ? alpha * xin[(int64_t)r1 * Xin.rs] : T(0);

    if (fwd) {
        for (int k = 0; k < n; ++k) {
            const T src = (k < 64) ? x0 : x1;
            const T xk = group_bcast<64>(src, k & 63) * sD[k];
            const T *col = sMt + k * LD;  // M(i, k), i > k
            if (k < 64) {
                x0 = (r0 == k) ? xk : ((r0 > k && r0 < n) ? fma(-col[c0], xk, x0) : x0);
                if (r1 < n)
                    x1 = fma(-col[c1], xk, x1);
            } else {
                x1 = (r1 == k) ? xk : ((r1 > k && r1 < n) ? fma(-col[c1], xk, x1) : x1);
            }
        }
    } else {
        for (int k = n - 1; k >= 0; --k) {
            const T src = (k < 64) ? x0 : x1;
            const T xk = group_bcast<64>(src, k & 63) * sD[k];
            const T *col = sMt + k * LD;  // M(i, k), i < k
            if (k >= 64) {
                x1 = (r1 == k) ? xk : ((r1 < k) ? fma(-col[c1], xk, x1) : x1);
                x0 = fma(-col[c0], xk, x0);
            } else {
                x0 = (r0 == k) ? xk : ((r0 < k) ? fma(-col[c0], xk, x0) : x0);
            }
        }
    }
    if (r0 < n)
        xout[(int64_t)r0 * X.rs] = x0;
    if (r1 < n)
        xout[(int64_t)r1 * X.rs] = x1;
}

template <typename T>
la_status launch_trsm_small(View<const T> Lam, View<const T> Xin, View<T> X, int64_t batch, int n, int m, T alpha,
                            bool fwd, hipStream_t st)
{
    if (batch <= 0 || n <= 0 || m <= 0)
        return LA_OK;
    if (n > SMALL_N)
        return LA_ERR_UNSUPPORTED;
    const int vchunks = (m + 3) / 4;
    const int64_t blocks = (int64_t)vchunks * batch;
    if (blocks > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    const size_t lds = ((size_t)n * (n + 1) + n) * sizeof(T);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_trsm_small<T>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) {
            set_error(e, "hipFuncSetAttribute(trsm_small)");
            return LA_ERR_RUNTIME;
        }
    }
    hipLaunchKernelGGL((k_trsm_small<T>), dim3((unsigned)blocks), dim3(256), lds, st, Lam, Xin, X, batch, n, m, alpha,
                       fwd ? 1 : 0, vchunks);
    return launch_check("trsm_small");
}

template la_status launch_trsm_small<float>(View<const float>, View<const float>, View<float>, int64_t, int, int, float,
                                            bool, hipStream_t);
template la_status launch_trsm_small<double>(View<const double>, View<const double>, View<double>, int64_t, int, int,
                                             double, bool, hipStream_t);
template la_status launch_tile_inverse<float>(View<const float>, View<float>, int64_t, int, hipStream_t);
template la_status launch_tile_inverse<double>(View<const double>, View<double>, int64_t, int, hipStream_t);

}  // namespace la
