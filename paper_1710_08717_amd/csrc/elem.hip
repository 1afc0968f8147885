// Memory-bound helper kernels: masked / scaled copies, the symmetrisation that ends the
// potrf backward expression (appendix "potrf": Abar must be symmetric), copyltu-style
// mirroring for syrk's full symmetric output, log|L| = sum_i log l_ii (section 3.1) and
// the Gaussian-process criterion glue (section 3.1 with the trsm backward rule of
// section 4.2).
#include "common.hpp"

namespace la {

constexpr int ET = 32;  // tile edge of the transposing helpers

template <typename T>
__global__ __launch_bounds__(256) void k_copy(View<const T> src, View<T> dst, int64_t batch, int rows, int cols,
                                              T alpha, int keep, int tiles_r, int tiles_c)
{
    const int64_t per = (int64_t)tiles_r * tiles_c;
    const int64_t b = blockIdx.x / per;
    const int tile = (int)(blockIdx.x % per);
    const int r0 = (tile / tiles_c) * ET, c0 = (tile % tiles_c) * ET;
    const bool colfast = (dst.cs == 1) || (dst.rs != 1);
    const T *sp = src.p + b * src.bs;
    T *dp = dst.p + b * dst.bs;
    const bool src_colfast = (src.cs == 1) || (src.rs != 1);
    if (src_colfast != colfast && (src.cs == 1 || src.rs == 1)) {
        // A transposing copy: the tile is read along the source's contiguous direction, turned in LDS
        // and written along the destination's (an element-wise copy would read with a stride).
        __shared__ T turn[ET][ET + 1];
        for (int t = threadIdx.x; t < ET * ET; t += 256) {
            const int u = t / ET, w = t % ET;  // w runs along the source's contiguous direction
            const int r = r0 + (src_colfast ? u : w), c = c0 + (src_colfast ? w : u);
            T v = T(0);
            if (r < rows && c < cols && !(keep != 0 && r < c))
                v = alpha * sp[(int64_t)r * src.rs + (int64_t)c * src.cs];
            turn[u][w] = v;
        }
        __syncthreads();
        for (int t = threadIdx.x; t < ET * ET; t += 256) {
            const int u = t / ET, w = t % ET;  // w runs along the destination's contiguous direction
            const int r = r0 + (colfast ? u : w), c = c0 + (colfast ? w : u);
            if (r < rows && c < cols && !(keep == 2 && r < c))
                dp[(int64_t)r * dst.rs + (int64_t)c * dst.cs] = turn[w][u];
        }
        return;
    }
    for (int t = threadIdx.x; t < ET * ET; t += 256) {
        const int u = t / ET, w = t % ET;
        const int r = r0 + (colfast ? u : w), c = c0 + (colfast ? w : u);
        if (r < rows && c < cols && !(keep == 2 && r < c)) {
            T v = T(0);
            if (!(keep == 1 && r < c))
                v = alpha * sp[(int64_t)r * src.rs + (int64_t)c * src.cs];
            dp[(int64_t)r * dst.rs + (int64_t)c * dst.cs] = v;
        }
    }
}

template <typename T>
la_status launch_copy(View<const T> src, View<T> dst, int64_t batch, int rows, int cols, T alpha, int keep,
                      hipStream_t st)
{
    if (batch <= 0 || rows <= 0 || cols <= 0)
        return LA_OK;
    const int tr = (rows + ET - 1) / ET, tc = (cols + ET - 1) / ET;
    const int64_t blocks = (int64_t)tr * tc * batch;
    if (blocks > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    LA_LAUNCH((k_copy<T>), dim3((unsigned)blocks), dim3(256), 0, st, src, dst, batch, rows, cols, alpha, keep,
                       tr, tc);
    return launch_check("copy");
}

// work(i,j) = src(i,j) for i >= j (nothing else of work is written) and out(i,j) = 0 for i < j
// (nothing else of out is written).  out may alias src.
template <typename T>
__global__ __launch_bounds__(256) void k_tril_split(View<const T> src, View<T> work, View<T> out, int64_t batch, int n,
                                                    int nt)
{
    const int64_t per = (int64_t)nt * nt;
    const int64_t b = blockIdx.x / per;
    const int tile = (int)(blockIdx.x % per);
    const int r0 = (tile / nt) * ET, c0 = (tile % nt) * ET;
    const bool colfast = (src.cs == 1) || (src.rs != 1);
    const T *sp = src.p + b * src.bs;
    T *wp = work.p + b * work.bs;
    T *op = out.p + b * out.bs;
    for (int t = threadIdx.x; t < ET * ET; t += 256) {
        const int u = t / ET, w = t % ET;
        const int r = r0 + (colfast ? u : w), c = c0 + (colfast ? w : u);
        if (r < n && c < n) {
            if (r >= c)
                wp[(int64_t)r * work.rs + (int64_t)c * work.cs] = sp[(int64_t)r * src.rs + (int64_t)c * src.cs];
            else
                op[(int64_t)r * out.rs + (int64_t)c * out.cs] = T(0);
        }
    }
}

template <typename T>
la_status launch_tril_split(View<const T> src, View<T> work, View<T> out, int64_t batch, int n, hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    const int nt = (n + ET - 1) / ET;
    const int64_t blocks = (int64_t)nt * nt * batch;
    if (blocks > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    LA_LAUNCH((k_tril_split<T>), dim3((unsigned)blocks), dim3(256), 0, st, src, work, out, batch, n, nt);
    return launch_check("tril_split");
}

// X(i,j) = 0 for i < j on n x n (nothing else is written).
template <typename T>
__global__ __launch_bounds__(256) void k_zero_strict_upper(View<T> X, int64_t batch, int n, int nt)
{
    const int64_t per = (int64_t)nt * nt;
    const int64_t b = blockIdx.x / per;
    const int tile = (int)(blockIdx.x % per);
    const int r0 = (tile / nt) * ET, c0 = (tile % nt) * ET;
    if (r0 > c0 + ET - 1)
        return;  // tile entirely below the diagonal
    const bool colfast = (X.cs == 1) || (X.rs != 1);
    T *xp = X.p + b * X.bs;
    for (int t = threadIdx.x; t < ET * ET; t += 256) {
        const int u = t / ET, w = t % ET;
        const int r = r0 + (colfast ? u : w), c = c0 + (colfast ? w : u);
        if (r < n && c < n && r < c)
            xp[(int64_t)r * X.rs + (int64_t)c * X.cs] = T(0);
    }
}

template <typename T>
la_status launch_zero_strict_upper(View<T> X, int64_t batch, int n, hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    const int nt = (n + ET - 1) / ET;
    const int64_t blocks = (int64_t)nt * nt * batch;
    if (blocks > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    LA_LAUNCH((k_zero_strict_upper<T>), dim3((unsigned)blocks), dim3(256), 0, st, X, batch, n, nt);
    return launch_check("zero_strict_upper");
}

// mode 0: X <- scale * (X + X^T).   mode 1: X(i,j) <- X(j,i) for i < j (lower copied to upper).
// One block per tile pair (ti >= tj); both tiles pass through LDS so every global access is
// along the contiguous direction.
template <typename T>
__global__ __launch_bounds__(256) void k_sym(View<T> X, int64_t batch, int n, T scale, int mode, int nt)
{
    __shared__ T sa[ET][ET + 1];
    __shared__ T sb[ET][ET + 1];
    const int64_t per = (int64_t)nt * nt;
    const int64_t b = blockIdx.x / per;
    const int tile = (int)(blockIdx.x % per);
    const int ti = tile / nt, tj = tile % nt;
    if (tj > ti)
        return;
    T *xp = X.p + b * X.bs;
    // treat the matrix in memory order: for a symmetric operation the orientation is immaterial
    const bool tr = (X.cs != 1);
    const int64_t ld = tr ? X.cs : X.rs;
    const int r0 = ti * ET, c0 = tj * ET;
    for (int t = threadIdx.x; t < ET * ET; t += 256) {
        const int u = t / ET, w = t % ET;
        sa[u][w] = (r0 + u < n && c0 + w < n) ? xp[(int64_t)(r0 + u) * ld + c0 + w] : T(0);  // tile (ti,tj)
        sb[u][w] = (c0 + u < n && r0 + w < n) ? xp[(int64_t)(c0 + u) * ld + r0 + w] : T(0);  // tile (tj,ti)
    }
    __syncthreads();
    // In memory order "lower" means row >= column; when the view is transposed the logical
    // lower triangle is the memory upper triangle.
    for (int t = threadIdx.x; t < ET * ET; t += 256) {
        const int u = t / ET, w = t % ET;
        // entry (r0+u, c0+w) of tile (ti,tj) pairs with entry (c0+w, r0+u) = sb[w][u]
        if (mode == 0) {
            const T v = scale * (sa[u][w] + sb[w][u]);
            if (r0 + u < n && c0 + w < n)
                xp[(int64_t)(r0 + u) * ld + c0 + w] = v;
        } else {
            const int r = r0 + u, c = c0 + w;
            if (r < n && c < n) {
                const bool src_is_here = tr ? (r < c) : (r > c);  // this entry lies in the logical lower triangle
                if (!src_is_here && r != c)
                    xp[(int64_t)r * ld + c] = sb[w][u];
            }
        }
    }
    if (ti != tj) {
        for (int t = threadIdx.x; t < ET * ET; t += 256) {
            const int u = t / ET, w = t % ET;
            // entry (c0+u, r0+w) of tile (tj,ti) pairs with entry (r0+w, c0+u) = sa[w][u]
            const int r = c0 + u, c = r0 + w;
            if (r < n && c < n) {
                if (mode == 0) {
                    xp[(int64_t)r * ld + c] = scale * (sa[w][u] + sb[u][w]);
                } else {
                    const bool src_is_here = tr ? (r < c) : (r > c);
                    if (!src_is_here)
                        xp[(int64_t)r * ld + c] = sa[w][u];
                }
            }
        }
    }
}

template <typename T>
static la_status launch_sym(View<T> X, int64_t batch, int n, T scale, int mode, hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    const int nt = (n + ET - 1) / ET;
    const int64_t blocks = (int64_t)nt * nt * batch;
    if (blocks > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    LA_LAUNCH((k_sym<T>), dim3((unsigned)blocks), dim3(256), 0, st, X, batch, n, scale, mode, nt);
    return launch_check("sym");
}
template <typename T>
la_status launch_symmetrize(View<T> X, int64_t batch, int n, T scale, hipStream_t st)
{
    return launch_sym<T>(X, batch, n, scale, 0, st);
}
template <typename T>
la_status launch_mirror_lower(View<T> X, int64_t batch, int n, hipStream_t st)
{
    return launch_sym<T>(X, batch, n, T(1), 1, st);
}

// One wavefront per matrix: out[b] = sum_i log L[b,i,i].
template <typename T>
__global__ __launch_bounds__(WAVE) void k_sumlogdiag(const T *L, T *out, int64_t batch, int n)
{
    const int64_t b = blockIdx.x;
    const T *lp = L + b * (int64_t)n * n;
    double s = 0.0;
    for (int i = threadIdx.x; i < n; i += WAVE)
        s += (double)log(lp[(int64_t)i * n + i]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        s += __shfl_xor(s, off, WAVE);
    if (threadIdx.x == 0)
        out[b] = (T)s;
}

// n <= 32: G = 2^g >= n lanes per matrix, 64 / G matrices per wavefront (a wavefront per matrix
// leaves most lanes idle and needs a workgroup per matrix).
template <typename T>
__global__ __launch_bounds__(256) void k_sumlogdiag_small(const T *L, T *out, int64_t batch, int n, int G)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t b = t / G;
    const int i = (int)(t % G);
    double s = 0.0;
    if (b < batch && i < n)
        s = (double)log(L[b * (int64_t)n * n + (int64_t)i * n + i]);
    for (int off = G >> 1; off >= 1; off >>= 1)
        s += __shfl_xor(s, off, WAVE);
    if (b < batch && i == 0)
        out[b] = (T)s;
}

template <typename T>
la_status launch_sumlogdiag(const T *L, T *out, int64_t batch, int n, hipStream_t st)
{
    if (batch <= 0)
        return LA_OK;
    if (batch > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    if (n >= 1 && n <= 32) {
        int G = 1;
        while (G < n)
            G *= 2;
        const int64_t blocks = (batch * G + 255) / 256;
        if (blocks > 0x7fffffffll)
            return LA_ERR_UNSUPPORTED;
        LA_LAUNCH((k_sumlogdiag_small<T>), dim3((unsigned)blocks), dim3(256), 0, st, L, out, batch, n, G);
        return launch_check("sumlogdiag_small");
    }
    LA_LAUNCH((k_sumlogdiag<T>), dim3((unsigned)batch), dim3(WAVE), 0, st, L, out, batch, n);
    return launch_check("sumlogdiag");
}

// loss = 1/2 y.alpha + sum log l_ii, Lbar = -tril(alpha z^T) + diag(1/l_ii).  A workgroup writes
// GLUE_ROWS rows of Lbar, a wavefront whole rows (no index arithmetic beyond the row loop); the
// first workgroup of a matrix also computes its loss.
constexpr int GLUE_THREADS = 1024;
constexpr int GLUE_ROWS = 64;
template <typename T>
__global__ __launch_bounds__(GLUE_THREADS) void k_gp_glue(const T *L, const T *y, const T *z, const T *alpha, T *loss,
                                                          T *Lbar, int64_t batch, int n, int chunks)
{
    __shared__ double red[GLUE_THREADS / WAVE];
    const int64_t b = blockIdx.x / chunks;
    const int chunk = (int)(blockIdx.x % chunks);
    const T *lp = L + b * (int64_t)n * n;
    const T *yp = y + b * n, *zp = z + b * n, *ap = alpha + b * n;
    T *gp = Lbar + b * (int64_t)n * n;
    const int w = threadIdx.x / WAVE, l = threadIdx.x % WAVE;
    const int r1 = min(n, (chunk + 1) * GLUE_ROWS);
    for (int i = chunk * GLUE_ROWS + w; i < r1; i += GLUE_THREADS / WAVE) {
        const T ai = ap[i];
        const T dinv = T(1) / lp[(int64_t)i * n + i];
        T *row = gp + (int64_t)i * n;
        for (int j = l; j < n; j += WAVE) {
            T g = (j <= i) ? -ai * zp[j] : T(0);
            if (j == i)
                g += dinv;
            row[j] = g;
        }
    }
    if (chunk != 0)
        return;
    double s = 0.0;
    for (int i = threadIdx.x; i < n; i += GLUE_THREADS)
        s += 0.5 * (double)yp[i] * (double)ap[i] + (double)log(lp[(int64_t)i * n + i]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        s += __shfl_xor(s, off, WAVE);
    if (l == 0)
        red[w] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int q = 0; q < GLUE_THREADS / WAVE; ++q)
            t += red[q];
        loss[b] = (T)t;
    }
}

template <typename T>
la_status launch_gp_glue(const T *L, const T *y, const T *z, const T *alpha, T *loss, T *Lbar, int64_t batch, int n,
                         hipStream_t st)
{
    if (batch <= 0)
        return LA_OK;
    const int chunks = n > 0 ? (n + GLUE_ROWS - 1) / GLUE_ROWS : 1;
    if (batch * chunks > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    LA_LAUNCH((k_gp_glue<T>), dim3((unsigned)(batch * chunks)), dim3(GLUE_THREADS), 0, st, L, y, z, alpha, loss,
                       Lbar, batch, n, chunks);
    return launch_check("gp_glue");
}

// ---------------------------------------------------------------------------------------
// Small pieces of the sparse-GP criterion (section 3.2): sums, a diagonal shift, a rank-1 update,
// the scalar formulas.
// ---------------------------------------------------------------------------------------
constexpr int RED_BLOCKS = SGP_PARTIALS;  // partial sums per quantity

// kind 0: sum a_i^2, 1: sum a_i, 2: sum a_i b_i, 3: sum of a_{i (ld + 1)} (trace of an ld x ld matrix),
// 4: sum log a_{i (ld + 1)}.  One fp64 partial sum per block; k_sgp_scalars adds them up.
template <typename T>
__global__ __launch_bounds__(256) void k_partial_sums(int kind, const T *a, const T *b, int64_t count, int64_t ld,
                                                      double *partial)
{
    __shared__ double red[4];
    double s = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) {
        if (kind == 0)
            s += (double)a[i] * (double)a[i];
        else if (kind == 1)
            s += (double)a[i];
        else if (kind == 2)
            s += (double)a[i] * (double)b[i];
        else if (kind == 3)
            s += (double)a[i * (ld + 1)];
        else
            s += log((double)a[i * (ld + 1)]);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        s += __shfl_xor(s, off, WAVE);
    if ((threadIdx.x & 63) == 0)
        red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0)
        partial[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}

template <typename T>
la_status launch_partial_sums(int kind, const T *a, const T *b, int64_t count, int64_t ld, double *partial,
                              hipStream_t st)
{
    LA_LAUNCH((k_partial_sums<T>), dim3(RED_BLOCKS), dim3(256), 0, st, kind, a, b, count, ld, partial);
    return launch_check("partial_sums");
}

// A(i,i) += v on an n x n row-major matrix
template <typename T>
__global__ void k_add_diag(T *A, int n, T v)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n)
        A[(int64_t)i * n + i] += v;
}
template <typename T>
la_status launch_add_diag(T *A, int n, T v, hipStream_t st)
{
    LA_LAUNCH((k_add_diag<T>), dim3((n + 255) / 256), dim3(256), 0, st, A, n, v);
    return launch_check("add_diag");
}

// C(i,j) += u_i v_j on rows x cols (row-major); fill != 0: C(i, j) = value instead (rows = 1)
template <typename T>
__global__ __launch_bounds__(256) void k_rank1_add(T *C, const T *u, const T *v, int rows, int cols)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t row = e / cols;  // one division per thread
    if (row < rows)
        C[e] += u[row] * v[e - row * cols];
}
template <typename T>
la_status launch_rank1_add(T *C, const T *u, const T *v, int rows, int cols, hipStream_t st)
{
    const int64_t total = (int64_t)rows * cols;
    LA_LAUNCH((k_rank1_add<T>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, C, u, v, rows, cols);
    return launch_check("rank1_add");
}

// Scalars of the criterion from the partial sums.  sums[q * RED_BLOCKS ..]: q = 0 |y|^2, 1 |w|^2,
// 2 |B|_F^2, 3 sum Kff_diag, 4 sum log La_ii, 5 sum Abar o A, 6 trace Abar.
// stage 0: phi.  stage 1: noise_bar and the constant Kff_diag_bar (first entry; a copy kernel spreads it).
template <typename T>
__global__ void k_sgp_scalars(int stage, const double *sums, double lam, int n, T *phi, T *noise_bar, T *kff_bar, int nk)
{
    __shared__ double tot[7];
    if (threadIdx.x < 7) {
        double t = 0.0;
        for (int i = 0; i < RED_BLOCKS; ++i)
            t += sums[threadIdx.x * RED_BLOCKS + i];
        tot[threadIdx.x] = t;
    }
    __syncthreads();
    const double yy = tot[0], ww = tot[1], bb = tot[2], kk = tot[3], logdet = tot[4], sa = tot[5] - tot[6];
    if (stage == 0) {
        if (threadIdx.x == 0)
            phi[0] = (T)((1.8378770664093454835606594728112 + log(lam)) * n / 2.0 + logdet + yy / (2.0 * lam) -
                         ww / (2.0 * lam * lam) - (bb - kk) / (2.0 * lam));
    } else {
        if (threadIdx.x == 0 && blockIdx.x == 0)
            noise_bar[0] = (T)(n / (2.0 * lam) - yy / (2.0 * lam * lam) + ww / (lam * lam * lam) +
                               (bb - kk) / (2.0 * lam * lam) - sa / lam);
        for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < nk; i += gridDim.x * blockDim.x)
            kff_bar[i] = (T)(1.0 / (2.0 * lam));
    }
}
template <typename T>
la_status launch_sgp_scalars(int stage, const double *sums, double lam, int n, T *phi, T *noise_bar, T *kff_bar, int nk,
                             hipStream_t st)
{
    const int blocks = stage == 0 ? 1 : (nk + 255) / 256;
    LA_LAUNCH((k_sgp_scalars<T>), dim3(blocks > 0 ? blocks : 1), dim3(256), 0, st, stage, sums, lam, n, phi,
                       noise_bar, kff_bar, nk);
    return launch_check("sgp_scalars");
}

__global__ void k_fill_i32(int32_t *p, int64_t count, int32_t v)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count)
        p[i] = v;
}

la_status launch_fill_i32(int32_t *p, int64_t count, int32_t v, hipStream_t st)
{
    if (count <= 0)
        return LA_OK;
    LA_LAUNCH(k_fill_i32, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, p, count, v);
    return launch_check("fill");
}

#define LA_INST(T)                                                                                              \
    template la_status launch_copy<T>(View<const T>, View<T>, int64_t, int, int, T, int, hipStream_t);          \
    template la_status launch_tril_split<T>(View<const T>, View<T>, View<T>, int64_t, int, hipStream_t);        \
    template la_status launch_zero_strict_upper<T>(View<T>, int64_t, int, hipStream_t);                         \
    template la_status launch_symmetrize<T>(View<T>, int64_t, int, T, hipStream_t);                             \
    template la_status launch_mirror_lower<T>(View<T>, int64_t, int, hipStream_t);                              \
    template la_status launch_sumlogdiag<T>(const T *, T *, int64_t, int, hipStream_t);                         \
    template la_status launch_partial_sums<T>(int, const T *, const T *, int64_t, int64_t, double *, hipStream_t); \
    template la_status launch_add_diag<T>(T *, int, T, hipStream_t);                                            \
    template la_status launch_rank1_add<T>(T *, const T *, const T *, int, int, hipStream_t);                   \
    template la_status launch_sgp_scalars<T>(int, const double *, double, int, T *, T *, T *, int, hipStream_t); \
    template la_status launch_gp_glue<T>(const T *, const T *, const T *, const T *, T *, T *, int64_t, int,    \
                                         hipStream_t);
LA_INST(float)
LA_INST(double)

}  // namespace la
