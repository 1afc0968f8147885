// Batched strided GEMM on the gfx950 matrix cores: the dense contraction inside every
// blocked algorithm of the library (trailing syrk/gemm update of the right-looking potrf,
// the off-diagonal updates of blocked trsm / trmm, and the three triangular phases of the
// potrf backward expression of arXiv 1710.08717, section 4.2).
//
//   C(i,j) = beta * C(i,j) + alpha * sum_k A(i,k) B(k,j)
//
// Operands are strided views (either index may be the contiguous one), so transposes and
// upper/lower variants never copy.  Triangular operands are masked while they are staged
// in LDS and their structurally-zero K range is skipped.
//
// Tiling: a 256-thread workgroup owns a BM x BN tile of C, four wavefronts in a 2 x 2
// arrangement, each accumulating (BM/2) x (BN/2) with 16x16x4 MFMA tiles
// (v_mfma_f64_16x16x4_f64 / v_mfma_f32_16x16x4_f32).  K advances in slabs of BK staged in LDS.
#include "common.hpp"

namespace la {

typedef double d4_t __attribute__((ext_vector_type(4)));
typedef float f4_t __attribute__((ext_vector_type(4)));

template <typename T>
struct Mfma;
template <>
struct Mfma<double> {
    using acc_t = d4_t;
    static __device__ __forceinline__ acc_t run(double a, double b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
    // accumulator register v of lane l holds D[row][l % 16]
    static __device__ __forceinline__ int row(int l, int v) { return (l >> 4) + 4 * v; }
};
template <>
struct Mfma<float> {
    using acc_t = f4_t;
    static __device__ __forceinline__ acc_t run(float a, float b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row(int l, int v) { return 4 * (l >> 4) + v; }
};

template <int BM, int BN, int BK>
struct GemmCfg {
    static constexpr int THREADS = 256;
    static constexpr int PAD = 16;
    // an operand slab is kept either "outer-fast" ([k][outer + PAD]) or "k-fast" ([outer][BK + 1]),
    // whichever matches the contiguous direction of its global memory
    static constexpr int A_ELEMS = (BK * (BM + PAD) > BM * (BK + 1)) ? BK * (BM + PAD) : BM * (BK + 1);
    static constexpr int B_ELEMS = (BK * (BN + PAD) > BN * (BK + 1)) ? BK * (BN + PAD) : BN * (BK + 1);
};

// Stage a (OUT x BK) slab: element (o, k) of the operand is src[o*so + k*sk] for o < no, k in
// [k0, k0+BK) & k < kmax; tri: 1 keeps o_glob >= k, 2 keeps o_glob <= k (o_glob = o0 + o), else zero.
template <typename T, int OUT, int BK, int PAD>
__device__ __forceinline__ void stage_slab(T *s, const T *src, int64_t so, int64_t sk, int o0, int no, int k0,
                                           int kmax, int tri, bool kfast)
{
    const int tid = threadIdx.x;
    constexpr int N = OUT * BK;
#pragma unroll
    for (int t = 0; t < N / 256; ++t) {
        const int idx = t * 256 + tid;
        int o, k;
        if (kfast) {
            o = idx / BK;
            k = idx % BK;
        } else {
            k = idx / OUT;
            o = idx % OUT;
        }
        const int og = o0 + o, kg = k0 + k;
        T v = T(0);
        bool ok = (og < no) && (kg < kmax);
        if (tri == 1)
            ok = ok && (og >= kg);
        else if (tri == 2)
            ok = ok && (og <= kg);
        if (ok)
            v = src[(int64_t)og * so + (int64_t)kg * sk];
        s[kfast ? (o * (BK + 1) + k) : (k * (OUT + PAD) + o)] = v;
    }
}

template <typename T, int BM, int BN, int BK>
__global__ __launch_bounds__(256) void k_gemm(View<const T> A, View<const T> B, View<T> C, int64_t batch, int M, int N,
                                              int K, T alpha, T beta, GemmOpts o, int tiles_m, int tiles_n)
{
    using Cfg = GemmCfg<BM, BN, BK>;
    using MF = Mfma<T>;
    using acc_t = typename MF::acc_t;
    constexpr int PAD = Cfg::PAD;
    constexpr int WM = BM / 2, WN = BN / 2;  // wave tile
    constexpr int TM = WM / 16, TN = WN / 16;
    __shared__ T sA[Cfg::A_ELEMS];
    __shared__ T sB[Cfg::B_ELEMS];

    const int64_t bid = blockIdx.x;
    const int64_t per = (int64_t)tiles_m * tiles_n;
    const int64_t b = bid / per;
    const int tile = (int)(bid % per);
    const int tm = tile / tiles_n, tn = tile % tiles_n;
    const int i0 = tm * BM, j0 = tn * BN;
    if (o.maskC == 1 && j0 > i0 + BM - 1)
        return;  // tile entirely above the diagonal

    int kbeg = 0, kend = K;
    if (o.triA == 1)
        kend = min(kend, i0 + BM);
    else if (o.triA == 2)
        kbeg = max(kbeg, i0);
    if (o.triB == 1)
        kbeg = max(kbeg, j0);
    else if (o.triB == 2)
        kend = min(kend, j0 + BN);
    kbeg = (kbeg / BK) * BK;

    const T *Ap = A.p + b * A.bs;
    const T *Bp = B.p + b * B.bs;
    T *Cp = C.p + b * C.bs;
    const bool a_kfast = (A.cs == 1);  // A(i,k): k contiguous
    const bool b_kfast = (B.rs == 1);  // B(k,j): k contiguous

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wm = (w >> 1) * WM, wn = (w & 1) * WN;
    const int l16 = lane & 15, lk = lane >> 4;

    acc_t acc[TM][TN];
#pragma unroll
    for (int x = 0; x < TM; ++x)
#pragma unroll
        for (int y = 0; y < TN; ++y)
            acc[x][y] = acc_t{0, 0, 0, 0};

    const int a_si = a_kfast ? (BK + 1) : 1, a_sk = a_kfast ? 1 : (BM + PAD);
    const int b_sj = b_kfast ? (BK + 1) : 1, b_sk = b_kfast ? 1 : (BN + PAD);

    for (int k0 = kbeg; k0 < kend; k0 += BK) {
        stage_slab<T, BM, BK, PAD>(sA, Ap, A.rs, A.cs, i0, M, k0, kend, o.triA, a_kfast);
        // B(k,j): "outer" index is j; its triangle test compares k against j, so swap the sense
        stage_slab<T, BN, BK, PAD>(sB, Bp, B.cs, B.rs, j0, N, k0, kend, o.triB == 1 ? 2 : (o.triB == 2 ? 1 : 0),
                                   b_kfast);
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; kk += 4) {
            T af[TM], bf[TN];
#pragma unroll
            for (int x = 0; x < TM; ++x)
                af[x] = sA[(wm + x * 16 + l16) * a_si + (kk + lk) * a_sk];
#pragma unroll
            for (int y = 0; y < TN; ++y)
                bf[y] = sB[(wn + y * 16 + l16) * b_sj + (kk + lk) * b_sk];
#pragma unroll
            for (int x = 0; x < TM; ++x)
#pragma unroll
                for (int y = 0; y < TN; ++y)
                    acc[x][y] = MF::run(af[x], bf[y], acc[x][y]);
        }
        __syncthreads();
    }

#pragma unroll
    for (int x = 0; x < TM; ++x)
#pragma unroll
        for (int y = 0; y < TN; ++y)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = i0 + wm + x * 16 + MF::row(lane, v);
                const int j = j0 + wn + y * 16 + l16;
                if (i < M && j < N && !(o.maskC == 1 && i < j)) {
                    T upd = alpha * acc[x][y][v];
                    if (o.halfDiag && i == j)
                        upd *= T(0.5);
                    T *c = Cp + (int64_t)i * C.rs + (int64_t)j * C.cs;
                    *c = (beta == T(0)) ? upd : fma(beta, *c, upd);
                }
            }
}

template <typename T>
la_status launch_gemm(View<const T> A, View<const T> B, View<T> C, int64_t batch, int M, int N, int K, T alpha, T beta,
                      GemmOpts o, hipStream_t st)
{
    if (batch <= 0 || M <= 0 || N <= 0)
        return LA_OK;
    constexpr int BM = 64, BN = 64, BK = 16;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int64_t blocks = (int64_t)tiles_m * tiles_n * batch;
    if (blocks > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((k_gemm<T, BM, BN, BK>), dim3((unsigned)blocks), dim3(256), 0, st, A, B, C, batch, M, N, K,
                       alpha, beta, o, tiles_m, tiles_n);
    return launch_check("gemm");
}

template la_status launch_gemm<float>(View<const float>, View<const float>, View<float>, int64_t, int, int, int, float,
                                      float, GemmOpts, hipStream_t);
template la_status launch_gemm<double>(View<const double>, View<const double>, View<double>, int64_t, int, int, int,
                                       double, double, GemmOpts, hipStream_t);

}  // namespace la
