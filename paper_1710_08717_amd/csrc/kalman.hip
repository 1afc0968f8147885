// Kalman filter over a batch of sequences (section 3.4, "Kalman Filtering"): every matrix of
// the recursion is at most 16 x 16, so one sequence lives in D = 16 lanes for its whole length --
// lane r holds row r of each matrix in registers (zero padded to D columns), vectors have one
// element per lane -- and a wavefront carries four sequences; with all dimensions <= 4 the same
// code runs with D = 4 and sixteen sequences per wavefront.  Nothing but the observation v_t
// is read and nothing but f_t, F_t is written per step.
//
// With rows in lanes, both product shapes of the recursion are chains of one instruction, a
// multiply-add whose second factor is broadcast from one lane of the group (DPP row_newbcast for
// 16 lanes, DPP quad_perm for 4):
//   C = X Y    C[r][j] += X[r][k] * (Y[k][j]: register j of lane k)
//   C = X Y^T  C[r][j] += X[r][k] * (Y[j][k]: register k of lane j)
// and the right-side triangular solves of the gain matrix work on rows, i.e. inside a lane.
// The parameters (A, B, S_h, S_v) wait in LDS and a lane fetches its row before each use.
#include "common.hpp"

namespace la {

template <typename T, int D>  // D: lanes per sequence = padded dimension (16, 8 or 4)
struct KfLds {
    static constexpr int GROUPS = 64 / D;                // sequences per workgroup (one wavefront)
    static constexpr int PS = D + 16 / (int)sizeof(T);   // row stride: 16-byte row reads of 16 lanes hit all banks
    static constexpr int MAT = D * PS;
    static constexpr int GROUP = 4 * MAT;  // A, B, S_h, S_v
    static constexpr size_t BYTES = (size_t)GROUPS * GROUP * sizeof(T);
};

// acc <- acc +- other * (src of lane K of the D-lane group)
template <int K>
__device__ __forceinline__ void fmac_quad(float &acc, float src, float other, bool neg)
{
    if (neg)
        asm volatile("v_fmac_f32_dpp %0, -%1, %2 quad_perm:[%3,%3,%3,%3] row_mask:0xf bank_mask:0xf"
                     : "+v"(acc)
                     : "v"(src), "v"(other), "n"(K));
    else
        asm volatile("v_fmac_f32_dpp %0, %1, %2 quad_perm:[%3,%3,%3,%3] row_mask:0xf bank_mask:0xf"
                     : "+v"(acc)
                     : "v"(src), "v"(other), "n"(K));
}
template <int K>
__device__ __forceinline__ void fmac_quad(double &acc, double src, double other, bool neg)
{
    // 64-bit DPP has no quad_perm: two 32-bit lane moves, then a plain multiply-add
    constexpr int ctrl = K | (K << 2) | (K << 4) | (K << 6);
    const long long v = __builtin_bit_cast(long long, src);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(v & 0xffffffffll), ctrl, 0xf, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(v >> 32), ctrl, 0xf, 0xf, false);
    const double b = __builtin_bit_cast(double, ((long long)hi << 32) | (unsigned int)lo);
    acc = fma(neg ? -other : other, b, acc);
}
template <int D, int K, typename T>
__device__ __forceinline__ void kf_fma(T &acc, T src, T other, bool neg)
{
    if constexpr (D == 16 || D == 8)  // D == 8: two sequences per 16-lane row, the instruction once per half
        fma_bcast<D, K>(acc, src, other, neg);
    else
        fmac_quad<K>(acc, src, other, neg);
}
// two wait states between a vector write of a register and a DPP read of it inside inline asm
template <typename T, int N>
__device__ __forceinline__ void kf_settle(T (&v)[N])
{
#pragma unroll
    for (int i = 0; i < N; ++i)
        asm volatile("" : "+v"(v[i]));
    asm volatile("s_nop 1");
}
template <typename T>
__device__ __forceinline__ void kf_settle1(T &v)
{
    asm volatile("s_nop 1" : "+v"(v));
}

template <typename T>
struct KfArgs {
    const T *A, *B, *Sh, *Sv, *mu0, *S0, *v;
    T *f, *F, *nll;
    int32_t *info;
    int64_t batch;
    int T_, dh, dv, shared;
};

// f(k) for k = 0 .. D-1 in ascending (or descending) order, in blocks of four; a block is skipped
// when all of it lies at or beyond `dim`.  (One uniform branch per block: a branch per index
// costs more scalar registers than there are.)  Indices between dim and the end of its block
// see the zero / identity padding.
template <int D, class Fn>
__device__ __forceinline__ void kf_upto(int dim, Fn &&fn)
{
    static_for<0, D / 4>([&](auto bc) {
        constexpr int b0 = 4 * decltype(bc)::value;
        if (b0 < dim) {
            static_for<0, 4>([&](auto ic) { fn(std::integral_constant<int, b0 + decltype(ic)::value>{}); });
        }
    });
}
template <int D, class Fn>
__device__ __forceinline__ void kf_downfrom(int dim, Fn &&fn)
{
    static_for<0, D / 4>([&](auto bc) {
        constexpr int b0 = D - 4 - 4 * decltype(bc)::value;
        if (b0 < dim) {
            static_for<0, 4>([&](auto ic) { fn(std::integral_constant<int, b0 + 3 - decltype(ic)::value>{}); });
        }
    });
}

// C[r][j] += sum_{k < kdim} X[r][k] Y[k][j]   (neg: subtract)
template <typename T, int D>
__device__ __forceinline__ void kf_nn(T (&C)[D], const T (&X)[D], T (&Y)[D], int kdim, bool neg = false)
{
    kf_settle(Y);
    kf_upto<D>(kdim, [&](auto kc) {
        constexpr int k = decltype(kc)::value;
        static_for<0, D>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            kf_fma<D, k>(C[j], Y[j], X[k], neg);
        });
    });
}

// C[r][j] += sum_k X[r][k] Y[j][k] for j < jdim
template <typename T, int D>
__device__ __forceinline__ void kf_nt(T (&C)[D], const T (&X)[D], T (&Y)[D], int jdim)
{
    kf_settle(Y);
    static_for<0, D / 4>([&](auto bc) {  // four columns at a time: their chains of multiply-adds interleave
        constexpr int b0 = 4 * decltype(bc)::value;
        if (b0 < jdim) {
            static_for<0, D>([&](auto kc) {
                constexpr int k = decltype(kc)::value;
                static_for<0, 4>([&](auto ic) {
                    constexpr int j = b0 + decltype(ic)::value;
                    kf_fma<D, j>(C[j], Y[k], X[k], false);
                });
            });
        }
    });
}

// c[r] += sum_{k < kdim} X[r][k] y[k]
template <typename T, int D>
__device__ __forceinline__ void kf_mv(T &c, const T (&X)[D], T &y, int kdim)
{
    kf_settle1(y);
    kf_upto<D>(kdim, [&](auto kc) {
        constexpr int k = decltype(kc)::value;
        kf_fma<D, k>(c, y, X[k], false);
    });
}

template <typename T, int D>
__device__ __forceinline__ void kf_zero(T (&x)[D])
{
#pragma unroll
    for (int j = 0; j < D; ++j)
        x[j] = T(0);
}

template <typename T, int D>
__device__ __forceinline__ void kf_row(T (&x)[D], const T *row)
{
#pragma unroll
    for (int j = 0; j < D; ++j)
        x[j] = row[j];
}

template <typename T, int D>
__global__ __launch_bounds__(64) void k_kalman(KfArgs<T> a)
{
    using Lds = KfLds<T, D>;
    constexpr int KF_D = D, KF_GROUPS = Lds::GROUPS;
    extern __shared__ __align__(16) unsigned char kf_smem[];
    const int lane = threadIdx.x, g = lane / D, r = lane % D;
    const int dh = a.dh, dv = a.dv, steps = a.T_;
    const int64_t b_raw = (int64_t)blockIdx.x * KF_GROUPS + g;
    const bool live = b_raw < a.batch;
    const int64_t b = live ? b_raw : a.batch - 1;  // a spare group repeats the last sequence and stores nothing
    const int64_t pb = a.shared ? 0 : b;

    // one copy of the parameters per sequence, or one for the workgroup when all sequences share them
    T *sA = reinterpret_cast<T *>(kf_smem) + (a.shared ? 0 : g * Lds::GROUP), *sB = sA + Lds::MAT,
      *sSh = sB + Lds::MAT, *sSv = sSh + Lds::MAT;
    if (!a.shared || g == 0) {   // parameters, zero padded (S_v: identity padded, so that the padded S_vv keeps a unit pivot)
        const T *Ap = a.A + pb * dh * dh, *Bp = a.B + pb * dv * dh, *Shp = a.Sh + pb * dh * dh, *Svp = a.Sv + pb * dv * dv;
#pragma unroll
        for (int j = 0; j < KF_D; ++j) {
            sA[r * Lds::PS + j] = (r < dh && j < dh) ? Ap[r * dh + j] : T(0);
            sB[r * Lds::PS + j] = (r < dv && j < dh) ? Bp[r * dh + j] : T(0);
            sSh[r * Lds::PS + j] = (r < dh && j < dh) ? Shp[r * dh + j] : T(0);
            sSv[r * Lds::PS + j] = (r < dv && j < dv) ? Svp[r * dv + j] : (r == j ? T(1) : T(0));
        }
    }
    __syncthreads();

    T F[KF_D];  // filtered covariance, row r
    T f = (r < dh) ? a.mu0[pb * dh + r] : T(0);
#pragma unroll
    for (int j = 0; j < KF_D; ++j)
        F[j] = (r < dh && j < dh) ? a.S0[pb * dh * dh + r * dh + j] : T(0);

    const T *vp = a.v + b * (int64_t)steps * dv;
    T vnext = (steps > 0 && r < dv) ? vp[r] : T(0);
    double nll_acc = 0.0;
    int32_t bad = 0;
    const T one = T(1);

    for (int t = 0; t < steps; ++t) {
        const T vt = vnext;
        if (t + 1 < steps && r < dv)
            vnext = vp[(int64_t)(t + 1) * dv + r];

        // ---- predicted state: mu_h, S_hh (the prior at t = 0) ----
        T Shh[KF_D];
        T muh;
        if (t == 0) {
            muh = f;
#pragma unroll
            for (int j = 0; j < KF_D; ++j)
                Shh[j] = F[j];
        } else {
            T Ar[KF_D], T1[KF_D];
            kf_row(Ar, sA + r * Lds::PS);
            muh = T(0);
            kf_mv(muh, Ar, f, dh);           // A f
            kf_zero(T1);
            kf_nt(T1, F, Ar, dh);            // F A^T
            kf_row(Shh, sSh + r * Lds::PS);
            kf_nn(Shh, Ar, T1, dh);          // S_h + A (F A^T)
        }

        // ---- predicted observation: mu_v, M = S_hh B^T, S_vv = B M + S_v ----
        T M[KF_D], S[KF_D];
        T muv = T(0);
        {
            T Br[KF_D];
            kf_row(Br, sB + r * Lds::PS);
            kf_mv(muv, Br, muh, dh);
            kf_zero(M);
            kf_nt(M, Shh, Br, dv);
            kf_row(S, sSv + r * Lds::PS);
            kf_nn(S, Br, M, dh);
        }

        // ---- S_vv = L L^T in place (lower triangle of S; lane r keeps 1 / L_rr) ----
        T invd = one;
        kf_upto<D>(dv, [&](auto kc) {
            constexpr int k = decltype(kc)::value;
            kf_settle1(S[k]);
            T d = T(0);
            kf_fma<D, k>(d, S[k], one, false);  // pivot, from lane k
            if (!(d > T(0)) && bad == 0)
                bad = t + 1;
            const T rs = one / sqrt(d);
            S[k] *= rs;
            if (r == k)
                invd = rs;
            kf_settle1(S[k]);
            static_for<k + 1, KF_D>([&](auto jc) {
                constexpr int j = decltype(jc)::value;
                kf_fma<D, j>(S[j], S[k], S[k], true);  // S[r][j] -= L[r][k] L[j][k]
            });
        });
#pragma unroll
        for (int j = 0; j < KF_D; ++j)
            S[j] = (j > r) ? T(0) : S[j];

        // ---- gain K = M L^-T L^-1, row by row inside each lane ----
        kf_settle(S);
        kf_settle1(invd);
        kf_upto<D>(dv, [&](auto jc) {  // X L^T = M
            constexpr int j = decltype(jc)::value;
            T x = T(0);
            kf_fma<D, j>(x, invd, M[j], false);
            M[j] = x;
            static_for<j + 1, KF_D>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                kf_fma<D, i>(M[i], S[j], x, true);  // M[r][i] -= x L[i][j]
            });
        });
        kf_downfrom<D>(dv, [&](auto jc) {  // K L = X
            constexpr int j = decltype(jc)::value;
            T y = T(0);
            kf_fma<D, j>(y, invd, M[j], false);
            M[j] = y;
            static_for<0, j>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                kf_fma<D, j>(M[i], S[i], y, true);  // M[r][i] -= y L[j][i]
            });
        });
        // M now holds K

        // ---- innovation, its likelihood term, filtered mean ----
        T delta = (r < dv) ? vt - muv : T(0);
        T fn = muh;
        kf_mv(fn, M, delta, dv);  // mu_h + K delta
        {
            T dl = delta, zfin = T(0);
            kf_upto<D>(dv, [&](auto kc) {  // z = L^-1 delta, one element per lane
                constexpr int k = decltype(kc)::value;
                T zs = dl * invd;
                if (r == k)
                    zfin = zs;
                kf_settle1(zs);
                kf_fma<D, k>(dl, zs, S[k], true);  // dl[r] -= L[r][k] z[k]
            });
            if (r < dv)
                nll_acc += 0.5 * (double)zfin * (double)zfin - (double)log(invd);
        }
        f = fn;

        // ---- filtered covariance F = (I - K B) S_hh (I - K B)^T + K S_v K^T ----
        T G[KF_D];
        {
            T Br[KF_D];
            kf_row(Br, sB + r * Lds::PS);
#pragma unroll
            for (int j = 0; j < KF_D; ++j)
                G[j] = (j == r) ? one : T(0);
            kf_nn(G, M, Br, dv, true);  // I - K B
        }
        {
            T T2[KF_D];
            kf_zero(T2);
            kf_nt(T2, Shh, G, dh);      // S_hh (I - K B)^T
            kf_zero(F);
            kf_nn(F, G, T2, dh);
        }
        {
            T Svr[KF_D], T3[KF_D];
            kf_row(Svr, sSv + r * Lds::PS);
            kf_zero(T3);
            kf_nt(T3, Svr, M, dh);      // S_v K^T
            kf_nn(F, M, T3, dv);        // + K (S_v K^T)
        }

        if (live && r < dh) {
            if (a.f)
                a.f[(b * steps + t) * dh + r] = f;
            if (a.F) {
                T *Fo = a.F + ((b * steps + t) * dh + r) * dh;
#pragma unroll
                for (int j = 0; j < KF_D; ++j)
                    if (j < dh)
                        Fo[j] = F[j];
            }
        }
    }

    // sum of the per-lane likelihood terms over the group, plus the constant
#pragma unroll
    for (int off = D / 2; off >= 1; off >>= 1)
        nll_acc += __shfl_xor(nll_acc, off, D);
    if (live && r == 0) {
        a.nll[b] = (T)(nll_acc + 0.5 * steps * dv * 1.8378770664093454835606594728112);  // log(2 pi)
        if (a.info)
            a.info[b] = bad;
    }
}

template <typename T, int D>
static la_status launch_kalman_d(const KfArgs<T> &a, hipStream_t st)
{
    using Lds = KfLds<T, D>;
    const int64_t blocks = (a.batch + Lds::GROUPS - 1) / Lds::GROUPS;
    if (blocks > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    const size_t lds = a.shared ? Lds::BYTES / Lds::GROUPS : Lds::BYTES;
    LA_LAUNCH((k_kalman<T, D>), dim3((unsigned)blocks), dim3(64), lds, st, a);
    return launch_check("kalman");
}

template <typename T>
la_status launch_kalman(const T *A, const T *B, const T *Sh, const T *Sv, const T *mu0, const T *S0, const T *v, T *f,
                        T *F, T *nll, int32_t *info, int64_t batch, int steps, int dh, int dv, int shared,
                        hipStream_t st)
{
    if (batch <= 0)
        return LA_OK;
    if (dh < 1 || dv < 1 || dh > 16 || dv > 16)
        return LA_ERR_UNSUPPORTED;
    KfArgs<T> a{A, B, Sh, Sv, mu0, S0, v, f, F, nll, info, batch, steps, dh, dv, shared};
    if (dh <= 4 && dv <= 4)
        return launch_kalman_d<T, 4>(a, st);
    // 8 lanes per sequence pay in fp32 only (1.76 -> 0.89 ms per 65536 x 32 steps at d = 8): in fp64 the
    // broadcast is four 32-bit lane moves beside the multiply-add and 16 lanes stay 4 % ahead
    if constexpr (sizeof(T) == 4) {
        if (dh <= 8 && dv <= 8)
            return launch_kalman_d<T, 8>(a, st);
    }
    return launch_kalman_d<T, 16>(a, st);
}

template la_status launch_kalman<float>(const float *, const float *, const float *, const float *, const float *,
                                        const float *, const float *, float *, float *, float *, int32_t *, int64_t,
                                        int, int, int, int, hipStream_t);
template la_status launch_kalman<double>(const double *, const double *, const double *, const double *,
                                         const double *, const double *, const double *, double *, double *, double *,
                                         int32_t *, int64_t, int, int, int, int, hipStream_t);

}  // namespace la
