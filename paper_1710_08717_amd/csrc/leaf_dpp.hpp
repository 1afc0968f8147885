// Row-per-lane helpers of the 16 x 16 tile routines (leaf.hip, trsm_stream.hip): multiply-adds whose
// second operand is a DPP row broadcast, and the inverse of a lower-triangular tile in registers.
#pragma once
#include "common.hpp"

namespace la {

constexpr int LT = 16;  // tile edge

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

// x = row r of the inverse of a 16 x 16 lower-triangular tile (a[c] = row r of the tile, dr its
// diagonal entry), columns shared out over the lane rows as in diag_factor_invert.  With
// m_rk = l_rk / l_kk the unit-triangular factor M = L diag(l)^-1 is inverted by
//   y_r. -= m_rk y_k.  (r > k),   k = 0, 1, ...   and   L^-1 = diag(l)^-1 M^-1.
template <typename T>
__device__ __forceinline__ void diag_invert(const T (&a)[LT], T dr, T (&x)[4], int r, int g)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        x[j] = (4 * j + g == r) ? T(1) : T(0);
        settle(x[j]);  // inside a loop the start values are copies made right here: keep them two wait states away
    }
    T rinv = rcp_newton(dr);
    settle(rinv);
    static_for<0, LT - 1>([&](auto kc) {
        constexpr int k = decltype(kc)::value;
        const T am = (r > k) ? a[k] : T(0);
        const T t = mul_row<k>(rinv, am);
        static_for<0, k / 4 + 1>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            fnmac_row_self<k>(x[j], t);
        });
    });
#pragma unroll
    for (int j = 0; j < 4; ++j)
        x[j] *= rinv;
}

}  // namespace la
