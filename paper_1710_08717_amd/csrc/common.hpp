// Shared declarations of the gfx950 batched Cholesky library: status codes, the
// strided-view descriptors passed from the host dispatcher to the kernels, wavefront
// broadcast helpers and launcher prototypes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "la.h"

namespace la {

constexpr int WAVE = 64;
constexpr int NB = 64;  // edge of the triangular base-case tile of the blocked algorithms

// View of one matrix operand inside a batched buffer: element (i, j) of item b lives at
// base + b*bs + i*rs + j*cs (element units).  Row-major storage has cs == 1; the
// transposed view of the same memory swaps rs and cs, which is how an upper factor
// R = L^T (appendix, potrf, last paragraph) is handled without copying.
template <typename T>
struct View {
    T *p;
    int64_t bs, rs, cs;
    // optional second batch level: batch index q addresses item (q / nb2) and sub-item (q % nb2),
    // the latter bs2 elements apart (e.g. the diagonal blocks of one matrix)
    int64_t bs2 = 0;
    int32_t nb2 = 1;
    __host__ __device__ View<T> sub(int64_t i, int64_t j) const { return {p + i * rs + j * cs, bs, rs, cs, bs2, nb2}; }
    __host__ __device__ View<T> t() const { return {p, bs, cs, rs, bs2, nb2}; }
    __host__ __device__ View<T> level2(int64_t stride2, int32_t count2) const { return {p, bs, rs, cs, stride2, count2}; }
    __device__ T *item(int64_t q) const { return nb2 == 1 ? p + q * bs : p + (q / nb2) * bs + (q % nb2) * bs2; }
};

void set_error(hipError_t e, const char *where);

#define LA_HIP(call)                         \
    do {                                     \
        hipError_t e__ = (call);             \
        if (e__ != hipSuccess) {             \
            ::la::set_error(e__, #call);     \
            return LA_ERR_RUNTIME;           \
        }                                    \
    } while (0)

#define LA_TRY(call)                \
    do {                            \
        la_status s__ = (call);     \
        if (s__ != LA_OK)           \
            return s__;             \
    } while (0)

// ---------------------------------------------------------------------------------
// Scratch memory of one call.  The library owns no device memory: whatever a blocked path needs
// beyond its inputs and outputs (explicit inverses, working copies, partial results of products
// split along K) is carved out of the workspace the caller passed to that call, by a bump
// allocator that lives on the calling thread for the duration of the call.  A function that
// takes memory opens an ArenaFrame; what it took is handed back when the frame ends, so
// consecutive steps reuse the same bytes (the work is ordered by the stream).
// In a SIZING pass (dry) nothing is launched and no HIP call is made: the host code of the
// operator runs as usual and the arena only records the most it was asked for.
// ---------------------------------------------------------------------------------
struct Arena {
    char *base = nullptr;
    size_t cap = 0, used = 0, peak = 0;
    bool dry = false;
};
Arena *&current_arena();
inline bool dry_run()
{
    const Arena *a = current_arena();
    return a && a->dry;
}
// `bytes` of scratch (256-byte aligned) from the current call's workspace; LA_ERR_WORKSPACE if it is too small
la_status arena_take(size_t bytes, void **out);
struct ArenaFrame {
    size_t mark;
    ArenaFrame() : mark(current_arena() ? current_arena()->used : 0) {}
    ~ArenaFrame()
    {
        if (current_arena())
            current_arena()->used = mark;
    }
};
// every kernel launch of the library goes through here: a sizing pass launches nothing
#define LA_LAUNCH(...)                      \
    do {                                    \
        if (!::la::dry_run())               \
            hipLaunchKernelGGL(__VA_ARGS__); \
    } while (0)

inline la_status launch_check(const char *where)
{
    if (dry_run())
        return LA_OK;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error(e, where);
        return LA_ERR_RUNTIME;
    }
    return LA_OK;
}

// ---------------------------------------------------------------------------------
// Broadcast of one lane's value to the G lanes of its group (G = 4, 8, 16, 32 or 64).
// G = 16: DPP row_newbcast, folded by the compiler into the consuming VALU op.  G = 8: two such
// moves, one per half of the 16-lane row (bank mask).  G = 4: DPP quad_perm.
// G = 32: ds_bpermute through the LDS crossbar.  G = 64: v_readlane into an SGPR.
// ---------------------------------------------------------------------------------
template <int K>
__device__ __forceinline__ int dpp_row_bcast_i(int x)
{
    return __builtin_amdgcn_update_dpp(0, x, 0x150 + K, 0xf, 0xf, false);
}

__device__ __forceinline__ int row_bcast_i(int x, int k)
{
    switch (k & 15) {
    case 0: return dpp_row_bcast_i<0>(x);
    case 1: return dpp_row_bcast_i<1>(x);
    case 2: return dpp_row_bcast_i<2>(x);
    case 3: return dpp_row_bcast_i<3>(x);
    case 4: return dpp_row_bcast_i<4>(x);
    case 5: return dpp_row_bcast_i<5>(x);
    case 6: return dpp_row_bcast_i<6>(x);
    case 7: return dpp_row_bcast_i<7>(x);
    case 8: return dpp_row_bcast_i<8>(x);
    case 9: return dpp_row_bcast_i<9>(x);
    case 10: return dpp_row_bcast_i<10>(x);
    case 11: return dpp_row_bcast_i<11>(x);
    case 12: return dpp_row_bcast_i<12>(x);
    case 13: return dpp_row_bcast_i<13>(x);
    case 14: return dpp_row_bcast_i<14>(x);
    default: return dpp_row_bcast_i<15>(x);
    }
}

// lane K of its own HALF of the 16-lane row to all 8 lanes of that half: the row broadcast of
// lane K written to banks 0-1 (lanes 0..7), that of lane 8 + K to banks 2-3 (lanes 8..15)
template <int K>
__device__ __forceinline__ int dpp_half_bcast_i(int x)
{
    const int lo = __builtin_amdgcn_update_dpp(x, x, 0x150 + K, 0xf, 0x3, false);
    return __builtin_amdgcn_update_dpp(lo, x, 0x158 + K, 0xf, 0xc, false);
}
__device__ __forceinline__ int half_bcast_i(int x, int k)
{
    switch (k) {
    case 0: return dpp_half_bcast_i<0>(x);
    case 1: return dpp_half_bcast_i<1>(x);
    case 2: return dpp_half_bcast_i<2>(x);
    case 3: return dpp_half_bcast_i<3>(x);
    case 4: return dpp_half_bcast_i<4>(x);
    case 5: return dpp_half_bcast_i<5>(x);
    case 6: return dpp_half_bcast_i<6>(x);
    default: return dpp_half_bcast_i<7>(x);
    }
}

// lane k of each group of four lanes to the four of them (DPP quad_perm)
__device__ __forceinline__ int quad_bcast_i(int x, int k)
{
    switch (k & 3) {
    case 0: return __builtin_amdgcn_update_dpp(0, x, 0x00, 0xf, 0xf, false);
    case 1: return __builtin_amdgcn_update_dpp(0, x, 0x55, 0xf, 0xf, false);
    case 2: return __builtin_amdgcn_update_dpp(0, x, 0xaa, 0xf, 0xf, false);
    default: return __builtin_amdgcn_update_dpp(0, x, 0xff, 0xf, 0xf, false);
    }
}

template <int G>
__device__ __forceinline__ int group_bcast_i(int x, int k)
{
    if constexpr (G == 16) {
        return row_bcast_i(x, k);
    } else if constexpr (G == 8) {
        return half_bcast_i(x, k);
    } else if constexpr (G == 4) {
        return quad_bcast_i(x, k);
    } else if constexpr (G == 32) {
        int lane = __lane_id();
        return __builtin_amdgcn_ds_bpermute(((lane & 32) | k) << 2, x);
    } else {
        return __builtin_amdgcn_readlane(x, k);
    }
}

template <int G>
__device__ __forceinline__ float group_bcast(float x, int k)
{
    return __builtin_bit_cast(float, group_bcast_i<G>(__builtin_bit_cast(int, x), k));
}

template <int G>
__device__ __forceinline__ double group_bcast(double x, int k)
{
    long long v = __builtin_bit_cast(long long, x);
    int lo = group_bcast_i<G>((int)(v & 0xffffffffll), k);
    int hi = group_bcast_i<G>((int)(v >> 32), k);
    long long r = ((long long)hi << 32) | (unsigned int)lo;
    return __builtin_bit_cast(double, r);
}

// acc <- acc + other * (value of src in lane k of the group)   (neg: minus instead of plus)
//
// fp32 with 16-lane groups is the throughput-critical case: there the multiply-add and the
// broadcast are ONE instruction, v_fmac_f32 with a DPP row_newbcast source operand.  The
// compiler only forms that for plain multiplies, so it is written out.  The hardware needs
// two wait states between a VALU write of a register and a DPP read of it and nothing
// checks that inside inline asm: callers keep the broadcast source untouched for at least
// two instructions before the call (see dpp_settle()).
template <int K>
__device__ __forceinline__ void fmac_dpp16(float &acc, float src, float other)
{
    asm volatile("v_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
                 : "+v"(acc)
                 : "v"(src), "v"(other), "n"(K));
}
template <int K>
__device__ __forceinline__ void fnmac_dpp16(float &acc, float src, float other)
{
    asm volatile("v_fmac_f32_dpp %0, -%1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
                 : "+v"(acc)
                 : "v"(src), "v"(other), "n"(K));
}
// fp64: the same single instruction exists (64-bit DPP supports exactly this broadcast control)
template <int K>
__device__ __forceinline__ void fmac_dpp16(double &acc, double src, double other)
{
    asm volatile("v_fmac_f64_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
                 : "+v"(acc)
                 : "v"(src), "v"(other), "n"(K));
}
template <int K>
__device__ __forceinline__ void fnmac_dpp16(double &acc, double src, double other)
{
    asm volatile("v_fmac_f64_dpp %0, -%1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
                 : "+v"(acc)
                 : "v"(src), "v"(other), "n"(K));
}

// 8 lanes per group, two groups per 16-lane row: the same instruction twice, each writing one
// half of the row (bank mask) with the broadcast of that half's lane K.
template <int K>
__device__ __forceinline__ void fmac_dpp8(float &acc, float src, float other)
{
    asm volatile("v_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0x3\n\t"
                 "v_fmac_f32_dpp %0, %1, %2 row_newbcast:%4 row_mask:0xf bank_mask:0xc"
                 : "+v"(acc)
                 : "v"(src), "v"(other), "n"(K), "n"(K + 8));
}
template <int K>
__device__ __forceinline__ void fnmac_dpp8(float &acc, float src, float other)
{
    asm volatile("v_fmac_f32_dpp %0, -%1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0x3\n\t"
                 "v_fmac_f32_dpp %0, -%1, %2 row_newbcast:%4 row_mask:0xf bank_mask:0xc"
                 : "+v"(acc)
                 : "v"(src), "v"(other), "n"(K), "n"(K + 8));
}
// 4 lanes per group: the broadcast is a quad permutation (fp32 only; 64-bit DPP has no such control)
template <int K>
__device__ __forceinline__ void fmac_dpp4(float &acc, float src, float other)
{
    asm volatile("v_fmac_f32_dpp %0, %1, %2 quad_perm:[%3,%3,%3,%3] row_mask:0xf bank_mask:0xf"
                 : "+v"(acc)
                 : "v"(src), "v"(other), "n"(K));
}
template <int K>
__device__ __forceinline__ void fnmac_dpp4(float &acc, float src, float other)
{
    asm volatile("v_fmac_f32_dpp %0, -%1, %2 quad_perm:[%3,%3,%3,%3] row_mask:0xf bank_mask:0xf"
                 : "+v"(acc)
                 : "v"(src), "v"(other), "n"(K));
}
template <int G, int K, typename T>
__device__ __forceinline__ void fma_bcast(T &acc, T src, T other, bool neg)
{
    if constexpr (G == 16) {
        if (neg)
            fnmac_dpp16<K>(acc, src, other);
        else
            fmac_dpp16<K>(acc, src, other);
    } else if constexpr (G == 8 && sizeof(T) == 4) {
        if (neg)
            fnmac_dpp8<K>(acc, src, other);
        else
            fmac_dpp8<K>(acc, src, other);
    } else if constexpr (G == 4 && sizeof(T) == 4) {
        if (neg)
            fnmac_dpp4<K>(acc, src, other);
        else
            fmac_dpp4<K>(acc, src, other);
    } else {  // (fp64 with 8-lane groups too: the 64-bit DPP form gave wrong values with a partial bank mask)
        const T b = group_bcast<G>(src, K);
        acc = fma(neg ? -other : other, b, acc);
    }
}

// The 16-lane form for kernels whose fp64 state overflows the 256 vector registers: the compiler
// then parks values in accumulation registers and may copy one back (a vector write) right before
// the inline asm that reads it through DPP, which it cannot see; an s_nop inside the asm statement
// restores the two wait states.  fp32 kernels of that kind do not overflow and take the plain form.
template <int K, typename T>
__device__ __forceinline__ void fma_bcast16_guarded(T &acc, T src, T other, bool neg)
{
    if constexpr (sizeof(T) == 8) {
        if (neg)
            asm volatile("s_nop 1\n\tv_fmac_f64_dpp %0, -%1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
                         : "+v"(acc)
                         : "v"(src), "v"(other), "n"(K));
        else
            asm volatile("s_nop 1\n\tv_fmac_f64_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
                         : "+v"(acc)
                         : "v"(src), "v"(other), "n"(K));
    } else {
        fma_bcast<16, K, T>(acc, src, other, neg);
    }
}

// acc <- acc -/+ other * (acc's own value in lane K of the group).  With 8-lane groups the first
// instruction of the pair writes the register the second one reads through DPP (other lanes of
// it, but the wait states go by register), hence the s_nop between them.
template <int G, int K, typename T>
__device__ __forceinline__ void fma_bcast_self(T &acc, T other, bool neg)
{
    if constexpr (G == 8 && sizeof(T) == 4) {
        if (neg)
            asm volatile("v_fmac_f32_dpp %0, -%0, %1 row_newbcast:%2 row_mask:0xf bank_mask:0x3\n\ts_nop 1\n\t"
                         "v_fmac_f32_dpp %0, -%0, %1 row_newbcast:%3 row_mask:0xf bank_mask:0xc"
                         : "+v"(acc)
                         : "v"(other), "n"(K), "n"(K + 8));
        else
            asm volatile("v_fmac_f32_dpp %0, %0, %1 row_newbcast:%2 row_mask:0xf bank_mask:0x3\n\ts_nop 1\n\t"
                         "v_fmac_f32_dpp %0, %0, %1 row_newbcast:%3 row_mask:0xf bank_mask:0xc"
                         : "+v"(acc)
                         : "v"(other), "n"(K), "n"(K + 8));
    } else {
        fma_bcast<G, K, T>(acc, acc, other, neg);
    }
}

// Compile-time loop: f(std::integral_constant<int, I>) for I = B .. E-1, so that lane numbers
// reach the DPP / readlane encodings as constants without relying on the unroller.
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

// Makes every register of v[] "settled" for a following DPP read: two wait states, and the
// values are routed through the statement so that nothing that computes them can be moved
// after it.
template <int G, typename T, int N>
__device__ __forceinline__ void dpp_settle(T (&v)[N])
{
    if constexpr (G == 16 || (G <= 8 && sizeof(T) == 4)) {
#pragma unroll
        for (int i = 0; i < N; ++i)
            asm volatile("" : "+v"(v[i]));
        asm volatile("s_nop 1");
    }
}
template <int G, typename T>
__device__ __forceinline__ void dpp_settle1(T &v)
{
    if constexpr (G == 16 || (G <= 8 && sizeof(T) == 4)) {
        asm volatile("s_nop 1" : "+v"(v));
    }
}

// 16x16x4 matrix-core instruction of each element type and where its operands live:
// lane l supplies A(l % 16, l / 16) and B(l / 16, l % 16); accumulator register v of lane l
// holds D(row(l, v), l % 16).
typedef double d4_t __attribute__((ext_vector_type(4)));
typedef float f4_t __attribute__((ext_vector_type(4)));

template <typename T>
struct Mfma;
template <>
struct Mfma<double> {
    using acc_t = d4_t;
    using vec_t = double2;
    static constexpr int VW = 2;
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
    using vec_t = float4;
    static constexpr int VW = 4;
    static __device__ __forceinline__ acc_t run(float a, float b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row(int l, int v) { return 4 * (l >> 4) + v; }
};

// Reciprocal square root and reciprocal accurate to a few ulp of T.
__device__ __forceinline__ float rsqrt_acc(float x) { return __builtin_amdgcn_rsqf(x); }
__device__ __forceinline__ double rsqrt_acc(double x)
{
    // hardware seed (about 2^-26 relative), two Newton steps r <- r (1.5 - 0.5 x r^2)
    double r = __builtin_amdgcn_rsq(x);
    double h = 0.5 * x;
    r = r * fma(-h * r, r, 1.5);
    r = r * fma(-h * r, r, 1.5);
    return r;
}
__device__ __forceinline__ float rcp_acc(float x) { return 1.0f / x; }
__device__ __forceinline__ double rcp_acc(double x) { return 1.0 / x; }

// ---------------------------------------------------------------------------------
// Launchers (defined one per .hip file).  All take element-unit strides.
// ---------------------------------------------------------------------------------

// Register-resident potrf of blocks of edge nb <= G (G lanes per matrix), reading the
// lower triangle of A(i,j) and writing L(i,j) (zeros above the diagonal of the block).
// info (may be null): set to info_off + failing column (1-based) where it is still 0.
template <typename T>
la_status launch_potrf_tiny(View<const T> A, View<T> L, int32_t *info, int info_off, int64_t batch, int nb,
                            hipStream_t st);

// potrf of many matrices of 32 < n <= 64: four wavefronts per matrix, tiles in LDS, no inverse.  Writes the factor
// and zeros above the diagonal; A may alias L.  info as above (offset 0).
template <typename T>
la_status launch_potrf_small16(View<const T> A, View<T> L, int32_t *info, int64_t batch, int n, hipStream_t st);
// potrf of blocks of edge nb <= 128 together with the inverse of the factor, one workgroup per
// block: writes the factor's lower triangle (zeros above the diagonal inside the 16 x 16
// diagonal tiles; nothing else above it is written unless zero_upper, which zeroes all of L
// above the diagonal) and the lower triangle of its inverse (not stored when Inv.p is null).
// A may alias L.
// info (may be null): set to info_off + failing column (1-based) where it is still 0.
template <typename T>
la_status launch_potrf_leaf16(View<const T> A, View<T> L, View<T> Inv, int32_t *info, int info_off, int64_t batch,
                              int nb, bool zero_upper, hipStream_t st);

// Inverses of the 128 x 128 diagonal blocks of Lam (n x n lower triangular; the last block may be
// smaller) written onto the diagonal blocks of Inv (lower triangles; nothing else is written).
template <typename T>
la_status launch_tri_inverse128(View<const T> Lam, View<T> Inv, int64_t batch, int n, hipStream_t st);

// X <- alpha * Lam^-1 Xin (fwd) or alpha * Lam^-T Xin (!fwd) for n <= 128 and m <= 48 vectors
// X(e, v), one workgroup per batch item.  X may alias Xin.
template <typename T>
la_status launch_trsm_leaf16(View<const T> Lam, View<const T> Xin, View<T> X, int64_t batch, int n, int m, T alpha,
                             bool fwd, hipStream_t st);

// The same solve for 128 < n <= 512 as one launch: one workgroup per batch item and slab of 16
// vectors, the factor streamed from memory.  trsm_stream_takes says for which shapes that is the
// quicker way.  X may alias Xin.
template <typename T>
bool trsm_stream_takes(int64_t batch, int n, int m);
template <typename T>
la_status launch_trsm_stream(View<const T> Lam, View<const T> Xin, View<T> X, int64_t batch, int n, int m, T alpha,
                             bool fwd, hipStream_t st);

// potrf backward with one workgroup per matrix, everything in LDS as 16 x 16 tiles, for
// n <= backward_leaf16_max_n<T>() (128 in fp32, 96 in fp64).  Abar may alias G.
template <typename T>
int backward_leaf16_max_n();
template <typename T>
la_status launch_backward_leaf16(View<const T> Lam, View<const T> G, View<T> Abar, int64_t batch, int n, hipStream_t st);
// C = alpha U V^T for many items of 16 < n <= 128 (U, V: n x k views; C n x n), one workgroup per item, operands in
// LDS.  tri 0: V is U and C is written with both triangles, exactly symmetric; tri 1 / 2: the lower / upper triangle of
// the product is kept and the other one written as zeros.  outer_leaf_takes says whether the shape fits.
template <typename T>
bool outer_leaf_takes(int64_t batch, int n, int k, bool two);
template <typename T>
la_status launch_outer_leaf(int tri, T alpha, int64_t batch, int n, int k, View<const T> U, View<const T> V, View<T> C,
                            hipStream_t st);
// syrk backward in the same form: Out = alpha (G + G^T) A with G n x n, A and Out n x k views
template <typename T>
bool symm_leaf_takes(int64_t batch, int n, int k);
template <typename T>
la_status launch_symm_leaf(T alpha, int64_t batch, int n, int k, View<const T> G, View<const T> A, View<T> Out,
                           hipStream_t st);
// trmm in the same form: X = alpha M Xin with M = Lam (fwd) or Lam^T, Lam lower triangular, Xin and X n x m views
// (X may be Xin); no scratch
template <typename T>
bool trmm_leaf_takes(int64_t batch, int n, int m);
template <typename T>
la_status launch_trmm_leaf(View<const T> Lam, View<const T> Xin, View<T> X, int64_t batch, int n, int m, T alpha, bool fwd,
                           hipStream_t st);
// potri of matrices of edge n <= 128, one workgroup per matrix, no scratch: B = A^-1 (both triangles, exactly
// symmetric) from the lower factor Lam of A.  B may alias Lam.
template <typename T>
la_status launch_potri_leaf16(View<const T> Lam, View<T> B, int64_t batch, int n, hipStream_t st);

// trsm / trmm for n <= 64 with at most 16 vectors, any batch: the operand as flat items of n * m
// elements (stored m x n when img_tr), M = Lam (fwd) or Lam^T
template <typename T>
la_status launch_tri_tiny(bool solve, bool fwd, T alpha, int64_t batch, int n, int m, View<const T> Lam, const T *Bin,
                          T *Bout, bool img_tr, hipStream_t st);
// syrk for n <= 16 and inner dimension <= 32: A as flat items of n * k elements (stored k x n when img_tr)
template <typename T>
la_status launch_syrk_tiny(bool img_tr, T alpha, int64_t batch, int n, int k, const T *A, View<T> C, hipStream_t st);
// C = alpha U V^T (same shapes and limits; tri: 0 whole square, 1 / 2 lower / upper triangle kept, zeros elsewhere)
template <typename T>
la_status launch_outer_tiny(bool img_tr, int tri, T alpha, int64_t batch, int n, int k, const T *U, const T *V, View<T> C,
                            hipStream_t st);
// gemm2 for m, n, k <= 16: C = alpha op(A) op(B), contiguous row-major items
template <typename T>
la_status launch_gemm2_tiny(int ta, int tb, T alpha, int64_t batch, int m, int n, int k, const T *A, const T *B, T *C,
                            hipStream_t st);
// syrk backward for n <= 16, inner dimension <= 32: Out = alpha (Gb + Gb^T) A on flat items (stored k x n when img_tr)
template <typename T>
la_status launch_symm_tiny(bool img_tr, T alpha, int64_t batch, int n, int k, View<const T> Gb, const T *A, T *Out,
                           hipStream_t st);
// The same products for 16 < n <= 32 and k <= 32 (16 lanes per matrix, two rows per lane); outer_rows_takes
// says whether the shape fits (two images of fp64 operands can exceed the LDS of one workgroup).
template <typename T>
bool outer_rows_takes(int n, int k, bool two);
template <typename T>
la_status launch_outer_rows(bool img_tr, int tri, T alpha, int64_t batch, int n, int k, const T *U, const T *V, View<T> C,
                            hipStream_t st);
// trsm / trmm for 16 < n <= 32 and at most 16 vectors in that form (arguments as launch_tri_tiny)
template <typename T>
la_status launch_tri_rows(bool solve, bool fwd, T alpha, int64_t batch, int n, int m, View<const T> Lam, const T *Bin, T *Bout,
                          bool img_tr, hipStream_t st);
// syrk backward and gemm2 in the same form (n, respectively m, n and k, up to 32)
template <typename T>
bool symm_rows_takes(int n, int k);
template <typename T>
la_status launch_symm_rows(bool img_tr, T alpha, int64_t batch, int n, int k, View<const T> Gb, const T *A, T *Out,
                           hipStream_t st);
template <typename T>
bool gemm2_rows_takes(int m, int n, int k);
template <typename T>
la_status launch_gemm2_rows(int ta, int tb, T alpha, int64_t batch, int m, int n, int k, const T *A, const T *B, T *C,
                            hipStream_t st);
// potri for n <= 32: B = Lam^-T Lam^-1, exactly symmetric
template <typename T>
la_status launch_potri_tiny(View<const T> Lam, View<T> B, int64_t batch, int n, hipStream_t st);
// Register-resident potrf backward for n <= 32: Abar = sym(L^-T Phi(L^T Lbar) L^-1).
template <typename T>
la_status launch_backward_tiny(View<const T> L, View<const T> G, View<T> Abar, int64_t batch, int n,
                               hipStream_t st);

// C(i,j) = beta*C(i,j) + alpha * sum_k A(i,k) B(k,j), i < M, j < N, k < K, per batch item.
struct GemmOpts {
    int triA = 0;      // 1: A(i,k) is zero for i < k (lower), 2: zero for i > k (upper)
    int triB = 0;      // same on (k,j)
    int maskC = 0;     // 1: only entries with i >= j are written, 2: only i <= j; 3 (set by the launcher): only the
                       // tiles with tile column <= tile row, written whole
    int halfDiag = 0;  // 1: the update of entries with i == j is halved
    int reverse = 0;   // 1: schedule the tiles last-to-first (heavy tiles of triangular work first)
    int shells = 0;    // 1: square problem whose K range depends on max(i, j): schedule by shells
    int order = 0;     // tile enumeration, chosen by the launcher
    int ksplit = 0;      // set by the launcher: the batch index also counts `ksplit` slices of a K range of `ktotal`
    int ktotal = 0;
    int xcd_batch = 0;   // set by the launcher: batched launch, items dealt to the XCDs, tile-major inside
    int min_tile64 = 0;  // 1: no workgroup tiles smaller than 64 x 64 (a caller that updates C in place over <= 64 rows)
    int symsum = 0;      // 1: C = alpha (A B + (A B)^T) on a square C, both triangles written, exactly symmetric.  The
                         // tiles on and below the diagonal accumulate A B and then B^T A^T -- B^T must have A's strides and
                         // A^T B's, so the second pass only swaps the two base pointers -- and store every entry with its
                         // mirror image.  beta and maskC are not used.
};
template <typename T>
la_status launch_gemm(View<const T> A, View<const T> B, View<T> C, int64_t batch, int M, int N, int K, T alpha,
                      T beta, GemmOpts o, hipStream_t st);


// Element-wise helpers.
// dst(i,j) = alpha * src(i,j) on rows x cols; keep: 0 all, 1 only i >= j (rest written as 0), 2 only i >= j
// (rest not written).
template <typename T>
la_status launch_copy(View<const T> src, View<T> dst, int64_t batch, int rows, int cols, T alpha, int keep,
                      hipStream_t st);
// work(i,j) = src(i,j) for i >= j and out(i,j) = 0 for i < j on n x n; nothing else is written
// (out may alias src).
template <typename T>
la_status launch_tril_split(View<const T> src, View<T> work, View<T> out, int64_t batch, int n, hipStream_t st);
// X(i,j) = 0 for i < j on n x n; nothing else is written (pass X.t() to clear below the diagonal).
template <typename T>
la_status launch_zero_strict_upper(View<T> X, int64_t batch, int n, hipStream_t st);
// X <- scale * (X + X^T) on n x n (exactly symmetric result).
template <typename T>
la_status launch_symmetrize(View<T> X, int64_t batch, int n, T scale, hipStream_t st);
// X(i,j) <- X(j,i) for i < j (copy the lower triangle over the upper).
template <typename T>
la_status launch_mirror_lower(View<T> X, int64_t batch, int n, hipStream_t st);
template <typename T>
la_status launch_sumlogdiag(const T *L, T *out, int64_t batch, int n, hipStream_t st);
template <typename T>
la_status launch_gp_glue(const T *L, const T *y, const T *z, const T *alpha, T *loss, T *Lbar, int64_t batch, int n,
                         hipStream_t st);
la_status launch_fill_i32(int32_t *p, int64_t count, int32_t v, hipStream_t st);

// Pieces of the sparse-GP criterion (section 3.2).
constexpr int SGP_PARTIALS = 256;  // fp64 partial sums per reduced quantity
// kind 0: sum a^2, 1: sum a, 2: sum a b, 3: trace of the ld x ld matrix a (count = ld), 4: sum of the
// logs of its diagonal; writes SGP_PARTIALS partial sums
template <typename T>
la_status launch_partial_sums(int kind, const T *a, const T *b, int64_t count, int64_t ld, double *partial,
                              hipStream_t st);
template <typename T>
la_status launch_add_diag(T *A, int n, T v, hipStream_t st);
template <typename T>
la_status launch_rank1_add(T *C, const T *u, const T *v, int rows, int cols, hipStream_t st);
// sums: 7 x SGP_PARTIALS partial sums (|y|^2, |w|^2, |B|^2, sum Kff_diag, sum log La_ii, sum Abar o A,
// trace Abar); stage 0 writes phi, stage 1 noise_bar and the constant Kff_diag_bar
template <typename T>
la_status launch_sgp_scalars(int stage, const double *sums, double lam, int n, T *phi, T *noise_bar, T *kff_bar, int nk,
                             hipStream_t st);

// Gaussian-process criterion and gradient, one workgroup per matrix (leaf.hip); n <= backward_leaf16_max_n.
template <typename T>
la_status launch_gp_leaf16(View<const T> A, const T *y, T *loss, View<T> Abar, int32_t *info, int64_t batch, int n,
                           hipStream_t st);

// Kalman filter over a batch of sequences, dimensions up to 16 (kalman.hip).
template <typename T>
la_status launch_kalman(const T *A, const T *B, const T *Sh, const T *Sv, const T *mu0, const T *S0, const T *v, T *f,
                        T *F, T *nll, int32_t *info, int64_t batch, int steps, int dh, int dv, int shared,
                        hipStream_t st);

}  // namespace la
