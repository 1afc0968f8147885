// Staging helpers shared by the small-matrix kernels (tiny.hip, tiny_ops.hip): the padded LDS stage of
// G x G matrices, its coalesced fill and drain, and row / column reads by the lanes.
#pragma once
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
// (Leaving out the 16-byte pieces that lie entirely in the unused triangle was tried twice: the
// count of read requests from the L2 to memory did not move -- 1 049 966 against 1 050 040 per
// launch for 65536 fp32 matrices of 16 x 16, none of them of the 32-byte kind; a request moves a
// 128-byte line, i.e. two whole rows -- and the predicated loads made the kernel slower, 42.5
// against 36.6 us.)
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
        for (int t = 0; t < (NV + WAVE - 1) / WAVE; ++t) {
            if (NV % WAVE != 0 && t * WAVE + lane >= NV)
                break;
            int e = (t * WAVE + lane) * VN;
            int q = e / (G * G), r = (e / G) % G, c = e % G;
            // streamed once: non-temporal, so the lines do not linger in the caches
            *reinterpret_cast<V4 *>(sm + q * S::MS + r * S::LD + c) = __builtin_nontemporal_load(&src[t * WAVE + lane]);
        }
        return;
    }
    // all loads of a batch of 16 first, then the LDS writes: the loads are in flight together
    constexpr int NE = S::MPW * G * G, NIT = (NE + WAVE - 1) / WAVE, CH = NIT < 16 ? NIT : 16;
    for (int t0 = 0; t0 < NIT; t0 += CH) {
        T v[CH];
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int e = (t0 + u) * WAVE + lane;
            const int q = e / (G * G), r = (e / G) % G, c = e % G;
            v[u] = (r == c) ? T(1) : T(0);
            if (e < NE && b0 + q < batch && r < nb && c < nb)
                v[u] = M.p[(b0 + q) * M.bs + r * M.ld + c];
        }
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int e = (t0 + u) * WAVE + lane;
            const int q = e / (G * G), r = (e / G) % G, c = e % G;
            if (e < NE)
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
        for (int t = 0; t < (NV + WAVE - 1) / WAVE; ++t) {
            if (NV % WAVE != 0 && t * WAVE + lane >= NV)
                break;
            int e = (t * WAVE + lane) * VN;
            int q = e / (G * G), r = (e / G) % G, c = e % G;
            __builtin_nontemporal_store(*reinterpret_cast<const V4 *>(sm + q * S::MS + r * S::LD + c),
                                        &dst[t * WAVE + lane]);
        }
        return;
    }
#pragma unroll 4
    for (int t = 0; t < (S::MPW * G * G + WAVE - 1) / WAVE; ++t) {
        int e = t * WAVE + lane;
        int q = e / (G * G);
        int r = (e / G) % G, c = e % G;
        if (e < S::MPW * G * G && b0 + q < batch && r < nb && c < nb)
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
// Operands that are not square travel as flat memory images of whole items through LDS.  The LDS
// index of image element e is e + e / 16, so that 16 lanes reading a column of a 16-wide image
// (stride 16) fall into different banks.
// ---------------------------------------------------------------------------------
__device__ __forceinline__ int img_idx(int e) { return e + (e >> 4); }

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

}  // namespace la
