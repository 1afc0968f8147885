// Diagonal-block leaf of the blocked potrf (section 4.2 of arXiv 1710.08717: A = L L^T):
// one workgroup factors a block of edge nb <= 128 AND inverts the factor, because every panel
// solve against this block later multiplies by that inverse.
//
// The block is cut into 16 x 16 tiles that live in LDS for the whole kernel.  Step k of the
// right-looking sweep over the K = ceil(nb / 16) tile columns:
//   (a) one wavefront factors the diagonal tile A_kk and inverts the factor in registers
//       (lane = row, registers = columns, column broadcasts are DPP operands of the
//       multiply-adds): L_kk, Li_kk;
//   (b) panel      L_ik = A_ik Li_kk^T  (i > k)   and   X_kj <- Li_kk X_kj  (j < k), which
//       completes row k of the inverse X = L^-1;
//   (c) trailing   A_ij -= L_ik L_jk^T  (k < j <= i)   and   X_ij -= L_ik X_kj  (i > k, j <= k).
// (b) and (c) are 16 x 16 x 16 products on the matrix cores, one tile per wavefront at a
// time.  The 16 * K pivots are strictly sequential, so what counts is the chain
//   (a) -> panel tile (k+1, k) -> update of tile (k+1, k+1) -> (a) of the next step:
// wavefront 0 walks exactly that chain while the other seven do the rest of (b) and (c) of
// step k behind it (two workgroup barriers per step).
#include "common.hpp"
#include "leaf_dpp.hpp"

#ifndef LEAF16_STAMP
#define LEAF16_STAMP(i)
#endif

namespace la {

constexpr int LK = 8;               // tiles per block edge (128 / 16)
constexpr int LEAF16_THREADS = 1024;
constexpr int LEAF16_WAVES = LEAF16_THREADS / 64;

template <typename T>
struct Leaf16 {
    // row stride of the diagonal tiles (padded so that "lane = row" accesses spread over the
    // banks and stay 16-byte aligned)
    static constexpr int PS = LT + 16 / (int)sizeof(T);
    static constexpr int DT = LT * PS;            // elements of a padded diagonal tile
    static constexpr int OT = LT * LT;            // elements of an off-diagonal tile
    static constexpr int NOFF = LK * (LK - 1) / 2;
    // LDS map (elements): diagonal tiles of A/L, diagonal tiles of X, off-diagonal of A/L, of X
    static constexpr int OFF_D = 0;
    static constexpr int OFF_XD = OFF_D + LK * DT;
    static constexpr int OFF_A = OFF_XD + LK * DT;
    static constexpr int OFF_X = OFF_A + NOFF * OT;
    static constexpr int TOTAL = OFF_X + NOFF * OT;
};

__device__ __forceinline__ int tri_off(int i, int j) { return i * (i - 1) / 2 + j; }  // i > j

// Factor and invert one 16 x 16 tile held one row per lane.  All four 16-lane rows of the
// wavefront factor copies of the same tile; the inverse is shared out between them: in lane row
// g register x[j] is column 4 j + g of the inverse.
// In: a[c] = A(r, c) for c <= r (what lies above the diagonal is never looked at).
// Out: a[c] = L(r, c) for c <= r, x[j] = L^-1(r, 4 j + g) (entries above the diagonal hold
// leftovers, respectively zero) and the return value is the 1-based index of the first pivot that
// is not > 0, or 0.
//
// The pivots run on the unscaled matrix,   a_rc -= a_rk a_ck / a_kk,   x_rc -= a_rk x_kc / a_kk,
// which needs only a reciprocal on the critical path (started as soon as the next pivot is final);
// the square roots are taken for all 16 pivots at once afterwards:
// L = A_raw diag(d)^-1/2,  L^-1 = diag(d)^-1/2 X_raw.
template <typename T>
__device__ __forceinline__ int diag_factor_invert(T (&a)[LT], T (&x)[4], int r, int g)
{
    T d = T(1);
#pragma unroll
    for (int j = 0; j < 4; ++j)
        x[j] = (4 * j + g == r) ? T(1) : T(0);
    T rinv = rcp_newton(a[0]);  // meaningful in the pivot's lane only
    static_for<0, LT>([&](auto kc) {
        constexpr int k = decltype(kc)::value;
        const T am = (r > k) ? a[k] : T(0);
        d = (r == k) ? a[k] : d;
        settle(rinv);
        const T t = mul_row<k>(rinv, am);  // a_rk / a_kk below the pivot, zero elsewhere
        if constexpr (k + 1 < LT) {
            fnmac_row<k + 1>(a[k + 1], a[k], t);
            rinv = rcp_newton(a[k + 1]);  // overlaps the rest of this pivot's updates
        }
        static_for<k + 2, LT>([&](auto cc) {
            constexpr int c = decltype(cc)::value;
            fnmac_row<c>(a[c], a[k], t);  // a_rc -= a_ck t_r
        });
        static_for<0, k / 4 + 1>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            fnmac_row_self<k>(x[j], t);  // x_rc -= x_kc t_r (a no-op where column c > k)
        });
    });
    const unsigned long long bad = __ballot(!(d > T(0)));
    T rs = rsqrt_acc(d);
    settle(rs);
    static_for<0, LT>([&](auto cc) {
        constexpr int c = decltype(cc)::value;
        a[c] = mul_row<c>(rs, a[c]);  // column c times d_c^-1/2
    });
#pragma unroll
    for (int j = 0; j < 4; ++j)
        x[j] *= rs;  // row r times d_r^-1/2
    const unsigned first = (unsigned)(bad & 0xffffu);
    return first ? __builtin_ctz(first) + 1 : 0;
}

// ---------------------------------------------------------------------------------------
// Tiles in LDS.  Diagonal tiles are stored with padded rows (stride PS) for the row-per-lane
// accesses of the factorisation.  Off-diagonal tiles are 16 x 16 without padding, with the
// 16-byte chunks of every row permuted by the row number, so that both access patterns of the
// matrix-core operands sweep all banks: a lane reading four consecutive elements of "its" row
// (rows 128 or 64 bytes apart would otherwise all start in the same bank), and 16 lanes reading
// one row.
// ---------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ int sw(int u, int w)  // element (u, w) of an off-diagonal tile
{
    constexpr int EPC = 16 / (int)sizeof(T);  // elements per 16-byte chunk
    constexpr int CPR = LT / EPC;             // chunks per row
    const int key = (sizeof(T) == 8 ? u : (u >> 1)) & (CPR - 1);
    return u * LT + (((w / EPC) ^ key) * EPC) + (w % EPC);
}

template <typename T>
struct TileRef {
    T *p;
    bool diag;  // padded diagonal tile (row stride PS, no permutation)
    __device__ __forceinline__ int at(int u, int w) const { return diag ? u * Leaf16<T>::PS + w : sw<T>(u, w); }
};

// Operand element k of the 16 x 16 x 16 contraction is dealt to lane group q = lane / 16 and
// register s as k = 4 q + s, the same for both operands, so that an operand stored with k
// contiguous is read as four consecutive elements (one or two 16-byte chunks) per lane.
//   op_rows: operand(i, k) = tile(i, k), this lane supplies i = lane % 16
//   op_nat:  operand(k, j) = tile(k, j), this lane supplies j = lane % 16
template <typename T>
__device__ __forceinline__ void op_rows(TileRef<T> t, int lane, T (&v)[4])
{
    using V = typename Mfma<T>::vec_t;
    const int u = lane & 15, q = lane >> 4;
    if constexpr (sizeof(T) == 8) {
        const V lo = *reinterpret_cast<const V *>(t.p + t.at(u, 4 * q));
        const V hi = *reinterpret_cast<const V *>(t.p + t.at(u, 4 * q + 2));
        v[0] = lo.x;
        v[1] = lo.y;
        v[2] = hi.x;
        v[3] = hi.y;
    } else {
        const V w = *reinterpret_cast<const V *>(t.p + t.at(u, 4 * q));
        v[0] = w.x;
        v[1] = w.y;
        v[2] = w.z;
        v[3] = w.w;
    }
}
template <typename T>
__device__ __forceinline__ void op_nat(TileRef<T> t, int lane, T (&v)[4])
{
#pragma unroll
    for (int s = 0; s < 4; ++s)
        v[s] = t.p[t.at(4 * (lane >> 4) + s, lane & 15)];
}
template <typename T>
__device__ __forceinline__ typename Mfma<T>::acc_t acc_load(TileRef<T> t, int lane)
{
    typename Mfma<T>::acc_t c;
#pragma unroll
    for (int v = 0; v < 4; ++v)
        c[v] = t.p[t.at(Mfma<T>::row(lane, v), lane & 15)];
    return c;
}
template <typename T>
__device__ __forceinline__ void acc_store(TileRef<T> t, int lane, typename Mfma<T>::acc_t c)
{
#pragma unroll
    for (int v = 0; v < 4; ++v)
        t.p[t.at(Mfma<T>::row(lane, v), lane & 15)] = c[v];
}
template <typename T>
__device__ __forceinline__ typename Mfma<T>::acc_t mma4(const T (&a)[4], const T (&b)[4], typename Mfma<T>::acc_t c,
                                                        bool neg)
{
#pragma unroll
    for (int s = 0; s < 4; ++s)
        c = Mfma<T>::run(neg ? -a[s] : a[s], b[s], c);
    return c;
}

template <typename T>
struct LeafLds {
    T *sD, *sXD, *sA, *sX;
    __device__ __forceinline__ TileRef<T> a(int i, int j) const  // tile (i, j) of A / L, i >= j
    {
        return i == j ? TileRef<T>{sD + i * Leaf16<T>::DT, true} : TileRef<T>{sA + tri_off(i, j) * Leaf16<T>::OT, false};
    }
    __device__ __forceinline__ TileRef<T> x(int i, int j) const  // tile (i, j) of the inverse, i >= j
    {
        return i == j ? TileRef<T>{sXD + i * Leaf16<T>::DT, true} : TileRef<T>{sX + tri_off(i, j) * Leaf16<T>::OT, false};
    }
};

// (a): diagonal tile k, by one whole wavefront
template <typename T>
__device__ __forceinline__ int leaf_diag(const LeafLds<T> &m, int k, int lane)
{
    constexpr int PS = Leaf16<T>::PS;
    const int r = lane & 15, g = lane >> 4;
    T a[LT], x[4];
    T *dk = m.sD + k * Leaf16<T>::DT + r * PS, *xk = m.sXD + k * Leaf16<T>::DT + r * PS;
    using V = typename Mfma<T>::vec_t;
    constexpr int VW = Mfma<T>::VW;
#pragma unroll
    for (int c = 0; c < LT; c += VW) {
        const V w = *reinterpret_cast<const V *>(dk + c);
        a[c] = w.x;
        a[c + 1] = w.y;
        if constexpr (VW == 4) {
            a[c + 2] = w.z;
            a[c + 3] = w.w;
        }
    }
    const int f = diag_factor_invert<T>(a, x, r, g);
    if (lane < LT) {
#pragma unroll
        for (int c = 0; c < LT; ++c)
            dk[c] = (c <= r) ? a[c] : T(0);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
        xk[4 * j + g] = (4 * j + g <= r) ? x[j] : T(0);
    return f;
}

// (b): L_ik = A_ik Li_kk^T
template <typename T>
__device__ __forceinline__ void leaf_panel(const LeafLds<T> &m, int i, int k, int lane)
{
    T av[4], bv[4];
    typename Mfma<T>::acc_t acc = {0, 0, 0, 0};
    op_rows<T>(m.a(i, k), lane, av);
    op_rows<T>(m.x(k, k), lane, bv);
    acc = mma4<T>(av, bv, acc, false);
    acc_store<T>(m.a(i, k), lane, acc);
}
// (b): X_kj <- Li_kk X_kj, j < k
template <typename T>
__device__ __forceinline__ void leaf_xrow(const LeafLds<T> &m, int k, int j, int lane)
{
    T av[4], bv[4];
    typename Mfma<T>::acc_t acc = {0, 0, 0, 0};
    op_rows<T>(m.x(k, k), lane, av);
    op_nat<T>(m.x(k, j), lane, bv);
    acc = mma4<T>(av, bv, acc, false);
    acc_store<T>(m.x(k, j), lane, acc);
}
// (c): A_ij -= L_ik L_jk^T, k < j <= i
template <typename T>
__device__ __forceinline__ void leaf_update_a(const LeafLds<T> &m, int i, int j, int k, int lane)
{
    T av[4], bv[4];
    op_rows<T>(m.a(i, k), lane, av);
    op_rows<T>(m.a(j, k), lane, bv);
    typename Mfma<T>::acc_t acc = acc_load<T>(m.a(i, j), lane);
    acc = mma4<T>(av, bv, acc, true);
    acc_store<T>(m.a(i, j), lane, acc);
}
// (c): X_ij -= L_ik X_kj, i > k, j <= k (tile (i, k) of the inverse starts from zero)
template <typename T>
__device__ __forceinline__ void leaf_update_x(const LeafLds<T> &m, int i, int j, int k, int lane)
{
    T av[4], bv[4];
    op_rows<T>(m.a(i, k), lane, av);
    op_nat<T>(m.x(k, j), lane, bv);
    typename Mfma<T>::acc_t acc = {0, 0, 0, 0};
    if (j < k)
        acc = acc_load<T>(m.x(i, j), lane);
    acc = mma4<T>(av, bv, acc, true);
    acc_store<T>(m.x(i, j), lane, acc);
}

// tile (ti, tj) number t < LK (LK + 1) / 2 of the lower triangle counted row by row
__device__ __forceinline__ void tri_decode(int t, int &ti, int &tj)
{
    static_assert(LK == 8, "the row starts below are those of eight tile rows");
    ti = (t >= 1) + (t >= 3) + (t >= 6) + (t >= 10) + (t >= 15) + (t >= 21) + (t >= 28);
    tj = t - ti * (ti + 1) / 2;
}

// Whole 16-byte pieces can move between a block at p and the tiles: rows contiguous and 16-byte
// aligned, no ragged last tile.
template <typename T>
__device__ __forceinline__ bool leaf_vec_ok(const T *p, int64_t rs, int64_t cs, int nb)
{
    constexpr int VW = Mfma<T>::VW;
    return cs == 1 && (rs % VW) == 0 && (reinterpret_cast<uintptr_t>(p) & 15) == 0 && (nb % LT) == 0;
}
// Lane -> 16-byte piece of a 16 x 16 tile: row `row0 + pass * RPP`, elements col .. col + VW - 1.
template <typename T>
struct TileVec {
    using V = typename Mfma<T>::vec_t;
    static constexpr int VW = Mfma<T>::VW;
    static constexpr int CPR = LT / VW;   // pieces per tile row
    static constexpr int RPP = 64 / CPR;  // tile rows a wavefront covers at once
    static constexpr int NP = LT / RPP;   // passes per tile
};

// leaf_load_lower for blocks that satisfy leaf_vec_ok: no predicates, half (a quarter of) the
// memory instructions, the 64-bit address arithmetic once per tile.  The pieces of a diagonal tile
// that reach above the diagonal are cleared element by element.
template <typename T, int W, int MAXK>
__device__ __forceinline__ void leaf_load_lower_vec(const LeafLds<T> &m, const T *p, int64_t rs, int K, int wave,
                                                    int lane, bool into_x)
{
    using TV = TileVec<T>;
    using V = typename TV::V;
    constexpr int TPW = (MAXK * (MAXK + 1) / 2 + W - 1) / W;
    const int ntl = K * (K + 1) / 2;
    const int row0 = lane / TV::CPR, col = (lane % TV::CPR) * TV::VW;
    V val[TPW][TV::NP];
#pragma unroll
    for (int q = 0; q < TPW; ++q) {
        const int t = wave + q * W;
        if (t < ntl) {
            int ti, tj;
            tri_decode(t, ti, tj);
            const T *tp = p + (int64_t)(ti * LT + row0) * rs + (tj * LT + col);
#pragma unroll
            for (int ps = 0; ps < TV::NP; ++ps)
                val[q][ps] = *reinterpret_cast<const V *>(tp + (int64_t)(ps * TV::RPP) * rs);
        }
    }
#pragma unroll
    for (int q = 0; q < TPW; ++q) {
        const int t = wave + q * W;
        if (t < ntl) {
            int ti, tj;
            tri_decode(t, ti, tj);
            const TileRef<T> tr = into_x ? m.x(ti, tj) : m.a(ti, tj);
#pragma unroll
            for (int ps = 0; ps < TV::NP; ++ps) {
                const int row = row0 + ps * TV::RPP;
                V v = val[q][ps];
                if (ti == tj) {
                    T *e = reinterpret_cast<T *>(&v);
#pragma unroll
                    for (int u = 0; u < TV::VW; ++u)
                        e[u] = (col + u <= row) ? e[u] : T(0);
                }
                *reinterpret_cast<V *>(tr.p + tr.at(row, col)) = v;
            }
        }
    }
}

// Lower triangle of an nb x nb block at p (element strides rs, cs) into the tiles of A (or of the
// inverse's area with into_x); outside nb x nb the tiles get pad_diag on the diagonal and zero
// elsewhere.  Per tile a lane moves four elements, 16 lanes along the contiguous direction of the
// operand; all loads of a wavefront are in flight together.
// W wavefronts share the work; the block has at most MAXK tile rows.
template <typename T, int W = LEAF16_WAVES, int MAXK = LK>
__device__ __forceinline__ void leaf_load_lower(const LeafLds<T> &m, const T *p, int64_t rs, int64_t cs, int nb,
                                                int wave, int lane, bool into_x = false, T pad_diag = T(1))
{
    if (leaf_vec_ok<T>(p, rs, cs, nb)) {
        leaf_load_lower_vec<T, W, MAXK>(m, p, rs, nb / LT, wave, lane, into_x);
        return;
    }
    constexpr int TPW = (MAXK * (MAXK + 1) / 2 + W - 1) / W;  // lower tiles per wavefront, at most
    const int K = (nb + LT - 1) / LT;
    const int ntl = K * (K + 1) / 2;
    const bool colfast = (cs == 1) || (rs != 1);
    const int f = lane & 15, s0 = lane >> 4;  // fast and slow coordinate inside the tile (slow: s0 + 4 v)
    const int64_t fs = colfast ? cs : rs, ss = colfast ? rs : cs;  // their strides
    const int64_t lane_off = (int64_t)f * fs + (int64_t)s0 * ss;
    T val[TPW][4];
#pragma unroll
    for (int q = 0; q < TPW; ++q) {
        const int t = wave + q * W;
        int ti, tj;
        tri_decode(t < ntl ? t : 0, ti, tj);
        const T *tp = p + (int64_t)(ti * LT) * rs + (int64_t)(tj * LT) * cs + lane_off;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int u = colfast ? s0 + 4 * v : f, w = colfast ? f : s0 + 4 * v;
            const int r = ti * LT + u, c = tj * LT + w;
            T x = (r == c) ? pad_diag : T(0);
            if (t < ntl && r < nb && c <= r)
                x = *tp;
            val[q][v] = x;
            tp += 4 * ss;
        }
    }
#pragma unroll
    for (int q = 0; q < TPW; ++q) {
        const int t = wave + q * W;
        if (t < ntl) {
            int ti, tj;
            tri_decode(t, ti, tj);
            const TileRef<T> tr = into_x ? m.x(ti, tj) : m.a(ti, tj);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int u = colfast ? s0 + 4 * v : f, w = colfast ? f : s0 + 4 * v;
                tr.p[tr.at(u, w)] = val[q][v];
            }
        }
    }
}

// The lower tiles of A / L (inverse == false) or of the inverse back to an nb x nb block at p;
// zero_upper also writes zeros to the tiles above the diagonal.
// leaf_store_lower for blocks that satisfy leaf_vec_ok
template <typename T, int W, int MAXK>
__device__ __forceinline__ void leaf_store_lower_vec(const LeafLds<T> &m, bool inverse, T *p, int64_t rs, int K,
                                                     bool zero_upper, int wave, int lane)
{
    using TV = TileVec<T>;
    using V = typename TV::V;
    constexpr int TPW = (MAXK * (MAXK + 1) / 2 + W - 1) / W;
    const int ntl = K * (K + 1) / 2;
    const int row0 = lane / TV::CPR, col = (lane % TV::CPR) * TV::VW;
#pragma unroll
    for (int q = 0; q < TPW; ++q) {
        const int t = wave + q * W;
        if (t < ntl) {
            int ti, tj;
            tri_decode(t, ti, tj);
            const TileRef<T> tr = inverse ? m.x(ti, tj) : m.a(ti, tj);
            T *tp = p + (int64_t)(ti * LT + row0) * rs + (tj * LT + col);
            V v0 = *reinterpret_cast<const V *>(tr.p + tr.at(row0, col));
            if constexpr (TV::NP == 2) {
                V v1 = *reinterpret_cast<const V *>(tr.p + tr.at(row0 + TV::RPP, col));
                *reinterpret_cast<V *>(tp) = v0;
                *reinterpret_cast<V *>(tp + (int64_t)TV::RPP * rs) = v1;
            } else {
                static_assert(TV::NP == 1 || TV::NP == 2, "one or two passes per tile");
                *reinterpret_cast<V *>(tp) = v0;
            }
        }
    }
    if (zero_upper) {
        V z;
        T *e = reinterpret_cast<T *>(&z);
#pragma unroll
        for (int u = 0; u < TV::VW; ++u)
            e[u] = T(0);
        for (int t = wave; t < ntl - K; t += W) {
            int tj, ti;
            tri_decode(t, tj, ti);  // strictly lower (tj + 1, ti), mirrored
            T *tp = p + (int64_t)(ti * LT + row0) * rs + ((tj + 1) * LT + col);
#pragma unroll
            for (int ps = 0; ps < TV::NP; ++ps)
                *reinterpret_cast<V *>(tp + (int64_t)(ps * TV::RPP) * rs) = z;
        }
    }
}

template <typename T, int W = LEAF16_WAVES, int MAXK = LK>
__device__ __forceinline__ void leaf_store_lower(const LeafLds<T> &m, bool inverse, T *p, int64_t rs, int64_t cs,
                                                 int nb, bool zero_upper, int wave, int lane)
{
    if (leaf_vec_ok<T>(p, rs, cs, nb)) {
        leaf_store_lower_vec<T, W, MAXK>(m, inverse, p, rs, nb / LT, zero_upper, wave, lane);
        return;
    }
    const int K = (nb + LT - 1) / LT;
    const int ntl = K * (K + 1) / 2;
    const bool colfast = (cs == 1) || (rs != 1);
    const int f = lane & 15, s0 = lane >> 4;
    const int64_t fs = colfast ? cs : rs, ss = colfast ? rs : cs;
    const int64_t lane_off = (int64_t)f * fs + (int64_t)s0 * ss;
    for (int t = wave; t < ntl; t += W) {
        int ti, tj;
        tri_decode(t, ti, tj);
        const TileRef<T> tr = inverse ? m.x(ti, tj) : m.a(ti, tj);
        T *tp = p + (int64_t)(ti * LT) * rs + (int64_t)(tj * LT) * cs + lane_off;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int u = colfast ? s0 + 4 * v : f, w = colfast ? f : s0 + 4 * v;
            if (ti * LT + u < nb && tj * LT + w < nb)
                *tp = tr.p[tr.at(u, w)];
            tp += 4 * ss;
        }
    }
    if (zero_upper) {
        for (int t = wave; t < ntl - K; t += W) {
            int tj, ti;
            tri_decode(t, tj, ti);  // strictly lower (tj + 1, ti), mirrored
            tj += 1;
            T *tp = p + (int64_t)(ti * LT) * rs + (int64_t)(tj * LT) * cs + lane_off;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int u = colfast ? s0 + 4 * v : f, w = colfast ? f : s0 + 4 * v;
                if (ti * LT + u < nb && tj * LT + w < nb)
                    *tp = T(0);
                tp += 4 * ss;
            }
        }
    }
}

// The factorisation loop shared by the kernels below: on entry the lower tiles of the block are in
// the A / L areas of m (and a workgroup barrier has passed), on return they hold the factor and the
// X areas its inverse.  Returns, in wavefront 0, the 1-based index of the first pivot that is not
// > 0 (0: none); ends with a workgroup barrier.
template <typename T>
__device__ __forceinline__ int leaf_factor(const LeafLds<T> &m, int K, int wave, int lane)
{
    constexpr int W = LEAF16_WAVES;
    int fail = 0;
    if (wave == 0)
        fail = leaf_diag<T>(m, 0, lane);
    __syncthreads();
    LEAF16_STAMP(1);

    for (int k = 0; k < K; ++k) {
        const int rows = K - 1 - k;  // tile rows below the pivot row
        // ---- (b): wavefront 0 takes the panel tile the next diagonal tile depends on ------------
        if (wave == 0) {
            if (rows > 0)
                leaf_panel<T>(m, k + 1, k, lane);
        } else {
            const int np = rows > 0 ? rows - 1 : 0;
            for (int it = wave - 1; it < np + k; it += W - 1) {
                if (it < np)
                    leaf_panel<T>(m, k + 2 + it, k, lane);
                else
                    leaf_xrow<T>(m, k, it - np, lane);
            }
        }
        __syncthreads();
        LEAF16_STAMP(2 + 2 * k);
        if (rows == 0)
            break;
        // ---- (c): wavefront 0 updates the next diagonal tile and factors it -----------------------
        if (wave == 0) {
            leaf_update_a<T>(m, k + 1, k + 1, k, lane);
            const int f = leaf_diag<T>(m, k + 1, lane);
            if (fail == 0 && f != 0)
                fail = (k + 1) * LT + f;
        } else {
            const int nx = rows * (k + 1);           // tiles of the inverse to update
            const int na = rows * (rows + 1) / 2 - 1;  // tiles of A, without tile (k+1, k+1)
            int xi = 0, xj = wave - 1;                // item number it = xi * (k + 1) + xj
            for (int it = wave - 1; it < nx + na; it += W - 1) {
                if (it < nx) {
                    while (xj > k) {
                        xj -= k + 1;
                        ++xi;
                    }
                    leaf_update_x<T>(m, k + 1 + xi, xj, k, lane);
                    xj += W - 1;
                } else {
                    int ii, jj;
                    tri_decode(it - nx + 1, ii, jj);
                    leaf_update_a<T>(m, k + 1 + ii, k + 1 + jj, k, lane);
                }
            }
        }
        __syncthreads();
        LEAF16_STAMP(3 + 2 * k);
    }
    return fail;
}

template <typename T>
__global__ __launch_bounds__(LEAF16_THREADS) void k_potrf_leaf16(View<const T> A, View<T> L, View<T> Inv, int32_t *info,
                                                                 int info_off, int64_t batch, int nb, int zero_upper)
{
    using C = Leaf16<T>;
    extern __shared__ __align__(16) unsigned char leaf16_lds[];
    T *lds = reinterpret_cast<T *>(leaf16_lds);
    const LeafLds<T> m{lds + C::OFF_D, lds + C::OFF_XD, lds + C::OFF_A, lds + C::OFF_X};

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int K = (nb + LT - 1) / LT;  // tile columns in use
    const int64_t b = blockIdx.x;
    LEAF16_STAMP(31);

    leaf_load_lower<T>(m, A.p + b * A.bs, A.rs, A.cs, nb, wave, lane);
    __syncthreads();
    LEAF16_STAMP(0);

    const int fail = leaf_factor<T>(m, K, wave, lane);

    // ---- factor and inverse back to memory (lower tiles; zeros above the diagonal inside the
    //      diagonal tiles) -----------------------------------------------------------------------
    leaf_store_lower<T>(m, false, L.p + b * L.bs, L.rs, L.cs, nb, zero_upper != 0, wave, lane);
    if (Inv.p != nullptr)  // a stand-alone factorisation has no use for the inverse
        leaf_store_lower<T>(m, true, Inv.p + b * Inv.bs, Inv.rs, Inv.cs, nb, false, wave, lane);
    LEAF16_STAMP(30);
    if (info != nullptr && tid == 0 && fail != 0 && fail <= nb) {
        if (info[b] == 0)
            info[b] = info_off + fail;
    }
}

// ---------------------------------------------------------------------------------------
// potrf of many matrices of at most four tile rows (32 < n <= 64), four wavefronts per matrix and LDS for
// the tiles in use only, so that several workgroups share a compute unit.  Nobody wants the inverse of
// the factor here: per tile column one wavefront factors the diagonal tile (and inverts it in registers,
// for the panel), then the panel tiles L_ik = A_ik Li_kk^T and the trailing updates are dealt over the four.
// ---------------------------------------------------------------------------------------
constexpr int SMALL16_WAVES = 4, SMALL16_MAXK = 4;
template <typename T>
__host__ __device__ constexpr int small16_lds_elems(int K)
{
    return 2 * K * Leaf16<T>::DT + K * (K - 1) / 2 * Leaf16<T>::OT;
}

template <typename T>
__global__ __launch_bounds__(SMALL16_WAVES * 64) void k_potrf_small16(View<const T> A, View<T> L, int32_t *info,
                                                                      int64_t batch, int n)
{
    using C = Leaf16<T>;
    extern __shared__ __align__(16) unsigned char leaf16_lds[];
    T *lds = reinterpret_cast<T *>(leaf16_lds);
    constexpr int W = SMALL16_WAVES;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t b = blockIdx.x;
    const int K = (n + LT - 1) / LT;
    // diagonal tiles of A / L, diagonal tiles of the inverse, tiles below the diagonal (no other tiles of the inverse)
    const LeafLds<T> m{lds, lds + K * C::DT, lds + 2 * K * C::DT, lds + 2 * K * C::DT};

    leaf_load_lower<T, W, SMALL16_MAXK>(m, A.p + b * A.bs, A.rs, A.cs, n, wave, lane);
    __syncthreads();
    int fail = 0;
    for (int k = 0; k < K; ++k) {
        if (wave == 0) {
            const int f = leaf_diag<T>(m, k, lane);
            if (fail == 0 && f != 0)
                fail = k * LT + f;
        }
        __syncthreads();
        const int rows = K - 1 - k;
        if (rows == 0)
            break;
        for (int i = k + 1 + wave; i < K; i += W)
            leaf_panel<T>(m, i, k, lane);
        __syncthreads();
        for (int t = wave; t < rows * (rows + 1) / 2; t += W) {
            int ii, jj;
            tri_decode(t, ii, jj);
            leaf_update_a<T>(m, k + 1 + ii, k + 1 + jj, k, lane);
        }
        __syncthreads();
    }
    leaf_store_lower<T, W, SMALL16_MAXK>(m, false, L.p + b * L.bs, L.rs, L.cs, n, true, wave, lane);
    if (info != nullptr && tid == 0 && fail != 0 && fail <= n) {
        if (info[b] == 0)
            info[b] = fail;
    }
}

// ---------------------------------------------------------------------------------------
// Inverse of a GIVEN lower-triangular factor (the potrf backward pass and trsm need L^-1 of their
// input, section 4.2): the diagonal blocks of edge 128 of Lam (n x n), one workgroup each, written
// onto the diagonal blocks of Inv.  Same tiles and matrix-core steps as above without the
// factorisation, so the 16 x 16 diagonal tiles are inverted all at once.
// ---------------------------------------------------------------------------------------

template <typename T>
__global__ __launch_bounds__(LEAF16_THREADS) void k_tri_inv_leaf16(View<const T> Lam, View<T> Inv, int64_t batch, int n,
                                                                   int nblk)
{
    using C = Leaf16<T>;
    extern __shared__ __align__(16) unsigned char leaf16_lds[];
    T *lds = reinterpret_cast<T *>(leaf16_lds);
    const LeafLds<T> m{lds + C::OFF_D, lds + C::OFF_XD, lds + C::OFF_A, lds + C::OFF_X};
    constexpr int W = LEAF16_WAVES;
    constexpr int PS = C::PS;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t b = blockIdx.x / nblk;
    const int64_t o0 = (int64_t)(blockIdx.x % nblk) * (LT * LK);
    const int nb = (int)((n - o0) < LT * LK ? (n - o0) : LT * LK);
    const int K = (nb + LT - 1) / LT;

    leaf_load_lower<T>(m, Lam.p + b * Lam.bs + o0 * (Lam.rs + Lam.cs), Lam.rs, Lam.cs, nb, wave, lane);
    __syncthreads();

    if (wave < K) {  // all diagonal tiles at once
        const int r = lane & 15, g = lane >> 4;
        const T *dk = m.sD + wave * C::DT + r * PS;
        T *xk = m.sXD + wave * C::DT + r * PS;
        T a[LT], x[4];
#pragma unroll
        for (int c = 0; c < LT; ++c)
            a[c] = dk[c];
        diag_invert<T>(a, dk[r], x, r, g);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            xk[4 * j + g] = (4 * j + g <= r) ? x[j] : T(0);
    }
    __syncthreads();

    for (int k = 0; k < K; ++k) {
        if (k > 0) {  // X_kj <- Li_kk X_kj, j < k
            for (int j = wave; j < k; j += W)
                leaf_xrow<T>(m, k, j, lane);
            __syncthreads();
        }
        const int rows = K - 1 - k;
        if (rows > 0) {  // X_ij -= L_ik X_kj, i > k, j <= k
            int xi = 0, xj = wave;
            for (int it = wave; it < rows * (k + 1); it += W) {
                while (xj > k) {
                    xj -= k + 1;
                    ++xi;
                }
                leaf_update_x<T>(m, k + 1 + xi, xj, k, lane);
                xj += W;
            }
            __syncthreads();
        }
    }
    leaf_store_lower<T>(m, true, Inv.p + b * Inv.bs + o0 * (Inv.rs + Inv.cs), Inv.rs, Inv.cs, nb, false, wave, lane);
}

// ---------------------------------------------------------------------------------------
// potrf backward (section 4.2; appendix "potrf") for one matrix per workgroup, everything in
// LDS:  Abar = sym(L^-T Phi(L^T Lbar) L^-1),  Phi = lower triangle with halved diagonal.
//   P = Phi(tril(L^T Lbar));   Li = L^-1 (as in k_tri_inv_leaf16);   Z = P Li;
//   Abar_ij = 1/2 sum_{k >= i} (Li_ki^T Z_kj + Z_ki^T Li_kj)   for tiles i >= j, mirrored,
// which is the symmetrised W = Li^T Z without ever forming W.  Three tile areas are enough:
// [L, later Z], [Lbar, later Li], [P, later staging for the mirrored store].
// ---------------------------------------------------------------------------------------
template <typename T>
__host__ __device__ constexpr int backward16_area(int K)  // elements of one tile area for K tile rows
{
    return K * Leaf16<T>::DT + K * (K - 1) / 2 * Leaf16<T>::OT;
}

// NW wavefronts per matrix: 16, or 4 for at most MAXK = 4 tile rows when there are many matrices (ten tiles
// keep four wavefronts busy, and seven or eight such workgroups fit a compute unit instead of two).
template <typename T, int NW, int MAXK>
__global__ __launch_bounds__(NW * 64) void k_backward_leaf16(View<const T> Lam, View<const T> G, View<T> Abar,
                                                             int64_t batch, int n)
{
    using C = Leaf16<T>;
    using MF = Mfma<T>;
    extern __shared__ __align__(16) unsigned char leaf16_lds[];
    T *lds = reinterpret_cast<T *>(leaf16_lds);
    constexpr int W = NW;
    constexpr int PS = C::PS, DT = C::DT, OT = C::OT;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t b = blockIdx.x;
    const int K = (n + LT - 1) / LT;
    const int ntl = K * (K + 1) / 2;
    const int area = backward16_area<T>(K);
    // a: L, later Z.  x: Lbar, later Li.
    const LeafLds<T> m{lds, lds + area, lds + K * DT, lds + area + K * DT};
    T *pD = lds + 2 * area, *pO = pD + K * DT;
    auto ptile = [&](int i, int j) { return i == j ? TileRef<T>{pD + i * DT, true} : TileRef<T>{pO + tri_off(i, j) * OT, false}; };

    leaf_load_lower<T, NW, MAXK>(m, Lam.p + b * Lam.bs, Lam.rs, Lam.cs, n, wave, lane, false, T(1));
    leaf_load_lower<T, NW, MAXK>(m, G.p + b * G.bs, G.rs, G.cs, n, wave, lane, true, T(0));
    __syncthreads();

    // ---- P_ij = sum_{k >= i} L_ki^T Lbar_kj, i >= j; Phi on the diagonal tiles ------------------
    for (int t = wave; t < ntl; t += W) {
        int i, j;
        tri_decode(t, i, j);
        typename MF::acc_t acc = {0, 0, 0, 0};
        for (int k = i; k < K; ++k) {
            T av[4], bv[4];
            op_nat<T>(m.a(k, i), lane, av);
            op_nat<T>(m.x(k, j), lane, bv);
            acc = mma4<T>(av, bv, acc, false);
        }
        if (i == j) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = MF::row(lane, v), col = lane & 15;
                acc[v] = row < col ? T(0) : (row == col ? T(0.5) * acc[v] : acc[v]);
            }
        }
        acc_store<T>(ptile(i, j), lane, acc);
    }
    __syncthreads();

    // ---- Li = L^-1 into the area Lbar occupied ------------------------------------------------
    if (wave < K) {
        const int r = lane & 15, g = lane >> 4;
        const T *dk = m.sD + wave * DT + r * PS;
        T *xk = m.sXD + wave * DT + r * PS;
        T a[LT], x[4];
#pragma unroll
        for (int c = 0; c < LT; ++c)
            a[c] = dk[c];
        diag_invert<T>(a, dk[r], x, r, g);
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
            xk[4 * jj + g] = (4 * jj + g <= r) ? x[jj] : T(0);
    }
    __syncthreads();
    for (int k = 0; k < K; ++k) {
        if (k > 0) {  // X_kj <- Li_kk X_kj, j < k
            for (int j = wave; j < k; j += W)
                leaf_xrow<T>(m, k, j, lane);
            __syncthreads();
        }
        const int rows = K - 1 - k;
        if (rows > 0) {  // X_ij -= L_ik X_kj, i > k, j <= k
            int xi = 0, xj = wave;
            for (int it = wave; it < rows * (k + 1); it += W) {
                while (xj > k) {
                    xj -= k + 1;
                    ++xi;
                }
                leaf_update_x<T>(m, k + 1 + xi, xj, k, lane);
                xj += W;
            }
            __syncthreads();
        }
    }

    // ---- Z_ij = sum_{k = j..i} P_ik Li_kj, i >= j, into the area L occupied -----------------------
    for (int t = wave; t < ntl; t += W) {
        int i, j;
        tri_decode(t, i, j);
        typename MF::acc_t acc = {0, 0, 0, 0};
        for (int k = j; k <= i; ++k) {
            T av[4], bv[4];
            op_rows<T>(ptile(i, k), lane, av);
            op_nat<T>(m.x(k, j), lane, bv);
            acc = mma4<T>(av, bv, acc, false);
        }
        acc_store<T>(m.a(i, j), lane, acc);
    }
    __syncthreads();

    // ---- Abar_ij = 1/2 sum_{k >= i} (Li_ki^T Z_kj + Z_ki^T Li_kj), i >= j, stored with its mirror ----
    {
        T *op = Abar.p + b * Abar.bs;
        const bool colfast = (Abar.cs == 1) || (Abar.rs != 1);
        const int f = lane & 15, s0 = lane >> 4;
        for (int t = wave; t < ntl; t += W) {
            int i, j;
            tri_decode(t, i, j);
            typename MF::acc_t acc = {0, 0, 0, 0};
            for (int k = i; k < K; ++k) {
                T av[4], bv[4];
                op_nat<T>(m.x(k, i), lane, av);
                op_nat<T>(m.a(k, j), lane, bv);
                acc = mma4<T>(av, bv, acc, false);
                op_nat<T>(m.a(k, i), lane, av);
                op_nat<T>(m.x(k, j), lane, bv);
                acc = mma4<T>(av, bv, acc, false);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v)
                acc[v] *= T(0.5);
            // through this tile's slot of the (finished) P area: the mirror image is read back
            // transposed; on diagonal tiles both halves take the lower half's values, which makes
            // the result exactly symmetric
            const TileRef<T> st = ptile(i, j);
            acc_store<T>(st, lane, acc);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int u = colfast ? s0 + 4 * v : f, w = colfast ? f : s0 + 4 * v;
                const T direct = st.p[st.at(u, w)], mirror = st.p[st.at(w, u)];
                const int r = i * LT + u, c = j * LT + w;
                if (r < n && c < n)
                    op[(int64_t)r * Abar.rs + (int64_t)c * Abar.cs] = (i == j && u < w) ? mirror : direct;
                const int r2 = j * LT + u, c2 = i * LT + w;
                if (i != j && r2 < n && c2 < n)
                    op[(int64_t)r2 * Abar.rs + (int64_t)c2 * Abar.cs] = mirror;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// potri (section 4.2 "potri": B = A^-1 from the factor of A = L L^T) for one matrix per workgroup,
// everything in LDS:  Li = L^-1 as in k_tri_inv_leaf16, then  B_ij = sum_{k >= i} Li_ki^T Li_kj  for
// tiles i >= j, stored with the mirror image.  Two tile areas: [L, later staging of B], [Li].
// NW and MAXK as in k_backward_leaf16.
// ---------------------------------------------------------------------------------------
template <typename T, int NW, int MAXK>
__global__ __launch_bounds__(NW * 64) void k_potri_leaf16(View<const T> Lam, View<T> B, int64_t batch, int n)
{
    using C = Leaf16<T>;
    using MF = Mfma<T>;
    extern __shared__ __align__(16) unsigned char leaf16_lds[];
    T *lds = reinterpret_cast<T *>(leaf16_lds);
    constexpr int W = NW;
    constexpr int PS = C::PS, DT = C::DT;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t b = blockIdx.x;
    const int K = (n + LT - 1) / LT;
    const int ntl = K * (K + 1) / 2;
    const int area = backward16_area<T>(K);
    const LeafLds<T> m{lds, lds + area, lds + K * DT, lds + area + K * DT};

    leaf_load_lower<T, NW, MAXK>(m, Lam.p + b * Lam.bs, Lam.rs, Lam.cs, n, wave, lane, false, T(1));
    __syncthreads();

    if (wave < K) {  // all diagonal tiles at once
        const int r = lane & 15, g = lane >> 4;
        const T *dk = m.sD + wave * DT + r * PS;
        T *xk = m.sXD + wave * DT + r * PS;
        T a[LT], x[4];
#pragma unroll
        for (int c = 0; c < LT; ++c)
            a[c] = dk[c];
        diag_invert<T>(a, dk[r], x, r, g);
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
            xk[4 * jj + g] = (4 * jj + g <= r) ? x[jj] : T(0);
    }
    __syncthreads();
    for (int k = 0; k < K; ++k) {
        if (k > 0) {  // X_kj <- Li_kk X_kj, j < k
            for (int j = wave; j < k; j += W)
                leaf_xrow<T>(m, k, j, lane);
            __syncthreads();
        }
        const int rows = K - 1 - k;
        if (rows > 0) {  // X_ij -= L_ik X_kj, i > k, j <= k
            int xi = 0, xj = wave;
            for (int it = wave; it < rows * (k + 1); it += W) {
                while (xj > k) {
                    xj -= k + 1;
                    ++xi;
                }
                leaf_update_x<T>(m, k + 1 + xi, xj, k, lane);
                xj += W;
            }
            __syncthreads();
        }
    }

    // ---- B_ij = sum_{k >= i} Li_ki^T Li_kj, i >= j, through the tile's slot of the (finished) L area ----
    T *op = B.p + b * B.bs;
    const bool colfast = (B.cs == 1) || (B.rs != 1);
    const int f = lane & 15, s0 = lane >> 4;
    for (int t = wave; t < ntl; t += W) {
        int i, j;
        tri_decode(t, i, j);
        typename MF::acc_t acc = {0, 0, 0, 0};
        for (int k = i; k < K; ++k) {
            T av[4], bv[4];
            op_nat<T>(m.x(k, i), lane, av);
            op_nat<T>(m.x(k, j), lane, bv);
            acc = mma4<T>(av, bv, acc, false);
        }
        const TileRef<T> st = m.a(i, j);
        acc_store<T>(st, lane, acc);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int u = colfast ? s0 + 4 * v : f, w = colfast ? f : s0 + 4 * v;
            const T direct = st.p[st.at(u, w)], mirror = st.p[st.at(w, u)];
            const int r = i * LT + u, c = j * LT + w;
            if (r < n && c < n)
                op[(int64_t)r * B.rs + (int64_t)c * B.cs] = (i == j && u < w) ? mirror : direct;
            const int r2 = j * LT + u, c2 = i * LT + w;
            if (i != j && r2 < n && c2 < n)
                op[(int64_t)r2 * B.rs + (int64_t)c2 * B.cs] = mirror;
        }
    }
}

// ---------------------------------------------------------------------------------------
// Outer products of small matrices, one workgroup per item, operands in LDS as 16 x 16 tiles:
//   C = alpha U V^T,  U and V n x k (any strides), C n x n.
// tri 0: U and V are the same matrix (syrk, section 4.2): the tiles on and below the diagonal are
//        computed and stored with their mirror image, so C is exactly symmetric;
// tri 1 / 2: only the lower / upper triangle of the product is kept, the other one is written as
//        zeros (the triangular operand's gradient in the trmm and trsm backward rules).
// ---------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void rect_load(T *tiles, int Kc, const T *p, int64_t rs, int64_t cs, int rows, int cols,
                                          int Kr, int wave, int lane, int W)
{
    const bool colfast = (cs == 1) || (rs != 1);
    const int f = lane & 15, s0 = lane >> 4;
    for (int t = wave; t < Kr * Kc; t += W) {
        const int ti = t / Kc, tk = t % Kc;
        const TileRef<T> tr{tiles + t * Leaf16<T>::OT, false};
        T val[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int u = colfast ? s0 + 4 * v : f, w = colfast ? f : s0 + 4 * v;
            const int r = ti * LT + u, c = tk * LT + w;
            val[v] = (r < rows && c < cols) ? p[(int64_t)r * rs + (int64_t)c * cs] : T(0);
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int u = colfast ? s0 + 4 * v : f, w = colfast ? f : s0 + 4 * v;
            tr.p[tr.at(u, w)] = val[v];
        }
    }
}

template <typename T, int NW>
__global__ __launch_bounds__(NW * 64) void k_outer_leaf16(View<const T> U, View<const T> V, View<T> Cv, int64_t batch,
                                                          int n, int k, T alpha, int tri)
{
    using C = Leaf16<T>;
    using MF = Mfma<T>;
    extern __shared__ __align__(16) unsigned char leaf16_lds[];
    T *lds = reinterpret_cast<T *>(leaf16_lds);
    constexpr int OT = C::OT;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t b = blockIdx.x;
    const int Kn = (n + LT - 1) / LT, Kk = (k + LT - 1) / LT;
    T *tu = lds, *tv = tri == 0 ? lds : lds + Kn * Kk * OT;
    T *stage = lds + (tri == 0 ? 1 : 2) * Kn * Kk * OT + wave * OT;  // one tile per wavefront

    rect_load<T>(tu, Kk, U.p + b * U.bs, U.rs, U.cs, n, k, Kn, wave, lane, NW);
    if (tri != 0)
        rect_load<T>(tv, Kk, V.p + b * V.bs, V.rs, V.cs, n, k, Kn, wave, lane, NW);
    __syncthreads();

    T *op = Cv.p + b * Cv.bs;
    const bool colfast = (Cv.cs == 1) || (Cv.rs != 1);
    const int f = lane & 15, s0 = lane >> 4;
    for (int t = wave; t < Kn * Kn; t += NW) {
        const int i = t / Kn, j = t % Kn;
        const bool kept = tri == 2 ? (i <= j) : (i >= j);
        if (tri == 0 && !kept)
            continue;  // written as the mirror image of tile (j, i)
        typename MF::acc_t acc = {0, 0, 0, 0};
        if (kept) {
            for (int kk = 0; kk < Kk; ++kk) {
                T av[4], bv[4];
                op_rows<T>(TileRef<T>{tu + (i * Kk + kk) * OT, false}, lane, av);
                op_rows<T>(TileRef<T>{tv + (j * Kk + kk) * OT, false}, lane, bv);
                acc = mma4<T>(av, bv, acc, false);
            }
        }
        const TileRef<T> st{stage, false};
#pragma unroll
        for (int v = 0; v < 4; ++v)
            acc[v] *= alpha;
        acc_store<T>(st, lane, acc);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int u = colfast ? s0 + 4 * v : f, w = colfast ? f : s0 + 4 * v;
            const T direct = st.p[st.at(u, w)], mirror = st.p[st.at(w, u)];
            const int r = i * LT + u, c = j * LT + w;
            T val = direct;
            if (i == j) {
                if (tri == 0)
                    val = u < w ? mirror : direct;
                else if (tri == 1 ? (u < w) : (u > w))
                    val = T(0);
            }
            if (r < n && c < n)
                op[(int64_t)r * Cv.rs + (int64_t)c * Cv.cs] = val;
            const int r2 = j * LT + u, c2 = i * LT + w;
            if (tri == 0 && i != j && r2 < n && c2 < n)
                op[(int64_t)r2 * Cv.rs + (int64_t)c2 * Cv.cs] = mirror;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();  // the staging tile is free again
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

// ---------------------------------------------------------------------------------------
// syrk backward (section 4.2 "syrk", backward) for small matrices, one workgroup per item:
//   Out = alpha (G + G^T) A,   G n x n (need not be symmetric), A and Out n x k (any strides).
// G and A sit in LDS as tiles; the left operand of each 16 x 16 x 16 product is G_ij + G_ji^T, added
// in the operand registers.
// ---------------------------------------------------------------------------------------
template <typename T, int NW>
__global__ __launch_bounds__(NW * 64) void k_symm_leaf16(View<const T> G, View<const T> A, View<T> Out, int64_t batch, int n,
                                                         int k, T alpha)
{
    using C = Leaf16<T>;
    using MF = Mfma<T>;
    extern __shared__ __align__(16) unsigned char leaf16_lds[];
    T *lds = reinterpret_cast<T *>(leaf16_lds);
    constexpr int OT = C::OT;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t b = blockIdx.x;
    const int Kn = (n + LT - 1) / LT, Kk = (k + LT - 1) / LT;
    T *tg = lds, *ta = lds + Kn * Kn * OT;
    T *stage = ta + Kn * Kk * OT + wave * OT;  // one tile per wavefront

    rect_load<T>(tg, Kn, G.p + b * G.bs, G.rs, G.cs, n, n, Kn, wave, lane, NW);
    rect_load<T>(ta, Kk, A.p + b * A.bs, A.rs, A.cs, n, k, Kn, wave, lane, NW);
    __syncthreads();

    T *op = Out.p + b * Out.bs;
    const bool colfast = (Out.cs == 1) || (Out.rs != 1);
    const int f = lane & 15, s0 = lane >> 4;
    for (int t = wave; t < Kn * Kk; t += NW) {
        const int i = t / Kk, c = t % Kk;
        typename MF::acc_t acc = {0, 0, 0, 0};
        for (int j = 0; j < Kn; ++j) {
            T av[4], at[4], bv[4];
            op_rows<T>(TileRef<T>{tg + (i * Kn + j) * OT, false}, lane, av);
            op_nat<T>(TileRef<T>{tg + (j * Kn + i) * OT, false}, lane, at);  // as a left operand: the transpose
            op_nat<T>(TileRef<T>{ta + (j * Kk + c) * OT, false}, lane, bv);
#pragma unroll
            for (int s = 0; s < 4; ++s)
                av[s] += at[s];
            acc = mma4<T>(av, bv, acc, false);
        }
        const TileRef<T> st{stage, false};
#pragma unroll
        for (int v = 0; v < 4; ++v)
            acc[v] *= alpha;
        acc_store<T>(st, lane, acc);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int u = colfast ? s0 + 4 * v : f, w = colfast ? f : s0 + 4 * v;
            const int r = i * LT + u, cc = c * LT + w;
            if (r < n && cc < k)
                op[(int64_t)r * Out.rs + (int64_t)cc * Out.cs] = st.p[st.at(u, w)];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();  // the staging tile is free again
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

// ---------------------------------------------------------------------------------------
// trmm (section 4.2 "trmm") for small matrices, one workgroup per item:  X = alpha M Xin with M = Lam
// (fwd) or Lam^T, Lam lower triangular n x n, Xin and X n x m (any strides; X may be Xin).  The lower
// tiles of Lam and the tiles of Xin sit in LDS; what lies above Lam's diagonal is never read.
// ---------------------------------------------------------------------------------------
template <typename T, int NW, int MAXK>
__global__ __launch_bounds__(NW * 64) void k_trmm_leaf16(View<const T> Lam, View<const T> Xin, View<T> X, int64_t batch, int n,
                                                         int m, T alpha, int fwd)
{
    using C = Leaf16<T>;
    using MF = Mfma<T>;
    extern __shared__ __align__(16) unsigned char leaf16_lds[];
    T *lds = reinterpret_cast<T *>(leaf16_lds);
    constexpr int OT = C::OT, DT = C::DT;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t b = blockIdx.x;
    const int Kn = (n + LT - 1) / LT, Km = (m + LT - 1) / LT;
    const int area = backward16_area<T>(Kn);
    const LeafLds<T> ml{lds, lds, lds + Kn * DT, lds + Kn * DT};  // only the A / L areas are used
    T *tx = lds + area;
    T *stage = tx + Kn * Km * OT + wave * OT;  // one tile per wavefront

    leaf_load_lower<T, NW, MAXK>(ml, Lam.p + b * Lam.bs, Lam.rs, Lam.cs, n, wave, lane, false, T(0));
    rect_load<T>(tx, Km, Xin.p + b * Xin.bs, Xin.rs, Xin.cs, n, m, Kn, wave, lane, NW);
    __syncthreads();

    T *op = X.p + b * X.bs;
    const bool colfast = (X.cs == 1) || (X.rs != 1);
    const int f = lane & 15, s0 = lane >> 4;
    for (int t = wave; t < Kn * Km; t += NW) {
        const int i = t / Km, c = t % Km;
        typename MF::acc_t acc = {0, 0, 0, 0};
        const int j0 = fwd ? 0 : i, j1 = fwd ? i : Kn - 1;
        for (int j = j0; j <= j1; ++j) {
            T av[4], bv[4];
            if (fwd)
                op_rows<T>(ml.a(i, j), lane, av);
            else
                op_nat<T>(ml.a(j, i), lane, av);  // as a left operand: the transpose
            op_nat<T>(TileRef<T>{tx + (j * Km + c) * OT, false}, lane, bv);
            acc = mma4<T>(av, bv, acc, false);
        }
        const TileRef<T> st{stage, false};
#pragma unroll
        for (int v = 0; v < 4; ++v)
            acc[v] *= alpha;
        acc_store<T>(st, lane, acc);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int u = colfast ? s0 + 4 * v : f, w = colfast ? f : s0 + 4 * v;
            const int r = i * LT + u, cc = c * LT + w;
            if (r < n && cc < m)
                op[(int64_t)r * X.rs + (int64_t)cc * X.cs] = st.p[st.at(u, w)];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();  // the staging tile is free again
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

// ---------------------------------------------------------------------------------------
// Gaussian-process criterion and its gradient in one launch (section 3.1: potrf, two trsm,
// sumlogdiag; backward of trsm (first case) and of potrf from section 4.2), one workgroup per
// matrix, everything in LDS.  For A = K + noise, targets y:
//   L = potrf(A) with Li = L^-1 (the factorisation loop of k_potrf_leaf16);
//   z = Li y,  alpha = Li^T z,  loss = 1/2 |z|^2 + sum_i log l_ii;
//   Lbar = -tril(alpha z^T) + diag(1 / l_ii) is never stored: its tiles are built in registers
//   where P = Phi(tril(L^T Lbar)) needs them;
//   Z = P Li;  Abar_ij = 1/2 sum_{k >= i} (Li_ki^T Z_kj + Z_ki^T Li_kj)   (as in k_backward_leaf16).
// Three tile areas: [A -> L -> Z], [Li], [P -> staging of the mirrored store], and 4 vectors.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(LEAF16_THREADS) void k_gp_leaf16(View<const T> A, const T *y, T *loss, View<T> Abar,
                                                              int32_t *info, int64_t batch, int n)
{
    using C = Leaf16<T>;
    using MF = Mfma<T>;
    extern __shared__ __align__(16) unsigned char leaf16_lds[];
    T *lds = reinterpret_cast<T *>(leaf16_lds);
    constexpr int W = LEAF16_WAVES;
    constexpr int DT = C::DT, OT = C::OT;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t b = blockIdx.x;
    const int K = (n + LT - 1) / LT;
    const int ntl = K * (K + 1) / 2;
    const int area = backward16_area<T>(K);
    const LeafLds<T> m{lds, lds + area, lds + K * DT, lds + area + K * DT};
    T *pD = lds + 2 * area, *pO = pD + K * DT;
    T *sy = lds + 3 * area, *sz = sy + LT * LK, *sal = sz + LT * LK, *sdi = sal + LT * LK;  // y, z, alpha, 1 / l_ii
    auto ptile = [&](int i, int j) { return i == j ? TileRef<T>{pD + i * DT, true} : TileRef<T>{pO + tri_off(i, j) * OT, false}; };

    leaf_load_lower<T>(m, A.p + b * A.bs, A.rs, A.cs, n, wave, lane);
    if (tid < LT * LK)
        sy[tid] = tid < n ? y[b * n + tid] : T(0);
    __syncthreads();

    // ---- L and Li ------------------------------------------------------------------------------
    const int fail = leaf_factor<T>(m, K, wave, lane);
    if (info != nullptr && tid == 0 && fail != 0 && fail <= n)
        info[b] = fail;

    // ---- z = Li y: eight threads per row, one tile column each ----------------------------------
    {
        const int r = tid >> 3, tj = tid & 7, ti = r >> 4, u = r & 15;
        T part = T(0);
        if (ti < K && tj <= ti) {
            const TileRef<T> t = m.x(ti, tj);
#pragma unroll
            for (int w = 0; w < LT; ++w)
                part = fma(t.p[t.at(u, w)], sy[tj * LT + w], part);
        }
        part += __shfl_xor(part, 1, 8);
        part += __shfl_xor(part, 2, 8);
        part += __shfl_xor(part, 4, 8);
        if (tj == 0) {
            sz[r] = part;
            const TileRef<T> d = m.x(ti < K ? ti : 0, ti < K ? ti : 0);
            sdi[r] = (r < n) ? d.p[d.at(u, u)] : T(0);
        }
    }
    __syncthreads();
    // ---- alpha = Li^T z: eight threads per column, one tile row each; the loss -------------------
    {
        const int c = tid >> 3, ti = tid & 7, tj = c >> 4, w = c & 15;
        T part = T(0);
        if (ti < K && tj <= ti) {
            const TileRef<T> t = m.x(ti, tj);
#pragma unroll
            for (int u = 0; u < LT; ++u)
                part = fma(t.p[t.at(u, w)], sz[ti * LT + u], part);
        }
        part += __shfl_xor(part, 1, 8);
        part += __shfl_xor(part, 2, 8);
        part += __shfl_xor(part, 4, 8);
        if (ti == 0)
            sal[c] = part;
    }
    if (wave == 0) {  // loss = 1/2 |z|^2 - sum log(1 / l_ii)
        double acc = 0.0;
        for (int r = lane; r < n; r += 64)
            acc += 0.5 * (double)sz[r] * (double)sz[r] - (double)log(sdi[r]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1)
            acc += __shfl_xor(acc, off, 64);
        if (lane == 0)
            loss[b] = (T)acc;
    }
    __syncthreads();

    // ---- P_ij = sum_{k >= i} L_ki^T Lbar_kj, i >= j, with Lbar_kj built in registers; Phi ----------
    for (int t = wave; t < ntl; t += W) {
        int i, j;
        tri_decode(t, i, j);
        typename MF::acc_t acc = {0, 0, 0, 0};
        const int w = lane & 15;
        const T zc = sz[j * LT + w];
        for (int k = i; k < K; ++k) {
            T av[4], bv[4];
            op_nat<T>(m.a(k, i), lane, av);
#pragma unroll
            for (int s = 0; s < 4; ++s) {  // element (u, w) of tile (k, j) of Lbar, u = 4 (lane / 16) + s
                const int u = 4 * (lane >> 4) + s;
                const int r = k * LT + u, c = j * LT + w;
                T v = -sal[r] * zc;
                if (r == c)
                    v += sdi[r];
                bv[s] = (r >= c) ? v : T(0);
            }
            acc = mma4<T>(av, bv, acc, false);
        }
        if (i == j) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = MF::row(lane, v), col = lane & 15;
                acc[v] = row < col ? T(0) : (row == col ? T(0.5) * acc[v] : acc[v]);
            }
        }
        acc_store<T>(ptile(i, j), lane, acc);
    }
    __syncthreads();

    // ---- Z_ij = sum_{k = j..i} P_ik Li_kj, i >= j, into the area L occupied -----------------------
    for (int t = wave; t < ntl; t += W) {
        int i, j;
        tri_decode(t, i, j);
        typename MF::acc_t acc = {0, 0, 0, 0};
        for (int k = j; k <= i; ++k) {
            T av[4], bv[4];
            op_rows<T>(ptile(i, k), lane, av);
            op_nat<T>(m.x(k, j), lane, bv);
            acc = mma4<T>(av, bv, acc, false);
        }
        acc_store<T>(m.a(i, j), lane, acc);
    }
    __syncthreads();

    // ---- Abar_ij = 1/2 sum_{k >= i} (Li_ki^T Z_kj + Z_ki^T Li_kj), i >= j, stored with its mirror ----
    {
        T *op = Abar.p + b * Abar.bs;
        const bool colfast = (Abar.cs == 1) || (Abar.rs != 1);
        const int f = lane & 15, s0 = lane >> 4;
        for (int t = wave; t < ntl; t += W) {
            int i, j;
            tri_decode(t, i, j);
            typename MF::acc_t acc = {0, 0, 0, 0};
            for (int k = i; k < K; ++k) {
                T av[4], bv[4];
                op_nat<T>(m.x(k, i), lane, av);
                op_nat<T>(m.a(k, j), lane, bv);
                acc = mma4<T>(av, bv, acc, false);
                op_nat<T>(m.a(k, i), lane, av);
                op_nat<T>(m.x(k, j), lane, bv);
                acc = mma4<T>(av, bv, acc, false);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v)
                acc[v] *= T(0.5);
            const TileRef<T> st = ptile(i, j);
            acc_store<T>(st, lane, acc);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int u = colfast ? s0 + 4 * v : f, w = colfast ? f : s0 + 4 * v;
                const T direct = st.p[st.at(u, w)], mirror = st.p[st.at(w, u)];
                const int r = i * LT + u, c = j * LT + w;
                if (r < n && c < n)
                    op[(int64_t)r * Abar.rs + (int64_t)c * Abar.cs] = (i == j && u < w) ? mirror : direct;
                const int r2 = j * LT + u, c2 = i * LT + w;
                if (i != j && r2 < n && c2 < n)
                    op[(int64_t)r2 * Abar.rs + (int64_t)c2 * Abar.cs] = mirror;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// trsm (section 4.2) with a small triangular matrix and a few right-hand sides: n <= 128 and
// m <= 48 vectors X(e, v), one workgroup per batch item.  Block substitution over the 16-row
// tiles with the inverted diagonal tiles:
//   fwd:  X_k = Li_kk B_k,    B_i -= L_ik X_k   (i > k),   k = 0, 1, ...
//   !fwd: X_k = Li_kk^T B_k,  B_i -= L_ki^T X_k (i < k),   k = K-1, K-2, ...
// Each 16-column tile of right-hand sides has its own chain wavefront, which also applies the
// update the next step depends on; the remaining updates belong to fixed other wavefronts (one
// owner per tile, so successive updates of a tile are ordered).  One barrier per step.
// ---------------------------------------------------------------------------------------
constexpr int TRSM16_MAX_CT = 3;  // column tiles of right-hand sides (they live in the inverse's tile area)

// LDS of k_trsm_leaf16 (elements): diagonal tiles of Lam and of their inverses, the tiles below the diagonal, the
// right-hand sides
template <typename T>
__host__ __device__ constexpr int trsm16_lds_elems(int K, int MT)
{
    return 2 * K * Leaf16<T>::DT + (K * (K - 1) / 2 + K * MT) * Leaf16<T>::OT;
}

// W wavefronts per item: 16, or 4 for at most MAXK = 4 tile rows when there are many items.
template <typename T, int W, int MAXK>
__global__ __launch_bounds__(W * 64) void k_trsm_leaf16(View<const T> Lam, View<const T> Xin, View<T> X,
                                                        int64_t batch, int n, int m, T alpha, int fwd)
{
    using C = Leaf16<T>;
    extern __shared__ __align__(16) unsigned char leaf16_lds[];
    T *lds = reinterpret_cast<T *>(leaf16_lds);
    constexpr int PS = C::PS, OT = C::OT;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t b = blockIdx.x;
    const int K = (n + LT - 1) / LT, MT = (m + LT - 1) / LT;
    const LeafLds<T> mm{lds, lds + K * C::DT, lds + 2 * K * C::DT, lds + 2 * K * C::DT + K * (K - 1) / 2 * OT};
    auto btile = [&](int k, int ct) { return TileRef<T>{mm.sX + (k * MT + ct) * OT, false}; };

    leaf_load_lower<T, W, MAXK>(mm, Lam.p + b * Lam.bs, Lam.rs, Lam.cs, n, wave, lane);
    {  // right-hand sides, scaled by alpha, zero outside n x m
        const T *xp = Xin.p + b * Xin.bs;
        const bool colfast = (Xin.cs == 1) || (Xin.rs != 1);
        const int f = lane & 15, s0 = lane >> 4;
        for (int t = wave; t < K * MT; t += W) {
            const int k = t / MT, ct = t % MT;
            const TileRef<T> tr = btile(k, ct);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int u = colfast ? s0 + 4 * v : f, w = colfast ? f : s0 + 4 * v;
                const int e = k * LT + u, vec = ct * LT + w;
                T val = T(0);
                if (e < n && vec < m)
                    val = alpha * xp[(int64_t)e * Xin.rs + (int64_t)vec * Xin.cs];
                tr.p[tr.at(u, w)] = val;
            }
        }
    }
    __syncthreads();

    if (wave < K) {  // all diagonal tiles at once
        const int r = lane & 15, g = lane >> 4;
        const T *dk = mm.sD + wave * C::DT + r * PS;
        T *xk = mm.sXD + wave * C::DT + r * PS;
        T a[LT], x[4];
#pragma unroll
        for (int c = 0; c < LT; ++c)
            a[c] = dk[c];
        diag_invert<T>(a, dk[r], x, r, g);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            xk[4 * j + g] = (4 * j + g <= r) ? x[j] : T(0);
    }
    __syncthreads();

    const int NW = W - MT;  // wavefronts that own the far updates
    for (int s = 0; s < K; ++s) {
        const int k = fwd ? s : K - 1 - s;
        if (wave < MT) {  // X_k = Li_kk B_k  (Li_kk^T when solving with the transpose)
            T av[4], bv[4];
            typename Mfma<T>::acc_t acc = {0, 0, 0, 0};
            if (fwd)
                op_rows<T>(mm.x(k, k), lane, av);
            else
                op_nat<T>(mm.x(k, k), lane, av);
            op_nat<T>(btile(k, wave), lane, bv);
            acc = mma4<T>(av, bv, acc, false);
            acc_store<T>(btile(k, wave), lane, acc);
        }
        __syncthreads();
        if (s + 1 == K)
            break;
        if (wave < MT) {  // the tile the next step starts from
            const int i = fwd ? k + 1 : k - 1;
            T av[4], bv[4];
            if (fwd)
                op_rows<T>(mm.a(i, k), lane, av);
            else
                op_nat<T>(mm.a(k, i), lane, av);
            op_nat<T>(btile(k, wave), lane, bv);
            typename Mfma<T>::acc_t acc = acc_load<T>(btile(i, wave), lane);
            acc = mma4<T>(av, bv, acc, true);
            acc_store<T>(btile(i, wave), lane, acc);
        } else {
            for (int d = 2; s + d < K; ++d) {
                const int i = fwd ? k + d : k - d;
                for (int ct = 0; ct < MT; ++ct) {
                    if ((i * MT + ct) % NW != wave - MT)
                        continue;
                    T av[4], bv[4];
                    if (fwd)
                        op_rows<T>(mm.a(i, k), lane, av);
                    else
                        op_nat<T>(mm.a(k, i), lane, av);
                    op_nat<T>(btile(k, ct), lane, bv);
                    typename Mfma<T>::acc_t acc = acc_load<T>(btile(i, ct), lane);
                    acc = mma4<T>(av, bv, acc, true);
                    acc_store<T>(btile(i, ct), lane, acc);
                }
            }
        }
    }
    __syncthreads();
    {
        T *xp = X.p + b * X.bs;
        const bool colfast = (X.cs == 1) || (X.rs != 1);
        const int f = lane & 15, s0 = lane >> 4;
        for (int t = wave; t < K * MT; t += W) {
            const int k = t / MT, ct = t % MT;
            const TileRef<T> tr = btile(k, ct);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int u = colfast ? s0 + 4 * v : f, w = colfast ? f : s0 + 4 * v;
                const int e = k * LT + u, vec = ct * LT + w;
                if (e < n && vec < m)
                    xp[(int64_t)e * X.rs + (int64_t)vec * X.cs] = tr.p[tr.at(u, w)];
            }
        }
    }
}

template <typename T>
la_status launch_potrf_leaf16(View<const T> A, View<T> L, View<T> Inv, int32_t *info, int info_off, int64_t batch,
                              int nb, bool zero_upper, hipStream_t st)
{
    if (batch <= 0 || nb <= 0)
        return LA_OK;
    if (nb > LT * LK || batch > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    constexpr size_t lds_bytes = (size_t)Leaf16<T>::TOTAL * sizeof(T);
    if (dry_run())
        return LA_OK;
    static bool configured[64] = {};
    int dev = 0;
    LA_HIP(hipGetDevice(&dev));
    if (dev >= 0 && dev < 64 && !configured[dev]) {
        LA_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_potrf_leaf16<T>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
        configured[dev] = true;
    }
    LA_LAUNCH((k_potrf_leaf16<T>), dim3((unsigned)batch), dim3(LEAF16_THREADS), lds_bytes, st, A, L, Inv, info,
                       info_off, batch, nb, zero_upper ? 1 : 0);
    return launch_check("potrf_leaf16");
}

template la_status launch_potrf_leaf16<float>(View<const float>, View<float>, View<float>, int32_t *, int, int64_t, int,
                                              bool, hipStream_t);
template la_status launch_potrf_leaf16<double>(View<const double>, View<double>, View<double>, int32_t *, int, int64_t,
                                               int, bool, hipStream_t);

template <typename T>
la_status launch_potrf_small16(View<const T> A, View<T> L, int32_t *info, int64_t batch, int n, hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    if (n > LT * SMALL16_MAXK || batch > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    const int K = (n + LT - 1) / LT;
    if (dry_run())
        return LA_OK;
    LA_LAUNCH((k_potrf_small16<T>), dim3((unsigned)batch), dim3(SMALL16_WAVES * 64), (size_t)small16_lds_elems<T>(K) * sizeof(T),
              st, A, L, info, batch, n);
    return launch_check("potrf_small16");
}
template la_status launch_potrf_small16<float>(View<const float>, View<float>, int32_t *, int64_t, int, hipStream_t);
template la_status launch_potrf_small16<double>(View<const double>, View<double>, int32_t *, int64_t, int, hipStream_t);

template <typename T>
la_status launch_tri_inverse128(View<const T> Lam, View<T> Inv, int64_t batch, int n, hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    const int nblk = (n + LT * LK - 1) / (LT * LK);
    if (batch * nblk > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    constexpr size_t lds_bytes = (size_t)Leaf16<T>::TOTAL * sizeof(T);
    if (dry_run())
        return LA_OK;
    static bool configured[64] = {};
    int dev = 0;
    LA_HIP(hipGetDevice(&dev));
    if (dev >= 0 && dev < 64 && !configured[dev]) {
        LA_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_tri_inv_leaf16<T>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
        configured[dev] = true;
    }
    LA_LAUNCH((k_tri_inv_leaf16<T>), dim3((unsigned)(batch * nblk)), dim3(LEAF16_THREADS), lds_bytes, st, Lam,
                       Inv, batch, n, nblk);
    return launch_check("tri_inverse128");
}

template la_status launch_tri_inverse128<float>(View<const float>, View<float>, int64_t, int, hipStream_t);
template la_status launch_tri_inverse128<double>(View<const double>, View<double>, int64_t, int, hipStream_t);

template <typename T>
la_status launch_trsm_leaf16(View<const T> Lam, View<const T> Xin, View<T> X, int64_t batch, int n, int m, T alpha,
                             bool fwd, hipStream_t st)
{
    if (batch <= 0 || n <= 0 || m <= 0)
        return LA_OK;
    if (n > LT * LK || m > LT * TRSM16_MAX_CT || batch > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    const int K = (n + LT - 1) / LT, MT = (m + LT - 1) / LT;
    const size_t lds_bytes = (size_t)trsm16_lds_elems<T>(K, MT) * sizeof(T);
    if (dry_run())
        return LA_OK;
    static bool configured[64] = {};
    int dev = 0;
    LA_HIP(hipGetDevice(&dev));
    if (dev >= 0 && dev < 64 && !configured[dev]) {
        LA_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_trsm_leaf16<T, LEAF16_WAVES, LK>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        LA_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_trsm_leaf16<T, 4, 4>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        configured[dev] = true;
    }
    // many items of at most four tile rows: four wavefronts each (one per tile of right-hand sides walks the
    // chain, which leaves at least one for the far updates), several workgroups per compute unit
    if (K <= 4 && batch > 1024 && lds_bytes <= 40 * 1024)
        LA_LAUNCH((k_trsm_leaf16<T, 4, 4>), dim3((unsigned)batch), dim3(4 * 64), lds_bytes, st, Lam, Xin, X, batch, n, m, alpha,
                  fwd ? 1 : 0);
    else
        LA_LAUNCH((k_trsm_leaf16<T, LEAF16_WAVES, LK>), dim3((unsigned)batch), dim3(LEAF16_THREADS), lds_bytes, st, Lam, Xin, X,
                  batch, n, m, alpha, fwd ? 1 : 0);
    return launch_check("trsm_leaf16");
}

template la_status launch_trsm_leaf16<float>(View<const float>, View<const float>, View<float>, int64_t, int, int, float,
                                             bool, hipStream_t);
template la_status launch_trsm_leaf16<double>(View<const double>, View<const double>, View<double>, int64_t, int, int,
                                              double, bool, hipStream_t);

// largest n the one-workgroup backward kernel takes: three tile areas must fit the 160 KB of LDS
template <typename T>
int backward_leaf16_max_n()
{
    int K = LK;
    while (K > 0 && 3 * (size_t)backward16_area<T>(K) * sizeof(T) > 160 * 1024)
        --K;
    return K * LT;
}
template int backward_leaf16_max_n<float>();
template int backward_leaf16_max_n<double>();

template <typename T>
la_status launch_backward_leaf16(View<const T> Lam, View<const T> G, View<T> Abar, int64_t batch, int n, hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    if (n > backward_leaf16_max_n<T>() || batch > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    const int K = (n + LT - 1) / LT;
    const size_t lds_bytes = 3 * (size_t)backward16_area<T>(K) * sizeof(T);
    if (dry_run())
        return LA_OK;
    static bool configured[64] = {};
    int dev = 0;
    LA_HIP(hipGetDevice(&dev));
    if (dev >= 0 && dev < 64 && !configured[dev]) {
        LA_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_backward_leaf16<T, LEAF16_WAVES, LK>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        LA_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_backward_leaf16<T, 4, 4>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        configured[dev] = true;
    }
    // more matrices than two rounds of the 512 places that 16-wavefront workgroups have on the chip, and small
    // enough for four workgroups per compute unit (fp64 with four tile rows needs 65 KB: no gain there)
    if (K <= 4 && batch > 1024 && lds_bytes <= 40 * 1024)
        LA_LAUNCH((k_backward_leaf16<T, 4, 4>), dim3((unsigned)batch), dim3(4 * 64), lds_bytes, st, Lam, G, Abar, batch, n);
    else
        LA_LAUNCH((k_backward_leaf16<T, LEAF16_WAVES, LK>), dim3((unsigned)batch), dim3(LEAF16_THREADS), lds_bytes, st, Lam,
                  G, Abar, batch, n);
    return launch_check("backward_leaf16");
}

template la_status launch_backward_leaf16<float>(View<const float>, View<const float>, View<float>, int64_t, int,
                                                 hipStream_t);
template la_status launch_backward_leaf16<double>(View<const double>, View<const double>, View<double>, int64_t, int,
                                                  hipStream_t);

template <typename T>
la_status launch_potri_leaf16(View<const T> Lam, View<T> B, int64_t batch, int n, hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    if (n > LT * LK || batch > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    const int K = (n + LT - 1) / LT;
    const size_t lds_bytes = 2 * (size_t)backward16_area<T>(K) * sizeof(T);
    if (dry_run())
        return LA_OK;
    static bool configured[64] = {};
    int dev = 0;
    LA_HIP(hipGetDevice(&dev));
    if (dev >= 0 && dev < 64 && !configured[dev]) {
        LA_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_potri_leaf16<T, LEAF16_WAVES, LK>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        LA_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_potri_leaf16<T, 4, 4>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        configured[dev] = true;
    }
    if (K <= 4 && batch > 1024 && lds_bytes <= 40 * 1024)  // as for the backward kernel
        LA_LAUNCH((k_potri_leaf16<T, 4, 4>), dim3((unsigned)batch), dim3(4 * 64), lds_bytes, st, Lam, B, batch, n);
    else
        LA_LAUNCH((k_potri_leaf16<T, LEAF16_WAVES, LK>), dim3((unsigned)batch), dim3(LEAF16_THREADS), lds_bytes, st, Lam, B,
                  batch, n);
    return launch_check("potri_leaf16");
}
template la_status launch_potri_leaf16<float>(View<const float>, View<float>, int64_t, int, hipStream_t);
template la_status launch_potri_leaf16<double>(View<const double>, View<double>, int64_t, int, hipStream_t);

// LDS of k_outer_leaf16 with NW wavefronts: the operand tiles and a staging tile per wavefront
template <typename T>
static size_t outer_leaf_lds(int n, int k, bool two, int nw)
{
    const int Kn = (n + LT - 1) / LT, Kk = (k + LT - 1) / LT;
    return ((size_t)(two ? 2 : 1) * Kn * Kk + nw) * Leaf16<T>::OT * sizeof(T);
}
template <typename T>
bool outer_leaf_takes(int64_t batch, int n, int k, bool two)
{
    // worth it while a matrix is too small for the tiles of the general product to fill the chip, and as
    // long as a few workgroups fit a compute unit
    // (measured against the general product, 4096 items of 64 x 64 with k = 64 in fp32: one operand 80 -> 40 us,
    // two operands 157 -> 181 us for the whole trmm backward rule, hence the tile limit on two operands)
    const int Kn = (n + LT - 1) / LT, Kk = (k + LT - 1) / LT;
    if (two && Kn * Kk > 8)
        return false;
    return n > 16 && n <= 128 && k >= 1 && k <= 128 && batch >= 64 && outer_leaf_lds<T>(n, k, two, LEAF16_WAVES) <= 64 * 1024;
}
template bool outer_leaf_takes<float>(int64_t, int, int, bool);
template bool outer_leaf_takes<double>(int64_t, int, int, bool);

template <typename T>
la_status launch_outer_leaf(int tri, T alpha, int64_t batch, int n, int k, View<const T> U, View<const T> V, View<T> C,
                            hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    if (!outer_leaf_takes<T>(batch, n, k, tri != 0) || batch > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    if (dry_run())
        return LA_OK;
    static bool configured[64] = {};
    int dev = 0;
    LA_HIP(hipGetDevice(&dev));
    if (dev >= 0 && dev < 64 && !configured[dev]) {
        LA_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_outer_leaf16<T, LEAF16_WAVES>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024));
        LA_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_outer_leaf16<T, 4>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024));
        configured[dev] = true;
    }
    const int Kn = (n + LT - 1) / LT;
    const int tiles = tri == 0 ? Kn * (Kn + 1) / 2 : Kn * Kn;
    if (tiles <= 16 && batch > 1024) {  // many small items: four wavefronts each
        LA_LAUNCH((k_outer_leaf16<T, 4>), dim3((unsigned)batch), dim3(4 * 64), outer_leaf_lds<T>(n, k, tri != 0, 4), st, U, V,
                  C, batch, n, k, alpha, tri);
    } else {
        LA_LAUNCH((k_outer_leaf16<T, LEAF16_WAVES>), dim3((unsigned)batch), dim3(LEAF16_THREADS),
                  outer_leaf_lds<T>(n, k, tri != 0, LEAF16_WAVES), st, U, V, C, batch, n, k, alpha, tri);
    }
    return launch_check("outer_leaf16");
}
template la_status launch_outer_leaf<float>(int, float, int64_t, int, int, View<const float>, View<const float>, View<float>,
                                            hipStream_t);
template la_status launch_outer_leaf<double>(int, double, int64_t, int, int, View<const double>, View<const double>,
                                             View<double>, hipStream_t);

template <typename T>
static size_t symm_leaf_lds(int n, int k, int nw)
{
    const int Kn = (n + LT - 1) / LT, Kk = (k + LT - 1) / LT;
    return ((size_t)Kn * Kn + (size_t)Kn * Kk + nw) * Leaf16<T>::OT * sizeof(T);
}
template <typename T>
bool symm_leaf_takes(int64_t batch, int n, int k)
{
    const int Kn = (n + LT - 1) / LT, Kk = (k + LT - 1) / LT;
    const int nw = (Kn * Kk <= 16 && batch > 1024) ? 4 : LEAF16_WAVES;  // as launch_symm_leaf chooses
    return n > 16 && n <= 128 && k >= 1 && k <= 128 && batch >= 64 && symm_leaf_lds<T>(n, k, nw) <= 64 * 1024;
}
template bool symm_leaf_takes<float>(int64_t, int, int);
template bool symm_leaf_takes<double>(int64_t, int, int);

template <typename T>
la_status launch_symm_leaf(T alpha, int64_t batch, int n, int k, View<const T> G, View<const T> A, View<T> Out,
                           hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    if (!symm_leaf_takes<T>(batch, n, k) || batch > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    if (dry_run())
        return LA_OK;
    const int Kn = (n + LT - 1) / LT, Kk = (k + LT - 1) / LT;
    if (Kn * Kk <= 16 && batch > 1024) {  // many small items: four wavefronts each
        LA_LAUNCH((k_symm_leaf16<T, 4>), dim3((unsigned)batch), dim3(4 * 64), symm_leaf_lds<T>(n, k, 4), st, G, A, Out, batch,
                  n, k, alpha);
    } else {
        LA_LAUNCH((k_symm_leaf16<T, LEAF16_WAVES>), dim3((unsigned)batch), dim3(LEAF16_THREADS),
                  symm_leaf_lds<T>(n, k, LEAF16_WAVES), st, G, A, Out, batch, n, k, alpha);
    }
    return launch_check("symm_leaf16");
}
template la_status launch_symm_leaf<float>(float, int64_t, int, int, View<const float>, View<const float>, View<float>,
                                           hipStream_t);
template la_status launch_symm_leaf<double>(double, int64_t, int, int, View<const double>, View<const double>, View<double>,
                                            hipStream_t);

template <typename T>
static size_t trmm_leaf_lds(int n, int m, int nw)
{
    const int Kn = (n + LT - 1) / LT, Km = (m + LT - 1) / LT;
    return ((size_t)backward16_area<T>(Kn) + ((size_t)Kn * Km + nw) * Leaf16<T>::OT) * sizeof(T);
}
template <typename T>
bool trmm_leaf_takes(int64_t batch, int n, int m)
{
    return n >= 1 && n <= 128 && m >= 1 && m <= 128 && batch >= 64 && trmm_leaf_lds<T>(n, m, LEAF16_WAVES) <= 64 * 1024;
}
template bool trmm_leaf_takes<float>(int64_t, int, int);
template bool trmm_leaf_takes<double>(int64_t, int, int);

template <typename T>
la_status launch_trmm_leaf(View<const T> Lam, View<const T> Xin, View<T> X, int64_t batch, int n, int m, T alpha, bool fwd,
                           hipStream_t st)
{
    if (batch <= 0 || n <= 0 || m <= 0)
        return LA_OK;
    if (!trmm_leaf_takes<T>(batch, n, m) || batch > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    if (dry_run())
        return LA_OK;
    const int Kn = (n + LT - 1) / LT, Km = (m + LT - 1) / LT;
    if (Kn <= 4 && Kn * Km <= 16 && batch > 1024) {  // many small items: four wavefronts each
        LA_LAUNCH((k_trmm_leaf16<T, 4, 4>), dim3((unsigned)batch), dim3(4 * 64), trmm_leaf_lds<T>(n, m, 4), st, Lam, Xin, X,
                  batch, n, m, alpha, fwd ? 1 : 0);
    } else {
        LA_LAUNCH((k_trmm_leaf16<T, LEAF16_WAVES, LK>), dim3((unsigned)batch), dim3(LEAF16_THREADS),
                  trmm_leaf_lds<T>(n, m, LEAF16_WAVES), st, Lam, Xin, X, batch, n, m, alpha, fwd ? 1 : 0);
    }
    return launch_check("trmm_leaf16");
}
template la_status launch_trmm_leaf<float>(View<const float>, View<const float>, View<float>, int64_t, int, int, float, bool,
                                           hipStream_t);
template la_status launch_trmm_leaf<double>(View<const double>, View<const double>, View<double>, int64_t, int, int, double,
                                            bool, hipStream_t);

template <typename T>
la_status launch_gp_leaf16(View<const T> A, const T *y, T *loss, View<T> Abar, int32_t *info, int64_t batch, int n,
                           hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    if (n > backward_leaf16_max_n<T>() || batch > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    const int K = (n + LT - 1) / LT;
    const size_t lds_bytes = (3 * (size_t)backward16_area<T>(K) + 4 * LT * LK) * sizeof(T);
    if (dry_run())
        return LA_OK;
    static bool configured[64] = {};
    int dev = 0;
    LA_HIP(hipGetDevice(&dev));
    if (dev >= 0 && dev < 64 && !configured[dev]) {
        const size_t most = (3 * (size_t)backward16_area<T>(backward_leaf16_max_n<T>() / LT) + 4 * LT * LK) * sizeof(T);
        LA_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gp_leaf16<T>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)most));
        configured[dev] = true;
    }
    LA_LAUNCH((k_gp_leaf16<T>), dim3((unsigned)batch), dim3(LEAF16_THREADS), lds_bytes, st, A, y, loss, Abar,
                       info, batch, n);
    return launch_check("gp_leaf16");
}
template la_status launch_gp_leaf16<float>(View<const float>, const float *, float *, View<float>, int32_t *, int64_t,
                                           int, hipStream_t);
template la_status launch_gp_leaf16<double>(View<const double>, const double *, double *, View<double>, int32_t *,
                                            int64_t, int, hipStream_t);

}  // namespace la
