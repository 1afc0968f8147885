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
// Two kernels:
//  * k_gemm_fast: 16-byte vector loads, register prefetch of the next K slab while the
//    current one is multiplied out of LDS, 128x128 (K slabs of 16, double-buffered LDS, one
//    barrier per slab), 64x64 or 32x32 workgroup tiles (K slabs of 64 for the small,
//    latency-bound grids of the recursion's lower levels; 32x32 when 64x64 tiles would leave
//    most compute units idle), four wavefronts in a 2 x 2 arrangement, 16x16x4
//    MFMA (v_mfma_f64_16x16x4_f64 / v_mfma_f32_16x16x4_f32).  Needs 16-byte aligned operands
//    and K a multiple of 16.
//  * k_gemm: element-wise staged fallback for everything else (ragged / unaligned shapes).
#include <algorithm>

#include "common.hpp"

namespace la {

__device__ __forceinline__ bool tri_keep(int tri, int o, int k)
{
    // tri 1 keeps o >= k, tri 2 keeps o <= k
    return tri == 0 || (tri == 1 ? (o >= k) : (o <= k));
}

// ---------------------------------------------------------------------------------------
// Workgroup -> work slot mapping.  Consecutive workgroups are dealt round-robin to the 8 XCDs
// (each with its own L2).  Slots are regrouped in chunks of 8 x 16: inside a chunk every XCD
// gets 16 consecutive slots (neighbouring tiles of one tile row share their A panel in that
// XCD's L2), while all XCDs still advance through the slot list at the same pace, which
// matters because triangular operands make the work per tile vary along the list.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ int64_t xcd_slot(int64_t w, int64_t total, int CH = 16)
{
    const int64_t c = w / (8 * CH);
    if ((c + 1) * 8 * CH > total)
        return w;  // incomplete last chunk keeps its order
    const int r = (int)(w % (8 * CH));
    return c * 8 * CH + (r % 8) * CH + r / 8;
}

// Tile enumeration.  Workgroups go to XCDs in a fixed round-robin, so the list of tiles must be
// (a) free of tiles that have nothing to do and (b) ordered so that the work per tile changes
// slowly along it; then every XCD ends up with the same share.
//   order 0: all tiles, row-major.
//   order 1: tiles on or below the diagonal only (tn <= tm), row by row.
//   order 2: tiles on or above the diagonal only (tm <= tn), column by column.
//   order 3: all tiles of a square grid in "shells" max(tm, tn) = s, s ascending: every tile of
//            a shell has the same K range when both operands are triangular.
//   order 4: all tiles, column-major (the K range depends on the column only when just B is
//            triangular).
//   order 5: tiles on or below the diagonal in bands of 8 diagonals tm - tn = d, the band with the
//            largest d first; inside a band row by row from the last row up, a row's tiles by
//            falling d.  For lower x lower = lower products the K range of a tile is d + 1 tile
//            edges, so this list is nearly sorted by work (which the slots need to fill evenly:
//            the heaviest tile is three times the mean) while the (up to) 8 consecutive tiles of a
//            row still share their A panel.
__device__ __forceinline__ void decode_tile(int order, int t, int tiles_m, int tiles_n, int &tm, int &tn)
{
    if (order == 0) {
        tm = t / tiles_n;
        tn = t % tiles_n;
    } else if (order == 4) {
        tn = t / tiles_m;
        tm = t % tiles_m;
    } else if (order == 5) {
        const int T = tiles_m;
        int b = (T - 1) / 8;
        for (;; --b) {  // band: diagonals 8 b .. min(T - 1, 8 b + 7)
            const int dlo = 8 * b, dhi = min(T - 1, dlo + 7);
            const int cnt = (dhi - dlo + 1) * T - (dlo + dhi) * (dhi - dlo + 1) / 2;  // sum of T - d
            if (t < cnt || b == 0)
                break;
            t -= cnt;
        }
        const int dlo = 8 * b, dhi = min(T - 1, dlo + 7);
        int i = T - 1;
        for (;; --i) {  // row i holds the diagonals min(dhi, i) .. dlo of the band
            const int cnt = min(dhi, i) - dlo + 1;
            if (t < cnt || i == dlo)
                break;
            t -= cnt;
        }
        tm = i;
        tn = i - (min(dhi, i) - t);
    } else if (order == 3) {
        int s_ = (int)sqrt((double)t);
        while ((s_ + 1) * (s_ + 1) <= t)
            ++s_;
        while (s_ * s_ > t)
            --s_;
        const int r = t - s_ * s_;
        if (r <= s_) {
            tm = s_;
            tn = r;
        } else {
            tm = r - s_ - 1;
            tn = s_;
        }
    } else {
        int a = (int)((sqrt(8.0 * (double)t + 1.0) - 1.0) * 0.5);
        while ((a + 1) * (a + 2) / 2 <= t)
            ++a;
        while (a * (a + 1) / 2 > t)
            --a;
        const int b = t - a * (a + 1) / 2;
        tm = order == 1 ? a : b;
        tn = order == 1 ? b : a;
    }
}

__device__ __forceinline__ int64_t tile_count_dev(int order, int tiles_m, int tiles_n)
{
    if (order == 1 || order == 2 || order == 5)
        return (int64_t)tiles_m * (tiles_m + 1) / 2;
    return (int64_t)tiles_m * tiles_n;
}
static inline int64_t tile_count(int order, int tiles_m, int tiles_n)
{
    if (order == 1 || order == 2 || order == 5)
        return (int64_t)tiles_m * (tiles_m + 1) / 2;
    return (int64_t)tiles_m * tiles_n;
}

// ---------------------------------------------------------------------------------------
// Fallback kernel: element-wise staging, any strides / sizes.
// ---------------------------------------------------------------------------------------
template <int BM, int BN, int BK>
struct GemmCfg {
    static constexpr int PAD = 16;
    static constexpr int A_ELEMS = (BK * (BM + PAD) > BM * (BK + 1)) ? BK * (BM + PAD) : BM * (BK + 1);
    static constexpr int B_ELEMS = (BK * (BN + PAD) > BN * (BK + 1)) ? BK * (BN + PAD) : BN * (BK + 1);
};

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
        if ((og < no) && (kg < kmax) && tri_keep(tri, og, kg))
            v = src[(int64_t)og * so + (int64_t)kg * sk];
        s[kfast ? (o * (BK + 1) + k) : (k * (OUT + PAD) + o)] = v;
    }
}

__device__ __forceinline__ void k_range(const GemmOpts &o, int i0, int j0, int BM, int BN, int K, int &kbeg, int &kend)
{
    kbeg = 0;
    kend = K;
    if (o.triA == 1)
        kend = min(kend, i0 + BM);
    else if (o.triA == 2)
        kbeg = max(kbeg, i0);
    if (o.triB == 1)
        kbeg = max(kbeg, j0);
    else if (o.triB == 2)
        kend = min(kend, j0 + BN);
}

// GemmOpts::symsum: the lower triangle's values go to both triangles
template <typename T>
__device__ __forceinline__ void store_c_sym(T *Cp, int64_t rs, int64_t cs, int i, int j, int M, T acc, T alpha)
{
    if (i < M && j <= i) {
        const T upd = alpha * acc;
        Cp[(int64_t)i * rs + (int64_t)j * cs] = upd;
        if (j < i)
            Cp[(int64_t)j * rs + (int64_t)i * cs] = upd;
    }
}

template <typename T>
__device__ __forceinline__ void store_c(T *Cp, int64_t rs, int64_t cs, int i, int j, int M, int N, T acc, T alpha,
                                        T beta, const GemmOpts &o)
{
    if (i < M && j < N && !(o.maskC == 1 && i < j) && !(o.maskC == 2 && i > j)) {
        T upd = alpha * acc;
        if (o.halfDiag && i == j)
            upd *= T(0.5);
        T *c = Cp + (int64_t)i * rs + (int64_t)j * cs;
        *c = (beta == T(0)) ? upd : fma(beta, *c, upd);
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
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int TM = WM / 16, TN = WN / 16;
    __shared__ T sA[Cfg::A_ELEMS];
    __shared__ T sB[Cfg::B_ELEMS];

    const int64_t bid = blockIdx.x;
    const int64_t per = tile_count_dev(o.order, tiles_m, tiles_n);
    const int64_t b = bid / per;
    int tile = (int)(bid % per);
    if (o.reverse && o.order != 5)
        tile = (int)per - 1 - tile;
    int tm, tn;
    decode_tile(o.order, tile, tiles_m, tiles_n, tm, tn);
    const int i0 = tm * BM, j0 = tn * BN;
    if ((o.maskC == 1 && j0 > i0 + BM - 1) || (o.maskC == 2 && i0 > j0 + BN - 1))
        return;  // tile entirely on the masked side of the diagonal

    int kbeg, kend;
    k_range(o, i0, j0, BM, BN, K, kbeg, kend);
    kbeg = (kbeg / BK) * BK;

    const T *Ap = A.item(b);
    const T *Bp = B.item(b);
    T *Cp = C.item(b);
    const bool a_kfast = (A.cs == 1);
    const bool b_kfast = (B.rs == 1);

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
    const int triB_o = o.triB == 1 ? 2 : (o.triB == 2 ? 1 : 0);  // in (j, k) order

    for (int pass = 0; pass <= o.symsum; ++pass) {
    if (pass == 1) {  // second half of A B + B^T A^T: same strides, the base pointers change places
        const T *t = Ap;
        Ap = Bp;
        Bp = t;
    }
    for (int k0 = kbeg; k0 < kend; k0 += BK) {
        stage_slab<T, BM, BK, PAD>(sA, Ap, A.rs, A.cs, i0, M, k0, kend, o.triA, a_kfast);
        stage_slab<T, BN, BK, PAD>(sB, Bp, B.cs, B.rs, j0, N, k0, kend, triB_o, b_kfast);
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
    }

#pragma unroll
    for (int x = 0; x < TM; ++x)
#pragma unroll
        for (int y = 0; y < TN; ++y)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = i0 + wm + x * 16 + MF::row(lane, v), j = j0 + wn + y * 16 + l16;
                if (o.symsum)
                    store_c_sym<T>(Cp, C.rs, C.cs, i, j, M, acc[x][y][v], alpha);
                else
                    store_c<T>(Cp, C.rs, C.cs, i, j, M, N, acc[x][y][v], alpha, beta, o);
            }
}

// ---------------------------------------------------------------------------------------
// Fast kernel.  AKF: A(i,k) has k contiguous (A.cs == 1), else i contiguous (A.rs == 1).
// BKF: B(k,j) has k contiguous (B.rs == 1), else j contiguous (B.cs == 1).
// LDS slab layouts (chosen so that global->LDS stores are 16-byte vectors and the MFMA
// fragment reads are bank-conflict free):
//   k contiguous:     s[o][BK + VW]      (row stride 18 doubles / 20 floats)
//   outer contiguous: s[k][OUT + 16]
// ---------------------------------------------------------------------------------------
template <typename T, int OUT, int BK, bool KF>
struct Slab {
    using MF = Mfma<T>;
    static constexpr int VW = MF::VW;
    static constexpr int LD = KF ? (BK + VW) : (OUT + 16);
    static constexpr int ELEMS = KF ? OUT * LD : BK * LD;
    static constexpr int NCH = OUT * BK / VW / 256;  // 16-byte chunks per thread
    static_assert(NCH >= 1, "tile too small for 256 threads");
    static constexpr int so = KF ? LD : 1;  // LDS stride of the outer index
    static constexpr int sk = KF ? 1 : LD;  // LDS stride of k

    // (outer, k) of chunk c of this thread
    static __device__ __forceinline__ void coords(int c, int &o, int &k)
    {
        const int q = c * 256 + threadIdx.x;
        if constexpr (KF) {
            o = q / (BK / VW);
            k = (q % (BK / VW)) * VW;
        } else {
            k = q / (OUT / VW);
            o = (q % (OUT / VW)) * VW;
        }
    }
};

template <typename T, int OUT, int BK, bool KF, typename RV>
__device__ __forceinline__ void slab_fetch(RV &r, const T *src, int64_t so, int64_t sk, int o0, int no, int k0)
{
    using S = Slab<T, OUT, BK, KF>;
    using V = typename Mfma<T>::vec_t;
#pragma unroll
    for (int c = 0; c < S::NCH; ++c) {
        int o, k;
        S::coords(c, o, k);
        V v;
        if constexpr (S::VW == 2)
            v = V{0, 0};
        else
            v = V{0, 0, 0, 0};
        if (o0 + o < no)  // whole chunk in range: K is a multiple of BK, `no` a multiple of VW when !KF
            v = *reinterpret_cast<const V *>(src + (int64_t)(o0 + o) * so + (int64_t)(k0 + k) * sk);
        r[c] = v;
    }
}

template <typename T, int OUT, int BK, bool KF, typename RV>
__device__ __forceinline__ void slab_commit(T *s, RV &r, int o0, int k0, int tri)
{
    using S = Slab<T, OUT, BK, KF>;
    using V = typename Mfma<T>::vec_t;
    // Does this slab touch the zero side of a triangular operand at all?  Decided once per slab
    // (a scalar branch); most slabs do not and take the plain copy below.
    bool need_mask = false;
    if (tri == 1)
        need_mask = (o0 < k0 + BK - 1);  // keep o >= k: some (o, k) with o < k exists
    else if (tri == 2)
        need_mask = (o0 + OUT - 1 > k0);
    if (!need_mask) {
#pragma unroll
        for (int c = 0; c < S::NCH; ++c) {
            int o, k;
            S::coords(c, o, k);
            *reinterpret_cast<V *>(s + o * S::so + k * S::sk) = r[c];
        }
        return;
    }
    // keep o >= k (tri 1) or o <= k (tri 2): with d = (o - k) for tri 1 and (k - o) for tri 2, keep d >= 0
    const int sgn = tri == 1 ? 1 : -1;
#pragma unroll
    for (int c = 0; c < S::NCH; ++c) {
        int o, k;
        S::coords(c, o, k);
        V v = r[c];
        T *e = reinterpret_cast<T *>(&v);
        const int d0 = sgn * ((o0 + o) - (k0 + k));
#pragma unroll
        for (int u = 0; u < S::VW; ++u) {
            const int d = d0 + (KF ? -sgn * u : sgn * u);  // element u moves along k (KF) or along o
            e[u] = d >= 0 ? e[u] : T(0);
        }
        *reinterpret_cast<V *>(s + o * S::so + k * S::sk) = v;
    }
}

template <typename T, int BM, int BN, int BK, int NBUF, bool AKF, bool BKF, bool SYM = false>
__global__ __launch_bounds__(256, 2) void k_gemm_fast(View<const T> A, View<const T> B, View<T> C, int64_t batch, int M,
                                                   int N, int K, T alpha, T beta, GemmOpts o, int tiles_m, int tiles_n)
{
    using MF = Mfma<T>;
    using acc_t = typename MF::acc_t;
    using V = typename MF::vec_t;
    using SA = Slab<T, BM, BK, AKF>;
    using SB = Slab<T, BN, BK, BKF>;
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int TM = WM / 16, TN = WN / 16;
    __shared__ __align__(16) T sA[NBUF][SA::ELEMS];
    __shared__ __align__(16) T sB[NBUF][SB::ELEMS];

    const int64_t per = tile_count_dev(o.order, tiles_m, tiles_n);
    int64_t b;
    int tile;
    if (o.xcd_batch) {
        // Batched launch: XCD x (workgroups x, x + 8, ...) owns the items b = x, x + 8, ... and
        // goes through the tile list once for all of them, tile by tile.  The tile lists are
        // heaviest-first, so the uneven tiles of triangular problems pack well over the
        // workgroup slots, and the tiles of one item still meet in one L2.
        const int x = (int)(blockIdx.x & 7);
        const int64_t q = blockIdx.x >> 3, mpx = (batch + 7) >> 3;
        tile = (int)(q / mpx);
        b = (q % mpx) * 8 + x;
        if (b >= batch)
            return;
    } else {
        // a few items: tile-major too (tile t of every item, then tile t + 1, ...)
        const int64_t slot = xcd_slot(blockIdx.x, per * batch, o.order == 5 ? 8 : 16);
        tile = (int)(slot / batch);
        b = slot % batch;
    }
    if (o.reverse && o.order != 5)
        tile = (int)per - 1 - tile;  // heaviest tiles first when the work grows along the tile list
    int tm, tn;
    decode_tile(o.order, tile, tiles_m, tiles_n, tm, tn);
    const int i0 = tm * BM, j0 = tn * BN;
    if ((o.maskC == 1 && j0 > i0 + BM - 1) || (o.maskC == 2 && i0 > j0 + BN - 1))
        return;

    int Kl = K;  // slice s of a split K range: K elements from s * K on, fewer for the last slice
    if (o.ksplit > 1)
        Kl = min(K, o.ktotal - (int)(b % o.ksplit) * K);
    int kbeg, kend;
    k_range(o, i0, j0, BM, BN, Kl, kbeg, kend);
    kbeg = (kbeg / BK) * BK;
    kend = ((kend + BK - 1) / BK) * BK;  // K is a multiple of BK, so this stays <= K

    const T *Ap = A.item(b);
    const T *Bp = B.item(b);
    T *Cp = C.item(b);
    const int triB_o = o.triB == 1 ? 2 : (o.triB == 2 ? 1 : 0);

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wm = (w >> 1) * WM, wn = (w & 1) * WN;
    const int l16 = lane & 15, lk = lane >> 4;

    acc_t acc[TM][TN];
#pragma unroll
    for (int x = 0; x < TM; ++x)
#pragma unroll
        for (int y = 0; y < TN; ++y)
            acc[x][y] = acc_t{0, 0, 0, 0};

    // Software pipeline.  Slabs travel global memory -> registers -> LDS -> matrix cores.
    // Two LDS buffers: while slab s is multiplied out of one buffer, slab s+1 (already in
    // registers) is written into the other and slab s+2 is requested from memory, so the only
    // thing between two blocks of MFMAs is one barrier: it orders the reads of slab s before
    // the overwrite by slab s+2 and the writes of slab s+1 before their reads.
    // One LDS buffer: slab s+1 is fetched into registers while slab s is multiplied, and written
    // once everybody is done reading (two barriers per slab).
    V ra[SA::NCH], rb[SB::NCH];
    auto multiply = [&](const T *a_s, const T *b_s) {
#pragma unroll
        for (int kk = 0; kk < BK; kk += 4) {
            T af[TM], bf[TN];
#pragma unroll
            for (int x = 0; x < TM; ++x)
                af[x] = a_s[(wm + x * 16 + l16) * SA::so + (kk + lk) * SA::sk];
#pragma unroll
            for (int y = 0; y < TN; ++y)
                bf[y] = b_s[(wn + y * 16 + l16) * SB::so + (kk + lk) * SB::sk];
#pragma unroll
            for (int x = 0; x < TM; ++x)
#pragma unroll
                for (int y = 0; y < TN; ++y)
                    acc[x][y] = MF::run(af[x], bf[y], acc[x][y]);
        }
    };
    // SYM (GemmOpts::symsum): a second pass adds B^T A^T -- same strides, the base pointers change places
    for (int pass = 0; pass < (SYM ? 2 : 1); ++pass) {
    if (SYM && pass == 1) {
        const T *t = Ap;
        Ap = Bp;
        Bp = t;
    }
    if constexpr (NBUF == 2) {
        if (kbeg < kend) {
            slab_fetch<T, BM, BK, AKF>(ra, Ap, A.rs, A.cs, i0, M, kbeg);
            slab_fetch<T, BN, BK, BKF>(rb, Bp, B.cs, B.rs, j0, N, kbeg);
            slab_commit<T, BM, BK, AKF>(sA[0], ra, i0, kbeg, o.triA);
            slab_commit<T, BN, BK, BKF>(sB[0], rb, j0, kbeg, triB_o);
            if (kbeg + BK < kend) {
                slab_fetch<T, BM, BK, AKF>(ra, Ap, A.rs, A.cs, i0, M, kbeg + BK);
                slab_fetch<T, BN, BK, BKF>(rb, Bp, B.cs, B.rs, j0, N, kbeg + BK);
            }
            __syncthreads();
        }
        int buf = 0;
        for (int k0 = kbeg; k0 < kend; k0 += BK) {
            if (k0 + BK < kend) {
                slab_commit<T, BM, BK, AKF>(sA[buf ^ 1], ra, i0, k0 + BK, o.triA);
                slab_commit<T, BN, BK, BKF>(sB[buf ^ 1], rb, j0, k0 + BK, triB_o);
            }
            if (k0 + 2 * BK < kend) {
                slab_fetch<T, BM, BK, AKF>(ra, Ap, A.rs, A.cs, i0, M, k0 + 2 * BK);
                slab_fetch<T, BN, BK, BKF>(rb, Bp, B.cs, B.rs, j0, N, k0 + 2 * BK);
            }
            multiply(sA[buf], sB[buf]);
            __syncthreads();
            buf ^= 1;
        }
    } else {
        if (kbeg < kend) {
            slab_fetch<T, BM, BK, AKF>(ra, Ap, A.rs, A.cs, i0, M, kbeg);
            slab_fetch<T, BN, BK, BKF>(rb, Bp, B.cs, B.rs, j0, N, kbeg);
        }
        for (int k0 = kbeg; k0 < kend; k0 += BK) {
            slab_commit<T, BM, BK, AKF>(sA[0], ra, i0, k0, o.triA);
            slab_commit<T, BN, BK, BKF>(sB[0], rb, j0, k0, triB_o);
            __syncthreads();
            if (k0 + BK < kend) {
                slab_fetch<T, BM, BK, AKF>(ra, Ap, A.rs, A.cs, i0, M, k0 + BK);
                slab_fetch<T, BN, BK, BKF>(rb, Bp, B.cs, B.rs, j0, N, k0 + BK);
            }
            multiply(sA[0], sB[0]);
            __syncthreads();
        }
    }
    }

#pragma unroll
    for (int x = 0; x < TM; ++x)
#pragma unroll
        for (int y = 0; y < TN; ++y)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = i0 + wm + x * 16 + MF::row(lane, v), j = j0 + wn + y * 16 + l16;
                if constexpr (SYM)
                    store_c_sym<T>(Cp, C.rs, C.cs, i, j, M, acc[x][y][v], alpha);
                else
                    store_c<T>(Cp, C.rs, C.cs, i, j, M, N, acc[x][y][v], alpha, beta, o);
            }
}

// ---------------------------------------------------------------------------------------
// Thin products: at most GEMV_N columns (matrix times a few vectors).  They are bound by reading A
// once, which the tile kernels above are not built for.  A may be masked (triA); B and C are plain.
//   A with k contiguous: one wavefront per row, lanes stride over k, shuffle reduction.
//   A with i contiguous: a block takes 64 rows, its eight wavefronts an eighth of the k range each
//   (every load is 64 consecutive elements), LDS reduction.
// ---------------------------------------------------------------------------------------
constexpr int GEMV_N = 8;
constexpr int GEMV_THREADS = 512;

template <typename T>
__global__ __launch_bounds__(GEMV_THREADS) void k_gemv(View<const T> A, View<const T> B, View<T> C, int64_t batch, int M, int N,
                                              int K, T alpha, T beta, int triA, int tiles)
{
    constexpr int NW = GEMV_THREADS / 64;  // wavefronts: rows per block (k contiguous) or slices of k
    __shared__ T red[NW][64][GEMV_N];
    const int64_t b = blockIdx.x / tiles;
    const int tile = (int)(blockIdx.x % tiles);
    const T *Ap = A.item(b);
    const T *Bp = B.item(b);
    T *Cp = C.item(b);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    T acc[GEMV_N];
#pragma unroll
    for (int j = 0; j < GEMV_N; ++j)
        acc[j] = T(0);
    if (A.cs == 1) {
        const int i = tile * NW + w;
        if (i < M) {
            const int kb = triA == 2 ? i : 0, ke = triA == 1 ? min(K, i + 1) : K;
            const T *ar = Ap + (int64_t)i * A.rs;
            for (int k = kb + lane; k < ke; k += 64) {
                const T a = ar[k];
#pragma unroll
                for (int j = 0; j < GEMV_N; ++j)
                    if (j < N)
                        acc[j] = fma(a, Bp[(int64_t)k * B.rs + (int64_t)j * B.cs], acc[j]);
            }
#pragma unroll
            for (int j = 0; j < GEMV_N; ++j) {
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1)
                    acc[j] += __shfl_xor(acc[j], off, WAVE);
                if (lane == 0 && j < N) {
                    T *c = Cp + (int64_t)i * C.rs + (int64_t)j * C.cs;
                    const T upd = alpha * acc[j];
                    *c = (beta == T(0)) ? upd : fma(beta, *c, upd);
                }
            }
        }
        return;
    }
    const int i = tile * 64 + lane;
    if (i < M) {
        const int kb = triA == 2 ? i : 0, ke = triA == 1 ? min(K, i + 1) : K;
        for (int k = w; k < K; k += NW) {
            if (k < kb || k >= ke)
                continue;
            const T a = Ap[(int64_t)i * A.rs + (int64_t)k * A.cs];
#pragma unroll
            for (int j = 0; j < GEMV_N; ++j)
                if (j < N)
                    acc[j] = fma(a, Bp[(int64_t)k * B.rs + (int64_t)j * B.cs], acc[j]);
        }
    }
#pragma unroll
    for (int j = 0; j < GEMV_N; ++j)
        red[w][lane][j] = acc[j];
    __syncthreads();
    if (w == 0 && i < M) {
#pragma unroll
        for (int j = 0; j < GEMV_N; ++j)
            if (j < N) {
                T sum = T(0);
#pragma unroll
                for (int q = 0; q < NW; ++q)
                    sum += red[q][lane][j];
                T *c = Cp + (int64_t)i * C.rs + (int64_t)j * C.cs;
                const T upd = alpha * sum;
                *c = (beta == T(0)) ? upd : fma(beta, *c, upd);
            }
    }
}

template <typename T>
static la_status launch_gemv(View<const T> A, View<const T> B, View<T> C, int64_t batch, int M, int N, int K, T alpha,
                             T beta, int triA, hipStream_t st)
{
    const int tiles = (A.cs == 1) ? (M + GEMV_THREADS / 64 - 1) / (GEMV_THREADS / 64) : (M + 63) / 64;
    const int64_t blocks = (int64_t)tiles * batch;
    if (blocks > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    LA_LAUNCH((k_gemv<T>), dim3((unsigned)blocks), dim3(GEMV_THREADS), 0, st, A, B, C, batch, M, N, K, alpha, beta, triA,
                       tiles);
    return launch_check("gemv");
}

// ---------------------------------------------------------------------------------------
// Split along K for products with few output tiles and a long K (A^T A of a tall A, the syrk of a
// wide panel): the K range is cut into slices that run as extra batch items into a buffer of
// partial results, which a second kernel sums in a fixed order (no atomics: results are
// reproducible) while applying alpha, beta and the output mask.  The buffer comes out of the
// calling operator's workspace (at most SPLITK_MAX_BYTES of it).
// ---------------------------------------------------------------------------------------
constexpr size_t SPLITK_MAX_BYTES = (size_t)64 << 20;

template <typename T>
__global__ __launch_bounds__(256) void k_splitk_reduce(const T *partial, View<T> C, int64_t batch, int M, int N,
                                                       int splits, T alpha, T beta, GemmOpts o)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t mn = (int64_t)M * N;
    if (e >= batch * mn)
        return;
    const int64_t b = e / mn;
    const int64_t r = e - b * mn;
    const int i = (int)(r / N), j = (int)(r - (int64_t)i * N);
    if ((o.maskC == 1 && i < j) || (o.maskC == 2 && i > j))
        return;
    const T *p = partial + b * splits * mn + r;
    T s = T(0);
    for (int q = 0; q < splits; ++q)
        s += p[q * mn];
    store_c<T>(C.item(b), C.rs, C.cs, i, j, M, N, s, alpha, beta, o);
}

template <typename T>
static bool aligned16(const View<const T> &V, int64_t lead)
{
    constexpr int VW = Mfma<T>::VW;
    return (reinterpret_cast<uintptr_t>(V.p) & 15) == 0 && (lead % VW) == 0 && (V.bs % VW) == 0 && (V.bs2 % VW) == 0;
}

static inline int pick_order(const GemmOpts &o, int tiles_m, int tiles_n)
{
    if (o.maskC == 0 && o.triA == 0 && o.triB != 0)
        return 4;  // work depends on the column only
    if (o.symsum)
        return 1;
    if (tiles_m != tiles_n)
        return 0;
    if (o.maskC == 1 && o.triA == 1 && o.triB == 1 && tiles_m >= 16)
        return 5;
    if (o.maskC == 1 || o.maskC == 3)
        return 1;
    if (o.maskC == 2)
        return 2;
    return o.shells ? 3 : 0;
}

template <typename T, int BM, int BN, int BK, int NBUF>
static void launch_fast(bool akf, bool bkf, View<const T> A, View<const T> B, View<T> C, int64_t batch, int M, int N,
                        int K, T alpha, T beta, GemmOpts o, hipStream_t st)
{
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    o.order = pick_order(o, tiles_m, tiles_n);
    const int64_t per = tile_count(o.order, tiles_m, tiles_n);
    o.xcd_batch = (batch >= 8 && per > 1) ? 1 : 0;
    const int64_t wgs = o.xcd_batch ? 8 * ((batch + 7) / 8) * per : per * batch;
    const dim3 grid((unsigned)wgs), block(256);
#define LA_GO(AK, BKF_)                                                                                              \
    LA_LAUNCH((k_gemm_fast<T, BM, BN, BK, NBUF, AK, BKF_>), grid, block, 0, st, A, B, C, batch, M, N, K,    \
                       alpha, beta, o, tiles_m, tiles_n)
    if constexpr (BM <= 64) {  // the symmetric sum exists for the small tiles only (launch_gemm picks them)
        if (o.symsum) {         // and its operands have mirrored strides, so akf == bkf
            if (akf)
                LA_LAUNCH((k_gemm_fast<T, BM, BN, BK, NBUF, true, true, true>), grid, block, 0, st, A, B, C, batch, M, N,
                          K, alpha, beta, o, tiles_m, tiles_n);
            else
                LA_LAUNCH((k_gemm_fast<T, BM, BN, BK, NBUF, false, false, true>), grid, block, 0, st, A, B, C, batch, M,
                          N, K, alpha, beta, o, tiles_m, tiles_n);
            return;
        }
    }
    if (akf && bkf)
        LA_GO(true, true);
    else if (akf && !bkf)
        LA_GO(true, false);
    else if (!akf && bkf)
        LA_GO(false, true);
    else
        LA_GO(false, false);
#undef LA_GO
}

static inline int flip_tri(int t) { return t == 1 ? 2 : (t == 2 ? 1 : 0); }

template <typename T>
la_status launch_gemm(View<const T> A, View<const T> B, View<T> C, int64_t batch, int M, int N, int K, T alpha, T beta,
                      GemmOpts o, hipStream_t st)
{
    if (batch <= 0 || M <= 0 || N <= 0)
        return LA_OK;
    if (o.symsum) {
        if (M != N || A.rs != B.cs || A.cs != B.rs || A.bs != B.bs || A.nb2 != 1 || B.nb2 != 1 || C.nb2 != 1)
            return LA_ERR_UNSUPPORTED;
        o.maskC = 0;
        o.halfDiag = 0;
        if (C.cs != 1 && C.rs == 1)  // the result is symmetric: its transpose is the same matrix
            C = C.t();
    }
    // a few vectors on either side: one pass over the big operand
    if (!o.maskC && !o.halfDiag && !o.min_tile64 && !o.symsum && K > 0) {
        if (N <= GEMV_N && o.triB == 0)
            return launch_gemv<T>(A, B, C, batch, M, N, K, alpha, beta, o.triA, st);
        if (M <= GEMV_N && o.triA == 0)  // C^T = B^T A^T
            return launch_gemv<T>(B.t(), A.t(), C.t(), batch, N, M, K, alpha, beta, flip_tri(o.triB), st);
    }
    // Keep the stores of C along its contiguous direction: if C is stored with i contiguous,
    // compute C^T = B^T A^T instead (a pure re-labelling of the views).
    if (C.cs != 1 && C.rs == 1 && !o.symsum) {
        GemmOpts t;
        t.triA = flip_tri(o.triB);
        t.triB = flip_tri(o.triA);
        t.maskC = flip_tri(o.maskC);
        t.halfDiag = o.halfDiag;
        t.reverse = o.reverse;
        t.shells = o.shells;
        t.min_tile64 = o.min_tile64;
        return launch_gemm<T>(B.t(), A.t(), C.t(), batch, N, M, K, alpha, beta, t, st);
    }
    constexpr int VW = Mfma<T>::VW;
    const bool akf = (A.cs == 1), bkf = (B.rs == 1);
    const bool a_ok = akf ? aligned16<T>(A, A.rs) : (A.rs == 1 && aligned16<T>(A, A.cs) && M % VW == 0);
    const bool b_ok = bkf ? aligned16<T>(B, B.cs) : (B.cs == 1 && aligned16<T>(B, B.rs) && N % VW == 0);
    if (K > 0 && K % 16 == 0 && a_ok && b_ok) {
        const int64_t t64 = (int64_t)((M + 63) / 64) * ((N + 63) / 64) * batch;
        if (t64 > 0x1fffffffll)  // (quarter tiles and the batched mapping round the grid up)
            return LA_ERR_UNSUPPORTED;
        // Workgroups a launch would have with each tile size (empty tiles of triangular outputs
        // left out).
        auto wgs = [&](int e) {
            const int tm = (M + e - 1) / e, tn = (N + e - 1) / e;
            return tile_count(pick_order(o, tm, tn), tm, tn) * batch;
        };
        const int64_t wg128 = wgs(128), wg64 = wgs(64);
        const bool k64 = (K % 64 == 0);
        if (!o.triA && !o.triB && !o.min_tile64 && !o.ksplit && wg64 <= 128 && K >= 2048 && A.nb2 == 1 && B.nb2 == 1 &&
            C.nb2 == 1) {
            int splits = (int)std::min<int64_t>(512 / wg64, K / 256);
            const int Kc = ((K / 16 + splits - 1) / splits) * 16;
            splits = (K + Kc - 1) / Kc;
            const size_t bytes = (size_t)batch * splits * M * N * sizeof(T);
            if (splits >= 2 && bytes <= SPLITK_MAX_BYTES) {
                ArenaFrame frame;
                void *buf = nullptr;
                LA_TRY(arena_take(bytes, &buf));
                const int64_t mn = (int64_t)M * N;
                View<const T> As = A.level2((int64_t)Kc * A.cs, splits), Bs = B.level2((int64_t)Kc * B.rs, splits);
                View<T> Ps{(T *)buf, (int64_t)splits * mn, N, 1, mn, splits};
                GemmOpts ps;
                ps.maskC = o.maskC;  // tiles beyond the kept triangle are not computed (nor read back)
                ps.ksplit = splits;
                ps.ktotal = K;
                launch_fast<T, 64, 64, 16, 2>(akf, bkf, As, Bs, Ps, batch * splits, M, N, Kc, T(1), T(0), ps, st);
                LA_TRY(launch_check("gemm_splitk"));
                const int64_t total = batch * mn;
                LA_LAUNCH((k_splitk_reduce<T>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                                   (const T *)buf, C, batch, M, N, splits, alpha, beta, o);
                return launch_check("splitk_reduce");
            }
        }
        int e;
        if (o.triA | o.triB) {
            // Triangular operands make the K range, hence the time, of a tile vary along the tile
            // list (heaviest first): the 512 workgroup slots only fill evenly if there are several
            // rounds of tiles, so take the largest tile that still gives 1024 workgroups.
            e = wg128 >= 1024 ? 128 : ((wg64 >= 1024 || !k64 || o.min_tile64) ? 64 : 32);
            if (o.symsum && e == 128)
                e = 64;
        } else {
            // Equal tiles: big tiles once they fill most of the chip, quarter tiles while 64 x 64 tiles
            // would fill the 512 workgroup slots less than twice -- with so few rounds the last one runs
            // part empty (32 x 384 x 384 lower triangle, K = 128: 672 tiles of 64, 38 -> 30 us; potrf of
            // 32 x 512 x 512 0.245 -> 0.231 ms, of 4 x 2048 x 2048 1.14 -> 1.10, 8192 x 8192 with 512
            // vectors trsm 1.19 -> 1.12 ms).
            const int64_t t128 = o.maskC ? wg128 : (int64_t)((M + 127) / 128) * ((N + 127) / 128) * batch;
            const bool big = o.maskC ? (M >= 2048 && N >= 2048) : (M >= 128 && N >= 128);
            e = (t128 >= 192 && big) ? 128 : ((wg64 < 1024 && k64 && !o.min_tile64) ? 32 : 64);
        }
        if (e >= 64 && o.maskC == 1 && !o.triA && !o.triB && !o.halfDiag && !o.shells && !o.min_tile64 && M == N &&
            M % e == 0 && A.nb2 == 1 && B.nb2 == 1 && C.nb2 == 1) {
            // Lower triangle in e x e tiles: T (T + 1) / 2 of them.  When that is a few tiles more than
            // whole rounds of the 512 workgroup slots (T = 32: 528), the last round runs nearly empty.
            // The T diagonal tiles only need their lower halves anyway: take the T (T - 1) / 2 tiles
            // below the diagonal in one launch (whole tiles, no masking) and the diagonal blocks as a
            // batch of T small lower-triangle products.
            const int64_t Tt = M / e, per = Tt * (Tt + 1) / 2, spill = per % 512, below = (per - Tt) % 512;
            if (batch == 1 && per > 512 && spill > 0 && spill <= 64 && (below == 0 || below > 256)) {
                GemmOpts lo = o;
                lo.maskC = 3;  // tiles with tn <= tm of the view that starts e rows down, nothing masked inside
                View<const T> A1 = A.sub(e, 0);
                View<T> C1 = C.sub(e, 0);
                if (e == 128)
                    launch_fast<T, 128, 128, 16, 2>(akf, bkf, A1, B, C1, batch, M - e, N - e, K, alpha, beta, lo, st);
                else if (k64)
                    launch_fast<T, 64, 64, 64, 1>(akf, bkf, A1, B, C1, batch, M - e, N - e, K, alpha, beta, lo, st);
                else
                    launch_fast<T, 64, 64, 16, 2>(akf, bkf, A1, B, C1, batch, M - e, N - e, K, alpha, beta, lo, st);
                LA_TRY(launch_check("gemm_fast"));
                return launch_gemm<T>(A.level2((int64_t)e * A.rs, (int)Tt), B.level2((int64_t)e * B.cs, (int)Tt),
                                      C.level2((int64_t)e * (C.rs + C.cs), (int)Tt), batch * Tt, e, e, K, alpha, beta, o, st);
            }
        }
        if (e == 128)
            launch_fast<T, 128, 128, 16, 2>(akf, bkf, A, B, C, batch, M, N, K, alpha, beta, o, st);
        else if (e == 32)
            launch_fast<T, 32, 32, 64, 1>(akf, bkf, A, B, C, batch, M, N, K, alpha, beta, o, st);
        else if (k64)  // small grids are latency bound: fewer, fatter K slabs
            launch_fast<T, 64, 64, 64, 1>(akf, bkf, A, B, C, batch, M, N, K, alpha, beta, o, st);
        else
            launch_fast<T, 64, 64, 16, 2>(akf, bkf, A, B, C, batch, M, N, K, alpha, beta, o, st);
        return launch_check("gemm_fast");
    }
    constexpr int BM = 64, BN = 64, BK = 16;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    o.order = pick_order(o, tiles_m, tiles_n);
    const int64_t blocks = tile_count(o.order, tiles_m, tiles_n) * batch;
    if (blocks > 0x7fffffffll)
        return LA_ERR_UNSUPPORTED;
    LA_LAUNCH((k_gemm<T, BM, BN, BK>), dim3((unsigned)blocks), dim3(256), 0, st, A, B, C, batch, M, N, K,
                       alpha, beta, o, tiles_m, tiles_n);
    return launch_check("gemm");
}

template la_status launch_gemm<float>(View<const float>, View<const float>, View<float>, int64_t, int, int, int, float,
                                      float, GemmOpts, hipStream_t);
template la_status launch_gemm<double>(View<const double>, View<const double>, View<double>, int64_t, int, int, int,
                                       double, double, GemmOpts, hipStream_t);

}  // namespace la
