// Triangular solve against one factor of middling size (128 < n <= 512) as one
// launch (section 4.2 of arXiv 1710.08717, operator trsm: X = alpha Lam^-1 B).
//
// One workgroup takes one batch item and one slab of 16 vectors and runs the substitution over
// tile rows of 16:   X_j = Lam_jj^-1 (B_j - sum_{k<j} Lam_jk X_k).
// Wavefront w of eight owns the tile rows i = w, w + 8, ...: their right-hand sides stay in its matrix-core
// accumulators from the first load to the final store, and the tiles Lam_ij of "its" rows come
// straight from memory into operand registers, a few steps ahead of their use.  The only shared
// state is the solved tile X_j, published through a double-buffered 16 x 16 area of LDS: after the
// barrier of step j every wavefront subtracts Lam_ij X_j from its rows, and the owner of row j + 1
// multiplies by the inverse of its diagonal tile right after its first product, so the sequential
// chain per step is   barrier -> X_j from LDS -> 4 + 4 matrix-core instructions -> X_{j+1} to LDS.
// The inverses of the 16 x 16 diagonal tiles are formed in registers at the start (row per lane,
// DPP broadcasts) and kept in LDS.
//
// The backward substitution (Lam^T X = B) is the same kernel on views with negated strides: with
// both index ranges reversed Lam^T is lower triangular again.
#include "common.hpp"
#include "leaf_dpp.hpp"

#ifndef TS_STAMP
#define TS_STAMP(i)
#endif

namespace la {

constexpr int TS_WAVES = 8;  // 256 registers per lane: room for the tiles in flight
constexpr int TS_THREADS = TS_WAVES * WAVE;

template <typename T>
struct TrsmStream {
    static constexpr int PS = LT + 1;        // row stride of an inverse tile in LDS (elements)
    static constexpr int IT = LT * PS;       // elements of an inverse tile
    static size_t lds_bytes(int K) { return sizeof(T) * ((size_t)K * IT + 2 * LT * LT); }
};

// R: tile rows per wavefront (n <= 128 R), D: steps the loads of Lam run ahead, VEC: Lam is read with
// 16-byte loads along its rows
template <typename T, int R, int D, bool VEC>
__global__ __launch_bounds__(TS_THREADS) void k_trsm_stream(View<const T> Lam, View<const T> Bin, View<T> X, int n,
                                                            int m, T alpha)
{
    using C = TrsmStream<T>;
    using acc_t = typename Mfma<T>::acc_t;
    extern __shared__ __align__(16) unsigned char ts_lds[];
    T *inv = reinterpret_cast<T *>(ts_lds);  // K tiles of Lam_ii^-1, rows padded
    const int K = (n + LT - 1) / LT;
    T *xbuf = inv + (size_t)K * C::IT;       // two 16 x 16 tiles, X_j in buffer j % 2, element (k, c) at 16 k + c

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int u = lane & 15, q = lane >> 4;
    const int c0 = blockIdx.x * LT;
    const int64_t b = blockIdx.y;
    const T *Lp = Lam.p + b * Lam.bs;
    const T *Bp = Bin.p + b * Bin.bs;
    T *Xp = X.p + b * X.bs;
    const bool col_ok = c0 + u < m;
    const int cu = col_ok ? c0 + u : m - 1;
    // element offsets inside one item fit 32 bits (checked by the launcher): scalar base + 32-bit lane offset
    const int lrs = (int)Lam.rs, lcs = (int)Lam.cs, brs = (int)Bin.rs, bcs = (int)Bin.cs, xrs = (int)X.rs, xcs = (int)X.cs;

    TS_STAMP(0);
    // ---- set-up: right-hand sides into the accumulators, inverses of the diagonal tiles into LDS ----
    acc_t acc[R];
    static_for<0, R>([&](auto H) {
        constexpr int h = decltype(H)::value;
        const int i = wave + TS_WAVES * h;
        // addresses are clamped into the operand and the value masked afterwards: no per-lane branches
        acc[h] = acc_t{0, 0, 0, 0};
        if (i < K) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int r = i * LT + Mfma<T>::row(lane, v);
                const T x = Bp[(r < n ? r : n - 1) * brs + cu * bcs];
                acc[h][v] = (r < n && col_ok) ? alpha * x : T(0);
            }
        }
    });
    {
        // the diagonal tiles of this wavefront's rows: all loads in flight together (lane (u, q) takes the
        // entries (4 q + v, u), a row of the tile per 16 lanes), parked in the LDS area of the inverse
        T raw[R][4];
        static_for<0, R>([&](auto H) {
            constexpr int h = decltype(H)::value;
            const int i = wave + TS_WAVES * h;
            if (i < K) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    // row and column clamped into the triangle of the operand that may be read (with a ragged
                    // last tile the rows past n would otherwise reach past the matrix; with negated strides,
                    // before it)
                    const int tr = 4 * q + v;
                    const int rr = i * LT + tr, rc = rr < n ? rr : n - 1;
                    const int cc = i * LT + (u <= tr ? u : tr);
                    raw[h][v] = Lp[rc * lrs + (cc < rc ? cc : rc) * lcs];
                }
            }
        });
        static_for<0, R>([&](auto H) {
            constexpr int h = decltype(H)::value;
            const int i = wave + TS_WAVES * h;
            if (i < K) {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    inv[(size_t)i * C::IT + (4 * q + v) * C::PS + u] = raw[h][v];
            }
        });
    }
    __syncthreads();
    TS_STAMP(1);
#pragma unroll 1
    for (int i = wave; i < K; i += TS_WAVES) {  // lane (u, q): row u of the tile, columns 4 j + q of its inverse
        const int r = i * LT + u;
        T *tile = inv + (size_t)i * C::IT + u * C::PS;
        T a[LT], dr = T(1);
#pragma unroll
        for (int c = 0; c < LT; ++c) {
            const T x = tile[c];
            a[c] = (r < n && c <= u) ? x : ((c == u) ? T(1) : T(0));  // rows past n: identity
        }
#pragma unroll
        for (int c = 0; c < LT; ++c)
            dr = (c == u) ? a[c] : dr;
        T x[4];
        diag_invert<T>(a, dr, x, u, q);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            tile[4 * j + q] = (4 * j + q <= u) ? x[j] : T(0);  // every lane has read its row by now
    }

    // tiles Lam(i, j) of this wavefront's rows as the first operand: lane (u, q) supplies element
    // (u, 4 q + s) for instruction s
    // Every step issues the same number of loads, needed or not (a tile on or above the diagonal is
    // replaced by one address at the start of the item and never used): with a fixed count the wait
    // for the tile of this step leaves the loads of the later steps in flight.
    T ring[D][R][4];
    auto fetch = [&](auto Dd, int j) {
        constexpr int d = decltype(Dd)::value;
        static_for<0, R>([&](auto H) {
            constexpr int h = decltype(H)::value;
            const int i = wave + TS_WAVES * h;
            const bool live = (i > j) && (i < K);  // the same for the whole wavefront
            const int r = i * LT + u, rc = r < n ? r : n - 1;
            if constexpr (VEC) {
                // Lam has unit column stride and 16-byte aligned rows: the four entries are one or two
                // 16-byte loads (a live tile lies below the diagonal tile, so nothing needs clamping); a tile
                // that is not needed reads the first entries of the item, one cache line for all lanes
                using V = typename Mfma<T>::vec_t;
                const int off = live ? rc * lrs + j * LT + 4 * q : 0;
                if constexpr (sizeof(T) == 8) {
                    const V lo = *reinterpret_cast<const V *>(Lp + off), hi = *reinterpret_cast<const V *>(Lp + off + 2);
                    ring[d][h][0] = lo.x; ring[d][h][1] = lo.y; ring[d][h][2] = hi.x; ring[d][h][3] = hi.y;
                } else {
                    const V w = *reinterpret_cast<const V *>(Lp + off);
                    ring[d][h][0] = w.x; ring[d][h][1] = w.y; ring[d][h][2] = w.z; ring[d][h][3] = w.w;
                }
            } else {
                // (a live tile lies below the diagonal tile: its columns need no clamping)
                const int off = live ? rc * lrs + (j * LT + 4 * q) * lcs : 0, step = live ? lcs : 0;
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    ring[d][h][s] = Lp[off + s * step];
            }
        });
    };
    static_for<0, D>([&](auto Dd) { fetch(Dd, decltype(Dd)::value); });

    // rows of the inverse of diagonal tile j as the first operand: the contraction index instruction s
    // sees in lane group q is the row that accumulator register s holds there
    auto inv_rows = [&](int j, T (&av)[4]) {
        const T *ij = inv + (size_t)j * C::IT + u * C::PS;
#pragma unroll
        for (int s = 0; s < 4; ++s)
            av[s] = ij[Mfma<T>::row(q * 16, s)];
    };
    // solve tile row j (held in slot h of its owner): X_j = inv_j acc; publish and store
    auto solve = [&](auto H, int j, const T (&av)[4]) {
        constexpr int h = decltype(H)::value;
        acc_t xa = {0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < 4; ++s)
            xa = Mfma<T>::run(av[s], acc[h][s], xa);  // the accumulator is the second operand as it stands
        T *xb = xbuf + (j & 1) * LT * LT;
#pragma unroll
        for (int v = 0; v < 4; ++v)
            xb[Mfma<T>::row(lane, v) * LT + u] = xa[v];
        acc[h] = xa;  // the row is done: its accumulator carries the solution to the stores at the end
    };

    TS_STAMP(2);
    __syncthreads();  // the inverses are in LDS
    TS_STAMP(3);
    if (wave == 0) {
        T av[4];
        inv_rows(0, av);
        solve(std::integral_constant<int, 0>{}, 0, av);
    }

    for (int j0 = 0; j0 < K; j0 += D) {
        static_for<0, D>([&](auto Dd) {
            constexpr int d = decltype(Dd)::value;
            const int j = j0 + d;
            if (j < K) {  // the same for the whole workgroup
                __syncthreads();  // X_j is in its buffer; buffer (j + 1) % 2 is no longer read
                TS_STAMP(4 + j);
                // the wavefront that owns row j + 1 carries the sequential chain of this step: its
                // matrix-core instructions go ahead of those of the wavefront it shares a SIMD with
                const bool chain = (j + 1 < K) && ((j + 1) % TS_WAVES == wave);
                T av[4] = {T(0), T(0), T(0), T(0)};
                if (chain) {
                    __builtin_amdgcn_s_setprio(3);
                    inv_rows(j + 1, av);
                }
                const T *xb = xbuf + (j & 1) * LT * LT;
                T bv[4];
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    bv[s] = xb[(4 * q + s) * LT + u];
                static_for<0, R>([&](auto H) {
                    constexpr int h = decltype(H)::value;
                    const int i = wave + TS_WAVES * h;
                    if (i > j && i < K) {
                        const bool row_ok = i * LT + u < n;
#pragma unroll
                        for (int s = 0; s < 4; ++s)
                            acc[h] = Mfma<T>::run(row_ok ? -ring[d][h][s] : T(0), bv[s], acc[h]);
                        if (i == j + 1) {
                            solve(H, j + 1, av);
                            __builtin_amdgcn_s_setprio(0);
                        }
                    }
                });
                fetch(Dd, j + D);
            }
        });
    }

    TS_STAMP(60);
    // (stores inside the loop would make the number of outstanding memory operations vary from step to step)
    static_for<0, R>([&](auto H) {
        constexpr int h = decltype(H)::value;
        const int i = wave + TS_WAVES * h;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int r = i * LT + Mfma<T>::row(lane, v);
            if (i < K && r < n && col_ok)
                Xp[r * xrs + (c0 + u) * xcs] = acc[h][v];
        }
    });
}

template <typename T>
bool trsm_stream_takes(int64_t batch, int n, int m)
{
    // Measured against the blocked path (explicit inverses of the diagonal blocks and products), fp64,
    // us, blocked / streamed: 32 x 512 with 64 vectors 89 / 51, 1 x 512 with 16: 62 / 45, 256 x 512 with
    // 16: 359 / 75, 256 x 512 with 64: 434 / 239, 4096 x 256 with 16: 2223 / 279, 32 x 256 with 1024:
    // 106 / 100, 16 x 512 with 1024: 168 / 193.  The blocked path only gets ahead with many vectors per
    // item once the slabs no longer fit the chip twice.
    const int64_t slabs = (m + LT - 1) / LT;
    return n > 128 && n <= 512 && (m <= 512 || batch * slabs <= 512) && batch <= 65535;
}
template bool trsm_stream_takes<float>(int64_t, int, int);
template bool trsm_stream_takes<double>(int64_t, int, int);

template <typename T>
la_status launch_trsm_stream(View<const T> Lam, View<const T> Xin, View<T> X, int64_t batch, int n, int m, T alpha,
                             bool fwd, hipStream_t st)
{
    if (batch <= 0 || n <= 0 || m <= 0)
        return LA_OK;
    if (n > 512 || batch > 65535 || Lam.nb2 != 1 || Xin.nb2 != 1 || X.nb2 != 1)
        return LA_ERR_UNSUPPORTED;
    {  // the kernel addresses one item with 32-bit element offsets
        auto span = [](int64_t rs, int64_t cs, int rows, int cols) {
            return (rs < 0 ? -rs : rs) * rows + (cs < 0 ? -cs : cs) * cols;
        };
        const int64_t lim = 0x7fffffffll;
        if (span(Lam.rs, Lam.cs, n, n) > lim || span(Xin.rs, Xin.cs, n, m) > lim || span(X.rs, X.cs, n, m) > lim)
            return LA_ERR_UNSUPPORTED;
    }
    if (!fwd) {  // Lam^T with both index ranges reversed is lower triangular: M(a, b) = Lam(n-1-b, n-1-a)
        Lam = View<const T>{Lam.p + (int64_t)(n - 1) * (Lam.rs + Lam.cs), Lam.bs, -Lam.cs, -Lam.rs};
        Xin = View<const T>{Xin.p + (int64_t)(n - 1) * Xin.rs, Xin.bs, -Xin.rs, Xin.cs};
        X = View<T>{X.p + (int64_t)(n - 1) * X.rs, X.bs, -X.rs, X.cs};
    }
    const int K = (n + LT - 1) / LT;
    const size_t lds = TrsmStream<T>::lds_bytes(K);
    if (dry_run())
        return LA_OK;
    constexpr int D = sizeof(T) == 8 ? 3 : 4;
    constexpr int64_t EPV = 16 / sizeof(T);  // elements per 16-byte load
    const bool vec = Lam.cs == 1 && Lam.rs % EPV == 0 && Lam.bs % EPV == 0 && (reinterpret_cast<uintptr_t>(Lam.p) & 15) == 0;
    const dim3 grid((unsigned)((m + LT - 1) / LT), (unsigned)batch);
    const int R = K <= 2 * TS_WAVES ? 2 : (K <= 3 * TS_WAVES ? 3 : 4);
    static bool configured[64] = {};
    int dev = 0;
    LA_HIP(hipGetDevice(&dev));
    const bool first = dev >= 0 && dev < 64 && !configured[dev];
    la_status status = LA_OK;
    auto go = [&](auto kernel) {
        if (first && hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)TrsmStream<T>::lds_bytes(32)) != hipSuccess)
            status = LA_ERR_RUNTIME;
    };
    if (first) {  // all six forms once per device
        go(&k_trsm_stream<T, 2, D, false>);
        go(&k_trsm_stream<T, 3, D, false>);
        go(&k_trsm_stream<T, 4, D, false>);
        go(&k_trsm_stream<T, 2, D, true>);
        go(&k_trsm_stream<T, 3, D, true>);
        go(&k_trsm_stream<T, 4, D, true>);
        if (status != LA_OK)
            return status;
        configured[dev] = true;
    }
#define TS_GO(RR, VV) LA_LAUNCH((k_trsm_stream<T, RR, D, VV>), grid, dim3(TS_THREADS), lds, st, Lam, Xin, X, n, m, alpha)
    if (vec) {
        if (R == 2) TS_GO(2, true); else if (R == 3) TS_GO(3, true); else TS_GO(4, true);
    } else {
        if (R == 2) TS_GO(2, false); else if (R == 3) TS_GO(3, false); else TS_GO(4, false);
    }
#undef TS_GO
    return launch_check("trsm_stream");
}

template la_status launch_trsm_stream<float>(View<const float>, View<const float>, View<float>, int64_t, int, int, float,
                                             bool, hipStream_t);
template la_status launch_trsm_stream<double>(View<const double>, View<const double>, View<double>, int64_t, int, int,
                                              double, bool, hipStream_t);

}  // namespace la
