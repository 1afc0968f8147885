// Operators on many small matrices with 16 < n <= 32 in 16 lanes per matrix: lane i holds the rows i and
// i + 16 (row slot h = 0, 1) of every operand, so that all broadcasts are DPP row broadcasts fused into
// the multiply-adds (as in the kernels of tiny.hip with two rows per lane); four matrices per
// wavefront.  Row j = 16 jh + jl lives in slot jh of lane jl.  syrk and the outer products of the
// trmm / trsm backward rules, the syrk backward rule, gemm2 (section 4.2 of arXiv 1710.08717 and its
// appendix).  Operands that are not square travel as flat memory images through LDS; the long dimension
// is taken in passes of CH columns to bound the registers.
#include "tiny_stage.hpp"

namespace la {

constexpr int ROWS_G = 16, ROWS_MPW = WAVE / ROWS_G;
constexpr int ROWS_KMAX = 32;  // inner dimension (syrk, outer products, syrk backward), at most
constexpr int ROWS_CH = 8;     // columns per pass

// elements of the padded LDS image of ROWS_MPW items of `per` elements, a multiple of 16 bytes
static inline __host__ __device__ int rows_image_elems(int per) { return (ROWS_MPW * per * 17 / 16 + 4 + 3) / 4 * 4; }

// ---------------------------------------------------------------------------------
// C = alpha U V^T for n x k operands U, V (V == U: syrk), 16 < n <= N, k <= 32.  tri = 0 writes the whole
// square, 1 / 2 keep the lower / upper triangle and write zeros to the other one.  In the syrk case lane
// pairs form the same products in the same order, so the result is exactly symmetric.
// ---------------------------------------------------------------------------------
template <typename T, int N, bool TWO>
__global__ __launch_bounds__(WAVE) void k_syrk_rows(const T *Uin, const T *Vin, View<T> C, int64_t batch, int n, int k,
                                                    int img_tr, int tri, T alpha)
{
    constexpr int G = ROWS_G, MPW = ROWS_MPW, CH = ROWS_CH;
    constexpr int IMG = MPW * N * ROWS_KMAX;
    using S = Stage<T, N, MPW>;
    extern __shared__ __align__(16) unsigned char tiny_lds[];
    // the result's stage overlays the images: they are dead by the time it is written
    T *sm = reinterpret_cast<T *>(tiny_lds), *img = sm, *img2 = img + rows_image_elems(n * k);
    const int lane = threadIdx.x;
    const int q = lane / G, i = lane % G;
    const int64_t b0 = (int64_t)blockIdx.x * MPW;
    const int cnt = (int)((batch - b0) < MPW ? (batch - b0) : MPW);
    const int nk = n * k;
    image_load<T, IMG, MPW>(img, Uin, b0, cnt, nk, lane);
    if constexpr (TWO)
        image_load<T, IMG, MPW>(img2, Vin, b0, cnt, nk, lane);
    __syncthreads();

    const bool live0 = (i < n) && (q < cnt), live1 = (i + G < n) && (q < cnt);
    const int e0 = q * nk + (img_tr ? i : i * k), e1 = q * nk + (img_tr ? i + G : (i + G) * k), estep = img_tr ? n : 1;
    T o0[N], o1[N];
#pragma unroll
    for (int j = 0; j < N; ++j) {
        o0[j] = T(0);
        o1[j] = T(0);
    }
    static_for<0, ROWS_KMAX / CH>([&](auto CB) {
        constexpr int c0 = CH * decltype(CB)::value;
        if (c0 < k) {  // the same for all lanes
            T a0[CH], a1[CH], v0[TWO ? CH : 1], v1[TWO ? CH : 1];
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                a0[u] = (live0 && c0 + u < k) ? img[img_idx(e0 + (c0 + u) * estep)] : T(0);
                a1[u] = (live1 && c0 + u < k) ? img[img_idx(e1 + (c0 + u) * estep)] : T(0);
            }
            if constexpr (TWO) {
#pragma unroll
                for (int u = 0; u < CH; ++u) {
                    v0[u] = (live0 && c0 + u < k) ? img2[img_idx(e0 + (c0 + u) * estep)] : T(0);
                    v1[u] = (live1 && c0 + u < k) ? img2[img_idx(e1 + (c0 + u) * estep)] : T(0);
                }
                dpp_settle<G>(v0);
                dpp_settle<G>(v1);
            } else {
                dpp_settle<G>(a0);
                dpp_settle<G>(a1);
            }
            static_for<0, N>([&](auto Jj) {
                constexpr int j = decltype(Jj)::value;
                constexpr int jl = j % G, jh = j / G;
                if (j < n) {
                    static_for<0, CH>([&](auto U) {
                        constexpr int u = decltype(U)::value;
                        // c_rj += u_rc v_jc, v_jc from slot jh of lane jl
                        // (the broadcast operand is named register by register: a copy made for the asm
                        // statement would be written right before its DPP read)
                        if constexpr (TWO && jh == 0) {
                            fma_bcast<G, jl>(o0[j], v0[u], a0[u], false);
                            fma_bcast<G, jl>(o1[j], v0[u], a1[u], false);
                        } else if constexpr (TWO) {
                            fma_bcast<G, jl>(o0[j], v1[u], a0[u], false);
                            fma_bcast<G, jl>(o1[j], v1[u], a1[u], false);
                        } else if constexpr (jh == 0) {
                            fma_bcast<G, jl>(o0[j], a0[u], a0[u], false);
                            fma_bcast<G, jl>(o1[j], a0[u], a1[u], false);
                        } else {
                            fma_bcast<G, jl>(o0[j], a1[u], a0[u], false);
                            fma_bcast<G, jl>(o1[j], a1[u], a1[u], false);
                        }
                    });
                }
            });
        }
    });
#pragma unroll
    for (int j = 0; j < N; ++j) {
        const bool keep0 = tri == 0 || (tri == 1 ? j <= i : j >= i);
        const bool keep1 = tri == 0 || (tri == 1 ? j <= i + G : j >= i + G);
        o0[j] = keep0 ? o0[j] * alpha : T(0);
        o1[j] = keep1 ? o1[j] * alpha : T(0);
    }
    __syncthreads();
    write_row<T, N>(sm + q * S::MS, i, o0);
    if (N == 2 * G || i + G < N)
        write_row<T, N>(sm + q * S::MS, i + G, o1);
    __syncthreads();
    stage_store<T, N, MPW>(sm, Mem<T>{C.p, C.bs, C.rs, false}, b0, batch, n);
}

template <typename T>
static size_t syrk_rows_lds(int N, int n, int k, int images)
{
    const size_t stage = (size_t)(N == 24 ? Stage<T, 24, ROWS_MPW>::ELEMS : Stage<T, 32, ROWS_MPW>::ELEMS);
    const size_t imgs = (size_t)images * rows_image_elems(n * k);
    return (stage > imgs ? stage : imgs) * sizeof(T);
}

template <typename T>
bool outer_rows_takes(int n, int k, bool two)
{
    return n > 16 && n <= 32 && k >= 1 && k <= ROWS_KMAX && syrk_rows_lds<T>(n <= 24 ? 24 : 32, n, k, two ? 2 : 1) <= 64 * 1024;
}
template bool outer_rows_takes<float>(int, int, bool);
template bool outer_rows_takes<double>(int, int, bool);

template <typename T>
la_status launch_outer_rows(bool img_tr, int tri, T alpha, int64_t batch, int n, int k, const T *U, const T *V, View<T> C,
                            hipStream_t st)
{
    if (batch <= 0 || n <= 0)
        return LA_OK;
    if (!outer_rows_takes<T>(n, k, U != V) || (batch + 3) / 4 > 0x7fffffffll || C.cs != 1)
        return LA_ERR_UNSUPPORTED;
    const bool two = (U != V);
    const dim3 grid((unsigned)((batch + ROWS_MPW - 1) / ROWS_MPW)), blk(WAVE);
    const int itr = img_tr ? 1 : 0;
#define LA_SYRK_ROWS(NN, TW)                                                                                         \
    LA_LAUNCH((k_syrk_rows<T, NN, TW>), grid, blk, syrk_rows_lds<T>(NN, n, k, TW ? 2 : 1), st, U, V, C, batch, n, k, \
              itr, tri, alpha)
    if (n <= 24) {
        if (two)
            LA_SYRK_ROWS(24, true);
        else
            LA_SYRK_ROWS(24, false);
    } else {
        if (two)
            LA_SYRK_ROWS(32, true);
        else
            LA_SYRK_ROWS(32, false);
    }
#undef LA_SYRK_ROWS
    return launch_check("syrk_rows");
}

template la_status launch_outer_rows<float>(bool, int, float, int64_t, int, int, const float *, const float *, View<float>,
                                            hipStream_t);
template la_status launch_outer_rows<double>(bool, int, double, int64_t, int, int, const double *, const double *,
                                             View<double>, hipStream_t);

}  // namespace la
