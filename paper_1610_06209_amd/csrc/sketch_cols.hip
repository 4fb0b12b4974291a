// Newton sketch without a transposition (Supplement, "Additional experiments": S W^{1/2} A with S the first m rows
// of a scaled spinner): the spinner acts on the COLUMNS of the row-major n x d matrix, and this kernel loads them as
// they lie.  A tile is all n rows by 16 or 32 contiguous columns (64- or 128-byte segments of each row): the low four
// or five index bits of a tile element are the column and are never transformed, the rest is the row index, on which the three rounds
// run with the same register / lane / LDS stages as the projection kernels.  A diagonal entry belongs to a row, so
// one 4-byte load serves the four columns a thread holds of it; the row weights multiply with the first diagonal.
// Only rows below m are stored.  A whole column group has to be on chip: n <= 2^12 (2^16 elements per workgroup),
// and the number of workgroups is d / 16, so this form pays for wide matrices and for small ones (one launch instead
// of three); the caller picks it by shape (sketch_cols_pays).
#include "launch.hpp"
namespace spinner {

struct SketchColsParams {
    const float* A;        // [n][d] row-major
    const float* w;        // [n] row weights or null
    const float* d[3];     // [n] each
    float* B;              // [m][d] row-major
    long long dcols;       // d
    long long tiles;       // column groups
    int m;
    float factor;          // n^{-3/2} * scale
};

// 32 columns per tile (128-byte segments) where such a tile fits (n <= 2^11) and the matrix is wide enough to fill the chip
// with them; 16 columns otherwise.  Measured on 256 MiB matrices: n = 1024 0.191 -> 0.125 ms with 32 columns (64 no better).
constexpr long long kSketchWideMinCols = 8192;
// With 16 columns two neighbouring tiles share every 128-byte line; workgroups go to the XCDs in turn, so each XCD takes
// runs of four consecutive tiles (xcd_tile): n = 4096, 256 MiB: 0.219 -> 0.184 ms.  No effect with 32 columns.
constexpr int sketch_cols_xcd_group_log(int c) { return c == 4 ? 2 : -1; }
// values per thread (log2) for tiles held by one wave; larger tiles take the geometry of the projection kernels
constexpr int sketch_cols_rmax(int nt) { return nt - 6; }
template <int NT>
using SketchColsGeom = std::conditional_t<(NT >= 12), GeomFor<float, NT>, TileGeom<NT, sketch_cols_rmax(NT), 4>>;

template <typename G, int C, int LAY>
__device__ __forceinline__ void row_diag_multiply(float (&v)[G::R], int ebase, const float* __restrict__ diag, const float* __restrict__ w)
{
#pragma unroll
    for (int jh = 0; jh < G::R / 4; ++jh) {
        const int row = (ebase | G::reg_index(LAY, jh * 4)) >> C;
        float f = diag[row];
        if (w) f *= w[row];
        v[jh * 4] *= f; v[jh * 4 + 1] *= f; v[jh * 4 + 2] *= f; v[jh * 4 + 3] *= f;
    }
}

template <typename G, int C>
__global__ void __launch_bounds__(G::THREADS) sketch_cols_kernel(SketchColsParams p)
{
    constexpr int NT = G::NT, R = G::R;
    static_assert(G::LB == 6 && !G::WIDE && NT - C >= 4 && C >= 2 && C <= 8, "a wave holds one tile or a part of one; column tiles never use wide exchanges");
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    ThreadCtx<G> c;
    c.lit = lane;
    long long tile;
    if constexpr (G::WB > 0) {
        tile = xcd_tile(blockIdx.x, gridDim.x, sketch_cols_xcd_group_log(C));
        c.wv = __builtin_amdgcn_readfirstlane(wave);
    } else {
        tile = xcd_tile(blockIdx.x, gridDim.x, sketch_cols_xcd_group_log(C)) * G::WAVES + wave;
        c.wv = 0;
    }
#pragma unroll
    for (int b = 0; b < 6; ++b) c.sg[b] = ((c.lit >> b) & 1) ? -1.0f : 1.0f;

    __shared__ float4 lds_store[G::LDS_FLOAT4];
    float4* lds = lds_store;

    // a tile past the end works on tile 0 and stores nothing (no load sits under a condition); the same for the
    // columns of the last tile that lie beyond d, which read the tile's first four columns
    const bool active = tile < p.tiles;
    const long long first_col = (active ? tile : 0) << C;
    const int col_in_tile = (lane << 2) & ((1 << C) - 1);          // index bits 2, 3 are lane bits in both layouts
    const bool col_ok = first_col + col_in_tile < p.dcols;
    const long long col = first_col + (col_ok ? col_in_tile : 0);

    constexpr int LAY0 = G::layout_after(0), LAY1 = G::layout_after(1), LAY2 = G::layout_after(2), LAYF = G::layout_after(3);
    float v[R];
    {
        const int e0 = c.base_index(LAY0);
#pragma unroll
        for (int jh = 0; jh < R / 4; ++jh) {
            const long long row = (e0 | G::reg_index(LAY0, jh * 4)) >> C;
            const float4 t = load4<true>(p.A + row * p.dcols + col);
            v[jh * 4] = t.x; v[jh * 4 + 1] = t.y; v[jh * 4 + 2] = t.z; v[jh * 4 + 3] = t.w;
        }
    }
    row_diag_multiply<G, C, LAY0>(v, c.base_index(LAY0), p.d[0], p.w);
    spinner_step<G, C, C, LAY0, false, true, false, false, float>(v, c, nullptr, nullptr, 0, lds);
    row_diag_multiply<G, C, LAY1>(v, c.base_index(LAY1), p.d[1], nullptr);
    spinner_step<G, C, C, LAY1, false, false, true, false, float>(v, c, nullptr, nullptr, 0, lds);
    row_diag_multiply<G, C, LAY2>(v, c.base_index(LAY2), p.d[2], nullptr);
    spinner_step<G, C, C, LAY2, false, false, false, false, float>(v, c, nullptr, nullptr, 0, lds);

    if (active && col_ok) {
        // held values carry the tracked lane sign after an odd number of transforms
        const float f = p.factor * tracked_sign<G, C, float>(c);
        const int ef = c.base_index(LAYF);
#pragma unroll
        for (int jh = 0; jh < R / 4; ++jh) {
            const int row = (ef | G::reg_index(LAYF, jh * 4)) >> C;
            if (row < p.m)
                store4<true>(p.B + (long long)row * p.dcols + col, v[jh * 4] * f, v[jh * 4 + 1] * f, v[jh * 4 + 2] * f, v[jh * 4 + 3] * f);
        }
    }
}

template <int NT, int C>
static hipError_t launch_cols_nt(SketchColsParams p, hipStream_t s)
{
    if constexpr (NT - C < 4 || NT > 16) return hipErrorInvalidValue;
    else {
    p.tiles = (p.dcols + (1 << C) - 1) >> C;
    using G = SketchColsGeom<NT>;
    const long long blocks = (p.tiles + G::TILES_PER_WG - 1) / G::TILES_PER_WG;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((sketch_cols_kernel<G, C>), dim3((unsigned)blocks), dim3(G::THREADS), 0, s, p);
    return hipGetLastError();
    }
}

// n = 2^4 .. 2^12, d a multiple of 4, every pointer 16-byte aligned (the caller checks)
template <int C>
static hipError_t launch_cols_c(int log2n, const SketchColsParams& p, hipStream_t s)
{
    switch (log2n) {
    case 4: return launch_cols_nt<4 + C, C>(p, s);
    case 5: return launch_cols_nt<5 + C, C>(p, s);
    case 6: return launch_cols_nt<6 + C, C>(p, s);
    case 7: return launch_cols_nt<7 + C, C>(p, s);
    case 8: return launch_cols_nt<8 + C, C>(p, s);
    case 9: return launch_cols_nt<9 + C, C>(p, s);
    case 10: return launch_cols_nt<10 + C, C>(p, s);
    case 11: return launch_cols_nt<11 + C, C>(p, s);
    case 12: return launch_cols_nt<12 + C, C>(p, s);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_sketch_cols(const float* A, int log2n, long long d, const float* w, const float* d1, const float* d2, const float* d3,
                              int m, float factor, float* B, hipStream_t s)
{
    SketchColsParams p;
    p.A = A; p.w = w; p.d[0] = d1; p.d[1] = d2; p.d[2] = d3; p.B = B;
    p.dcols = d; p.tiles = 0;
    p.m = m; p.factor = factor;
    if (log2n <= 11 && d >= kSketchWideMinCols) return launch_cols_c<5>(log2n, p, s);
    return launch_cols_c<4>(log2n, p, s);
}
}  // namespace spinner
