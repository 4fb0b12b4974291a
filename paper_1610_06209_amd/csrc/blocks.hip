// Stacked independent blocks in one launch (Section 3.2: independently constructed m x n spinners stacked vertically;
// Section 5 takes k = L m > n random features this way).  One contiguous tile is one whole vector; x is loaded once
// and stays in registers while the L diagonal triples are applied one after the other, each block's epilogue going
// to its own column range of the output row.  fp32 diagonals [L][3][n]; n = 2^4 .. 2^14.
#include "launch.hpp"
namespace spinner {

struct BlockParams {
    TileParams t;             // x, out, batch, m, out_stride, factor, factor_rev, inv_sqrt_m, sin_off as for one block
    const float* diag_sets;   // [L][3][n]
    int L;
};

// EPI_STORE_NONE:   out[vec][l m + i]              = factor * y_l[i]
// EPI_STORE_COSSIN: out[vec][l m + i]              = cos(w_l[i]) / sqrt(L m),
//                   out[vec][sin_off + l m + i]    = sin(w_l[i]) / sqrt(L m),   sin_off = L m
// m and the row stride are multiples of 4 (checked by the caller), so a thread's four consecutive coordinates are kept
// or dropped together and every store is a 16-byte store.
template <typename T, typename G, int EPI>
__global__ void __launch_bounds__(G::THREADS) __attribute__((amdgpu_waves_per_eu(1)))
spinner_blocks_kernel(BlockParams p)
{
    constexpr int NT = G::NT, R = G::R, n = 1 << NT;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    ThreadCtx<G> c;
    long long vec;
    if constexpr (G::WB > 0) {
        vec = blockIdx.x;
        c.lit = lane;
        c.wv = __builtin_amdgcn_readfirstlane(wave);
    } else {
        vec = ((long long)blockIdx.x * G::WAVES + wave) * G::TPW + (lane >> G::LB);
        c.lit = lane & ((1 << G::LB) - 1);
        c.wv = 0;
    }
#pragma unroll
    for (int b = 0; b < 6; ++b) c.sg[b] = ((c.lit >> b) & 1) ? -1.0f : 1.0f;
    const bool active = vec < p.t.batch;

    __shared__ float4 lds_store[(std::is_same<T, float>::value || G::WB == 0) ? G::LDS_FLOAT4 : (1 << NT) / 4];
    float4* lds = lds_store;

    float x0[R];
    {
        const float* src = p.t.x + (active ? vec : 0) * (long long)n + c.base_index(0);      // a vector past the end reads the first one
#pragma unroll
        for (int jh = 0; jh < R / 4; ++jh) {
            const float4 t = load4<true>(src + G::reg_index(0, jh * 4));
            x0[jh * 4] = t.x; x0[jh * 4 + 1] = t.y; x0[jh * 4 + 2] = t.z; x0[jh * 4 + 3] = t.w;
        }
    }
    constexpr int LAYF = G::layout_after(3);
    const int ebase = c.base_index(LAYF);
    const float lane_factor = p.t.factor * tracked_sign<G, 0, T>(c);      // three transforms leave the tracked lane sign
    float* row = p.t.out + (active ? vec : 0) * p.t.out_stride;
    const int m = active ? p.t.m : 0;

    for (int l = 0; l < p.L; ++l) {
        const float* d = p.diag_sets + (long long)l * 3 * n;
        T v[R];
#pragma unroll
        for (int j = 0; j < R; ++j) v[j] = (T)x0[j];
        if constexpr (G::WB > 0) __syncthreads();      // the exchange buffer is free again (a block starts in layout 0)
        spinner_step<G, NT, 0, G::layout_after(0), true, true, false, false, T>(v, c, d, nullptr, 0, lds);
        spinner_step<G, NT, 0, G::layout_after(1), true, false, true, false, T>(v, c, d + n, nullptr, 0, lds);
        spinner_step<G, NT, 0, G::layout_after(2), true, false, false, false, T>(v, c, d + 2 * n, nullptr, 0, lds);

        float* dst = row + (long long)l * p.t.m;
#pragma unroll
        for (int jh = 0; jh < R / 4; ++jh) {
            const int i = ebase | G::reg_index(LAYF, jh * 4);
            if constexpr (EPI == EPI_STORE_NONE) {
                const float a0 = (float)(v[jh * 4] * (T)lane_factor), a1 = (float)(v[jh * 4 + 1] * (T)lane_factor);
                const float a2 = (float)(v[jh * 4 + 2] * (T)lane_factor), a3 = (float)(v[jh * 4 + 3] * (T)lane_factor);
                if (i < m) store4<true>(dst + i, a0, a1, a2, a3);
            } else {
                float sn[4], cs[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    feature_sincos(v[jh * 4 + k], p.t, lane_factor, sn[k], cs[k]);
                    sn[k] *= p.t.inv_sqrt_m;
                    cs[k] *= p.t.inv_sqrt_m;
                }
                if (i < m) {
                    store4<true>(dst + i, cs[0], cs[1], cs[2], cs[3]);
                    store4<true>(dst + p.t.sin_off + i, sn[0], sn[1], sn[2], sn[3]);
                }
            }
        }
    }
}

// 32 values per thread at most, so that the resident copy of x fits beside the working values
template <typename T, int NT> struct BlocksTuning : Tuning<T, NT> {};
template <> struct BlocksTuning<float, 11> : NotWide { static constexpr int rmax = 5, waves = 4, min_waves = 0, trips = 0; };
template <> struct BlocksTuning<float, 12> : NotWide { static constexpr int rmax = 5, waves = 4, min_waves = 0, trips = 0; };
template <> struct BlocksTuning<float, 13> : NotWide { static constexpr int rmax = 5, waves = 4, min_waves = 0, trips = 0; };
template <> struct BlocksTuning<float, 14> : NotWide { static constexpr int rmax = 5, waves = 4, min_waves = 0, trips = 0; };

template <typename T, int NT, int EPI>
static hipError_t launch_blocks_nt(const BlockParams& p, hipStream_t s)
{
    using G = GeomFrom<BlocksTuning<T, NT>, NT>;
    static_assert(G::R <= 32, "resident x beside the working values");
    const long long blocks = (p.t.batch + G::TILES_PER_WG - 1) / G::TILES_PER_WG;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((spinner_blocks_kernel<T, G, EPI>), dim3((unsigned)blocks), dim3(G::THREADS), 0, s, p);
    return hipGetLastError();
}

#define CASE(NT) case NT: return cossin ? launch_blocks_nt<double, NT, EPI_STORE_COSSIN>(bp, s) : launch_blocks_nt<float, NT, EPI_STORE_NONE>(bp, s);
hipError_t launch_blocks(int log2n, bool cossin, const TileParams& p, const float* diag_sets, int L, hipStream_t s)
{
    BlockParams bp;
    bp.t = p;
    bp.diag_sets = diag_sets;
    bp.L = L;
    switch (log2n) {
        CASE(4) CASE(5) CASE(6) CASE(7) CASE(8) CASE(9) CASE(10) CASE(11) CASE(12) CASE(13) CASE(14)
    default: return hipErrorInvalidValue;
    }
}
#undef CASE
}  // namespace spinner
