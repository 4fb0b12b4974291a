// Fused three-round kernels with fp32 diagonals in which one workgroup carries V vectors through the rounds together,
// so that every 16-byte load of a diagonal serves V vectors.  The diagonals are shared by the whole batch (Section 5:
// the parameters of the matrix are fixed in advance), and with fp32 diagonals their 12 bytes per element of L2 -> L1
// traffic, used once per load, is what holds the one-vector kernels back from n = 2^12 on (n = 2^12, 2^13 here).  Full-width output only
// (every coordinate kept, rows 16-byte aligned): the general kernels serve the rest.
#include "launch.hpp"
namespace spinner {

template <typename G, int V>
__global__ void __launch_bounds__(G::THREADS) __attribute__((amdgpu_waves_per_eu(G::MIN_WAVES > 0 ? G::MIN_WAVES : 1)))
spinner_shared_diag_kernel(TileParams p)
{
    static_assert(G::WB > 0 && G::LB == 6, "tiles that span several waves");
    constexpr int NT = G::NT, R = G::R, n = 1 << NT;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    ThreadCtx<G> c;
    c.lit = lane;
    c.wv = __builtin_amdgcn_readfirstlane(wave);
#pragma unroll
    for (int b = 0; b < 6; ++b) c.sg[b] = ((c.lit >> b) & 1) ? -1.0f : 1.0f;
    const long long vec0 = (long long)blockIdx.x * V;

    __shared__ float4 lds_store[G::LDS_FLOAT4];
    float4* lds = lds_store;

    float v[V][R];
    {
        const int e0 = c.base_index(G::layout_after(0));
#pragma unroll
        for (int vv = 0; vv < V; ++vv) {
            // a vector past the end of the batch reads the first one and stores nothing (no load under a condition)
            const long long vec = vec0 + vv < p.batch ? vec0 + vv : 0;
            const float* src = p.x + vec * (long long)n + e0;
#pragma unroll
            for (int jh = 0; jh < R / 4; ++jh) {
                const float4 t = load4<true>(src + G::reg_index(G::layout_after(0), jh * 4));
                v[vv][jh * 4] = t.x; v[vv][jh * 4 + 1] = t.y; v[vv][jh * 4 + 2] = t.z; v[vv][jh * 4 + 3] = t.w;
            }
        }
    }
    static_for<0, 3>([&](auto k) {
        constexpr int LAY = G::layout_after(k.value);
        // one diagonal load, V products
        const float* dk = p.d[k.value] + c.base_index(LAY);
#pragma unroll
        for (int jh = 0; jh < R / 4; ++jh) {
            const float4 t = *reinterpret_cast<const float4*>(dk + G::reg_index(LAY, jh * 4));
#pragma unroll
            for (int vv = 0; vv < V; ++vv) {
                v[vv][jh * 4] *= t.x; v[vv][jh * 4 + 1] *= t.y; v[vv][jh * 4 + 2] *= t.z; v[vv][jh * 4 + 3] *= t.w;
            }
        }
        // the transforms of the V vectors one after the other through the one exchange buffer (every exchange ends with a barrier)
#pragma unroll
        for (int vv = 0; vv < V; ++vv)
            spinner_step<G, NT, 0, LAY, false, (k.value == 0), (k.value == 1), false, float>(v[vv], c, nullptr, nullptr, 0, lds);
    });
    constexpr int LAYF = G::layout_after(3);
    const int ebase = c.base_index(LAYF);
    const float lane_factor = p.factor * tracked_sign<G, 0, float>(c);
#pragma unroll
    for (int vv = 0; vv < V; ++vv) {
        if (vec0 + vv < p.batch) {
            float* dst = p.out + (vec0 + vv) * p.out_stride + ebase;
#pragma unroll
            for (int jh = 0; jh < R / 4; ++jh)
                store4<true>(dst + G::reg_index(LAYF, jh * 4), v[vv][jh * 4] * lane_factor, v[vv][jh * 4 + 1] * lane_factor,
                             v[vv][jh * 4 + 2] * lane_factor, v[vv][jh * 4 + 3] * lane_factor);
        }
    }
}

// Measured in one run against one vector per workgroup (V = 1): n = 2^12 0.397 -> 0.384 ms with V = 2 (0.382 with 3, 0.402 with
// 4), n = 2^13 0.431 -> 0.421 ms with V = 2 (0.50-0.52 with 3 and 4: over 128 registers).  n = 2^14 lost with every V > 1
// (0.444 -> 0.472 ms with V = 2) and stays on the one-vector kernel.
template <int NT> struct SharedDiagTuning;
template <> struct SharedDiagTuning<12> : NotWide { static constexpr int rmax = 4, waves = 4, min_waves = 0, trips = 0, V = 2; };
template <> struct SharedDiagTuning<13> : NotWide { static constexpr int rmax = 5, waves = 4, min_waves = 0, trips = 2, V = 2; };

template <int NT>
static hipError_t launch_shared_nt(const TileParams& p, hipStream_t s)
{
    using TU = SharedDiagTuning<NT>;
    using G = GeomFrom<TU, NT>;
    const long long blocks = (p.batch + TU::V - 1) / TU::V;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((spinner_shared_diag_kernel<G, TU::V>), dim3((unsigned)blocks), dim3(G::THREADS), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_fused_shared_diag(int log2n, const TileParams& p, hipStream_t s)
{
    switch (log2n) {
    case 12: return launch_shared_nt<12>(p, s);
    case 13: return launch_shared_nt<13>(p, s);
    default: return hipErrorInvalidValue;
    }
}
}  // namespace spinner
