// Adaptive-layer kernels: forward with saved activations, backward, n = 2^4 .. 2^14.
#include "launch.hpp"
#include "layer_kernels.hpp"
namespace spinner {
// 16 values per thread up to n = 2^12, 32 above: the backward kernel keeps three running sums per
// value in registers beside the signal itself
constexpr int layer_rmax(int nt) { return nt <= 5 ? 2 : (nt <= 9 ? 3 : (nt <= 12 ? 4 : 5)); }
template <int NT>
using LayerGeom = TileGeom<NT, layer_rmax(NT), 4>;

// dd[i] = factor * sum over slots of partial[slot][i], summed in fp64 in a fixed order.  A block owns 16
// columns; its 16 slot lanes walk the slots with stride 16 and are then added up through LDS.
__global__ void __launch_bounds__(256) layer_reduce_kernel(const float* __restrict__ partial, long long slots, long long len,
                                                           double factor, float* __restrict__ dd)
{
    __shared__ double sh[16][17];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const long long i = (long long)blockIdx.x * 16 + tx;
    double s = 0.0;
    if (i < len) {
        long long k = ty;
        for (; k + 48 < slots; k += 64) {        // four independent loads in flight per thread
            const float a0 = partial[k * len + i], a1 = partial[(k + 16) * len + i];
            const float a2 = partial[(k + 32) * len + i], a3 = partial[(k + 48) * len + i];
            s += ((double)a0 + (double)a1) + ((double)a2 + (double)a3);
        }
        for (; k < slots; k += 16) s += (double)partial[k * len + i];
    }
    sh[ty][tx] = s;
    __syncthreads();
    if (ty == 0 && i < len) {
        double t = 0.0;
#pragma unroll
        for (int r = 0; r < 16; ++r) t += sh[r][tx];
        dd[i] = (float)(factor * t);
    }
}

template <int NT>
static hipError_t forward_nt(const LayerForwardParams& p, hipStream_t s)
{
    using G = LayerGeom<NT>;
    const long long blocks = (p.batch + G::TILES_PER_WG - 1) / G::TILES_PER_WG;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((layer_forward_kernel<G>), dim3((unsigned)blocks), dim3(G::THREADS), 0, s, p);
    return hipGetLastError();
}

template <int NT>
static long long slots_nt(long long batch)
{
    using G = LayerGeom<NT>;
    // four workgroups for each of the 256 compute units (as many as the kernel's registers let a compute unit hold
    // where it is compiled for a given number of waves per SIMD), fewer when the batch is small
    // (32 values per thread: two waves per SIMD, 512 workgroups are resident)
    long long wgs = (G::R == 16 && G::WB > 0) ? 256 * 4 * kLayerBackwardWaves / G::WAVES : (G::R == 32 ? 512 : 1024);
    const long long need = (batch + G::TILES_PER_WG - 1) / G::TILES_PER_WG;
    if (wgs > need) wgs = need;
    // small vectors put many tiles into one workgroup: keep the number of partial rows bounded
    if (wgs * G::TILES_PER_WG > 8192) wgs = 8192 / G::TILES_PER_WG;
    return wgs * G::TILES_PER_WG;
}

template <int NT>
static hipError_t backward_nt(const LayerBackwardParams& p, hipStream_t s)
{
    using G = LayerGeom<NT>;
    const long long blocks = p.slots / G::TILES_PER_WG;
    if (blocks <= 0) return hipSuccess;
    hipLaunchKernelGGL((layer_backward_kernel<G>), dim3((unsigned)blocks), dim3(G::THREADS), 0, s, p);
    return hipGetLastError();
}

#define CASES(F, ...) switch (log2n) { case 4: return F<4>(__VA_ARGS__); case 5: return F<5>(__VA_ARGS__); case 6: return F<6>(__VA_ARGS__); \
    case 7: return F<7>(__VA_ARGS__); case 8: return F<8>(__VA_ARGS__); case 9: return F<9>(__VA_ARGS__); case 10: return F<10>(__VA_ARGS__); \
    case 11: return F<11>(__VA_ARGS__); case 12: return F<12>(__VA_ARGS__); case 13: return F<13>(__VA_ARGS__); case 14: return F<14>(__VA_ARGS__); \
    default: break; }

hipError_t launch_layer_forward(int log2n, const LayerForwardParams& p, hipStream_t s)
{
    CASES(forward_nt, p, s)
    return hipErrorInvalidValue;
}
long long layer_backward_slots(int log2n, long long batch)
{
    CASES(slots_nt, batch)
    return 0;
}
hipError_t launch_layer_backward(int log2n, const LayerBackwardParams& p, hipStream_t s)
{
    CASES(backward_nt, p, s)
    return hipErrorInvalidValue;
}
hipError_t launch_layer_reduce(const float* partial, long long slots, long long len, double factor, float* dd, hipStream_t s)
{
    const long long blocks = (len + 15) / 16;
    hipLaunchKernelGGL(layer_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, s, partial, slots, len, factor, dd);
    return hipGetLastError();
}
#undef CASES
}  // namespace spinner
