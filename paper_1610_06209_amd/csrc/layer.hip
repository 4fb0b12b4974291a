// Adaptive-layer kernels: forward with saved activations, backward, n = 2^4 .. 2^14; batch sums of the backward pass above that.
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

// Above the fused range the backward pass materialises the signal that arrives at each diagonal; the gradient of
// that diagonal is then a sum over the batch of (signal x activation), per coordinate.  Block (bx, by) owns four
// coordinates per thread and the vectors by, by + S, by + 2S, ... (S = gridDim.y) and writes row `by` of `partial`
// (fp64 sums, rounded once); layer_reduce_kernel adds the S rows in fp64 in a fixed order.  With d1 != null the same
// sweep also writes dx = d1 .* g (the last step of the backward pass).
__global__ void __launch_bounds__(256) layer_large_dd_kernel(const float* __restrict__ g, const float* __restrict__ a, long long n,
                                                             long long batch, float* __restrict__ partial,
                                                             const float* __restrict__ d1, float* __restrict__ dx)
{
    const long long i = ((long long)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= n) return;
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    float4 dv = make_float4(0.f, 0.f, 0.f, 0.f);
    if (d1) dv = *reinterpret_cast<const float4*>(d1 + i);
    for (long long b = blockIdx.y; b < batch; b += gridDim.y) {
        const float4 gv = *reinterpret_cast<const float4*>(g + b * n + i);
        const float4 av = *reinterpret_cast<const float4*>(a + b * n + i);
        s0 += (double)gv.x * (double)av.x; s1 += (double)gv.y * (double)av.y;
        s2 += (double)gv.z * (double)av.z; s3 += (double)gv.w * (double)av.w;
        if (d1) *reinterpret_cast<float4*>(dx + b * n + i) = make_float4(dv.x * gv.x, dv.y * gv.y, dv.z * gv.z, dv.w * gv.w);
    }
    *reinterpret_cast<float4*>(partial + (long long)blockIdx.y * n + i) = make_float4((float)s0, (float)s1, (float)s2, (float)s3);
}

// rows of `partial` the large-n backward pass uses: enough blocks to fill the chip, never more than the batch
long long layer_large_slabs(int log2n, long long batch)
{
    const long long per_row = ((1LL << log2n) / 4 + 255) / 256;       // blocks along the coordinates
    long long slabs = (2048 + per_row - 1) / per_row;
    if (slabs > batch) slabs = batch;
    if (slabs > 1024) slabs = 1024;
    return slabs < 1 ? 1 : slabs;
}

hipError_t launch_layer_large_dd(const float* g, const float* a, int log2n, long long batch, float* partial, float* dd,
                                 const float* d1, float* dx, hipStream_t s)
{
    const long long n = 1LL << log2n;
    const long long per_row = (n / 4 + 255) / 256;
    const long long slabs = layer_large_slabs(log2n, batch);
    if (per_row > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(layer_large_dd_kernel, dim3((unsigned)per_row, (unsigned)slabs), dim3(256), 0, s, g, a, n, batch, partial, d1, dx);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_layer_reduce(partial, slabs, n, 1.0, dd, s);
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
