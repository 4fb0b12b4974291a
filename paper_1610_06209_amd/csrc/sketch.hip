// Newton-sketch helpers: transposition with optional row weights (the sketch acts on the columns
// of a row-major data matrix) and the Gram matrix B^T B on the fp32 matrix pipe.
#include <mutex>

#include "launch.hpp"
namespace spinner {

// dst[c][r] = src[r][c] * (row_scale ? row_scale[r] : 1), src is [rows][cols] row-major.
// 64 x 64 tiles through LDS (row padded by one word), both sides coalesced.  All sixteen loads of a thread are
// issued before the first is used: rows and columns past the end are clamped to the last one (and not stored), so
// that no load sits under a condition.
template <bool SCALED>
__global__ void __launch_bounds__(256) transpose_scale_kernel(const float* __restrict__ src, long long rows, long long cols,
                                                              const float* __restrict__ row_scale, float* __restrict__ dst)
{
    __shared__ float tile[64][65];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const long long r0 = (long long)blockIdx.y * 64, c0 = (long long)blockIdx.x * 64;
    const long long cc = c0 + tx < cols ? c0 + tx : cols - 1;
    float v[16], w[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const long long r = r0 + ty + 4 * k;
        const long long rr = r < rows ? r : rows - 1;
        v[k] = src[rr * cols + cc];
        w[k] = SCALED ? row_scale[rr] : 1.0f;
    }
#pragma unroll
    for (int k = 0; k < 16; ++k) tile[ty + 4 * k][tx] = SCALED ? v[k] * w[k] : v[k];
    __syncthreads();
    const long long r = r0 + tx;
    if (r0 + 64 <= rows && c0 + 64 <= cols) {
#pragma unroll
        for (int k = 0; k < 16; ++k) dst[(c0 + ty + 4 * k) * rows + r] = tile[tx][ty + 4 * k];
    } else {
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const long long c = c0 + ty + 4 * k;
            if (r < rows && c < cols) dst[c * rows + r] = tile[tx][ty + 4 * k];
        }
    }
}

hipError_t launch_transpose_scale(const float* src, long long rows, long long cols, const float* row_scale, float* dst,
                                  hipStream_t s)
{
    if (rows <= 0 || cols <= 0) return hipSuccess;
    const long long gx = (cols + 63) / 64, gy = (rows + 63) / 64;
    if (gx > 0x7fffffffLL || gy > 65535) return hipErrorInvalidConfiguration;
    if (row_scale)
        hipLaunchKernelGGL(transpose_scale_kernel<true>, dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, s, src, rows, cols, row_scale, dst);
    else
        hipLaunchKernelGGL(transpose_scale_kernel<false>, dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, s, src, rows, cols, row_scale, dst);
    return hipGetLastError();
}

// G = B^T B for B [m][d] row-major: G[a][b] = sum_k B[k][a] B[k][b].  A workgroup of four waves owns a
// 128 x 128 block of G (each wave 64 x 64 = 2 x 2 tiles of v_mfma_f32_32x32x2_f32) and walks k in chunks
// of 16 rows of B staged in LDS.  Both MFMA operands are rows of B: lane l supplies B[k + l / 32][. + l % 32].
typedef float floatx16 __attribute__((ext_vector_type(16)));
constexpr int kGramBlock = 128, kGramK = 16;
// Split over k: block z handles rows [z * kchunk, (z + 1) * kchunk) of B and writes its own d x d slab of `out`
// (G itself when there is a single slab); the slabs are added up afterwards in a fixed order.
__global__ void __launch_bounds__(256) sketch_gram_kernel(const float* __restrict__ B, int m_total, int d, int kchunk,
                                                          float* __restrict__ out)
{
    const int k_begin = blockIdx.z * kchunk;
    const int m = k_begin + kchunk < m_total ? k_begin + kchunk : m_total;
    float* G = out + (long long)blockIdx.z * d * d;
    __shared__ float sa[kGramK][kGramBlock];
    __shared__ float sb[kGramK][kGramBlock];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wa = wave >> 1, wb = wave & 1;
    const int a0 = blockIdx.y * kGramBlock, b0 = blockIdx.x * kGramBlock;
    floatx16 acc[2][2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][u][v] = 0.f;

    // 16 rows x 128 columns per operand, 256 threads: 8 values per thread and operand.  A chunk is loaded into
    // registers while the chunk before it is multiplied (addresses clamped to the last row / column, what lies
    // outside set to zero afterwards: no load under a condition).
    float ra[8], rb[8];
    auto load_chunk = [&](int k0) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int idx = q * 256 + threadIdx.x;
            const int kk = idx >> 7, col = idx & 127;
            const int row = k0 + kk < m ? k0 + kk : m - 1;
            const int ca = a0 + col < d ? a0 + col : d - 1, cb = b0 + col < d ? b0 + col : d - 1;
            ra[q] = B[(long long)row * d + ca];
            rb[q] = B[(long long)row * d + cb];
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int idx = q * 256 + threadIdx.x;
            const int kk = idx >> 7, col = idx & 127;
            const bool row_ok = k0 + kk < m;
            if (!(row_ok && a0 + col < d)) ra[q] = 0.f;
            if (!(row_ok && b0 + col < d)) rb[q] = 0.f;
        }
    };
    if (k_begin < m) load_chunk(k_begin);
    for (int k0 = k_begin; k0 < m; k0 += kGramK) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int idx = q * 256 + threadIdx.x;
            sa[idx >> 7][idx & 127] = ra[q];
            sb[idx >> 7][idx & 127] = rb[q];
        }
        __syncthreads();
        if (k0 + kGramK < m) load_chunk(k0 + kGramK);
#pragma unroll
        for (int kk = 0; kk < kGramK; kk += 2) {
            float fa[2], fb[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                fa[t] = sa[kk + (lane >> 5)][wa * 64 + t * 32 + (lane & 31)];
                fb[t] = sb[kk + (lane >> 5)][wb * 64 + t * 32 + (lane & 31)];
            }
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int u = 0; u < 2; ++u) acc[t][u] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[t], fb[u], acc[t][u], 0, 0, 0);
        }
        __syncthreads();
    }
    // result register v of lane l holds row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32 of its 32 x 32 tile
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = a0 + wa * 64 + t * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                const int col = b0 + wb * 64 + u * 32 + (lane & 31);
                if (row < d && col < d) G[(long long)row * d + col] = acc[t][u][v];
            }
}

__global__ void __launch_bounds__(256) gram_reduce_kernel(const float* __restrict__ slabs, int count, long long len,
                                                          float* __restrict__ G)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= len) return;
    float s = 0.f;
    int k = 0;
    for (; k + 3 < count; k += 4) {         // four loads in flight; the order of the additions stays fixed
        const float a0 = slabs[k * len + i], a1 = slabs[(k + 1) * len + i], a2 = slabs[(k + 2) * len + i], a3 = slabs[(k + 3) * len + i];
        s += a0; s += a1; s += a2; s += a3;
    }
    for (; k < count; ++k) s += slabs[k * len + i];
    G[i] = s;
}

// number of k-slabs: enough blocks to fill the chip, at least 64 rows of B per slab, at most 64 slabs
int sketch_gram_slabs(int m, int d)
{
    const long long tiles = (long long)((d + kGramBlock - 1) / kGramBlock) * ((d + kGramBlock - 1) / kGramBlock);
    constexpr int kGramWorkgroups = 256;      // workgroups aimed at when the sum over k is split (128 .. 1024 measured alike)
    long long ks = (kGramWorkgroups + tiles - 1) / tiles;
    if (ks > (m + 63) / 64) ks = (m + 63) / 64;
    if (ks > 64) ks = 64;
    return ks < 1 ? 1 : (int)ks;
}

// Scratch of the entry point that allocates nothing: the slabs of the split sum live in a file-scope device array.
// Every GPU the library runs on holds its own copy at its own address; in host code the array's name is only a
// handle, so its device address is asked for once per device (hipGetSymbolAddress with that device current) and
// kept, and that pointer - never the name - is what reaches the kernels.
static __device__ __align__(256) unsigned char gram_static_scratch[kGramStaticScratchBytes];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_lock;
static float* g_scratch_ptr[kMaxDevices];     // device address of gram_static_scratch on each device, once known

hipError_t gram_static_scratch_ptr(float** ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(gram_static_scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<float*>(p);
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

hipError_t launch_sketch_gram(const float* B, int m, int d, float* G, float* slabs, hipStream_t s)
{
    if (m <= 0 || d <= 0) return hipSuccess;
    const int g = (d + kGramBlock - 1) / kGramBlock;
    if (g > 65535) return hipErrorInvalidConfiguration;
    const int ks = sketch_gram_slabs(m, d);
    int kchunk = (m + ks - 1) / ks;
    kchunk = (kchunk + kGramK - 1) / kGramK * kGramK;
    hipLaunchKernelGGL(sketch_gram_kernel, dim3((unsigned)g, (unsigned)g, (unsigned)ks), dim3(256), 0, s, B, m, d, kchunk,
                       ks > 1 ? slabs : G);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || ks == 1) return e;
    const long long len = (long long)d * d;
    hipLaunchKernelGGL(gram_reduce_kernel, dim3((unsigned)((len + 255) / 256)), dim3(256), 0, s, slabs, ks, len, G);
    return hipGetLastError();
}
}  // namespace spinner
