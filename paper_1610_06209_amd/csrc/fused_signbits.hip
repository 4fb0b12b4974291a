// Fused three-round kernels with the sign-code epilogue (angular-kernel features),
// n = 2^8 .. 2^16, with fp32 diagonals or packed sign words; the last round is pruned
// when m <= n / 16.  Also the code-packing kernel used above the fused range and the
// Hamming-distance Gram kernel.
#include "launch.hpp"
namespace spinner {
// The epilogue needs a whole wave per 256 coordinates (six lane bits per tile), so the
// values per thread are capped at n / 64.
#ifndef SPINNER_CODE_RMAX       // tuning experiments: cap on the values per thread (log2) of the sign-code kernels
#define SPINNER_CODE_RMAX 6
#endif
template <typename TU, int NT>
using GeomCodeFrom = TileGeom<NT, clamp_rmax(NT, (TU::rmax < NT - 6 ? (TU::rmax < SPINNER_CODE_RMAX ? TU::rmax : SPINNER_CODE_RMAX) : NT - 6)),
                              TU::waves, TU::min_waves, TU::trips>;
// Without pruning, n = 2^12 .. 2^14 take the wide exchanges of the plain kernels, loading in layout 1 so that
// the three rounds end in layout 0, where a wave's lanes hold index bits 2..7 (one code word per register).
#ifndef SPINNER_CODE_WIDE
#define SPINNER_CODE_WIDE 0x7000
#endif
template <int NT> struct CodeWide { static constexpr int rmax = NT >= 13 ? 6 : 5, waves = 4, min_waves = NT >= 13 ? 4 : 0, trips = 2, wide = 1, start = 1; };
template <int NT, bool PRUNED>
using GeomCode = std::conditional_t<PRUNED, GeomCodeFrom<PrunedTuning<float, NT>, NT>,
                                    std::conditional_t<((SPINNER_CODE_WIDE >> NT) & 1) != 0, GeomFrom<CodeWide<NT>, NT>, GeomCodeFrom<Tuning<float, NT>, NT>>>;

template <int NT, bool SIGNS, int PRUNE>
static hipError_t launch_code_tile(const TileParams& p, long long tiles, hipStream_t stream)
{
    using G = GeomCode<NT, (PRUNE > 0)>;
    static_assert(G::TILES_PER_WG >= 1 && G::LB == 6, "one tile per wave or several waves per tile");
    const long long blocks = (tiles + G::TILES_PER_WG - 1) / G::TILES_PER_WG;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((spinner_tile_kernel<float, G, NT, 3, true, EPI_STORE_SIGNBITS, SIGNS, PRUNE>),
                       dim3((unsigned)blocks), dim3(G::THREADS), 0, stream, p);
    return hipGetLastError();
}

#define CASE(NT) case NT: return signs ? launch_code_tile<NT, true, 0>(p, tiles, s) : launch_code_tile<NT, false, 0>(p, tiles, s);
#define PCASE(NT) case NT: return signs ? launch_code_tile<NT, true, kPruneBits>(p, tiles, s) \
                                        : launch_code_tile<NT, false, kPruneBits>(p, tiles, s);
hipError_t launch_fused_signbits(int log2n, bool signs, int prune, const TileParams& p, long long tiles, hipStream_t s)
{
    if (prune >= kPruneBits) {
        switch (log2n) {
            PCASE(12) PCASE(13) PCASE(14)
        default: break;
        }
    }
    switch (log2n) {
        CASE(8) CASE(9) CASE(10) CASE(11) CASE(12) CASE(13) CASE(14) CASE(15) CASE(16)
    default: return hipErrorInvalidValue;
    }
}
#undef CASE
#undef PCASE

// One wave per code word: lane l looks at coordinate ((w >> 2) << 8) | (l << 2) | (w & 3)
// of its vector and the wave's ballot of "negative" is the word.
__global__ void __launch_bounds__(256) pack_codes_kernel(const float* __restrict__ y, long long y_stride,
                                                         unsigned long long* __restrict__ codes, int words_per_vec,
                                                         long long total_words)
{
    const long long gw = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (gw >= total_words) return;
    const long long vec = gw / words_per_vec;
    const int w = (int)(gw - vec * words_per_vec);
    const long long e = ((long long)(w >> 2) << 8) | (lane << 2) | (w & 3);
    const unsigned long long mk = __ballot(y[vec * y_stride + e] < 0.0f);
    if (lane == 0) codes[gw] = mk;
}

hipError_t launch_pack_codes(const float* y, long long y_stride, unsigned long long* codes, int m, long long batch, hipStream_t s)
{
    const int words = m / 64;
    const long long total = batch * words;
    const long long blocks = (total + 3) / 4;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(pack_codes_kernel, dim3((unsigned)blocks), dim3(256), 0, s, y, y_stride, codes, words, total);
    return hipGetLastError();
}

// out[i][j] = 1 - popcount(a_i xor b_j) / m.  A workgroup of 16 x 16 threads owns a block of
// 64 x 64 pairs (4 x 4 per thread) and walks the code words in chunks of 32 staged in LDS
// (rows padded by one word so that the 16 rows a wave reads at once fall into different banks).
constexpr int kGramTile = 64, kGramChunk = 32;
__global__ void __launch_bounds__(256) hamming_gram_kernel(const unsigned long long* __restrict__ a, long long na,
                                                           const unsigned long long* __restrict__ b, long long nb,
                                                           int words, float inv_m, float* __restrict__ out)
{
    __shared__ unsigned long long sa[kGramTile][kGramChunk + 1];
    __shared__ unsigned long long sb[kGramTile][kGramChunk + 1];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const long long i0 = (long long)blockIdx.y * kGramTile, j0 = (long long)blockIdx.x * kGramTile;
    int dh[4][4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int w = 0; w < 4; ++w) dh[u][w] = 0;

    for (int k0 = 0; k0 < words; k0 += kGramChunk) {
        // 64 rows x 32 words per operand, 256 threads: 8 words per thread and operand
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int idx = t * 256 + threadIdx.x;
            const int row = idx >> 5, col = idx & 31;
            const bool in_k = k0 + col < words;
            sa[row][col] = (in_k && i0 + row < na) ? a[(i0 + row) * words + k0 + col] : 0ull;
            sb[row][col] = (in_k && j0 + row < nb) ? b[(j0 + row) * words + k0 + col] : 0ull;
        }
        __syncthreads();
#pragma unroll 4
        for (int k = 0; k < kGramChunk; ++k) {
            unsigned long long ra[4], rb[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { ra[u] = sa[ty * 4 + u][k]; rb[u] = sb[tx + 16 * u][k]; }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int w = 0; w < 4; ++w) dh[u][w] += __popcll(ra[u] ^ rb[w]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const long long i = i0 + ty * 4 + u;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const long long j = j0 + tx + 16 * w;
            if (i < na && j < nb) out[i * nb + j] = 1.0f - (float)dh[u][w] * inv_m;
        }
    }
}

hipError_t launch_hamming_gram(const unsigned long long* a, long long na, const unsigned long long* b, long long nb, int m,
                               float* out, hipStream_t s)
{
    if (na <= 0 || nb <= 0) return hipSuccess;
    const long long gx = (nb + kGramTile - 1) / kGramTile, gy = (na + kGramTile - 1) / kGramTile;
    if (gx > 0x7fffffffLL || gy > 65535) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(hamming_gram_kernel, dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, s, a, na, b, nb, m / 64,
                       1.0f / (float)m, out);
    return hipGetLastError();
}
}  // namespace spinner
