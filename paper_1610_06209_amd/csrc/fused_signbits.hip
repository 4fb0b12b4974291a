// Fused three-round kernels with the sign-code epilogue (angular-kernel features),
// n = 2^8 .. 2^16, with fp32 diagonals or packed sign words; the last round is pruned
// when m <= n / 16.  Also the code-packing kernel used above the fused range and the
// Hamming-distance Gram kernel.
#include "launch.hpp"
namespace spinner {
// The epilogue needs a whole wave per 256 coordinates (six lane bits per tile), so the
// values per thread are capped at n / 64.
template <typename TU, int NT>
using GeomCodeFrom = TileGeom<NT, clamp_rmax(NT, (TU::rmax < NT - 6 ? TU::rmax : NT - 6)),
                              TU::waves, TU::min_waves, TU::trips>;
// Without pruning, n = 2^12 .. 2^14 take the wide exchanges of the plain kernels, loading in layout 1 so that
// the three rounds end in layout 0, where a wave's lanes hold index bits 2..7 (one code word per register).
template <int NT> struct CodeWide { static constexpr int rmax = NT >= 13 ? 6 : 5, waves = 4, min_waves = NT >= 13 ? 4 : 0, trips = 2, wide = 1, start = 1, chunk = kLaneChunk; };
template <int NT, bool PRUNED>
using GeomCode = std::conditional_t<PRUNED, GeomCodeFrom<PrunedTuning<float, NT>, NT>,
                                    std::conditional_t<has_wide_words(NT), GeomFrom<CodeWide<NT>, NT>, GeomCodeFrom<Tuning<float, NT>, NT>>>;

template <int NT, bool SIGNS, int PRUNE>
static hipError_t launch_code_tile(const TileParams& p, long long tiles, hipStream_t stream)
{
    using G = GeomCode<NT, (PRUNE > 0)>;
    static_assert(G::TILES_PER_WG >= 1 && G::LB == 6, "one tile per wave or several waves per tile");
    const long long blocks = (tiles + G::TILES_PER_WG - 1) / G::TILES_PER_WG;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    TileParams q = p;
    q.xcd_group_log = SIGNS ? xcd_group_log_for<G>() : -1;
    hipLaunchKernelGGL((spinner_tile_kernel<float, G, NT, 3, true, EPI_STORE_SIGNBITS, SIGNS, PRUNE>),
                       dim3((unsigned)blocks), dim3(G::THREADS), 0, stream, q);
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

// out[i][j] = 1 - popcount(a_i xor b_j) / m.  With the code bits as 0 / 1 numbers,
//     popcount(a xor b) = |a| + |b| - 2 <a, b>,
// and the table of inner products <a_i, b_j> is a dense contraction over the m code bits: it runs on the matrix
// pipe in the narrowest format that holds 0 and 1, fp4 (E2M1, 0x2 = 1.0; v_mfma_scale_f32_32x32x64_f8f6f4 with
// unit scales; products and fp32 sums of at most 2^24 ones: exact).  A workgroup of four waves owns 128 x 128 pairs
// (each wave 64 x 64 = 2 x 2 tiles) and walks the code words in chunks of 16 staged in LDS (rows padded by one
// word: the 2 x 32 half words a wave reads at once fall on 64 different banks).  One instruction consumes a whole
// 64-bit code word: lane group g = lane / 32 takes half word g and spreads it into nibbles in registers, dword q
// holding bits q, q + 4, .., q + 28 (each moved to bit 1 of its nibble).  Which bit lands in which of the 64
// k-slots does not matter, as long as both operands are spread the same way.  The row weights |a_i|, |b_j| are
// counted on the way (v_bcnt, each lane group its half), |a_i| goes through LDS to the lanes that hold row i of
// the result.  (Bits as +1 / -1, which need no weights, take one more instruction per dword to spread: slower.)
typedef int intx8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
constexpr int kGramRows = 128, kGramCols = 128, kGramChunk = 16;

// the 32 bits of w as 32 fp4 numbers (0 or 1.0) in four dwords
__device__ __forceinline__ intx8 spread_bits_fp4(unsigned w)
{
    intx8 f = {0, 0, 0, 0, 0, 0, 0, 0};
    f[0] = (int)((w << 1) & 0x22222222u);
    f[1] = (int)(w & 0x22222222u);
    f[2] = (int)((w >> 1) & 0x22222222u);
    f[3] = (int)((w >> 2) & 0x22222222u);
    return f;
}

__global__ void __launch_bounds__(256) hamming_gram_kernel(const unsigned long long* __restrict__ a, long long na,
                                                           const unsigned long long* __restrict__ b, long long nb,
                                                           int words, float inv_m, float* __restrict__ out)
{
    __shared__ unsigned long long sa[kGramRows][kGramChunk + 1];
    __shared__ unsigned long long sb[kGramCols][kGramChunk + 1];
    __shared__ int weight_a[kGramRows];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wr = wave >> 1, wc = wave & 1, g = lane >> 5, l32 = lane & 31;
    const long long i0 = (long long)blockIdx.y * kGramRows, j0 = (long long)blockIdx.x * kGramCols;
    floatx16 acc[2][2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][u][v] = 0.0f;
    int wa[2] = {0, 0}, wb[2] = {0, 0};
    const int one = 0x7f7f7f7f;                      // scale exponents (E8M0): 2^0
    // this lane's half words: row (.. + l32) of each tile, 32-bit half g of word k
    const unsigned* ha[2];
    const unsigned* hb[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        ha[t] = reinterpret_cast<const unsigned*>(&sa[wr * 64 + t * 32 + l32][0]) + g;
        hb[t] = reinterpret_cast<const unsigned*>(&sb[wc * 64 + t * 32 + l32][0]) + g;
    }

    // staging: 128 rows x 16 words per operand, 256 threads: 8 words per thread and operand
    const int srow = threadIdx.x >> 4, scol = threadIdx.x & 15;
    for (int k0 = 0; k0 < words; k0 += kGramChunk) {
        unsigned long long pa[8], pb[8];
        const bool in_k = k0 + scol < words;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            pa[t] = (in_k && i0 + t * 16 + srow < na) ? a[(i0 + t * 16 + srow) * words + k0 + scol] : 0ull;
            pb[t] = (in_k && j0 + t * 16 + srow < nb) ? b[(j0 + t * 16 + srow) * words + k0 + scol] : 0ull;
        }
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            sa[t * 16 + srow][scol] = pa[t];
            sb[t * 16 + srow][scol] = pb[t];
        }
        __syncthreads();
#pragma unroll 4
        for (int k = 0; k < kGramChunk; ++k) {
            intx8 fa[2], fb[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const unsigned xa = ha[t][2 * k], xb = hb[t][2 * k];
                wa[t] += __popc(xa);
                wb[t] += __popc(xb);
                fa[t] = spread_bits_fp4(xa);
                fb[t] = spread_bits_fp4(xb);
            }
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int u = 0; u < 2; ++u)
                    acc[t][u] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa[t], fb[u], acc[t][u], 4, 4, 0, one, 0, one);
        }
        __syncthreads();
    }
    // a row's weight is the sum of what the two lane groups counted
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        wa[t] += lane_xor_i<32>(wa[t]);
        wb[t] += lane_xor_i<32>(wb[t]);
    }
    if (wc == 0 && g == 0) {
        weight_a[wr * 64 + l32] = wa[0];
        weight_a[wr * 64 + 32 + l32] = wa[1];
    }
    __syncthreads();
    // result register v of lane l holds row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32 of its 32 x 32 tile
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int rl = wr * 64 + t * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                const long long i = i0 + rl, j = j0 + wc * 64 + u * 32 + l32;
                const int dh = weight_a[rl] + wb[u] - 2 * (int)acc[t][u][v];
                if (i < na && j < nb) out[i * nb + j] = 1.0f - (float)dh * inv_m;
            }
}

hipError_t launch_hamming_gram(const unsigned long long* a, long long na, const unsigned long long* b, long long nb, int m,
                               float* out, hipStream_t s)
{
    if (na <= 0 || nb <= 0) return hipSuccess;
    const long long gx = (nb + kGramCols - 1) / kGramCols, gy = (na + kGramRows - 1) / kGramRows;
    if (gx > 0x7fffffffLL || gy > 65535) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(hamming_gram_kernel, dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, s, a, na, b, nb, m / 64,
                       1.0f / (float)m, out);
    return hipGetLastError();
}
}  // namespace spinner
