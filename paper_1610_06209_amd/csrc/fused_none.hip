// Fused three-round kernels, first-m-rows epilogue, n = 2^4 .. 2^16,
// with fp32 diagonals or with packed sign words; for n >= 2^8 also with the last
// round pruned to the rows that are kept (m <= n / 16).
#include "launch.hpp"
namespace spinner {
// whole: every tile lies inside the kept rows and output rows are 16-byte aligned: kernels without row-limit tests
#define CASE(NT) case NT: return signs ? (whole ? launch_tile<float, NT, NT, 3, true, EPI_STORE_NONE, true, 0, false>(p, tiles, s)  \
                                                : launch_tile<float, NT, NT, 3, true, EPI_STORE_NONE, true>(p, tiles, s))            \
                                       : (whole ? launch_tile<float, NT, NT, 3, true, EPI_STORE_NONE, false, 0, false>(p, tiles, s) \
                                                : launch_tile<float, NT, NT, 3, true, EPI_STORE_NONE, false>(p, tiles, s));
#define PCASE(NT) case NT: return signs ? launch_tile<float, NT, NT, 3, true, EPI_STORE_NONE, true, kPruneBits>(p, tiles, s) \
                                        : launch_tile<float, NT, NT, 3, true, EPI_STORE_NONE, false, kPruneBits>(p, tiles, s);
hipError_t launch_fused_none(int log2n, bool signs, int prune, const TileParams& p, long long tiles, hipStream_t s)
{
    const bool whole = p.m == (1 << log2n) && (p.out_stride & 3) == 0;
    if (prune >= kPruneBits) {
        switch (log2n) {
            PCASE(8) PCASE(9) PCASE(10) PCASE(11) PCASE(12) PCASE(13) PCASE(14) PCASE(15) PCASE(16)
        default: break;
        }
    }
    switch (log2n) {
        CASE(4) CASE(5) CASE(6) CASE(7) CASE(8) CASE(9) CASE(10) CASE(11) CASE(12) CASE(13) CASE(14)
        // 2^15: the kernel without row-limit tests measured 1 % faster with sign words and 4 % slower with fp32 diagonals
        case 15: return signs ? (whole ? launch_tile<float, 15, 15, 3, true, EPI_STORE_NONE, true, 0, false>(p, tiles, s)
                                       : launch_tile<float, 15, 15, 3, true, EPI_STORE_NONE, true>(p, tiles, s))
                              : launch_tile<float, 15, 15, 3, true, EPI_STORE_NONE, false>(p, tiles, s);
        CASE(16)
    default: return hipErrorInvalidValue;
    }
}
#undef CASE
#undef PCASE

// Lane masks of the sign flips in layout 1 of the wide geometries (n = 2^12 .. 2^14), behind the other words of
// each triple: word (wave << r) | register of diagonal k has, in bit l, the sign of the entry that lane l of that
// wave holds in that register.  One thread per word.
template <typename G>
__global__ void __launch_bounds__(256) pack_wide_words_kernel(const float* __restrict__ diag, unsigned long long* __restrict__ out,
                                                              long long triple_words, long long offset)
{
    static_assert(G::WIDE, "layout 1 of a wide geometry");
    constexpr int W = (1 << G::NT) / 64;
    const int t = blockIdx.y * 256 + threadIdx.x;       // word within the diagonal
    if (t >= W) return;
    const long long dg = blockIdx.x;                     // 3 * triple + k
    const float* d = diag + (dg << G::NT);
    const int wv = t >> G::r, j = t & (G::R - 1);
    int e0 = G::reg_index(1, j);
    for (int b = 0; b < G::WB; ++b) e0 |= ((wv >> b) & 1) << G::wave_pos(1, b);
    unsigned long long m = 0;
    for (int l = 0; l < 64; ++l) {
        const int e = e0 | ((l & 15) << 2) | (((l >> 4) & 1) << G::lane_pos(1, 4)) | (((l >> 5) & 1) << G::lane_pos(1, 5));
        m |= (unsigned long long)(__float_as_uint(d[e]) >> 31) << l;
    }
    out[(dg / 3) * triple_words + offset + (dg % 3) * W + t] = m;
}

template <int NT>
static hipError_t launch_pack_wide_nt(const float* diag_sets, int L, unsigned long long* signs, hipStream_t s)
{
    using G = GeomFrom<WideF32<NT>, NT>;
    constexpr int W = (1 << NT) / 64;
    hipLaunchKernelGGL((pack_wide_words_kernel<G>), dim3((unsigned)(3 * L), (unsigned)((W + 255) / 256)), dim3(256), 0, s, diag_sets,
                       signs, sign_words_per_triple(1 << NT, NT), wide_words_offset(1 << NT, NT));
    return hipGetLastError();
}

hipError_t launch_pack_wide_words(const float* diag_sets, int log2n, int L, unsigned long long* signs, hipStream_t s)
{
    switch (log2n) {
    case 12: return launch_pack_wide_nt<12>(diag_sets, L, signs, s);
    case 13: return launch_pack_wide_nt<13>(diag_sets, L, signs, s);
    case 14: return launch_pack_wide_nt<14>(diag_sets, L, signs, s);
    default: return hipSuccess;
    }
}
}  // namespace spinner
