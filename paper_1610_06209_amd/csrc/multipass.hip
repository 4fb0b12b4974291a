// Passes of the four-pass schedule for n above the fused range.  The vector is viewed as a
// 2^R x 2^(N-R) row-major matrix (R = 7 up to n = 2^21, then 8, 9, 10: col_shape_for); H_n = H_rows (x)
// H_cols acts as a transform along rows (contiguous tiles) and along columns
// (tiles of all 2^R rows x 32 or 16 contiguous columns).  Row and column transforms commute and a diagonal is elementwise, so
//   P1: D1, rows   P2: cols, D2, cols   P3: rows, D3, rows   P4: cols, epilogue
// equals H D3 H D2 H D1 with four trips through HBM instead of six.
#include "launch.hpp"
namespace spinner {
#define ROWCASE(NT, STEPS, FD)                                                                                        \
    case NT:                                                                                                          \
        if constexpr (NT >= kRowSignsMinLog) { if (signs) return launch_tile<float, NT, NT, STEPS, FD, EPI_STORE_NONE, true>(p, tiles, s); } \
        else if (signs) return hipErrorInvalidValue;                                                                  \
        return launch_tile<float, NT, NT, STEPS, FD, EPI_STORE_NONE>(p, tiles, s);
hipError_t launch_row_first(int nt, bool signs, const TileParams& p, long long tiles, hipStream_t s)
{
    switch (nt) {
        ROWCASE(5, 1, true) ROWCASE(6, 1, true) ROWCASE(7, 1, true) ROWCASE(8, 1, true) ROWCASE(9, 1, true)
        ROWCASE(10, 1, true) ROWCASE(11, 1, true) ROWCASE(12, 1, true) ROWCASE(13, 1, true) ROWCASE(14, 1, true)
    default: return hipErrorInvalidValue;
    }
}
hipError_t launch_row_middle(int nt, bool signs, const TileParams& p, long long tiles, hipStream_t s)
{
    switch (nt) {
        ROWCASE(5, 2, false) ROWCASE(6, 2, false) ROWCASE(7, 2, false) ROWCASE(8, 2, false) ROWCASE(9, 2, false)
        ROWCASE(10, 2, false) ROWCASE(11, 2, false) ROWCASE(12, 2, false) ROWCASE(13, 2, false) ROWCASE(14, 2, false)
    default: return hipErrorInvalidValue;
    }
}
// rows only, no diagonal (single transforms of the adaptive layer above its fused range)
#define ROWPLAIN(NT) case NT: return launch_tile<float, NT, NT, 1, false, EPI_STORE_NONE>(p, tiles, s);
hipError_t launch_row_plain(int nt, const TileParams& p, long long tiles, hipStream_t s)
{
    switch (nt) {
        ROWPLAIN(5) ROWPLAIN(6) ROWPLAIN(7) ROWPLAIN(8) ROWPLAIN(9) ROWPLAIN(10) ROWPLAIN(11) ROWPLAIN(12) ROWPLAIN(13) ROWPLAIN(14)
    default: return hipErrorInvalidValue;
    }
}
#undef ROWPLAIN
#undef ROWCASE
#define COLCASE(NT, C, STEPS, EPI) if (rows_log + contig_log == NT && contig_log == C) return launch_tile<float, NT, C, STEPS, false, EPI>(p, tiles, s);
#define COLMID(NT, C)                                                                                     \
    if (rows_log + contig_log == NT && contig_log == C)                                                   \
        return signs ? launch_tile<float, NT, C, 2, false, EPI_STORE_NONE, true>(p, tiles, s)             \
                     : launch_tile<float, NT, C, 2, false, EPI_STORE_NONE>(p, tiles, s);
hipError_t launch_col_middle(int rows_log, int contig_log, bool signs, const TileParams& p, long long tiles, hipStream_t s)
{
    COLMID(12, 5) COLMID(13, 5) COLMID(14, 5) COLMID(14, 4)
    return hipErrorInvalidValue;
}
#undef COLMID

// Lane masks of the second diagonal for that pass, one 64-bit word per register of a wave: the tile of columns
// [q 2^C, (q + 1) 2^C) has its 2^NT / 64 words at q 2^NT / 64, word (wave << r) | register, and bit l of a word is
// the sign of the entry that lane l of that wave holds in that register in layout 1, where the pass multiplies.
// One wave per word; the word is the wave's ballot.
template <typename G, int C>
__global__ void __launch_bounds__(256) pack_col_words_kernel(const float* __restrict__ diag_sets, unsigned long long* __restrict__ signs,
                                                             long long n, int sl, long long triple_words, long long offset,
                                                             long long total_words)
{
    static_assert(G::WB > 0 && G::LB == 6 && !G::WIDE && C < G::NT, "column tile held by several waves");
    const long long gw = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (gw >= total_words) return;
    const long long W = n >> 6;
    const long long triple = gw / W, w = gw - triple * W;
    const long long q = w >> (G::NT - 6);
    const int wj = (int)(w & ((1 << (G::NT - 6)) - 1));
    const int wv = wj >> G::r, j = wj & (G::R - 1);
    int e = G::reg_index(1, j) | (lane << 2);
    for (int b = 0; b < G::WB; ++b) e |= ((wv >> b) & 1) << G::wave_pos(1, b);
    const long long idx = (q << C) + tile_offset<G::NT, C>(e, sl);
    const bool neg = (__float_as_uint(diag_sets[(triple * 3 + 1) * n + idx]) >> 31) != 0;
    const unsigned long long m = __ballot(neg);
    if (lane == 0) signs[triple * triple_words + offset + w] = m;
}

#define COLPACK(NT, C)                                                                                                     \
    if (cs.rows_log + cs.contig_log == NT && cs.contig_log == C) {                                                         \
        hipLaunchKernelGGL((pack_col_words_kernel<GeomFor<float, NT>, C>), dim3((unsigned)blocks), dim3(256), 0, s, diag_sets, signs, \
                           n, log2n - cs.rows_log, sign_words_per_triple((int)n, log2n), col_words_offset((int)n, log2n), total); \
        return hipGetLastError();                                                                                          \
    }
hipError_t launch_pack_col_words(const float* diag_sets, int log2n, int L, unsigned long long* signs, hipStream_t s)
{
    const ColShape cs = col_shape_for(log2n);
    const long long n = 1LL << log2n;
    const long long total = (long long)L * (n >> 6);
    const long long blocks = (total + 3) / 4;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    COLPACK(12, 5) COLPACK(13, 5) COLPACK(14, 5) COLPACK(14, 4)
    return hipErrorInvalidValue;
}
#undef COLPACK
hipError_t launch_col_last(int rows_log, int contig_log, int epi, const TileParams& p, long long tiles, hipStream_t s)
{
    if (epi == EPI_STORE_COSSIN) {
        COLCASE(12, 5, 1, EPI_STORE_COSSIN)
        COLCASE(13, 5, 1, EPI_STORE_COSSIN)
    COLCASE(14, 5, 1, EPI_STORE_COSSIN)
        COLCASE(14, 4, 1, EPI_STORE_COSSIN)
        return hipErrorInvalidValue;
    }
    COLCASE(12, 5, 1, EPI_STORE_NONE)
    COLCASE(13, 5, 1, EPI_STORE_NONE)
    COLCASE(14, 5, 1, EPI_STORE_NONE)
    COLCASE(14, 4, 1, EPI_STORE_NONE)
    return hipErrorInvalidValue;
}
#undef COLCASE
}  // namespace spinner
