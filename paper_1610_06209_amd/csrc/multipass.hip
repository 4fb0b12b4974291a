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
#undef ROWCASE
#define COLCASE(NT, C, STEPS, EPI) if (rows_log + contig_log == NT && contig_log == C) return launch_tile<float, NT, C, STEPS, false, EPI>(p, tiles, s);
hipError_t launch_col_middle(int rows_log, int contig_log, const TileParams& p, long long tiles, hipStream_t s)
{
    COLCASE(12, 5, 2, EPI_STORE_NONE)
    COLCASE(13, 5, 2, EPI_STORE_NONE)
    COLCASE(14, 5, 2, EPI_STORE_NONE)
    COLCASE(14, 4, 2, EPI_STORE_NONE)
#ifdef SPINNER_TUNING_HOOKS
    COLCASE(12, 4, 2, EPI_STORE_NONE) COLCASE(12, 6, 2, EPI_STORE_NONE) COLCASE(13, 6, 2, EPI_STORE_NONE)
#endif
    return hipErrorInvalidValue;
}
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
#ifdef SPINNER_TUNING_HOOKS
    COLCASE(12, 4, 1, EPI_STORE_NONE) COLCASE(12, 6, 1, EPI_STORE_NONE) COLCASE(13, 6, 1, EPI_STORE_NONE)
#endif
    return hipErrorInvalidValue;
}
#undef COLCASE
}  // namespace spinner
