// Fused three-round kernels, first-m-rows epilogue, n = 2^4 .. 2^16,
// with fp32 diagonals or with packed sign words; for n >= 2^8 also with the last
// round pruned to the rows that are kept (m <= n / 16).
#include "launch.hpp"
namespace spinner {
#define CASE(NT) case NT: return signs ? launch_tile<float, NT, NT, 3, true, EPI_STORE_NONE, true>(p, tiles, s) \
                                       : launch_tile<float, NT, NT, 3, true, EPI_STORE_NONE, false>(p, tiles, s);
#define PCASE(NT) case NT: return signs ? launch_tile<float, NT, NT, 3, true, EPI_STORE_NONE, true, kPruneBits>(p, tiles, s) \
                                        : launch_tile<float, NT, NT, 3, true, EPI_STORE_NONE, false, kPruneBits>(p, tiles, s);
hipError_t launch_fused_none(int log2n, bool signs, int prune, const TileParams& p, long long tiles, hipStream_t s)
{
    if (prune >= kPruneBits) {
        switch (log2n) {
            PCASE(8) PCASE(9) PCASE(10) PCASE(11) PCASE(12) PCASE(13) PCASE(14)
        default: break;
        }
    }
    switch (log2n) {
        CASE(4) CASE(5) CASE(6) CASE(7) CASE(8) CASE(9) CASE(10) CASE(11) CASE(12) CASE(13) CASE(14)
        CASE(15) CASE(16)
    default: return hipErrorInvalidValue;
    }
}
#undef CASE
#undef PCASE
}  // namespace spinner
