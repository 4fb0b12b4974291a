// Fused three-round kernels, cos/sin random-feature epilogue, n = 2^4 .. 2^14.
// The butterflies run in fp64: with w = scale * y of magnitude ~10^2 the rounding
// of 3 log2(n) fp32 stages alone would exceed a 1e-5 relative feature error.
#include "launch.hpp"
namespace spinner {
#define CASE(NT) case NT: return signs ? launch_tile<double, NT, NT, 3, true, EPI_STORE_COSSIN, true>(p, tiles, s) \
                                       : launch_tile<double, NT, NT, 3, true, EPI_STORE_COSSIN, false>(p, tiles, s);
hipError_t launch_fused_cossin(int log2n, bool signs, const TileParams& p, long long tiles, hipStream_t s)
{
    switch (log2n) {
        CASE(4) CASE(5) CASE(6) CASE(7) CASE(8) CASE(9) CASE(10) CASE(11) CASE(12) CASE(13) CASE(14)
    default: return hipErrorInvalidValue;
    }
}
#undef CASE
}  // namespace spinner
