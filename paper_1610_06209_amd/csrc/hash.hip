// Cross-polytope hash kernels, n = 2^4 .. 2^14.
#include "launch.hpp"
#ifndef SPINNER_HASH_RMAX      // values per thread (log2) of the hash kernels: 32 values leave room for four waves per
                               // SIMD beside the resident copy of x (measured 16 % faster than 64 at n = 1024, L = 16)
#define SPINNER_HASH_RMAX 5
#endif
namespace spinner {
template <int NT, bool SIGNS>
static hipError_t launch_hash_nt(const HashParams& p, hipStream_t s)
{
    using G = TileGeom<NT, clamp_rmax(NT, SPINNER_HASH_RMAX)>;
    const long long blocks = (p.batch + G::TILES_PER_WG - 1) / G::TILES_PER_WG;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((spinner_hash_kernel<G, SIGNS>), dim3((unsigned)blocks), dim3(G::THREADS), 0, s, p);
    return hipGetLastError();
}
#define CASE(NT) case NT: return signs ? launch_hash_nt<NT, true>(p, s) : launch_hash_nt<NT, false>(p, s);
hipError_t launch_hash(int log2n, bool signs, const HashParams& p, hipStream_t s)
{
    switch (log2n) {
        CASE(4) CASE(5) CASE(6) CASE(7) CASE(8) CASE(9) CASE(10) CASE(11) CASE(12) CASE(13) CASE(14)
    default: return hipErrorInvalidValue;
    }
}
#undef CASE
}  // namespace spinner
