// Fused three-round kernels, cos/sin random-feature epilogue, n = 2^4 .. 2^14.
// The butterflies run in fp64: with w = scale * y of magnitude ~10^2 the rounding
// of 3 log2(n) fp32 stages alone would exceed a 1e-5 relative feature error.
#include "launch.hpp"
#include "allreg.hpp"
namespace spinner {

// ------------------------------------------------------------------ feature kernel with every butterfly between registers
// The fp64 feature map is bound by the vector ALU, and a lane butterfly on fp64 values costs two lane moves
// and an addition at half rate.  For the sizes below (n = 2^(2r), one wave per 64 / 2^r vectors, +-1 diagonals
// as lane masks) all 3 * 2r stages are register stages of the two layouts of allreg.hpp; fp64 values cross the
// wave-private exchange buffer in two trips (low words, high words), so the buffer stays 4 bytes per element.
// x arrives through the same buffer after coalesced 16-byte loads; the three exchanges end in layout B, where
// register j of consecutive lanes holds consecutive coordinates: the cos and sin rows are written 4 bytes per
// lane, 64 lanes on 256 consecutive bytes.
template <typename G>
__device__ __forceinline__ void feat_ar_flip(double (&v)[G::R], const unsigned long long* words)
{
    sign_words_t w = (sign_words_t)words;
#pragma unroll
    for (int j = 0; j < G::R; ++j) flip_by_mask(v[j], w[j]);
}

template <typename G>
__device__ __forceinline__ void feat_ar_a_to_b(double (&v)[G::R], float4* pa, float* pb)
{
    int4* ia = reinterpret_cast<int4*>(pa);
    int* ib = reinterpret_cast<int*>(pb);
    int lo[G::R];
#pragma unroll
    for (int k = 0; k < G::R / 4; ++k)
        ia[k] = make_int4(__double2loint(v[4 * k]), __double2loint(v[4 * k + 1]), __double2loint(v[4 * k + 2]), __double2loint(v[4 * k + 3]));
    wave_lds_fence();
#pragma unroll
    for (int j = 0; j < G::R; ++j) lo[j] = ib[j * G::STRIDE];
    wave_lds_fence();
#pragma unroll
    for (int k = 0; k < G::R / 4; ++k)
        ia[k] = make_int4(__double2hiint(v[4 * k]), __double2hiint(v[4 * k + 1]), __double2hiint(v[4 * k + 2]), __double2hiint(v[4 * k + 3]));
    wave_lds_fence();
#pragma unroll
    for (int j = 0; j < G::R; ++j) v[j] = __hiloint2double(ib[j * G::STRIDE], lo[j]);
    wave_lds_fence();
}

template <typename G>
__device__ __forceinline__ void feat_ar_b_to_a(double (&v)[G::R], float4* pa, float* pb)
{
    int4* ia = reinterpret_cast<int4*>(pa);
    int* ib = reinterpret_cast<int*>(pb);
    int lo[G::R];
#pragma unroll
    for (int j = 0; j < G::R; ++j) ib[j * G::STRIDE] = __double2loint(v[j]);
    wave_lds_fence();
#pragma unroll
    for (int k = 0; k < G::R / 4; ++k) {
        const int4 t = ia[k];
        lo[4 * k] = t.x; lo[4 * k + 1] = t.y; lo[4 * k + 2] = t.z; lo[4 * k + 3] = t.w;
    }
    wave_lds_fence();
#pragma unroll
    for (int j = 0; j < G::R; ++j) ib[j * G::STRIDE] = __double2hiint(v[j]);
    wave_lds_fence();
#pragma unroll
    for (int k = 0; k < G::R / 4; ++k) {
        const int4 t = ia[k];
        v[4 * k] = __hiloint2double(t.x, lo[4 * k]);
        v[4 * k + 1] = __hiloint2double(t.y, lo[4 * k + 1]);
        v[4 * k + 2] = __hiloint2double(t.z, lo[4 * k + 2]);
        v[4 * k + 3] = __hiloint2double(t.w, lo[4 * k + 3]);
    }
    wave_lds_fence();
}

// fp32 diagonals for the same kernel.  In layout A a thread's entries are 2^r consecutive floats: the diagonal goes
// through the exchange buffer like x (coalesced 16-byte loads, 16-byte reads in layout A).  In layout B register j of
// consecutive lanes wants consecutive entries: 4-byte loads, 64 lanes on 256 consecutive bytes (the diagonal is
// cache-resident).
template <typename G>
__device__ __forceinline__ void feat_ar_diag_a(double (&v)[G::R], const float* d, float* w, float4* pa, int l)
{
#pragma unroll
    for (int k = 0; k < G::R / 4; ++k)
        *reinterpret_cast<float4*>(w + ar_word_of<G>(4 * (k * G::LANES + l))) = *reinterpret_cast<const float4*>(d + 4 * (k * G::LANES + l));
    wave_lds_fence();
#pragma unroll
    for (int k = 0; k < G::R / 4; ++k) {
        const float4 t = pa[k];
        v[4 * k] *= (double)t.x; v[4 * k + 1] *= (double)t.y; v[4 * k + 2] *= (double)t.z; v[4 * k + 3] *= (double)t.w;
    }
    wave_lds_fence();
}
template <typename G>
__device__ __forceinline__ void feat_ar_diag_b(double (&v)[G::R], const float* d, int ebase)
{
    // a few at a time: with all 2^r entries in flight at once the register allocator runs out
    constexpr int CH = G::R < 16 ? G::R : 16;
#pragma unroll
    for (int j0 = 0; j0 < G::R; j0 += CH) {
        float t[CH];
#pragma unroll
        for (int j = 0; j < CH; ++j) t[j] = d[ebase + ((j0 + j) << G::r)];
#pragma unroll
        for (int j = 0; j < CH; ++j) v[j0 + j] *= (double)t[j];
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <typename G, bool SIGNS>
__global__ void __launch_bounds__(G::THREADS) __attribute__((amdgpu_waves_per_eu(G::r >= 6 ? 2 : 4)))
spinner_feature_ar_kernel(TileParams p)
{
    static_assert(G::LB == G::r, "no lane bit is shared by the two layouts");
    constexpr int R = G::R, r = G::r, n = 1 << G::NT;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int g = lane >> G::LB, l = lane & (G::LANES - 1);
    const long long wvec = ((long long)blockIdx.x * G::WAVES + wave) * G::TPW;     // first vector of this wave (wave-uniform)
    // a wave with no vector at all leaves (the exchange buffer is private to the wave: no barrier waits for it)
    if (wvec >= p.batch) return;

    __shared__ float4 lds_store[G::WAVES * G::TPW * G::VEC_WORDS / 4];
    float* w = reinterpret_cast<float*>(lds_store) + (wave * G::TPW + g) * G::VEC_WORDS;
    float4* pa = ar_ptr_a<G>(w, l);
    float* pb = ar_ptr_b<G>(w, l);
    constexpr int W = n / 64 < 4 ? 4 : n / 64;      // sign words per diagonal
    const unsigned long long* hw = p.sw[0] + 3 * W; // lane masks behind the triple's sign words: [3 diagonals][2 layouts][R]
    const int ebase = ar_base_b<G>(l);              // layout B: register j holds coordinate ebase + (j << r)
    const long long so = p.sin_off;

    {
        const long long vec = wvec + g;
        const bool active = vec < p.batch;
        double v[R];
        // x: coalesced 16-byte loads, then through the buffer into layout A
        const float* src = p.x + (active ? vec : 0) * p.in_stride + 4 * l;
#pragma unroll
        for (int k = 0; k < R / 4; ++k) {
            const float4 t = load4<true>(src + 4 * k * G::LANES);      // a vector past the end reads the first one
            *reinterpret_cast<float4*>(w + ar_word_of<G>(4 * (k * G::LANES + l))) = t;
        }
        wave_lds_fence();
#pragma unroll
        for (int k = 0; k < R / 4; ++k) {
            const float4 t = pa[k];
            v[4 * k] = (double)t.x; v[4 * k + 1] = (double)t.y; v[4 * k + 2] = (double)t.z; v[4 * k + 3] = (double)t.w;
        }
        wave_lds_fence();

        if constexpr (SIGNS) feat_ar_flip<G>(v, hw);                 // D1 in layout A
        else feat_ar_diag_a<G>(v, p.d[0], w, pa, l);
        ar_stages<G>(v);
        feat_ar_a_to_b<G>(v, pa, pb);
        ar_stages<G>(v);
        if constexpr (SIGNS) feat_ar_flip<G>(v, hw + 3 * R);         // D2 in layout B
        else feat_ar_diag_b<G>(v, p.d[1], ebase);
        ar_stages<G>(v);
        feat_ar_b_to_a<G>(v, pa, pb);
        ar_stages<G>(v);
        if constexpr (SIGNS) feat_ar_flip<G>(v, hw + 4 * R);         // D3 in layout A
        else feat_ar_diag_a<G>(v, p.d[2], w, pa, l);
        ar_stages<G>(v);
        feat_ar_a_to_b<G>(v, pa, pb);
        ar_stages<G>(v);

        float* dst = p.out + (active ? vec : 0) * p.out_stride + ebase;
        if (p.m == n) {                         // every coordinate is kept: straight-line stores
#pragma unroll
            for (int j = 0; j < R; ++j) {
                float sn, cs;
                feature_sincos(v[j], p, 0.0f, sn, cs);
                if (G::TPW == 1 || active) {
                    __builtin_nontemporal_store(cs * p.inv_sqrt_m, dst + (j << r));
                    __builtin_nontemporal_store(sn * p.inv_sqrt_m, dst + so + (j << r));
                }
            }
        } else {
            const int m = active ? p.m : 0;
#pragma unroll
            for (int j = 0; j < R; ++j) {
                float sn, cs;
                feature_sincos(v[j], p, 0.0f, sn, cs);
                if (ebase + (j << r) < m) {
                    __builtin_nontemporal_store(cs * p.inv_sqrt_m, dst + (j << r));
                    __builtin_nontemporal_store(sn * p.inv_sqrt_m, dst + so + (j << r));
                }
            }
        }
    }
}

// one wave per workgroup (each wave owns its vectors and its exchange buffer): measured 3-4 % faster than two
constexpr int kFeatureArWaves = 1;
template <int NT, bool SIGNS>
static hipError_t launch_cossin(const TileParams& p, long long tiles, hipStream_t s)
{
    if constexpr (feature_ar_log2r(NT) != 0) {
        using GA = HashArGeom<NT, feature_ar_log2r(NT), kFeatureArWaves>;
        const long long blocks = (tiles + GA::VECS_PER_WG - 1) / GA::VECS_PER_WG;
        if (blocks <= 0) return hipSuccess;
        if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
        hipLaunchKernelGGL((spinner_feature_ar_kernel<GA, SIGNS>), dim3((unsigned)blocks), dim3(GA::THREADS), 0, s, p);
        return hipGetLastError();
    }
    return launch_tile<double, NT, NT, 3, true, EPI_STORE_COSSIN, SIGNS>(p, tiles, s);
}

#define CASE(NT) case NT: return signs ? launch_cossin<NT, true>(p, tiles, s) : launch_cossin<NT, false>(p, tiles, s);
hipError_t launch_fused_cossin(int log2n, bool signs, const TileParams& p, long long tiles, hipStream_t s)
{
    switch (log2n) {
        CASE(4) CASE(5) CASE(6) CASE(7) CASE(8) CASE(9) CASE(10) CASE(11) CASE(12) CASE(13) CASE(14)
    default: return hipErrorInvalidValue;
    }
}
#undef CASE
}  // namespace spinner
