// Cross-polytope hash kernels, n = 2^4 .. 2^14.
#include "launch.hpp"
#include "allreg.hpp"
namespace spinner {
// values per thread (log2) of the hash kernels: 32 values leave room for four waves per SIMD beside the resident
// copy of x (measured 16 % faster than 64 at n = 1024, L = 16)
constexpr int kHashRmax = 5;

template <typename G>
__device__ __forceinline__ void hash_ar_stages(float (&v)[G::R])
{
    static_for<0, G::r>([&](auto q) { reg_stage<q.value>(v); });
}
template <typename G>
__device__ __forceinline__ void hash_ar_shared_lane_stages(float (&v)[G::R], int l)
{
    static_for<G::r, G::LB>([&](auto b) { lane_stage<b.value>(v, ((l >> b.value) & 1) ? -1.0f : 1.0f); });
}
template <typename G>
__device__ __forceinline__ void hash_ar_flip(float (&v)[G::R], const unsigned long long* words)
{
    sign_words_t w = (sign_words_t)words;
#pragma unroll
    for (int j = 0; j < G::R; ++j) flip_by_mask(v[j], w[j]);
}
// v = D x for a diagonal given as lane masks (reads the resident copy, writes the working registers)
template <typename G>
__device__ __forceinline__ void hash_ar_flip_from(float (&v)[G::R], const float (&x)[G::R], const unsigned long long* words)
{
    sign_words_t w = (sign_words_t)words;
#pragma unroll
    for (int j = 0; j < G::R; ++j) asm("v_cndmask_b32_e64 %0, %1, -%1, %2" : "=v"(v[j]) : "v"(x[j]), "s"(w[j]));
}
template <typename G>
__device__ __forceinline__ void hash_ar_a_to_b(float (&v)[G::R], float4* pa, float* pb)
{
#pragma unroll
    for (int k = 0; k < G::R / 4; ++k) pa[k] = make_float4(v[4 * k], v[4 * k + 1], v[4 * k + 2], v[4 * k + 3]);
    wave_lds_fence();
#pragma unroll
    for (int j = 0; j < G::R; ++j) v[j] = pb[j * G::STRIDE];
    wave_lds_fence();
}
template <typename G>
__device__ __forceinline__ void hash_ar_b_to_a(float (&v)[G::R], float4* pa, float* pb)
{
#pragma unroll
    for (int j = 0; j < G::R; ++j) pb[j * G::STRIDE] = v[j];
    wave_lds_fence();
#pragma unroll
    for (int k = 0; k < G::R / 4; ++k) {
        const float4 t = pa[k];
        v[4 * k] = t.x; v[4 * k + 1] = t.y; v[4 * k + 2] = t.z; v[4 * k + 3] = t.w;
    }
    wave_lds_fence();
}

template <typename G>
__global__ void __launch_bounds__(G::THREADS) spinner_hash_ar_kernel(HashParams p)
{
    constexpr int R = G::R, r = G::r, n = 1 << G::NT;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int g = lane >> G::LB, l = lane & (G::LANES - 1);
    const long long vec = ((long long)blockIdx.x * G::WAVES + wave) * G::TPW + g;
    const bool active = vec < p.batch;

    __shared__ float4 lds_store[G::WAVES * G::TPW * G::VEC_WORDS / 4];
    float* w = reinterpret_cast<float*>(lds_store) + (wave * G::TPW + g) * G::VEC_WORDS;
    float4* pa = reinterpret_cast<float4*>(w + l * G::STRIDE + (l >> r) * R);
    float* pb = w + (l & (R - 1)) + ((l >> r) << r) * G::STRIDE + (l >> r) * R;

    // x: coalesced 16-byte loads, then through the buffer into layout A
    float x0[R];
    {
        const float* src = p.x + (active ? vec : 0) * (long long)n;
#pragma unroll
        for (int k = 0; k < R / 4; ++k) {
            const int e = 4 * (k * G::LANES + l);
            const float4 t = *reinterpret_cast<const float4*>(src + e);      // a vector past the end reads the first one (nothing is stored for it)
            *reinterpret_cast<float4*>(w + (e >> r) * G::STRIDE + (e & (R - 1)) + (e >> (2 * r)) * R) = t;
        }
        wave_lds_fence();
#pragma unroll
        for (int k = 0; k < R / 4; ++k) {
            const float4 t = pa[k];
            x0[4 * k] = t.x; x0[4 * k + 1] = t.y; x0[4 * k + 2] = t.z; x0[4 * k + 3] = t.w;
        }
        wave_lds_fence();
    }

    constexpr int W = n / 64 < 4 ? 4 : n / 64;
    for (int t = 0; t < p.L; ++t) {
        const unsigned long long* hw = p.signs + (long long)t * p.triple_words + 3 * W;   // [3][2][R]: diagonal, layout
        float v[R];
        hash_ar_flip_from<G>(v, x0, hw);            // D1 in layout A
        hash_ar_stages<G>(v);
        hash_ar_a_to_b<G>(v, pa, pb);
        hash_ar_stages<G>(v);
        hash_ar_shared_lane_stages<G>(v, l);
        hash_ar_flip<G>(v, hw + 3 * R);             // D2 in layout B
        hash_ar_stages<G>(v);
        hash_ar_b_to_a<G>(v, pa, pb);
        hash_ar_stages<G>(v);
        hash_ar_shared_lane_stages<G>(v, l);
        hash_ar_flip<G>(v, hw + 4 * R);             // D3 in layout A
        hash_ar_stages<G>(v);
        hash_ar_a_to_b<G>(v, pa, pb);
        hash_ar_stages<G>(v);
        hash_ar_shared_lane_stages<G>(v, l);

        // layout B: register j holds element ebase + (j << r); increasing j is increasing index, strict '>' keeps the lowest
        const int ebase = (l & (R - 1)) + ((l >> r) << (2 * r));
        float best = v[0];
        int best_i = ebase;
#pragma unroll
        for (int j = 1; j < R; ++j) {
            const bool take = __builtin_fabsf(v[j]) > __builtin_fabsf(best);
            best = take ? v[j] : best;
            best_i = take ? (ebase + (j << r)) : best_i;
        }
        static_for<0, G::LB>([&](auto b) {
            const float ov = lane_xor<(1 << b.value)>(best);
            const int oi = lane_xor_i<(1 << b.value)>(best_i);
            const float fa = __builtin_fabsf(ov), fb = __builtin_fabsf(best);
            const bool take = (fa > fb) || (fa == fb && oi < best_i);
            best = take ? ov : best;
            best_i = take ? oi : best_i;
        });
        if (active && l == 0) p.out_idx[vec * p.L + t] = best_i + ((best < 0.0f) ? n : 0);
    }
}

// Lane masks of the sign flips in the two layouts above, behind the sign words of each triple:
// word [k][0][j] (layout A): bit l of each vector's lane group = sign of d_k[j + (l << r)];
// word [k][1][j] (layout B): sign of d_k[(l mod 2^r) + (j << r) + ((l >> r) << 2r)].
__global__ void __launch_bounds__(256) pack_hash_words_kernel(const float* __restrict__ diag, unsigned long long* __restrict__ out,
                                                              int log2n, int r, long long triple_words, long long std_words, long long total)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int R = 1 << r, LB = log2n - r;
    const int j = (int)(i % R);
    const int lay = (int)((i / R) % 2);
    const long long dg = i / (2 * R);               // 3 * triple + k
    const float* d = diag + (dg << log2n);
    unsigned long long m = 0;
    for (int l = 0; l < (1 << LB); ++l) {
        const int e = lay == 0 ? j + (l << r) : (l & (R - 1)) + (j << r) + ((l >> r) << (2 * r));
        m |= (unsigned long long)(__float_as_uint(d[e]) >> 31) << l;
    }
    for (int sft = 1 << LB; sft < 64; sft <<= 1) m |= m << sft;     // one copy per vector of the wave
    out[(dg / 3) * triple_words + std_words + ((dg % 3) * 2 + lay) * R + j] = m;
}

hipError_t launch_pack_hash_words(const float* diag_sets, int log2n, int L, unsigned long long* signs, hipStream_t s)
{
    const int r = ar_log2r(log2n);
    if (!r) return hipSuccess;
    const int n = 1 << log2n;
    const long long total = (long long)L * 3 * 2 * (1 << r);
    hipLaunchKernelGGL(pack_hash_words_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, diag_sets, signs, log2n, r,
                       sign_words_per_triple(n, log2n), 3 * sign_words_per_diag(n), total);
    return hipGetLastError();
}

template <int NT, bool SIGNS>
static hipError_t launch_hash_nt(const HashParams& p, hipStream_t s)
{
    if constexpr (SIGNS && hash_ar_log2r(NT) != 0) {
        using GA = HashArGeom<NT, hash_ar_log2r(NT)>;
        const long long blocks = (p.batch + GA::VECS_PER_WG - 1) / GA::VECS_PER_WG;
        if (blocks <= 0) return hipSuccess;
        if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
        hipLaunchKernelGGL((spinner_hash_ar_kernel<GA>), dim3((unsigned)blocks), dim3(GA::THREADS), 0, s, p);
        return hipGetLastError();
    }
    using G = TileGeom<NT, clamp_rmax(NT, kHashRmax)>;
    const long long blocks = (p.batch + G::TILES_PER_WG - 1) / G::TILES_PER_WG;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((spinner_hash_kernel<G, SIGNS>), dim3((unsigned)blocks), dim3(G::THREADS), 0, s, p);
    return hipGetLastError();
}
// n = 2^15, 2^16: a vector fills the registers of a whole workgroup, so no copy of x can stay resident beside the
// working values; each triple is one launch of the fused plain kernel with the bucket as its epilogue (x is read once
// per triple).  p describes one triple; p.out points at its column of the int32 [batch][L] result, p.out_stride = L.
hipError_t launch_hash_tile(int log2n, bool signs, const TileParams& p, long long tiles, hipStream_t s)
{
    switch (log2n) {
    case 15: return signs ? launch_tile<float, 15, 15, 3, true, EPI_STORE_HASH, true>(p, tiles, s)
                          : launch_tile<float, 15, 15, 3, true, EPI_STORE_HASH, false>(p, tiles, s);
    case 16: return signs ? launch_tile<float, 16, 16, 3, true, EPI_STORE_HASH, true>(p, tiles, s)
                          : launch_tile<float, 16, 16, 3, true, EPI_STORE_HASH, false>(p, tiles, s);
    default: return hipErrorInvalidValue;
    }
}

// ------------------------------------------------------------------ buckets of a projection that lies in memory (n > 2^16)
// Above the fused range the projection y is produced by the four-pass schedule; the bucket of each vector is then
// taken from y in two steps.  Step 1: a workgroup scans one chunk of 2^kArgmaxChunkLog coordinates of one vector and
// leaves the chunk's candidate (value, index): largest |y_i|, lowest index on exact ties.  Step 2: one wave per vector
// picks among the candidates by the same rule and writes index + n when the value is negative.
constexpr int kArgmaxChunkLog = 16;

__device__ __forceinline__ void argmax_take(float& best, int& best_i, float ov, int oi)
{
    const float fa = __builtin_fabsf(ov), fb = __builtin_fabsf(best);
    const bool take = (fa > fb) || (fa == fb && oi < best_i);
    best = take ? ov : best;
    best_i = take ? oi : best_i;
}

__global__ void __launch_bounds__(256) hash_argmax_chunks_kernel(const float* __restrict__ y, int log2n, float* __restrict__ cand_val,
                                                                 int* __restrict__ cand_idx)
{
    const int chunks_log = log2n - kArgmaxChunkLog;
    const long long vec = blockIdx.x >> chunks_log;
    const int chunk = blockIdx.x & ((1 << chunks_log) - 1);
    const int first = chunk << kArgmaxChunkLog;
    const float4* src = reinterpret_cast<const float4*>(y + (vec << log2n) + first);
    float best = 0.0f;
    int best_i = 0x7fffffff;
    // a thread meets its coordinates in increasing order, so the strict comparison keeps the lowest index
    for (int q = threadIdx.x; q < (1 << (kArgmaxChunkLog - 2)); q += 256) {
        const float4 t = src[q];
        const int i = first + 4 * q;
        argmax_take(best, best_i, t.x, i);
        argmax_take(best, best_i, t.y, i + 1);
        argmax_take(best, best_i, t.z, i + 2);
        argmax_take(best, best_i, t.w, i + 3);
    }
    static_for<0, 6>([&](auto b) {
        const float ov = lane_xor<(1 << b.value)>(best);
        const int oi = lane_xor_i<(1 << b.value)>(best_i);
        argmax_take(best, best_i, ov, oi);
    });
    __shared__ float red_val[4];
    __shared__ int red_idx[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { red_val[wave] = best; red_idx[wave] = best_i; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) argmax_take(best, best_i, red_val[w], red_idx[w]);
        cand_val[blockIdx.x] = best;
        cand_idx[blockIdx.x] = best_i;
    }
}

__global__ void __launch_bounds__(64) hash_argmax_pick_kernel(const float* __restrict__ cand_val, const int* __restrict__ cand_idx,
                                                              int log2n, int* __restrict__ out_idx, long long out_stride)
{
    const int chunks = 1 << (log2n - kArgmaxChunkLog);
    const long long vec = blockIdx.x;
    float best = 0.0f;
    int best_i = 0x7fffffff;
    for (int k = threadIdx.x; k < chunks; k += 64) argmax_take(best, best_i, cand_val[vec * chunks + k], cand_idx[vec * chunks + k]);
    static_for<0, 6>([&](auto b) {
        const float ov = lane_xor<(1 << b.value)>(best);
        const int oi = lane_xor_i<(1 << b.value)>(best_i);
        argmax_take(best, best_i, ov, oi);
    });
    if (best_i == 0x7fffffff) best_i = 0;      // no coordinate compared at all (NaN input): bucket 0
    if (threadIdx.x == 0) out_idx[vec * out_stride] = best_i + ((best < 0.0f) ? (1 << log2n) : 0);
}

size_t hash_candidates_bytes(int log2n, long long batch)
{
    return log2n > kArgmaxChunkLog ? (size_t)batch * ((size_t)1 << (log2n - kArgmaxChunkLog)) * 8 : 0;
}

// y: fp32 [batch][n]; candidates: hash_candidates_bytes(log2n, batch) bytes of scratch; out_idx[vec * out_stride]
hipError_t launch_hash_argmax(const float* y, int log2n, long long batch, void* candidates, int* out_idx, long long out_stride,
                              hipStream_t s)
{
    if (log2n <= kArgmaxChunkLog) return hipErrorInvalidValue;
    if (batch <= 0) return hipSuccess;
    const long long blocks = batch << (log2n - kArgmaxChunkLog);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    float* cand_val = static_cast<float*>(candidates);
    int* cand_idx = reinterpret_cast<int*>(cand_val + blocks);
    hipLaunchKernelGGL(hash_argmax_chunks_kernel, dim3((unsigned)blocks), dim3(256), 0, s, y, log2n, cand_val, cand_idx);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(hash_argmax_pick_kernel, dim3((unsigned)batch), dim3(64), 0, s, cand_val, cand_idx, log2n, out_idx, out_stride);
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
