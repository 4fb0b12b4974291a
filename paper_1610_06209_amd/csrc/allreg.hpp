// Kernels that keep every butterfly between registers (cross-polytope hash, fp64 feature map).
//
// Where the vector ALU is the limit, a butterfly between two registers costs half of one across lanes
// (DPP forms issue at half rate; fp64 values need two lane moves each) and uses no LDS.  These kernels
// therefore keep two layouts of a vector of 2^NT = 2^(r + LB) elements on 2^LB lanes:
//   layout A: register j, lane l hold element j + (l << r)                    (registers = index bits 0 .. r-1)
//   layout B: register j, lane l hold element (l mod 2^r) + (j << r) + ((l >> r) << 2r)   (registers = bits r .. 2r-1)
// and go from one to the other through a wave-private LDS buffer once per transform, so that a transform is
// r register stages, the exchange, r register stages (plus lane stages for the LB - r lane bits both layouts
// share).  Element e sits at word (e >> r) * (2^r + 4) + (e mod 2^r) (+ a skew per group of 2^r lanes and per
// vector): layout A accesses it 16 bytes per lane, layout B 4 bytes per lane with consecutive lanes on
// consecutive words; the padding of 4 words keeps both free of bank conflicts.  No barrier is needed: the buffer
// belongs to one wave, whose LDS accesses only have to be ordered among themselves.
// The lane masks of the sign flips in these layouts are prepared by spinner_pack_signs (pack_hash_words_kernel).
#pragma once
#include "spinner_kernels.hpp"

namespace spinner {

template <int NT_, int r_, int WAVES_ = 4>
struct HashArGeom {
    static constexpr int NT = NT_, r = r_, R = 1 << r_, LB = NT_ - r_, LANES = 1 << LB, TPW = 64 >> LB;
    static_assert(LB >= r && LB <= 6 && r >= 2, "two register layouts must cover all but the shared lane bits");
    static constexpr int WAVES = WAVES_, THREADS = 64 * WAVES, VECS_PER_WG = WAVES * TPW;
    static constexpr int STRIDE = R + 4;
    static constexpr int GROUPS = LANES >> r;                          // runs of 2^r lanes per vector
    static constexpr int VEC_WORDS = LANES * STRIDE + GROUPS * R;      // the skews fit, and vectors of a wave start on different banks
    static_assert((LANES * STRIDE) % 64 == 0 && GROUPS * R * TPW <= 64, "bank layout of the exchange buffer");
    static_assert(WAVES * TPW * VEC_WORDS * 4 <= 65536, "exchange buffers of a workgroup");
};

__device__ __forceinline__ void wave_lds_fence()
{
    // orders this wave's LDS writes before its later LDS reads (the buffer is private to the wave)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Where a thread finds its elements in the wave's exchange buffer `w` (start of its vector's words):
// pa: its 2^r consecutive words in layout A; pb: its first word in layout B, the others STRIDE words apart.
template <typename G>
__device__ __forceinline__ float4* ar_ptr_a(float* w, int l) { return reinterpret_cast<float4*>(w + l * G::STRIDE + (l >> G::r) * G::R); }
template <typename G>
__device__ __forceinline__ float* ar_ptr_b(float* w, int l)
{
    return w + (l & (G::R - 1)) + ((l >> G::r) << G::r) * G::STRIDE + (l >> G::r) * G::R;
}
// word of element e (a multiple of 4) for the 16-byte accesses of coalesced loads
template <typename G>
__device__ __forceinline__ int ar_word_of(int e) { return (e >> G::r) * G::STRIDE + (e & (G::R - 1)) + (e >> (2 * G::r)) * G::R; }
// first element of lane l in layout B; register j adds j << r
template <typename G>
__device__ __forceinline__ int ar_base_b(int l) { return (l & (G::R - 1)) + ((l >> G::r) << (2 * G::r)); }

template <typename G, typename T>
__device__ __forceinline__ void ar_stages(T (&v)[G::R])
{
    static_for<0, G::r>([&](auto q) { reg_stage<q.value>(v); });
}

}  // namespace spinner
