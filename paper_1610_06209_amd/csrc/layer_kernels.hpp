// Adaptive setting: the HD3HD2HD1 block as a layer with learned diagonals (forward pass that keeps
// the activations entering D2 and D3, and the backward pass).  Built from the same tile geometry,
// butterfly stages and LDS transposes as the projection kernels in spinner_kernels.hpp.
//
// Nothing is normalised on the way: with H_u the +-1 Hadamard matrix,
//   saved1 = H_u D1 x            (= sqrt(n) * b1),
//   saved2 = H_u D2 saved1       (= n * b2),
//   y      = scale n^{-3/2} H_u D3 saved2.
// Backward, with t1 = H_u dy, t2 = H_u D3 t1, t3 = H_u D2 t2 and c = scale n^{-3/2}:
//   dD3 = c sum_b t1 * saved2,  dD2 = c sum_b t2 * saved1,  dD1 = c sum_b t3 * x,  dx = c D1 t3.
#pragma once
#include "layer_params.hpp"
#include "spinner_kernels.hpp"

namespace spinner {
// waves per SIMD that the backward kernel of tiles of several waves, 16 values per thread, is compiled for
constexpr int kLayerBackwardWaves = 3;

// `base` must be readable also for a tile past the end of the batch (the callers pass the first vector then and
// store nothing): loads under a condition end up in a branch each, with waits where the branches join
template <typename G, int LAY>
__device__ __forceinline__ void tile_load(float (&v)[G::R], const ThreadCtx<G>& c, const float* base)
{
    const float* src = base + c.base_index(LAY);
#pragma unroll
    for (int jh = 0; jh < G::R / 4; ++jh) {
        const float4 t = *reinterpret_cast<const float4*>(src + G::reg_index(LAY, jh * 4));
        v[jh * 4] = t.x; v[jh * 4 + 1] = t.y; v[jh * 4 + 2] = t.z; v[jh * 4 + 3] = t.w;
    }
}

template <typename G, int LAY>
__device__ __forceinline__ void tile_store(const float (&v)[G::R], const ThreadCtx<G>& c, float* base, float f)
{
    float* dst = base + c.base_index(LAY);
#pragma unroll
    for (int jh = 0; jh < G::R / 4; ++jh)
        *reinterpret_cast<float4*>(dst + G::reg_index(LAY, jh * 4)) =
            make_float4(v[jh * 4] * f, v[jh * 4 + 1] * f, v[jh * 4 + 2] * f, v[jh * 4 + 3] * f);
}

// acc += g * (tile of `base` in layout LAY)
template <typename G, int LAY>
__device__ __forceinline__ void tile_mac(float (&acc)[G::R], const float (&g)[G::R], const ThreadCtx<G>& c, const float* base)
{
    const float* src = base + c.base_index(LAY);
#pragma unroll
    for (int jh = 0; jh < G::R / 4; ++jh) {
        const float4 t = *reinterpret_cast<const float4*>(src + G::reg_index(LAY, jh * 4));
        acc[jh * 4] = __builtin_fmaf(g[jh * 4], t.x, acc[jh * 4]);
        acc[jh * 4 + 1] = __builtin_fmaf(g[jh * 4 + 1], t.y, acc[jh * 4 + 1]);
        acc[jh * 4 + 2] = __builtin_fmaf(g[jh * 4 + 2], t.z, acc[jh * 4 + 2]);
        acc[jh * 4 + 3] = __builtin_fmaf(g[jh * 4 + 3], t.w, acc[jh * 4 + 3]);
    }
}

// v *= (tile of the diagonal d in layout LAY); GROUPED: all loads are issued before the first product (a scheduling
// barrier keeps them together where the compiler would otherwise wait for each by itself)
template <typename G, int LAY, bool GROUPED>
__device__ __forceinline__ void tile_scale(float (&v)[G::R], const ThreadCtx<G>& c, const float* d)
{
    const float* src = d + c.base_index(LAY);
    float4 t[G::R / 4];
#pragma unroll
    for (int jh = 0; jh < G::R / 4; ++jh) t[jh] = *reinterpret_cast<const float4*>(src + G::reg_index(LAY, jh * 4));
    if constexpr (GROUPED) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int jh = 0; jh < G::R / 4; ++jh) {
        v[jh * 4] *= t[jh].x; v[jh * 4 + 1] *= t[jh].y; v[jh * 4 + 2] *= t[jh].z; v[jh * 4 + 3] *= t[jh].w;
    }
}

// acc += g * t for a tile already in registers
template <int R>
__device__ __forceinline__ void tile_fma(float (&acc)[R], const float (&g)[R], const float (&t)[R])
{
#pragma unroll
    for (int j = 0; j < R; ++j) acc[j] = __builtin_fmaf(g[j], t[j], acc[j]);
}

template <typename G>
__device__ __forceinline__ void layer_ctx(ThreadCtx<G>& c, long long& slot)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    if constexpr (G::WB > 0) {
        slot = blockIdx.x;
        c.lit = lane;
        c.wv = __builtin_amdgcn_readfirstlane(wave);
    } else {
        slot = ((long long)blockIdx.x * G::WAVES + wave) * G::TPW + (lane >> G::LB);
        c.lit = lane & ((1 << G::LB) - 1);
        c.wv = 0;
    }
#pragma unroll
    for (int b = 0; b < 6; ++b) c.sg[b] = ((c.lit >> b) & 1) ? -1.0f : 1.0f;
}

// One vector per tile.  The held values carry the tracked lane sign after an odd number of
// transforms (see lane_stage_fmac_dpp); it is folded into the factors of what is stored.
template <typename G>
__global__ void __launch_bounds__(G::THREADS) layer_forward_kernel(LayerForwardParams p)
{
    constexpr int NT = G::NT;
    constexpr int n = 1 << NT;
    ThreadCtx<G> c;
    long long vec;
    layer_ctx(c, vec);
    const bool active = vec < p.batch;
    const long long off = (active ? vec : 0) * (long long)n;
    __shared__ float4 lds_store[G::LDS_FLOAT4];
    float4* lds = lds_store;
    const float sgn = tracked_sign<G, 0, float>(c);

    float v[G::R];
    tile_load<G, G::layout_after(0)>(v, c, p.x + off);
    spinner_step<G, NT, 0, G::layout_after(0), true, true, false, false>(v, c, p.d[0], nullptr, 0, lds);
    if (active) tile_store<G, G::layout_after(1)>(v, c, p.saved1 + off, sgn);
    spinner_step<G, NT, 0, G::layout_after(1), true, false, true, false>(v, c, p.d[1], nullptr, 0, lds);
    if (active) tile_store<G, G::layout_after(2)>(v, c, p.saved2 + off, 1.0f);
    spinner_step<G, NT, 0, G::layout_after(2), true, false, false, false>(v, c, p.d[2], nullptr, 0, lds);
    if (active) tile_store<G, G::layout_after(3)>(v, c, p.y + off, p.factor * sgn);
}

// Slot s (one tile position of one workgroup) handles vectors s, s + slots, s + 2 slots, ... and
// keeps its three per-coordinate sums in registers; they are written once at the end.
template <typename G>
__global__ void __launch_bounds__(G::THREADS) __attribute__((amdgpu_waves_per_eu((G::R == 16 && G::WB > 0) ? kLayerBackwardWaves : (G::R == 32 ? 2 : 1))))
layer_backward_kernel(LayerBackwardParams p)
{
    constexpr int NT = G::NT;
    constexpr int n = 1 << NT;
    constexpr int R = G::R;
    constexpr int L1 = G::layout_after(1), L2 = G::layout_after(2), L3 = G::layout_after(3);
    // with 32 values per thread the loads of a diagonal are issued together, ahead of its products
    constexpr bool GROUPED_DIAG = R >= 32;
    // (tiles of several waves, n = 2^11 .. 2^14: measured -7 % at n = 2^12, -29 % at 2^13, -20 % at 2^14; with fewer
    // values per thread nothing is gained, with 16 on one wave the registers for it are not there)
    constexpr bool PREFETCH = (R == 16 || R == 32) && G::WB > 0;
    ThreadCtx<G> c;
    long long slot;
    layer_ctx(c, slot);
    __shared__ float4 lds_store[G::LDS_FLOAT4];
    float4* lds = lds_store;
    const float sgn = tracked_sign<G, 0, float>(c);

    float acc1[R], acc2[R], acc3[R];
#pragma unroll
    for (int j = 0; j < R; ++j) { acc1[j] = 0.f; acc2[j] = 0.f; acc3[j] = 0.f; }

    // every wave of a workgroup runs the same number of rounds (the barriers inside the steps need that)
    const long long first = G::WB > 0 ? (long long)blockIdx.x : (long long)blockIdx.x * G::TILES_PER_WG;
    for (long long base = first; base < p.batch; base += p.slots) {
        const long long vec = base + (slot - first);
        const bool active = vec < p.batch;
        const long long off = (active ? vec : 0) * (long long)n;
        float g[R];
        tile_load<G, G::layout_after(0)>(g, c, p.dy + off);
        if constexpr (PREFETCH) {
            // each saved tile is asked for one transform ahead of its use (the scheduling barriers keep the loads
            // where they are written: left alone, the compiler moves each next to its use to save registers)
            float ta[R];
            tile_load<G, L1>(ta, c, p.saved2 + off);
            __builtin_amdgcn_sched_barrier(0);
            spinner_step<G, NT, 0, G::layout_after(0), false, true, false, false>(g, c, nullptr, nullptr, 0, lds);
            if (active) tile_fma<R>(acc3, g, ta);
            tile_load<G, L2>(ta, c, p.saved1 + off);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (GROUPED_DIAG) {
                tile_scale<G, L1, true>(g, c, p.d[2]);
                spinner_step<G, NT, 0, L1, false, false, true, false>(g, c, nullptr, nullptr, 0, lds);
            } else {
                spinner_step<G, NT, 0, L1, true, false, true, false>(g, c, p.d[2], nullptr, 0, lds);
            }
            if (active) tile_fma<R>(acc2, g, ta);
            tile_load<G, L3>(ta, c, p.x + off);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (GROUPED_DIAG) {
                tile_scale<G, L2, true>(g, c, p.d[1]);
                spinner_step<G, NT, 0, L2, false, false, false, false>(g, c, nullptr, nullptr, 0, lds);
            } else {
                spinner_step<G, NT, 0, L2, true, false, false, false>(g, c, p.d[1], nullptr, 0, lds);
            }
            if (active) tile_fma<R>(acc1, g, ta);
        } else {
            spinner_step<G, NT, 0, G::layout_after(0), false, true, false, false>(g, c, nullptr, nullptr, 0, lds);
            if (active) tile_mac<G, L1>(acc3, g, c, p.saved2 + off);
            spinner_step<G, NT, 0, L1, true, false, true, false>(g, c, p.d[2], nullptr, 0, lds);
            if (active) tile_mac<G, L2>(acc2, g, c, p.saved1 + off);
            spinner_step<G, NT, 0, L2, true, false, false, false>(g, c, p.d[1], nullptr, 0, lds);
            if (active) tile_mac<G, L3>(acc1, g, c, p.x + off);
        }
        if (active) {
            // dx = factor * D1 t3
            const float* d1 = p.d[0] + c.base_index(L3);
            float* dst = p.dx + off + c.base_index(L3);
            const float f = p.factor * sgn;
            if constexpr (R >= 32) {
                // all of D1's entries are asked for before the first product is stored: the scheduling barrier keeps the
                // compiler from pairing each load with its store, one load in flight at a time (n = 2^14: 1.305 -> 1.137 ms;
                // with 16 values per thread the pairing measured 3 % faster at n = 2^11 and is left alone)
                float4 t[R / 4];
#pragma unroll
                for (int jh = 0; jh < R / 4; ++jh) t[jh] = *reinterpret_cast<const float4*>(d1 + G::reg_index(L3, jh * 4));
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int jh = 0; jh < R / 4; ++jh)
                    *reinterpret_cast<float4*>(dst + G::reg_index(L3, jh * 4)) =
                        make_float4(g[jh * 4] * f * t[jh].x, g[jh * 4 + 1] * f * t[jh].y, g[jh * 4 + 2] * f * t[jh].z, g[jh * 4 + 3] * f * t[jh].w);
            } else {
#pragma unroll
                for (int jh = 0; jh < R / 4; ++jh) {
                    const float4 t = *reinterpret_cast<const float4*>(d1 + G::reg_index(L3, jh * 4));
                    *reinterpret_cast<float4*>(dst + G::reg_index(L3, jh * 4)) =
                        make_float4(g[jh * 4] * f * t.x, g[jh * 4 + 1] * f * t.y, g[jh * 4 + 2] * f * t.z, g[jh * 4 + 3] * f * t.w);
                }
            }
        }
    }
    if (slot < p.slots) {
        float* part = p.partial + slot * 3LL * n;
        tile_store<G, L3>(acc1, c, part, sgn);            // t3 carries the tracked sign (three transforms)
        tile_store<G, L2>(acc2, c, part + n, 1.0f);       // t2: two transforms
        tile_store<G, L1>(acc3, c, part + 2 * n, sgn);    // t1: one transform
    }
}

}  // namespace spinner
