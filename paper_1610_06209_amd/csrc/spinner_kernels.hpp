// Device code of the structured spinner y = H D3 H D2 H D1 x for gfx950 (wave64).
//
// One "tile" is 2^NT fp32 elements that live on chip for a whole kernel: a
// complete vector when n <= 2^14 (all three rounds fused, Section 1 / Section 3
// of the paper define the product), or a row / column block of the Kronecker
// view H_{ab} = H_a (x) H_b when n is larger.  Every thread keeps R = 2^r
// elements in registers.  A Walsh-Hadamard transform is a butterfly stage per
// index bit and the stages commute, so each index bit is handled where it is
// cheapest:
//   * bits held by the register index  : plain add/sub between two registers;
//   * bits held by the lane id         : exchange with lane^mask (DPP, LDS
//                                        crossbar swizzle, bpermute) + one FMA;
//   * bits held by the wave id (NT>12) : an LDS transpose swaps them with
//                                        register bits, then register stages.
// The lane id holds index bits 2..7 (in the second layout of a "wide" geometry:
// bits 2..5 and two high bits), so every global and LDS access is a 16-byte-per-
// lane access in runs of 64 (16) lanes, and diagonals are read with the same
// addresses as the data.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace spinner {

// Fixed choices, each the best of a timing sweep on MI355X.
constexpr int kWavesPerWorkgroup = 4;     // waves per workgroup when a tile fits one wave
constexpr int kLaneChunk = 32;            // registers exchanged per batch in the lane stages that cross the LDS crossbar
constexpr int kMaskPrefetch = 16;         // lane masks of the next step's sign flips fetched before the current step's exchange
                                          // (each takes two scalar registers)

typedef float v4f __attribute__((ext_vector_type(4)));

template <bool STREAM>
__device__ __forceinline__ float4 load4(const float* p)
{
    if constexpr (STREAM) {
        const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
        return make_float4(t.x, t.y, t.z, t.w);
    } else {
        return *reinterpret_cast<const float4*>(p);
    }
}
template <bool STREAM>
__device__ __forceinline__ void store4(float* p, float a, float b, float c, float d)
{
    if constexpr (STREAM) {
        v4f t = {a, b, c, d};
        __builtin_nontemporal_store(t, reinterpret_cast<v4f*>(p));
    } else {
        *reinterpret_cast<float4*>(p) = make_float4(a, b, c, d);
    }
}

// ------------------------------------------------------------------ helpers
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// Value of `v` held by lane (id ^ MASK); MASK is a single bit.
template <int MASK>
__device__ __forceinline__ float lane_xor(float v)
{
    const int s = __builtin_bit_cast(int, v);
    int t;
    if constexpr (MASK == 1)        // quad_perm:[1,0,3,2]
        t = __builtin_amdgcn_update_dpp(0, s, 0xB1, 0xF, 0xF, true);
    else if constexpr (MASK == 2)   // quad_perm:[2,3,0,1]
        t = __builtin_amdgcn_update_dpp(0, s, 0x4E, 0xF, 0xF, true);
    else if constexpr (MASK == 8)   // row_ror:8 (rotation by half a 16-lane row)
        t = __builtin_amdgcn_update_dpp(0, s, 0x128, 0xF, 0xF, true);
    else if constexpr (MASK == 4)   // swizzle, bit mode: and=0x1f or=0 xor=4
        t = __builtin_amdgcn_ds_swizzle(s, (4 << 10) | 0x1F);
    else if constexpr (MASK == 16)  // swizzle, bit mode: xor=16
        t = __builtin_amdgcn_ds_swizzle(s, (16 << 10) | 0x1F);
    else {                          // MASK == 32: crosses the 32-lane halves
        static_assert(MASK == 32, "single lane bit expected");
        const int lane = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
        t = __builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, s);
    }
    return __builtin_bit_cast(float, t);
}

template <int MASK>
__device__ __forceinline__ int lane_xor_i(int v)
{
    return __builtin_bit_cast(int, lane_xor<MASK>(__builtin_bit_cast(float, v)));
}

template <int MASK>
__device__ __forceinline__ double lane_xor(double v)
{
    const int lo = lane_xor_i<MASK>(__double2loint(v));
    const int hi = lane_xor_i<MASK>(__double2hiint(v));
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ float fused_mul_add(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ double fused_mul_add(double a, double b, double c) { return __builtin_fma(a, b, c); }

// ------------------------------------------------------------------ geometry
// Which index bit each register / lane / wave bit holds.  Two layouts:
//   layout 0 ("top"): registers hold bits {0,1} and the top r-2 bits
//   layout 1 ("mid"): registers hold bits {0,1} and the r-2 bits just above the
//                     lane bits (only used when a tile spans several waves)
// Lanes hold bits 2 .. 2+LB-1 in both layouts, except with WIDE_ (below).
// MINW_: occupancy (waves per SIMD) the register allocator must allow; 0 leaves it to the knobs above
// TRIPS_: 2 sends the exchanges of a tile of up to 2^14 elements through an LDS buffer of half the tile, in two trips
// WIDE_: the exchange between the layouts also trades lane bits 4, 5 for register bits.  Layout 1 then keeps
//        bits {0,1}, 6, 7 and layout 0's wave bits in registers, layout 0's register bits 2, 3 in lane bits
//        4, 5 and layout 0's next register bits in the wave id (what is left stays where it was).  A transform
//        is then register stages, four lane stages (bits 2..5), the exchange, and register stages again:
//        lane bits 4, 5 never need a cross-lane butterfly.  Accesses stay 16 bytes per lane in runs of 16 lanes.
// START_: layout in which a kernel loads its tile (1: a three-round kernel ends in layout 0, where the lanes
//        hold index bits 2..7 again, which the sign-code epilogue needs)
// CHUNK_: registers exchanged per batch in the lane stages that go through the LDS crossbar (the exchanged copies of one
//        batch are alive at once, so a smaller batch lowers the register count; 0: all registers at once)
template <int NT_, int RMAX = 6, int WAVES_1 = kWavesPerWorkgroup, int MINW_ = 0, int TRIPS_ = 0, int WIDE_ = 0, int START_ = 0,
          int CHUNK_ = kLaneChunk>
struct TileGeom {
    static constexpr int MIN_WAVES = MINW_;
    static constexpr int LANE_CHUNK = CHUNK_;
    static constexpr int NT = NT_;
    static_assert(WAVES_1 == 1 || WAVES_1 == 2 || WAVES_1 == 4 || WAVES_1 == 8, "waves per workgroup");
    static_assert(NT >= 4 && NT <= 16, "tile of 2^4 .. 2^16 elements");
    static_assert(RMAX >= 2 && RMAX <= 7, "4 .. 128 elements per thread");
    static constexpr int r = NT >= RMAX + 2 ? RMAX : NT - 2;
    static constexpr int R = 1 << r;
    static constexpr int LB = (NT - r) < 6 ? (NT - r) : 6;   // lane bits per tile
    static constexpr int WB = NT - r - LB;                   // wave bits per tile
    // one transpose per transform must bring every wave-held bit into a register bit
    static_assert(WB <= r - 2, "too few registers per thread for this many waves per tile");
    static constexpr int TPW = 64 >> LB;                     // tiles per wave
    // the LDS exchange buffer holds the whole tile, or half of it (two trips per transpose)
    // (tiles above 2^14 elements always take two trips: 64 KiB at 2^15, where two tiles share a compute unit, and
    // 128 KiB at 2^16, where one tile fills the registers of a compute unit anyway; four trips through 64 KiB
    // measured 6 % slower there)
    static constexpr int LDS_HALVES = NT_ > 14 ? 2 : ((TRIPS_ == 2 && WB >= 1) ? 2 : 1);
    static constexpr int LDS_FLOAT4 = WB > 0 ? ((1 << NT_) / 4) / LDS_HALVES : 1;
    static constexpr int WAVES = WB ? (1 << WB) : WAVES_1;   // waves per workgroup
    static constexpr int THREADS = 64 * WAVES;
    static constexpr int TILES_PER_WG = WB ? 1 : WAVES * TPW;

    static constexpr bool WIDE = WIDE_ != 0 && LB == 6 && WB >= 1 && (r - 2) >= 2 + WB;
    static constexpr int LANE_STAGES = WIDE ? 4 : LB;        // lane bits that are transformed by lane exchanges
    static constexpr int reg_pos(int lay, int q)
    {
        if (q < 2) return q;
        if (lay == 0) return NT - r + q;
        if (!WIDE) return LB + q;
        return q < 4 + WB ? 4 + q : NT - r + q;
    }
    static constexpr int lane_pos(int lay, int b) { return (WIDE && lay == 1 && b >= 4) ? NT - r + 2 + (b - 4) : 2 + b; }
    static constexpr int wave_pos(int lay, int b) { return lay == 0 ? 2 + LB + b : (WIDE ? NT - r + 4 + b : LB + r + b); }
    static constexpr int reg_index(int lay, int j)
    {
        int e = 0;
        for (int q = 0; q < r; ++q)
            if ((j >> q) & 1) e |= 1 << reg_pos(lay, q);
        return e;
    }
    // "Swapped" state of a tile (see lane_swap_stages): physical register bits 2, 3 hold the index
    // bits of lane bits 4, 5 (positions 6, 7) and the lanes hold the index bits of register bits 2, 3.
    static constexpr bool LANE_SWAPS = WB > 0 && LB == 6 && r >= 4 && !WIDE;
    static constexpr int reg_index_sw(int lay, int j)
    {
        int e = 0;
        for (int q = 0; q < r; ++q)
            if ((j >> q) & 1) e |= 1 << (q == 2 ? 6 : (q == 3 ? 7 : reg_pos(lay, q)));
        return e;
    }
    static constexpr bool is_reg_pos(int lay, int pos)
    {
        for (int q = 0; q < r; ++q)
            if (reg_pos(lay, q) == pos) return true;
        return false;
    }
    // layout in force after `steps` complete (diag, transform) steps
    static constexpr int layout_after(int steps) { return WB ? ((steps + START_) & 1) : 0; }
};

struct TileParams {
    const float* x;           // input, row stride in_stride
    float* out;               // output, row stride out_stride
    const float* d[3];        // diagonals used by step 0, 1, 2 (unused entries may be null)
    const unsigned long long* sw[3];   // packed sign words of the same diagonals (sign-word kernels only)
    int wide_off;             // words from sw[k] to the lane masks of layout 1 of the same diagonal (wide geometries)
    long long batch;
    long long in_stride;
    long long out_stride;
    int tiles_per_vec_log;    // log2(tiles per vector)
    int tb;                   // tile number -> first element: q << tb
    int sl;                   // log2(row stride) of a column tile (ignored for contiguous tiles)
    int m;                    // coordinates kept by the epilogue
    float factor;             // n^{-3/2} * scale (or 1 for an intermediate pass)
    double factor_rev;        // factor / (2 pi), fp64: w in revolutions for the fp64 feature path
    float inv_sqrt_m;         // COSSIN only: 1 / sqrt(number of features of the whole row)
    long long sin_off;        // COSSIN only: distance from a cos entry to its sin entry (m for a single block)
    int xcd_group_log;        // tiles that span several waves: log2 of the run of consecutive tiles an XCD takes (see xcd_tile); -1: none
};

// Workgroups go to the eight XCDs in turn (workgroup b runs on XCD b mod 8).  With tile = b each XCD would touch
// every eighth tile: pieces of one tile size at eight times that stride, so that for tiles of 32 KiB and more the
// address bits that pick a tile's place among its seven neighbours are fixed per XCD.  Here each XCD takes runs of
// 2^group_log consecutive tiles instead: within a chunk of 8 * 2^group_log tiles, XCD k walks tiles
// [k 2^group_log, (k + 1) 2^group_log).  Tiles beyond the last whole chunk keep tile = b.  group_log < 0: tile = b.
__device__ __forceinline__ long long xcd_tile(unsigned b, long long total, int group_log)
{
    if (group_log < 0) return b;
    const long long chunk = 8LL << group_log;
    const long long whole = total - total % chunk;
    if (b >= whole) return b;
    const long long cidx = b / chunk, r = b % chunk;
    return cidx * chunk + ((r & 7) << group_log) + (r >> 3);
}

enum { EPI_STORE_NONE = 0, EPI_STORE_COSSIN = 1, EPI_STORE_SIGNBITS = 2, EPI_STORE_HASH = 3 };

// Position of tile element e inside its vector, relative to the tile's base:
// the low C bits are contiguous, the rest walks rows of 2^sl elements.
template <int NT, int C>
__device__ __forceinline__ long long tile_offset(int e, int sl)
{
    if constexpr (C >= NT) {
        return e;
    } else {
        return (long long)(e & ((1 << C) - 1)) + ((long long)(e >> C) << sl);
    }
}

// ------------------------------------------------------------------ per-thread state
template <typename G>
struct ThreadCtx {
    int lit;        // lane within tile
    int wv;         // wave bits of the tile index held by this thread
    int wide_off = 0;   // wide geometries: words from a diagonal's sign words to its lane masks of layout 1
    float sg[6];    // +1 / -1 by lane bit: sign of the own value in a lane butterfly
    __device__ __forceinline__ int base_index(int lay) const
    {
        int e = lit << 2;
        if constexpr (G::WIDE)
            if (lay == 1) e = ((lit & 15) << 2) | (((lit >> 4) & 1) << G::lane_pos(1, 4)) | (((lit >> 5) & 1) << G::lane_pos(1, 5));
        for (int b = 0; b < G::WB; ++b)
            e |= ((wv >> b) & 1) << G::wave_pos(lay, b);
        return e;
    }
    // the same in the swapped state: lane bits 4, 5 carry the index bits of register bits 2, 3
    __device__ __forceinline__ int base_index_sw(int lay) const
    {
        int e = ((lit & 15) << 2) | (((lit >> 4) & 1) << G::reg_pos(lay, 2)) | (((lit >> 5) & 1) << G::reg_pos(lay, 3));
        for (int b = 0; b < G::WB; ++b)
            e |= ((wv >> b) & 1) << G::wave_pos(lay, b);
        return e;
    }
};

// ------------------------------------------------------------------ butterflies
// RL: number of leading registers that are still needed (all R unless the last round is pruned)
template <int Q, int RL = 0, typename T, int R>
__device__ __forceinline__ void reg_stage(T (&v)[R])
{
#pragma unroll
    for (int j = 0; j < (RL ? RL : R); ++j) {
        if (!(j & (1 << Q))) {
            const T a = v[j], b = v[j | (1 << Q)];
            v[j] = a + b;
            v[j | (1 << Q)] = a - b;
        }
    }
}

// Exact lane butterfly: the lane with the mask bit clear gets own + partner,
// the other one partner - own.
template <int B, int RL = 0, int CHUNK = kLaneChunk, typename T, int RR>
__device__ __forceinline__ void lane_stage(T (&v)[RR], float sign_own)
{
    constexpr int R = RL ? RL : RR;
    // exchange and combine a few registers at a time so that the exchanged copies of
    // only one chunk are alive at once (register pressure decides occupancy here)
    constexpr int CH = (CHUNK > 0 && CHUNK < R) ? CHUNK : R;
#pragma unroll
    for (int j0 = 0; j0 < R; j0 += CH) {
        T t[CH];
#pragma unroll
        for (int j = 0; j < CH; ++j) t[j] = lane_xor<(1 << B)>(v[j0 + j]);
#pragma unroll
        for (int j = 0; j < CH; ++j) v[j0 + j] = fused_mul_add(v[j0 + j], (T)sign_own, t[j]);
        if (CH < R) __builtin_amdgcn_sched_barrier(0);
    }
}

// One-instruction lane butterfly for the masks a DPP control can express
// (xor 1, xor 2 inside a quad, xor 8 inside a row of 16):
//     own <- own + coef * partner          (v_fmac_f32 with a DPP source)
// With coef = +1 on the lower lane and -1 on the upper lane this gives a+b on
// the lower lane and b-a = -(a-b) on the upper one: the upper lane holds the
// NEGATED difference.  Every later stage is linear, so the kernel keeps a
// per-lane sign s (true value = s * held value) instead of fixing it at once:
// in a transform that starts with all s = +1 the coefficients are (+1,-1) and
// it ends with s = prod over these masks of (-1)^bit; the next transform
// starts from that state, uses the negated coefficients (-1,+1) and ends with
// all s = +1 again.  Partners of every other kind of stage (registers, swizzle,
// bpermute, LDS transpose across waves) share the same s, so those stay exact.
// An odd number of transforms leaves s to be folded into the output factor.
// The two wait states a DPP read needs after a VALU write of the same register
// are supplied by the s_nop at the head of each block.
#define SPINNER_FMAC_DPP8(CTRL)                                                             \
    asm volatile("s_nop 1\n\t"                                                              \
                 "v_fmac_f32_dpp %0, %0, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"          \
                 "v_fmac_f32_dpp %1, %1, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"          \
                 "v_fmac_f32_dpp %2, %2, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"          \
                 "v_fmac_f32_dpp %3, %3, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"          \
                 "v_fmac_f32_dpp %4, %4, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"          \
                 "v_fmac_f32_dpp %5, %5, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"          \
                 "v_fmac_f32_dpp %6, %6, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"          \
                 "v_fmac_f32_dpp %7, %7, %8 " CTRL " row_mask:0xf bank_mask:0xf"               \
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7]) \
                 : "v"(coef))

#define SPINNER_FMAC_DPP4(CTRL)                                                             \
    asm volatile("s_nop 1\n\t"                                                              \
                 "v_fmac_f32_dpp %0, %0, %4 " CTRL " row_mask:0xf bank_mask:0xf\n\t"          \
                 "v_fmac_f32_dpp %1, %1, %4 " CTRL " row_mask:0xf bank_mask:0xf\n\t"          \
                 "v_fmac_f32_dpp %2, %2, %4 " CTRL " row_mask:0xf bank_mask:0xf\n\t"          \
                 "v_fmac_f32_dpp %3, %3, %4 " CTRL " row_mask:0xf bank_mask:0xf"               \
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3])                             \
                 : "v"(coef))

template <int MASK>
__device__ __forceinline__ void fmac_dpp_block4(float* a, float coef)
{
    if constexpr (MASK == 1) SPINNER_FMAC_DPP4("quad_perm:[1,0,3,2]");
    else if constexpr (MASK == 2) SPINNER_FMAC_DPP4("quad_perm:[2,3,0,1]");
    else { static_assert(MASK == 8, "mask without a DPP control"); SPINNER_FMAC_DPP4("row_ror:8"); }
}

template <int MASK>
__device__ __forceinline__ void fmac_dpp_block8(float* a, float coef)
{
    if constexpr (MASK == 1) SPINNER_FMAC_DPP8("quad_perm:[1,0,3,2]");
    else if constexpr (MASK == 2) SPINNER_FMAC_DPP8("quad_perm:[2,3,0,1]");
    else { static_assert(MASK == 8, "mask without a DPP control"); SPINNER_FMAC_DPP8("row_ror:8"); }
}

template <typename T, int R>
constexpr bool lane_mask_uses_fmac_dpp(int mask)
{
    return std::is_same<T, float>::value && R >= 8 && (mask == 1 || mask == 2 || mask == 8);
}

template <int B, int RL = 0, int R>
__device__ __forceinline__ void lane_stage_fmac_dpp(float (&v)[R], float coef)
{
    constexpr int N = RL ? RL : R;
    if constexpr (N >= 8) {
#pragma unroll
        for (int j = 0; j < N; j += 8) fmac_dpp_block8<(1 << B)>(&v[j], coef);
    } else {
        static_assert(N == 4, "register groups come in fours");
        fmac_dpp_block4<(1 << B)>(&v[0], coef);
    }
}

// Lane bits 4 and 5 without the LDS crossbar.  v_permlane16_swap exchanges the odd 16-lane rows
// of its first register with the even rows of its second, v_permlane32_swap the upper half of the
// first with the lower half of the second.  Applied to a register pair (a, b) that differs in one
// register bit, either leaves in a and b the two inputs of every butterfly across that lane bit,
// so a plain register stage finishes it.  Afterwards the register bit holds what the lane bit
// held and vice versa ("swapped" state); the next LDS transpose reads the data from there.
typedef unsigned uint2v __attribute__((ext_vector_type(2)));
template <int LANE_BIT>
__device__ __forceinline__ void lane_swap(float& a, float& b)
{
    uint2v t;
    if constexpr (LANE_BIT == 4) t = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    else t = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    a = __uint_as_float(t.x);
    b = __uint_as_float(t.y);
}
template <int LANE_BIT>
__device__ __forceinline__ void lane_swap(double& a, double& b)
{
    float alo = __int_as_float(__double2loint(a)), ahi = __int_as_float(__double2hiint(a));
    float blo = __int_as_float(__double2loint(b)), bhi = __int_as_float(__double2hiint(b));
    lane_swap<LANE_BIT>(alo, blo);
    lane_swap<LANE_BIT>(ahi, bhi);
    a = __hiloint2double(__float_as_int(ahi), __float_as_int(alo));
    b = __hiloint2double(__float_as_int(bhi), __float_as_int(blo));
}
template <int LANE_BIT, int Q, typename T, int R>
__device__ __forceinline__ void lane_swap_stage(T (&v)[R])
{
#pragma unroll
    for (int j = 0; j < R; ++j)
        if (!(j & (1 << Q))) lane_swap<LANE_BIT>(v[j], v[j | (1 << Q)]);
    reg_stage<Q>(v);
}

// All stages of one transform that the current layout can do without moving
// data between waves: register bits and lane bits at index positions >= CB.
// SKIP_WAVE_OWNED: skip register bits that the *other* layout's waves hold
// (those are finished after the transpose instead, so do not do them twice).
// NEGATE selects the coefficient set of the tracked-sign butterflies (true in
// every second transform of a kernel, see lane_stage_fmac_dpp).
template <typename G, int CB, int LAY, bool NEGATE, bool SWAP = false, typename T>
__device__ __forceinline__ void local_stages(T (&v)[G::R], const ThreadCtx<G>& c)
{
    static_assert(!G::WIDE || CB == 0, "wide exchanges are for contiguous tiles");
    static_assert(!SWAP || CB <= G::lane_pos(LAY, 4), "lane swaps: lane bits 4 and 5 must be among the transformed ones");
    static_for<0, G::r>([&](auto q) {
        if constexpr (G::reg_pos(LAY, q.value) >= CB)
            reg_stage<q.value>(v);
    });
    static_for<0, G::LANE_STAGES>([&](auto b) {
        if constexpr (G::lane_pos(LAY, b.value) >= CB && !(SWAP && b.value >= 4)) {
            if constexpr (lane_mask_uses_fmac_dpp<T, G::R>(1 << b.value)) {
                lane_stage_fmac_dpp<b.value>(v, NEGATE ? -c.sg[b.value] : c.sg[b.value]);
            } else {
                lane_stage<b.value, 0, G::LANE_CHUNK>(v, c.sg[b.value]);
            }
        }
    });
    if constexpr (SWAP) {
        lane_swap_stage<4, 2>(v);
        lane_swap_stage<5, 3>(v);
    }
}

// Sign s of the value a lane holds after an odd number of transforms (+1 after
// an even number): the product of sg over the tracked-sign lane masks.
template <typename G, int CB, typename T>
__device__ __forceinline__ float tracked_sign(const ThreadCtx<G>& c)
{
    float s = 1.0f;
    static_for<0, G::LB>([&](auto b) {
        if constexpr (G::lane_pos(0, b.value) >= CB && lane_mask_uses_fmac_dpp<T, G::R>(1 << b.value)) s *= c.sg[b.value];
    });
    return s;
}

// Register stages, in layout LAY, for exactly those index bits that layout
// 1-LAY does not keep in registers (the part of a transform left after a transpose).
template <typename G, int CB, int LAY, typename T>
__device__ __forceinline__ void wave_owned_stages(T (&v)[G::R])
{
    static_for<0, G::r>([&](auto q) {
        constexpr int pos = G::reg_pos(LAY, q.value);
        if constexpr (pos >= CB && !G::is_reg_pos(1 - LAY, pos)) reg_stage<q.value>(v);
    });
}

// Slots of the two-trip exchange of a WIDE geometry: element e goes to slot
//     (e >> 2) ^ (bit P4 of e) << 4 ^ (bit P5 of e) << 5,      P4, P5 = index bits of lane bits 4, 5 in layout 1.
// In layout 0 those two bits are register bits (the xor is known per register: four bases), in layout 1 they
// are lane bits and slot bits 4, 5 are register bits (again four bases, one per value of those register bits).
template <typename G>
constexpr int wide_slot_k(int lay, int rj)
{
    return lay == 0 ? (((rj >> G::lane_pos(1, 4)) & 1) | (((rj >> G::lane_pos(1, 5)) & 1) << 1)) : ((rj >> 6) & 3);
}
template <typename G>
constexpr int wide_slot_off(int lay, int rj) { return lay == 0 ? (rj >> 2) : ((rj >> 2) & ~48); }
template <typename G, int LAY>
__device__ __forceinline__ void wide_slot_bases(const ThreadCtx<G>& c, int ebase, int (&b)[4])
{
    const int x = (c.lit >> 4) & 3;
#pragma unroll
    for (int k = 0; k < 4; ++k) b[k] = LAY == 0 ? ((ebase >> 2) ^ (k << 4)) : ((ebase >> 2) | ((k ^ x) << 4));
}

// ------------------------------------------------------------------ LDS transpose between layouts
// Moves every element from its (wave, lane, register) place in layout FROM to
// its place in the other layout.  Both sides access the LDS as 16 bytes per
// lane with consecutive lanes on consecutive addresses (no bank conflicts).
// RW / RR: how many leading registers are written / read (all of them unless the last
// round is pruned); `reads` is false for a wave that needs nothing from this exchange.
// SW: the data start in the swapped state (lane_swap_stages); they always arrive in the normal one.
template <typename G, int FROM, bool SYNC_BEFORE, int RW = 0, int RR = 0, bool SW = false>
__device__ __forceinline__ void transpose(float (&v)[G::R], const ThreadCtx<G>& c, float4* lds, bool reads = true)
{
    constexpr int TO = 1 - FROM;
    static_assert(!SW || (RW == 0 && RR == 0), "pruned rounds do not use lane swaps");
    constexpr int NW = RW ? RW : G::R, NR = RR ? RR : G::R;
    if constexpr (G::LDS_HALVES == 1) {
        const int ef = SW ? c.base_index_sw(FROM) : c.base_index(FROM);
#pragma unroll
        for (int jh = 0; jh < NW / 4; ++jh) {
            const int e = ef | (SW ? G::reg_index_sw(FROM, jh * 4) : G::reg_index(FROM, jh * 4));
            lds[e >> 2] = make_float4(v[jh * 4], v[jh * 4 + 1], v[jh * 4 + 2], v[jh * 4 + 3]);
        }
        __syncthreads();
        const int et = c.base_index(TO);
        if (reads) {
#pragma unroll
            for (int jh = 0; jh < NR / 4; ++jh) {
                const int e = et | G::reg_index(TO, jh * 4);
                const float4 t = lds[e >> 2];
                v[jh * 4] = t.x; v[jh * 4 + 1] = t.y; v[jh * 4 + 2] = t.z; v[jh * 4 + 3] = t.w;
            }
        }
        __syncthreads();   // buffer free for the next exchange
    } else {
        // Two trips through an LDS buffer of half the tile: trip h moves registers 4k+2h, 4k+2h+1
        // of every thread, i.e. the elements with a given value of index bit 1: 8 bytes per lane,
        // consecutive lanes on consecutive addresses.  Each thread receives exactly the register slots it has just
        // sent, so nothing is overwritten before it is sent.  A smaller footprint lets a CU
        // hold more workgroups, and lets tiles of 2^15 and 2^16 elements fit at all.
        const int ef = SW ? c.base_index_sw(FROM) : c.base_index(FROM);
        const int et = c.base_index(TO);
        if constexpr (G::LDS_HALVES == 2 && G::WIDE) {
            // 8 bytes per lane: in layout 1 lane bits 4, 5 hold high index bits, so the four runs of 16 lanes would
            // fall on the same banks.  Slot bits 4, 5 (index bits 6, 7) are therefore xored with those two high
            // bits: every access of a wave then covers 64 different 8-byte slots of a 512-byte window.
            float2* lds2 = reinterpret_cast<float2*>(lds);
            int bw[4], br[4];
            wide_slot_bases<G, FROM>(c, ef, bw);
            wide_slot_bases<G, TO>(c, et, br);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (h == 1) __syncthreads();
#pragma unroll
                for (int jh = 0; jh < NW / 4; ++jh) {
                    const int rj = G::reg_index(FROM, jh * 4);
                    lds2[bw[wide_slot_k<G>(FROM, rj)] + wide_slot_off<G>(FROM, rj)] = make_float2(v[jh * 4 + 2 * h], v[jh * 4 + 2 * h + 1]);
                }
                __syncthreads();
                if (reads) {
#pragma unroll
                    for (int jh = 0; jh < NR / 4; ++jh) {
                        const int rj = G::reg_index(TO, jh * 4);
                        const float2 t = lds2[br[wide_slot_k<G>(TO, rj)] + wide_slot_off<G>(TO, rj)];
                        v[jh * 4 + 2 * h] = t.x; v[jh * 4 + 2 * h + 1] = t.y;
                    }
                }
            }
        } else {
            static_assert(G::LDS_HALVES == 2, "one or two trips");
            float2* lds2 = reinterpret_cast<float2*>(lds);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (h == 1) __syncthreads();
#pragma unroll
                for (int jh = 0; jh < NW / 4; ++jh) {
                    const int e = ef | (SW ? G::reg_index_sw(FROM, jh * 4) : G::reg_index(FROM, jh * 4));
                    lds2[e >> 2] = make_float2(v[jh * 4 + 2 * h], v[jh * 4 + 2 * h + 1]);
                }
                __syncthreads();
                if (reads) {
#pragma unroll
                    for (int jh = 0; jh < NR / 4; ++jh) {
                        const int e = et | G::reg_index(TO, jh * 4);
                        const float2 t = lds2[e >> 2];
                        v[jh * 4 + 2 * h] = t.x; v[jh * 4 + 2 * h + 1] = t.y;
                    }
                }
            }
        }
        __syncthreads();
    }
}

// fp64 values cross in two trips (low words, then high words) so that the LDS
// footprint stays 4 bytes per element.
template <typename G, int FROM, bool SYNC_BEFORE, bool SW = false>
__device__ __forceinline__ void transpose(double (&v)[G::R], const ThreadCtx<G>& c, float4* lds)
{
    constexpr int TO = 1 - FROM;
    int4* ilds = reinterpret_cast<int4*>(lds);
    const int ef = SW ? c.base_index_sw(FROM) : c.base_index(FROM);
    const int et = c.base_index(TO);
    int lo[G::R];
    if constexpr (SYNC_BEFORE) __syncthreads();
#pragma unroll
    for (int jh = 0; jh < G::R / 4; ++jh) {
        const int e = ef | (SW ? G::reg_index_sw(FROM, jh * 4) : G::reg_index(FROM, jh * 4));
        ilds[e >> 2] = make_int4(__double2loint(v[jh * 4]), __double2loint(v[jh * 4 + 1]),
                                 __double2loint(v[jh * 4 + 2]), __double2loint(v[jh * 4 + 3]));
    }
    __syncthreads();
#pragma unroll
    for (int jh = 0; jh < G::R / 4; ++jh) {
        const int4 t = ilds[(et | G::reg_index(TO, jh * 4)) >> 2];
        lo[jh * 4] = t.x; lo[jh * 4 + 1] = t.y; lo[jh * 4 + 2] = t.z; lo[jh * 4 + 3] = t.w;
    }
    __syncthreads();
#pragma unroll
    for (int jh = 0; jh < G::R / 4; ++jh) {
        const int e = ef | (SW ? G::reg_index_sw(FROM, jh * 4) : G::reg_index(FROM, jh * 4));
        ilds[e >> 2] = make_int4(__double2hiint(v[jh * 4]), __double2hiint(v[jh * 4 + 1]),
                                 __double2hiint(v[jh * 4 + 2]), __double2hiint(v[jh * 4 + 3]));
    }
    __syncthreads();
#pragma unroll
    for (int jh = 0; jh < G::R / 4; ++jh) {
        const int4 t = ilds[(et | G::reg_index(TO, jh * 4)) >> 2];
        v[jh * 4] = __hiloint2double(t.x, lo[jh * 4]);
        v[jh * 4 + 1] = __hiloint2double(t.y, lo[jh * 4 + 1]);
        v[jh * 4 + 2] = __hiloint2double(t.z, lo[jh * 4 + 2]);
        v[jh * 4 + 3] = __hiloint2double(t.w, lo[jh * 4 + 3]);
    }
}

// ------------------------------------------------------------------ diagonal product
template <typename G, int C, int LAY, typename T>
__device__ __forceinline__ void diag_multiply(T (&v)[G::R], const ThreadCtx<G>& c,
                                              const float* dtile, int sl)
{
    constexpr int NT = G::NT;
    const float* base = dtile + tile_offset<NT, C>(c.base_index(LAY), sl);
#pragma unroll
    for (int jh = 0; jh < G::R / 4; ++jh) {
        const float4 t = *reinterpret_cast<const float4*>(base + tile_offset<NT, C>(G::reg_index(LAY, jh * 4), sl));
        v[jh * 4] *= (T)t.x; v[jh * 4 + 1] *= (T)t.y; v[jh * 4 + 2] *= (T)t.z; v[jh * 4 + 3] *= (T)t.w;
    }
}

// ------------------------------------------------------------------ +-1 diagonals as packed sign words
// Packed format of one diagonal (any n; n / 64 words, at least 4): 64-bit words; element e has its
// sign bit at bit (e >> 2) & 63 of word ((e >> 8) << 2) | (e & 3).  Because the
// lane id holds index bits 2..7 (except in layout 1 of a wide geometry and in column tiles), one word is exactly the lane mask "which
// lanes hold a negated element" of one register, so it is fetched with a scalar
// load and applied with one v_cndmask (x or -x by lane mask): no vector memory
// traffic and no registers spent on staging the diagonal.
typedef const __attribute__((address_space(4))) unsigned long long* sign_words_t;

__device__ __forceinline__ void flip_by_mask(float& x, unsigned long long mask)
{
    asm("v_cndmask_b32_e64 %0, %0, -%0, %1" : "+v"(x) : "s"(mask));
}
__device__ __forceinline__ void flip_by_mask(double& x, unsigned long long mask)
{
    int hi = __double2hiint(x);
    asm("v_cndmask_b32_e64 %0, %0, -%0, %1" : "+v"(hi) : "s"(mask));    // the modifier flips bit 31
    x = __hiloint2double(hi, __double2loint(x));
}

// index bits held by the (uniform) wave id in layout LAY
template <typename G, int LAY>
__device__ __forceinline__ int wave_index_bits(const ThreadCtx<G>& c)
{
    int ew = 0;
    for (int b = 0; b < G::WB; ++b) ew |= ((c.wv >> b) & 1) << G::wave_pos(LAY, b);
    return ew;
}

// lane mask "which lanes hold a negated element" of register j in layout LAY
// DIRECT: `w` holds this tile's masks as they are used, word (wave << r) | register (column tiles of the four-pass
// schedule, whose lanes hold no run of the packed format)
template <typename G, int LAY, bool DIRECT = false>
__device__ __forceinline__ unsigned long long sign_mask(sign_words_t w, const ThreadCtx<G>& c, int ew, int j)
{
    if constexpr (DIRECT) {
        return w[(c.wv << G::r) | j];
    } else if constexpr (G::WIDE && LAY == 1) {
        // lanes hold index bits 2..5 and two high bits: no word of the packed format is this register's lane mask;
        // spinner_pack_signs leaves the masks of this layout, word (wave << r) | register, wide_off words further on
        return w[c.wide_off + ((c.wv << G::r) | j)];
    } else {
        const int e = ew | G::reg_index(LAY, j);  // lane bits (2 .. 2+LB-1) are zero here
        unsigned long long m = w[((e >> 8) << 2) | (e & 3)];
        if constexpr (G::LB < 6) {
            // several tiles share the wave: take this register's 2^LB-lane pattern and repeat it
            constexpr int span = 1 << G::LB;
            m = (m >> ((e >> 2) & 63)) & ((1ull << span) - 1ull);
#pragma unroll
            for (int sft = span; sft < 64; sft <<= 1) m |= m << sft;
        }
        return m;
    }
}

// Lane masks of the first N registers, fetched ahead of their use: the scalar loads of a step's masks would
// otherwise start only after the exchange that precedes the step, with nothing to hide their latency behind.
template <int N>
struct SignMasks { unsigned long long m[N > 0 ? N : 1]; };

template <typename G, int LAY, int N, bool DIRECT = false>
__device__ __forceinline__ void fetch_sign_masks(SignMasks<N>& pm, const ThreadCtx<G>& c, const unsigned long long* words)
{
    sign_words_t w = (sign_words_t)words;
    const int ew = wave_index_bits<G, LAY>(c);
#pragma unroll
    for (int j = 0; j < N; ++j) pm.m[j] = sign_mask<G, LAY, DIRECT>(w, c, ew, j);
}

// NPF: the masks of registers 0 .. NPF-1 come from `pm` instead of from memory
template <typename G, int LAY, int NPF = 0, bool DIRECT = false, typename T>
__device__ __forceinline__ void sign_flip(T (&v)[G::R], const ThreadCtx<G>& c, const unsigned long long* words,
                                          const SignMasks<NPF>* pm = nullptr)
{
    sign_words_t w = (sign_words_t)words;
    const int ew = wave_index_bits<G, LAY>(c);
#pragma unroll
    for (int j = 0; j < G::R; ++j) {
        if (j < NPF) flip_by_mask(v[j], pm->m[j]);
        else flip_by_mask(v[j], sign_mask<G, LAY, DIRECT>(w, c, ew, j));
    }
}

// One (diagonal, transform) step starting in layout LAY; it ends in the other
// layout when the tile spans several waves.  Every index bit >= CB is
// transformed exactly once: register and lane bits of LAY before the transpose,
// the bits LAY keeps in the wave id after it.
// NPF > 0: `pm` holds the first NPF lane masks of this step's sign flips unless this is the first step, and, with
// PF_NEXT, receives those of the next step (packed words at next_words) before this step's exchange.
template <typename G, int C, int CB, int LAY, bool HAS_DIAG, bool FIRST_TRANSPOSE, bool NEGATE, bool SIGNS, typename T, int NPF = 0,
          bool PF_NEXT = false>
__device__ __forceinline__ void spinner_step(T (&v)[G::R], const ThreadCtx<G>& c,
                                             const float* dtile, const unsigned long long* words, int sl, float4* lds,
                                             SignMasks<NPF>* pm = nullptr, const unsigned long long* next_words = nullptr)
{
    constexpr bool DIRECT = SIGNS && C < G::NT;      // column tiles bring their lane masks as they are used
    if constexpr (HAS_DIAG) {
        if constexpr (SIGNS) {
            if constexpr (NPF > 0 && !FIRST_TRANSPOSE) sign_flip<G, LAY, NPF, DIRECT>(v, c, words, pm);
            else sign_flip<G, LAY, 0, DIRECT>(v, c, words);
        }
        else diag_multiply<G, C, LAY>(v, c, dtile, sl);
    }
    constexpr bool SWAP = G::LANE_SWAPS && CB <= G::lane_pos(LAY, 4);
    local_stages<G, CB, LAY, NEGATE, SWAP>(v, c);
    if constexpr (NPF > 0 && PF_NEXT) fetch_sign_masks<G, (G::WB > 0 ? 1 - LAY : LAY), NPF, DIRECT>(*pm, c, next_words);
    if constexpr (G::WB > 0) {
        if constexpr (std::is_same<T, float>::value) transpose<G, LAY, !FIRST_TRANSPOSE, 0, 0, SWAP>(v, c, lds);
        else transpose<G, LAY, !FIRST_TRANSPOSE, SWAP>(v, c, lds);
        wave_owned_stages<G, CB, 1 - LAY>(v);
    }
}

// ------------------------------------------------------------------ last round when only m <= n / 2^P outputs are kept
// Rows 0 .. n/2^P - 1 of H_n are (1^T (x) H_{n/2^P}) / sqrt(n): on the P highest index
// bits the last transform only needs the "sum" output of each butterfly.  Where such a
// bit is held by the register index, the stage is a plain add that halves the set of
// live registers (always a leading block, because pruned bits are the highest register
// bits of either layout); where it is held by the wave id, the waves whose bit is 1 have
// nothing left to do after the transpose; where it is held by the lane id nothing is
// saved.  All later stages, the exchange and the store touch live registers only.
template <typename G>
constexpr unsigned prune_positions(int P) { return P > 0 ? (((1u << P) - 1u) << (G::NT - P)) : 0u; }

// live registers in layout lay once the pruned positions in `done` have been reduced
template <typename G>
constexpr int live_regs(int lay, unsigned done)
{
    int rl = G::R;
    for (int q = 0; q < G::r; ++q)
        if ((done >> G::reg_pos(lay, q)) & 1u) rl >>= 1;
    return rl;
}
template <typename G>
constexpr unsigned reg_positions(int lay)
{
    unsigned m = 0;
    for (int q = 0; q < G::r; ++q) m |= 1u << G::reg_pos(lay, q);
    return m;
}
template <typename G>
constexpr unsigned lane_positions(int lay)
{
    unsigned m = 0;
    for (int b = 0; b < G::LB; ++b) m |= 1u << G::lane_pos(lay, b);
    return m;
}
// registers live at the end of a pruned last step that started in layout LAY
template <typename G>
constexpr int pruned_final_regs(int lay, int P)
{
    const unsigned pm = prune_positions<G>(P);
    if (G::WB == 0) return live_regs<G>(lay, pm & reg_positions<G>(lay));
    return live_regs<G>(1 - lay, pm & (reg_positions<G>(lay) | reg_positions<G>(1 - lay)));
}

template <int HALF, typename T, int R>
__device__ __forceinline__ void sum_stage(T (&v)[R])
{
#pragma unroll
    for (int j = 0; j < HALF; ++j) v[j] = v[j] + v[j + HALF];
}

// register stages of layout LAY over positions in `want`: pruned ones (sum only) first,
// from the highest register bit down, then the ordinary ones on what is still live
template <typename G, int LAY, unsigned WANT, unsigned PM, unsigned DONE0, typename T>
__device__ __forceinline__ void pruned_reg_stages(T (&v)[G::R])
{
    static_for<0, G::r>([&](auto qq) {
        constexpr int q = G::r - 1 - qq.value;
        constexpr unsigned bit = 1u << G::reg_pos(LAY, q);
        if constexpr ((WANT & bit) && (PM & bit)) {
            static_assert(live_regs<G>(LAY, DONE0 | (PM & WANT & ~(bit | (bit - 1u)))) == (2 << q), "pruned bits must top the live block");
            sum_stage<(1 << q)>(v);
        }
    });
    constexpr int RL = live_regs<G>(LAY, DONE0 | (PM & WANT));
    static_for<0, G::r>([&](auto q) {
        constexpr unsigned bit = 1u << G::reg_pos(LAY, q.value);
        if constexpr ((WANT & bit) && !(PM & bit) && (1 << q.value) < RL) reg_stage<q.value, RL>(v);
    });
}

// The last (diagonal, transform) step with the P highest index bits pruned.  Returns,
// through wave_live, whether this wave still holds outputs; pruned_final_regs() tells
// how many leading registers do.
template <typename G, int C, int CB, int LAY, bool NEGATE, bool SIGNS, int P, int NPF = 0>
__device__ __forceinline__ void spinner_step_pruned(float (&v)[G::R], const ThreadCtx<G>& c, const float* dtile,
                                                    const unsigned long long* words, int sl, float4* lds,
                                                    bool& wave_live, const SignMasks<NPF>* pm = nullptr)
{
    static_assert(C >= G::NT && CB == 0, "pruning is for whole-vector tiles");
    constexpr unsigned PM = prune_positions<G>(P);
    constexpr unsigned REGS = reg_positions<G>(LAY);
    if constexpr (SIGNS) sign_flip<G, LAY, NPF>(v, c, words, pm);
    else diag_multiply<G, C, LAY>(v, c, dtile, sl);
    pruned_reg_stages<G, LAY, REGS, PM, 0u>(v);
    constexpr unsigned DONE1 = PM & REGS;
    constexpr int RL1 = live_regs<G>(LAY, DONE1);
    static_for<0, G::LANE_STAGES>([&](auto b) {
        if constexpr (lane_mask_uses_fmac_dpp<float, G::R>(1 << b.value))
            lane_stage_fmac_dpp<b.value, RL1>(v, NEGATE ? -c.sg[b.value] : c.sg[b.value]);
        else
            lane_stage<b.value, RL1, G::LANE_CHUNK>(v, c.sg[b.value]);
    });
    wave_live = true;
    if constexpr (G::WB > 0) {
        constexpr int TO = 1 - LAY;
        constexpr unsigned POST = reg_positions<G>(TO) & ~REGS;     // bits that become register bits only now
        constexpr int RL2 = live_regs<G>(TO, DONE1);
        // a thread of the new layout is live iff its wave- and lane-held bits avoid the reduced positions
        wave_live = (c.base_index(TO) & (int)DONE1) == 0;
        transpose<G, LAY, true, RL1, RL2>(v, c, lds, wave_live);
        if (wave_live) pruned_reg_stages<G, TO, POST, PM, DONE1>(v);
    }
}

// ------------------------------------------------------------------ cos / sin of w = y * factor
// fp32 values: plain library sincos of the fp32 product.
__device__ __forceinline__ void feature_sincos(float y, const TileParams&, float lane_factor, float& s, float& c)
{
    sincosf(y * lane_factor, &s, &c);
}
// fp64 values: w / (2 pi) is formed in fp64 and reduced to its fractional part in fp64
// (exact), then the hardware sine / cosine, which take their argument in revolutions,
// evaluate it in fp32.  On reduced arguments they are accurate to 1.2e-7 absolute
// (measured over 4M points), far inside the 1e-5 feature tolerance.
__device__ __forceinline__ void feature_sincos(double y, const TileParams& p, float, float& s, float& c)
{
    const double t = y * p.factor_rev;
    const float fr = (float)__builtin_amdgcn_fract(t);
    s = __builtin_amdgcn_sinf(fr);
    c = __builtin_amdgcn_cosf(fr);
}

// ------------------------------------------------------------------ the tile kernel
// T       arithmetic type of the butterflies (float, or double for the feature map)
// NT      log2(tile elements)
// C       log2(contiguous run) - NT for a contiguous tile, 4 for a column tile
// NSTEPS  number of (diagonal, transform) steps run on chip (1..3)
// FIRST_DIAG  whether step 0 multiplies by p.d[0] first
// EPI     EPI_STORE_NONE, EPI_STORE_COSSIN (applied with p.factor, limit p.m) or EPI_STORE_SIGNBITS
//         (p.out holds 64-bit code words, p.out_stride counts words, p.m is a multiple of 256) or EPI_STORE_HASH
//         (whole-vector tiles; p.out holds int32 buckets, one per vector, p.out_stride apart)
// RAGGED  false: the caller guarantees that every tile lies entirely inside the kept range [0, m) and that output rows
//         are 16-byte aligned (EPI_STORE_NONE only); the kernel then has no per-store row-limit test at all.  With the
//         tests compiled in, the compiler forms their predicates before the rounds and carries them through the
//         whole kernel (dozens of scalar register pairs, spilled to vector-register lanes and read back at the end).
template <typename T, typename G, int C, int NSTEPS, bool FIRST_DIAG, int EPI, bool SIGNS, int PRUNE = 0, bool RAGGED = true>
__global__ void __launch_bounds__(G::THREADS)
__attribute__((amdgpu_waves_per_eu(G::MIN_WAVES > 0 && std::is_same<T, float>::value ? G::MIN_WAVES : 1)))
spinner_tile_kernel(TileParams p)
{
    // packed sign words describe contiguous tiles; the column pass that applies the second diagonal takes lane masks
    // prepared for its layout (see sign_mask)
    static_assert(!SIGNS || C >= G::NT || (NSTEPS == 2 && !FIRST_DIAG && G::WB > 0), "sign words and column tiles");
    // a pass over tiles of longer vectors reads the words of its own tile: one tile per wave
    static_assert(!SIGNS || NSTEPS == 3 || G::LB == 6, "sign words of a pass: a wave holds one tile");
    constexpr int NT = G::NT;
    constexpr int R = G::R;
    constexpr int CB = C >= NT ? 0 : C;          // index bits below CB are not transformed
    // data touched once bypass cache retention: x and out of the fused kernels, and, in the four-pass schedule,
    // x read by the first pass and what the last pass reads and writes (what lies between is read again soon)
    constexpr bool FIRST_PASS = NSTEPS == 1 && FIRST_DIAG && C >= NT, LAST_PASS = NSTEPS == 1 && !FIRST_DIAG && C < NT;
    // (measured on the four-pass schedule: the hint on the first pass alone +2-3 % at n = 2^17 .. 2^20, on the last pass too +0.4 .. 4 %)
    constexpr bool STREAM_LD = NSTEPS == 3 || FIRST_PASS || LAST_PASS;
    constexpr bool STREAM = NSTEPS == 3 || LAST_PASS;

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    ThreadCtx<G> c;
    long long tile;
    if constexpr (G::WB > 0) {
        tile = xcd_tile(blockIdx.x, p.batch << p.tiles_per_vec_log, p.xcd_group_log);
        c.lit = lane;
        c.wv = __builtin_amdgcn_readfirstlane(wave);
    } else if constexpr (SIGNS && NSTEPS < 3) {
        tile = (long long)blockIdx.x * G::WAVES + __builtin_amdgcn_readfirstlane(wave);      // wave-uniform: it places the sign words
        c.lit = lane;
        c.wv = 0;
    } else {
        const long long wg = NSTEPS == 3 ? xcd_tile(blockIdx.x, gridDim.x, p.xcd_group_log) : (long long)blockIdx.x;
        tile = (wg * G::WAVES + wave) * G::TPW + (lane >> G::LB);
        c.lit = lane & ((1 << G::LB) - 1);
        c.wv = 0;
    }
#pragma unroll
    for (int b = 0; b < 6; ++b) c.sg[b] = ((c.lit >> b) & 1) ? -1.0f : 1.0f;
    c.wide_off = p.wide_off;

    const long long total = p.batch << p.tiles_per_vec_log;

    __shared__ float4 lds_store[(std::is_same<T, float>::value || G::WB == 0) ? G::LDS_FLOAT4 : (1 << NT) / 4];
    float4* lds = lds_store;

    {
        const bool active = tile < total;
        long long vec = 0, q = 0;
        if (active) {
            // tiles are numbered vector by vector: consecutive row tiles are consecutive memory, consecutive column
            // tiles read neighbouring segments of the same rows
            if constexpr (NSTEPS == 3) { vec = tile; }      // all three rounds on chip: the tile is a whole vector
            else { vec = tile >> p.tiles_per_vec_log; q = tile - (vec << p.tiles_per_vec_log); }
        }
        const long long tile_first = q << p.tb;      // first element of the tile inside its vector

        T v[R];
        {
            const float* src = p.x + vec * p.in_stride + tile_first + tile_offset<NT, C>(c.base_index(G::layout_after(0)), p.sl);
#pragma unroll
            for (int jh = 0; jh < R / 4; ++jh) {
                // no test of `active` here: a tile past the end reads the first tile of the first vector (vec = q = 0)
                // and stores nothing; loads under a condition end up in a branch each, with waits where they join
                const float4 t = load4<STREAM_LD>(src + tile_offset<NT, C>(G::reg_index(G::layout_after(0), jh * 4), p.sl));
                v[jh * 4] = (T)t.x; v[jh * 4 + 1] = (T)t.y; v[jh * 4 + 2] = (T)t.z; v[jh * 4 + 3] = (T)t.w;
            }
        }

        // lane masks of the next step's sign flips travel in scalar registers across the exchange (see SignMasks)
        // (measured: 1.4 % at n = 2^14, nothing elsewhere; only tiles of several waves with 64 values per thread use it)
        constexpr int NPF = (SIGNS && G::WB > 0 && R == 64) ? kMaskPrefetch : 0;
        SignMasks<NPF> pm;
        // words of this tile's part of the diagonals (tile q of a longer vector: 2^NT / 64 words per tile)
        const unsigned long long* sw0 = p.sw[0];
        const unsigned long long* sw1 = p.sw[1];
        if constexpr (SIGNS && NSTEPS < 3) { sw0 += q << (NT - 6); sw1 += q << (NT - 6); }
        // steps (layout alternates only when a tile spans several waves)
        spinner_step<G, C, CB, G::layout_after(0), FIRST_DIAG, true, false, SIGNS, T, NPF, (NSTEPS > 1)>(v, c, p.d[0] + tile_first, sw0, p.sl, lds, &pm, sw1);
        if constexpr (NSTEPS > 1)
            spinner_step<G, C, CB, G::layout_after(1), true, false, true, SIGNS, T, NPF, (NSTEPS > 2)>(v, c, p.d[1] + tile_first, sw1, p.sl, lds, &pm, p.sw[2]);
        bool wave_live = true;
        if constexpr (NSTEPS > 2) {
            if constexpr (PRUNE > 0)
                spinner_step_pruned<G, C, CB, G::layout_after(2), false, SIGNS, PRUNE, NPF>(v, c, p.d[2] + tile_first, p.sw[2], p.sl, lds, wave_live, &pm);
            else
                spinner_step<G, C, CB, G::layout_after(2), true, false, false, SIGNS, T, NPF, false>(v, c, p.d[2] + tile_first, p.sw[2], p.sl, lds, &pm);
        }
        static_assert(PRUNE == 0 || (NSTEPS == 3 && std::is_same<T, float>::value), "pruning: fused fp32 kernels only");
        constexpr int RF = PRUNE > 0 ? pruned_final_regs<G>(G::layout_after(2), PRUNE) : R;   // registers that hold outputs

        constexpr int LAYF = G::layout_after(NSTEPS);
        const int ebase = c.base_index(LAYF);
        if (active && wave_live) {
            const long long m = p.m;
            // held values carry the tracked lane sign after an odd number of transforms
            float lane_factor = p.factor;
            if constexpr (NSTEPS & 1) lane_factor *= tracked_sign<G, CB, T>(c);
            // whole tile inside the kept range and rows 16-byte aligned: no per-store checks
            // (with a pruned last round, lanes whose pruned bits are set hold nothing to store)
            constexpr bool LANES_PRUNED = PRUNE > 0 && (prune_positions<G>(PRUNE) & lane_positions<G>(LAYF)) != 0;
            static_assert(RAGGED || (EPI == EPI_STORE_NONE && !LANES_PRUNED), "kernels without row-limit tests: plain stores of whole tiles");
            const bool full = !RAGGED || (!LANES_PRUNED && (tile_first + tile_offset<NT, C>((1 << (NT - PRUNE)) - 1, p.sl) < m) &&
                                          ((p.out_stride & 3) == 0));
            float* dst = p.out + vec * p.out_stride;
            if constexpr (EPI == EPI_STORE_NONE) {
                if (full) {
                    float* d0 = dst + tile_first + tile_offset<NT, C>(ebase, p.sl);
        #pragma unroll
                    for (int jh = 0; jh < RF / 4; ++jh) {
                        const float a0 = (float)(v[jh * 4] * (T)lane_factor), a1 = (float)(v[jh * 4 + 1] * (T)lane_factor);
                        const float a2 = (float)(v[jh * 4 + 2] * (T)lane_factor), a3 = (float)(v[jh * 4 + 3] * (T)lane_factor);
                        store4<STREAM>(d0 + tile_offset<NT, C>(G::reg_index(LAYF, jh * 4), p.sl), a0, a1, a2, a3);
                    }
                } else {
        #pragma unroll
                    for (int jh = 0; jh < RF / 4; ++jh) {
                        const long long i = tile_first + tile_offset<NT, C>(ebase | G::reg_index(LAYF, jh * 4), p.sl);
                        const float a0 = (float)(v[jh * 4] * (T)lane_factor), a1 = (float)(v[jh * 4 + 1] * (T)lane_factor);
                        const float a2 = (float)(v[jh * 4 + 2] * (T)lane_factor), a3 = (float)(v[jh * 4 + 3] * (T)lane_factor);
                        if (i + 3 < m && (p.out_stride & 3) == 0) {
                            *reinterpret_cast<float4*>(dst + i) = make_float4(a0, a1, a2, a3);
                        } else {
                            if (i < m) dst[i] = a0;
                            if (i + 1 < m) dst[i + 1] = a1;
                            if (i + 2 < m) dst[i + 2] = a2;
                            if (i + 3 < m) dst[i + 3] = a3;
                        }
                    }
                }
            } else if constexpr (EPI == EPI_STORE_HASH) {
                // Cross-polytope bucket of the whole vector: argmax of |y_i|, lowest index on exact ties, + n when that
                // coordinate is negative.  Per thread, then across the lanes, then across the waves through the
                // exchange buffer (free again: every exchange ends with a barrier).  `active` is uniform over a
                // workgroup whose tile spans several waves, so every wave reaches the barrier below.
                static_assert(C >= NT && NSTEPS == 3 && PRUNE == 0 && std::is_same<T, float>::value && G::WB > 0 && G::LB == 6,
                              "hash epilogue: fused fp32 kernels of tiles that span several waves");
                float best = v[0];
                int best_i = ebase | G::reg_index(LAYF, 0);
#pragma unroll
                for (int j = 1; j < R; ++j) {
                    const int ij = ebase | G::reg_index(LAYF, j);
                    const float fa = __builtin_fabsf(v[j]), fb = __builtin_fabsf(best);
                    const bool take = (fa > fb) || (fa == fb && ij < best_i);
                    best = take ? v[j] : best;
                    best_i = take ? ij : best_i;
                }
                best *= lane_factor;      // positive factor times the tracked lane sign
                static_for<0, 6>([&](auto b) {
                    const float ov = lane_xor<(1 << b.value)>(best);
                    const int oi = lane_xor_i<(1 << b.value)>(best_i);
                    const float fa = __builtin_fabsf(ov), fb = __builtin_fabsf(best);
                    const bool take = (fa > fb) || (fa == fb && oi < best_i);
                    best = take ? ov : best;
                    best_i = take ? oi : best_i;
                });
                float* red_val = reinterpret_cast<float*>(lds);
                int* red_idx = reinterpret_cast<int*>(lds) + G::WAVES;
                if (lane == 0) { red_val[wave] = best; red_idx[wave] = best_i; }
                __syncthreads();
                if (threadIdx.x == 0) {
                    for (int w = 1; w < G::WAVES; ++w) {
                        const float ov = red_val[w];
                        const int oi = red_idx[w];
                        const float fa = __builtin_fabsf(ov), fb = __builtin_fabsf(best);
                        const bool take = (fa > fb) || (fa == fb && oi < best_i);
                        best = take ? ov : best;
                        best_i = take ? oi : best_i;
                    }
                    reinterpret_cast<int*>(p.out)[vec * p.out_stride] = best_i + ((best < 0.0f) ? (1 << NT) : 0);
                }
            } else if constexpr (EPI == EPI_STORE_SIGNBITS) {
                // Code word ((e >> 8) << 2) | (e & 3) holds, in bit (e >> 2) & 63, whether coordinate e
                // is negative.  Lanes hold index bits 2..7, so the wave-wide comparison mask of one
                // register is one whole word; lane j then stores the word of register j.
                static_assert(G::LB == 6 && (!G::WIDE || LAYF == 0) && C >= NT && std::is_same<T, float>::value && RF <= 64,
                              "sign codes: fp32 contiguous tiles with a whole wave per 256 coordinates");
                // The compare is written out with an explicit scalar destination: through the VCC alias
                // (what the compiler would pick) a lane write right behind it reads a stale mask, and
                // inline asm is invisible to the compiler's hazard pass.  Four compares are issued before
                // their lane writes, and the lane writes feed four independent accumulators so that they
                // do not form one long dependent chain.
                static_assert(RF % 4 == 0, "registers come in groups of four");
                int lo4[4] = {0, 0, 0, 0}, hi4[4] = {0, 0, 0, 0};
#pragma unroll
                for (int j0 = 0; j0 < RF; j0 += 4) {
                    unsigned long long mk[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const float yk = (float)v[j0 + k] * lane_factor;
                        asm volatile("v_cmp_gt_f32_e64 %0, 0, %1" : "=s"(mk[k]) : "v"(yk));
                    }
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        asm volatile("v_writelane_b32 %0, %1, %2" : "+v"(lo4[k]) : "s"((int)(unsigned)mk[k]), "n"(j0 + k));
                        asm volatile("v_writelane_b32 %0, %1, %2" : "+v"(hi4[k]) : "s"((int)(unsigned)(mk[k] >> 32)), "n"(j0 + k));
                    }
                }
                const int lo = lo4[0] | lo4[1] | lo4[2] | lo4[3], hi = hi4[0] | hi4[1] | hi4[2] | hi4[3];
                if (lane < RF) {
                    const int wavebits = ebase & ~(63 << 2);
                    const int e = wavebits | (lane & 3) | ((lane >> 2) << G::reg_pos(LAYF, 2));
                    if (tile_first + e < m) {
                        unsigned long long* codes = reinterpret_cast<unsigned long long*>(p.out) + vec * p.out_stride;
                        const long long i = tile_first + e;
                        codes[((i >> 8) << 2) | (i & 3)] = ((unsigned long long)(unsigned)hi << 32) | (unsigned)lo;
                    }
                }
            } else {
                // dst row is [cos block | sin block]; the sin entry of coordinate i sits sin_off floats after its cos entry
                const long long so = p.sin_off;
        #pragma unroll
                for (int jh = 0; jh < RF / 4; ++jh) {
                    const long long i = tile_first + tile_offset<NT, C>(ebase | G::reg_index(LAYF, jh * 4), p.sl);
                    float sn[4], cs[4];
        #pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        feature_sincos(v[jh * 4 + k], p, lane_factor, sn[k], cs[k]);
                        sn[k] *= p.inv_sqrt_m;
                        cs[k] *= p.inv_sqrt_m;
                    }
                    if (full && ((m | so) & 3) == 0) {
                        *reinterpret_cast<float4*>(dst + i) = make_float4(cs[0], cs[1], cs[2], cs[3]);
                        *reinterpret_cast<float4*>(dst + so + i) = make_float4(sn[0], sn[1], sn[2], sn[3]);
                    } else if (i + 3 < m && ((m | so | p.out_stride) & 3) == 0) {
                        *reinterpret_cast<float4*>(dst + i) = make_float4(cs[0], cs[1], cs[2], cs[3]);
                        *reinterpret_cast<float4*>(dst + so + i) = make_float4(sn[0], sn[1], sn[2], sn[3]);
                    } else {
        #pragma unroll
                        for (int k = 0; k < 4; ++k)
                            if (i + k < m) { dst[i + k] = cs[k]; dst[so + i + k] = sn[k]; }
                    }
                }
            }
        }   // active
    }
}

// ------------------------------------------------------------------ cross-polytope hash kernel
// One contiguous tile = one whole vector (n = 2^NT).  x stays in registers while
// L diagonal triples are applied one after the other.
struct HashParams {
    const float* x;
    const float* diag_sets;   // [L][3][n] fp32 diagonals, or null when sign words are used
    const unsigned long long* signs;   // packed sign words of L triples, or null
    long long triple_words;   // 64-bit words from one triple's sign words to the next
    int* out_idx;             // [batch][L]
    long long batch;
    int L;
};

template <typename G, bool SIGNS>
__global__ void __launch_bounds__(G::THREADS)
spinner_hash_kernel(HashParams p)
{
    constexpr int NT = G::NT;
    constexpr int R = G::R;
    constexpr int n = 1 << NT;

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    ThreadCtx<G> c;
    long long vec;
    if constexpr (G::WB > 0) {
        vec = blockIdx.x;
        c.lit = lane;
        c.wv = __builtin_amdgcn_readfirstlane(wave);
    } else {
        vec = ((long long)blockIdx.x * G::WAVES + wave) * G::TPW + (lane >> G::LB);
        c.lit = lane & ((1 << G::LB) - 1);
        c.wv = 0;
    }
#pragma unroll
    for (int b = 0; b < 6; ++b) c.sg[b] = ((c.lit >> b) & 1) ? -1.0f : 1.0f;
    const bool active = vec < p.batch;

    __shared__ float4 lds_store[G::LDS_FLOAT4];
    __shared__ float red_val[G::WB > 0 ? G::WAVES : 1];
    __shared__ int red_idx[G::WB > 0 ? G::WAVES : 1];
    float4* lds = lds_store;

    float x0[R];
    {
        const float* src = p.x + (active ? vec : 0) * (long long)n + c.base_index(0);
#pragma unroll
        for (int jh = 0; jh < R / 4; ++jh) {
            const float4 t = *reinterpret_cast<const float4*>(src + G::reg_index(0, jh * 4));   // a vector past the end reads the first one
            x0[jh * 4] = t.x; x0[jh * 4 + 1] = t.y; x0[jh * 4 + 2] = t.z; x0[jh * 4 + 3] = t.w;
        }
    }

    for (int l = 0; l < p.L; ++l) {
        const float* d = p.diag_sets + (long long)l * 3 * n;
        constexpr int W = n / 64 < 4 ? 4 : n / 64;              // sign words per diagonal
        const unsigned long long* sw = p.signs + (long long)l * p.triple_words;
        float v[R];
#pragma unroll
        for (int j = 0; j < R; ++j) v[j] = x0[j];
        // a fresh triple starts in layout 0 again, so re-sync before reusing the LDS
        if constexpr (G::WB > 0) __syncthreads();
        spinner_step<G, NT, 0, G::layout_after(0), true, true, false, SIGNS>(v, c, d, sw, 0, lds);
        spinner_step<G, NT, 0, G::layout_after(1), true, false, true, SIGNS>(v, c, d + n, sw + W, 0, lds);
        spinner_step<G, NT, 0, G::layout_after(2), true, false, false, SIGNS>(v, c, d + 2 * n, sw + 2 * W, 0, lds);

        constexpr int LAYF = G::layout_after(3);
        const int ebase = c.base_index(LAYF);
        // per-thread candidate: visit registers in increasing index order, strict '>' keeps the lowest index
        float best = v[0];
        int best_i = ebase | G::reg_index(LAYF, 0);
#pragma unroll
        for (int j = 1; j < R; ++j) {
            const bool take = __builtin_fabsf(v[j]) > __builtin_fabsf(best);
            best = take ? v[j] : best;
            best_i = take ? (ebase | G::reg_index(LAYF, j)) : best_i;
        }
        best *= tracked_sign<G, 0, float>(c);     // three transforms: undo the tracked lane sign
        // across the lanes of the tile
        static_for<0, G::LB>([&](auto b) {
            const float ov = lane_xor<(1 << b.value)>(best);
            const int oi = lane_xor_i<(1 << b.value)>(best_i);
            const float fa = __builtin_fabsf(ov), fb = __builtin_fabsf(best);
            const bool take = (fa > fb) || (fa == fb && oi < best_i);
            best = take ? ov : best;
            best_i = take ? oi : best_i;
        });
        if constexpr (G::WB > 0) {
            if (lane == 0) { red_val[wave] = best; red_idx[wave] = best_i; }
            __syncthreads();
            if (active && threadIdx.x == 0) {
                for (int w = 1; w < G::WAVES; ++w) {
                    const float ov = red_val[w];
                    const int oi = red_idx[w];
                    const float fa = __builtin_fabsf(ov), fb = __builtin_fabsf(best);
                    const bool take = (fa > fb) || (fa == fb && oi < best_i);
                    best = take ? ov : best;
                    best_i = take ? oi : best_i;
                }
                p.out_idx[vec * p.L + l] = best_i + ((best < 0.0f) ? n : 0);
            }
        } else {
            if (active && c.lit == 0) p.out_idx[vec * p.L + l] = best_i + ((best < 0.0f) ? n : 0);
        }
    }
}

}  // namespace spinner
