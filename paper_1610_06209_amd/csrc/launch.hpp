// Host-side launch helpers shared by the translation units that instantiate
// the kernels (split only to compile them in parallel).
#pragma once
#include "spinner_kernels.hpp"

namespace spinner {

constexpr int clamp_rmax(int nt, int want) { return (nt - 3) / 2 > want ? (nt - 3) / 2 : want; }

// largest n (log2) that a single fused kernel handles, per epilogue / entry point
constexpr int kFusedMaxLogPlain = 16;     // fp32 butterflies, first-m-rows epilogue
constexpr int kFusedMaxLogOther = 14;     // fp64 feature map, hash

// Registers per thread (2^rmax values) and waves per workgroup for each tile
// size, from timing sweeps on MI355X: fewer registers per thread buy occupancy
// (more waves to hide HBM latency) at the price of more lane / LDS stages.
// fp64 butterflies keep 32 values per thread (64 registers), 16 at n = 2^12.
struct NotWide { static constexpr int wide = 0, start = 0, chunk = kLaneChunk; };
template <typename T, int NT> struct Tuning : NotWide { static constexpr int rmax = std::is_same<T, double>::value ? clamp_rmax(NT, 5) : 6, waves = 4, min_waves = 0, trips = 0; };
template <> struct Tuning<double, 12> : NotWide { static constexpr int rmax = 4, waves = 4, min_waves = 0, trips = 0; };
template <> struct Tuning<float, 4> : NotWide { static constexpr int rmax = 2, waves = 4, min_waves = 0, trips = 0; };
template <> struct Tuning<float, 5> : NotWide { static constexpr int rmax = 2, waves = 4, min_waves = 0, trips = 0; };
template <> struct Tuning<float, 6> : NotWide { static constexpr int rmax = 3, waves = 4, min_waves = 0, trips = 0; };
template <> struct Tuning<float, 7> : NotWide { static constexpr int rmax = 3, waves = 4, min_waves = 0, trips = 0; };
template <> struct Tuning<float, 8> : NotWide { static constexpr int rmax = 3, waves = 4, min_waves = 0, trips = 0; };
template <> struct Tuning<float, 9> : NotWide { static constexpr int rmax = 3, waves = 4, min_waves = 0, trips = 0; };
template <> struct Tuning<float, 10> : NotWide { static constexpr int rmax = 4, waves = 4, min_waves = 0, trips = 0; };
template <> struct Tuning<float, 11> : NotWide { static constexpr int rmax = 6, waves = 1, min_waves = 0, trips = 0; };
template <> struct Tuning<float, 12> : NotWide { static constexpr int rmax = 4, waves = 4, min_waves = 0, trips = 0; };   // 4 waves per tile, 16 KiB LDS
template <> struct Tuning<float, 13> : NotWide { static constexpr int rmax = 5, waves = 4, min_waves = 0, trips = 0; };
// n = 2^14: four waves of 64 values per tile, held to 128 registers, exchanging through half-size LDS buffers:
// four tiles share a compute unit (two with 32 values on eight waves and a whole-tile buffer); measured +5 %
template <> struct Tuning<float, 14> : NotWide { static constexpr int rmax = 6, waves = 4, min_waves = 4, trips = 2; };
template <> struct Tuning<float, 15> : NotWide { static constexpr int rmax = 6, waves = 4, min_waves = 4, trips = 0; };   // 8 waves per tile; 128 registers let two tiles share a compute unit
template <> struct Tuning<float, 16> : NotWide { static constexpr int rmax = 6, waves = 4, min_waves = 0, trips = 0; };   // 16 waves per tile
template <typename TU, int NT>
using GeomFrom = TileGeom<NT, TU::rmax, TU::waves, TU::min_waves, TU::trips, TU::wide, TU::start, TU::chunk>;   // wide, start: see WideF32 below
template <typename T, int NT>
using GeomFor = GeomFrom<Tuning<T, NT>, NT>;
// Fused fp32 kernels with packed sign words for vectors of 2^12 .. 2^14 elements use exchanges that also
// trade lane bits 4, 5 for register bits (TileGeom's WIDE_; column tiles never do), through half-size LDS buffers:
// 32 values per thread on two waves at 2^12, 64 values held to 128 registers on two / four waves at 2^13 / 2^14.
// Measured against the tables above: 2^12 0.374 -> 0.345 ms (the copy kernel's time), 2^13 -8 %, 2^14 -2 to -4 %;
// no gain for fp64 butterflies, which keep the narrow exchanges.
constexpr bool has_wide_words(int log2n) { return log2n >= 12 && log2n <= 14; }      // sizes of the wide geometries
template <int NT> struct WideF32 { static constexpr int rmax = NT >= 13 ? 6 : 5, waves = 4, min_waves = NT >= 13 ? 4 : 0, trips = 2, wide = 1, start = 0, chunk = kLaneChunk; };
template <typename T, int NT>
using ContigTuning = std::conditional_t<std::is_same<T, float>::value && has_wide_words(NT), WideF32<NT>, Tuning<T, NT>>;
template <typename T, int NT>
using ContigGeomFor = GeomFrom<ContigTuning<T, NT>, NT>;
// Row passes of the four-pass schedule that flip signs by packed words need one tile per wave (a wave's scalar
// loads fetch the words of one tile): 2^11-element rows then take 32 values per thread instead of 64.
struct RowSigns11 : NotWide { static constexpr int rmax = 5, waves = 4, min_waves = 0, trips = 0; };
constexpr int kRowSignsMinLog = 9;      // shorter rows share a wave: those passes multiply by the fp32 diagonals
// Fused three-round kernels with fp32 diagonals at n = 2^13, 2^14: 32 values per thread (four / eight waves per tile)
// and half-size exchange buffers.  With 64 values the diagonal loads of the second and third round do not fit the
// 128 registers beside the data (the 2^14 kernel spilled); measured in one run: 2^14 0.518 -> 0.483 ms, 2^13 0.438 -> 0.431.
template <int NT> struct FusedF32DiagTuning : Tuning<float, NT> {};
template <> struct FusedF32DiagTuning<13> : NotWide { static constexpr int rmax = 5, waves = 4, min_waves = 0, trips = 2; };
// eight waves per tile: crossbar lane stages in batches of eight registers keep the kernel at 64 registers (four tiles
// per compute unit instead of three; 0.479 -> 0.447 ms)
template <> struct FusedF32DiagTuning<14> { static constexpr int rmax = 5, waves = 4, min_waves = 0, trips = 2, wide = 0, start = 0, chunk = 8; };
// geometry of the kernels whose last round is pruned (a separate table so that it can be tuned apart)
template <typename T, int NT> struct PrunedTuning : Tuning<T, NT> {};
template <typename T, int NT>
using PrunedGeomFor = GeomFrom<PrunedTuning<T, NT>, NT>;

// XCD-aware numbering of the workgroups of the fused sign-word kernels (xcd_tile): each XCD takes runs of consecutive
// workgroups that cover 512 KiB of x (tiles of several waves) or 1 MiB (tiles of one wave).  Measured against plain
// numbering, in one process: n = 2^8 80.2 -> 83.9 % of the HBM peak, 2^10 75.8 -> 76.7, 2^11 75.1 -> 77.8, 2^12
// 76.5 -> 77.9, 2^13 69.4 -> 72.2-72.8, 2^14 69.6 -> 70.5; runs of 128 KiB and less lose up to 8 %, the kernels with
// fp32 diagonals and the sizes 2^15, 2^16 gain nothing (not applied there).
template <typename G>
constexpr int xcd_group_log_for()
{
    int wg_bytes_log = G::NT + 2;
    for (int t = G::TILES_PER_WG; t > 1; t >>= 1) ++wg_bytes_log;
    const int target = G::WB > 0 ? 19 : 20;
    return G::NT > 14 ? -1 : (target > wg_bytes_log ? target - wg_bytes_log : 0);
}

template <typename T, int NT, int C, int NSTEPS, bool FIRST_DIAG, int EPI, bool SIGNS = false, int PRUNE = 0, bool RAGGED = true>
inline hipError_t launch_tile(const TileParams& p, long long total_tiles, hipStream_t stream)
{
    // wide exchanges pay with packed sign words only: fp32 diagonals read in layout 1 come in 256-byte runs,
    // which measured 2-5 % slower than the narrow exchange (also for the row passes of the four-pass schedule)
    // the sign-word kernels with a pruned last round use the wide exchanges too
    // (first n/16 rows: 2^12 0.494 -> 0.451 ms, 2^13 0.528 -> 0.490, 2^14 0.545 -> 0.524)
    constexpr bool kWidePruned = PRUNE > 0 && SIGNS && C >= NT && NSTEPS == 3 && EPI == EPI_STORE_NONE && std::is_same<T, float>::value &&
                                 has_wide_words(NT);
    constexpr bool kFusedF32Diag = PRUNE == 0 && !SIGNS && C >= NT && NSTEPS == 3 && EPI == EPI_STORE_NONE && std::is_same<T, float>::value;
    using G = std::conditional_t<(PRUNE > 0 && !kWidePruned), PrunedGeomFor<T, NT>,
                                 std::conditional_t<(C >= NT && SIGNS && NSTEPS == 3), ContigGeomFor<T, NT>,
                                                    std::conditional_t<(SIGNS && NSTEPS < 3 && NT == 11), GeomFrom<RowSigns11, NT>,
                                                                       std::conditional_t<kFusedF32Diag, GeomFrom<FusedF32DiagTuning<NT>, NT>, GeomFor<T, NT>>>>>;
    const long long blocks = (total_tiles + G::TILES_PER_WG - 1) / G::TILES_PER_WG;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    TileParams q = p;
    q.xcd_group_log = (SIGNS && NSTEPS == 3 && C >= NT) ? xcd_group_log_for<G>() : -1;
    hipLaunchKernelGGL((spinner_tile_kernel<T, G, C, NSTEPS, FIRST_DIAG, EPI, SIGNS, PRUNE, RAGGED>), dim3((unsigned)blocks),
                       dim3(G::THREADS), 0, stream, q);
    return hipGetLastError();
}

// implemented in fused_none.hip / fused_cossin.hip / multipass.hip / hash.hip
hipError_t launch_fused_none(int log2n, bool signs, int prune, const TileParams& p, long long tiles, hipStream_t s);
// fp32 diagonals, full-width output, n = 2^12, 2^13: a workgroup carries two vectors per diagonal load (fused_shared.hip)
constexpr bool has_shared_diag_kernel(int log2n) { return log2n == 12 || log2n == 13; }
hipError_t launch_fused_shared_diag(int log2n, const TileParams& p, hipStream_t s);
constexpr int kPruneBits = 4;   // the pruned variant drops the 4 highest index bits in the last round (m <= n/16)
hipError_t launch_fused_cossin(int log2n, bool signs, const TileParams& p, long long tiles, hipStream_t s);
// signs: the diagonal of the pass comes as packed words p.sw[] (rows of at least 2^kRowSignsMinLog elements), not as p.d[]
hipError_t launch_row_first(int nt, bool signs, const TileParams& p, long long tiles, hipStream_t s);    // D1 then rows
hipError_t launch_row_middle(int nt, bool signs, const TileParams& p, long long tiles, hipStream_t s);   // rows, D3, rows
hipError_t launch_row_plain(int nt, const TileParams& p, long long tiles, hipStream_t s);                 // rows
// signs: the pass flips by the lane masks p.sw[1] that launch_pack_col_words prepared for its tiles
hipError_t launch_col_middle(int rows_log, int contig_log, bool signs, const TileParams& p, long long tiles, hipStream_t s);   // cols, D2, cols
hipError_t launch_col_last(int rows_log, int contig_log, int epi, const TileParams& p, long long tiles, hipStream_t s);   // cols, epilogue
hipError_t launch_hash(int log2n, bool signs, const HashParams& p, hipStream_t s);
hipError_t launch_hash_tile(int log2n, bool signs, const TileParams& p, long long tiles, hipStream_t s);   // n = 2^15, 2^16, one triple
// n > 2^16: buckets of a projection y [batch][n] that the four-pass schedule left in memory (two small kernels)
size_t hash_candidates_bytes(int log2n, long long batch);
hipError_t launch_hash_argmax(const float* y, int log2n, long long batch, void* candidates, int* out_idx, long long out_stride,
                              hipStream_t s);
// sign codes (angular-kernel features): fused kernels for n = 2^8 .. 2^16, packing of an fp32 projection, Gram matrix
constexpr int kCodeMinLog = 8;
hipError_t launch_fused_signbits(int log2n, bool signs, int prune, const TileParams& p, long long tiles, hipStream_t s);
hipError_t launch_pack_codes(const float* y, long long y_stride, unsigned long long* codes, int m, long long batch, hipStream_t s);
hipError_t launch_hamming_gram(const unsigned long long* a, long long na, const unsigned long long* b, long long nb, int m,
                               float* out, hipStream_t s);

// stacked blocks in one launch (blocks.hip): L fp32 triples [L][3][n] applied to a resident copy of x, n <= 2^kBlocksMaxLog;
// p as for one block (out_stride = the whole row, sin_off = L m, inv_sqrt_m = 1 / sqrt(L m))
constexpr int kBlocksMaxLog = 14;
hipError_t launch_blocks(int log2n, bool cossin, const TileParams& p, const float* diag_sets, int L, hipStream_t s);

// sign words per diagonal in the packed format
inline long long sign_words_per_diag(int n) { return n / 64 < 4 ? 4 : n / 64; }
// Sizes whose hash kernel keeps every butterfly between registers (hash.hip) take, behind the three diagonals'
// sign words of a triple, the lane masks of that kernel's two layouts: [3 diagonals][2 layouts][2^r words].
constexpr int hash_ar_log2r(int log2n)      // values per thread (log2) at n = 2^8 and 2^10; 0: size not covered
{
    return log2n == 8 ? 4 : (log2n == 10 ? 5 : 0);
}
// The fp64 feature map has such a kernel too (fused_cossin.hip), for n = 2^(2r), and reads the same lane masks.
constexpr int feature_ar_log2r(int log2n) { return log2n == 12 ? 6 : 0; }
constexpr int ar_log2r(int log2n) { return hash_ar_log2r(log2n) ? hash_ar_log2r(log2n) : feature_ar_log2r(log2n); }
// n = 2^12 .. 2^14: the wide geometries flip signs in a layout whose lane masks are no words of the packed format;
// they follow as a block of their own, [3 diagonals][n / 64 words], word (wave << r) | register (fused_none.hip).
inline long long wide_words_offset(int n, int log2n)      // from a triple's first sign word
{
    return 3 * sign_words_per_diag(n) + (ar_log2r(log2n) ? 6LL << ar_log2r(log2n) : 0);
}
hipError_t launch_pack_wide_words(const float* diag_sets, int log2n, int L, unsigned long long* signs, hipStream_t s);
// Shape of the column tiles of the four-pass schedule: 2^rows_log rows (all rows of the
// matrix view) by 2^contig_log contiguous columns.  Up to n = 2^21 the matrix view has
// 2^7 rows and a column tile is 128 rows x 32 columns (128-byte segments, 2^12 elements:
// one wave, no LDS, no barriers); larger n take more rows so that a row (a contiguous
// tile of n / rows elements) still fits on chip.  128-byte segments measured 25-30 %
// faster than 64-byte ones.
struct ColShape { int rows_log, contig_log; };
inline ColShape col_shape_for(int log2n)
{
    // rows_log grows only as far as needed to keep a row (n / rows elements) within 2^14
    return log2n <= 21 ? ColShape{7, 5} : (log2n == 22 ? ColShape{8, 5} : (log2n == 23 ? ColShape{9, 5} : ColShape{10, 4}));
}

// n > 2^14 (sizes that the four-pass schedule serves): that schedule multiplies by the second diagonal in column
// tiles, whose lanes hold no run of the packed format; the lane masks of that pass follow the three diagonals' words
// (n / 64 words, multipass.hip), and then, where the rows of the matrix view are too short for the row passes to flip
// by sign words (n = 2^15), the fp32 diagonals.
inline long long col_words_offset(int n, int log2n) { return wide_words_offset(n, log2n); }
inline long long fp32_copy_offset(int n, int log2n) { return col_words_offset(n, log2n) + sign_words_per_diag(n); }
inline bool has_fp32_copy(int log2n) { return log2n > kFusedMaxLogOther && log2n - col_shape_for(log2n).rows_log < kRowSignsMinLog; }
inline long long sign_words_per_triple(int n, int log2n)
{
    if (log2n > kFusedMaxLogOther) return fp32_copy_offset(n, log2n) + (has_fp32_copy(log2n) ? 3LL * n / 2 : 0);
    return wide_words_offset(n, log2n) + (has_wide_words(log2n) ? 3 * sign_words_per_diag(n) : 0);
}
hipError_t launch_pack_col_words(const float* diag_sets, int log2n, int L, unsigned long long* signs, hipStream_t s);
hipError_t launch_pack_hash_words(const float* diag_sets, int log2n, int L, unsigned long long* signs, hipStream_t s);

// adaptive layer (forward with saved activations, backward); the parameter structs are in layer_kernels.hpp
struct LayerForwardParams;
struct LayerBackwardParams;
constexpr int kLayerMaxLog = 14;
hipError_t launch_layer_forward(int log2n, const LayerForwardParams& p, hipStream_t s);
long long layer_backward_slots(int log2n, long long batch);      // partial-sum rows the backward kernel writes
hipError_t launch_layer_backward(int log2n, const LayerBackwardParams& p, hipStream_t s);
hipError_t launch_layer_reduce(const float* partial, long long slots, long long len, double factor, float* dd, hipStream_t s);
// n > 2^14: dd[i] = sum over the batch of g[b][i] a[b][i] (partial: layer_large_slabs(log2n, batch) rows of n floats);
// with d1 != null the same sweep writes dx = d1 .* g
long long layer_large_slabs(int log2n, long long batch);
hipError_t launch_layer_large_dd(const float* g, const float* a, int log2n, long long batch, float* partial, float* dd,
                                 const float* d1, float* dx, hipStream_t s);

// Newton sketch: transposition with optional row weights, Gram matrix on the matrix pipe
hipError_t launch_transpose_scale(const float* src, long long rows, long long cols, const float* row_scale, float* dst,
                                  hipStream_t s);
// the sketch on the columns as they lie (sketch_cols.hip): n = 2^4 .. 2^kSketchColsMaxLog, d a multiple of 4; factor = n^{-3/2} scale
constexpr int kSketchColsMaxLog = 12;
// Shapes for which that form is the faster one.  Measured against transposition + projection + transposition (ms):
// n = 4096: d = 512 0.035 / 0.017, 1024 0.037 / 0.023, 2048 0.040 / 0.036, 4096 0.044 / 0.062, 16384 0.184 / 0.252;
// n = 2048: d = 2048 0.022 / 0.024, 8192 0.039 / 0.058; n = 1024: d = 256 0.012 / 0.013, 4096 0.016 / 0.022,
// 65536 0.125 / 0.239; n = 256, d = 65536: 0.026 / 0.050.
inline bool sketch_cols_pays(int log2n, long long d)
{
    return log2n <= kSketchColsMaxLog && (d & 3) == 0 && d >= (log2n == 12 ? 4096 : (log2n == 11 ? 1024 : 64));
}
hipError_t launch_sketch_cols(const float* A, int log2n, long long d, const float* w, const float* d1, const float* d2, const float* d3,
                              int m, float factor, float* B, hipStream_t s);
int sketch_gram_slabs(int m, int d);      // d x d slabs of scratch the Gram kernel needs (1: none)
hipError_t launch_sketch_gram(const float* B, int m, int d, float* G, float* slabs, hipStream_t s);
// scratch of spinner_sketch_gram_static: a file-scope device array in sketch.hip; gram_static_scratch_ptr gives its
// address on the current device (looked up on the first call per device, no allocation)
constexpr size_t kGramStaticScratchBytes = (size_t)16 << 20;
hipError_t gram_static_scratch_ptr(float** ptr);

// G_struct D2 H D1 members: spectrum of the structured block, FFT convolution (structured.hip)
hipError_t launch_struct_prepare(const float* params, int kind, int n, int log2p, float2* spec, float2* tw, hipStream_t s);
hipError_t launch_struct_conv(const float* x, const float* d1, const float* d2, const float2* spec, const float2* tw, float* out,
                              long long batch, int n, int log2n, int log2p, int m, int reverse, float factor, hipStream_t s);

// transforms of length P = 2^15 .. 2^kStructLargeMaxLog2pHost through global memory (structured.hip)
constexpr int kStructLargeMaxLog2pHost = 22;
hipError_t launch_struct_prepare_large(const float* params, int kind, int n, int log2p, float2* spec, float2* tw, float2* tw_b,
                                       hipStream_t s);
hipError_t launch_struct_conv_large(const float* t, const float* d2, const float2* spec, const float2* tw, const float2* tw_b, float2* z,
                                    float* out, long long batch, int n, int log2p, int m, int reverse, float factor, hipStream_t s);

}  // namespace spinner
