// C ABI of the structured-spinner library: argument validation and dispatch.
// The declarations, their meaning and the passages of the paper they follow
// are in include/spinner.h.
#include "spinner.h"

#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "launch.hpp"
#include "layer_params.hpp"

namespace spinner {
// ------------------------------------------------------------------ plain copy (measurement aid)
__global__ void __launch_bounds__(256) stream_copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst,
                                                          size_t count4)
{
    // one 16-byte element per thread, 4 KiB per workgroup: the shape that reached the
    // highest read+write rate in bandwidth probes on MI355X
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < count4) dst[i] = src[i];
}

// One wave per output word: lane l looks at element ((w >> 2) << 8) | (l << 2) | (w & 3)
// of its diagonal and the wave's ballot of the sign bits is the word.
// Diagonal dg = 3 * triple + k; a triple's words start triple_words apart.
__global__ void __launch_bounds__(256) pack_signs_kernel(const float* __restrict__ diag, unsigned long long* __restrict__ out,
                                                         int n, int W, long long triple_words, long long total_words)
{
    const long long gw = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (gw >= total_words) return;
    const long long dg = gw / W;
    const int w = (int)(gw - dg * W);
    const long long e = ((long long)(w >> 2) << 8) | (lane << 2) | (w & 3);
    bool neg = false;
    if (e < n) neg = (__float_as_uint(diag[dg * n + e]) >> 31) != 0;
    const unsigned long long m = __ballot(neg);
    if (lane == 0) out[(dg / 3) * triple_words + (dg % 3) * W + w] = m;
}
}  // namespace spinner

namespace {

thread_local char g_hip_msg[256] = "HIP error";

int hip_fail(hipError_t e)
{
    snprintf(g_hip_msg, sizeof(g_hip_msg), "HIP error: %s", hipGetErrorString(e));
    return SPINNER_ERR_HIP;
}

bool pow2_in_range(int n, int* log2n)
{
    if (n < 16 || n > (1 << 24) || (n & (n - 1))) return false;
    int l = 0;
    while ((1 << l) < n) ++l;
    *log2n = l;
    return true;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// internal epilogue id of the sign-code entry points (not part of spinner_epilogue_t)
constexpr int kEpiSignBits = 2;

int fused_max_log(int epilogue)
{
    return epilogue == SPINNER_EPI_COSSIN ? spinner::kFusedMaxLogOther : spinner::kFusedMaxLogPlain;
}


}  // namespace

extern "C" {

int spinner_version(void) { return 140; }

const char* spinner_strerror(int status)
{
    switch (status) {
    case SPINNER_OK: return "success";
    case SPINNER_ERR_BAD_N: return "n must be a power of two in [2^4, 2^24]";
    case SPINNER_ERR_BAD_M: return "m must satisfy 1 <= m <= n";
    case SPINNER_ERR_NULL_PTR: return "a required pointer is NULL";
    case SPINNER_ERR_BAD_EPILOGUE: return "unknown epilogue";
    case SPINNER_ERR_BAD_BATCH: return "batch is negative or too large";
    case SPINNER_ERR_WORKSPACE: return "workspace required but NULL";
    case SPINNER_ERR_HIP: return g_hip_msg;
    case SPINNER_ERR_BAD_L: return "L must be >= 1";
    case SPINNER_ERR_ALIGNMENT: return "data pointers must be 16-byte aligned";
    case SPINNER_ERR_UNSUPPORTED: return "combination not supported";
    case SPINNER_ERR_SCRATCH_LIMIT: return "problem needs more scratch than the library's built-in buffer holds";
    default: return "unknown status";
    }
}

size_t spinner_workspace_bytes(int n, long batch, int m, int epilogue)
{
    int log2n;
    if (!pow2_in_range(n, &log2n) || batch <= 0 || m < 1 || m > n) return 0;
    if (log2n <= fused_max_log(epilogue)) return 0;
    if (m == n && epilogue == SPINNER_EPI_NONE) return 0;
    return (size_t)batch * (size_t)n * sizeof(float);
}

// Shared body of spinner_apply / spinner_apply_signs.  For n <= 2^14 `signs`
// (if non-null) replaces d1..d3; above that size the caller passes fp32 diagonals.
// blocks > 1: this call writes block `block` of a row that stacks `blocks` independent m-row blocks
// (out already points at the block's first column; see spinner_apply_blocks).
static int apply_impl(const float* x, int n, int log2n, long batch, const float* d1, const float* d2, const float* d3,
                      const unsigned long long* signs, int m, int epilogue, float scale, float* out,
                      void* workspace, void* stream, int blocks = 1)
{
    using namespace spinner;
    // a block of a stacked row never runs its passes in place: its output rows are wider than n
    const size_t ws = (blocks > 1 && log2n > fused_max_log(epilogue)) ? (size_t)batch * (size_t)n * sizeof(float)
                                                                      : spinner_workspace_bytes(n, batch, m, epilogue);
    if (ws && !workspace) return SPINNER_ERR_WORKSPACE;
    if (ws && !aligned16(workspace)) return SPINNER_ERR_ALIGNMENT;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const int epi = epilogue == SPINNER_EPI_COSSIN ? EPI_STORE_COSSIN : EPI_STORE_NONE;
    // row stride of the output: floats, or 64-bit words for sign codes
    const long long out_stride = (epilogue == SPINNER_EPI_COSSIN ? 2LL * m : (epilogue == kEpiSignBits ? m / 64 : (long long)m)) * blocks;
    // n^{-3/2} * scale, formed in double and rounded once
    const double factor_d = (double)scale / ((double)n * sqrt((double)n));

    TileParams p;
    memset(&p, 0, sizeof(p));
    p.batch = batch;
    p.m = m;
    p.inv_sqrt_m = (float)(1.0 / sqrt((double)m * blocks));
    p.sin_off = (long long)m * blocks;
    p.factor_rev = factor_d / 6.283185307179586476925286766559;
    p.xcd_group_log = -1;

    if (log2n <= fused_max_log(epilogue)) {
        if (batch > 0x7fffffffLL) return SPINNER_ERR_BAD_BATCH;
        p.x = x; p.out = out;
        p.d[0] = d1; p.d[1] = d2; p.d[2] = d3;
        if (signs) {
            const long long W = sign_words_per_diag(n);
            p.sw[0] = signs; p.sw[1] = signs + W; p.sw[2] = signs + 2 * W;
            p.wide_off = (int)wide_words_offset(n, log2n);      // both blocks hold a diagonal every W words
        }
        p.in_stride = n; p.out_stride = out_stride;
        p.tiles_per_vec_log = 0; p.tb = log2n; p.sl = 0;
        p.factor = (float)factor_d;
        // how many of the highest index bits lie entirely above the kept rows
        int prune = 0;
        while (prune < log2n && (long long)m <= ((long long)n >> (prune + 1))) ++prune;
        const bool shared_diag = !signs && epilogue == SPINNER_EPI_NONE && m == n && blocks == 1 && has_shared_diag_kernel(log2n);
        const hipError_t e = shared_diag                ? launch_fused_shared_diag(log2n, p, s)
                             : epilogue == kEpiSignBits ? launch_fused_signbits(log2n, signs != nullptr, prune, p, batch, s)
                             : epi == EPI_STORE_COSSIN ? launch_fused_cossin(log2n, signs != nullptr, p, batch, s)
                                                       : launch_fused_none(log2n, signs != nullptr, prune, p, batch, s);
        return e == hipSuccess ? SPINNER_OK : hip_fail(e);
    }

    // four passes; rows are contiguous runs of 2^nr elements, there are 2^kColRowsLog of them
    const ColShape cs = col_shape_for(log2n);
    const int kColRowsLog = cs.rows_log, kColContigLog = cs.contig_log;
    const int nr = log2n - kColRowsLog;
    float* buf_all = ws ? static_cast<float*>(workspace) : out;
    // with packed sign words the passes flip by lane mask: the row passes if a row fills a wave (else they multiply
    // by the fp32 diagonal), the column pass by the masks prepared for its tiles
    const bool row_signs = signs != nullptr && nr >= kRowSignsMinLog;
    const bool col_signs = signs != nullptr;
    if ((!row_signs && (!d1 || !d3)) || (!col_signs && !d2)) return SPINNER_ERR_NULL_PTR;
    // The batch is walked in slices of at most 256 MiB, all four passes per slice, so that the
    // three intermediate trips of a slice find it in the 256 MB memory-side cache (measured
    // 20 % faster than pass-by-pass over the whole batch; slices of 340 MiB are already as slow
    // as that, smaller ones lose 1 % at 224 MiB, 2 % at 192, 6 % at 128).
    const long long slice_bytes = 256LL << 20;
    long long slice = slice_bytes / (4LL * n);
    if (slice < 8) slice = 8;          // very long vectors: keep enough tiles per launch to fill the chip
    if (slice > batch) slice = batch;
    // equal slices: a short last slice would run its four launches on a partly empty chip
    const long long nslices = (batch + slice - 1) / slice;
    slice = (batch + nslices - 1) / nslices;
    if ((slice << kColRowsLog) > 0x7fffffffLL * 4 || (slice << (nr - kColContigLog)) > 0x7fffffffLL) return SPINNER_ERR_BAD_BATCH;

    for (long long b0 = 0; b0 < batch; b0 += slice) {
        const long long nb = batch - b0 < slice ? batch - b0 : slice;
        const long long row_tiles = nb << kColRowsLog;
        const long long col_tiles = nb << (nr - kColContigLog);
        float* buf = buf_all + b0 * (long long)n;
        hipError_t e;
        p.batch = nb;
        // P1: D1, rows : x -> buf
        p.x = x + b0 * (long long)n; p.out = buf; p.d[0] = d1; p.d[1] = nullptr; p.d[2] = nullptr;
        p.in_stride = n; p.out_stride = n; p.tiles_per_vec_log = kColRowsLog; p.tb = nr; p.sl = 0;
        p.m = n; p.factor = 1.0f;
        p.sw[0] = signs;
        if ((e = launch_row_first(nr, row_signs, p, row_tiles, s)) != hipSuccess) return hip_fail(e);
        // P2: cols, D2, cols : buf -> buf
        p.x = buf; p.out = buf; p.d[0] = nullptr; p.d[1] = d2;
        p.tiles_per_vec_log = nr - kColContigLog; p.tb = kColContigLog; p.sl = nr;
        if (col_signs) p.sw[1] = signs + col_words_offset(n, log2n);
        if ((e = launch_col_middle(kColRowsLog, kColContigLog, col_signs, p, col_tiles, s)) != hipSuccess) return hip_fail(e);
        // P3: rows, D3, rows : buf -> buf
        p.d[1] = d3; p.tiles_per_vec_log = kColRowsLog; p.tb = nr; p.sl = 0;
        if (row_signs) p.sw[1] = signs + 2 * sign_words_per_diag(n);
        if ((e = launch_row_middle(nr, row_signs, p, row_tiles, s)) != hipSuccess) return hip_fail(e);
        // P4: cols, epilogue : buf -> out
        p.out = out + b0 * out_stride; p.d[1] = nullptr; p.out_stride = out_stride;
        p.tiles_per_vec_log = nr - kColContigLog; p.tb = kColContigLog; p.sl = nr;
        p.m = m; p.factor = (float)factor_d;
        if ((e = launch_col_last(kColRowsLog, kColContigLog, epi, p, col_tiles, s)) != hipSuccess) return hip_fail(e);
    }
    return SPINNER_OK;
}

static int check_apply_args(const float* x, int n, long batch, int m, int epilogue, const float* out, int* log2n)
{
    if (!pow2_in_range(n, log2n)) return SPINNER_ERR_BAD_N;
    if (m < 1 || m > n) return SPINNER_ERR_BAD_M;
    if (epilogue != SPINNER_EPI_NONE && epilogue != SPINNER_EPI_COSSIN) return SPINNER_ERR_BAD_EPILOGUE;
    if (batch < 0 || (double)batch * (double)n > 9.0e15) return SPINNER_ERR_BAD_BATCH;
    if (batch == 0) return SPINNER_OK;
    if (!x || !out) return SPINNER_ERR_NULL_PTR;
    if (!aligned16(x) || !aligned16(out)) return SPINNER_ERR_ALIGNMENT;
    return SPINNER_OK;
}

int spinner_apply(const float* x, int n, long batch, const float* d1, const float* d2, const float* d3, int m,
                  int epilogue, float scale, float* out, void* workspace, void* stream)
{
    int log2n;
    const int rc = check_apply_args(x, n, batch, m, epilogue, out, &log2n);
    if (rc != SPINNER_OK || batch == 0) return rc;
    if (!d1 || !d2 || !d3) return SPINNER_ERR_NULL_PTR;
    if (!aligned16(d1) || !aligned16(d2) || !aligned16(d3)) return SPINNER_ERR_ALIGNMENT;
    return apply_impl(x, n, log2n, batch, d1, d2, d3, nullptr, m, epilogue, scale, out, workspace, stream);
}

size_t spinner_signs_bytes(int n, int L)
{
    int log2n;
    if (!pow2_in_range(n, &log2n) || L < 1) return 0;
    return (size_t)L * (size_t)spinner::sign_words_per_triple(n, log2n) * 8;
}

int spinner_pack_signs(const float* diag_sets, int n, int L, void* signs, void* stream)
{
    int log2n;
    if (!pow2_in_range(n, &log2n)) return SPINNER_ERR_BAD_N;
    if (L < 1) return SPINNER_ERR_BAD_L;
    if (!diag_sets || !signs) return SPINNER_ERR_NULL_PTR;
    if (!aligned16(diag_sets) || !aligned16(signs)) return SPINNER_ERR_ALIGNMENT;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int W = (int)spinner::sign_words_per_diag(n);
    const long long total_words = (long long)L * 3 * W;
    const long long blocks = (total_words + 3) / 4;
    hipLaunchKernelGGL(spinner::pack_signs_kernel, dim3((unsigned)blocks), dim3(256), 0, s, diag_sets,
                       static_cast<unsigned long long*>(signs), n, W, spinner::sign_words_per_triple(n, log2n), total_words);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && spinner::ar_log2r(log2n))
        e = spinner::launch_pack_hash_words(diag_sets, log2n, L, static_cast<unsigned long long*>(signs), s);
    if (e == hipSuccess && spinner::has_wide_words(log2n))
        e = spinner::launch_pack_wide_words(diag_sets, log2n, L, static_cast<unsigned long long*>(signs), s);
    // sizes of the four-pass schedule: lane masks of its column pass, then (short rows only) an fp32 copy of each triple
    if (e == hipSuccess && log2n > spinner::kFusedMaxLogOther)
        e = spinner::launch_pack_col_words(diag_sets, log2n, L, static_cast<unsigned long long*>(signs), s);
    if (e == hipSuccess && spinner::has_fp32_copy(log2n))
        e = hipMemcpy2DAsync(static_cast<unsigned long long*>(signs) + spinner::fp32_copy_offset(n, log2n),
                             (size_t)spinner::sign_words_per_triple(n, log2n) * 8,
                             diag_sets, (size_t)3 * n * sizeof(float), (size_t)3 * n * sizeof(float), (size_t)L,
                             hipMemcpyDeviceToDevice, s);
    return e == hipSuccess ? SPINNER_OK : hip_fail(e);
}

int spinner_apply_signs(const float* x, int n, long batch, const void* signs, int m, int epilogue, float scale,
                        float* out, void* workspace, void* stream)
{
    int log2n;
    const int rc = check_apply_args(x, n, batch, m, epilogue, out, &log2n);
    if (rc != SPINNER_OK || batch == 0) return rc;
    if (!signs) return SPINNER_ERR_NULL_PTR;
    if (!aligned16(signs)) return SPINNER_ERR_ALIGNMENT;
    if (log2n > fused_max_log(epilogue) && spinner::has_fp32_copy(log2n)) {      // four passes whose row passes multiply by the fp32 diagonals behind the words
        const unsigned long long* w = static_cast<const unsigned long long*>(signs);
        const float* d = reinterpret_cast<const float*>(w + spinner::fp32_copy_offset(n, log2n));
        return apply_impl(x, n, log2n, batch, d, d + n, d + 2 * (size_t)n, w, m, epilogue, scale, out, workspace, stream);
    }
    return apply_impl(x, n, log2n, batch, nullptr, nullptr, nullptr, static_cast<const unsigned long long*>(signs), m,
                      epilogue, scale, out, workspace, stream);
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

size_t spinner_hash_workspace_bytes(int n, long batch)
{
    int log2n;
    if (!pow2_in_range(n, &log2n) || batch <= 0 || log2n <= spinner::kFusedMaxLogPlain) return 0;
    return align256((size_t)batch * (size_t)n * sizeof(float)) + spinner::hash_candidates_bytes(log2n, batch);
}

// with_workspace: the call has a workspace argument (spinner_hash_ws / spinner_hash_signs_ws), which n > 2^16 needs
static int hash_impl(const float* x, int n, long batch, int L, const float* diag_sets, const unsigned long long* signs,
                     int* out_idx, void* stream, bool with_workspace = false, void* workspace = nullptr)
{
    using namespace spinner;
    int log2n;
    if (!pow2_in_range(n, &log2n)) return SPINNER_ERR_BAD_N;
    if (L < 1) return SPINNER_ERR_BAD_L;
    if (batch < 0 || (double)batch * (double)n > 9.0e15 || batch > 0x7fffffffL) return SPINNER_ERR_BAD_BATCH;
    if (batch == 0) return SPINNER_OK;
    if (!x || (!diag_sets && !signs) || !out_idx) return SPINNER_ERR_NULL_PTR;
    if (!aligned16(x) || !aligned16(diag_sets) || !aligned16(signs)) return SPINNER_ERR_ALIGNMENT;
    if (log2n > kFusedMaxLogPlain) {
        // four passes per triple leave the projection in the workspace; its bucket is taken from there
        if (!with_workspace) return SPINNER_ERR_UNSUPPORTED;
        if (!workspace) return SPINNER_ERR_WORKSPACE;
        if (!aligned16(workspace)) return SPINNER_ERR_ALIGNMENT;
        float* y = static_cast<float*>(workspace);
        void* candidates = static_cast<char*>(workspace) + align256((size_t)batch * (size_t)n * sizeof(float));
        for (int l = 0; l < L; ++l) {
            const float* d = diag_sets ? diag_sets + (size_t)l * 3 * n : nullptr;
            const unsigned long long* sw = signs ? signs + (long long)l * sign_words_per_triple(n, log2n) : nullptr;
            const int rc = apply_impl(x, n, log2n, batch, d, d ? d + n : nullptr, d ? d + 2 * (size_t)n : nullptr, sw, n,
                                      SPINNER_EPI_NONE, 1.0f, y, nullptr, stream);
            if (rc != SPINNER_OK) return rc;
            const hipError_t e = launch_hash_argmax(y, log2n, batch, candidates, out_idx + l, L, static_cast<hipStream_t>(stream));
            if (e != hipSuccess) return hip_fail(e);
        }
        return SPINNER_OK;
    }
    if (log2n > kFusedMaxLogOther) {
        // one launch of the fused plain kernel per triple, the bucket as its epilogue
        const long long W = sign_words_per_diag(n);
        for (int l = 0; l < L; ++l) {
            TileParams p;
            memset(&p, 0, sizeof(p));
            p.x = x; p.batch = batch; p.m = n;
            p.out = reinterpret_cast<float*>(out_idx + l);
            p.in_stride = n; p.out_stride = L;
            p.tiles_per_vec_log = 0; p.tb = log2n; p.sl = 0;
            p.factor = 1.0f;      // the bucket does not depend on a positive scale
            p.xcd_group_log = -1;
            if (signs) {
                const unsigned long long* sw = signs + (long long)l * sign_words_per_triple(n, log2n);
                p.sw[0] = sw; p.sw[1] = sw + W; p.sw[2] = sw + 2 * W;
            } else {
                const float* d = diag_sets + (size_t)l * 3 * n;
                p.d[0] = d; p.d[1] = d + n; p.d[2] = d + 2 * (size_t)n;
            }
            const hipError_t e = launch_hash_tile(log2n, signs != nullptr, p, batch, static_cast<hipStream_t>(stream));
            if (e != hipSuccess) return hip_fail(e);
        }
        return SPINNER_OK;
    }
    HashParams p;
    p.x = x; p.diag_sets = diag_sets; p.signs = signs; p.out_idx = out_idx; p.batch = batch; p.L = L;
    p.triple_words = sign_words_per_triple(n, log2n);
    const hipError_t e = launch_hash(log2n, signs != nullptr, p, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SPINNER_OK : hip_fail(e);
}

int spinner_hash(const float* x, int n, long batch, int L, const float* diag_sets, int* out_idx, void* stream)
{
    return hash_impl(x, n, batch, L, diag_sets, nullptr, out_idx, stream);
}

int spinner_hash_signs(const float* x, int n, long batch, int L, const void* signs, int* out_idx, void* stream)
{
    return hash_impl(x, n, batch, L, nullptr, static_cast<const unsigned long long*>(signs), out_idx, stream);
}

int spinner_hash_ws(const float* x, int n, long batch, int L, const float* diag_sets, int* out_idx, void* workspace, void* stream)
{
    return hash_impl(x, n, batch, L, diag_sets, nullptr, out_idx, stream, true, workspace);
}

int spinner_hash_signs_ws(const float* x, int n, long batch, int L, const void* signs, int* out_idx, void* workspace, void* stream)
{
    return hash_impl(x, n, batch, L, nullptr, static_cast<const unsigned long long*>(signs), out_idx, stream, true, workspace);
}

// ------------------------------------------------------------------ sign codes (angular kernel)
size_t spinner_code_bytes(int m) { return (m >= 256 && m % 256 == 0) ? (size_t)m / 8 : 0; }

size_t spinner_codes_workspace_bytes(int n, long batch)
{
    int log2n;
    if (!pow2_in_range(n, &log2n) || batch <= 0) return 0;
    return log2n <= spinner::kFusedMaxLogPlain ? 0 : (size_t)batch * (size_t)n * sizeof(float);
}

int spinner_code_position(int coordinate, int* word, int* bit)
{
    if (!word || !bit) return SPINNER_ERR_NULL_PTR;
    if (coordinate < 0) return SPINNER_ERR_BAD_M;
    *word = ((coordinate >> 8) << 2) | (coordinate & 3);
    *bit = (coordinate >> 2) & 63;
    return SPINNER_OK;
}

static int codes_impl(const float* x, int n, long batch, const float* d1, const float* d2, const float* d3,
                      const unsigned long long* signs, int m, void* codes, void* workspace, void* stream)
{
    int log2n;
    if (!pow2_in_range(n, &log2n)) return SPINNER_ERR_BAD_N;
    if (log2n < spinner::kCodeMinLog) return SPINNER_ERR_UNSUPPORTED;
    if (m < 256 || m > n || m % 256) return SPINNER_ERR_BAD_M;
    if (batch < 0 || (double)batch * (double)n > 9.0e15) return SPINNER_ERR_BAD_BATCH;
    if (batch == 0) return SPINNER_OK;
    if (!x || !codes) return SPINNER_ERR_NULL_PTR;
    if (!aligned16(x) || !aligned16(codes)) return SPINNER_ERR_ALIGNMENT;
    if (log2n <= spinner::kFusedMaxLogPlain)
        return apply_impl(x, n, log2n, batch, d1, d2, d3, signs, m, kEpiSignBits, 1.0f, static_cast<float*>(codes), nullptr,
                          stream);
    // above the fused range: the whole projection goes to the workspace (four passes), then its signs are packed
    if (!workspace) return SPINNER_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SPINNER_ERR_ALIGNMENT;
    float* y = static_cast<float*>(workspace);
    const int rc = apply_impl(x, n, log2n, batch, d1, d2, d3, signs, n, SPINNER_EPI_NONE, 1.0f, y, nullptr, stream);
    if (rc != SPINNER_OK) return rc;
    const hipError_t e = spinner::launch_pack_codes(y, n, static_cast<unsigned long long*>(codes), m, batch,
                                                    static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SPINNER_OK : hip_fail(e);
}

int spinner_sign_codes(const float* x, int n, long batch, const float* d1, const float* d2, const float* d3, int m,
                       void* codes, void* workspace, void* stream)
{
    if (batch > 0 && (!d1 || !d2 || !d3)) return SPINNER_ERR_NULL_PTR;
    if (!aligned16(d1) || !aligned16(d2) || !aligned16(d3)) return SPINNER_ERR_ALIGNMENT;
    return codes_impl(x, n, batch, d1, d2, d3, nullptr, m, codes, workspace, stream);
}

int spinner_sign_codes_signs(const float* x, int n, long batch, const void* signs, int m, void* codes, void* workspace,
                             void* stream)
{
    if (batch > 0 && !signs) return SPINNER_ERR_NULL_PTR;
    if (!aligned16(signs)) return SPINNER_ERR_ALIGNMENT;
    return codes_impl(x, n, batch, nullptr, nullptr, nullptr, static_cast<const unsigned long long*>(signs), m, codes,
                      workspace, stream);
}

int spinner_angular_gram(const void* codes_a, long na, const void* codes_b, long nb, int m, float* out, void* stream)
{
    if (m < 256 || m % 256) return SPINNER_ERR_BAD_M;
    if (na < 0 || nb < 0 || (double)na * (double)nb > 9.0e15) return SPINNER_ERR_BAD_BATCH;
    if (na == 0 || nb == 0) return SPINNER_OK;
    if (!codes_a || !codes_b || !out) return SPINNER_ERR_NULL_PTR;
    if (!aligned16(codes_a) || !aligned16(codes_b) || !aligned16(out)) return SPINNER_ERR_ALIGNMENT;
    if ((na + 127) / 128 > 65535) return SPINNER_ERR_BAD_BATCH;
    const hipError_t e = spinner::launch_hamming_gram(static_cast<const unsigned long long*>(codes_a), na,
                                                      static_cast<const unsigned long long*>(codes_b), nb, m, out,
                                                      static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SPINNER_OK : hip_fail(e);
}

// ------------------------------------------------------------------ adaptive layer
size_t spinner_layer_saved_bytes(int n, long batch)
{
    int log2n;
    if (!pow2_in_range(n, &log2n) || batch <= 0) return 0;
    return 2 * (size_t)batch * (size_t)n * sizeof(float);
}

size_t spinner_layer_workspace_bytes(int n, long batch)
{
    int log2n;
    if (!pow2_in_range(n, &log2n) || batch <= 0) return 0;
    if (log2n > spinner::kLayerMaxLog)      // two signal buffers and the partial rows of the batch sums
        return 2 * (size_t)batch * (size_t)n * sizeof(float) + (size_t)spinner::layer_large_slabs(log2n, batch) * (size_t)n * sizeof(float);
    return (size_t)spinner::layer_backward_slots(log2n, batch) * 3 * (size_t)n * sizeof(float);
}

static int check_layer_args(int n, long batch, int* log2n)
{
    if (!pow2_in_range(n, log2n)) return SPINNER_ERR_BAD_N;
    if (batch < 0 || batch > 0x7fffffffL || (double)batch * (double)n > 9.0e15) return SPINNER_ERR_BAD_BATCH;
    return SPINNER_OK;
}

// One transform of vectors longer than the fused layer kernels serve: out = factor * H (diag .* in), or factor * H in
// when diag is null, as a pass over the rows and a pass over the columns of the 2^rows x 2^nr view of each vector
// (the passes of the four-pass schedule, one transform each).  in == out is allowed.  The batch is walked in slices of
// 256 MiB so that the second pass finds what the first wrote in the memory-side cache.
static int large_round(const float* in, const float* diag, float* out, int n, int log2n, long long batch, double factor,
                       hipStream_t s)
{
    using namespace spinner;
    const ColShape cs = col_shape_for(log2n);
    const int nr = log2n - cs.rows_log;
    long long slice = (256LL << 20) / (4LL * n);
    if (slice < 8) slice = 8;
    if (slice > batch) slice = batch;
    const long long nslices = (batch + slice - 1) / slice;
    slice = (batch + nslices - 1) / nslices;
    if ((slice << cs.rows_log) > 0x7fffffffLL * 4 || (slice << (nr - cs.contig_log)) > 0x7fffffffLL) return SPINNER_ERR_BAD_BATCH;
    TileParams p;
    memset(&p, 0, sizeof(p));
    p.xcd_group_log = -1;
    p.in_stride = n; p.out_stride = n; p.m = n;
    for (long long b0 = 0; b0 < batch; b0 += slice) {
        const long long nb = batch - b0 < slice ? batch - b0 : slice;
        hipError_t e;
        p.batch = nb;
        p.x = in + b0 * (long long)n; p.out = out + b0 * (long long)n; p.d[0] = diag;
        p.tiles_per_vec_log = cs.rows_log; p.tb = nr; p.sl = 0; p.factor = 1.0f;
        e = diag ? launch_row_first(nr, false, p, nb << cs.rows_log, s) : launch_row_plain(nr, p, nb << cs.rows_log, s);
        if (e != hipSuccess) return hip_fail(e);
        p.x = p.out; p.d[0] = nullptr;
        p.tiles_per_vec_log = nr - cs.contig_log; p.tb = cs.contig_log; p.sl = nr; p.factor = (float)factor;
        if ((e = launch_col_last(cs.rows_log, cs.contig_log, EPI_STORE_NONE, p, nb << (nr - cs.contig_log), s)) != hipSuccess)
            return hip_fail(e);
    }
    return SPINNER_OK;
}

int spinner_layer_forward(const float* x, int n, long batch, const float* d1, const float* d2, const float* d3,
                          float scale, float* y, void* saved, void* stream)
{
    int log2n;
    const int rc = check_layer_args(n, batch, &log2n);
    if (rc != SPINNER_OK || batch == 0) return rc;
    if (!x || !d1 || !d2 || !d3 || !y || !saved) return SPINNER_ERR_NULL_PTR;
    if (!aligned16(x) || !aligned16(d1) || !aligned16(d2) || !aligned16(d3) || !aligned16(y) || !aligned16(saved))
        return SPINNER_ERR_ALIGNMENT;
    if (log2n > spinner::kLayerMaxLog) {
        // three single transforms; the activations entering D2 and D3 are kept normalised
        hipStream_t s = static_cast<hipStream_t>(stream);
        float* a2 = static_cast<float*>(saved);
        float* a3 = a2 + (size_t)batch * n;
        const double h = 1.0 / sqrt((double)n);
        int r = large_round(x, d1, a2, n, log2n, batch, h, s);
        if (r == SPINNER_OK) r = large_round(a2, d2, a3, n, log2n, batch, h, s);
        if (r == SPINNER_OK) r = large_round(a3, d3, y, n, log2n, batch, h * (double)scale, s);
        return r;
    }
    spinner::LayerForwardParams p;
    p.x = x; p.d[0] = d1; p.d[1] = d2; p.d[2] = d3; p.y = y;
    p.saved1 = static_cast<float*>(saved);
    p.saved2 = p.saved1 + (size_t)batch * n;
    p.batch = batch;
    p.factor = (float)((double)scale / ((double)n * sqrt((double)n)));
    const hipError_t e = spinner::launch_layer_forward(log2n, p, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SPINNER_OK : hip_fail(e);
}

int spinner_layer_backward(const float* dy, const float* x, const void* saved, int n, long batch, const float* d1,
                           const float* d2, const float* d3, float scale, float* dx, float* dd, void* workspace,
                           void* stream)
{
    int log2n;
    const int rc = check_layer_args(n, batch, &log2n);
    if (rc != SPINNER_OK) return rc;
    if (batch == 0) return SPINNER_OK;
    if (!dy || !x || !saved || !d1 || !d2 || !d3 || !dx || !dd) return SPINNER_ERR_NULL_PTR;
    if (!workspace) return SPINNER_ERR_WORKSPACE;
    if (!aligned16(dy) || !aligned16(x) || !aligned16(saved) || !aligned16(d1) || !aligned16(d2) || !aligned16(d3) ||
        !aligned16(dx) || !aligned16(dd) || !aligned16(workspace))
        return SPINNER_ERR_ALIGNMENT;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (log2n > spinner::kLayerMaxLog) {
        // the signal arriving at D3, D2, D1 from the output side is materialised in turn (g3 = scale H dy, g2 = H D3 g3,
        // g1 = H D2 g2); each diagonal's gradient is the batch sum of signal times saved activation; dx = D1 g1
        const float* a2 = static_cast<const float*>(saved);
        const float* a3 = a2 + (size_t)batch * n;
        float* w0 = static_cast<float*>(workspace);
        float* w1 = w0 + (size_t)batch * n;
        float* partial = w1 + (size_t)batch * n;
        const double h = 1.0 / sqrt((double)n);
        int r = large_round(dy, nullptr, w0, n, log2n, batch, h * (double)scale, s);
        if (r != SPINNER_OK) return r;
        hipError_t e = spinner::launch_layer_large_dd(w0, a3, log2n, batch, partial, dd + 2 * (size_t)n, nullptr, nullptr, s);
        if (e != hipSuccess) return hip_fail(e);
        if ((r = large_round(w0, d3, w1, n, log2n, batch, h, s)) != SPINNER_OK) return r;
        if ((e = spinner::launch_layer_large_dd(w1, a2, log2n, batch, partial, dd + (size_t)n, nullptr, nullptr, s)) != hipSuccess)
            return hip_fail(e);
        if ((r = large_round(w1, d2, w0, n, log2n, batch, h, s)) != SPINNER_OK) return r;
        e = spinner::launch_layer_large_dd(w0, x, log2n, batch, partial, dd, d1, dx, s);
        return e == hipSuccess ? SPINNER_OK : hip_fail(e);
    }
    const double factor = (double)scale / ((double)n * sqrt((double)n));
    spinner::LayerBackwardParams p;
    p.dy = dy; p.x = x;
    p.saved1 = static_cast<const float*>(saved);
    p.saved2 = p.saved1 + (size_t)batch * n;
    p.d[0] = d1; p.d[1] = d2; p.d[2] = d3;
    p.dx = dx;
    p.partial = static_cast<float*>(workspace);
    p.batch = batch;
    p.slots = spinner::layer_backward_slots(log2n, batch);
    p.factor = (float)factor;
    hipError_t e = spinner::launch_layer_backward(log2n, p, s);
    if (e != hipSuccess) return hip_fail(e);
    e = spinner::launch_layer_reduce(p.partial, p.slots, 3LL * n, factor, dd, s);
    return e == hipSuccess ? SPINNER_OK : hip_fail(e);
}

// ------------------------------------------------------------------ Newton sketch

size_t spinner_sketch_workspace_bytes(int n, int d, int m)
{
    int log2n;
    if (!pow2_in_range(n, &log2n) || d < 1 || m < 1 || m > n) return 0;
    return align256((size_t)d * n * sizeof(float)) + align256((size_t)d * m * sizeof(float)) +
           spinner_workspace_bytes(n, d, m, SPINNER_EPI_NONE);
}

int spinner_sketch(const float* A, int n, int d, const float* w, const float* d1, const float* d2, const float* d3, int m,
                   float scale, float* B, void* workspace, void* stream)
{
    int log2n;
    if (!pow2_in_range(n, &log2n)) return SPINNER_ERR_BAD_N;
    if (m < 1 || m > n) return SPINNER_ERR_BAD_M;
    if (d < 0 || (double)d * (double)n > 9.0e15) return SPINNER_ERR_BAD_BATCH;
    if (d == 0) return SPINNER_OK;
    if (!A || !d1 || !d2 || !d3 || !B) return SPINNER_ERR_NULL_PTR;
    if (!workspace) return SPINNER_ERR_WORKSPACE;
    if (!aligned16(A) || !aligned16(w) || !aligned16(d1) || !aligned16(d2) || !aligned16(d3) || !aligned16(B) ||
        !aligned16(workspace))
        return SPINNER_ERR_ALIGNMENT;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (spinner::sketch_cols_pays(log2n, d)) {
        // the columns as they lie: one pass over A
        const double factor_d = (double)scale / ((double)n * sqrt((double)n));
        const hipError_t e = spinner::launch_sketch_cols(A, log2n, d, w, d1, d2, d3, m, (float)factor_d, B, s);
        return e == hipSuccess ? SPINNER_OK : hip_fail(e);
    }
    char* base = static_cast<char*>(workspace);
    float* At = reinterpret_cast<float*>(base);                                             // [d][n]
    float* Ut = reinterpret_cast<float*>(base + align256((size_t)d * n * sizeof(float)));   // [d][m]
    void* ws2 = base + align256((size_t)d * n * sizeof(float)) + align256((size_t)d * m * sizeof(float));
    hipError_t e = spinner::launch_transpose_scale(A, n, d, w, At, s);
    if (e != hipSuccess) return hip_fail(e);
    const int rc = apply_impl(At, n, log2n, d, d1, d2, d3, nullptr, m, SPINNER_EPI_NONE, scale, Ut,
                              spinner_workspace_bytes(n, d, m, SPINNER_EPI_NONE) ? ws2 : nullptr, stream);
    if (rc != SPINNER_OK) return rc;
    e = spinner::launch_transpose_scale(Ut, d, m, nullptr, B, s);
    return e == hipSuccess ? SPINNER_OK : hip_fail(e);
}

size_t spinner_sketch_gram_workspace_bytes(int m, int d)
{
    if (m < 1 || d < 1) return 0;
    const int ks = spinner::sketch_gram_slabs(m, d);
    return ks > 1 ? (size_t)ks * d * d * sizeof(float) : 0;
}

int spinner_sketch_gram(const float* B, int m, int d, float* G, void* workspace, void* stream)
{
    if (m < 0 || d < 0) return SPINNER_ERR_BAD_BATCH;
    if (m == 0 || d == 0) return SPINNER_OK;
    if (!B || !G) return SPINNER_ERR_NULL_PTR;
    if (spinner_sketch_gram_workspace_bytes(m, d) && !workspace) return SPINNER_ERR_WORKSPACE;
    if (!aligned16(B) || !aligned16(G) || !aligned16(workspace)) return SPINNER_ERR_ALIGNMENT;
    const hipError_t e = spinner::launch_sketch_gram(B, m, d, G, static_cast<float*>(workspace),
                                                     static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SPINNER_OK : hip_fail(e);
}

size_t spinner_sketch_gram_static_limit(void) { return spinner::kGramStaticScratchBytes; }

int spinner_sketch_gram_static(const float* B, int m, int d, float* G, void* stream)
{
    if (m < 0 || d < 0) return SPINNER_ERR_BAD_BATCH;
    if (m == 0 || d == 0) return SPINNER_OK;
    if (!B || !G) return SPINNER_ERR_NULL_PTR;
    if (!aligned16(B) || !aligned16(G)) return SPINNER_ERR_ALIGNMENT;
    if (spinner_sketch_gram_workspace_bytes(m, d) > spinner::kGramStaticScratchBytes) return SPINNER_ERR_SCRATCH_LIMIT;
    float* slabs = nullptr;
    hipError_t e = spinner::gram_static_scratch_ptr(&slabs);
    if (e != hipSuccess) return hip_fail(e);
    // every slab entry the reduction reads is written by the first kernel of this call: nothing has to start at zero
    e = spinner::launch_sketch_gram(B, m, d, G, slabs, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SPINNER_OK : hip_fail(e);
}

// ------------------------------------------------------------------ stacked independent blocks
size_t spinner_blocks_workspace_bytes(int n, long batch, int m, int epilogue)
{
    // above the fused range every block runs its passes in the workspace (its output is a slice of wider rows)
    int log2n;
    if (!pow2_in_range(n, &log2n) || batch <= 0 || m < 1 || m > n) return 0;
    return log2n <= fused_max_log(epilogue) ? 0 : (size_t)batch * (size_t)n * sizeof(float);
}

int spinner_apply_blocks(const float* x, int n, long batch, int L, const float* diag_sets, int m, int epilogue, float scale,
                         float* out, void* workspace, void* stream)
{
    int log2n;
    const int rc = check_apply_args(x, n, batch, m, epilogue, out, &log2n);
    if (rc != SPINNER_OK) return rc;
    if (L < 1) return SPINNER_ERR_BAD_L;
    if (L > 1 && (m & 3)) return SPINNER_ERR_BAD_M;
    if (batch == 0) return SPINNER_OK;
    if (!diag_sets) return SPINNER_ERR_NULL_PTR;
    if (!aligned16(diag_sets)) return SPINNER_ERR_ALIGNMENT;
    if (spinner_blocks_workspace_bytes(n, batch, m, epilogue) && !workspace) return SPINNER_ERR_WORKSPACE;
    if (L > 1 && log2n <= spinner::kBlocksMaxLog) {
        // one launch: x is read once and stays in registers while the L triples are applied
        if (batch > 0x7fffffffLL) return SPINNER_ERR_BAD_BATCH;
        const double factor_d = (double)scale / ((double)n * sqrt((double)n));
        spinner::TileParams p;
        memset(&p, 0, sizeof(p));
        p.x = x; p.out = out; p.batch = batch; p.m = m;
        p.in_stride = n;
        p.out_stride = (epilogue == SPINNER_EPI_COSSIN ? 2LL : 1LL) * m * L;
        p.factor = (float)factor_d;
        p.factor_rev = factor_d / 6.283185307179586476925286766559;
        p.inv_sqrt_m = (float)(1.0 / sqrt((double)m * L));
        p.sin_off = (long long)m * L;
        p.xcd_group_log = -1;
        const hipError_t e = spinner::launch_blocks(log2n, epilogue == SPINNER_EPI_COSSIN, p, diag_sets, L,
                                                    static_cast<hipStream_t>(stream));
        return e == hipSuccess ? SPINNER_OK : hip_fail(e);
    }
    for (int l = 0; l < L; ++l) {
        const float* d = diag_sets + (size_t)l * 3 * n;
        // block l owns columns [l m, (l + 1) m) of the cos part (and of the sin part, L m further on)
        const int r = apply_impl(x, n, log2n, batch, d, d + n, d + 2 * (size_t)n, nullptr, m, epilogue, scale,
                                 out + (size_t)l * m, workspace, stream, L);
        if (r != SPINNER_OK) return r;
    }
    return SPINNER_OK;
}

// ------------------------------------------------------------------ G_struct D2 H D1 members
static int struct_log2p(int kind, int log2n) { return kind == SPINNER_STRUCT_CIRCULANT ? log2n : log2n + 1; }

constexpr int kStructLdsMaxLog2p = 14;      // longest transform one workgroup holds in LDS

// with_workspace: the call can take the path through global memory (transforms of 2^15 .. 2^22 points)
static int check_struct(int kind, int n, int* log2n, bool with_workspace = true)
{
    if (kind < SPINNER_STRUCT_CIRCULANT || kind > SPINNER_STRUCT_HANKEL) return SPINNER_ERR_BAD_EPILOGUE;
    if (!pow2_in_range(n, log2n)) return SPINNER_ERR_BAD_N;
    // H D1 x comes from the one-step tile kernels (n >= 32)
    const int lp = struct_log2p(kind, *log2n);
    if (*log2n < 5 || lp > (with_workspace ? spinner::kStructLargeMaxLog2pHost : kStructLdsMaxLog2p)) return SPINNER_ERR_UNSUPPORTED;
    return SPINNER_OK;
}

size_t spinner_struct_params(int kind, int n)
{
    int log2n;
    if (check_struct(kind, n, &log2n) != SPINNER_OK) return 0;
    return (kind == SPINNER_STRUCT_CIRCULANT || kind == SPINNER_STRUCT_SKEW_CIRCULANT) ? (size_t)n : 2 * (size_t)n - 1;
}

size_t spinner_struct_spectrum_bytes(int kind, int n)
{
    int log2n;
    if (check_struct(kind, n, &log2n) != SPINNER_OK) return 0;
    const int lp = struct_log2p(kind, log2n);
    const size_t P = (size_t)1 << lp;
    // spectrum, then the twiddle table; long transforms also carry the table of their blocks of 2^12 points
    return P * 8 + (P / 2) * 8 + (lp > kStructLdsMaxLog2p ? 2048 * 8 : 0);
}

size_t spinner_struct_workspace_bytes(int kind, int n, long batch)
{
    int log2n;
    if (check_struct(kind, n, &log2n) != SPINNER_OK || batch <= 0) return 0;
    const int lp = struct_log2p(kind, log2n);
    if (lp <= kStructLdsMaxLog2p) return 0;
    // H D1 x of every vector, then one complex work buffer of P points per pair of vectors
    return align256((size_t)batch * (size_t)n * sizeof(float)) + (size_t)((batch + 1) / 2) * ((size_t)8 << lp);
}

int spinner_struct_prepare(int kind, const float* params, int n, void* spectrum, void* stream)
{
    int log2n;
    const int rc = check_struct(kind, n, &log2n);
    if (rc != SPINNER_OK) return rc;
    if (!params || !spectrum) return SPINNER_ERR_NULL_PTR;
    if (!aligned16(params) || !aligned16(spectrum)) return SPINNER_ERR_ALIGNMENT;
    const int lp = struct_log2p(kind, log2n);
    float2* spec = static_cast<float2*>(spectrum);
    float2* tw = spec + ((size_t)1 << lp);
    const hipError_t e = lp > kStructLdsMaxLog2p
                             ? spinner::launch_struct_prepare_large(params, kind, n, lp, spec, tw, tw + ((size_t)1 << (lp - 1)),
                                                                    static_cast<hipStream_t>(stream))
                             : spinner::launch_struct_prepare(params, kind, n, lp, spec, tw, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SPINNER_OK : hip_fail(e);
}

static int struct_apply_impl(const float* x, int n, long batch, int kind, const void* spectrum, const float* d1, const float* d2,
                             int m, float scale, float* out, bool with_workspace, void* workspace, void* stream)
{
    int log2n;
    const int rc = check_struct(kind, n, &log2n, with_workspace);
    if (rc != SPINNER_OK) return rc;
    if (m < 1 || m > n) return SPINNER_ERR_BAD_M;
    if (batch < 0 || batch > 0x7fffffffL || (double)batch * (double)n > 9.0e15) return SPINNER_ERR_BAD_BATCH;
    if (batch == 0) return SPINNER_OK;
    if (!x || !spectrum || !d1 || !d2 || !out) return SPINNER_ERR_NULL_PTR;
    if (!aligned16(x) || !aligned16(spectrum) || !aligned16(d1) || !aligned16(d2) || !aligned16(out)) return SPINNER_ERR_ALIGNMENT;
    const int lp = struct_log2p(kind, log2n);
    const float2* spec = static_cast<const float2*>(spectrum);
    // the Hadamard stages and both transforms of the convolution run unnormalised: 1 / sqrt(n) and 1 / P go into the last scale
    const double factor = (double)scale / ((double)((size_t)1 << lp) * sqrt((double)n));
    if (lp > kStructLdsMaxLog2p) {
        // H D1 x (unnormalised) of every vector by a pass over rows and a pass over columns, then the convolution
        // through global memory: column stages, blocks of 2^12 points (with the spectrum product), column stages back
        if (!workspace) return SPINNER_ERR_WORKSPACE;
        if (!aligned16(workspace)) return SPINNER_ERR_ALIGNMENT;
        hipStream_t s = static_cast<hipStream_t>(stream);
        float* t = static_cast<float*>(workspace);
        float2* z = reinterpret_cast<float2*>(static_cast<char*>(workspace) + align256((size_t)batch * (size_t)n * sizeof(float)));
        const int r = large_round(x, d1, t, n, log2n, batch, 1.0, s);
        if (r != SPINNER_OK) return r;
        const float2* tw = spec + ((size_t)1 << lp);
        const hipError_t e = spinner::launch_struct_conv_large(t, d2, spec, tw, tw + ((size_t)1 << (lp - 1)), z, out, batch, n, lp, m,
                                                               kind == SPINNER_STRUCT_HANKEL ? 1 : 0, (float)factor, s);
        return e == hipSuccess ? SPINNER_OK : hip_fail(e);
    }
    const hipError_t e = spinner::launch_struct_conv(x, d1, d2, spec, spec + ((size_t)1 << lp), out, batch, n, log2n, lp, m,
                                                     kind == SPINNER_STRUCT_HANKEL ? 1 : 0, (float)factor,
                                                     static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SPINNER_OK : hip_fail(e);
}

int spinner_struct_apply(const float* x, int n, long batch, int kind, const void* spectrum, const float* d1, const float* d2,
                         int m, float scale, float* out, void* stream)
{
    return struct_apply_impl(x, n, batch, kind, spectrum, d1, d2, m, scale, out, false, nullptr, stream);
}

int spinner_struct_apply_ws(const float* x, int n, long batch, int kind, const void* spectrum, const float* d1, const float* d2,
                            int m, float scale, float* out, void* workspace, void* stream)
{
    return struct_apply_impl(x, n, batch, kind, spectrum, d1, d2, m, scale, out, true, workspace, stream);
}

int spinner_stream_copy(const float* src, float* dst, size_t count, void* stream)
{
    if (!src || !dst) return SPINNER_ERR_NULL_PTR;
    if (!aligned16(src) || !aligned16(dst) || (count & 3)) return SPINNER_ERR_ALIGNMENT;
    if (count == 0) return SPINNER_OK;
    const size_t count4 = count / 4;
    const size_t blocks = (count4 + 255) / 256;
    if (blocks > 0x7fffffffULL) return SPINNER_ERR_BAD_BATCH;
    hipLaunchKernelGGL(spinner::stream_copy_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       static_cast<hipStream_t>(stream), reinterpret_cast<const float4*>(src),
                       reinterpret_cast<float4*>(dst), count4);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? SPINNER_OK : hip_fail(e);
}

}  // extern "C"
