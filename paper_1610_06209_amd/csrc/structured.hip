// The G_struct D2 H D1 members of the family: third block a circulant, skew-circulant, Toeplitz or Hankel
// matrix given by its generating vector.  One workgroup holds two vectors in LDS as the real and imaginary
// parts of complex points (the generator is real, so the two stay apart): H D1 x by Walsh-Hadamard stages on
// those points, then the product with G_struct as a cyclic convolution of length P (n for a circulant, 2n
// otherwise) by a complex FFT in the same buffer.
#include "launch.hpp"
namespace spinner {

struct StructParams {
    const float* x;        // [batch][n]
    const float* d1;       // [n]
    const float* d2;       // [n]
    const float2* spec;    // [P] spectrum of the convolution kernel, in the order the forward transform leaves it
    const float2* tw;      // [P/2] exp(-2 pi i k / P)
    float* out;            // [batch][m]
    long long batch;
    int n, log2p, m, reverse;
    float factor;          // scale / (P sqrt(n)): both transforms are left unnormalised on the way
    int log2n;
};

__device__ __forceinline__ float2 cmul(float2 a, float2 b) { return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x); }
__device__ __forceinline__ float2 cmul_conj(float2 a, float2 b) { return make_float2(a.x * b.x + a.y * b.y, a.y * b.x - a.x * b.y); }

__device__ __forceinline__ float2 cadd(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ float2 csub(float2 a, float2 b) { return make_float2(a.x - b.x, a.y - b.y); }

// Point i of a transform sits at X[pad(i)]: one unused slot after every 16 points keeps the strided accesses of the
// passes below on different LDS banks.
__device__ __forceinline__ int pad(int i) { return i + (i >> 4); }
inline size_t fft_lds_bytes(int log2p) { return (((size_t)1 << log2p) + ((size_t)1 << log2p) / 16) * sizeof(float2); }

// A radix-2 stage on index bit s pairs points 2^s apart; with o the offset of the lower point inside its group of
// 2^s, the twiddle is exp(-2 pi i o / 2^(s+1)): the forward transform (decimation in frequency) multiplies the
// difference by it after the butterfly, the inverse (decimation in time) multiplies the upper point by its conjugate
// before the butterfly.  Four stages (bits top .. top-3) run on sixteen points k * 2^(top-3) + j, k = 0 .. 15, held
// in registers, one trip through LDS for the four; their twiddles are a base factor per stage (a function of j,
// read from the table) times a constant power of exp(-2 pi i / 16).
struct Twiddles16 { float2 a[8], b[4], c[2], d; };     // stages on bits top, top-1, top-2, top-3

__device__ __forceinline__ void twiddles16(Twiddles16& t, const float2* __restrict__ tw, int j, int top, int log2p)
{
    const int sh = log2p - 1 - top;
    const float2 b1 = tw[j << sh], b2 = tw[j << (sh + 1)], b3 = tw[j << (sh + 2)], b4 = tw[j << (sh + 3)];
    constexpr float c1 = 0.92387953251128674f, s1 = 0.38268343236508977f, h = 0.70710678118654752f;
    t.a[0] = b1;
    t.a[1] = cmul(b1, make_float2(c1, -s1));
    t.a[2] = cmul(b1, make_float2(h, -h));
    t.a[3] = cmul(b1, make_float2(s1, -c1));
    t.a[4] = make_float2(b1.y, -b1.x);                      // times -i
    t.a[5] = cmul(b1, make_float2(-s1, -c1));
    t.a[6] = cmul(b1, make_float2(-h, -h));
    t.a[7] = cmul(b1, make_float2(-c1, -s1));
    t.b[0] = b2;
    t.b[1] = cmul(b2, make_float2(h, -h));
    t.b[2] = make_float2(b2.y, -b2.x);
    t.b[3] = cmul(b2, make_float2(-h, -h));
    t.c[0] = b3;
    t.c[1] = make_float2(b3.y, -b3.x);
    t.d = b4;
}

template <bool INVERSE>
__device__ __forceinline__ void butterfly(float2& lo, float2& hi, float2 w)
{
    if constexpr (INVERSE) {
        const float2 t = cmul_conj(hi, w);
        hi = csub(lo, t);
        lo = cadd(lo, t);
    } else {
        const float2 d = csub(lo, hi);
        lo = cadd(lo, hi);
        hi = cmul(d, w);
    }
}

// the four stages on bits top .. top-3 (forward: in that order; inverse: from bit top-3 up).  load(i) brings point i,
// store(i, v) takes it: LDS by default; the first forward trip reads the vectors and the last inverse trip writes the
// result straight from / to global memory, and a trip next to the spectrum product multiplies on its way
template <bool INVERSE, typename Load, typename Store>
__device__ __forceinline__ void fft_trip16(const float2* __restrict__ tw, int top, int log2p, Load load, Store store)
{
    const int qb = top - 3, q = 1 << qb;
    for (int b = threadIdx.x; b < (1 << (log2p - 4)); b += blockDim.x) {
        const int j = b & (q - 1);
        const int i0 = ((b >> qb) << (top + 1)) | j;
        float2 v[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = load(i0 + (k << qb));
        Twiddles16 t;
        twiddles16(t, tw, j, top, log2p);
        if constexpr (!INVERSE) {
#pragma unroll
            for (int k = 0; k < 8; ++k) butterfly<false>(v[k], v[k + 8], t.a[k]);
#pragma unroll
            for (int k = 0; k < 16; ++k) if (!(k & 4)) butterfly<false>(v[k], v[k + 4], t.b[k & 3]);
#pragma unroll
            for (int k = 0; k < 16; ++k) if (!(k & 2)) butterfly<false>(v[k], v[k + 2], t.c[k & 1]);
#pragma unroll
            for (int k = 0; k < 16; k += 2) butterfly<false>(v[k], v[k + 1], t.d);
        } else {
#pragma unroll
            for (int k = 0; k < 16; k += 2) butterfly<true>(v[k], v[k + 1], t.d);
#pragma unroll
            for (int k = 0; k < 16; ++k) if (!(k & 2)) butterfly<true>(v[k], v[k + 2], t.c[k & 1]);
#pragma unroll
            for (int k = 0; k < 16; ++k) if (!(k & 4)) butterfly<true>(v[k], v[k + 4], t.b[k & 3]);
#pragma unroll
            for (int k = 0; k < 8; ++k) butterfly<true>(v[k], v[k + 8], t.a[k]);
        }
#pragma unroll
        for (int k = 0; k < 16; ++k) store(i0 + (k << qb), v[k]);
    }
    __syncthreads();
}
template <bool INVERSE>
__device__ __forceinline__ void fft_trip16(float2* X, const float2* __restrict__ tw, int top, int log2p)
{
    fft_trip16<INVERSE>(tw, top, log2p, [&](int i) { return X[pad(i)]; }, [&](int i, float2 v) { X[pad(i)] = v; });
}

// The stages on the LOW lowest bits (LOW = log2p mod 4, what the radix-16 trips leave) act on 2^LOW neighbouring
// points with constant twiddles (powers of exp(-2 pi i / 8)): forward stages, product with the spectrum and inverse
// stages are one pass over registers.
template <int LOW>
__device__ __forceinline__ void fft_middle(float2* X, const float2* __restrict__ spec, int log2p)
{
    constexpr int M = 1 << LOW;
    constexpr float h = 0.70710678118654752f;
    const float2 w8[4] = {make_float2(1.f, 0.f), make_float2(h, -h), make_float2(0.f, -1.f), make_float2(-h, -h)};
    for (int b = threadIdx.x; b < (1 << (log2p - LOW)); b += blockDim.x) {
        float2 v[M];
#pragma unroll
        for (int k = 0; k < M; ++k) v[k] = X[pad(b * M + k)];
#pragma unroll
        for (int st = LOW - 1; st >= 0; --st)
#pragma unroll
            for (int k = 0; k < M; ++k)
                if (!(k & (1 << st))) butterfly<false>(v[k], v[k + (1 << st)], w8[(k & ((1 << st) - 1)) * (4 >> st)]);
#pragma unroll
        for (int k = 0; k < M; ++k) v[k] = cmul(v[k], spec[b * M + k]);
#pragma unroll
        for (int st = 0; st < LOW; ++st)
#pragma unroll
            for (int k = 0; k < M; ++k)
                if (!(k & (1 << st))) butterfly<true>(v[k], v[k + (1 << st)], w8[(k & ((1 << st) - 1)) * (4 >> st)]);
#pragma unroll
        for (int k = 0; k < M; ++k) X[pad(b * M + k)] = v[k];
    }
    __syncthreads();
}

// two stages (bits s and s-1) on four points, and a single stage on bit 0: what is left below the radix-16 trips
template <bool INVERSE>
__device__ __forceinline__ void fft_trip4(float2* X, const float2* __restrict__ tw, int s, int log2p)
{
    const int q = 1 << (s - 1);
    const int sh = log2p - 1 - s;
    for (int b = threadIdx.x; b < (1 << (log2p - 2)); b += blockDim.x) {
        const int j = b & (q - 1);
        const int i0 = ((b >> (s - 1)) << (s + 1)) | j;
        float2 a0 = X[pad(i0)], a1 = X[pad(i0 + q)], a2 = X[pad(i0 + 2 * q)], a3 = X[pad(i0 + 3 * q)];
        const float2 w0 = tw[j << sh], w1 = tw[(j + q) << sh], wl = tw[j << (sh + 1)];
        if constexpr (!INVERSE) {
            butterfly<false>(a0, a2, w0);
            butterfly<false>(a1, a3, w1);
            butterfly<false>(a0, a1, wl);
            butterfly<false>(a2, a3, wl);
        } else {
            butterfly<true>(a0, a1, wl);
            butterfly<true>(a2, a3, wl);
            butterfly<true>(a0, a2, w0);
            butterfly<true>(a1, a3, w1);
        }
        X[pad(i0)] = a0; X[pad(i0 + q)] = a1; X[pad(i0 + 2 * q)] = a2; X[pad(i0 + 3 * q)] = a3;
    }
    __syncthreads();
}
__device__ __forceinline__ void fft_bit0(float2* X, int log2p)      // twiddle 1 in both directions
{
    for (int b = threadIdx.x; b < (1 << (log2p - 1)); b += blockDim.x) {
        const float2 a = X[pad(2 * b)], c = X[pad(2 * b + 1)];
        X[pad(2 * b)] = cadd(a, c);
        X[pad(2 * b + 1)] = csub(a, c);
    }
    __syncthreads();
}

// forward transform, decimation in frequency: natural order in, bit-reversed order out, in place (used for the
// spectrum of the generator; the convolution kernel runs the same stages, fused with its loads and stores)
__device__ __forceinline__ void fft_forward(float2* X, const float2* __restrict__ tw, int log2p)
{
    int s = log2p - 1;
    for (; s >= 3; s -= 4) fft_trip16<false>(X, tw, s, log2p);
    if (s >= 1) { fft_trip4<false>(X, tw, s, log2p); s -= 2; }
    if (s == 0) fft_bit0(X, log2p);
}

// Walsh-Hadamard stages on the BITS index bits top .. top-BITS+1 of the 2^log2n points in LDS, 2^BITS points per
// thread in registers (one trip through LDS for all of them)
template <int BITS, typename Load>
__device__ __forceinline__ void wht_trip(float2* X, int top, int log2n, Load load)
{
    constexpr int M = 1 << BITS;
    const int qb = top - (BITS - 1), q = 1 << qb;
    for (int b = threadIdx.x; b < (1 << (log2n - BITS)); b += blockDim.x) {
        const int j = b & (q - 1);
        const int i0 = ((b >> qb) << (top + 1)) | j;
        float2 v[M];
#pragma unroll
        for (int k = 0; k < M; ++k) v[k] = load(i0 + (k << qb));
#pragma unroll
        for (int st = 0; st < BITS; ++st)
#pragma unroll
            for (int k = 0; k < M; ++k)
                if (!(k & (1 << st))) {
                    const float2 a = v[k], c = v[k + (1 << st)];
                    v[k] = cadd(a, c);
                    v[k + (1 << st)] = csub(a, c);
                }
#pragma unroll
        for (int k = 0; k < M; ++k) X[pad(i0 + (k << qb))] = v[k];
    }
    __syncthreads();
}

// H D1 x of two vectors, times D2 (reversed for a Hankel block), zero-padded to P; forward transform, product with
// the spectrum, inverse transform.  The first trip of the Hadamard stages reads x from global memory, the last
// inverse trip writes the result there; everything between stays in LDS.
__global__ void __launch_bounds__(512) struct_conv_kernel(StructParams p)
{
    extern __shared__ float2 X[];
    const int L = p.log2p, N = p.log2n;
    const long long v0 = 2LL * blockIdx.x, v1 = v0 + 1;
    const bool two = v1 < p.batch;
    const float* __restrict__ x0 = p.x + v0 * p.n;
    const float* __restrict__ x1 = p.x + (two ? v1 : v0) * p.n;      // a lone last vector is read twice, its copy dropped
    auto from_lds = [&](int i) { return X[pad(i)]; };
    auto to_lds = [&](int i, float2 v) { X[pad(i)] = v; };

    // t = H_u D1 x on the points 0 .. n-1 (H_u the +-1 matrix): four bits per trip, then what is left
    int top = N - 1;
    wht_trip<4>(X, top, N, [&](int i) { const float d = p.d1[i]; return make_float2(x0[i] * d, x1[i] * d); });
    for (top -= 4; top >= 3; top -= 4) wht_trip<4>(X, top, N, from_lds);
    if (top == 2) wht_trip<3>(X, 2, N, from_lds);
    else if (top == 1) wht_trip<2>(X, 1, N, from_lds);
    else if (top == 0) wht_trip<1>(X, 0, N, from_lds);
    if (p.reverse) {                                                  // Hankel: G acts on the reversed vector
        for (int i = threadIdx.x; i < p.n / 2; i += blockDim.x) {
            const float2 a = X[pad(i)], c = X[pad(p.n - 1 - i)];
            X[pad(i)] = c;
            X[pad(p.n - 1 - i)] = a;
        }
        __syncthreads();
    }
    // every point is read and written by the same thread in a trip, so the transforms run in place
    auto padded_times_d2 = [&](int i) {
        const int ic = i < p.n ? i : p.n - 1;                         // clamped: no load under a condition
        const float dd = p.d2[p.reverse ? p.n - 1 - ic : ic];
        const float2 t = X[pad(ic)];
        return i < p.n ? make_float2(t.x * dd, t.y * dd) : make_float2(0.f, 0.f);
    };
    auto to_global = [&](int i, float2 r) {
        if (i < p.m) {
            p.out[v0 * p.m + i] = r.x * p.factor;
            if (two) p.out[v1 * p.m + i] = r.y * p.factor;
        }
    };
    const int low = L & 3;
    // forward: bits L-1 .. low in radix-16 trips (the last one multiplies by the spectrum when no bits are left)
    int s = L - 1;
    fft_trip16<false>(p.tw, s, L, padded_times_d2, to_lds);
    for (s -= 4; s >= 3; s -= 4) {
        if (low == 0 && s == 3) fft_trip16<false>(p.tw, s, L, from_lds, [&](int i, float2 v) { X[pad(i)] = cmul(v, p.spec[i]); });
        else fft_trip16<false>(X, p.tw, s, L);
    }
    if (low == 1) fft_middle<1>(X, p.spec, L);
    else if (low == 2) fft_middle<2>(X, p.spec, L);
    else if (low == 3) fft_middle<3>(X, p.spec, L);
    // inverse: bits low .. L-1
    for (s = low; s + 7 < L; s += 4) fft_trip16<true>(X, p.tw, s + 3, L);
    fft_trip16<true>(p.tw, s + 3, L, from_lds, to_global);
}

// tw[k] = exp(-2 pi i k / P), formed in fp64
__global__ void __launch_bounds__(256) struct_twiddle_kernel(float2* tw, int half_p)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= half_p) return;
    double s, c;
    sincospi((double)k / (double)half_p, &s, &c);
    tw[k] = make_float2((float)c, (float)-s);
}

// Convolution kernel c of the structured matrix: (G v)_i = sum_j c[(i - j) mod P] v_j, then its spectrum.
//   kind 0 circulant       G[i][j] = g[(j - i) mod n]:            c[k] = g[(-k) mod n],            P = n
//   kind 1 skew-circulant  wrapped entries negated:               c[0] = g[0], c[k] = -g[n - k], c[2n - q] = g[q]
//   kind 2 Toeplitz        G[i][j] = t[j - i + n - 1]:            c[k] = t[n - 1 - k], c[2n - q] = t[n - 1 + q]
//   kind 3 Hankel          G[i][j] = h[i + j], v reversed:        Toeplitz with t'[e] = h[2n - 2 - e]
__device__ __forceinline__ float conv_kernel_entry(const float* __restrict__ params, int kind, int n, int k)
{
    float v = 0.f;
    if (kind == 0) {
        v = params[(n - k) & (n - 1)];
    } else if (k < n) {                       // k = i - j >= 0
        if (kind == 1) v = k == 0 ? params[0] : -params[n - k];
        else if (kind == 2) v = params[n - 1 - k];
        else v = params[2 * n - 2 - (n - 1 - k)];
    } else if (k > n) {                       // k = 2n - q, q = j - i > 0
        const int q = 2 * n - k;
        if (kind == 1) v = params[q];
        else if (kind == 2) v = params[n - 1 + q];
        else v = params[2 * n - 2 - (n - 1 + q)];
    }
    return v;
}

__global__ void __launch_bounds__(512) struct_spectrum_kernel(const float* __restrict__ params, int kind, int n, int log2p,
                                                              const float2* __restrict__ tw, float2* __restrict__ spec)
{
    extern __shared__ float2 X[];
    const int P = 1 << log2p;
    for (int k = threadIdx.x; k < P; k += blockDim.x) {
        const float v = conv_kernel_entry(params, kind, n, k);
        X[pad(k)] = make_float2(v, 0.f);
    }
    __syncthreads();
    fft_forward(X, tw, log2p);
    for (int k = threadIdx.x; k < P; k += blockDim.x) spec[k] = X[pad(k)];
}


// ------------------------------------------------------------------ transforms longer than the LDS holds (P = 2^15 .. 2^22)
// The decimation-in-frequency transform of length P = 2^L is split after its top La = L - 12 stages.  Those stages
// pair points 2^12 and more apart: for every offset b below 2^12 they are a transform over the 2^La points
// a 2^12 + b, with twiddles exp(-2 pi i o / 2^(s+1)), o = the point's offset in its group of 2^s.  A workgroup of
// struct_col_kernel takes all a for sixteen or more consecutive b (runs of 128 bytes and up) through LDS, one stage per pass.  The
// twelve stages below act inside each contiguous block of 2^12 points and are the in-LDS transform of that length
// with its own twiddle table (struct_block_kernel), which multiplies by the block's part of the spectrum and runs
// the inverse stages on the way back; the inverse (decimation in time) column stages then mirror the forward ones,
// so the points return to natural order without any reordering pass.  Two real vectors travel as one complex one.
constexpr int kBlockLog = 12;
constexpr int kStructLargeMaxLog2p = kBlockLog + 10;      // a column tile of 2^(La + 4) points must fit the LDS
// consecutive b per column tile (log2): sixteen (128-byte runs) for long columns, more for short ones so that a
// workgroup still has 2^11 points to work on
constexpr int struct_col_log(int log2p) { return 11 - (log2p - kBlockLog) > 4 ? 11 - (log2p - kBlockLog) : 4; }

struct StructLargeParams {
    const float* t;        // [batch][n]: H D1 x (unnormalised), input of the forward column stages
    const float* d2;       // [n]
    float2* z;             // [pairs][P] complex work buffer
    const float2* tw;      // [P/2] exp(-2 pi i k / P)
    const float2* tw_b;    // [2^11] exp(-2 pi i k / 2^12)
    const float2* spec;    // [P] spectrum in the order the forward transform leaves it
    float* out;            // [batch][m]
    long long batch;
    int n, log2p, m, reverse;
    float factor;
    int col_log;
};

enum { COL_FWD_REAL = 0, COL_FWD_COMPLEX = 1, COL_INV_OUT = 2 };

template <int MODE>
__global__ void __launch_bounds__(256) struct_col_kernel(StructLargeParams p)
{
    extern __shared__ float2 X[];
    constexpr bool INVERSE = MODE == COL_INV_OUT;
    const int cl = p.col_log;                                         // log2 of the consecutive b of a tile
    const int L = p.log2p, T = L - kBlockLog + cl;              // index bits of a tile: a above, sixteen b below
    const long long pair = blockIdx.x >> (kBlockLog - cl);
    const int b0 = (int)(blockIdx.x & ((1 << (kBlockLog - cl)) - 1)) << cl;
    const long long v0 = 2 * pair, v1 = v0 + 1;
    const bool two = v1 < p.batch;
    float2* z = p.z + (pair << L);
    auto true_index = [&](int i) { return ((i >> cl) << kBlockLog) | (b0 + (i & ((1 << cl) - 1))); };

    for (int i = threadIdx.x; i < (1 << T); i += 256) {
        const int pt = true_index(i);
        float2 v;
        if constexpr (MODE == COL_FWD_REAL) {
            const int pc = pt < p.n ? pt : p.n - 1;                  // clamped: no load under a condition
            const int q = p.reverse ? p.n - 1 - pc : pc;             // Hankel: G acts on the reversed vector
            const float dd = p.d2[q];
            const float a = p.t[v0 * p.n + q], c = p.t[(two ? v1 : v0) * p.n + q];
            v = pt < p.n ? make_float2(a * dd, c * dd) : make_float2(0.f, 0.f);
        } else {
            v = z[pt];
        }
        X[pad(i)] = v;
    }
    __syncthreads();
    for (int step = 0; step < T - cl; ++step) {
        const int t = INVERSE ? cl + step : T - 1 - step;       // tile bit of this stage
        const int s = t - cl + kBlockLog;                        // its bit in the transform
        for (int bf = threadIdx.x; bf < (1 << (T - 1)); bf += 256) {
            const int o = bf & ((1 << t) - 1);
            const int lo = ((bf >> t) << (t + 1)) | o;
            const int ot = ((o >> cl) << kBlockLog) | (b0 + (o & ((1 << cl) - 1)));      // offset in the group of 2^s
            float2 a = X[pad(lo)], c = X[pad(lo + (1 << t))];
            butterfly<INVERSE>(a, c, p.tw[(long long)ot << (L - 1 - s)]);
            X[pad(lo)] = a;
            X[pad(lo + (1 << t))] = c;
        }
        __syncthreads();
    }
    for (int i = threadIdx.x; i < (1 << T); i += 256) {
        const int pt = true_index(i);
        const float2 v = X[pad(i)];
        if constexpr (MODE == COL_INV_OUT) {
            if (pt < p.m) {
                p.out[v0 * p.m + pt] = v.x * p.factor;
                if (two) p.out[v1 * p.m + pt] = v.y * p.factor;
            }
        } else {
            z[pt] = v;
        }
    }
}

// The same column stages for short columns (LA = 3 or 4 stages, transforms of 2^15 and 2^16 points): a thread holds the
// 2^LA points a 2^12 + b of one b in registers and runs all stages there; consecutive threads take consecutive b.
template <int MODE, int LA>
__global__ void __launch_bounds__(256) struct_col_reg_kernel(StructLargeParams p)
{
    constexpr bool INVERSE = MODE == COL_INV_OUT;
    constexpr int M = 1 << LA, L = kBlockLog + LA;
    const long long gid = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long pair = gid >> kBlockLog;
    const int b = (int)(gid & ((1 << kBlockLog) - 1));
    const long long v0 = 2 * pair, v1 = v0 + 1;
    const bool two = v1 < p.batch;
    float2* z = p.z + (pair << L);
    float2 v[M];
#pragma unroll
    for (int a = 0; a < M; ++a) {
        const int pt = (a << kBlockLog) | b;
        if constexpr (MODE == COL_FWD_REAL) {
            const int pc = pt < p.n ? pt : p.n - 1;
            const int q = p.reverse ? p.n - 1 - pc : pc;
            const float dd = p.d2[q];
            const float x0 = p.t[v0 * p.n + q], x1 = p.t[(two ? v1 : v0) * p.n + q];
            v[a] = pt < p.n ? make_float2(x0 * dd, x1 * dd) : make_float2(0.f, 0.f);
        } else {
            v[a] = z[pt];
        }
    }
#pragma unroll
    for (int step = 0; step < LA; ++step) {
        const int t = INVERSE ? step : LA - 1 - step;             // bit of a
        const int s = t + kBlockLog;
#pragma unroll
        for (int a = 0; a < M; ++a)
            if (!(a & (1 << t))) {
                const int ot = ((a & ((1 << t) - 1)) << kBlockLog) | b;      // offset in the group of 2^s
                butterfly<INVERSE>(v[a], v[a | (1 << t)], p.tw[ot << (L - 1 - s)]);
            }
    }
#pragma unroll
    for (int a = 0; a < M; ++a) {
        const int pt = (a << kBlockLog) | b;
        if constexpr (MODE == COL_INV_OUT) {
            if (pt < p.m) {
                p.out[v0 * p.m + pt] = v[a].x * p.factor;
                if (two) p.out[v1 * p.m + pt] = v[a].y * p.factor;
            }
        } else {
            z[pt] = v[a];
        }
    }
}

// The twelve low stages of one block of 2^12 points: forward, product with the spectrum, inverse, in place
// (FORWARD_ONLY: forward alone, for the spectrum of the generator).
template <bool FORWARD_ONLY>
__global__ void __launch_bounds__(256) struct_block_kernel(StructLargeParams p)
{
    extern __shared__ float2 X[];
    constexpr int L = kBlockLog;
    float2* z = p.z + ((long long)blockIdx.x << L);                  // block (pair, a): blocks of a pair are consecutive
    const float2* spec = p.spec + (((long long)blockIdx.x & ((1LL << (p.log2p - L)) - 1)) << L);
    auto from_lds = [&](int i) { return X[pad(i)]; };
    auto to_lds = [&](int i, float2 v) { X[pad(i)] = v; };
    fft_trip16<false>(p.tw_b, 11, L, [&](int i) { return z[i]; }, to_lds);
    fft_trip16<false>(X, p.tw_b, 7, L);
    if constexpr (FORWARD_ONLY) {
        fft_trip16<false>(p.tw_b, 3, L, from_lds, [&](int i, float2 v) { z[i] = v; });
    } else {
        fft_trip16<false>(p.tw_b, 3, L, from_lds, [&](int i, float2 v) { X[pad(i)] = cmul(v, spec[i]); });
        fft_trip16<true>(X, p.tw_b, 3, L);
        fft_trip16<true>(X, p.tw_b, 7, L);
        fft_trip16<true>(p.tw_b, 11, L, from_lds, [&](int i, float2 v) { z[i] = v; });
    }
}

// c[k] of the structured matrix as complex points in global memory (the generator of a long transform)
__global__ void __launch_bounds__(256) struct_fill_kernel(const float* __restrict__ params, int kind, int n, int log2p, float2* __restrict__ c)
{
    const long long k = (long long)blockIdx.x * 256 + threadIdx.x;
    if (k < (1LL << log2p)) c[k] = make_float2(conv_kernel_entry(params, kind, n, (int)k), 0.f);
}

static hipError_t allow_lds(const void* kernel, size_t bytes)
{
    return bytes > 65536 ? hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) : hipSuccess;
}

hipError_t launch_struct_prepare(const float* params, int kind, int n, int log2p, float2* spec, float2* tw, hipStream_t s)
{
    const int P = 1 << log2p;
    hipLaunchKernelGGL(struct_twiddle_kernel, dim3((P / 2 + 255) / 256), dim3(256), 0, s, tw, P / 2);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t lds = fft_lds_bytes(log2p);
    if ((e = allow_lds(reinterpret_cast<const void*>(struct_spectrum_kernel), lds)) != hipSuccess) return e;
    hipLaunchKernelGGL(struct_spectrum_kernel, dim3(1), dim3(512), lds, s, params, kind, n, log2p, tw, spec);
    return hipGetLastError();
}

hipError_t launch_struct_conv(const float* x, const float* d1, const float* d2, const float2* spec, const float2* tw, float* out,
                              long long batch, int n, int log2n, int log2p, int m, int reverse, float factor, hipStream_t s)
{
    if (batch <= 0) return hipSuccess;
    const long long blocks = (batch + 1) / 2;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    const size_t lds = fft_lds_bytes(log2p);
    hipError_t e = allow_lds(reinterpret_cast<const void*>(struct_conv_kernel), lds);
    if (e != hipSuccess) return e;
    StructParams p{x, d1, d2, spec, tw, out, batch, n, log2p, m, reverse, factor, log2n};
    // one thread per sixteen points of the transform
    const int threads = (1 << log2p) / 16 < 64 ? 64 : ((1 << log2p) / 16 > 512 ? 512 : (1 << log2p) / 16);
    hipLaunchKernelGGL(struct_conv_kernel, dim3((unsigned)blocks), dim3(threads), lds, s, p);
    return hipGetLastError();
}

template <int MODE>
static hipError_t launch_struct_col(const StructLargeParams& p, long long pairs, hipStream_t s)
{
    const int la = p.log2p - kBlockLog;
    if (la == 3 || la == 4) {
        const unsigned blocks = (unsigned)((pairs << kBlockLog) / 256);
        if (la == 3) hipLaunchKernelGGL((struct_col_reg_kernel<MODE, 3>), dim3(blocks), dim3(256), 0, s, p);
        else hipLaunchKernelGGL((struct_col_reg_kernel<MODE, 4>), dim3(blocks), dim3(256), 0, s, p);
        return hipGetLastError();
    }
    const size_t lds_col = fft_lds_bytes(la + p.col_log);
    const hipError_t e = allow_lds(reinterpret_cast<const void*>(struct_col_kernel<MODE>), lds_col);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(struct_col_kernel<MODE>, dim3((unsigned)(pairs << (kBlockLog - p.col_log))), dim3(256), lds_col, s, p);
    return hipGetLastError();
}

// spectrum of a generator whose transform does not fit the LDS: [P] spectrum, [P/2] twiddles, [2^11] twiddles of the blocks
hipError_t launch_struct_prepare_large(const float* params, int kind, int n, int log2p, float2* spec, float2* tw, float2* tw_b,
                                       hipStream_t s)
{
    if (log2p <= kBlockLog + 2 || log2p > kStructLargeMaxLog2p) return hipErrorInvalidValue;
    const long long P = 1LL << log2p;
    hipLaunchKernelGGL(struct_twiddle_kernel, dim3((unsigned)((P / 2 + 255) / 256)), dim3(256), 0, s, tw, (int)(P / 2));
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(struct_twiddle_kernel, dim3((1 << (kBlockLog - 1)) / 256), dim3(256), 0, s, tw_b, 1 << (kBlockLog - 1));
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(struct_fill_kernel, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, s, params, kind, n, log2p, spec);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const int cl = struct_col_log(log2p);
    StructLargeParams p{nullptr, nullptr, spec, tw, tw_b, nullptr, nullptr, 1, n, log2p, 0, 0, 1.0f, cl};
    const size_t lds_blk = fft_lds_bytes(kBlockLog);
    if ((e = launch_struct_col<COL_FWD_COMPLEX>(p, 1, s)) != hipSuccess) return e;
    hipLaunchKernelGGL(struct_block_kernel<true>, dim3(1 << (log2p - kBlockLog)), dim3(256), lds_blk, s, p);
    return hipGetLastError();
}

// t: H D1 x (unnormalised) [batch][n]; z: ceil(batch / 2) * P complex points of scratch
hipError_t launch_struct_conv_large(const float* t, const float* d2, const float2* spec, const float2* tw, const float2* tw_b, float2* z,
                                    float* out, long long batch, int n, int log2p, int m, int reverse, float factor, hipStream_t s)
{
    if (batch <= 0) return hipSuccess;
    if (log2p <= kBlockLog + 2 || log2p > kStructLargeMaxLog2p) return hipErrorInvalidValue;
    const long long pairs = (batch + 1) / 2;
    const int cl = struct_col_log(log2p);
    if ((pairs << (log2p - kBlockLog)) > 0x7fffffffLL || (pairs << (kBlockLog - cl)) > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    StructLargeParams p{t, d2, z, tw, tw_b, spec, out, batch, n, log2p, m, reverse, factor, cl};
    const size_t lds_blk = fft_lds_bytes(kBlockLog);
    hipError_t e;
    if ((e = launch_struct_col<COL_FWD_REAL>(p, pairs, s)) != hipSuccess) return e;
    hipLaunchKernelGGL(struct_block_kernel<false>, dim3((unsigned)(pairs << (log2p - kBlockLog))), dim3(256), lds_blk, s, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    return launch_struct_col<COL_INV_OUT>(p, pairs, s);
}
}  // namespace spinner
