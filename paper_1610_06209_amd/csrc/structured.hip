// The G_struct D2 H D1 members of the family: third block a circulant, skew-circulant, Toeplitz or Hankel
// matrix given by its generating vector.  H D1 x comes from the tile kernels; the product with G_struct is a
// cyclic convolution of length P (n for a circulant, 2n otherwise) done by a complex FFT held in LDS.  Two
// real vectors share one complex transform (the generator is real, so real and imaginary part stay apart).
#include "launch.hpp"
namespace spinner {

struct StructParams {
    const float* t;        // [batch][n]: H D1 x
    const float* d2;       // [n]
    const float2* spec;    // [P] spectrum of the convolution kernel, in the order the forward transform leaves it
    const float2* tw;      // [P/2] exp(-2 pi i k / P)
    float* out;            // [batch][m]
    long long batch;
    int n, log2p, m, reverse;
    float factor;          // scale / P
};

__device__ __forceinline__ float2 cmul(float2 a, float2 b) { return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x); }
__device__ __forceinline__ float2 cmul_conj(float2 a, float2 b) { return make_float2(a.x * b.x + a.y * b.y, a.y * b.x - a.x * b.y); }

__device__ __forceinline__ float2 cadd(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ float2 csub(float2 a, float2 b) { return make_float2(a.x - b.x, a.y - b.y); }

// forward transform, decimation in frequency: natural order in, bit-reversed order out.  Two radix-2 stages
// (index bits s and s-1) are done per trip through LDS on four points held in registers; a last single
// stage is left when the number of stages is odd.  The stage on bit s pairs points 2^s apart and multiplies
// the difference by exp(-2 pi i j / 2^(s+1)), j the offset inside the lower half.
__device__ __forceinline__ void fft_forward(float2* X, const float2* __restrict__ tw, int log2p)
{
    int s = log2p - 1;
    for (; s >= 1; s -= 2) {
        const int q = 1 << (s - 1);                         // quarter of the 2^(s+1)-point group
        for (int b = threadIdx.x; b < (1 << (log2p - 2)); b += blockDim.x) {
            const int j = b & (q - 1);
            const int i0 = ((b >> (s - 1)) << (s + 1)) | j;
            const float2 a0 = X[i0], a1 = X[i0 + q], a2 = X[i0 + 2 * q], a3 = X[i0 + 3 * q];
            const int sh = log2p - 1 - s;
            const float2 b0 = cadd(a0, a2), b2 = cmul(csub(a0, a2), tw[j << sh]);
            const float2 b1 = cadd(a1, a3), b3 = cmul(csub(a1, a3), tw[(j + q) << sh]);
            const float2 w = tw[j << (sh + 1)];
            X[i0] = cadd(b0, b1);
            X[i0 + q] = cmul(csub(b0, b1), w);
            X[i0 + 2 * q] = cadd(b2, b3);
            X[i0 + 3 * q] = cmul(csub(b2, b3), w);
        }
        __syncthreads();
    }
    if (s == 0) {                                           // bit 0: twiddle 1
        for (int b = threadIdx.x; b < (1 << (log2p - 1)); b += blockDim.x) {
            const float2 a = X[2 * b], c = X[2 * b + 1];
            X[2 * b] = cadd(a, c);
            X[2 * b + 1] = csub(a, c);
        }
        __syncthreads();
    }
}

// inverse transform (unnormalised), decimation in time: bit-reversed order in, natural order out; the
// mirror image of fft_forward with conjugate twiddles (bit 0 first when the number of stages is odd).
__device__ __forceinline__ void fft_inverse(float2* X, const float2* __restrict__ tw, int log2p)
{
    int s = 0;
    if (log2p & 1) {
        for (int b = threadIdx.x; b < (1 << (log2p - 1)); b += blockDim.x) {
            const float2 a = X[2 * b], c = X[2 * b + 1];
            X[2 * b] = cadd(a, c);
            X[2 * b + 1] = csub(a, c);
        }
        __syncthreads();
        s = 1;
    }
    for (; s + 1 < log2p; s += 2) {                         // bits s and s+1
        const int q = 1 << s;
        for (int b = threadIdx.x; b < (1 << (log2p - 2)); b += blockDim.x) {
            const int j = b & (q - 1);
            const int i0 = ((b >> s) << (s + 2)) | j;
            const float2 a0 = X[i0], a1 = X[i0 + q], a2 = X[i0 + 2 * q], a3 = X[i0 + 3 * q];
            const int sh = log2p - 1 - s;
            const float2 w = tw[j << sh];
            const float2 t1 = cmul_conj(a1, w), t3 = cmul_conj(a3, w);
            const float2 b0 = cadd(a0, t1), b1 = csub(a0, t1), b2 = cadd(a2, t3), b3 = csub(a2, t3);
            const float2 u2 = cmul_conj(b2, tw[j << (sh - 1)]), u3 = cmul_conj(b3, tw[(j + q) << (sh - 1)]);
            X[i0] = cadd(b0, u2);
            X[i0 + 2 * q] = csub(b0, u2);
            X[i0 + q] = cadd(b1, u3);
            X[i0 + 3 * q] = csub(b1, u3);
        }
        __syncthreads();
    }
}

__global__ void __launch_bounds__(512) struct_conv_kernel(StructParams p)
{
    extern __shared__ float2 X[];
    const int P = 1 << p.log2p;
    const long long v0 = 2LL * blockIdx.x, v1 = v0 + 1;
    const bool two = v1 < p.batch;
    for (int i = threadIdx.x; i < P; i += blockDim.x) {
        float re = 0.f, im = 0.f;
        if (i < p.n) {
            const int si = p.reverse ? p.n - 1 - i : i;
            const float dd = p.d2[si];
            re = p.t[v0 * p.n + si] * dd;
            if (two) im = p.t[v1 * p.n + si] * dd;
        }
        X[i] = make_float2(re, im);
    }
    __syncthreads();
    fft_forward(X, p.tw, p.log2p);
    for (int i = threadIdx.x; i < P; i += blockDim.x) X[i] = cmul(X[i], p.spec[i]);
    __syncthreads();
    fft_inverse(X, p.tw, p.log2p);
    for (int i = threadIdx.x; i < p.m; i += blockDim.x) {
        const float2 r = X[i];
        p.out[v0 * p.m + i] = r.x * p.factor;
        if (two) p.out[v1 * p.m + i] = r.y * p.factor;
    }
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
__global__ void __launch_bounds__(512) struct_spectrum_kernel(const float* __restrict__ params, int kind, int n, int log2p,
                                                              const float2* __restrict__ tw, float2* __restrict__ spec)
{
    extern __shared__ float2 X[];
    const int P = 1 << log2p;
    for (int k = threadIdx.x; k < P; k += blockDim.x) {
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
        X[k] = make_float2(v, 0.f);
    }
    __syncthreads();
    fft_forward(X, tw, log2p);
    for (int k = threadIdx.x; k < P; k += blockDim.x) spec[k] = X[k];
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
    const size_t lds = (size_t)P * sizeof(float2);
    if ((e = allow_lds(reinterpret_cast<const void*>(struct_spectrum_kernel), lds)) != hipSuccess) return e;
    hipLaunchKernelGGL(struct_spectrum_kernel, dim3(1), dim3(512), lds, s, params, kind, n, log2p, tw, spec);
    return hipGetLastError();
}

hipError_t launch_struct_conv(const float* t, const float* d2, const float2* spec, const float2* tw, float* out, long long batch,
                              int n, int log2p, int m, int reverse, float factor, hipStream_t s)
{
    if (batch <= 0) return hipSuccess;
    const long long blocks = (batch + 1) / 2;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    const size_t lds = ((size_t)1 << log2p) * sizeof(float2);
    hipError_t e = allow_lds(reinterpret_cast<const void*>(struct_conv_kernel), lds);
    if (e != hipSuccess) return e;
    StructParams p{t, d2, spec, tw, out, batch, n, log2p, m, reverse, factor};
    hipLaunchKernelGGL(struct_conv_kernel, dim3((unsigned)blocks), dim3(512), lds, s, p);
    return hipGetLastError();
}
}  // namespace spinner
