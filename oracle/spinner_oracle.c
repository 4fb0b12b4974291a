/*
 * TEST INFRASTRUCTURE - NOT PART OF THE PRODUCT PATH.
 *
 * Plain, slow, dense-matrix CPU oracle for the structured spinner
 *     y = H D3 H D2 H D1 x
 * (Structured Spinners, Section 1 and Section 3: H is the L2-normalised
 * Hadamard matrix, D_i are diagonal matrices, either random +-1 or arbitrary
 * "adaptive" ones; Lemma 1 lists sqrt(n) H D3 H D2 H D1 and the variant with
 * a Gaussian third diagonal as members of the family).
 *
 * The fast method reaches this result exactly (up to rounding order), so the
 * oracle is the definition written out: every H is a materialised n x n
 * matrix of +-1 entries (Sylvester / natural order, entry (i,j) is
 * (-1)^popcount(i & j)), every product is an O(n^2) matrix-vector product
 * accumulated in fp64, every diagonal is an explicit elementwise multiply.
 * There is no butterfly, no blocking, no fusion.
 *
 * For n too large to materialise H_n (n > 2^14) the oracle materialises the
 * two Kronecker factors of H_n = H_a (x) H_b (n = a*b) and applies
 * vec(H_a X H_b^T) with X the row-major a x b reshape of the vector.  The
 * factorisation itself is pinned entrywise against the popcount formula by
 * the CPU tests.
 *
 * Only tests/, the smoke check and the benchmark's cpu_baseline leg may call
 * this file.  It shares no code with the HIP path.
 *
 * Parallelism: OpenMP over vectors only (each vector is computed by one
 * thread with the plain loops below).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* +1 / -1 entry of the unnormalised Sylvester Hadamard matrix. */
int oracle_hadamard_sign(uint64_t i, uint64_t j)
{
    return (__builtin_popcountll(i & j) & 1) ? -1 : 1;
}

/* Fill H[n*n] (row-major int8) with the unnormalised Sylvester matrix. */
void oracle_hadamard_dense(int n, int8_t *H)
{
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j)
            H[(size_t)i * n + j] = (int8_t)oracle_hadamard_sign((uint64_t)i, (uint64_t)j);
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* out = (Hn / sqrt(n)) in,   Hn dense n x n. */
static void normalised_hadamard_matvec(int n, const int8_t *H, const double *in, double *out)
{
    const double inv_sqrt_n = 1.0 / sqrt((double)n);
    for (int i = 0; i < n; ++i) {
        const int8_t *row = H + (size_t)i * n;
        double acc = 0.0;
        for (int j = 0; j < n; ++j)
            acc += (double)row[j] * in[j];
        out[i] = acc * inv_sqrt_n;
    }
}

/*
 * out = ((Ha (x) Hb) / sqrt(a*b)) in, with in viewed as the row-major a x b
 * matrix X (element r*b + c): out = vec(Ha X Hb^T).
 * tmp has a*b doubles.
 */
static void normalised_hadamard_matvec_kron(int a, int b, const int8_t *Ha, const int8_t *Hb,
                                            const double *in, double *tmp, double *out)
{
    const double inv_sqrt_n = 1.0 / sqrt((double)a * (double)b);
    /* tmp = X Hb^T : tmp[r][c] = sum_c' Hb[c][c'] X[r][c'] */
    for (int r = 0; r < a; ++r)
        for (int c = 0; c < b; ++c) {
            const int8_t *hrow = Hb + (size_t)c * b;
            const double *xrow = in + (size_t)r * b;
            double acc = 0.0;
            for (int cc = 0; cc < b; ++cc)
                acc += (double)hrow[cc] * xrow[cc];
            tmp[(size_t)r * b + c] = acc;
        }
    /* out = Ha tmp : out[r][c] = sum_r' Ha[r][r'] tmp[r'][c] */
    for (int r = 0; r < a; ++r) {
        double *orow = out + (size_t)r * b;
        for (int c = 0; c < b; ++c)
            orow[c] = 0.0;
        for (int rr = 0; rr < a; ++rr) {
            const double h = (double)Ha[(size_t)r * a + rr];
            const double *trow = tmp + (size_t)rr * b;
            for (int c = 0; c < b; ++c)
                orow[c] += h * trow[c];
        }
        for (int c = 0; c < b; ++c)
            orow[c] *= inv_sqrt_n;
    }
}

static int is_pow2(long v) { return v > 0 && (v & (v - 1)) == 0; }

/*
 * One normalised Hadamard product on `batch` fp64 vectors (used by the CPU
 * tests to pin H on its own: isometry, involution, balancedness).
 * kron_a == 0: dense H_n.  kron_a > 0: H_n = H_a (x) H_{n/a}.
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int oracle_hadamard_apply(const double *in, int n, long batch, int kron_a, double *out)
{
    if (!in || !out || !is_pow2(n) || batch < 0)
        return -1;
    if (kron_a) {
        if (!is_pow2(kron_a) || kron_a > n)
            return -1;
        const int a = kron_a, b = n / kron_a;
        int8_t *Ha = malloc((size_t)a * a), *Hb = malloc((size_t)b * b);
        if (!Ha || !Hb) { free(Ha); free(Hb); return -1; }
        oracle_hadamard_dense(a, Ha);
        oracle_hadamard_dense(b, Hb);
        int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
        for (long v = 0; v < batch; ++v) {
            double *tmp = malloc(sizeof(double) * (size_t)n);
            if (!tmp) { fail = 1; continue; }
            normalised_hadamard_matvec_kron(a, b, Ha, Hb, in + (size_t)v * n, tmp, out + (size_t)v * n);
            free(tmp);
        }
        free(Ha); free(Hb);
        return fail ? -1 : 0;
    }
    int8_t *H = malloc((size_t)n * n);
    if (!H) return -1;
    oracle_hadamard_dense(n, H);
#pragma omp parallel for schedule(dynamic, 1)
    for (long v = 0; v < batch; ++v)
        normalised_hadamard_matvec(n, H, in + (size_t)v * n, out + (size_t)v * n);
    free(H);
    return 0;
}

/*
 * y[v] = H D3 H D2 H D1 x[v] for v in [0, batch), fp64 throughout.
 *   x      : fp32 [batch][n] (the exact bits handed to the GPU path, widened)
 *   d1..d3 : fp32 [n] diagonals (any values; +-1 in the random setting)
 *   y      : fp64 [batch][n]
 *   kron_a : 0 -> dense H_n (needs n*n bytes); > 0 -> H_n = H_a (x) H_{n/a}
 *   nthreads: 0 -> OpenMP default
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int oracle_spinner(const float *x, int n, long batch, const float *d1, const float *d2,
                   const float *d3, int kron_a, int nthreads, double *y)
{
    if (!x || !d1 || !d2 || !d3 || !y || !is_pow2(n) || batch < 0)
        return -1;
    if (kron_a && (!is_pow2(kron_a) || kron_a > n))
        return -1;
#ifdef _OPENMP
    if (nthreads > 0)
        omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
    const float *diag[3] = { d1, d2, d3 };
    const int a = kron_a ? kron_a : n, b = kron_a ? n / kron_a : 1;
    int8_t *Ha = malloc((size_t)a * a), *Hb = NULL;
    if (!Ha) return -1;
    oracle_hadamard_dense(a, Ha);
    if (kron_a) {
        Hb = malloc((size_t)b * b);
        if (!Hb) { free(Ha); return -1; }
        oracle_hadamard_dense(b, Hb);
    }
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long v = 0; v < batch; ++v) {
        double *t = malloc(sizeof(double) * (size_t)n);
        double *u = malloc(sizeof(double) * (size_t)n);
        double *tmp = kron_a ? malloc(sizeof(double) * (size_t)n) : NULL;
        if (!t || !u || (kron_a && !tmp)) { fail = 1; free(t); free(u); free(tmp); continue; }
        for (int i = 0; i < n; ++i)
            t[i] = (double)x[(size_t)v * n + i];
        for (int round = 0; round < 3; ++round) {
            for (int i = 0; i < n; ++i)          /* t <- D_round t */
                t[i] = (double)diag[round][i] * t[i];
            if (kron_a)                          /* u <- H t */
                normalised_hadamard_matvec_kron(a, b, Ha, Hb, t, tmp, u);
            else
                normalised_hadamard_matvec(n, Ha, t, u);
            memcpy(t, u, sizeof(double) * (size_t)n);
        }
        memcpy(y + (size_t)v * n, t, sizeof(double) * (size_t)n);
        free(t); free(u); free(tmp);
    }
    free(Ha); free(Hb);
    return fail ? -1 : 0;
}
