/*
 * spinner.h - C ABI of the MI355X (gfx950) structured-spinner library.
 *
 * The library computes, for a batch of fp32 vectors, the structured projection
 *
 *        y = H D3 H D2 H D1 x
 *
 * of "Structured Spinners" (Section 1; Section 3, Lemma 1), where H is the
 * L2-normalised Hadamard matrix in Sylvester (natural) order, entry (i,j) =
 * (-1)^popcount(i & j) / sqrt(n), and D1, D2, D3 are diagonal matrices given by
 * their fp32 diagonals (+-1 in the random setting, arbitrary in the adaptive
 * one, Gaussian D3 for the H D_g H D2 H D1 member).  H is never materialised:
 * each H is a fast Walsh-Hadamard transform that runs entirely on the GPU.
 * The projection is fused with the step that consumes it (Section 1 notes that
 * the projected data usually go straight into some nonlinear function).
 *
 * Conventions shared by every entry point
 *   - All data pointers are DEVICE pointers unless stated otherwise, must be
 *     16-byte aligned, and are owned by the caller.  The library never
 *     allocates, frees or synchronises; all work is enqueued on `stream`
 *     (a hipStream_t passed as void*, NULL = the default stream).  Buffers
 *     must stay alive until the stream has run the call.
 *   - Vectors are row-major and contiguous: x is fp32 [batch][n].
 *   - n must be a power of two in [2^4, 2^24].  Zero-padding other sizes is
 *     the caller's job.
 *   - Return value: SPINNER_OK (0) or a negative SPINNER_ERR_* code.  All
 *     validation happens before the first launch; a failed call enqueues
 *     nothing.  batch == 0 is a successful no-op.
 */
#ifndef SPINNER_H
#define SPINNER_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SPINNER_OK               =  0,
    SPINNER_ERR_BAD_N        = -1,  /* n not a power of two or outside [2^4, 2^24]          */
    SPINNER_ERR_BAD_M        = -2,  /* m < 1 or m > n                                       */
    SPINNER_ERR_NULL_PTR     = -3,  /* a required pointer is NULL                           */
    SPINNER_ERR_BAD_EPILOGUE = -4,  /* epilogue is not one of spinner_epilogue_t            */
    SPINNER_ERR_BAD_BATCH    = -5,  /* batch < 0, or batch * n does not fit the index range */
    SPINNER_ERR_WORKSPACE    = -6,  /* workspace required (see spinner_workspace_bytes) but NULL */
    SPINNER_ERR_HIP          = -7,  /* a kernel launch failed; see spinner_strerror         */
    SPINNER_ERR_BAD_L        = -8,  /* L < 1                                                */
    SPINNER_ERR_ALIGNMENT    = -9,  /* a data pointer is not 16-byte aligned                */
    SPINNER_ERR_UNSUPPORTED  = -10, /* combination not built (e.g. hashing with n > 2^16)   */
    SPINNER_ERR_SCRATCH_LIMIT = -11 /* needs more scratch than the built-in buffer of an allocation-free entry point */
};

typedef enum {
    /* out[batch][m]  = scale * (first m coordinates of y).
     * Section 3.2: an m x n spinner is the first m rows of the n x n one.      */
    SPINNER_EPI_NONE = 0,
    /* out[batch][2m] = (1/sqrt(m)) [cos(w_0..w_{m-1}), sin(w_0..w_{m-1})],
     * w = scale * y.  Section 5 (kernel approximation): random Fourier features
     * s(Ax) = exp(-i A x / sigma) scaled by 1/sqrt(d'), in real form; with
     * A = sqrt(n) H D3 H D2 H D1 pass scale = sqrt(n) / sigma.                  */
    SPINNER_EPI_COSSIN = 1
} spinner_epilogue_t;

/*
 * Apply one spinner (one triple of diagonals) to a batch and run an epilogue.
 *
 *   x         in   device fp32 [batch][n]; never written
 *   n         in   vector length, power of two in [2^4, 2^24]
 *   batch     in   number of vectors, >= 0
 *   d1,d2,d3  in   device fp32 [n] each: the diagonals of D1, D2, D3
 *   m         in   number of leading coordinates kept, 1 <= m <= n
 *   epilogue  in   spinner_epilogue_t
 *   scale     in   caller's factor on top of the normalised transform
 *                  (1 for the plain spinner, sqrt(n/m) for a norm-preserving
 *                  reduction, sqrt(n)/sigma for Gaussian-kernel features)
 *   out       out  device fp32 [batch][m] (NONE) or [batch][2m] (COSSIN).
 *                  May alias x only when n <= 2^16, m == n and epilogue is NONE.
 *   workspace      device scratch of spinner_workspace_bytes(...) bytes, or
 *                  NULL when that is 0
 *   stream         hipStream_t
 *
 * Up to the fused limit (n <= 2^16 for SPINNER_EPI_NONE, n <= 2^14 for
 * SPINNER_EPI_COSSIN) one kernel keeps the vector on chip for all three sign-flip +
 * transform rounds.  Above it the call makes four passes over HBM using the
 * Kronecker structure H_{ab} = H_a (x) H_b of the Sylvester matrix; intermediate
 * passes run in place in `out` when m == n, else in `workspace`.
 *
 * Accuracy: outputs of SPINNER_EPI_NONE carry the rounding of 3 log2 n fp32
 * butterfly stages (relative L2 error of a few 1e-7 per vector).  The fused
 * feature kernels (SPINNER_EPI_COSSIN, n <= 2^14) run their butterflies and the
 * reduction of w in fp64, so the unit-norm feature vector is good to 1e-5
 * relative at any scale.  Above 2^14 the four passes are fp32: each angle w
 * then carries an error of about 3.4e-8 * sqrt(3 log2 n) * rms(w) radians,
 * which is also the relative L2 error of the feature vector, i.e. at most
 * max(1e-5, 5e-7 * rms(w)); with scale = sqrt(n) / sigma that exceeds 1e-5
 * once |x| / sigma is above about 40.
 */
int spinner_apply(const float *x, int n, long batch,
                  const float *d1, const float *d2, const float *d3,
                  int m, int epilogue, float scale,
                  float *out, void *workspace, void *stream);

/*
 * Cross-polytope LSH (Section 4, Theorem 4): for each vector and each of L
 * independently drawn diagonal triples (Section 3.2: independently constructed
 * blocks), the hash is the signed canonical direction closest to the
 * projection: i* = argmax_i |y_i| (lowest index on exact ties), bucket = i* if
 * y_{i*} >= 0 else i* + n.  x is read once for all L triples.
 *
 *   x          in   device fp32 [batch][n]
 *   L          in   number of triples, >= 1
 *   diag_sets  in   device fp32 [L][3][n], order d1, d2, d3 within a triple
 *   out_idx    out  device int32 [batch][L], values in [0, 2n)
 *
 * Supported for n <= 2^16 (SPINNER_ERR_UNSUPPORTED above that: the call has no
 * workspace for the four-pass path; spinner_hash_ws does).  Up to n = 2^14 one
 * kernel keeps x in registers for all L triples; at n = 2^15 and 2^16 a vector
 * fills the registers of a workgroup and every triple is a launch of its own.
 */
int spinner_hash(const float *x, int n, long batch, int L,
                 const float *diag_sets, int *out_idx, void *stream);

/*
 * The same hash for every n in [2^4, 2^24].  Above 2^16 each triple runs the
 * four-pass projection into the workspace and the bucket is taken from there by
 * two small kernels (same rules: largest |y_i|, lowest index on exact ties, a
 * zero counts as positive); x is then read once per triple.  Up to 2^16 the
 * call is spinner_hash and the workspace may be NULL.
 *
 *   workspace  in   device scratch of spinner_hash_workspace_bytes(n, batch)
 *                   bytes (0 for n <= 2^16), 16-byte aligned;
 *                   SPINNER_ERR_WORKSPACE if it is needed and NULL
 * spinner_hash_signs_ws is the variant for packed sign words (see below).
 */
size_t spinner_hash_workspace_bytes(int n, long batch);
int spinner_hash_ws(const float *x, int n, long batch, int L,
                    const float *diag_sets, int *out_idx, void *workspace, void *stream);

/*
 * Random setting, parameters prepared in advance.  In the random setting the
 * diagonals are drawn from {-1,+1} (Section 3, notation paragraph), and the
 * paper's own timings prepare all parameters of the matrix beforehand and put
 * only the matrix-vector products on the clock (Section 5).  For such
 * diagonals only one bit per entry matters: spinner_pack_signs turns L triples
 * of fp32 diagonals into the library's packed sign words once, and
 * spinner_apply_signs / spinner_hash_signs then compute exactly what
 * spinner_apply / spinner_hash compute for those diagonals without reading the
 * fp32 diagonals again (the sign words travel through the scalar cache).
 *
 *   diag_sets  in   device fp32 [L][3][n]; only the SIGN BIT of each entry is
 *                   used, so entries are expected to be exactly +1 or -1
 *   signs      out  device buffer of spinner_signs_bytes(n, L) bytes, 16-byte
 *                   aligned, opaque; triple l starts at byte
 *                   l * spinner_signs_bytes(n, 1)
 *
 * spinner_apply_signs uses the first triple found at `signs`; all other
 * arguments, the output, the workspace rule and the error codes are those of
 * spinner_apply.  For n > 2^14 the buffer also holds the lane masks with
 * which the four-pass path flips signs in its pass over columns (its passes
 * over rows use the sign words), and at n = 2^15 a copy of the fp32
 * diagonals: about n / 2 bytes per triple otherwise.
 */
size_t spinner_signs_bytes(int n, int L);
int spinner_pack_signs(const float *diag_sets, int n, int L, void *signs, void *stream);
int spinner_apply_signs(const float *x, int n, long batch, const void *signs,
                        int m, int epilogue, float scale,
                        float *out, void *workspace, void *stream);
int spinner_hash_signs(const float *x, int n, long batch, int L,
                       const void *signs, int *out_idx, void *stream);
int spinner_hash_signs_ws(const float *x, int n, long batch, int L,
                          const void *signs, int *out_idx, void *workspace, void *stream);

/*
 * Stacked blocks (Section 3.2: independently constructed m x n spinners stacked
 * vertically give a k x n matrix, k = L m, for k <= n and k > n alike; Section 5
 * uses this when more random features than input dimensions are wanted).
 * spinner_apply_blocks applies L independent triples to the same x and writes the
 * L blocks side by side:
 *   NONE    out[batch][L m]:   columns [l m, (l+1) m) hold scale * (first m rows of
 *                              H D3 H D2 H D1 x) for triple l
 *   COSSIN  out[batch][2 L m]: (1/sqrt(L m)) [cos block of L m | sin block of L m],
 *                              triple l in columns [l m, (l+1) m) of either block
 *   diag_sets  in   device fp32 [L][3][n], order d1, d2, d3 within a triple
 *   workspace  in   spinner_blocks_workspace_bytes(n, batch, m, epilogue) bytes
 * For L > 1, m must be a multiple of 4.  Up to n = 2^14 the L blocks come from one
 * kernel launch that reads x once and keeps it in registers while the triples are
 * applied one after the other (the feature blocks in fp64 as in spinner_apply); above
 * that size every block runs the four-pass path and reads x again.  Otherwise as
 * spinner_apply (which is the case L = 1).
 */
size_t spinner_blocks_workspace_bytes(int n, long batch, int m, int epilogue);
int spinner_apply_blocks(const float *x, int n, long batch, int L,
                         const float *diag_sets, int m, int epilogue, float scale,
                         float *out, void *workspace, void *stream);

/*
 * Angular-kernel features (Section 5, kernel approximation): the non-linear
 * map applied pointwise to the projection is the sign function, and the
 * kernel 1 - theta/pi between two inputs is estimated by 1 - d_H / d' from
 * the Hamming distance d_H of their d' = m sign bits.
 *
 * spinner_sign_codes computes, for each row of x, the signs of the first m
 * coordinates of y = H D3 H D2 H D1 x, packed one bit per coordinate:
 * bit = 1 where y_i < 0, 0 otherwise (a zero of either sign counts as
 * positive, as in spinner_hash).  The bits are stored in 64-bit words in the
 * order in which the hardware produces them (the comparison mask of one
 * register over one wave): coordinate e lives in bit (e >> 2) & 63 of word
 * ((e >> 8) << 2) | (e & 3) of its row.  The order is part of this interface
 * (it will not change between versions); spinner_code_position is the call
 * that converts a coordinate into its (word, bit) pair on the host, for
 * consumers that need the sign of one particular coordinate.  Hamming
 * distances, which is what the estimate uses, are the same in any fixed order.
 *
 *   x, d1..d3  in   as for spinner_apply
 *   m          in   coordinates kept: a multiple of 256, 256 <= m <= n
 *   codes      out  device, spinner_code_bytes(m) = m / 8 bytes per row,
 *                   rows contiguous, 16-byte aligned
 *   workspace  in   device scratch of spinner_codes_workspace_bytes(n, batch)
 *                   bytes (0 for n <= 2^16: one fused pass; above that the
 *                   projection is formed in the workspace by the four-pass
 *                   path and its signs are packed by a second kernel)
 *
 * spinner_sign_codes_signs is the same for diagonals packed by
 * spinner_pack_signs.  n must be at least 256 (SPINNER_ERR_UNSUPPORTED below).
 *
 * spinner_angular_gram computes out[i][j] = 1 - d_H(a_i, b_j) / m (fp32,
 * row-major [na][nb]) for two sets of codes of the same m; the Hamming
 * distances are exact integers.  na is limited to 128 * 65535 rows per call.
 */
size_t spinner_code_bytes(int m);
size_t spinner_codes_workspace_bytes(int n, long batch);
int spinner_code_position(int coordinate, int *word, int *bit);   /* SPINNER_ERR_BAD_M for a negative coordinate */
int spinner_sign_codes(const float *x, int n, long batch,
                       const float *d1, const float *d2, const float *d3,
                       int m, void *codes, void *workspace, void *stream);
int spinner_sign_codes_signs(const float *x, int n, long batch, const void *signs,
                             int m, void *codes, void *workspace, void *stream);
int spinner_angular_gram(const void *codes_a, long na, const void *codes_b, long nb,
                         int m, float *out, void *stream);

/*
 * Adaptive setting (Section 1; Section 3.2: the diagonals may be learned; Section 5,
 * neural networks: a fully connected layer re-parametrised as H D3 H D2 H D1 with
 * learned diagonals).  spinner_layer_forward computes y = scale * H D3 H D2 H D1 x
 * like spinner_apply (m = n, epilogue NONE) and keeps the two activations the backward
 * pass needs (those entering D2 and D3) in `saved`; spinner_layer_backward computes,
 * from dy = dL/dy,
 *     dx  = scale * D1 H D2 H D3 H dy                       (H is symmetric)
 *     dd  = [dL/dd1, dL/dd2, dL/dd3], each summed over the batch:
 *           dL/ddk[i] = sum_b (signal arriving at Dk from the output side)[b][i]
 *                             * (activation entering Dk)[b][i].
 *
 *   x, dy      in   device fp32 [batch][n]
 *   d1..d3     in   device fp32 [n], arbitrary values
 *   y, dx      out  device fp32 [batch][n]; dx may alias dy
 *   saved      out/in  device, spinner_layer_saved_bytes(n, batch) = 2 * batch * n * 4
 *                   bytes, opaque; written by the forward call, passed unchanged to
 *                   the backward call of the same x, d1..d3
 *   dd         out  device fp32 [3][n], overwritten
 *   workspace  in   device scratch of spinner_layer_workspace_bytes(n, batch) bytes
 *                   (partial sums over the batch, added up in fp64 in a fixed order;
 *                   above 2^14 also two signal buffers of batch * n floats)
 *
 * n = 2^4 .. 2^24, batch < 2^31.  Up to 2^14 each call is one fused kernel (plus the
 * reduction of the partial sums).  Above, every one of the three transforms is a pass
 * over the rows and a pass over the columns of the matrix view of the vector (the
 * saved activations arise between transforms), the backward pass writes the signal
 * arriving at each diagonal to the workspace and sums signal times activation over
 * the batch: six passes forward, six passes and three batch sums backward.  Same
 * ownership, alignment and error rules as spinner_apply.
 */
size_t spinner_layer_saved_bytes(int n, long batch);
size_t spinner_layer_workspace_bytes(int n, long batch);
int spinner_layer_forward(const float *x, int n, long batch,
                          const float *d1, const float *d2, const float *d3,
                          float scale, float *y, void *saved, void *stream);
int spinner_layer_backward(const float *dy, const float *x, const void *saved,
                           int n, long batch,
                           const float *d1, const float *d2, const float *d3,
                           float scale, float *dx, float *dd, void *workspace, void *stream);

/*
 * Newton sketch (Supplement, "Additional experiments"): the Hessian A^T W A of a
 * generalised linear model is replaced by (S W^{1/2} A)^T (S W^{1/2} A), with S an
 * m x n sketching matrix - here scale * (first m rows of H D3 H D2 H D1), which acts
 * on the COLUMNS of the row-major data matrix.
 *
 * spinner_sketch computes B = S diag(w) A.
 *   A          in   device fp32 [n][d] row-major (n observations of dimension d)
 *   w          in   device fp32 [n] row weights (e.g. the square roots of the Hessian
 *                   weights), or NULL for none
 *   d1..d3     in   device fp32 [n]
 *   m, scale   in   rows of the sketch, extra factor (sqrt(n/m) makes E[S^T S] = I)
 *   B          out  device fp32 [m][d] row-major
 *   workspace  in   device scratch of spinner_sketch_workspace_bytes(n, d, m) bytes.
 *                   Two forms, picked by shape.  For n <= 2^12 with d a multiple of 4
 *                   (matrices wide enough to fill the chip with column groups, and small
 *                   ones) one kernel loads the columns as they lie in the row-major
 *                   matrix - a tile is all n rows by 16 or 32 contiguous columns - and A
 *                   is moved once; the workspace is then not touched.  Otherwise (n >> d,
 *                   a column does not fit on chip beside enough neighbours for coalesced
 *                   loads) the matrix is transposed (weights applied on the way) so that
 *                   each column becomes one contiguous vector, projected with the same
 *                   kernels as spinner_apply, and the result transposed back
 * spinner_sketch_gram computes G = B^T B (device fp32 [d][d], all of it, symmetric)
 * on the fp32 matrix pipe; the sum over the m rows is split into slabs that are added
 * up in a fixed order, for which it needs spinner_sketch_gram_workspace_bytes(m, d)
 * bytes of device scratch (0 for small m).
 * n a power of two in [2^4, 2^24]; d and m arbitrary (1 <= m <= n).
 */
size_t spinner_sketch_workspace_bytes(int n, int d, int m);
int spinner_sketch(const float *A, int n, int d, const float *w,
                   const float *d1, const float *d2, const float *d3,
                   int m, float scale, float *B, void *workspace, void *stream);
size_t spinner_sketch_gram_workspace_bytes(int m, int d);
int spinner_sketch_gram(const float *B, int m, int d, float *G, void *workspace, void *stream);

/*
 * spinner_sketch_gram for callers that cannot allocate device memory or pass a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels and bit-identical results; the
 * slabs of the split sum go to a buffer built into the library (a file-scope
 * device array of spinner_sketch_gram_static_limit() = 16 MiB that each GPU the
 * library runs on holds until the process ends).  The call allocates and frees
 * nothing.  Problems with spinner_sketch_gram_workspace_bytes(m, d) above the
 * limit return SPINNER_ERR_SCRATCH_LIMIT and enqueue nothing (every d <= 256
 * and the d = 512 of the paper's experiment fit; d > 1920 needs no scratch at
 * all).  All calls on one GPU share the one buffer: calls that may
 * overlap in time on the same GPU (different streams, different threads) race;
 * calls on one stream are safe.  Nothing in the buffer has to be cleared
 * between calls.
 */
size_t spinner_sketch_gram_static_limit(void);
int spinner_sketch_gram_static(const float *B, int m, int d, float *G, void *stream);

/*
 * The G_struct D2 H D1 members of the family (Lemma 1 and the remark after it; Theorem 3;
 * used beside H D3 H D2 H D1 in the experiments of Section 5): the third block is a
 * structured matrix given by a generating vector, Gaussian in the random setting.
 *   SPINNER_STRUCT_CIRCULANT       g[n]:    row 0 is g, every next row is the previous
 *                                           one shifted right cyclically: G[i][j] = g[(j - i) mod n]
 *   SPINNER_STRUCT_SKEW_CIRCULANT  g[n]:    the same, an entry that wraps around changes sign
 *   SPINNER_STRUCT_TOEPLITZ        t[2n-1]: G[i][j] = t[j - i + n - 1]
 *   SPINNER_STRUCT_HANKEL          h[2n-1]: G[i][j] = h[i + j]
 * spinner_struct_prepare turns the generating vector (device fp32,
 * spinner_struct_params(kind, n) entries) into the opaque `spectrum` (device,
 * spinner_struct_spectrum_bytes(kind, n) bytes) once, off the clock, as the paper
 * prepares all parameters in advance.  spinner_struct_apply computes
 *     out[batch][m] = scale * (first m rows of G_struct D2 H D1 x)
 * with H the normalised Hadamard matrix.  The product with G_struct is an O(n log n)
 * FFT convolution of length P = n (circulant) or 2n (the others).  While the transform
 * fits the LDS (P <= 2^14: n = 2^5 .. 2^14 for the circulant, .. 2^13 for the others)
 * the call is one kernel that needs no scratch memory; spinner_struct_apply returns
 * SPINNER_ERR_UNSUPPORTED above that.  spinner_struct_apply_ws takes a workspace of
 * spinner_struct_workspace_bytes(kind, n, batch) bytes (0 for the sizes above) and also
 * serves P = 2^15 .. 2^22 (n up to 2^22 / 2^21): H D1 x by a pass over rows and a pass
 * over columns, then the transform in three passes through global memory (its top
 * stages over column tiles, blocks of 2^12 points with the spectrum product, the top
 * stages back).  spinner_struct_prepare serves all of these sizes.  An unknown kind
 * gives SPINNER_ERR_BAD_EPILOGUE.
 */
enum { SPINNER_STRUCT_CIRCULANT = 0, SPINNER_STRUCT_SKEW_CIRCULANT = 1, SPINNER_STRUCT_TOEPLITZ = 2, SPINNER_STRUCT_HANKEL = 3 };
size_t spinner_struct_params(int kind, int n);
size_t spinner_struct_spectrum_bytes(int kind, int n);
int spinner_struct_prepare(int kind, const float *params, int n, void *spectrum, void *stream);
int spinner_struct_apply(const float *x, int n, long batch, int kind, const void *spectrum,
                         const float *d1, const float *d2, int m, float scale,
                         float *out, void *stream);
size_t spinner_struct_workspace_bytes(int kind, int n, long batch);
int spinner_struct_apply_ws(const float *x, int n, long batch, int kind, const void *spectrum,
                            const float *d1, const float *d2, int m, float scale,
                            float *out, void *workspace, void *stream);

/*
 * Bytes of device scratch spinner_apply needs for these arguments: 0 up to the
 * fused limit, and above it when m == n with epilogue NONE; otherwise batch * n * 4.
 * Returns 0 for invalid arguments (spinner_apply reports those).
 */
size_t spinner_workspace_bytes(int n, long batch, int m, int epilogue);

/* Static, NUL-terminated description of a status code (host memory). */
const char *spinner_strerror(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int spinner_version(void);

/*
 * Measurement aid, not part of the method: dst[i] = src[i] for count fp32
 * elements with the same 16-byte-per-lane access shape the spinner kernels
 * use.  It gives the achievable read+write HBM rate on the machine at hand
 * and calibrates hardware byte counters against a transfer of known size.
 * count must be a multiple of 4; pointers 16-byte aligned.
 */
int spinner_stream_copy(const float *src, float *dst, size_t count, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SPINNER_H */
