/*
 * CPU oracle for group-quantized matrix-vector products (QIGen, arXiv 2307.03738).
 *
 * TEST INFRASTRUCTURE, NOT PRODUCT CODE.  This file is the slow, plain statement of what
 * the GPU library must compute.  It shares nothing with the HIP sources: no header, no
 * table, no helper.  Only the tests, the smoke check and the cpu_baseline leg of the
 * benchmark may load it.
 *
 * Conventions (weights in PyTorch Linear orientation; the paper writes the transpose):
 *   W  [N][K] fp32, N outputs, K inputs          (paper: W in R^{n x m}, n = K, m = N)
 *   groups of G consecutive k share one (s, z)   (Section 2, "groups")
 *   b in {2,3,4} bits per code
 *   What[n][k] = s[n][k/G] * (q[n][k] - z[n][k/G])   (Section 2, dequantization D, eq. (1))
 *
 * All fp32 steps of the quantizer are single IEEE-754 binary32 operations, round to
 * nearest even, true division, no fused multiply-add (build with -ffp-contract=off and
 * without -ffast-math).  Products are accumulated in fp64 in index order.
 *
 * Every function returns 0 on success and a positive number on a bad argument.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

static int bad_shape(int64_t N, int64_t K, int bits, int group)
{
    if (N <= 0 || K <= 0 || group <= 0) return 1;
    if (bits != 2 && bits != 3 && bits != 4) return 1;
    if (K % group != 0) return 1;
    return 0;
}

int qgo_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Number of threads the loops over outputs use from now on (timing only; results do not
 * depend on it: every output is summed by one thread in index order). */
void qgo_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ---------------------------------------------------------------------------------------
 * Quantization (Section 2, "Quantization": Q(x,b) maps to integers in [0, 2^b); D(x_q) =
 * s (x_q - z) as fixed by eq. (1)).  Reading used here, stated in the task as
 * q = clamp(round(w/s) + z, 0, 2^b - 1) with an fp32 scale and an integer zero:
 *   lo = min(0, min_k w), hi = max(0, max_k w)       the range always contains 0
 *   s  = (hi - lo) / (2^b - 1)                       the dequantization step
 *   z  = clamp(rint(-lo / s), 0, 2^b - 1)            integer zero-point
 *   q  = clamp(rint(w / s) + z, 0, 2^b - 1)          round to nearest, ties to even
 * A group whose range is 0 (all entries equal 0 after including 0) gets s = 1, z = 0, q = 0.
 * ------------------------------------------------------------------------------------- */
int qgo_quantize(const float *W, int64_t N, int64_t K, int bits, int group,
                 uint8_t *q, float *s, uint8_t *z)
{
    if (bad_shape(N, K, bits, group) || !W || !q || !s || !z) return 1;
    const int qmax = (1 << bits) - 1;
    const int64_t ngroups = K / group;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t g = 0; g < ngroups; ++g) {
            const float *w = W + n * K + g * group;
            float lo = 0.0f, hi = 0.0f;
            for (int k = 0; k < group; ++k) {
                if (w[k] < lo) lo = w[k];
                if (w[k] > hi) hi = w[k];
            }
            const float range = hi - lo;
            float scale;
            int zero;
            if (range == 0.0f) {
                scale = 1.0f;
                zero = 0;
            } else {
                scale = range / (float)qmax;
                zero = (int)rintf(-lo / scale);
                if (zero < 0) zero = 0;
                if (zero > qmax) zero = qmax;
            }
            s[n * ngroups + g] = scale;
            z[n * ngroups + g] = (uint8_t)zero;
            uint8_t *qo = q + n * K + g * group;
            for (int k = 0; k < group; ++k) {
                int c = (int)rintf(w[k] / scale) + zero;
                if (c < 0) c = 0;
                if (c > qmax) c = qmax;
                qo[k] = (uint8_t)c;
            }
        }
    }
    return 0;
}

/* Dequantization D(x_q) = s (x_q - z), eq. (1).  Exact in fp64: a 24-bit significand times
 * an integer of at most 5 bits. */
int qgo_dequantize(const uint8_t *q, const float *s, const uint8_t *z, int64_t N, int64_t K,
                   int group, double *What)
{
    if (N <= 0 || K <= 0 || group <= 0 || K % group || !q || !s || !z || !What) return 1;
    const int64_t ngroups = K / group;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            const int64_t g = n * ngroups + k / group;
            What[n * K + k] = (double)s[g] * (double)((int)q[n * K + k] - (int)z[g]);
        }
    return 0;
}

/* ---------------------------------------------------------------------------------------
 * Canonical packed format (Section 3, "Data format"; Algorithm 2 fixes the field order).
 * The codes of one output n along k form a little-endian bit stream: code k occupies bits
 * [b*k, b*k + b).  The stream is cut into 32-bit words; word w of output n is stored at
 * P[w][n] (uint32 [K*b/32][N], n contiguous: the paper's compressed matrix of size
 * n/(32/b) x m).  4-bit: 8 codes per word, code j of the word in bits [4j, 4j+4).
 * 2-bit: 16 per word.  3-bit: every 32 codes fill exactly three consecutive words, so the
 * codes with k = 10 and 21 (mod 32) straddle a word boundary.
 * A stream of `count` items whose bit length is not a multiple of 32 is zero-padded to a
 * whole word (this only happens for the zero-points, see below).
 * ------------------------------------------------------------------------------------- */
static int64_t stream_words(int64_t count, int bits)
{
    return (count * bits + 31) / 32;
}

static int pack_stream(const uint8_t *v, int64_t N, int64_t count, int bits, uint32_t *P)
{
    const int64_t words = stream_words(count, bits);
    for (int64_t i = 0; i < N * count; ++i)
        if (v[i] >> bits) return 2; /* code out of range */
    memset(P, 0, (size_t)(words * N) * sizeof(uint32_t));
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < count; ++k) {
            const uint32_t c = v[n * count + k];
            const int64_t bit = k * bits;
            const int64_t w = bit / 32;
            const int off = (int)(bit % 32);
            P[w * N + n] |= c << off;
            if (off + bits > 32) P[(w + 1) * N + n] |= c >> (32 - off);
        }
    return 0;
}

static void unpack_stream(const uint32_t *P, int64_t N, int64_t count, int bits, uint8_t *v)
{
    const uint32_t mask = (1u << bits) - 1u;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < count; ++k) {
            const int64_t bit = k * bits;
            const int64_t w = bit / 32;
            const int off = (int)(bit % 32);
            uint32_t c = P[w * N + n] >> off;
            if (off + bits > 32) c |= P[(w + 1) * N + n] << (32 - off);
            v[n * count + k] = (uint8_t)(c & mask);
        }
}

int64_t qgo_code_words(int64_t K, int bits) { return stream_words(K, bits); }

/* q [N][K] one code per byte -> P [K*b/32][N].  K*b must be a multiple of 32. */
int qgo_pack_codes(const uint8_t *q, int64_t N, int64_t K, int bits, uint32_t *P)
{
    if (N <= 0 || K <= 0 || (bits != 2 && bits != 3 && bits != 4) || !q || !P) return 1;
    if ((K * bits) % 32 != 0) return 1;
    return pack_stream(q, N, K, bits, P);
}

int qgo_unpack_codes(const uint32_t *P, int64_t N, int64_t K, int bits, uint8_t *q)
{
    if (N <= 0 || K <= 0 || (bits != 2 && bits != 3 && bits != 4) || !q || !P) return 1;
    if ((K * bits) % 32 != 0) return 1;
    unpack_stream(P, N, K, bits, q);
    return 0;
}

/* Zero-points are themselves stored with b bits each (Section 3: the z_j "can also be
 * quantized", and the memory formula counts b bits per zero): the same bit-stream rule is
 * applied along the group index, zero-padded to a whole word.  z [N][ngroups] ->
 * Zp [ceil(ngroups*b/32)][N]. */
int qgo_pack_zeros(const uint8_t *z, int64_t N, int64_t ngroups, int bits, uint32_t *Zp)
{
    if (N <= 0 || ngroups <= 0 || (bits != 2 && bits != 3 && bits != 4) || !z || !Zp) return 1;
    return pack_stream(z, N, ngroups, bits, Zp);
}

int qgo_unpack_zeros(const uint32_t *Zp, int64_t N, int64_t ngroups, int bits, uint8_t *z)
{
    if (N <= 0 || ngroups <= 0 || (bits != 2 && bits != 3 && bits != 4) || !z || !Zp) return 1;
    unpack_stream(Zp, N, ngroups, bits, z);
    return 0;
}

/* Scales in the canonical format: float [ngroups][N] (one per output and group, output
 * index contiguous like the codes).  s [N][ngroups] -> St [ngroups][N] and back. */
int qgo_transpose_scales(const float *s, int64_t N, int64_t ngroups, float *St)
{
    if (N <= 0 || ngroups <= 0 || !s || !St) return 1;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t g = 0; g < ngroups; ++g) St[g * N + n] = s[n * ngroups + g];
    return 0;
}

/* Storage of the canonical format in bits: b per weight, 32 + b per (output, group)
 * (Section 3 memory formula, generalised from one group per output to K/G groups). */
int64_t qgo_storage_bits(int64_t N, int64_t K, int bits, int group)
{
    return (int64_t)bits * N * K + (int64_t)(32 + bits) * N * (K / group);
}

/* ---------------------------------------------------------------------------------------
 * Products.  y[n] = sum_k What[n][k] x[k], the definition, accumulated in fp64 in index
 * order (Algorithm 1 output, eq. (1)/(2) left-hand side).
 * ------------------------------------------------------------------------------------- */
int qgo_matvec(const uint8_t *q, const float *s, const uint8_t *z, int64_t N, int64_t K,
               int group, const float *x, double *y)
{
    if (N <= 0 || K <= 0 || group <= 0 || K % group || !q || !s || !z || !x || !y) return 1;
    const int64_t ngroups = K / group;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const int64_t g = n * ngroups + k / group;
            const double w = (double)s[g] * (double)((int)q[n * K + k] - (int)z[g]);
            acc += w * (double)x[k];
        }
        y[n] = acc;
    }
    return 0;
}

/* The factorised form, eq. (2) with the scale restored on the zero term:
 * y[n] = sum_g s_g <x_g, q_g> - sum_g s_g z_g <x_g, 1>.  Integer-code dot products first,
 * one scale and one zero correction per group.  Used to check the identity. */
int qgo_matvec_factored(const uint8_t *q, const float *s, const uint8_t *z, int64_t N,
                        int64_t K, int group, const float *x, double *y)
{
    if (N <= 0 || K <= 0 || group <= 0 || K % group || !q || !s || !z || !x || !y) return 1;
    const int64_t ngroups = K / group;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double first = 0.0, second = 0.0;
        for (int64_t g = 0; g < ngroups; ++g) {
            double dot = 0.0, ones = 0.0;
            for (int k = 0; k < group; ++k) {
                dot += (double)q[n * K + g * group + k] * (double)x[g * group + k];
                ones += (double)x[g * group + k];
            }
            first += (double)s[n * ngroups + g] * dot;
            second += (double)s[n * ngroups + g] * (double)z[n * ngroups + g] * ones;
        }
        y[n] = first - second;
    }
    return 0;
}

/* Same product, reading the canonical packed format directly and dequantizing on the fly
 * (what a kernel given only the packed matrix has to do; Algorithm 1's inputs).  P is
 * uint32 [K*b/32][N], St is float [K/G][N], Zp is the packed zero stream. */
int qgo_matvec_packed(const uint32_t *P, const float *St, const uint32_t *Zp, int64_t N,
                      int64_t K, int bits, int group, const float *x, double *y)
{
    if (bad_shape(N, K, bits, group) || (K * bits) % 32 || !P || !St || !Zp || !x || !y) return 1;
    const uint32_t mask = (1u << bits) - 1u;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const int64_t g = k / group;
            int64_t bit = k * bits;
            uint32_t c = P[(bit / 32) * N + n] >> (bit % 32);
            if (bit % 32 + bits > 32) c |= P[(bit / 32 + 1) * N + n] << (32 - bit % 32);
            c &= mask;
            bit = g * bits;
            uint32_t zz = Zp[(bit / 32) * N + n] >> (bit % 32);
            if (bit % 32 + bits > 32) zz |= Zp[(bit / 32 + 1) * N + n] << (32 - bit % 32);
            zz &= mask;
            const double w = (double)St[g * N + n] * (double)((int)c - (int)zz);
            acc += w * (double)x[k];
        }
        y[n] = acc;
    }
    return 0;
}

/* Small-batch form for prompt tokens: Y[m][n] = sum_k X[m][k] What[n][k], X [M][K]
 * row-major, Y [M][N] row-major, fp64 accumulation in index order, no rounding of either
 * operand to a shorter type. */
int qgo_matmul_small(const uint8_t *q, const float *s, const uint8_t *z, int64_t N, int64_t K,
                     int group, const float *X, int64_t M, double *Y)
{
    if (N <= 0 || K <= 0 || M <= 0 || group <= 0 || K % group || !q || !s || !z || !X || !Y)
        return 1;
    const int64_t ngroups = K / group;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t m = 0; m < M; ++m) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                const int64_t g = n * ngroups + k / group;
                const double w = (double)s[g] * (double)((int)q[n * K + k] - (int)z[g]);
                acc += w * (double)X[m * K + k];
            }
            Y[m * N + n] = acc;
        }
    return 0;
}

/* Row norms ||What[n,:]||_2, the scale of the error metric used to compare a
 * floating-point product with this oracle. */
int qgo_row_norms(const uint8_t *q, const float *s, const uint8_t *z, int64_t N, int64_t K,
                  int group, double *norms)
{
    if (N <= 0 || K <= 0 || group <= 0 || K % group || !q || !s || !z || !norms) return 1;
    const int64_t ngroups = K / group;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const int64_t g = n * ngroups + k / group;
            const double w = (double)s[g] * (double)((int)q[n * K + k] - (int)z[g]);
            acc += w * w;
        }
        norms[n] = sqrt(acc);
    }
    return 0;
}

/* The gated combination of two products that a LLaMA block applies after its "gate" and "up"
 * projections: h[i] = silu(g[i]) * u[i], silu(t) = t / (1 + exp(-t)), in fp64. */
void qgo_swiglu(const double *g, const double *u, int64_t n, double *h)
{
    for (int64_t i = 0; i < n; ++i) h[i] = g[i] / (1.0 + exp(-g[i])) * u[i];
}

