/*
 * CPU oracle, numerical part -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain fp64 definitions of what the tiled kernels must reproduce.  The paper's
 * matrix-multiplication application (Section 4.2, the application listing) accumulates
 * dot(input[k], other[k]) over the K tiles and stores the sum: that is exactly
 * C[m,n] = sum_k A[m,k] * B[k,n], so the oracle is that definition written out, with
 * no tiling, blocking or reordering beyond the i-k-j loop order (which only changes the
 * order of an fp64 sum).  The 2D convolution (Section 4.3) maps onto the same product by
 * implicit GEMM; its oracle is the direct 7-deep cross-correlation loop.
 *
 * Inputs are the 16-bit patterns (IEEE binary16 or bfloat16) the GPU receives; they are
 * decoded exactly to fp64 here.  Nothing in this file is shared with, or called by, the
 * HIP library.  Only tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * Parity pins (tests/test_oracle_numeric.py): identity and permutation matrices,
 * hand-worked 2x2 / 3x3 products, all-ones closed form, transpose identity,
 * conv == GEMM for 1x1 filters, conv hand-worked 3x3 example, numpy second opinion.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

enum { NTO_F16 = 0, NTO_BF16 = 1 };

/* Exact decode of IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
static double decode_f16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int f = h & 0x3FF;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);               /* subnormal: f * 2^-10 * 2^-14 */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(f | 0x400), e - 25);  /* (1024+f) * 2^(e-15-10) */
    return sign ? -v : v;
}

/* Exact decode of bfloat16: the upper 16 bits of an IEEE binary32. */
static double decode_bf16(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

double nto_decode_one(uint16_t bits, int dtype)
{
    return dtype == NTO_F16 ? decode_f16(bits) : decode_bf16(bits);
}

void nto_decode(const uint16_t *src, int64_t n, int dtype, double *dst)
{
    for (int64_t i = 0; i < n; ++i)
        dst[i] = nto_decode_one(src[i], dtype);
}

/*
 * C[m,n] = sum_k A[m,k] * B[k,n]   (Section 4.2).
 * A is addressed as A[m*sAm + k*sAk], B as B[k*sBk + n*sBn] (strides in elements);
 * C is a dense row-major M x N fp64 array.  nthreads > 1 partitions the rows of C.
 * Returns 0, or -1 if memory for the decoded operands cannot be obtained.
 */
int nto_gemm(const uint16_t *A, int64_t sAm, int64_t sAk,
             const uint16_t *B, int64_t sBk, int64_t sBn,
             double *C, int64_t M, int64_t N, int64_t K, int dtype, int nthreads)
{
    double *a = (double *)malloc(sizeof(double) * (size_t)(M * K > 0 ? M * K : 1));
    double *b = (double *)malloc(sizeof(double) * (size_t)(K * N > 0 ? K * N : 1));
    if (!a || !b) { free(a); free(b); return -1; }
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k)
            a[m * K + k] = nto_decode_one(A[m * sAm + k * sAk], dtype);
    for (int64_t k = 0; k < K; ++k)
        for (int64_t n = 0; n < N; ++n)
            b[k * N + n] = nto_decode_one(B[k * sBk + n * sBn], dtype);
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        double *c = C + m * N;
        for (int64_t n = 0; n < N; ++n) c[n] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double x = a[m * K + k];
            const double *br = b + k * N;
            for (int64_t n = 0; n < N; ++n) c[n] += x * br[n];
        }
    }
    free(a); free(b);
    return 0;
}

/* Selected entries C[ms[i], ns[i]] of the same product, one dot product each. */
void nto_gemm_samples(const uint16_t *A, int64_t sAm, int64_t sAk,
                      const uint16_t *B, int64_t sBk, int64_t sBn,
                      int64_t K, int dtype,
                      const int64_t *ms, const int64_t *ns, int64_t nsamp, double *out)
{
    for (int64_t i = 0; i < nsamp; ++i) {
        double s = 0.0;
        for (int64_t k = 0; k < K; ++k)
            s += nto_decode_one(A[ms[i] * sAm + k * sAk], dtype) *
                 nto_decode_one(B[k * sBk + ns[i] * sBn], dtype);
        out[i] = s;
    }
}

/*
 * Direct 2D cross-correlation (no filter flip), NCHW input, KCRS filter, NKPQ output
 * (shape names of Section 4.3):
 *   Y[n,f,p,q] = sum_{c,r,s} X[n,c,p*sh+r-ph, q*sw+s-pw] * Wt[f,c,r,s],  X = 0 outside.
 * All three tensors dense in their natural order.  P and Q are given by the caller.
 */
void nto_conv2d(const uint16_t *X, const uint16_t *Wt, double *Y,
                int64_t N, int64_t C, int64_t H, int64_t W,
                int64_t F, int64_t R, int64_t S, int64_t P, int64_t Q,
                int64_t sh, int64_t sw, int64_t ph, int64_t pw, int dtype, int nthreads)
{
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(static) collapse(2)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t f = 0; f < F; ++f)
            for (int64_t p = 0; p < P; ++p)
                for (int64_t q = 0; q < Q; ++q) {
                    double acc = 0.0;
                    for (int64_t c = 0; c < C; ++c)
                        for (int64_t r = 0; r < R; ++r)
                            for (int64_t s = 0; s < S; ++s) {
                                int64_t h = p * sh + r - ph;
                                int64_t w = q * sw + s - pw;
                                if (h < 0 || h >= H || w < 0 || w >= W) continue;
                                acc += nto_decode_one(X[((n * C + c) * H + h) * W + w], dtype) *
                                       nto_decode_one(Wt[((f * C + c) * R + r) * S + s], dtype);
                            }
                    Y[((n * F + f) * P + p) * Q + q] = acc;
                }
}

/* Selected outputs Y[n,f,p,q] of the same convolution; idx holds nsamp (n,f,p,q) rows. */
void nto_conv2d_samples(const uint16_t *X, const uint16_t *Wt,
                        int64_t C, int64_t H, int64_t W, int64_t R, int64_t S,
                        int64_t sh, int64_t sw, int64_t ph, int64_t pw, int dtype,
                        const int64_t *idx, int64_t nsamp, double *out)
{
    for (int64_t i = 0; i < nsamp; ++i) {
        int64_t n = idx[4 * i], f = idx[4 * i + 1], p = idx[4 * i + 2], q = idx[4 * i + 3];
        double acc = 0.0;
        for (int64_t c = 0; c < C; ++c)
            for (int64_t r = 0; r < R; ++r)
                for (int64_t s = 0; s < S; ++s) {
                    int64_t h = p * sh + r - ph;
                    int64_t w = q * sw + s - pw;
                    if (h < 0 || h >= H || w < 0 || w >= W) continue;
                    acc += nto_decode_one(X[((n * C + c) * H + h) * W + w], dtype) *
                           nto_decode_one(Wt[((f * C + c) * R + r) * S + s], dtype);
                }
        out[i] = acc;
    }
}
