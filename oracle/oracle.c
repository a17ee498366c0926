/*
 * CPU oracle for the three dense contractions.  TEST INFRASTRUCTURE ONLY: it is called by
 * the tests, by the smoke check and by the benchmark's CPU-baseline leg, never by the
 * product path, and it shares no code with the GPU kernels.
 *
 * Every function is the plain definition written out as nested loops, with each output
 * element accumulated in double (fp32 x fp32 products are exact in double) or in 64-bit
 * integers, reduction index ascending.  No blocking, no reordering, no intrinsics.  The
 * only parallelism is an OpenMP "parallel for" over independent output rows, which does
 * not change any element's sequence of operations.
 *
 * Definitions followed:
 *   - matrix multiplication: Section 2.1, Fig. 1 (loop nest and its Einstein form) with
 *     alpha = beta = 1, plus = +, times = *;
 *   - convolution: Section 2.1, first item of the list after the pre/post-operation
 *     formula, O[r,c] = I[r+k, c+j] * w[k,j] (a correlation: the filter is not flipped),
 *     with the affine index map of the generalised contraction supplying stride and
 *     zero padding;
 *   - signed 8-bit product with 32-bit sums: the same generalised contraction with
 *     integer plus/times, result taken modulo 2^32;
 *   - the product on transposed operands: the same loop nest with the affine index map of
 *     A or B swapped (Section 2.1 lists the transposition O[r,c] = I[c,r]);
 *   - single-operand contractions (Section 5.2): transposition, sub-tensor extraction and
 *     broadcast as one strided copy;
 *   - depth-wise convolution (the DWCONV rows of Table 1): the convolution formula with
 *     the channel index shared by input, filter and output instead of being reduced,
 *     O[r,c,ch] = I[r+k, c+j, ch] * w[k,j,ch]; only the filter taps are summed.
 *
 * All pointers are host pointers.  Strides (lda, ldb, ldc) are in elements.
 */
#include <stddef.h>
#include <stdint.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* One element of C_in + A.B and of |C_in| + sum |a.b| (Fig. 1, innermost loop). */
static void sgemm_element(int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb,
                          float c_in, int64_t i, int64_t j, double *value, double *absum)
{
    double acc = (double)c_in;
    double mag = fabs((double)c_in);
    for (int64_t k = 0; k < K; ++k) {
        double prod = (double)A[i * lda + k] * (double)B[k * ldb + j];
        acc += prod;
        mag += fabs(prod);
    }
    *value = acc;
    if (absum) *absum = mag;
}

/*
 * out[i*N + j] = Cin[i*ldc + j] + sum_k A[i*lda + k] * B[k*ldb + j]      (Fig. 1)
 * absum[i*N + j] = |Cin| + sum_k |A*B|   (optional, may be NULL)
 * out and absum are dense M x N doubles.
 */
int oracle_sgemm(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                 int64_t ldb, const float *Cin, int64_t ldc, double *out, double *absum)
{
    if (M < 0 || N < 0 || K < 0) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            double v, s;
            sgemm_element(K, A, lda, B, ldb, Cin[i * ldc + j], i, j, &v, &s);
            out[i * N + j] = v;
            if (absum) absum[i * N + j] = s;
        }
    }
    return 0;
}

/*
 * C = post(pre(C_in) + A.B): the contraction with the element-wise pre- and post-operation
 * of Section 2.1 (the formula that follows the generalised contraction).
 *   pre : 0 -> C_in[i,j]   1 -> 0   2 -> bias[j]
 *   post: 0 -> x           1 -> max(x, 0)   (the ReLU of the MLP listing in Section 3)
 * absum = |pre value| + sum |a.b|.
 */
int oracle_sgemm_fused(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                       int64_t ldb, const float *Cin, int64_t ldc, const float *bias, int pre,
                       int post, double *out, double *absum)
{
    if (M < 0 || N < 0 || K < 0 || pre < 0 || pre > 2 || post < 0 || post > 1) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            float init = 0.0f;
            if (pre == 0) init = Cin[i * ldc + j];
            if (pre == 2) init = bias[j];
            double v, s;
            sgemm_element(K, A, lda, B, ldb, init, i, j, &v, &s);
            if (post == 1 && v < 0.0) v = 0.0;
            out[i * N + j] = v;
            if (absum) absum[i * N + j] = s;
        }
    }
    return 0;
}

/*
 * The product with either operand stored transposed: the generalised contraction of
 * Section 2.1 with the affine index map of an operand swapped (its list of contractions
 * gives the transposition O[r,c] = I[c,r]):
 *   out[i*N + j] = Cin[i*ldc + j] + sum_k a(i,k) * b(k,j)
 *   a(i,k) = ta ? A[k*lda + i] : A[i*lda + k]      (ta: A is stored K x M)
 *   b(k,j) = tb ? B[j*ldb + k] : B[k*ldb + j]      (tb: B is stored N x K)
 * absum as in oracle_sgemm.  One double accumulator per element, k ascending.
 */
int oracle_sgemm_op(int ta, int tb, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
                    const float *B, int64_t ldb, const float *Cin, int64_t ldc, double *out,
                    double *absum)
{
    if (M < 0 || N < 0 || K < 0) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            double acc = (double)Cin[i * ldc + j];
            double mag = fabs(acc);
            for (int64_t k = 0; k < K; ++k) {
                double a = (double)(ta ? A[k * lda + i] : A[i * lda + k]);
                double b = (double)(tb ? B[j * ldb + k] : B[k * ldb + j]);
                acc += a * b;
                mag += fabs(a * b);
            }
            out[i * N + j] = acc;
            if (absum) absum[i * N + j] = mag;
        }
    }
    return 0;
}

/* The same element formula at npts chosen coordinates (ii[t], jj[t]). */
int oracle_sgemm_points(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
                        const float *B, int64_t ldb, const float *Cin, int64_t ldc, int64_t npts,
                        const int64_t *ii, const int64_t *jj, double *out, double *absum)
{
    if (M < 0 || N < 0 || K < 0 || npts < 0) return -1;
    for (int64_t t = 0; t < npts; ++t)
        if (ii[t] < 0 || ii[t] >= M || jj[t] < 0 || jj[t] >= N) return -2;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t t = 0; t < npts; ++t) {
        double v, s;
        sgemm_element(K, A, lda, B, ldb, Cin[ii[t] * ldc + jj[t]], ii[t], jj[t], &v, &s);
        out[t] = v;
        if (absum) absum[t] = s;
    }
    return 0;
}

/* C[i,j] = (Cin[i,j] + sum_k A[i,k]*B[k,j]) mod 2^32, operands signed 8-bit. */
int oracle_igemm_s8s32(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda,
                       const int8_t *B, int64_t ldb, const int32_t *Cin, int64_t ldc, int32_t *out)
{
    if (M < 0 || N < 0 || K < 0) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            /* |each product| <= 2^14, so int64 cannot overflow for any addressable K */
            int64_t acc = (int64_t)Cin[i * ldc + j];
            for (int64_t k = 0; k < K; ++k)
                acc += (int64_t)A[i * lda + k] * (int64_t)B[k * ldb + j];
            out[i * N + j] = (int32_t)(uint32_t)(uint64_t)acc; /* reduce modulo 2^32 */
        }
    }
    return 0;
}

static int conv_out_extent(int64_t in, int64_t filt, int64_t stride, int64_t pad)
{
    return (int)((in + 2 * pad - filt) / stride + 1);
}

/* One output element: the three reduction loops r, s, c of the seven-loop nest. */
static void conv_element(int64_t H, int64_t W, int64_t C, int64_t R, int64_t S, int64_t stride,
                         int64_t pad, const float *in, const float *w, int64_t n, int64_t p,
                         int64_t q, int64_t k, double *value, double *absum)
{
    double acc = 0.0, mag = 0.0;
    for (int64_t r = 0; r < R; ++r) {
        for (int64_t s = 0; s < S; ++s) {
            int64_t h = p * stride - pad + r; /* affine index into the input */
            int64_t x = q * stride - pad + s;
            if (h < 0 || h >= H || x < 0 || x >= W) continue; /* zero padding */
            for (int64_t c = 0; c < C; ++c) {
                double prod = (double)in[((n * H + h) * W + x) * C + c] *
                              (double)w[((k * R + r) * S + s) * C + c];
                acc += prod;
                mag += fabs(prod);
            }
        }
    }
    *value = acc;
    if (absum) *absum = mag;
}

/*
 * out[n,p,q,k] = sum_{r,s,c} in[n, p*stride-pad+r, q*stride-pad+s, c] * w[k,r,s,c]
 * in: N,H,W,C   w: K,R,S,C   out/absum: N,P,Q,K doubles (absum optional).
 */
int oracle_conv2d_nhwc_fused(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R,
                             int64_t S, int64_t stride, int64_t pad, const float *in, const float *w,
                             const float *bias, int post, double *out, double *absum);

int oracle_conv2d_nhwc(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                       int64_t stride, int64_t pad, const float *in, const float *w, double *out,
                       double *absum)
{
    return oracle_conv2d_nhwc_fused(N, H, W, C, K, R, S, stride, pad, in, w, NULL, 0, out, absum);
}

/*
 * out[n,p,q,k] = post(bias[k] + sum_{r,s,c} ...): the convolution above with a per-channel
 * bias as pre-operation (bias == NULL: none) and post as for oracle_sgemm_fused.
 * absum = |bias[k]| + sum |in.w|.
 */
int oracle_conv2d_nhwc_fused(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R,
                             int64_t S, int64_t stride, int64_t pad, const float *in, const float *w,
                             const float *bias, int post, double *out, double *absum)
{
    if (post < 0 || post > 1) return -1;
    if (N < 0 || H < 0 || W < 0 || C <= 0 || K <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0)
        return -1;
    if (H + 2 * pad < R || W + 2 * pad < S) return -1;
    const int64_t P = conv_out_extent(H, R, stride, pad), Q = conv_out_extent(W, S, stride, pad);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < P; ++p)
            for (int64_t q = 0; q < Q; ++q)
                for (int64_t k = 0; k < K; ++k) {
                    double v, s;
                    conv_element(H, W, C, R, S, stride, pad, in, w, n, p, q, k, &v, &s);
                    if (bias) {
                        v = (double)bias[k] + v;
                        s = fabs((double)bias[k]) + s;
                    }
                    if (post == 1 && v < 0.0) v = 0.0;
                    int64_t o = ((n * P + p) * Q + q) * K + k;
                    out[o] = v;
                    if (absum) absum[o] = s;
                }
    return 0;
}

/*
 * Depth-wise convolution, one filter per channel (Table 1, DWCONV rows; Section 2.1's
 * convolution with the channel kept as an output index):
 *   out[n,p,q,c] = post(bias[c] + sum_{r,s} in[n, p*stride-pad+r, q*stride-pad+s, c] * w[r,s,c])
 * in: N,H,W,C   w: R,S,C   bias: C or NULL   out/absum: N,P,Q,C doubles (absum optional).
 * absum = |bias[c]| + sum |in.w|.
 */
int oracle_dwconv2d_nhwc(int64_t N, int64_t H, int64_t W, int64_t C, int64_t R, int64_t S,
                         int64_t stride, int64_t pad, const float *in, const float *w,
                         const float *bias, int post, double *out, double *absum)
{
    if (post < 0 || post > 1) return -1;
    if (N < 0 || H < 0 || W < 0 || C <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0) return -1;
    if (H + 2 * pad < R || W + 2 * pad < S) return -1;
    const int64_t P = conv_out_extent(H, R, stride, pad), Q = conv_out_extent(W, S, stride, pad);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < P; ++p)
            for (int64_t q = 0; q < Q; ++q)
                for (int64_t c = 0; c < C; ++c) {
                    double acc = bias ? (double)bias[c] : 0.0;
                    double mag = fabs(acc);
                    for (int64_t r = 0; r < R; ++r) {
                        const int64_t h = p * stride - pad + r;
                        if (h < 0 || h >= H) continue;
                        for (int64_t t = 0; t < S; ++t) {
                            const int64_t x = q * stride - pad + t;
                            if (x < 0 || x >= W) continue;
                            double prod = (double)in[((n * H + h) * W + x) * C + c] *
                                          (double)w[(r * S + t) * C + c];
                            acc += prod;
                            mag += fabs(prod);
                        }
                    }
                    if (post == 1 && acc < 0.0) acc = 0.0;
                    int64_t o = ((n * P + p) * Q + q) * C + c;
                    out[o] = acc;
                    if (absum) absum[o] = mag;
                }
    return 0;
}

/*
 * Single-operand form of the contraction (Section 5.2, "Single Operand LoopNest"; the
 * transpositions and broadcasts of Section 2.1's list): no reduction index, one input,
 *   out[i0,i1,i2,i3] = in[i0*s0 + i1*s1 + i2*s2 + i3*s3]
 * out is dense row-major with extents d[0..3]; the input is addressed through element
 * strides s[0..3] (permuted strides transpose, a stride of 0 broadcasts, the strides of an
 * enclosing tensor extract a sub-tensor).  esize = bytes per element (1 or 4); pure data
 * movement, so the result is bit-exact.
 */
int oracle_tensor_copy(int64_t esize, const int64_t *d, const int64_t *s, const void *in, void *out)
{
    if (esize != 1 && esize != 4) return -1;
    for (int a = 0; a < 4; ++a)
        if (d[a] < 0 || s[a] < 0) return -1;
    const unsigned char *src = (const unsigned char *)in;
    unsigned char *dst = (unsigned char *)out;
    int64_t o = 0;
    for (int64_t i0 = 0; i0 < d[0]; ++i0)
        for (int64_t i1 = 0; i1 < d[1]; ++i1)
            for (int64_t i2 = 0; i2 < d[2]; ++i2)
                for (int64_t i3 = 0; i3 < d[3]; ++i3, ++o) {
                    const int64_t from = i0 * s[0] + i1 * s[1] + i2 * s[2] + i3 * s[3];
                    for (int64_t b = 0; b < esize; ++b) dst[o * esize + b] = src[from * esize + b];
                }
    return 0;
}

/*
 * The same product with the second operand given transposed, i.e. k-contiguous like A
 * (an operand reorganised by the single-operand contraction of Section 5.2 for the kernel
 * that follows): C[i,j] = (Cin[i,j] + sum_k A[i,k]*Bt[j,k]) mod 2^32, Bt: N x K.
 */
int oracle_igemm_s8s32_bt(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda,
                          const int8_t *Bt, int64_t ldbt, const int32_t *Cin, int64_t ldc, int32_t *out)
{
    if (M < 0 || N < 0 || K < 0) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            int64_t acc = (int64_t)Cin[i * ldc + j];
            for (int64_t k = 0; k < K; ++k)
                acc += (int64_t)A[i * lda + k] * (int64_t)Bt[j * ldbt + k];
            out[i * N + j] = (int32_t)(uint32_t)(uint64_t)acc;
        }
    }
    return 0;
}
