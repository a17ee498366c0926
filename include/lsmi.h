/*
 * lsmi - dense contraction kernels for gfx950 (MI355X) behind a C ABI.
 *
 * The three compute calls are instances of the generalised contraction of Section 2.1
 *     C = post(pre(C_in) (+) beta (A (x) B))
 * with alpha = beta = 1 and identity pre/post operations:
 *   sgemm        fp32 matrix product accumulated into C (Fig. 1 loop nest / Einstein form)
 *   igemm_s8s32  the same with signed 8-bit operands and 32-bit integer sums
 *   conv2d_nhwc  2-D convolution O[r,c] = I[r+k, c+j] * w[k,j] (first item of the list of
 *                contractions in Section 2.1; a correlation, the filter is not flipped)
 *                with stride and zero padding supplied by the affine index map
 * Tensors are dense row-major, i.e. the last listed dimension is contiguous (Section 4.2,
 * read/write nodes operate on user-provided memory in the listed dimension order).
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers, allocated, owned and freed by the caller.
 *     The library keeps no reference to them after the call returns.
 *   - Sizes and strides are int64_t; strides (lda, ldb, ldc) count ELEMENTS between the
 *     starts of consecutive rows.
 *   - Work is enqueued on the stream set by lsmi_set_stream() for the calling thread
 *     (default: the null stream) and the call returns without waiting for it.
 *   - The library allocates no device memory; only sgemm_ws takes a workspace, from the caller.
 *   - Return value: LSMI_OK (0) or a negative lsmi_status.  Arguments are validated on
 *     the host before any GPU call, so validation errors are reported even on a machine
 *     without a GPU.  On an error nothing has been enqueued.
 *   - A zero extent is a successful no-op (see each call).
 *   - Undefined: C (or out) overlapping an input; host pointers; two calls writing the
 *     same C concurrently on different streams; NaN, infinite or denormal inputs.
 *   - Outputs (C, out) must be ordinary device memory (hipMalloc, coarse-grained): where
 *     partial sums of several workgroups meet they are added with the hardware's
 *     floating-point atomic instructions (the library is built with -munsafe-fp-atomics),
 *     which fine-grained or host-mapped memory does not support.
 *   - Operand rows are fetched in 16-byte groups: a matrix whose last row ends off a
 *     16-byte boundary may be READ (never written) up to the end of that 16-byte granule,
 *     i.e. at most 12 bytes (fp32) or 15 bytes (int8) past its last element; what is read
 *     there never reaches a stored result.  The granule lies in the same page, so the read
 *     cannot fault.
 *   - Any alignment of pointers and strides is accepted; rows that are 16-byte aligned
 *     (bases and row pitches) take the fastest path, rows that are only 4-byte aligned (any
 *     fp32 matrix; int8 rows at multiples of 4) one within about a tenth of it, everything
 *     else (int8 rows at odd addresses) a path about three times slower; the results are
 *     the same.
 */
#ifndef LSMI_H
#define LSMI_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum lsmi_status {
    LSMI_OK = 0,
    LSMI_ERR_DIM = -1,       /* negative extent; conv: C,K,R,S,stride <= 0, pad < 0, filter larger than padded image */
    LSMI_ERR_LD = -2,        /* lda < max(1,K), ldb < max(1,N) or ldc < max(1,N) */
    LSMI_ERR_NULL = -3,      /* null pointer for a tensor with a non-zero extent */
    LSMI_ERR_TOO_LARGE = -4, /* an extent or offset beyond what the kernels index (see each call) */
    LSMI_ERR_NO_DEVICE = -5, /* no usable gfx950 device */
    LSMI_ERR_LAUNCH = -6,    /* the HIP runtime refused the launch; see lsmi_last_hip_error() */
    LSMI_ERR_OP = -7         /* unknown pre- or post-operation code */
} lsmi_status;

/*
 * Element-wise operations around a contraction, C = post(pre(C_in) (+) A (x) B): the
 * pre-operation initialises the output, the post-operation transforms a value before it
 * is stored (Section 2.1, the formula that adds pre/post to the generalised contraction;
 * the paper names biases and activation functions as their use).
 */
typedef enum lsmi_pre {
    LSMI_PRE_ACCUMULATE = 0, /* pre(C_in) = C_in: add to the existing contents */
    LSMI_PRE_ZERO = 1,       /* pre(C_in) = 0: overwrite */
    LSMI_PRE_BIAS = 2        /* pre(C_in)[i,j] = bias[j]: a bias broadcast along rows */
} lsmi_pre;
typedef enum lsmi_post {
    LSMI_POST_NONE = 0,      /* post(x) = x */
    LSMI_POST_RELU = 1       /* post(x) = max(x, 0), the activation of the paper's MLP listing */
} lsmi_post;

/*
 * C[i*ldc + j] += sum_{k<K} A[i*lda + k] * B[k*ldb + j]   for i<M, j<N     (Section 2.1, Fig. 1)
 *
 * A: M x K, B: K x N, C: M x N, fp32, row-major with row strides lda, ldb, ldc.
 * Products and sums are true fp32 (fused multiply-add on the matrix cores); the order of
 * the k-summation is unspecified and, for small outputs with long K (a few rows of C
 * against a large B among them) and for the tiles left
 * over when the tile count is not a multiple of the number of compute units, partial sums
 * from several workgroups are combined with floating-point atomic adds, so two runs may
 * differ in the last bits (lsmi_set_tuning(-1, 1) keeps the reduction of every element in
 * one workgroup).  C is read and written; A and B are only read.
 * M, N or K equal to 0: nothing is done, C is untouched, LSMI_OK.
 * Limits: M, N, K, lda, ldb, ldc < 2^31 (row offsets are formed in 64 bits), else
 * LSMI_ERR_TOO_LARGE.
 */
int sgemm(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
          int64_t ldb, float *C, int64_t ldc);

/*
 * C[i*ldc + j] += sum_{k<K} a(i,k) * b(k,j),
 *     a(i,k) = transa ? A[k*lda + i] : A[i*lda + k],   b(k,j) = transb ? B[j*ldb + k] : B[k*ldb + j]
 *
 * sgemm on operands stored transposed: the transposition O[r,c] = I[c,r] of Section 2.1's list
 * of contractions, taken as the affine index map of an operand of the product (Section 2.1)
 * instead of a separate single-operand pass (Section 5.2) over it.  With transa != 0 the array
 * A holds the K x M transpose of the left operand (lda >= max(1, M)); with transb != 0 the
 * array B holds the N x K transpose of the right operand (ldb >= max(1, K)).  The swap is
 * applied while a tile is fetched into LDS; no copy of an operand is made and HBM is read
 * once, as for sgemm.  transa = transb = 0 is sgemm.  Zero extents, limits, summation order
 * and errors as for sgemm (LSMI_ERR_LD against the stored row lengths).
 */
int sgemm_op(int transa, int transb, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
             const float *B, int64_t ldb, float *C, int64_t ldc);

/*
 * sgemm whose result does not depend on the order in which workgroups finish: where the
 * reduction of an element is cut over several workgroups (small outputs with a long K, the
 * tiles of an incomplete last round), the partial sums do not meet in atomic adds onto C
 * but in `workspace`, and the last workgroup to arrive adds them in a fixed order (the
 * split and reorder of the reduction loop of Section 2.2, with the combination made
 * explicit).  Same value as sgemm up to summation order; two calls with the same arguments
 * give bit-identical results.  It is also the faster form for those shapes: plain stores
 * instead of floating-point atomics.
 * workspace: device memory, 256-byte aligned (else LSMI_ERR_DIM), of workspace_bytes bytes
 * (negative: LSMI_ERR_DIM), owned by the caller.  Its first 65536 bytes hold arrival counters:
 * they must be ZERO before the first call that uses the workspace, and every call leaves them
 * zero again; the rest is scratch and may hold anything.  lsmi_sgemm_ws_bytes() gives a
 * size with which no call is limited by the workspace; with less, fewer slices are used, and
 * with NULL or too little for a single partial tile every reduction stays in one workgroup.
 * Two calls that use the same workspace must not overlap in time (same stream, or ordered by
 * events).  Other arguments, zero extents and errors as for sgemm.
 */
int sgemm_ws(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb,
             float *C, int64_t ldc, void *workspace, int64_t workspace_bytes);

/* Bytes of workspace with which sgemm_ws is not limited by it for this shape with dense,
 * 16-byte aligned operands: the counters plus the partial tiles of the split the library would
 * choose (0: an empty or invalid shape, or one whose reductions stay whole). */
int64_t lsmi_sgemm_ws_bytes(int64_t M, int64_t N, int64_t K);

/*
 * sgemm_ws for callers that cannot allocate a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  The workspace is an array of
 * 8 MiB + 64 KiB inside the library's device code (one copy per GPU, held until the process
 * ends); the call allocates and frees nothing, on the host or on the device.  Result and
 * determinism as for sgemm_ws with that workspace.
 * A call whose partial sums would not fit the array (the split the library would choose for
 * these arguments needs more than 8 MiB of partial tiles: outputs of a few hundred 64 x 64
 * tiles cut several times) is refused with LSMI_ERR_TOO_LARGE and nothing is enqueued; such a
 * caller passes sgemm_ws a workspace of lsmi_sgemm_ws_bytes().
 * Every call on a GPU shares that GPU's array: calls that may overlap in time on one GPU
 * (different streams without an ordering between them, different threads) race on it and must
 * not be made.  The arrival counters at its start are zero when the library is loaded and
 * every call leaves them zero.  The first call on a device looks the array's address up
 * (hipGetSymbolAddress); LSMI_ERR_LAUNCH if that fails.  Other arguments, zero extents and
 * errors as for sgemm.
 */
int sgemm_static(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb,
                 float *C, int64_t ldc);

/*
 * C[i*ldc + j] = post(pre(C)[i,j] + sum_{k<K} A[i*lda + k] * B[k*ldb + j])
 *
 * sgemm with the pre- and post-operation of Section 2.1 fused into the epilogue (a fully
 * connected layer with bias and ReLU is one call, as in the MLP of Section 3's listing).
 * pre, post: lsmi_pre / lsmi_post codes, else LSMI_ERR_OP.  bias: N device floats, read only
 * when pre == LSMI_PRE_BIAS (then NULL is LSMI_ERR_NULL), ignored otherwise.  With
 * pre == LSMI_PRE_ACCUMULATE and post == LSMI_POST_NONE this is sgemm.  Every other form
 * is one kernel that keeps each element's whole reduction in one workgroup, and its result
 * is deterministic -- except on a small output with a long reduction (fewer than two
 * 64 x 64 tiles per compute unit, e.g. a fully connected layer at a batch of 1 to 64), where
 * that kernel would use a fraction of the GPU: there the call writes pre(C) out, runs sgemm on it
 * with the reduction cut (partial sums added atomically: the last bits can differ from run to
 * run, as for sgemm) and applies post in place, three launches on the same stream.
 * lsmi_set_tuning(-1, 1) keeps every reduction whole and the result deterministic.
 * M or N equal to 0: no-op.  K == 0: C = post(pre(C)) (A and B
 * are not read).  Other arguments, limits and errors as for sgemm.
 */
int sgemm_fused(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                int64_t ldb, float *C, int64_t ldc, const float *bias, int pre, int post);

/*
 * C[i*ldc + j] = (C[i*ldc + j] + sum_{k<K} (int32)A[i*lda + k] * (int32)B[k*ldb + j]) mod 2^32
 *
 * The generalised contraction of Section 2.1 with integer (+, *).  A: M x K and B: K x N
 * hold SIGNED 8-bit values; C: M x N int32.  Each product is exact and the sum wraps
 * modulo 2^32, so the result does not depend on summation order and is bit-exact.
 * Zero extents, limits and errors as for sgemm.
 */
int igemm_s8s32(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *B,
                int64_t ldb, int32_t *C, int64_t ldc);

/*
 * C[i*ldc + j] = (C[i*ldc + j] + sum_{k<K} (int32)A[i*lda + k] * (int32)Bt[j*ldbt + k]) mod 2^32
 *
 * igemm_s8s32 with the second operand given transposed: Bt is N x K, k-contiguous like A,
 * ldbt >= max(1, K).  This is the layout the single-operand contraction of Section 5.2
 * (tensor_copy_s8 with permuted strides) packs an operand into for the kernel that follows:
 * both operands then reach the matrix cores with one 16-byte LDS read per block operand.
 * Everything else as for igemm_s8s32; the result is bit-identical to it on the transpose.
 */
int igemm_s8s32_bt(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *Bt,
                   int64_t ldbt, int32_t *C, int64_t ldc);

/*
 * out[n,p,q,k] = sum_{r<R} sum_{s<S} sum_{c<C}
 *                    in[n, p*stride - pad + r, q*stride - pad + s, c] * w[k,r,s,c]
 * (Section 2.1: convolution as a contraction with affine index maps), a term being zero
 * where the input row or column index falls outside [0,H) x [0,W).
 *
 * in : N x H x W x C fp32 (NHWC, dense)      w : K x R x S x C fp32 (dense)
 * out: N x P x Q x K fp32 (dense), P = (H + 2*pad - R)/stride + 1, Q = (W + 2*pad - S)/stride + 1
 * (floor division).  One stride and one symmetric zero padding for both image axes; no
 * dilation, no groups.  out is OVERWRITTEN (its previous contents are ignored).
 * N = 0 (or H, W such that the output is empty is not possible once the checks pass):
 * nothing is done.  Errors: LSMI_ERR_DIM if N,H,W < 0, any of C,K,R,S,stride <= 0, pad < 0,
 * or H + 2*pad < R or W + 2*pad < S; LSMI_ERR_TOO_LARGE if any tensor has 2^31 or more
 * elements or R*S*C >= 2^31.  Any C and alignment is accepted; 16-byte aligned tensors with
 * C % 16 == 0 take the fastest kernels, C % 4 == 0 and any other C (a stem of 3 channels)
 * forms of the same kernels that run at about 0.8 and 0.7 of their rate.
 */
int conv2d_nhwc(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                int64_t stride, int64_t pad, const float *in, const float *w, float *out);

/*
 * out[n,p,q,k] = post(bias[k] + conv2d_nhwc(...)[n,p,q,k]): the convolution with a per-channel
 * bias as pre-operation (bias == NULL: none) and `post` (lsmi_post code, else LSMI_ERR_OP)
 * as post-operation, fused into the epilogue.  bias: K device floats.  Everything else as
 * for conv2d_nhwc, which is this call with bias == NULL and post == LSMI_POST_NONE.
 */
int conv2d_nhwc_fused(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                      int64_t stride, int64_t pad, const float *in, const float *w, float *out,
                      const float *bias, int post);

/*
 * out[n,p,q,c] = sum_{r<R} sum_{s<S} in[n, p*stride - pad + r, q*stride - pad + s, c] * w[r,s,c]
 *
 * Depth-wise convolution (the DWCONV rows of Table 1): the convolution of Section 2.1 with
 * the channel index shared by input, filter and output instead of being reduced, one 2-D
 * filter per channel, channel multiplier 1.  A term is zero where the input row or column
 * index falls outside [0,H) x [0,W).
 *
 * in : N x H x W x C fp32 (NHWC, dense)      w : R x S x C fp32 (dense, channels contiguous)
 * out: N x P x Q x C fp32 (dense), P and Q as for conv2d_nhwc.  out is OVERWRITTEN.
 * N = 0: nothing is done.  Errors as for conv2d_nhwc (without K).  Any C, R, S, stride,
 * pad and alignment is accepted; C % 4 == 0 with 16-byte aligned tensors and a 3x3, 5x5 or
 * 7x7 filter at stride 1 or 2 takes the fastest kernels.
 */
int dwconv2d_nhwc(int64_t N, int64_t H, int64_t W, int64_t C, int64_t R, int64_t S, int64_t stride,
                  int64_t pad, const float *in, const float *w, float *out);

/*
 * out[n,p,q,c] = post(bias[c] + dwconv2d_nhwc(...)[n,p,q,c]): per-channel bias as
 * pre-operation (bias == NULL: none; else C device floats) and `post` (lsmi_post code, else
 * LSMI_ERR_OP) as post-operation of Section 2.1's general form, applied before the store.
 * dwconv2d_nhwc is this call with bias == NULL and post == LSMI_POST_NONE.
 */
int dwconv2d_nhwc_fused(int64_t N, int64_t H, int64_t W, int64_t C, int64_t R, int64_t S,
                        int64_t stride, int64_t pad, const float *in, const float *w, float *out,
                        const float *bias, int post);

/*
 * out[i0,i1,i2,i3] = in[i0*s0 + i1*s1 + i2*s2 + i3*s3]
 *
 * The single-operand form of the contraction (Section 5.2, "Single Operand LoopNest"; the
 * transpositions O[r,c] = I[c,r] and broadcasts O[r,c] = I[r] of Section 2.1): no reduction
 * index, one input.  out is dense row-major with extents d0 x d1 x d2 x d3; the input is
 * addressed through the non-negative element strides s0..s3 from `in`.  Permuted strides
 * transpose (NCHW <-> NHWC, a matrix transpose, packing a B operand k-contiguously), the
 * strides of an enclosing tensor extract a sub-tensor (point `in` at its first element), a
 * stride of 0 broadcasts.  Pure data movement: bit-exact.  in and out must not overlap.
 * Any extent 0: nothing is done.  Errors: LSMI_ERR_DIM for a negative extent or stride,
 * LSMI_ERR_TOO_LARGE if an extent or stride, the element count, or the largest input
 * offset exceeds 2^31 - 1, LSMI_ERR_NULL for a null pointer with a non-empty output.
 * Any alignment is accepted; 16-byte aligned bases and strides take the widest accesses.
 */
int tensor_copy_f32(int64_t d0, int64_t d1, int64_t d2, int64_t d3, int64_t s0, int64_t s1, int64_t s2,
                    int64_t s3, const float *in, float *out);

/* The same for 8-bit elements (the operands of igemm_s8s32). */
int tensor_copy_s8(int64_t d0, int64_t d1, int64_t d2, int64_t d3, int64_t s0, int64_t s1, int64_t s2,
                   int64_t s3, const int8_t *in, int8_t *out);

/*
 * Stream on which the calling thread's later calls enqueue their kernels.  hip_stream is
 * a hipStream_t passed as void*; NULL selects the null stream.  The stream must stay
 * alive while calls use it.  Always returns LSMI_OK.
 */
int lsmi_set_stream(void *hip_stream);

/* Static, NUL-terminated description of a status code (never NULL). */
const char *lsmi_strerror(int status);

/* hipError_t (as int) recorded by the calling thread's last LSMI_ERR_LAUNCH / LSMI_ERR_NO_DEVICE, else 0. */
int lsmi_last_hip_error(void);

/* Library version: major*10000 + minor*100 + patch. */
int lsmi_version(void);

/*
 * Name of the kernel variant the calling thread's last successful compute call launched
 * (static string such as "sgemm_128x128x16_splitk1"); "" before the first call.  For
 * benchmarks and tests that want to report or pin the dispatch decision.
 */
const char *lsmi_last_variant(void);

#ifdef __cplusplus
}
#endif
#endif /* LSMI_H */
