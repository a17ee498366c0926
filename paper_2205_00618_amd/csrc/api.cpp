// C ABI of the library: argument validation (pure host code, no GPU needed), per-thread
// state, and hand-off to the launchers.  The operations are the three instances of the
// generalised contraction of Section 2.1 described in the public header.
#include <atomic>
#include <cstring>
#include <initializer_list>
#include <mutex>

#include "common.hpp"

namespace lsmi {

ThreadState &tls()
{
    static thread_local ThreadState state;
    return state;
}

namespace {
std::once_flag g_device_once;
int g_device_status = LSMI_ERR_NO_DEVICE;
int g_device_hip_error = 0;
int g_cu_count = 0;
}  // namespace

int ensure_device()
{
    std::call_once(g_device_once, [] {
        int count = 0;
        hipError_t err = hipGetDeviceCount(&count);
        if (err != hipSuccess || count <= 0) {
            g_device_hip_error = static_cast<int>(err != hipSuccess ? err : hipErrorNoDevice);
            (void)hipGetLastError();
            return;
        }
        int dev = 0;
        err = hipGetDevice(&dev);
        hipDeviceProp_t prop;
        if (err == hipSuccess) err = hipGetDeviceProperties(&prop, dev);
        if (err != hipSuccess) {
            g_device_hip_error = static_cast<int>(err);
            (void)hipGetLastError();
            return;
        }
        if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) {
            g_device_hip_error = static_cast<int>(hipErrorInvalidDevice);
            return;
        }
        g_cu_count = prop.multiProcessorCount;
        g_device_status = LSMI_OK;
    });
    if (g_device_status != LSMI_OK) tls().last_hip_error = g_device_hip_error;
    return g_device_status;
}

int device_cu_count() { return g_cu_count > 0 ? g_cu_count : 256; }

int check_launch()
{
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) {
        tls().last_hip_error = static_cast<int>(err);
        return LSMI_ERR_LAUNCH;
    }
    return LSMI_OK;
}

namespace {

constexpr int64_t kMaxExtent = INT32_MAX;

// Shared by sgemm and igemm_s8s32.  Returns LSMI_OK with *empty set when there is no work.
int validate_gemm(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                  int64_t ldb, const void *C, int64_t ldc, bool *empty)
{
    *empty = false;
    if (M < 0 || N < 0 || K < 0) return LSMI_ERR_DIM;
    if (lda < (K > 1 ? K : 1) || ldb < (N > 1 ? N : 1) || ldc < (N > 1 ? N : 1)) return LSMI_ERR_LD;
    if (M > kMaxExtent || N > kMaxExtent || K > kMaxExtent || lda > kMaxExtent ||
        ldb > kMaxExtent || ldc > kMaxExtent)
        return LSMI_ERR_TOO_LARGE;
    if (M == 0 || N == 0 || K == 0) {
        *empty = true;
        return LSMI_OK;
    }
    if (A == nullptr || B == nullptr || C == nullptr) return LSMI_ERR_NULL;
    return LSMI_OK;
}

// Whether the product of the (non-negative, <= 2^31) factors stays within kMaxExtent.
bool product_fits(std::initializer_list<int64_t> factors)
{
    int64_t acc = 1;
    for (int64_t f : factors) {
        if (f == 0) return true;
        if (acc > kMaxExtent / f) return false;
        acc *= f;
    }
    return true;
}

}  // namespace
}  // namespace lsmi

using namespace lsmi;

extern "C" {

int sgemm(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
          int64_t ldb, float *C, int64_t ldc)
{
    bool empty;
    int rc = validate_gemm(M, N, K, A, lda, B, ldb, C, ldc, &empty);
    if (rc != LSMI_OK || empty) return rc;
    if ((rc = ensure_device()) != LSMI_OK) return rc;
    return launch_sgemm((int)M, (int)N, (int)K, A, lda, B, ldb, C, ldc, nullptr, LSMI_PRE_ACCUMULATE,
                        LSMI_POST_NONE);
}

int sgemm_op(int transa, int transb, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
             const float *B, int64_t ldb, float *C, int64_t ldc)
{
    if (M < 0 || N < 0 || K < 0) return LSMI_ERR_DIM;
    // the stored A is K x M when transposed, the stored B N x K
    const int64_t a_cols = transa ? M : K, b_cols = transb ? K : N;
    if (lda < (a_cols > 1 ? a_cols : 1) || ldb < (b_cols > 1 ? b_cols : 1) || ldc < (N > 1 ? N : 1)) return LSMI_ERR_LD;
    if (M > kMaxExtent || N > kMaxExtent || K > kMaxExtent || lda > kMaxExtent || ldb > kMaxExtent ||
        ldc > kMaxExtent)
        return LSMI_ERR_TOO_LARGE;
    if (M == 0 || N == 0 || K == 0) return LSMI_OK;
    if (A == nullptr || B == nullptr || C == nullptr) return LSMI_ERR_NULL;
    int rc = ensure_device();
    if (rc != LSMI_OK) return rc;
    return launch_sgemm((int)M, (int)N, (int)K, A, lda, B, ldb, C, ldc, nullptr, LSMI_PRE_ACCUMULATE,
                        LSMI_POST_NONE, transa != 0, transb != 0);
}

int64_t lsmi_sgemm_ws_bytes(int64_t M, int64_t N, int64_t K)
{
    if (M <= 0 || N <= 0 || K <= 0 || M > kMaxExtent || N > kMaxExtent || K > kMaxExtent) return 0;
    // the plan of the call with dense, 16-byte aligned operands and an unlimited workspace
    // (on a host without a device: for 256 compute units)
    (void)ensure_device();
    float *const aligned = reinterpret_cast<float *>(uintptr_t{4096});
    int64_t bytes = 0;
    launch_sgemm((int)M, (int)N, (int)K, aligned, K, aligned, N, aligned, N, nullptr, LSMI_PRE_ACCUMULATE,
                 LSMI_POST_NONE, false, false, aligned, INT64_MAX / 2, true, &bytes);
    return bytes;
}

int sgemm_ws(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb,
             float *C, int64_t ldc, void *workspace, int64_t workspace_bytes)
{
    bool empty;
    int rc = validate_gemm(M, N, K, A, lda, B, ldb, C, ldc, &empty);
    if (rc != LSMI_OK) return rc;
    if (workspace_bytes < 0) return LSMI_ERR_DIM;
    if (empty) return LSMI_OK;
    if (workspace != nullptr && (reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return LSMI_ERR_DIM;
    if ((rc = ensure_device()) != LSMI_OK) return rc;
    return launch_sgemm((int)M, (int)N, (int)K, A, lda, B, ldb, C, ldc, nullptr, LSMI_PRE_ACCUMULATE,
                        LSMI_POST_NONE, false, false, workspace, workspace != nullptr ? workspace_bytes : 0, true);
}

int sgemm_static(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb,
                 float *C, int64_t ldc)
{
    bool empty;
    int rc = validate_gemm(M, N, K, A, lda, B, ldb, C, ldc, &empty);
    if (rc != LSMI_OK || empty) return rc;
    if ((rc = ensure_device()) != LSMI_OK) return rc;
    // what this very call would put into an unlimited workspace must fit the library's array
    int64_t need = 0;
    launch_sgemm((int)M, (int)N, (int)K, A, lda, B, ldb, C, ldc, nullptr, LSMI_PRE_ACCUMULATE, LSMI_POST_NONE,
                 false, false, C, INT64_MAX / 2, true, &need);
    if (need > kSgemmCounterBytes + kSgemmStaticPartialBytes) return LSMI_ERR_TOO_LARGE;
    void *scratch_ptr = nullptr;
    if ((rc = sgemm_static_scratch(&scratch_ptr)) != LSMI_OK) return rc;
    return launch_sgemm((int)M, (int)N, (int)K, A, lda, B, ldb, C, ldc, nullptr, LSMI_PRE_ACCUMULATE,
                        LSMI_POST_NONE, false, false, scratch_ptr, kSgemmCounterBytes + kSgemmStaticPartialBytes, true);
}

int sgemm_fused(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                int64_t ldb, float *C, int64_t ldc, const float *bias, int pre, int post)
{
    if (pre != LSMI_PRE_ACCUMULATE && pre != LSMI_PRE_ZERO && pre != LSMI_PRE_BIAS) return LSMI_ERR_OP;
    if (post != LSMI_POST_NONE && post != LSMI_POST_RELU) return LSMI_ERR_OP;
    bool empty;
    int rc = validate_gemm(M, N, K, A, lda, B, ldb, C, ldc, &empty);  // no pointer checks when K == 0
    if (rc != LSMI_OK) return rc;
    // an empty reduction still applies pre and post to every element of C
    const bool identity = pre == LSMI_PRE_ACCUMULATE && post == LSMI_POST_NONE;
    if (M == 0 || N == 0 || (K == 0 && identity)) return LSMI_OK;
    if (C == nullptr) return LSMI_ERR_NULL;
    if (pre == LSMI_PRE_BIAS && bias == nullptr) return LSMI_ERR_NULL;
    if ((rc = ensure_device()) != LSMI_OK) return rc;
    return launch_sgemm((int)M, (int)N, (int)K, A, lda, B, ldb, C, ldc, bias, pre, post);
}

int igemm_s8s32(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *B,
                int64_t ldb, int32_t *C, int64_t ldc)
{
    bool empty;
    int rc = validate_gemm(M, N, K, A, lda, B, ldb, C, ldc, &empty);
    if (rc != LSMI_OK || empty) return rc;
    if ((rc = ensure_device()) != LSMI_OK) return rc;
    return launch_igemm((int)M, (int)N, (int)K, A, lda, B, ldb, C, ldc, false);
}

int igemm_s8s32_bt(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *Bt,
                   int64_t ldbt, int32_t *C, int64_t ldc)
{
    // Bt is N x K: its rows are as long as A's
    if (M < 0 || N < 0 || K < 0) return LSMI_ERR_DIM;
    if (lda < (K > 1 ? K : 1) || ldbt < (K > 1 ? K : 1) || ldc < (N > 1 ? N : 1)) return LSMI_ERR_LD;
    if (M > kMaxExtent || N > kMaxExtent || K > kMaxExtent || lda > kMaxExtent || ldbt > kMaxExtent ||
        ldc > kMaxExtent)
        return LSMI_ERR_TOO_LARGE;
    if (M == 0 || N == 0 || K == 0) return LSMI_OK;
    if (A == nullptr || Bt == nullptr || C == nullptr) return LSMI_ERR_NULL;
    int rc = ensure_device();
    if (rc != LSMI_OK) return rc;
    return launch_igemm((int)M, (int)N, (int)K, A, lda, Bt, ldbt, C, ldc, true);
}

int conv2d_nhwc(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                int64_t stride, int64_t pad, const float *in, const float *w, float *out)
{
    return conv2d_nhwc_fused(N, H, W, C, K, R, S, stride, pad, in, w, out, nullptr, LSMI_POST_NONE);
}

int conv2d_nhwc_fused(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                      int64_t stride, int64_t pad, const float *in, const float *w, float *out,
                      const float *bias, int post)
{
    if (post != LSMI_POST_NONE && post != LSMI_POST_RELU) return LSMI_ERR_OP;
    if (N < 0 || H < 0 || W < 0 || C <= 0 || K <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0)
        return LSMI_ERR_DIM;
    // every extent is bounded first so that the products below cannot overflow 64 bits
    const int64_t lim = kMaxExtent;
    if (N > lim || H > lim || W > lim || C > lim || K > lim || R > lim || S > lim || stride > lim ||
        pad > lim / 4)
        return LSMI_ERR_TOO_LARGE;
    if (H + 2 * pad < R || W + 2 * pad < S) return LSMI_ERR_DIM;
    const int64_t P = (H + 2 * pad - R) / stride + 1;
    const int64_t Q = (W + 2 * pad - S) / stride + 1;
    auto fits = [](int64_t a, int64_t b, int64_t c, int64_t d) {
        // a*b*c*d <= lim, evaluated without overflow (all factors are <= 2^31)
        int64_t acc = 1;
        for (int64_t f : {a, b, c, d}) {
            if (f == 0) return true;
            if (acc > lim / f) return false;
            acc *= f;
        }
        return true;
    };
    if (!fits(N, H, W, C) || !fits(K, R, S, C) || !fits(N, P, Q, K) || !fits(R, S, C, 1) ||
        H + 2 * pad > lim || W + 2 * pad > lim)
        return LSMI_ERR_TOO_LARGE;
    if (N == 0) return LSMI_OK;  // P, Q >= 1 once the checks above pass
    if (w == nullptr || out == nullptr) return LSMI_ERR_NULL;
    if (in == nullptr && H * W > 0) return LSMI_ERR_NULL;
    int rc = ensure_device();
    if (rc != LSMI_OK) return rc;
    return launch_conv2d((int)N, (int)H, (int)W, (int)C, (int)K, (int)R, (int)S, (int)stride,
                         (int)pad, (int)P, (int)Q, in, w, out, bias, post);
}

int dwconv2d_nhwc(int64_t N, int64_t H, int64_t W, int64_t C, int64_t R, int64_t S, int64_t stride,
                  int64_t pad, const float *in, const float *w, float *out)
{
    return dwconv2d_nhwc_fused(N, H, W, C, R, S, stride, pad, in, w, out, nullptr, LSMI_POST_NONE);
}

int dwconv2d_nhwc_fused(int64_t N, int64_t H, int64_t W, int64_t C, int64_t R, int64_t S,
                        int64_t stride, int64_t pad, const float *in, const float *w, float *out,
                        const float *bias, int post)
{
    if (post != LSMI_POST_NONE && post != LSMI_POST_RELU) return LSMI_ERR_OP;
    if (N < 0 || H < 0 || W < 0 || C <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0)
        return LSMI_ERR_DIM;
    const int64_t lim = kMaxExtent;
    if (N > lim || H > lim || W > lim || C > lim || R > lim || S > lim || stride > lim || pad > lim / 4)
        return LSMI_ERR_TOO_LARGE;
    if (H + 2 * pad < R || W + 2 * pad < S) return LSMI_ERR_DIM;
    const int64_t P = (H + 2 * pad - R) / stride + 1;
    const int64_t Q = (W + 2 * pad - S) / stride + 1;
    if (!product_fits({N, H, W, C}) || !product_fits({N, P, Q, C}) || !product_fits({R, S, C}) ||
        !product_fits({H + 2 * pad, stride}) || !product_fits({W + 2 * pad, stride}))
        return LSMI_ERR_TOO_LARGE;
    if (N == 0) return LSMI_OK;
    if (w == nullptr || out == nullptr) return LSMI_ERR_NULL;
    if (in == nullptr && H * W > 0) return LSMI_ERR_NULL;
    int rc = ensure_device();
    if (rc != LSMI_OK) return rc;
    return launch_dwconv2d((int)N, (int)H, (int)W, (int)C, (int)R, (int)S, (int)stride, (int)pad,
                           (int)P, (int)Q, in, w, out, bias, post);
}

static int tensor_copy_any(int esize, int64_t d0, int64_t d1, int64_t d2, int64_t d3, int64_t s0, int64_t s1,
                           int64_t s2, int64_t s3, const void *in, void *out)
{
    const int64_t d[4] = {d0, d1, d2, d3}, s[4] = {s0, s1, s2, s3};
    int64_t total = 1, last = 0;
    for (int a = 0; a < 4; ++a)
        if (d[a] < 0 || s[a] < 0) return LSMI_ERR_DIM;
    for (int a = 0; a < 4; ++a) {
        if (d[a] > kMaxExtent || s[a] > kMaxExtent) return LSMI_ERR_TOO_LARGE;
        if (d[a] == 0) return LSMI_OK;
        if (total > kMaxExtent / d[a]) return LSMI_ERR_TOO_LARGE;
        total *= d[a];
        last += (d[a] - 1) * s[a];  // each term below 2^62 / 4: no overflow
        if (last > kMaxExtent) return LSMI_ERR_TOO_LARGE;
    }
    if (in == nullptr || out == nullptr) return LSMI_ERR_NULL;
    int rc = ensure_device();
    if (rc != LSMI_OK) return rc;
    return launch_tensor_copy(esize, d, s, in, out);
}

int tensor_copy_f32(int64_t d0, int64_t d1, int64_t d2, int64_t d3, int64_t s0, int64_t s1, int64_t s2,
                    int64_t s3, const float *in, float *out)
{
    return tensor_copy_any(4, d0, d1, d2, d3, s0, s1, s2, s3, in, out);
}

int tensor_copy_s8(int64_t d0, int64_t d1, int64_t d2, int64_t d3, int64_t s0, int64_t s1, int64_t s2,
                   int64_t s3, const int8_t *in, int8_t *out)
{
    return tensor_copy_any(1, d0, d1, d2, d3, s0, s1, s2, s3, in, out);
}

int lsmi_set_stream(void *hip_stream)
{
    tls().stream = static_cast<hipStream_t>(hip_stream);
    return LSMI_OK;
}

const char *lsmi_strerror(int status)
{
    switch (status) {
    case LSMI_OK: return "success";
    case LSMI_ERR_DIM: return "invalid dimension";
    case LSMI_ERR_LD: return "leading dimension smaller than the row length";
    case LSMI_ERR_NULL: return "null pointer for a non-empty tensor";
    case LSMI_ERR_TOO_LARGE: return "extent beyond the supported index range";
    case LSMI_ERR_NO_DEVICE: return "no usable gfx950 device";
    case LSMI_ERR_LAUNCH: return "HIP runtime error at kernel launch";
    case LSMI_ERR_OP: return "unknown pre- or post-operation";
    default: return "unknown status";
    }
}

int lsmi_last_hip_error(void) { return tls().last_hip_error; }

int lsmi_version(void) { return 153; }

const char *lsmi_last_variant(void) { return tls().last_variant; }

int lsmi_last_split(void) { return tls().last_split; }

int lsmi_set_tuning(int sgemm_variant, int split_k)
{
    if (sgemm_variant < -1 || sgemm_variant >= sgemm_variant_count() || split_k < 0)
        return LSMI_ERR_DIM;
    tls().forced_variant = sgemm_variant;
    tls().forced_split_k = split_k;
    return LSMI_OK;
}

int lsmi_set_tile_walk(int band_rows)
{
    if (band_rows < 0 || band_rows > 65535) return LSMI_ERR_DIM;
    tls().forced_group_m = band_rows;
    return LSMI_OK;
}

int lsmi_set_dwconv_tuning(int dwconv_variant, int strip)
{
    if (dwconv_variant < -1 || dwconv_variant >= dwconv_variant_count() || strip < 0) return LSMI_ERR_DIM;
    tls().forced_dwconv_variant = dwconv_variant;
    tls().forced_dwconv_strip = strip;
    return LSMI_OK;
}

int lsmi_set_igemm_tuning(int igemm_variant)
{
    if (igemm_variant < -1 || igemm_variant >= igemm_variant_count()) return LSMI_ERR_DIM;
    tls().forced_igemm_variant = igemm_variant;
    return LSMI_OK;
}

const char *lsmi_igemm_variant_name(int index) { return igemm_variant_name(index); }

int lsmi_set_conv_split(int slices)
{
    if (slices < 0) return LSMI_ERR_DIM;
    tls().forced_conv_slices = slices;
    return LSMI_OK;
}

int lsmi_set_conv_tail(int tile_rows)
{
    if (tile_rows < -1) return LSMI_ERR_DIM;
    tls().forced_conv_tail = tile_rows;
    return LSMI_OK;
}

const char *lsmi_conv_variant_name(int index) { return conv_variant_name(index); }

int lsmi_set_dwconv_tile(int cols, int channels, int depth)
{
    if (cols < 0 || channels < 0 || depth < 0 || depth > 2) return LSMI_ERR_DIM;
    tls().forced_dwconv_cols = cols;
    tls().forced_dwconv_channels = channels;
    tls().forced_dwconv_depth = depth;
    return LSMI_OK;
}

const char *lsmi_dwconv_variant_name(int index) { return dwconv_variant_name(index); }

int lsmi_set_conv_tuning(int conv_variant)
{
    if (conv_variant < -1 || conv_variant >= conv_variant_count()) return LSMI_ERR_DIM;
    tls().forced_conv_variant = conv_variant;
    return LSMI_OK;
}

const char *lsmi_variant_name(int index) { return sgemm_variant_name(index); }

uint32_t lsmi_fast_divide(uint32_t n, uint32_t d) { return fast_divide(n, d); }

int lsmi_tile_of_workgroup(int wg, int tiles_m, int tiles_n, int group_m, int *tile_row,
                           int *tile_col)
{
    if (tiles_m < 1 || tiles_n < 1 || group_m < 1 || wg < 0 || tile_row == nullptr ||
        tile_col == nullptr || (int64_t)wg >= (int64_t)tiles_m * tiles_n)
        return LSMI_ERR_DIM;
    tile_of_workgroup(wg, tiles_m, tiles_n, group_m, tile_row, tile_col);
    return LSMI_OK;
}

}  // extern "C"
