// Shared host-side declarations of the library: status codes come from the public header,
// the per-thread state (stream, last variant, tuning override) and the launchers that the
// four .hip files define live here.
#pragma once

#include <cstdint>
#include <hip/hip_runtime.h>

#include "../../include/lsmi.h"
#include "../../include/lsmi_tune.h"

namespace lsmi {

struct ThreadState {
    hipStream_t stream = nullptr;
    int last_hip_error = 0;
    const char *last_variant = "";
    int last_split = 1;  // reduction slices of the last sgemm launch
    int forced_variant = -1;  // sgemm tile configuration override, -1 = built-in choice
    int forced_split_k = 0;   // 0 = built-in choice
    int forced_group_m = 0;   // tile rows per band of the tile walk, 0 = built-in choice
    int forced_conv_variant = -1;
    int forced_conv_slices = 0;  // reduction slices of the direct-to-LDS conv kernels, 0 = built-in choice
    int forced_conv_tail = -1;   // tile rows computed as quarter-tile pieces, -1 = built-in choice
    int forced_igemm_variant = -1;
    int forced_dwconv_variant = -1;
    int forced_dwconv_strip = 0;  // output rows per lane / per workgroup, 0 = built-in choice
    int forced_dwconv_cols = 0, forced_dwconv_channels = 0, forced_dwconv_depth = 0;  // LDS-staged tile
};

ThreadState &tls();

// Checks once per process that device 0.. current is a gfx950 part.  Returns LSMI_OK or
// LSMI_ERR_NO_DEVICE (recording the HIP error in the thread state).
int ensure_device();

// Number of compute units of the current device (cached after ensure_device()).
int device_cu_count();

// Converts the status of a kernel launch into a library status.
int check_launch();

// Launchers: arguments already validated, all extents non-zero.
// pre / post: the element-wise operations of the public header (lsmi_pre, lsmi_post)
// ta / tb: the operand is stored transposed (A as K x M, B as N x K).  workspace: device
// memory where the partial sums of a cut reduction meet instead of in atomic adds onto C, or
// nullptr; it starts with kSgemmCounterBytes of arrival counters (zero between calls), then
// partial tiles.  no_atomics: never combine partial sums with atomic adds.
// plan_bytes: when not null nothing is launched and *plan_bytes receives the bytes of workspace
// the call's partial sums would occupy if the workspace did not limit them (0: nothing is cut).
constexpr int64_t kSgemmCounterBytes = 65536;
int launch_sgemm(int M, int N, int K, const float *A, int64_t lda, const float *B, int64_t ldb,
                 float *C, int64_t ldc, const float *bias, int pre, int post, bool ta = false, bool tb = false,
                 void *workspace = nullptr, int64_t workspace_bytes = 0, bool no_atomics = false,
                 int64_t *plan_bytes = nullptr);

// The workspace of sgemm_static: a device array of kSgemmCounterBytes + kSgemmStaticPartialBytes
// bytes that lives in the library.  Stores this device's address of it in *ptr.
constexpr int64_t kSgemmStaticPartialBytes = 8 << 20;
int sgemm_static_scratch(void **ptr);
// bt: B is given transposed, N x K with row stride ldb
int launch_igemm(int M, int N, int K, const int8_t *A, int64_t lda, const int8_t *B, int64_t ldb,
                 int32_t *C, int64_t ldc, bool bt);
int launch_conv2d(int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int P,
                  int Q, const float *in, const float *w, float *out, const float *bias, int post);

int launch_dwconv2d(int N, int H, int W, int C, int R, int S, int stride, int pad, int P, int Q,
                    const float *in, const float *w, float *out, const float *bias, int post);

// esize 4 (fp32) or 1 (int8); extents non-zero
int launch_tensor_copy(int esize, const int64_t d[4], const int64_t s[4], const void *in, void *out);

void tile_of_workgroup(int wg, int tiles_m, int tiles_n, int group_m, int *tm, int *tn);
uint32_t fast_divide(uint32_t n, uint32_t d);  // FastDiv(d).div(n) of tile_f32.hpp, on the host
int sgemm_variant_count();
int conv_variant_count();
int igemm_variant_count();
const char *igemm_variant_name(int index);
int dwconv_variant_count();
const char *dwconv_variant_name(int index);
const char *conv_variant_name(int index);
const char *sgemm_variant_name(int index);

}  // namespace lsmi
