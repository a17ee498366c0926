// Calibration of the matrix pipes: a loop of matrix instructions on registers alone (no
// memory, no LDS), timed, with the shader clock read beside it.  It is the figure a kernel's
// rate is to be compared with besides the datasheet peak: what the part sustains under the
// instruction stream and operand activity in question.
//
// Every wave issues dependent chains on four independent accumulator blocks, which keeps the
// pipe of its SIMD full; four workgroups of four waves per CU.  The operands are either the
// same registers in every instruction (no switching activity at the multipliers' inputs) or
// eight different register sets of pseudo-random values taken in rotation, which is what a
// GEMM on random matrices presents.  The shader clock is the ratio of the cycle counter to
// the constant 100 MHz counter over the loop, averaged over the workgroups.
#include <vector>

#include "common.hpp"

namespace lsmi {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

__device__ inline uint32_t mix(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

template <bool INT8>
__global__ __launch_bounds__(256) void mfma_rate_kernel(uint64_t *counters, int iters, int random, float *sink)
{
    const uint32_t id = blockIdx.x * 256u + threadIdx.x;
    float fa[8], fb[8];
    i32x4 ia[8], ib[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const uint32_t h = random ? mix(id * 8u + r + 1u) : 0x3f803f80u;
        const uint32_t g = random ? mix(h) : 0x01010101u;
        fa[r] = random ? (float)(int)(h & 0xffffu) * (1.f / 32768.f) - 1.f : 1.f;
        fb[r] = random ? (float)(int)(g & 0xffffu) * (1.f / 32768.f) - 1.f : 1.f;
        ia[r] = i32x4{(int)h, (int)mix(h + 1), (int)mix(h + 2), (int)mix(h + 3)};
        ib[r] = i32x4{(int)g, (int)mix(g + 1), (int)mix(g + 2), (int)mix(g + 3)};
        if (!random) ia[r] = ib[r] = i32x4{0x01010101, 0x01010101, 0x01010101, 0x01010101};
    }
    f32x16 facc[4];
    i32x16 iacc[4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            facc[a][v] = 0.f;
            iacc[a][v] = 0;
        }
    const uint64_t c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int r = 0; r < 8; ++r)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                if constexpr (INT8)
                    iacc[a] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ia[r], ib[r], iacc[a], 0, 0, 0);
                else
                    facc[a] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[r], fb[r], facc[a], 0, 0, 0);
            }
    }
    float s = 0.f;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += INT8 ? (float)iacc[a][v] : facc[a][v];
    const uint64_t c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
    if (threadIdx.x == 0) {
        counters[2 * blockIdx.x] = c1 - c0;
        counters[2 * blockIdx.x + 1] = r1 - r0;
    }
    if (s == 12345.678f) *sink = s;  // keeps the accumulators alive; practically never taken
}

}  // namespace
}  // namespace lsmi

using namespace lsmi;

extern "C" int lsmi_mfma_rate(int int8, int random_operands, void *device_words, int64_t words,
                              double *ops_per_second, double *shader_clock_hz)
{
    if (ops_per_second == nullptr || shader_clock_hz == nullptr) return LSMI_ERR_NULL;
    int rc = ensure_device();
    if (rc != LSMI_OK) return rc;
    const int wgs = 4 * device_cu_count();
    if (device_words == nullptr) return LSMI_ERR_NULL;
    if (words < 2 * (int64_t)wgs + 1) return LSMI_ERR_DIM;
    uint64_t *counters = static_cast<uint64_t *>(device_words);
    float *sink = reinterpret_cast<float *>(counters + 2 * wgs);
    hipStream_t s = tls().stream;
    const int iters = int8 ? 8000 : 4000;  // 32 instructions per iteration, 32 (int8) or 64 (fp32) cycles each
    auto launch = [&](int n) {
        if (int8)
            hipLaunchKernelGGL(mfma_rate_kernel<true>, dim3(wgs), dim3(256), 0, s, counters, n, random_operands, sink);
        else
            hipLaunchKernelGGL(mfma_rate_kernel<false>, dim3(wgs), dim3(256), 0, s, counters, n, random_operands, sink);
    };
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return check_launch();
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return check_launch();
    }
    for (int w = 0; w < 3; ++w) launch(iters);  // clocks settle under this load
    hipError_t err = hipEventRecord(e0, s);
    launch(iters);
    if (err == hipSuccess) err = hipEventRecord(e1, s);
    if (err == hipSuccess) err = hipEventSynchronize(e1);
    float ms = 0.f;
    if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
    std::vector<uint64_t> host(2 * (size_t)wgs);
    if (err == hipSuccess) err = hipMemcpy(host.data(), counters, host.size() * sizeof(uint64_t), hipMemcpyDeviceToHost);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (err != hipSuccess) {
        tls().last_hip_error = (int)err;
        (void)hipGetLastError();
        return LSMI_ERR_LAUNCH;
    }
    double cycles = 0, ticks = 0;
    for (int i = 0; i < wgs; ++i) {
        cycles += (double)host[2 * i];
        ticks += (double)host[2 * i + 1];
    }
    // per instruction: 32 x 32 outputs x k multiply-adds x 2
    const double ops_per_instr = 2.0 * 32 * 32 * (int8 ? 32 : 2);
    *ops_per_second = ops_per_instr * 32.0 * iters * 4.0 * wgs / (ms * 1e-3);
    *shader_clock_hz = ticks > 0 ? cycles / ticks * 100e6 : 0.0;
    return LSMI_OK;
}
