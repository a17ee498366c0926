// sgemm for outputs of a few rows (M up to 16 or 32) against a large B: the loop nest of
// Fig. 1 with the i extent so small that the time goes into reading B once.  A 64-row tile
// would spend its matrix instructions on rows that do not exist (8 x 4096 x 4096: 23 us, all
// of it matrix-pipe time); here a wave multiplies 16-row blocks with MFMA 16x16x4 and takes B
// straight from global memory into the registers the instruction wants, without LDS and
// without barriers in the loop.
//
// A workgroup of four waves owns 64 columns and a slice of the reduction; wave w takes the
// w-th quarter of the slice, 16 reduction elements per step.  Lane (q, i) = (lane / 16,
// lane % 16) loads, for j = 0 .. 3, the 16 bytes B[k + 4q + j][4i .. 4i + 3]: a row of the step
// is 256 contiguous bytes over the sixteen lanes of a quarter wave.  Its four floats are the B
// operands of four instructions, one per column residue c = 0 .. 3: instruction c computes the
// columns 4i + c, so that the lane ends up with four consecutive columns of C.  The A operand
// of step j is element j of the 16 bytes A[m0 + i][k + 4q .. k + 4q + 3]: quarter q of the wave
// supplies the reduction index k + 4q + j to both operands.  Loads go through buffer
// descriptors: rows past M, columns past N and reduction indices past K read as zeros.
// The four partial tiles are added through LDS and go to C with atomic adds (the reduction
// is always cut: this form only serves the plain accumulate call).
#pragma once

#include "sgemm_dma.hpp"

namespace lsmi {

typedef float f32x4v __attribute__((ext_vector_type(4)));

template <int RB_>
struct RowsShape {
    static constexpr int RB = RB_;          // 16-row blocks per wave
    static constexpr int BM = 16 * RB, BN = 64, NT = 256;
    static constexpr int STEP = 16;         // reduction elements per wave and step
    static constexpr int BK = 4 * STEP;     // granularity of a workgroup's slice
};

template <class T>
__global__ __launch_bounds__(T::NT) void sgemm_rows_kernel(int M, int N, int K, const float *__restrict__ A,
                                                           int64_t lda, const float *__restrict__ B, int64_t ldb,
                                                           float *__restrict__ C, int64_t ldc, int tiles_n,
                                                           int k_per_split)
{
    __shared__ float partial[3][T::RB * 16][64];  // tiles of waves 1 .. 3: [wave][register][lane]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int q = lane >> 4, i = lane & 15;
    const int tn = (int)blockIdx.x % tiles_n, tm = (int)blockIdx.x / tiles_n;
    const int m0 = tm * T::BM, n0 = tn * T::BN;
    const int slice_begin = (int)blockIdx.y * k_per_split;
    const int slice_end = min(K, slice_begin + k_per_split);
    if (slice_begin >= slice_end) return;  // nothing to add (also K == 0): C stays untouched
    const int per_wave = k_per_split / 4;  // a multiple of STEP
    const int kb = slice_begin + wave * per_wave, ke = min(slice_end, kb + per_wave);

    const __amdgpu_buffer_rsrc_t buf_a = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(A + (int64_t)m0 * lda), 0, (int)kOutOfRange, 0x00020000);
    const __amdgpu_buffer_rsrc_t buf_b =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(B + n0), 0, (int)kOutOfRange, 0x00020000);
    uint32_t voff_a[T::RB], voff_b[4];
#pragma unroll
    for (int rb = 0; rb < T::RB; ++rb)
        voff_a[rb] = m0 + 16 * rb + i < M ? (uint32_t)(((int64_t)(16 * rb + i) * lda + 4 * q) * 4) : kOutOfRange;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        voff_b[j] = n0 + 4 * i < N ? (uint32_t)(((int64_t)(4 * q + j) * ldb + 4 * i) * 4) : kOutOfRange;

    f32x4v acc[T::RB][4];
#pragma unroll
    for (int rb = 0; rb < T::RB; ++rb)
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[rb][c][v] = 0.f;

    struct Operands {
        f32x4v a[T::RB], b[4];
    };
    // the operands of the step that starts at k; past the wave's share, or for a lane whose
    // four reduction indices lie past K (K is a multiple of 4), zeros
    auto request = [&](int k, Operands &x) {
        const bool live = k < ke && k + 4 * q < K;
        const int k_safe = k < ke ? k : kb;  // keeps the scalar offset inside the buffers
#pragma unroll
        for (int rb = 0; rb < T::RB; ++rb)
            x.a[rb] = __builtin_bit_cast(f32x4v, __builtin_amdgcn_raw_buffer_load_b128(
                                                     buf_a, (int)(live ? voff_a[rb] : kOutOfRange), k_safe * 4, 0));
#pragma unroll
        for (int j = 0; j < 4; ++j)
            x.b[j] = __builtin_bit_cast(f32x4v, __builtin_amdgcn_raw_buffer_load_b128(
                                                    buf_b, (int)(live ? voff_b[j] : kOutOfRange),
                                                    (int)((int64_t)k_safe * ldb * 4), 0));
    };
    auto multiply = [&](const Operands &x) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int rb = 0; rb < T::RB; ++rb)
                    acc[rb][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(x.a[rb][j], x.b[j][c], acc[rb][c], 0, 0, 0);
    };

    // two sets of operand registers: the loads of the next step are in flight while this one
    // is multiplied
    Operands x0, x1;
    request(kb, x0);
    for (int k = kb; k < ke; k += 2 * T::STEP) {
        request(k + T::STEP, x1);
        multiply(x0);
        request(k + 2 * T::STEP, x0);
        multiply(x1);
    }

    // ---- the four partial tiles added in a fixed order, then one atomic add per element ----
    if (wave > 0) {
#pragma unroll
        for (int rb = 0; rb < T::RB; ++rb)
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int v = 0; v < 4; ++v) partial[wave - 1][rb * 16 + c * 4 + v][lane] = acc[rb][c][v];
    }
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int rb = 0; rb < T::RB; ++rb)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            // register v of a 16 x 16 block: row 4 * (lane / 16) + v, column lane % 16
            const int row = m0 + 16 * rb + 4 * q + v;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int col = n0 + 4 * i + c;
                const int r = rb * 16 + c * 4 + v;
                const float sum = ((acc[rb][c][v] + partial[0][r][lane]) + partial[1][r][lane]) + partial[2][r][lane];
                if (row < M && col < N) atomicAdd(C + (int64_t)row * ldc + col, sum);
            }
        }
}

}  // namespace lsmi
