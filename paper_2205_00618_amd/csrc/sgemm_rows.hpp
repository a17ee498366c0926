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
//
// BT: the second operand is given transposed (N x K, k-contiguous: the weight matrix of a fully
// connected layer stored output-major).  A step is then 32 reduction elements, one 128-byte
// line of each of B's rows: lane (q, i) loads, for column block cb = 0 .. 3 and half t = 0, 1,
// the 16 bytes Bt[n0 + 16 cb + i][k + 16 t + 4 q .. + 3], whose element j is the B operand of
// instruction (cb, t, j), to which quarter q brings the reduction index k + 16 t + 4 q + j; the A
// operand is element j of A[m0 + i][k + 16 t + 4 q .. + 3].  The lane ends up with the columns
// 16 cb + i of C.  (Measured against the form in which each wave owns one column block over
// the whole slice, 512 contiguous bytes per row and step and no meeting in LDS: 8 x 4096 x 4096
// 16.8 against 19.8 us, 16 x 4096 x 4096 20.0 / 25.9, 8 x 8192 x 8192 60.8 / 56.6.)
//
// A few COLUMNS of C against a large A (a matrix-vector product, N up to 16) are the same
// problem transposed, C^T = B^T A^T: the BT form with the operands exchanged, A (M x K,
// k-contiguous) in the place of Bt.  Two more switches make the kernel serve it in place: AT,
// the small operand is stored with the reduction index along its columns (B as given, K x N):
// a lane then loads its four reduction indices as four single elements; OUT_T, the result
// goes to C transposed (the kernel's row is C's column).
#pragma once

#include "sgemm_dma.hpp"

namespace lsmi {

typedef float f32x4v __attribute__((ext_vector_type(4)));

template <int RB_, bool BT_ = false, bool AT_ = false, bool OUT_T_ = false>
struct RowsShape {
    static constexpr int RB = RB_;          // 16-row blocks per wave
    static constexpr bool BT = BT_, AT = AT_, OUT_T = OUT_T_;
    static constexpr int BM = 16 * RB, BN = 64, NT = 256;
    static constexpr int STEP = BT ? 32 : 16;   // reduction elements per wave and step
    static constexpr int GROUPS = STEP / 16;    // 16-byte groups of A per lane, row block and step
    static constexpr int BK = 64;               // granularity of a workgroup's slice
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
    const int per_wave = k_per_split / 4;  // a multiple of 16
    const int kb = slice_begin + wave * per_wave, ke = min(slice_end, kb + per_wave);

    const __amdgpu_buffer_rsrc_t buf_a = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(T::AT ? A + m0 : A + (int64_t)m0 * lda), 0, (int)kOutOfRange, 0x00020000);
    const __amdgpu_buffer_rsrc_t buf_b = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(T::BT ? B + (int64_t)n0 * ldb : B + n0), 0, (int)kOutOfRange, 0x00020000);
    uint32_t voff_a[T::RB], voff_b[4];
#pragma unroll
    for (int rb = 0; rb < T::RB; ++rb)
        voff_a[rb] = m0 + 16 * rb + i >= M ? kOutOfRange
                     : T::AT       ? (uint32_t)(((int64_t)(4 * q) * lda + 16 * rb + i) * 4)
                                   : (uint32_t)(((int64_t)(16 * rb + i) * lda + 4 * q) * 4);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if constexpr (T::BT)  // j: the column block; row n0 + 16 j + i of Bt
            voff_b[j] = n0 + 16 * j + i < N ? (uint32_t)(((int64_t)(16 * j + i) * ldb + 4 * q) * 4) : kOutOfRange;
        else
            voff_b[j] = n0 + 4 * i < N ? (uint32_t)(((int64_t)(4 * q + j) * ldb + 4 * i) * 4) : kOutOfRange;
    }

    f32x4v acc[T::RB][4];
#pragma unroll
    for (int rb = 0; rb < T::RB; ++rb)
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[rb][c][v] = 0.f;

    struct Operands {
        f32x4v a[T::RB][T::GROUPS], b[4][T::GROUPS];
    };
    // the operands of the step that starts at k; past the wave's share, or for a lane whose
    // four reduction indices lie past K (K is a multiple of 4), zeros
    auto request = [&](int k, Operands &x) {
        const int k_safe = k < ke ? k : kb;  // keeps the scalar offset inside the buffers
#pragma unroll
        for (int t = 0; t < T::GROUPS; ++t) {
            const bool live = k + 16 * t < ke && k + 16 * t + 4 * q < K;
#pragma unroll
            for (int rb = 0; rb < T::RB; ++rb) {
                if constexpr (T::AT) {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        x.a[rb][t][j] = __builtin_bit_cast(
                            float, __builtin_amdgcn_raw_buffer_load_b32(
                                       buf_a, (int)(live && voff_a[rb] != kOutOfRange ? voff_a[rb] + (uint32_t)(j * lda * 4) : kOutOfRange),
                                       (int)((int64_t)(k_safe + 16 * t) * lda * 4), 0));
                } else {
                    x.a[rb][t] = __builtin_bit_cast(
                        f32x4v, __builtin_amdgcn_raw_buffer_load_b128(buf_a, (int)(live ? voff_a[rb] : kOutOfRange),
                                                                      (k_safe + 16 * t) * 4, 0));
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
                x.b[j][t] = __builtin_bit_cast(
                    f32x4v, __builtin_amdgcn_raw_buffer_load_b128(
                                buf_b, (int)(live ? voff_b[j] : kOutOfRange),
                                T::BT ? (k_safe + 16 * t) * 4 : (int)((int64_t)k_safe * ldb * 4), 0));
        }
    };
    auto multiply = [&](const Operands &x) {
        if constexpr (T::BT) {
#pragma unroll
            for (int t = 0; t < T::GROUPS; ++t)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                        for (int rb = 0; rb < T::RB; ++rb)
                            acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(x.a[rb][t][j], x.b[cb][t][j],
                                                                               acc[rb][cb], 0, 0, 0);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int c = 0; c < 4; ++c)
#pragma unroll
                    for (int rb = 0; rb < T::RB; ++rb)
                        acc[rb][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(x.a[rb][0][j], x.b[j][0][c], acc[rb][c], 0, 0, 0);
        }
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
                const int col = T::BT ? n0 + 16 * c + i : n0 + 4 * i + c;
                const int r = rb * 16 + c * 4 + v;
                const float sum = ((acc[rb][c][v] + partial[0][r][lane]) + partial[1][r][lane]) + partial[2][r][lane];
                if (row < M && col < N)
                    atomicAdd(T::OUT_T ? C + (int64_t)col * ldc + row : C + (int64_t)row * ldc + col, sum);
            }
        }
}

}  // namespace lsmi
