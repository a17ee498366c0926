// The sgemm kernel variants and their table, one table per combination of operand layouts
// (plain or transposed A, plain or transposed B).  Each combination is compiled in a
// translation unit of its own (sgemm_gfx950.hip and sgemm_nt/tn/tt_gfx950.hip) so that the
// builds run side by side; the launcher picks the table by the call's flags.
//
// sgemm_kernel is the register-staged kernel for any shape and alignment: one workgroup owns
// one BM x BN tile of C (and, under split-K, one slice of the reduction).  Per BK chunk:
// global -> registers -> LDS staging of the A and B tiles, double-buffered so the loads of
// chunk t+1 are in flight while chunk t feeds the matrix cores; the wave's accumulators stay
// in registers until the epilogue adds them to C.  Tiles that touch the matrix edge, a K
// remainder, or rows that are not 16-byte aligned take element-wise predicated loads/stores
// inside the same kernel (tail handling as in the Section 6.2 walk-through); everything else
// moves 16 bytes per lane.
#pragma once

#include "common.hpp"
#include "sgemm_dma.hpp"
#include "sgemm_rows.hpp"
#include "tile_f32.hpp"

namespace lsmi {

template <class T, bool AT, bool BT>
__global__ __launch_bounds__(T::NT) void sgemm_kernel(int M, int N, int K,
                                                      const float *__restrict__ A, int64_t lda,
                                                      const float *__restrict__ B, int64_t ldb,
                                                      float *__restrict__ C, int64_t ldc, TileMap tmap,
                                                      int k_per_split, int split_k, Epilogue ep)
{
    __shared__ __attribute__((aligned(16))) float lds[T::LDS_FLOATS];
    float *const a_lds = lds;
    float *const b_lds = lds + 2 * T::A_STAGE;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, half = lane >> 5;
    const int wrow = (wave / T::WAVES_N) * T::WTM;
    const int wcol = (wave % T::WAVES_N) * T::WTN;

    int tm, tn;
    tmap.locate(blockIdx.x, tm, tn);
    const int m0 = tm * T::BM, n0 = tn * T::BN;
    const int kbeg = blockIdx.y * k_per_split;
    const int kend = (kbeg + k_per_split < K) ? kbeg + k_per_split : K;
    if (kbeg >= kend && split_k > 1) return;  // uniform for the workgroup, before any barrier

    // a transposed operand (AT: A is stored K x M, BT: B is stored N x K) is fetched element
    // by element through its swapped index map; the 16-byte loads serve the plain layouts
    const bool a_vec = !AT && (((uintptr_t)A | (uintptr_t)(lda * 4)) & 15) == 0 && m0 + T::BM <= M;
    const bool b_vec = !BT && (((uintptr_t)B | (uintptr_t)(ldb * 4)) & 15) == 0 && n0 + T::BN <= N;
    const int64_t a_sm = AT ? 1 : lda, a_sk = AT ? lda : 1;  // strides of (row, k) in A
    const int64_t b_sk = BT ? 1 : ldb, b_sn = BT ? ldb : 1;  // strides of (k, column) in B

    f32x4 ra[T::A_SLOTS], rb[T::B_SLOTS];

    auto gload = [&](int k0) {
        const bool kfull = k0 + T::BK <= kend;
        if (a_vec && kfull) {
#pragma unroll
            for (int v = 0; v < T::A_SLOTS; ++v) {
                const int slot = tid + v * T::NT;
                const int row = slot / (T::BK / 4), kq = slot % (T::BK / 4);
                ra[v] = *reinterpret_cast<const f32x4 *>(A + (int64_t)(m0 + row) * lda + k0 + kq * 4);
            }
        } else {
#pragma unroll
            for (int v = 0; v < T::A_SLOTS; ++v) {
                const int slot = tid + v * T::NT;
                const int row = slot / (T::BK / 4), kq = slot % (T::BK / 4);
                const float *src = A + (int64_t)(m0 + row) * a_sm + (int64_t)(k0 + kq * 4) * a_sk;
                const bool row_ok = m0 + row < M;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    ra[v][e] = (row_ok && k0 + kq * 4 + e < kend) ? src[e * a_sk] : 0.f;
            }
        }
        if (b_vec && kfull) {
#pragma unroll
            for (int v = 0; v < T::B_SLOTS; ++v) {
                const int slot = tid + v * T::NT;
                const int row = slot / (T::BN / 4), nq = slot % (T::BN / 4);
                rb[v] = *reinterpret_cast<const f32x4 *>(B + (int64_t)(k0 + row) * ldb + n0 + nq * 4);
            }
        } else {
#pragma unroll
            for (int v = 0; v < T::B_SLOTS; ++v) {
                const int slot = tid + v * T::NT;
                const int row = slot / (T::BN / 4), nq = slot % (T::BN / 4);
                const float *src = B + (int64_t)(k0 + row) * b_sk + (int64_t)(n0 + nq * 4) * b_sn;
                const bool row_ok = k0 + row < kend;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    rb[v][e] = (row_ok && n0 + nq * 4 + e < N) ? src[e * b_sn] : 0.f;
            }
        }
    };

    auto sstore = [&](int buf) {
        float *as = a_lds + buf * T::A_STAGE;
        float *bs = b_lds + buf * T::B_STAGE;
#pragma unroll
        for (int v = 0; v < T::A_SLOTS; ++v) {
            const int slot = tid + v * T::NT;
            const int row = slot / (T::BK / 4), kq = slot % (T::BK / 4);
            *reinterpret_cast<f32x4 *>(as + row * T::A_LD + kq * 4) = ra[v];
        }
#pragma unroll
        for (int v = 0; v < T::B_SLOTS; ++v) {
            const int slot = tid + v * T::NT;
            const int row = slot / (T::BN / 4), nq = slot % (T::BN / 4);
            *reinterpret_cast<f32x4 *>(bs + row * T::B_LD + nq * 4) = rb[v];
        }
    };

    WaveTile<T> wt;
    wt.clear();

    gload(kbeg);
    sstore(0);
    __syncthreads();
    int buf = 0;
    for (int k0 = kbeg; k0 < kend; k0 += T::BK) {
        const bool has_next = k0 + T::BK < kend;
        if (has_next) gload(k0 + T::BK);
        wt.consume_chunk(a_lds + buf * T::A_STAGE, b_lds + buf * T::B_STAGE, wrow, wcol, li, half);
        if (has_next) sstore(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }

    // Epilogue: C += acc.  Lane (li, half) holds, for block row a and register v, the TN
    // adjacent columns n0 + wcol + TN*li + {0..TN-1} of one row.
    typedef typename FVec<T::TN>::type CVec;
    const int col = n0 + wcol + T::TN * li;
    const bool c_vec = (((uintptr_t)C | (uintptr_t)(ldc * 4)) & (4 * T::TN - 1)) == 0 &&
                       m0 + T::BM <= M && n0 + T::BN <= N;
    // Old values of C are requested a block row at a time, ahead of the stores: a load behind
    // a store to C would wait for that store (the two may overlap as far as the compiler can
    // tell), one memory round trip per register.
    auto c_at = [&](int a, int v) {
        return C + (int64_t)(m0 + wrow + WaveTile<T>::acc_row(a, v, half)) * ldc + col;
    };
    if (split_k > 1) {
        // partial sums of several workgroups: only the plain accumulate form gets here
#pragma unroll
        for (int a = 0; a < T::TM; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wrow + WaveTile<T>::acc_row(a, v, half);
#pragma unroll
                for (int b = 0; b < T::TN; ++b)
                    if (row < M && col + b < N) atomicAdd(c_at(a, v) + b, wt.acc[a][b][v]);
            }
    } else if (c_vec) {
        CVec init;
        if constexpr (T::TN == 1) {
            init = ep.pre == kPreBias ? ep.bias[col] : 0.f;
        } else {
#pragma unroll
            for (int b = 0; b < T::TN; ++b) init[b] = ep.pre == kPreBias ? ep.bias[col + b] : 0.f;
        }
#pragma unroll
        for (int a = 0; a < T::TM; ++a) {
            CVec c[16];
#pragma unroll
            for (int v = 0; v < 16; ++v)
                c[v] = ep.pre == kPreAccumulate ? *reinterpret_cast<const CVec *>(c_at(a, v)) : init;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                if constexpr (T::TN == 1) {
                    c[v] = apply_post(c[v] + wt.acc[a][0][v], ep.post);
                } else {
#pragma unroll
                    for (int b = 0; b < T::TN; ++b) c[v][b] = apply_post(c[v][b] + wt.acc[a][b][v], ep.post);
                }
                *reinterpret_cast<CVec *>(c_at(a, v)) = c[v];
            }
        }
    } else {
#pragma unroll
        for (int a = 0; a < T::TM; ++a) {
            float c[16][T::TN];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const bool row_ok = m0 + wrow + WaveTile<T>::acc_row(a, v, half) < M;
#pragma unroll
                for (int b = 0; b < T::TN; ++b) {
                    c[v][b] = 0.f;
                    if (row_ok && col + b < N)
                        c[v][b] = ep.pre == kPreAccumulate ? c_at(a, v)[b]
                                  : ep.pre == kPreBias     ? ep.bias[col + b]
                                                           : 0.f;
                }
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const bool row_ok = m0 + wrow + WaveTile<T>::acc_row(a, v, half) < M;
#pragma unroll
                for (int b = 0; b < T::TN; ++b)
                    if (row_ok && col + b < N) c_at(a, v)[b] = apply_post(c[v][b] + wt.acc[a][b][v], ep.post);
            }
        }
    }
}

struct Variant {
    const char *name;
    const char *tail_name;  // reported when the last round's tiles run as slices
    int bm, bn, bk;
    bool dma;   // direct global->LDS loads: needs 16-byte aligned A, B and lda, ldb multiples of 4
    bool edge;  // dma kernel that also takes ragged M, N, K and split-K
    void (*launch)(dim3 grid, hipStream_t s, int M, int N, int K, const float *A, int64_t lda,
                   const float *B, int64_t ldb, float *C, int64_t ldc, int tiles_m, int tiles_n,
                   int group_m, int k_per_split, int split_k, int tail_first, int tail_split, Epilogue ep,
                   Meeting meet);
    bool dword = false;  // edge kernel with 4-byte loads: no alignment condition on A, B, lda, ldb, K
    bool rows = false;   // few-row kernel (sgemm_rows.hpp): operands straight into registers, always atomic adds
    int ksets = 1;       // chunks per step of the direct-to-LDS kernels (wave sets)
    bool cols = false;   // the few-row kernel on the transposed problem: a few columns of C against a large A
    int per_cu = 4;      // workgroups of a 128-row tile resident per CU (two for the eight-wave forms)
};

template <class T, bool AT, bool BT>
void launch_variant(dim3 grid, hipStream_t s, int M, int N, int K, const float *A, int64_t lda,
                    const float *B, int64_t ldb, float *C, int64_t ldc, int tiles_m, int tiles_n,
                    int group_m, int k_per_split, int split_k, int, int, Epilogue ep, Meeting)
{
    hipLaunchKernelGGL((sgemm_kernel<T, AT, BT>), grid, dim3(T::NT), 0, s, M, N, K, A, lda, B, ldb, C, ldc,
                       TileMap(tiles_m, tiles_n, group_m), k_per_split, split_k, ep);
}

template <class T>
void launch_dma_variant(dim3 grid, hipStream_t s, int M, int N, int K, const float *A, int64_t lda,
                        const float *B, int64_t ldb, float *C, int64_t ldc, int tiles_m,
                        int tiles_n, int group_m, int k_per_split, int split_k, int tail_first, int tail_split,
                        Epilogue ep, Meeting meet)
{
    // a uniform split of the buffer-load kernels runs as one dimension of tiles x slices workgroups
    const bool cut = T::EDGE && split_k > 1 && tail_split <= 1;
    if (cut) grid = dim3(grid.x * grid.y, 1u);
    hipLaunchKernelGGL(sgemm_dma_kernel<T>, grid, dim3(T::NT), 0, s, M, N, K, A, lda, B, ldb, C, ldc,
                       TileMap(tiles_m, tiles_n, group_m, cut ? split_k : 1), k_per_split, split_k, tail_first,
                       tail_split, ep, meet);
}

template <class T>
void launch_rows_variant(dim3 grid, hipStream_t s, int M, int N, int K, const float *A, int64_t lda,
                         const float *B, int64_t ldb, float *C, int64_t ldc, int, int tiles_n, int,
                         int k_per_split, int, int, int, Epilogue, Meeting)
{
    hipLaunchKernelGGL(sgemm_rows_kernel<T>, grid, dim3(T::NT), 0, s, M, N, K, A, lda, B, ldb, C, ldc, tiles_n,
                       k_per_split);
}

// the few-row kernels exist for A as given (rows of C are rows of A), B in either layout
template <bool AT, bool BT, int RB>
constexpr auto rows_launcher()
{
    if constexpr (AT) return static_cast<decltype(&launch_rows_variant<RowsShape<RB>>)>(nullptr);
    else return &launch_rows_variant<RowsShape<RB, BT>>;
}

// A few columns of C (N up to 16) against a large A as given: C^T = B^T A^T on the few-row kernel,
// A in the place of the streamed operand, B (stored K x N, or N x K when transposed) in the
// place of the few rows, the result stored transposed.
template <class T>
void launch_cols_variant(dim3 grid, hipStream_t s, int M, int N, int K, const float *A, int64_t lda,
                         const float *B, int64_t ldb, float *C, int64_t ldc, int tiles_m, int, int,
                         int k_per_split, int, int, int, Epilogue, Meeting)
{
    hipLaunchKernelGGL(sgemm_rows_kernel<T>, grid, dim3(T::NT), 0, s, N, M, K, B, ldb, A, lda, C, ldc, tiles_m,
                       k_per_split);
}

template <bool AT, bool BT>
constexpr auto cols_launcher()
{
    if constexpr (AT) return static_cast<decltype(&launch_cols_variant<RowsShape<1, true, true, true>>)>(nullptr);
    else return &launch_cols_variant<RowsShape<1, true, !BT, true>>;
}

// Indices of the variants the built-in choice names.
constexpr int kDefaultDma = 2, kLoneDma = 3, kOneRoundDma = 4, kWideDma = 5, kEdgeBigFour = 6, kEdgeBig = 18, kEdgeSingle = 7, kEdgePair = 8, kEdgeDword = 10, kEdgeBigDword = 11;
constexpr int kRows16 = 12, kCols16 = 13, kEdgeQuad = 15, kEdgeQuadDword = 17;  // 64 x 64 tiles shared by four wave sets
constexpr int kNumSgemmVariants = 20;

// Workgroups per CU the register allocation of a buffer-load kernel allows: four, except for
// 128 x 128 tiles with 4-byte loads of a transposed B, whose per-lane load offsets and reduction
// indices for both operands need the registers of three.
constexpr int edge_wgs(int bm, bool dword, bool bt) { return bm == 128 && dword && bt ? 3 : 4; }

// The table for one combination of layouts; SUFFIX ("" or "_nt", "_tn", "_tt") ends the names.
#define LSMI_REG(BM, BN, BK, WM, WN, AT, BT, SUFFIX)                                                       \
    {"sgemm_" #BM "x" #BN "x" #BK "_w" #WM "x" #WN SUFFIX, "", BM, BN, BK, false, false,                    \
     &launch_variant<TileShape<BM, BN, BK, WM, WN, true>, AT, BT>}
#define LSMI_DMA(BM, BN, WM, WN, NS, PC, MAXWG, AT, BT, SUFFIX)                                            \
    {"sgemm_dma_" #BM "x" #BN "x16_w" #WM "x" #WN "_s" #NS "_c" #PC SUFFIX, "", BM, BN, 16, true, false,    \
     &launch_dma_variant<DmaShape<BM, BN, WM, WN, NS, (PC != 0), false, MAXWG, 1, false, AT, BT>>}
#define LSMI_EDGE(TAG, BM, BN, BKSTEP, WM, WN, KS, KTAG, NS, DW, AT, BT, SUFFIX)                            \
    {"sgemm_dma_" TAG "_" #BM "x" #BN "x" #BKSTEP "_w" #WM "x" #WN KTAG "_s" #NS SUFFIX,                    \
     "sgemm_dma_" TAG "_" #BM "x" #BN "x" #BKSTEP "_w" #WM "x" #WN KTAG "_s" #NS "_tail" SUFFIX, BM, BN,    \
     BKSTEP, true, true, &launch_dma_variant<DmaShape<BM, BN, WM, WN, NS, false, true, edge_wgs(BM, DW, BT), KS, DW, AT, BT>>, \
     DW, false, KS}
#define LSMI_EDGE8(TAG, DW, AT, BT, SUFFIX)                                                                 \
    {"sgemm_dma_" TAG "_128x128x16_w4x2_s2" SUFFIX, "sgemm_dma_" TAG "_128x128x16_w4x2_s2_tail" SUFFIX, 128, 128, \
     16, true, true, &launch_dma_variant<DmaShape<128, 128, 4, 2, 2, false, true, 2, 1, DW, AT, BT>>, DW, false, 1, false, 2}
#define LSMI_DEFINE_SGEMM_TABLE(ACCESSOR, AT, BT, SUFFIX)                                                  \
    namespace {                                                                                            \
    const Variant kTable##ACCESSOR[kNumSgemmVariants] = {                                                  \
        LSMI_REG(128, 128, 16, 2, 2, AT, BT, SUFFIX),           /* 0: any shape and alignment, many tiles */ \
        LSMI_REG(64, 64, 16, 2, 2, AT, BT, SUFFIX),             /* 1: any shape, few tiles (with split-K) */ \
        LSMI_DMA(128, 128, 2, 2, 2, 0, 4, AT, BT, SUFFIX),  /* 2: aligned shapes; four workgroups per CU */ \
        LSMI_DMA(128, 128, 4, 2, 2, 0, 2, AT, BT, SUFFIX),  /* 3: eight waves of 32 x 64: a tile that has its CU to itself */ \
        LSMI_DMA(128, 128, 2, 2, 2, 1, 2, AT, BT, SUFFIX),   /* 4: C requested at the start, two per CU */ \
        LSMI_DMA(256, 128, 4, 2, 2, 0, 2, AT, BT, SUFFIX),  /* 5: eight waves of 64 x 64, two per CU */  \
        LSMI_EDGE("edge", 128, 128, 16, 2, 2, 1, "", 2, false, AT, BT, SUFFIX),   /* 6: ragged, aligned rows */ \
        LSMI_EDGE("edge", 64, 64, 16, 2, 1, 1, "", 3, false, AT, BT, SUFFIX),     /* 7: the same, few tiles */  \
        LSMI_EDGE("edge", 64, 64, 32, 2, 1, 2, "_k2", 3, false, AT, BT, SUFFIX),  /* 8: two wave sets */        \
        LSMI_EDGE("edge", 64, 64, 32, 2, 1, 2, "_k2", 4, false, AT, BT, SUFFIX),  /* 9 */                       \
        LSMI_EDGE("edge4", 64, 64, 32, 2, 1, 2, "_k2", 3, true, AT, BT, SUFFIX),  /* 10: 8 with 4-byte loads */ \
        LSMI_EDGE("edge4", 128, 128, 16, 2, 2, 1, "", 2, true, AT, BT, SUFFIX),   /* 11: 6 with 4-byte loads */ \
        {"sgemm_rows_16x64x64_w4" SUFFIX, "", 16, 64, 64, true, true, rows_launcher<AT, BT, 1>(), false, true}, /* 12 */ \
        {"sgemm_cols_64x16x64_w4" SUFFIX, "", 64, 16, 64, true, true, cols_launcher<AT, BT>(), false, true, 1, true}, /* 13 */ \
        LSMI_EDGE("edge", 64, 64, 64, 2, 1, 4, "_k4", 3, false, AT, BT, SUFFIX),  /* 14: four wave sets */      \
        LSMI_EDGE("edge", 64, 64, 64, 2, 1, 4, "_k4", 2, false, AT, BT, SUFFIX),  /* 15: two per CU */          \
        LSMI_EDGE("edge4", 64, 64, 64, 2, 1, 4, "_k4", 3, true, AT, BT, SUFFIX),  /* 16: 14 with 4-byte loads */ \
        LSMI_EDGE("edge4", 64, 64, 64, 2, 1, 4, "_k4", 2, true, AT, BT, SUFFIX),  /* 17 */                      \
        LSMI_EDGE8("edge", false, AT, BT, SUFFIX),   /* 18: 6 on eight waves of 32 x 64, two workgroups per CU */ \
        LSMI_EDGE8("edge4", true, AT, BT, SUFFIX),   /* 19: 11 likewise */                                       \
    };                                                                                                     \
    }                                                                                                      \
    const Variant *ACCESSOR() { return kTable##ACCESSOR; }

// the tables, one per translation unit: plain layouts, B transposed, A transposed, both
const Variant *sgemm_table_nn();
const Variant *sgemm_table_nt();
const Variant *sgemm_table_tn();
const Variant *sgemm_table_tt();

}  // namespace lsmi
