// fp32 GEMM, C += A.B (Section 2.1, Fig. 1 with alpha = beta = 1), for gfx950.
//
// One workgroup owns one BM x BN tile of C (and, under split-K, one slice of the
// reduction).  Per BK chunk: global -> registers -> LDS staging of the A and B tiles,
// double-buffered so the loads of chunk t+1 are in flight while chunk t feeds the matrix
// cores; the wave's accumulators stay in registers until the epilogue adds them to C.
// Tiles that touch the matrix edge, a K remainder, or rows that are not 16-byte aligned
// take element-wise predicated loads/stores inside the same kernel (tail handling as in
// the Section 6.2 walk-through); everything else moves 16 bytes per lane.
#include "common.hpp"
#include "sgemm_dma.hpp"
#include "sgemm_rows.hpp"
#include "tile_f32.hpp"

namespace lsmi {
namespace {

template <class T>
__global__ __launch_bounds__(T::NT) void sgemm_kernel(int M, int N, int K,
                                                      const float *__restrict__ A, int64_t lda,
                                                      const float *__restrict__ B, int64_t ldb,
                                                      float *__restrict__ C, int64_t ldc,
                                                      int tiles_m, int tiles_n, int group_m,
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
    map_tile(blockIdx.x, tiles_m, tiles_n, group_m, tm, tn);
    const int m0 = tm * T::BM, n0 = tn * T::BN;
    const int kbeg = blockIdx.y * k_per_split;
    const int kend = (kbeg + k_per_split < K) ? kbeg + k_per_split : K;
    if (kbeg >= kend && split_k > 1) return;  // uniform for the workgroup, before any barrier

    const bool a_vec = (((uintptr_t)A | (uintptr_t)(lda * 4)) & 15) == 0 && m0 + T::BM <= M;
    const bool b_vec = (((uintptr_t)B | (uintptr_t)(ldb * 4)) & 15) == 0 && n0 + T::BN <= N;

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
                const float *src = A + (int64_t)(m0 + row) * lda + k0 + kq * 4;
                const bool row_ok = m0 + row < M;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    ra[v][e] = (row_ok && k0 + kq * 4 + e < kend) ? src[e] : 0.f;
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
                const float *src = B + (int64_t)(k0 + row) * ldb + n0 + nq * 4;
                const bool row_ok = k0 + row < kend;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    rb[v][e] = (row_ok && n0 + nq * 4 + e < N) ? src[e] : 0.f;
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
    bool edge;  // dma kernel that also takes ragged M, N, K % 4 == 0 and split-K
    void (*launch)(dim3 grid, hipStream_t s, int M, int N, int K, const float *A, int64_t lda,
                   const float *B, int64_t ldb, float *C, int64_t ldc, int tiles_m, int tiles_n,
                   int group_m, int k_per_split, int split_k, int tail_first, int tail_split, Epilogue ep);
    bool dword = false;  // edge kernel with 4-byte loads: no alignment condition on A, B, lda, ldb, K
    bool rows = false;   // few-row kernel (sgemm_rows.hpp): operands straight into registers, always atomic adds
};

template <class T>
void launch_variant(dim3 grid, hipStream_t s, int M, int N, int K, const float *A, int64_t lda,
                    const float *B, int64_t ldb, float *C, int64_t ldc, int tiles_m, int tiles_n,
                    int group_m, int k_per_split, int split_k, int, int, Epilogue ep)
{
    hipLaunchKernelGGL(sgemm_kernel<T>, grid, dim3(T::NT), 0, s, M, N, K, A, lda, B, ldb, C, ldc,
                       tiles_m, tiles_n, group_m, k_per_split, split_k, ep);
}

template <class T>
void launch_dma_variant(dim3 grid, hipStream_t s, int M, int N, int K, const float *A, int64_t lda,
                        const float *B, int64_t ldb, float *C, int64_t ldc, int tiles_m,
                        int tiles_n, int group_m, int k_per_split, int split_k, int tail_first, int tail_split,
                        Epilogue ep)
{
    hipLaunchKernelGGL(sgemm_dma_kernel<T>, grid, dim3(T::NT), 0, s, M, N, K, A, lda, B, ldb, C, ldc,
                       tiles_m, tiles_n, group_m, k_per_split, split_k, tail_first, tail_split, ep);
}

template <class T>
void launch_rows_variant(dim3 grid, hipStream_t s, int M, int N, int K, const float *A, int64_t lda,
                         const float *B, int64_t ldb, float *C, int64_t ldc, int, int tiles_n, int,
                         int k_per_split, int, int, int, Epilogue)
{
    hipLaunchKernelGGL(sgemm_rows_kernel<T>, grid, dim3(T::NT), 0, s, M, N, K, A, lda, B, ldb, C, ldc, tiles_n,
                       k_per_split);
}

#define LSMI_VARIANT(BM, BN, BK, WM, WN)                                                     \
    {"sgemm_" #BM "x" #BN "x" #BK "_w" #WM "x" #WN, "", BM, BN, BK, false, false,             \
     &launch_variant<TileShape<BM, BN, BK, WM, WN, true>>}
#define LSMI_DMA_VARIANT(BM, BN, WM, WN, NS, PC)                                             \
    {"sgemm_dma_" #BM "x" #BN "x16_w" #WM "x" #WN "_s" #NS "_c" #PC, "", BM, BN, 16, true, false,  \
     &launch_dma_variant<DmaShape<BM, BN, WM, WN, NS, PC>>}
#define LSMI_DMA_EDGE_VARIANT(BM, BN, WM, WN, NS)                                            \
    {"sgemm_dma_edge_" #BM "x" #BN "x16_w" #WM "x" #WN "_s" #NS,                               \
     "sgemm_dma_edge_" #BM "x" #BN "x16_w" #WM "x" #WN "_s" #NS "_tail", BM, BN, 16, true, true, \
     &launch_dma_variant<DmaShape<BM, BN, WM, WN, NS, false, true>>}

const Variant kVariants[] = {
    LSMI_VARIANT(128, 128, 16, 2, 2),        // 0: any shape and alignment, many tiles
    LSMI_VARIANT(64, 64, 16, 2, 2),          // 1: any shape, few tiles (combined with split-K)
    LSMI_DMA_VARIANT(128, 128, 2, 2, 2, 0),  // 2: aligned shapes; four workgroups per CU
    LSMI_DMA_VARIANT(128, 128, 2, 2, 3, 0),  // 3: deeper load pipeline, three workgroups per CU
    {"sgemm_dma_128x128x16_w2x2_s2_c1", "", 128, 128, 16, true, false,  // 4: C requested at the start, two
     &launch_dma_variant<DmaShape<128, 128, 2, 2, 2, true, false, 2>>},  // workgroups per CU: outputs of one tile per CU
    LSMI_DMA_VARIANT(256, 128, 2, 2, 3, 0),  // 5: 128 x 64 wave tiles, two workgroups per CU
    LSMI_DMA_EDGE_VARIANT(128, 128, 2, 2, 2),  // 6: ragged M, N, K with aligned rows, many tiles
    LSMI_DMA_EDGE_VARIANT(64, 64, 2, 1, 3),    // 7: the same, few tiles (combined with split-K)
    {"sgemm_dma_edge_64x64x32_w2x1_k2_s3", "sgemm_dma_edge_64x64x32_w2x1_k2_s3_tail", 64, 64, 32, true, true,  // 8: two chunks per step, one per pair
     &launch_dma_variant<DmaShape<64, 64, 2, 1, 3, false, true, 4, true>>},  // of waves: all four SIMDs on a 64 x 64 tile
    {"sgemm_dma_edge_64x64x32_w2x1_k2_s4", "sgemm_dma_edge_64x64x32_w2x1_k2_s4_tail", 64, 64, 32, true, true,  // 9
     &launch_dma_variant<DmaShape<64, 64, 2, 1, 4, false, true, 4, true>>},
    {"sgemm_dma_edge4_64x64x32_w2x1_k2_s3", "sgemm_dma_edge4_64x64x32_w2x1_k2_s3_tail", 64, 64, 32, true, true,  // 10: 8 with
     &launch_dma_variant<DmaShape<64, 64, 2, 1, 3, false, true, 4, true, true>>, true},  // 4-byte loads: any lda, ldb, K
    {"sgemm_dma_edge4_128x128x16_w2x2_s2", "sgemm_dma_edge4_128x128x16_w2x2_s2_tail", 128, 128, 16, true, true,  // 11: 6 with
     &launch_dma_variant<DmaShape<128, 128, 2, 2, 2, false, true, 4, false, true>>, true},  // 4-byte loads
    {"sgemm_rows_16x64x64_w4", "", 16, 64, 64, true, true, &launch_rows_variant<RowsShape<1>>, false, true},  // 12: a few rows
    {"sgemm_rows_32x64x64_w4", "", 32, 64, 64, true, true, &launch_rows_variant<RowsShape<2>>, false, true},  // 13: two row
    // blocks per wave (B read once for 32 rows; slower than two 16-row tiles, whose second read of B comes from L2)
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);
constexpr int kDefaultDma = 2, kOneRoundDma = 4, kEdgeBig = 6, kEdgePair = 8, kEdgeDword = 10, kEdgeBigDword = 11;
constexpr int kRows16 = 12;

// Shapes the direct-to-LDS kernels accept (see sgemm_dma.hpp).
bool dma_supported(const Variant &v, int M, int N, int K, const float *A, int64_t lda,
                   const float *B, int64_t ldb, const float *C, int64_t ldc, const Epilogue &ep)
{
    // (the few-row kernels combine their slices with atomic adds: plain accumulate form only)
    if (v.rows && (ep.pre != kPreAccumulate || ep.post != kPostNone || (int64_t)K * ldb * 4 >= (int64_t)INT32_MAX))
        return false;
    if (v.dword)
        return K >= 1 && (int64_t)v.bm * lda * 4 + 64 < (int64_t)INT32_MAX &&
               16 * ldb * 4 + v.bn * 4 < (int64_t)INT32_MAX;
    if (v.edge)
        return K % 4 == 0 && K >= 4 && (((uintptr_t)A | (uintptr_t)B) & 15) == 0 && lda % 4 == 0 &&
               ldb % 4 == 0 && (int64_t)v.bm * lda * 4 < (int64_t)INT32_MAX &&
               16 * ldb * 4 + v.bn * 4 < (int64_t)INT32_MAX;
    if (ep.pre == kPreBias && ((uintptr_t)ep.bias & 7) != 0) return false;
    return M % v.bm == 0 && N % v.bn == 0 && K % 16 == 0 && K >= 16 &&
           (((uintptr_t)A | (uintptr_t)B) & 15) == 0 && lda % 4 == 0 && ldb % 4 == 0 &&
           ((uintptr_t)C & 7) == 0 && ldc % 2 == 0 &&
           (int64_t)v.bm * lda * 4 < (int64_t)UINT32_MAX && 16 * ldb * 4 + v.bn * 4 < (int64_t)UINT32_MAX;
}

// Slices for the tiles of an incomplete last round (0: none).  `gain_us` is the estimated
// time saved against running those tiles whole.
struct TailPlan {
    int split = 0;
    double gain_us = 0;
};

TailPlan plan_tail(const Variant &v, int64_t nt, int chunks, int cus)
{
    TailPlan p;
    const int64_t rem = nt % cus;
    if (nt <= cus || rem == 0) return p;
    int s = (int)(cus / rem);
    const int cap = chunks / 4 < 64 ? chunks / 4 : 64;  // at least four chunks per slice
    if (s > cap) s = cap;
    if (s < 2) return p;
    const double chunk_us = 2.0 * v.bm * v.bn * v.bk / 0.47e6;
    const double atomic_us = 4.0 * v.bm * v.bn * rem * s / 0.7e6;
    const int per = (chunks + s - 1) / s;
    const double gain = chunk_us * (chunks - per) - atomic_us;
    if (gain <= 0) return p;
    p.split = s;
    p.gain_us = gain;
    return p;
}

}  // namespace

int sgemm_variant_count() { return kNumVariants; }

const char *sgemm_variant_name(int index)
{
    return (index >= 0 && index < kNumVariants) ? kVariants[index].name : nullptr;
}

void tile_of_workgroup(int wg, int tiles_m, int tiles_n, int group_m, int *tm, int *tn)
{
    map_tile(wg, tiles_m, tiles_n, group_m, *tm, *tn);
}

int launch_sgemm(int M, int N, int K, const float *A, int64_t lda, const float *B, int64_t ldb,
                 float *C, int64_t ldc, const float *bias, int pre, int post)
{
    const Epilogue ep{bias, pre, post};
    // partial sums can only be combined by atomic adds onto the old C when nothing else
    // happens to the element: any other pre/post form keeps the whole reduction in one workgroup
    const bool may_split = pre == kPreAccumulate && post == kPostNone;
    ThreadState &st = tls();
    const int cus = device_cu_count();
    auto tiles = [&](const Variant &v) {
        return (int64_t)((M + v.bm - 1) / v.bm) * ((N + v.bn - 1) / v.bn);
    };
    int vi = st.forced_variant;
    if (vi >= 0 && kVariants[vi].dma && !dma_supported(kVariants[vi], M, N, K, A, lda, B, ldb, C, ldc, ep))
        vi = -1;  // a forced aligned-only kernel cannot take this problem: use the built-in choice
    if (vi < 0) {
        const Variant &d = kVariants[kDefaultDma];
        // Estimated time of a direct-to-LDS kernel on this problem: the CU with the most tiles
        // sets it, so a tile count is worth its whole rounds of the CUs plus one more round
        // for any remainder -- a tile's time, or a slice's when the remainder can be cut into
        // slices (plan_tail; buffer-load kernels in the plain accumulate form only).  Rates
        // per CU from sweeps of 20 shapes: 0.57 TFLOP/s for the full-tile 128 x 128 kernel,
        // 0.558 for its buffer-load form, 0.53 for 64 x 64 tiles shared by two pairs of waves.
        // 3072^3 (576 tiles of 128 x 128, 2.25 per CU): 532 us on whole tiles, 408 with the
        // last 64 tiles in four slices, 421 on 64 x 64 tiles (nine per CU exactly).
        auto estimate = [&](int index, double rate, bool tail_ok) {
            const Variant &c = kVariants[index];
            const int64_t t = tiles(c);
            const int chunks = (K + c.bk - 1) / c.bk;
            // a 128 x 128 workgroup alone on its CU runs below the rate it has in company
            // (2000^3, 256 tiles: 159 us on the buffer-load form, 131 at 2048^3 on the
            // full-tile form with C requested up front)
            if (t <= cus && c.bm >= 128) rate *= c.edge ? 0.75 : 0.9;
            const double chunk_us = 2.0 * c.bm * c.bn * c.bk / rate;
            double us = chunk_us * chunks * (double)(t / cus);
            if (t % cus != 0) {
                const TailPlan tp = tail_ok ? plan_tail(c, t, chunks, cus) : TailPlan{};
                if (tp.split > 1)
                    us += chunk_us * ((chunks + tp.split - 1) / tp.split) +
                          4.0 * c.bm * c.bn * (double)(t % cus) * tp.split / 0.7e6;
                else
                    us += chunk_us * chunks;
            }
            return us;
        };
        const bool tail_ok = may_split && st.forced_split_k <= 0;
        const bool edge_ok = dma_supported(kVariants[kEdgeBig], M, N, K, A, lda, B, ldb, C, ldc, ep);
        const int rows = kRows16;
        if (M <= 32 && (int64_t)N * K >= (1 << 20) && st.forced_split_k != 1 &&
            dma_supported(kVariants[rows], M, N, K, A, lda, B, ldb, C, ldc, ep)) {
            // a few rows against a B of 4 MB or more: the kernel that streams B straight into
            // registers (a caller who keeps the reduction in one workgroup does not get it:
            // its slices always meet in atomic adds).  N = K = 4096, B from HBM: M = 1
            // 24.1 -> 14.9 us, M = 8 22.9 -> 15.8, M = 16 23.7 -> 19.0, M = 32 (two row tiles)
            // 25.3 -> 23.9; from 48 rows on the 64-row tiles are level
            vi = rows;
        } else if (st.forced_split_k <= 1 && tiles(d) >= cus && K >= 64 &&
            dma_supported(d, M, N, K, A, lda, B, ldb, C, ldc, ep)) {
            // with one workgroup per CU (2048^3: 256 tiles) nothing else hides the latency of
            // the C tile in the epilogue: request it up front (5 %); with two or more per CU
            // the plain kernel is as fast or faster
            vi = (tiles(d) < 2 * cus && ep.pre == kPreAccumulate) ? kOneRoundDma : kDefaultDma;
            double best = estimate(kDefaultDma, 0.57e6, false);
            if (edge_ok) {
                const double big = estimate(kEdgeBig, 0.558e6, tail_ok);
                if (big < best) {
                    best = big;
                    vi = kEdgeBig;
                }
                if (estimate(kEdgePair, 0.53e6, tail_ok) < best) vi = kEdgePair;
            }
        } else if (K >= 64 && (tiles(kVariants[kEdgePair]) * 4096 * K >= (1LL << 28) || 2 * tiles(kVariants[kEdgePair]) >= cus) && edge_ok) {
            // ragged shapes with aligned rows, and whole-tile shapes too small for the 128 x 128
            // tiles: the buffer-load kernels, 128 x 128 tiles or the form in which two pairs of
            // waves share a 64 x 64 tile, each taking every other chunk (1024^3: 31 -> 22 us; it
            // is level with or ahead of the plain 64 x 64 form on every shape of the sweeps),
            // by the same estimate.  Problems with fewer than 2^28 multiply-adds (counted over
            // whole tiles: a few rows against a large B cost what 64 rows do, 8 x 4096 x 4096
            // 42 -> 23 us) and 64 x 64 tiles for less than half the CUs stay with the
            // register-staged kernel, which is as quick there (with more tiles and a short
            // reduction it is not: 1024 x 1024 x 128 10.8 -> 6.1 us)
            vi = kEdgePair;
            if (st.forced_split_k <= 1 && tiles(kVariants[kEdgeBig]) >= cus &&
                estimate(kEdgeBig, 0.558e6, tail_ok) < estimate(kEdgePair, 0.53e6, tail_ok))
                vi = kEdgeBig;
        } else if (K >= 64 && ((int64_t)M * N * K >= (1LL << 28) || 2 * tiles(kVariants[kEdgeDword]) >= cus) &&
                   dma_supported(kVariants[kEdgeDword], M, N, K, A, lda, B, ldb, C, ldc, ep)) {
            // rows that start at any element (lda, ldb or K not multiples of four, or bases not
            // 16-byte aligned): the same kernels with 4-byte loads, by the same estimate (rates
            // 0.544 and 0.51 TFLOP/s per CU; 4001^3: 965 us on 128 x 128 tiles, 1029 on 64 x 64)
            vi = kEdgeDword;
            if (st.forced_split_k <= 1 && tiles(kVariants[kEdgeBigDword]) >= cus &&
                estimate(kEdgeBigDword, 0.544e6, tail_ok) < estimate(kEdgeDword, 0.51e6, tail_ok))
                vi = kEdgeBigDword;
        } else {
            vi = tiles(kVariants[0]) >= 2 * cus ? 0 : 1;
        }
    }
    const Variant &v = kVariants[vi];
    const int tiles_m = (M + v.bm - 1) / v.bm, tiles_n = (N + v.bn - 1) / v.bn;
    const int64_t nt = (int64_t)tiles_m * tiles_n;
    if (nt > INT32_MAX) return LSMI_ERR_TOO_LARGE;

    // Split the reduction when the output alone cannot fill the machine: aim at about one and
    // a half workgroups per compute unit (sweeps over 512^3, 1000^3, 256x256x8192 and
    // 4097x129x511 all have their best time there; more slices add atomic traffic faster than
    // they shorten the reduction), keep at least four chunks per slice.
    const int chunks = K > 0 ? (K + v.bk - 1) / v.bk : 1;  // K == 0: one empty slice runs the epilogue
    int split = ((v.dma && !v.edge) || !may_split) ? 1 : st.forced_split_k;
    if (split <= 0 && v.rows) {
        // fitted to sweeps of M = 1 .. 32 against 16 to 180 MB of B read from HBM (several
        // copies of B in rotation): B streams at 6.3 TB/s, plus the time one workgroup needs
        // for its own share at 38.5 GB/s (what it keeps in flight; longer when there are fewer
        // workgroups than CUs), plus, per slice, the output through the atomic units at 3.7 us
        // per MB and 0.15 us; at least two 64-deep chunks per slice.  Three steps in flight
        // per wave instead of one changed nothing.
        const double stream_us = 4.0 * N * K / 6.3e6, share_us = 4.0 * 64 * K / 38.5e3;
        const double slice_us = 3.7e-6 * 4.0 * M * N + 0.15;
        const int cap = chunks / 2 > 1 ? (chunks / 2 < 256 ? chunks / 2 : 256) : 1;
        double best = 0;
        split = 1;
        for (int s = 1; s <= cap; ++s) {
            const double wgs = (double)tiles_n * s;
            const double cost = stream_us + share_us / s * (wgs < cus ? cus / wgs : 1.0) + slice_us * s;
            if (s == 1 || cost < best) {
                best = cost;
                split = s;
            }
        }
    }
    if (split <= 0 && (vi == kEdgePair || vi == kEdgeDword)) {
        // fitted to sweeps of 16 .. 784 tiles: 0.56 us per 32-deep step of a lone workgroup,
        // workgroups beyond one per CU share it, and s > 1 slices send s times the output
        // through the floating-point atomic units at about 0.7 TB/s
        const double atomic_us = 4.0 * M * N / 0.7e6;
        const int cap = chunks / 4 > 1 ? (chunks / 4 < 64 ? chunks / 4 : 64) : 1;
        double best = 0;
        split = 1;
        for (int s = 1; s <= cap; ++s) {
            const int per = (chunks + s - 1) / s;
            const int64_t rounds = (nt * s + cus - 1) / cus;
            const double cost = 0.56 * per * rounds + (s > 1 ? s * atomic_us : 0.0);
            if (s == 1 || cost < best) {
                best = cost;
                split = s;
            }
        }
    }
    // the tiles of an incomplete last round as slices, see below
    TailPlan tail;
    if (v.edge && !v.rows && may_split && st.forced_split_k <= 0) tail = plan_tail(v, nt, chunks, cus);
    if (split <= 0) {
        split = 1;
        if (nt < 2 * cus && tail.split <= 1) {
            int64_t want = (3 * (int64_t)cus + 2 * nt - 1) / (2 * nt);
            int64_t cap = chunks / 4 > 1 ? chunks / 4 : 1;
            split = (int)(want < cap ? want : cap);
        }
    }
    if (split > chunks) split = chunks;
    if (split > 65535) split = 65535;
    const int chunks_per_split = (chunks + split - 1) / split;
    const int k_per_split = chunks_per_split * v.bk;
    split = (chunks + chunks_per_split - 1) / chunks_per_split;

    const int group_m = 8;
    // Tail split (buffer-load kernels, plain accumulate form): the tiles left over after the
    // last whole round of the CUs are cut into as many slices as fill one more round, so that
    // round lasts a slice's time instead of a tile's.  Taken when the time saved (at the rate
    // of one tile per CU, 0.47 TFLOP/s) exceeds what the slices' atomic adds cost.
    if (tail.split > 1 && split == 1) {
        const int per = (chunks + tail.split - 1) / tail.split;
        const int slices = (chunks + per - 1) / per;
        const int64_t rem = nt % cus;
        v.launch(dim3((unsigned)(nt - rem + rem * slices), 1u), st.stream, M, N, K, A, lda, B, ldb, C, ldc,
                 tiles_m, tiles_n, group_m, per * v.bk, 1, (int)(nt - rem), slices, ep);
        int rc = check_launch();
        if (rc == LSMI_OK) st.last_variant = v.tail_name;
        return rc;
    }
    // More tiles than fit on the machine at once (four workgroups per CU): a single launch
    // hands the later tiles to whichever CU frees a slot first, and some CUs end up with a
    // tile more than others -- 8192 x 4096 x 4096, 2048 tiles: 2085 us, the time of nine tiles
    // per CU instead of eight.  One launch per generation of 4 x CUs tiles gives every CU the
    // same number (1888 us; 16384 x 4096 x 4096: 3951 -> 3767).  A last generation of less
    // than one tile per CU stays in one launch with the one before it.
    const int64_t generation = 4 * (int64_t)cus;
    // The buffer-load form of the same tile likewise when M or N leave partial tiles and the
    // reduction is long (8000 x 4000 x 4096, 2016 tiles: 2151 -> 1990 us; 8100 x 4096 x 4096:
    // 2090 -> 1925; with whole tiles only, or K = 1024, its single launch is 3 - 5 % ahead),
    // unless its left-over tiles run as slices.
    const bool whole_tiles = vi == kDefaultDma || ((vi == kEdgeBig || vi == kEdgeBigDword) && tail.split <= 1 &&
                                                   K >= 2048 && (M % 128 != 0 || N % 128 != 0));
    if (whole_tiles && split == 1 && nt >= generation + cus) {
        for (int64_t first = 0; first < nt;) {
            const int64_t count = nt - first < generation + cus ? nt - first : generation;
            v.launch(dim3((unsigned)count, 1u), st.stream, M, N, K, A, lda, B, ldb, C, ldc, tiles_m, tiles_n,
                     group_m, k_per_split, 1, (int)first, 0, ep);
            first += count;
        }
    } else {
        v.launch(dim3((unsigned)nt, (unsigned)split), st.stream, M, N, K, A, lda, B, ldb, C, ldc,
                 tiles_m, tiles_n, group_m, k_per_split, split, 0, 0, ep);
    }
    int rc = check_launch();
    if (rc == LSMI_OK) st.last_variant = v.name;
    return rc;
}

}  // namespace lsmi
