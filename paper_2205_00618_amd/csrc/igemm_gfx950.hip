// Signed 8-bit GEMM with 32-bit sums, C += A.B, for gfx950: the generalised contraction of
// Section 2.1 with integer plus/times on V_MFMA_I32_32X32X32_I8.
//
// Each lane feeds the instruction 16 consecutive-k bytes of one A row and of one B column.
// A is k-contiguous in memory, so its tile is staged in LDS as is and a lane reads its 16
// bytes with one 16-byte LDS load.  B is n-contiguous, so on the way into LDS every
// thread transposes a 4(k) x 4(n) byte block in registers and the tile is stored as
// [k/4][n] dwords, a dword holding four consecutive k of one column; a lane then gathers
// its 16 bytes with four dword reads down that column.  Lanes 0..31 take the first 16 k
// of each 32-k group, lanes 32..63 the second 16; integer sums are order-free, so only
// the agreement between the two operands matters.  Sums wrap modulo 2^32 like the
// hardware accumulators do, and split-K partial sums are combined with integer atomic
// adds, so the result is bit-exact for every dispatch.
#include <mutex>

#include "common.hpp"
#include "igemm_big.hpp"
#include "igemm_dma.hpp"

namespace lsmi {
namespace {

typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef int i32x16 __attribute__((ext_vector_type(16)));

constexpr int kXcdCount = 8;

// BT: the second operand is given transposed (N x K, k-contiguous); its tile is then staged
// and read like A's, [n][k] bytes, and block column b of a wave is columns 32b + lane%32.
template <int BM_, int BN_, int WAVES_M_, int WAVES_N_, bool BT_ = false>
struct ITile {
    static constexpr bool BT = BT_;
    static constexpr int BM = BM_, BN = BN_, BK = 64;
    static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
    static constexpr int NT = 64 * WAVES_M * WAVES_N;
    static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    static constexpr int TM = WTM / 32, TN = WTN / 32;
    static constexpr int A_LD = BK + 16;  // bytes per LDS row of A
    static constexpr int B_LD = BN + 8;   // dwords per LDS row of B (one row = four k)
    static constexpr int A_STAGE = BM * A_LD;       // bytes
    static constexpr int B_STAGE = BT ? BN * A_LD / 4 : (BK / 4) * B_LD; // dwords
    static constexpr int LDS_BYTES = 2 * (A_STAGE + 4 * B_STAGE);
    static constexpr int A_SLOTS = BM * BK / 16 / NT;        // 16-byte runs along k
    static constexpr int B_SLOTS = BT ? BN * BK / 16 / NT : (BK / 4) * (BN / 4) / NT; // 16-byte runs / 4x4 byte blocks
    static_assert(TN == 1 || TN == 2, "B fragment is read as 1 or 2 dwords");
    static_assert((BM * BK / 16) % NT == 0 && ((BK / 4) * (BN / 4)) % NT == 0 && (BN * BK / 16) % NT == 0,
                  "loads divide evenly");
};

template <class T>
__global__ __launch_bounds__(T::NT) void igemm_kernel(int M, int N, int K,
                                                      const int8_t *__restrict__ A, int64_t lda,
                                                      const int8_t *__restrict__ B, int64_t ldb,
                                                      int32_t *__restrict__ C, int64_t ldc,
                                                      int tiles_m, int tiles_n, int k_per_split,
                                                      int split_k)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[T::LDS_BYTES];
    unsigned char *const a_lds = lds;
    int *const b_lds = reinterpret_cast<int *>(lds + 2 * T::A_STAGE);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, half = lane >> 5;
    const int wrow = (wave / T::WAVES_N) * T::WTM;
    const int wcol = (wave % T::WAVES_N) * T::WTN;

    // XCD-contiguous, row-major walk over the tiles
    const int nt = tiles_m * tiles_n;
    const int q = nt / kXcdCount, rem = nt % kXcdCount;
    const int xcd = blockIdx.x % kXcdCount;
    const int logical = xcd * q + (xcd < rem ? xcd : rem) + blockIdx.x / kXcdCount;
    const int m0 = (logical / tiles_n) * T::BM, n0 = (logical % tiles_n) * T::BN;

    const int kbeg = blockIdx.y * k_per_split;
    const int kend = (kbeg + k_per_split < K) ? kbeg + k_per_split : K;
    if (kbeg >= kend) return;

    // A group (16 bytes along k, 4 bytes along n) that lies inside the matrix and the slice is
    // loaded whole at whatever address its row starts: the types say "alignment 1" and the
    // compiler picks the instructions the target allows for that (single wide loads where
    // unaligned access is on).  The group lies inside its row, so nothing past the operand is
    // read.  Rows past M (columns past N of a transposed B) are zeros without a load; only the
    // groups that straddle N and the chunk that crosses the end of the slice go byte by byte
    // under tests.
    typedef i32x4 i32x4_any __attribute__((aligned(1)));
    typedef unsigned unsigned_any __attribute__((aligned(1)));

    i32x4 ra[T::A_SLOTS];
    i32x4 rb[T::B_SLOTS];  // after the transpose: rb[v][c] = four k of column 4*nq + c

    auto gload = [&](int k0) {
        const bool kfull = k0 + T::BK <= kend;
#pragma unroll
        for (int v = 0; v < T::A_SLOTS; ++v) {
            const int slot = tid + v * T::NT;
            const int row = slot / (T::BK / 16), kq = slot % (T::BK / 16);
            const int8_t *src = A + (int64_t)(m0 + row) * lda + k0 + kq * 16;
            if (kfull) {
                ra[v] = i32x4{0, 0, 0, 0};
                if (m0 + row < M) ra[v] = *reinterpret_cast<const i32x4_any *>(src);
            } else {
                const bool row_ok = m0 + row < M;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    unsigned word = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int k = k0 + kq * 16 + d * 4 + e;
                        const unsigned byte = (row_ok && k < kend) ? (unsigned char)src[d * 4 + e] : 0u;
                        word |= byte << (8 * e);
                    }
                    ra[v][d] = (int)word;
                }
            }
        }
        if constexpr (T::BT) {
            // rows of Bt are output columns: the same 16-byte runs along k as for A
#pragma unroll
            for (int v = 0; v < T::B_SLOTS; ++v) {
                const int slot = tid + v * T::NT;
                const int row = slot / (T::BK / 16), kq = slot % (T::BK / 16);
                const int8_t *src = B + (int64_t)(n0 + row) * ldb + k0 + kq * 16;
                if (kfull) {
                    rb[v] = i32x4{0, 0, 0, 0};
                    if (n0 + row < N) rb[v] = *reinterpret_cast<const i32x4_any *>(src);
                } else {
                    const bool row_ok = n0 + row < N;
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        unsigned word = 0;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int k = k0 + kq * 16 + d * 4 + e;
                            const unsigned byte = (row_ok && k < kend) ? (unsigned char)src[d * 4 + e] : 0u;
                            word |= byte << (8 * e);
                        }
                        rb[v][d] = (int)word;
                    }
                }
            }
            return;
        }
#pragma unroll
        for (int v = 0; v < T::B_SLOTS; ++v) {
            const int slot = tid + v * T::NT;
            const int kq = slot / (T::BN / 4), nq = slot % (T::BN / 4);
            const int8_t *src = B + (int64_t)(k0 + kq * 4) * ldb + n0 + nq * 4;
            unsigned r[4];  // r[e] = bytes n..n+3 of row k0 + 4*kq + e
            if (kfull && n0 + nq * 4 + 4 <= N) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    r[e] = *reinterpret_cast<const unsigned_any *>(src + (int64_t)e * ldb);
            } else if (kfull && n0 + nq * 4 >= N) {
#pragma unroll
                for (int e = 0; e < 4; ++e) r[e] = 0u;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool row_ok = k0 + kq * 4 + e < kend;
                    unsigned word = 0;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const unsigned byte =
                            (row_ok && n0 + nq * 4 + c < N) ? (unsigned char)src[(int64_t)e * ldb + c] : 0u;
                        word |= byte << (8 * c);
                    }
                    r[e] = word;
                }
            }
            // 4x4 byte transpose: column c gathers byte c of the four rows
#pragma unroll
            for (int c = 0; c < 4; ++c)
                rb[v][c] = (int)(((r[0] >> (8 * c)) & 0xffu) | (((r[1] >> (8 * c)) & 0xffu) << 8) |
                                 (((r[2] >> (8 * c)) & 0xffu) << 16) | (((r[3] >> (8 * c)) & 0xffu) << 24));
        }
    };

    auto sstore = [&](int buf) {
        unsigned char *as = a_lds + buf * T::A_STAGE;
        int *bs = b_lds + buf * T::B_STAGE;
#pragma unroll
        for (int v = 0; v < T::A_SLOTS; ++v) {
            const int slot = tid + v * T::NT;
            const int row = slot / (T::BK / 16), kq = slot % (T::BK / 16);
            *reinterpret_cast<i32x4 *>(as + row * T::A_LD + kq * 16) = ra[v];
        }
#pragma unroll
        for (int v = 0; v < T::B_SLOTS; ++v) {
            const int slot = tid + v * T::NT;
            if constexpr (T::BT) {
                const int row = slot / (T::BK / 16), kq = slot % (T::BK / 16);
                *reinterpret_cast<i32x4 *>(reinterpret_cast<unsigned char *>(bs) + row * T::A_LD + kq * 16) = rb[v];
            } else {
                const int kq = slot / (T::BN / 4), nq = slot % (T::BN / 4);
                *reinterpret_cast<i32x4 *>(bs + kq * T::B_LD + nq * 4) = rb[v];
            }
        }
    };

    i32x16 acc[T::TM][T::TN];
#pragma unroll
    for (int a = 0; a < T::TM; ++a)
#pragma unroll
        for (int b = 0; b < T::TN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0;

    auto consume = [&](int buf) {
        const unsigned char *as = a_lds + buf * T::A_STAGE;
        const int *bs = b_lds + buf * T::B_STAGE;
#pragma unroll
        for (int u = 0; u < T::BK / 32; ++u) {
            i32x4 af[T::TM];
#pragma unroll
            for (int a = 0; a < T::TM; ++a)
                af[a] = *reinterpret_cast<const i32x4 *>(as + (wrow + 32 * a + li) * T::A_LD + 32 * u + 16 * half);
            i32x4 bf[T::TN];  // bf[b][d] = k-quad d of column TN*li + b (BT: of column 32b + li)
            if constexpr (T::BT) {
#pragma unroll
                for (int b = 0; b < T::TN; ++b)
                    bf[b] = *reinterpret_cast<const i32x4 *>(reinterpret_cast<const unsigned char *>(bs) +
                                                             (wcol + 32 * b + li) * T::A_LD + 32 * u + 16 * half);
            }
#pragma unroll
            for (int d = 0; d < (T::BT ? 0 : 4); ++d) {
                const int *p = bs + (8 * u + 4 * half + d) * T::B_LD + wcol + T::TN * li;
                if constexpr (T::TN == 1) {
                    bf[0][d] = *p;
                } else {
                    const i32x2 two = *reinterpret_cast<const i32x2 *>(p);
                    bf[0][d] = two[0];
                    bf[1][d] = two[1];
                }
            }
#pragma unroll
            for (int a = 0; a < T::TM; ++a)
#pragma unroll
                for (int b = 0; b < T::TN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[a], bf[b], acc[a][b], 0, 0, 0);
        }
    };

    gload(kbeg);
    sstore(0);
    __syncthreads();
    int buf = 0;
    for (int k0 = kbeg; k0 < kend; k0 += T::BK) {
        const bool has_next = k0 + T::BK < kend;
        if (has_next) gload(k0 + T::BK);
        consume(buf);
        if (has_next) sstore(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }

    // Epilogue.  Register v of block (a, b): row 32a + 8(v/4) + 4*half + v%4, column TN*li + b.
    constexpr int CSTEP = T::BT ? 32 : 1;  // distance between the columns of blocks b and b+1
    const int col = n0 + wcol + (T::BT ? li : T::TN * li);
    // the old values of a block row are requested together, ahead of the stores (a load behind
    // a store to C would wait for that store: one memory round trip per register)
#pragma unroll
    for (int a = 0; a < T::TM; ++a) {
        uint32_t old[16][T::TN];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = m0 + wrow + 32 * a + 8 * (v >> 2) + 4 * half + (v & 3);
            int32_t *dst = C + (int64_t)row * ldc + col;
#pragma unroll
            for (int b = 0; b < T::TN; ++b) {
                old[v][b] = 0;
                if (row < M && col + CSTEP * b < N) {
                    if (split_k > 1)
                        atomicAdd(dst + CSTEP * b, acc[a][b][v]);
                    else
                        old[v][b] = (uint32_t)dst[CSTEP * b];
                }
            }
        }
        if (split_k > 1) continue;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = m0 + wrow + 32 * a + 8 * (v >> 2) + 4 * half + (v & 3);
            int32_t *dst = C + (int64_t)row * ldc + col;
#pragma unroll
            for (int b = 0; b < T::TN; ++b)
                if (row < M && col + CSTEP * b < N) dst[CSTEP * b] = (int32_t)(old[v][b] + (uint32_t)acc[a][b][v]);
        }
    }
}

typedef ITile<128, 128, 2, 2> IBig;
typedef ITile<64, 64, 2, 2> ISmall;
typedef ITile<128, 128, 2, 2, true> IBigBt;
typedef ITile<64, 64, 2, 2, true> ISmallBt;

template <class T>
void launch_tile(hipStream_t s, int split, int k_per_split, int M, int N, int K, const int8_t *A,
                 int64_t lda, const int8_t *B, int64_t ldb, int32_t *C, int64_t ldc)
{
    const int tiles_m = (M + T::BM - 1) / T::BM, tiles_n = (N + T::BN - 1) / T::BN;
    hipLaunchKernelGGL(igemm_kernel<T>, dim3((unsigned)(tiles_m * tiles_n), (unsigned)split),
                       dim3(T::NT), 0, s, M, N, K, A, lda, B, ldb, C, ldc, tiles_m, tiles_n,
                       k_per_split, split);
}

// Direct-to-LDS kernels: tile rows x 128 columns x 128 reduction bytes per chunk.
struct IDmaVariant {
    const char *name, *bt_name;
    int bm, bn, bk, lds_bytes;
    bool splits;  // takes a reduction cut over gridDim.y
    hipError_t (*launch)(hipStream_t s, int slices, int chunks_per_slice, int M, int N, int K, const int8_t *A,
                         int64_t lda, const int8_t *B, int64_t ldb, int32_t *C, int64_t ldc);
    // the same tile for a transposed (k-contiguous) second operand
    hipError_t (*launch_bt)(hipStream_t s, int slices, int chunks_per_slice, int M, int N, int K, const int8_t *A,
                            int64_t lda, const int8_t *B, int64_t ldb, int32_t *C, int64_t ldc);
    bool edge = false;   // takes M, N, K that are not multiples of the tile (row pitches multiples of 16)
    bool dword = false;  // an edge form on 4-byte loads: row pitches multiples of 4
};

template <class T>
hipError_t launch_idma(hipStream_t s, int slices, int chunks_per_slice, int M, int N, int K, const int8_t *A,
                       int64_t lda, const int8_t *B, int64_t ldb, int32_t *C, int64_t ldc)
{
    static std::once_flag once;
    static hipError_t raised = hipSuccess;
    std::call_once(once, [] {
        raised = hipFuncSetAttribute(reinterpret_cast<const void *>(igemm_dma_kernel<T>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
    });
    if (raised != hipSuccess) return raised;
    const int tiles_m = (M + T::BM - 1) / T::BM, tiles_n = (N + T::BN - 1) / T::BN;  // whole tiles unless EDGE
    hipLaunchKernelGGL(igemm_dma_kernel<T>, dim3((unsigned)(tiles_m * tiles_n), (unsigned)slices), dim3(T::NT),
                       T::LDS_BYTES, s, M, N, K, A, lda, B, ldb, C, ldc,
                       TileMap(tiles_m, tiles_n, tls().forced_group_m > 0 ? tls().forced_group_m : T::BM >= 256 ? 2 : 8), chunks_per_slice);
    return hipSuccess;
}

// 256 x 256 tiles, one workgroup per CU: no reduction split (slices is always 1).  The workgroups walk C
// in bands of two tile rows, 512 rows of C (lsmi_set_tile_walk overrides): the int8 kernels feel what the order
// leaves for the L2s to fetch -- 8192 x 8192 x 4096 343.5 us in bands of eight tile rows, 346.6 in four, 317.7 in two,
// 359.6 in sixteen; 8192 x 4096 x 2048 on half tiles 98.9, 94.0, 88.0, 98.1; 4096^3 78.7, 78.9, 77.8, 80.1 -- while
// the 64-row tiles do best at eight or sixteen (8192 x 8192 x 1024: 148.3, 150.2, 164.6, 192.7).
template <class T>
hipError_t launch_ibig(hipStream_t s, int, int, int M, int N, int K, const int8_t *A, int64_t lda,
                       const int8_t *B, int64_t ldb, int32_t *C, int64_t ldc)
{
    static std::once_flag once;
    static hipError_t raised = hipSuccess;
    std::call_once(once, [] {
        raised = hipFuncSetAttribute(reinterpret_cast<const void *>(igemm_big_kernel<T>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
    });
    if (raised != hipSuccess) return raised;
    const int tiles_m = M / T::BM, tiles_n = N / T::BN;
    hipLaunchKernelGGL(igemm_big_kernel<T>, dim3((unsigned)(tiles_m * tiles_n)), dim3(T::NT), T::LDS_BYTES, s, K,
                       A, lda, B, ldb, C, ldc, TileMap(tiles_m, tiles_n, tls().forced_group_m > 0 ? tls().forced_group_m : 2));
    return hipSuccess;
}

#define LSMI_IBIG_VARIANT(NS)                                                                 \
    {"igemm_big_256x256x64_w2x2_s" #NS, "igemm_bt_big_256x256x64_w2x2_s" #NS, 256, 256, 64,    \
     IBigShape<NS, false>::LDS_BYTES, false, &launch_ibig<IBigShape<NS, false>>,               \
     &launch_ibig<IBigShape<NS, true>>}
#define LSMI_IBIG_HALF_VARIANT(NS)                                                            \
    {"igemm_big_256x128x64_w2x2_s" #NS, "igemm_bt_big_256x128x64_w2x2_s" #NS, 256, 128, 64,    \
     IBigShape<NS, false, 128>::LDS_BYTES, false, &launch_ibig<IBigShape<NS, false, 128>>,     \
     &launch_ibig<IBigShape<NS, true, 128>>}
#define LSMI_IDMA_VARIANT(BM, WM, WN, NS)                                                     \
    {"igemm_dma_" #BM "x128x128_w" #WM "x" #WN "_s" #NS, "igemm_bt_dma_" #BM "x128x128_w" #WM "x" #WN "_s" #NS, \
     BM, 128, 128, IDmaShape<BM, WM, WN, NS>::LDS_BYTES, true, &launch_idma<IDmaShape<BM, WM, WN, NS>>, \
     &launch_idma<IDmaShape<BM, WM, WN, NS, 128, true>>}
#define LSMI_IDMA_VARIANT64(BM, WM, WN, NS)                                                   \
    {"igemm_dma_" #BM "x128x64_w" #WM "x" #WN "_s" #NS, "igemm_bt_dma_" #BM "x128x64_w" #WM "x" #WN "_s" #NS, \
     BM, 128, 64, IDmaShape<BM, WM, WN, NS, 64>::LDS_BYTES, true, &launch_idma<IDmaShape<BM, WM, WN, NS, 64>>, \
     &launch_idma<IDmaShape<BM, WM, WN, NS, 64, true>>}

#define LSMI_IDMA_EDGE_VARIANT(BM, WM, WN, NS)                                                \
    {"igemm_dma_edge_" #BM "x128x128_w" #WM "x" #WN "_s" #NS,                                  \
     "igemm_bt_dma_edge_" #BM "x128x128_w" #WM "x" #WN "_s" #NS, BM, 128, 128,                 \
     IDmaShape<BM, WM, WN, NS>::LDS_BYTES, true, &launch_idma<IDmaShape<BM, WM, WN, NS, 128, false, true>>, \
     &launch_idma<IDmaShape<BM, WM, WN, NS, 128, true, true>>, true}

#define LSMI_IDMA_EDGE4_VARIANT(BM, WM, WN, NS)                                               \
    {"igemm_dma_edge4_" #BM "x128x128_w" #WM "x" #WN "_s" #NS,                                 \
     "igemm_bt_dma_edge4_" #BM "x128x128_w" #WM "x" #WN "_s" #NS, BM, 128, 128,                \
     IDmaShape<BM, WM, WN, NS>::LDS_BYTES, true,                                              \
     &launch_idma<IDmaShape<BM, WM, WN, NS, 128, false, true, true>>,                         \
     &launch_idma<IDmaShape<BM, WM, WN, NS, 128, true, true, true>>, true, true}

const IDmaVariant kIDmaVariants[] = {
    LSMI_IDMA_VARIANT(64, 1, 2, 3),   // 0: two waves of 64 x 64, small outputs
    LSMI_IDMA_VARIANT(128, 2, 2, 2),  // 1: four waves of 64 x 64, two workgroups per CU
    LSMI_IDMA_VARIANT(128, 2, 2, 3),  // 2
    LSMI_IDMA_VARIANT(256, 2, 2, 2),  // 3: four waves of 128 x 64
    LSMI_IDMA_VARIANT(256, 4, 2, 2),  // 4: eight waves of 64 x 64
    LSMI_IDMA_VARIANT(256, 4, 2, 3),  // 5
    LSMI_IDMA_VARIANT64(256, 4, 2, 4),  // 6: 64-byte chunks, four stages: same rate as 5, kept for sweeps
    LSMI_IDMA_VARIANT64(128, 2, 2, 4),  // 7
    LSMI_IBIG_VARIANT(4),               // 8: four waves of 128 x 128, hand-scheduled loop
    LSMI_IBIG_VARIANT(3),               // 9
    LSMI_IDMA_EDGE_VARIANT(64, 1, 2, 3),   // 10: 0 and 1 for ragged M, N, K (buffer loads, zero fill)
    LSMI_IDMA_EDGE_VARIANT(128, 2, 2, 2),  // 11
    LSMI_IBIG_HALF_VARIANT(3),             // 12: 8 on 256 x 128 tiles, two workgroups per CU
    LSMI_IDMA_VARIANT(64, 1, 2, 6),        // 13: 0 with a ring that holds most of a short reduction
    LSMI_IDMA_VARIANT(64, 2, 2, 6),        // 14: the same with four waves of 32 x 64
    LSMI_IDMA_VARIANT(64, 2, 2, 3),        // 15
    LSMI_IDMA_VARIANT(64, 2, 4, 3),        // 16: eight waves of 32 x 32: small outputs are bound by what one wave
                                           //     does per chunk, not by the matrix pipe (1024^3 6.7 -> 5.9 us,
                                           //     1024 x 1024 x 2048 10.0 -> 7.0, 2048 x 1024 x 1024 7.4 -> 5.9)
    LSMI_IDMA_VARIANT(64, 2, 4, 4),        // 17
    LSMI_IDMA_VARIANT(64, 2, 2, 4),        // 18
    LSMI_IDMA_EDGE_VARIANT(64, 2, 4, 3),   // 19: 16 for ragged M, N, K
    LSMI_IDMA_EDGE4_VARIANT(64, 2, 4, 3),  // 20: 19 on 4-byte loads, for rows that are only 4-byte aligned
    LSMI_IDMA_EDGE4_VARIANT(128, 2, 4, 2), // 21: eight waves of 64 x 32 (with four waves of 64 x 64 each wave issues
                                           //     32 loads per chunk: 4000^3 152 us against 96)
    LSMI_IDMA_EDGE_VARIANT(128, 2, 4, 2),  // 22: 11 on eight waves (4000^3 93.7 -> 92.0 us, 2200 x 2208 x 2064 26.2 -> 23.8,
                                           //     4100 x 4112 x 2048 75.9 -> 72.5, 8000 x 8000 x 1008 147.2 -> 148.8)
    LSMI_IDMA_VARIANT(128, 2, 4, 2),       // 23: 1 on eight waves of 64 x 32
};
constexpr int kISmall = 16, kIEdgeSmall = 19, kIEdgeBig = 22, kIMid = 23;
constexpr int kIEdge4Small = 20, kIEdge4Big = 21;
constexpr int kNumIDma = sizeof(kIDmaVariants) / sizeof(kIDmaVariants[0]);
constexpr int kNumIgemmVariants = 2 + kNumIDma;  // 0, 1: the register-staged kernels

}  // namespace

int igemm_variant_count() { return kNumIgemmVariants; }

const char *igemm_variant_name(int index)
{
    if (index == 0) return "igemm_128x128x64";
    if (index == 1) return "igemm_64x64x64";
    return index >= 2 && index < kNumIgemmVariants ? kIDmaVariants[index - 2].name : nullptr;
}

int launch_igemm(int M, int N, int K, const int8_t *A, int64_t lda, const int8_t *B, int64_t ldb,
                 int32_t *C, int64_t ldc, bool bt)
{
    ThreadState &st = tls();
    const int cus = device_cu_count();

    // ---- direct-to-LDS kernels: whole tiles, 16-byte aligned rows ----
    auto dma_fits = [&](const IDmaVariant &v) {
        // edge: a load's group of 16 (4) bytes never straddles the end of a row: a row pitch that
        // is a multiple of the group keeps a group that starts before N, or before K, inside its
        // row.  The bytes of A it brings from past K meet rows of B that the kernel has filled
        // with zeros, so K itself may be anything; with a k-contiguous B both operands would
        // bring such bytes, and K has to be a multiple of the group.  31-bit lane offsets.
        if (v.edge)
            return (!bt || K % (v.dword ? 4 : 16) == 0) &&
                   (((uintptr_t)A | (uintptr_t)B | (uintptr_t)lda | (uintptr_t)ldb) & (v.dword ? 3 : 15)) == 0 &&
                   ((uintptr_t)C & 3) == 0 && (int64_t)v.bm * lda + 256 < (1LL << 31) &&
                   (int64_t)128 * ldb + 256 < (1LL << 31) &&
                   (int64_t)v.bm * ldc * 4 < (1LL << 31);  // (an edge tile's part of C, through 32-bit offsets too)
        return M % v.bm == 0 && N % v.bn == 0 && K % v.bk == 0 && K >= v.bk &&
               (((uintptr_t)A | (uintptr_t)B | (uintptr_t)lda | (uintptr_t)ldb) & 15) == 0 &&
               ((uintptr_t)C & 3) == 0 && (int64_t)v.bm * lda < (1LL << 32) &&
               (int64_t)v.bn * ldb < (1LL << 32);  // bn rows of k-contiguous B, at most 128 of n-contiguous
    };
    int dv = -1;
    if (st.forced_igemm_variant >= 2) {
        if (dma_fits(kIDmaVariants[st.forced_igemm_variant - 2])) dv = st.forced_igemm_variant - 2;
    } else if (st.forced_igemm_variant < 0) {
        // measured: 256 x 256 tiles (four waves of 128 x 128) lead when they fill at least three
        // quarters of the CUs in every round (1.7 POP/s at 4096^3, 2.0 at 8192^3 on random
        // data, where the clock, not the kernel, sets the rate) and also in a single round on
        // half the CUs or more (3072^3, 144 tiles: 42 against 51 us; probably idle CUs leave the
        // busy ones a higher clock), then 256 x 128 tiles (the same hand-scheduled loop with four
        // waves of 128 x 64, two workgroups per CU; 4096 x 2048 x 4096: 40.6 us against 46.9 on
        // 256 x 256 tiles for half the CUs and 42.1 on eight waves of 64 x 64) when they give every
        // CU a workgroup, then 128 x 128 tiles when they give every CU more than one (with exactly
        // one, 2048^3, the 64-row tiles' two per CU cover each other's epilogue: 17 against
        // 22 us); smaller outputs take 64-row tiles and split the reduction
        for (int i : {8, 12, 1, kISmall}) {
            if (!dma_fits(kIDmaVariants[i])) continue;
            const int64_t tiles = (int64_t)(M / kIDmaVariants[i].bm) * (N / kIDmaVariants[i].bn);
            bool take = tiles >= cus;
            if (i == 8) {
                const int64_t rounds = (tiles + cus - 1) / cus;
                take = 2 * tiles >= cus && (tiles < cus || 4 * tiles >= 3 * rounds * cus);
            }
            if (i == 1) take = tiles > cus;
            if (take || i == kISmall) {
                dv = i;
                break;
            }
        }
        // (long reductions on 128 x 128 tiles: eight waves of 64 x 32 instead of four of 64 x 64 --
        // 9600 x 3456 x 8192 298 -> 268 us, 2.03 POP/s; 3968 x 9856 x 4096 194 -> 181; but 4096 x 4096 x 2048
        // 50.6 against 58.0 -- a shape the larger tiles take; 4992 x 5504 x 2048 85.5 -> 80.4, 9088 x 9600 x 3072
        // 364 -> 343)
        if (dv == 1 && K >= 2048 && dma_fits(kIDmaVariants[kIMid])) dv = kIMid;
        // More than a round of 256 x 256 tiles whose last round is partly empty, on a long reduction:
        // the eight-wave 128 x 128 tiles multiply nearly as fast there (9600 x 3456 x 8192: 2.03 POP/s) and
        // divide over the CUs four times as finely -- 9984 x 8960 x 3072, 1365 tiles in six rounds, 398 ->
        // 344 us; 9984 x 7168 x 4096 380 -> 343; whole rounds stay (8192 x 8192 x 4096 343 against 356).
        if (dv == 8 && K >= 2048 && dma_fits(kIDmaVariants[kIMid])) {
            const int64_t t256 = (int64_t)(M / 256) * (N / 256), t128 = 4 * t256;
            const double loss_big = (double)((t256 + cus - 1) / cus * cus) / (double)t256;
            const double loss_mid = (double)((t128 + cus - 1) / cus * cus) / (double)t128;
            // (from four rounds of full tiles on: with fewer the half tiles below do better still, 6144 x 6144 x 2048,
            // 2.25 rounds, 109.5 us here against 99.3)
            if (t256 >= 4 * (int64_t)cus && loss_big > 1.05 * loss_mid) dv = kIMid;
        }
        // (M a multiple of 64 only, a long reduction, more than a 128 x 128 tile per CU: the ragged
        // forms below choose better than the 64-row whole-tile kernel -- 5952 x 7808 x 4096: 264 us
        // against 214 on the ragged 128 x 128 tile)
        if (dv == kISmall && K > 1024 && (int64_t)((M + 127) / 128) * ((N + 127) / 128) > cus &&
            dma_fits(kIDmaVariants[kIEdgeBig]))
            dv = -1;
        // 256 x 256 tiles or their halves.  A CU's one workgroup of the full tile multiplies (0.79
        // us per 64-byte chunk under random data), then reads and writes its C tile with the
        // matrix pipe idle, and since every CU does that at the same time the memory system sets
        // the pace: 23 us for a full round (4096^2 outputs: 128 MB at 5.6 TB/s).  Two workgroups
        // on half tiles, the first given priority (igemm_big.hpp), are out of step, so only the
        // last epilogue (about 9 us) shows; but a half tile reads more of LDS per matrix
        // instruction, and a CU's two take 1.0 us per chunk between them.  So short reductions
        // and outputs of up to two rounds go to the half tiles by that estimate (4096 x 4096 x
        // 1024: 40.3 -> 33.9 us, x 2048: 54.1 -> 48.6, x 4096: 84.4 -> 79.8, 2048 x 4096 x 4096: 52.1 -> 41.4, 6144 x
        // 4096 x 4096: 127.0 -> 115.4); from three rounds on the full tiles' workgroups drift
        // apart by themselves (8192 x 8192 x 4096: 342 us against 385).
        if (dv == 8 && dma_fits(kIDmaVariants[12])) {
            const int64_t full = (int64_t)(M / 256) * (N / 256), halves = 2 * full;
            const int64_t rounds = (full + cus - 1) / cus;
            // (three rounds: 6144 x 6144 x 3072, 2.25 rounds of full tiles, 162 -> 140 us; with the walk in bands of two
            // tile rows the estimate holds for any number of rounds: 8192 x 8192 x 2048 226 us on full tiles, 198 on
            // halves, x 4096 330 / 316, x 8192 536 / 566)
            {
                const double nk = K / 64.0;
                const double t_full = rounds * nk * 0.79 + 23.0 * full / (double)cus;
                const double t_half = (double)((halves + cus - 1) / cus) * nk * 0.50 + 9.0;
                if (t_half * (rounds == 3 ? 1.05 : 1.0) < t_full) dv = 12;
            }
        }
        // Short reductions: the call is the C tiles' way to memory and back (8192 x 8192 x 256: 537
        // MB), which many small workgroups per CU keep going where a few large ones take turns: the
        // 64 x 128 tiles of eight waves, for any output (8192 x 8192 x 256 147 -> 101 us, x 1024 182 ->
        // 150, 6144 x 6912 x 256 78.5 -> 54.9, 4096 x 4096 x 512 28.8 -> 26.3); up to K = 2048 from four
        // rounds of full tiles on (8192 x 8192 x 2048 241 -> 226)
        // -- the 256-row tiles in bands of two tile rows take K = 1024 back (4096 x 4096 x 1024 35.7 -> 33.2 us on
        // half tiles, 8192 x 8192 x 1024 148.3 -> 139.7, x 2048 222.5 -> 198.4; at K = 512 the 64-row tiles lead, 26.1 / 27.4)
        if ((dv == 8 || dv == 12 || dv == 1) && dma_fits(kIDmaVariants[kISmall]) &&
            (K < 1024 || (dv == 1 && (K <= 1024 || (K <= 2048 && (int64_t)(M / 256) * (N / 256) >= 4 * (int64_t)cus)))))
            dv = kISmall;
        // M, N or K not multiples of a tile (rows 16-byte aligned, K a multiple of 16): the
        // same two smallest tiles through buffer loads that return zeros past the edges
        // (4000^3: 498 us on the register-staged kernel; 1000^3: 31.5 us), small problems
        // included: the register-staged kernel's element loads under tests cost a few tiles
        // two to four times what the zero fill does (432 x 32 x 416 21.3 against 5.2 us, 96 x 352 x 704
        // 19.3 / 5.5, 256 x 256 x 928 8.4 / 5.7).
        // A short reduction whose 128 x 128 tiles are all resident at once (two per CU) and cover at
        // least half the CUs: the eight-wave 128 x 128 tile, half the workgroups for the same way of
        // C to memory and back (3000 x 2000 x 768, 384 tiles, 15.5 -> 13.7 us; 1500 x 1504 x 512, 144 tiles,
        // 7.1 -> 6.4; 2782 x 2336 x 96 9.1 -> 7.9; 1000^3, 64 tiles, 7.8 against 9.3 stays on 64 rows)
        auto short_one_round = [&](int64_t big) { return K <= 1024 && 2 * big >= cus && big <= 2 * (int64_t)cus; };
        if (dv < 0 && dma_fits(kIDmaVariants[kIEdgeBig])) {
            const int64_t big = (int64_t)((M + 127) / 128) * ((N + 127) / 128);
            // (eight waves of 32 x 32 up to a tile per CU, two of 64 x 64 beyond: 1000 x 4096 x 4096,
            // 512 tiles, 24.1 against 25.5 us)
            const int64_t small = (int64_t)((M + 63) / 64) * ((N + 127) / 128);
            // (and eight waves again when the 128-row tiles' last round is mostly empty: 3000 x 3008 x 3008,
            // 576 tiles, 50.7 against 58.0 us; 4000^3, 1024 tiles, 118 / 96; 1024 x 7808 x 4560, 488 tiles,
            // 61.5 / 50.6; 7424 x 1984 x 640, 928 tiles, 29.9 / 26.1; but 4000 x 4000 x 512 28.5 / 31.2)
            // A CU works through ceil(tiles / CUs) tiles, and a 64-row tile costs 0.6 of a 128-row one.
            const int64_t per_cu_big = (big + cus - 1) / cus, per_cu_small = (small + cus - 1) / cus;
            dv = big > cus ? (0.6 * per_cu_small <= (double)per_cu_big ? kIEdgeSmall : kIEdgeBig)
                           : small <= cus ? kIEdgeSmall : 10;
            if (short_one_round(big)) dv = kIEdgeBig;
        }
        // Rows that are only 4-byte aligned (a dense 1000 x 1000 A or B): the same loop on 4-byte
        // loads, four times the load instructions for the same bytes, spread over eight waves
        // (1000^3: 30.2 us on the register-staged kernel, 7.8 here; 3000^3 554 -> 61; 8000 x 8000 x 1000
        // 748 -> 153; within 3 to 8 % of the 16-byte form on shapes that allow both)
        if (dv < 0 && dma_fits(kIDmaVariants[kIEdge4Big])) {
            const int64_t big = (int64_t)((M + 127) / 128) * ((N + 127) / 128);
            dv = big > 2 * (int64_t)cus || short_one_round(big) ? kIEdge4Big : kIEdge4Small;
        }
    }
    if (dv >= 0) {
        const IDmaVariant &v = kIDmaVariants[dv];
        const int64_t tiles = (int64_t)((M + v.bm - 1) / v.bm) * ((N + v.bn - 1) / v.bn);  // whole unless edge
        const int chunks = (K + v.bk - 1) / v.bk;
        int slices = v.splits ? st.forced_split_k : 1;
        if (slices <= 0) {
            slices = 1;
            if (tiles < cus) {
                // Cut the reduction when that shortens the longest workgroup by more than the
                // atomic adds cost.  Fitted to sweeps of 256^2 .. 1536^2 outputs: 3.3 us of
                // launch and ramp, 0.42 us per 128-byte chunk of a workgroup, and for s > 1
                // slices s times the output through the atomic units at about 2.3 TB/s.
                // (eight waves: 0.14 us per chunk, 0.24 in the ragged form with its tests per chunk:
                // 704 x 592 x 2512, 55 tiles, 9.6 us whole and 7.2 in two slices)
                // (on 4-byte loads 0.48: 200 x 200 x 4000, 8 tiles, 18.7 us whole, 11.0 in two slices, 7.2 in four;
                // 88 x 3560 x 1080, 56 tiles, 7.9 whole and 6.4 in two)
                const double per_chunk = dv == kISmall ? 0.14 : dv == kIEdgeSmall ? 0.24 : dv == kIEdge4Small ? 0.48 : 0.42;
                const double chunk_us = per_chunk * v.bk / 128.0, atomic_us = 4.0 * M * N / 2.3e6;
                const int cap = chunks / 2 > 1 ? (chunks / 2 < 32 ? chunks / 2 : 32) : 1;
                double best = 0;
                for (int s = 1; s <= cap; ++s) {
                    const int per = (chunks + s - 1) / s;
                    const int64_t rounds = (tiles * s + cus - 1) / cus;
                    const double cost = per * chunk_us * rounds + (s > 1 ? s * atomic_us : 0.0);
                    if (s == 1 || cost < best) {
                        best = cost;
                        slices = s;
                    }
                }
            }
        }
        if (slices > chunks) slices = chunks;
        if (slices > 65535) slices = 65535;
        const int per = (chunks + slices - 1) / slices;
        slices = (chunks + per - 1) / per;
        const hipError_t err = (bt ? v.launch_bt : v.launch)(st.stream, slices, per, M, N, K, A, lda, B, ldb, C, ldc);
        if (err != hipSuccess) {
            st.last_hip_error = (int)err;
            return LSMI_ERR_LAUNCH;
        }
        st.last_variant = bt ? v.bt_name : v.name;
        return check_launch();
    }

    // ---- register-staged kernels: any shape ----
    const int64_t big_tiles = (int64_t)((M + 127) / 128) * ((N + 127) / 128);
    // 128 x 128 tiles when there are two per CU and the reduction is not a handful of chunks
    // (4682 x 7472 x 81: 117 us on them, 85 on 64 x 64), and for long reductions from a few dozen
    // tiles on, their reduction cut (1514 x 1536 x 6900: 435 us on 64 x 64 tiles, 310 on 128 x 128 in
    // two slices; 2718 x 208 x 6626: 181 / 125)
    const bool big = st.forced_igemm_variant == 0 ||
                     (st.forced_igemm_variant != 1 &&
                      (big_tiles >= 2 * cus ? K >= 256
                                            : ((K >= 1024 && big_tiles >= 128) || (K >= 4096 && big_tiles >= 40))));
    const int bm = big ? 128 : 64;
    const int64_t nt = (int64_t)((M + bm - 1) / bm) * ((N + bm - 1) / bm);
    if (nt > INT32_MAX) return LSMI_ERR_TOO_LARGE;
    const int chunks = (K + 63) / 64;
    int split = st.forced_split_k;
    if (split <= 0) {
        split = 1;
        if (nt < 2 * cus && big) {
            // measured at 1024^3: two slices per tile beat one and four (integer atomics are slow)
            int64_t want = (2 * (int64_t)cus + nt - 1) / nt;
            int64_t cap = chunks / 4 > 1 ? chunks / 4 : 1;
            split = (int)(want < cap ? want : cap);
        } else if (nt < 2 * cus) {
            // The 64 x 64 tiles only see rows at odd addresses now (unaligned group loads): a chunk
            // of a lone workgroup costs 1.2 us, so up to two workgroups per CU the slices go down
            // to a single chunk (301^3, 25 tiles of 5 chunks: 11.1 us whole, 7.2 in five slices;
            // 545 x 1032 x 3733, 153 tiles: 48.3 whole, 23.2 in three; 1001^3, 256 tiles: 20.8 / 17.1)
            const int64_t want = 2 * (int64_t)cus / nt;
            split = (int)(want < chunks ? want : chunks);
            if (split < 1) split = 1;
        }
    }
    if (split > chunks) split = chunks;
    if (split > 65535) split = 65535;
    const int chunks_per_split = (chunks + split - 1) / split;
    const int k_per_split = chunks_per_split * 64;
    split = (chunks + chunks_per_split - 1) / chunks_per_split;
    if (big) {
        if (bt) launch_tile<IBigBt>(st.stream, split, k_per_split, M, N, K, A, lda, B, ldb, C, ldc);
        else launch_tile<IBig>(st.stream, split, k_per_split, M, N, K, A, lda, B, ldb, C, ldc);
        st.last_variant = bt ? "igemm_bt_128x128x64" : "igemm_128x128x64";
    } else {
        if (bt) launch_tile<ISmallBt>(st.stream, split, k_per_split, M, N, K, A, lda, B, ldb, C, ldc);
        else launch_tile<ISmall>(st.stream, split, k_per_split, M, N, K, A, lda, B, ldb, C, ldc);
        st.last_variant = bt ? "igemm_bt_64x64x64" : "igemm_64x64x64";
    }
    return check_launch();
}

}  // namespace lsmi
