// fp32 workgroup-tile machinery shared by the GEMM and the convolution kernels (gfx950).
//
// The schedule is the classical one the paper's Section 2.2 lists for contractions,
// mapped to this machine: the output is split into BM x BN workgroup tiles and the
// reduction into BK chunks; each chunk of both operands is staged ("packed", Section 4.3
// staging annotation) into LDS; each wave keeps a (32*TM) x (32*TN) sub-tile of the
// output in accumulator registers for the whole reduction (the no-spill register
// blocking of Section 5.1) and feeds V_MFMA_F32_32X32X2_F32 from LDS fragments.
//
// Operand convention of v_mfma_f32_32x32x2_f32: lane l supplies a = A[l%32][l/32] and
// b = B[l/32][l%32]; accumulator register v of lane l holds
// D[8*(v/4) + 4*(l/32) + v%4][l%32].  Which k of a chunk a given MFMA consumes is free as
// long as both operands agree, so lanes 0..31 take k = 8u+0..3 and lanes 32..63 take
// k = 8u+4..7 of each group of eight: an operand stored k-contiguous in LDS is then
// fetched with one 16-byte read per four MFMAs.
#pragma once

#include <cstdint>
#include <type_traits>
#include <utility>
#include <hip/hip_runtime.h>

namespace lsmi {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int N> struct FVec;
template <> struct FVec<1> { typedef float type; };
template <> struct FVec<2> { typedef f32x2 type; };
template <> struct FVec<4> { typedef f32x4 type; };

template <int N>
__device__ inline float vec_get(const typename FVec<N>::type &v, int i)
{
    if constexpr (N == 1) return v; else return v[i];
}

// Element-wise operations around the contraction, C = post(pre(C_in) + A.B), the general
// form of Section 2.1: `pre` initialises the output (its old contents, zero, or a bias
// broadcast along rows), `post` transforms the sum before it is stored.
enum : int { kPreAccumulate = 0, kPreZero = 1, kPreBias = 2 };
enum : int { kPostNone = 0, kPostRelu = 1 };
struct Epilogue {
    const float *bias;  // one value per output column / channel when pre == kPreBias
    int pre, post;
};

__device__ inline float apply_post(float x, int post) { return post == kPostRelu ? fmaxf(x, 0.f) : x; }

// Calls f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N-1>{}):
// a loop whose index is a compile-time constant inside the body.
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// Number of XCDs workgroup ids are dealt to round-robin.
constexpr int kXcds = 8;

// Division of a 32-bit unsigned number by a divisor that the host knows at launch: the
// quotient is a high multiply, an add and two shifts (division by an invariant through
// multiplication by its rounded-up reciprocal) instead of the forty-odd vector instructions of
// a general division.  A kernel's start is address arithmetic on every wave of every resident
// workgroup at once, with nothing to multiply yet: the tile walk and the pixel decoding of the
// convolution spent several microseconds there on divisions alone.  Exact for every n < 2^32.
struct FastDiv {
    uint32_t divisor, magic, shift1, shift2;

    FastDiv() : divisor(1), magic(1), shift1(0), shift2(0) {}
    explicit FastDiv(uint32_t d) : divisor(d ? d : 1)
    {
        uint32_t l = 0;  // ceil(log2(divisor))
        while (l < 32 && (uint64_t{1} << l) < divisor) ++l;
        magic = (uint32_t)(((uint64_t{1} << 32) * ((uint64_t{1} << l) - divisor)) / divisor + 1);
        shift1 = l < 1 ? l : 1;
        shift2 = l > 1 ? l - 1 : 0;
    }
    __host__ __device__ uint32_t div(uint32_t n) const
    {
#if defined(__HIP_DEVICE_COMPILE__)
        const uint32_t t = __umulhi(magic, n);
#else
        const uint32_t t = (uint32_t)(((uint64_t)magic * n) >> 32);
#endif
        return (t + ((n - t) >> shift1)) >> shift2;
    }
    __host__ __device__ uint32_t mod(uint32_t n) const { return n - div(n) * divisor; }
};

// Maps the linear workgroup id to a tile (tm, tn).  Consecutive ids land on different
// XCDs, each with a private L2, so ids are first regrouped such that every XCD owns one
// contiguous range of tiles; inside the range tiles are walked in column-major bands of
// `group_m` tile rows so that the tiles resident at the same time share A row panels and
// B column panels.  The divisors of the walk are fixed per launch (FastDiv).
struct TileMap {
    int tiles_m, tiles_n, group_m;
    int per_xcd, extra_xcds;     // tiles of every XCD, and how many XCDs take one more
    int cut_per_xcd, cut_extra;  // the same for the workgroups of a launch that cuts every tile into slices
    FastDiv band;                // tiles of a full band: group_m * tiles_n
    FastDiv rows_full, rows_last;  // tile rows of a full band and of the last, possibly shorter one
    FastDiv tiles;               // all tiles

    TileMap() : tiles_m(1), tiles_n(1), group_m(1), per_xcd(0), extra_xcds(0), cut_per_xcd(0), cut_extra(0) {}
    TileMap(int tm, int tn, int gm, int slices = 1) : tiles_m(tm), tiles_n(tn), group_m(gm)
    {
        const int64_t nt = (int64_t)tm * tn;
        per_xcd = (int)(nt / kXcds);
        extra_xcds = (int)(nt % kXcds);
        cut_per_xcd = (int)(nt * slices / kXcds);
        cut_extra = (int)(nt * slices % kXcds);
        band = FastDiv((uint32_t)(gm * tn));
        rows_full = FastDiv((uint32_t)gm);
        rows_last = FastDiv((uint32_t)(tm % gm ? tm % gm : gm));
        tiles = FastDiv((uint32_t)nt);
    }
    // position of workgroup wg in the order in which every XCD owns one contiguous range
    __host__ __device__ static uint32_t regroup(int wg, int each, int extra)
    {
        const int xcd = (int)((uint32_t)wg % kXcds), idx = (int)((uint32_t)wg / kXcds);
        return (uint32_t)(xcd * each + (xcd < extra ? xcd : extra) + idx);
    }
    // tile at position `logical` of the walk down the bands
    __host__ __device__ void walk(uint32_t logical, int &tm, int &tn) const
    {
        const uint32_t g = band.div(logical), in_band = logical - g * band.divisor;
        const int first_m = (int)g * group_m;
        const bool last = tiles_m - first_m < group_m;
        const uint32_t q = last ? rows_last.div(in_band) : rows_full.div(in_band);
        const uint32_t gm = last ? rows_last.divisor : rows_full.divisor;
        tm = first_m + (int)(in_band - q * gm);
        tn = (int)q;
    }
    __host__ __device__ void locate(int wg, int &tm, int &tn) const { walk(regroup(wg, per_xcd, extra_xcds), tm, tn); }
    // A launch of tiles x slices workgroups in one dimension: the order is slice-major, so an
    // XCD owns whole slices of the reduction -- every tile of a slice, which between them read
    // each row panel of A and each column panel of B of that slice once into the XCD's L2.
    // (With the slice as a second grid dimension an XCD got a few tiles of every slice, and
    // every panel was fetched by several XCDs: 256 x 256 x 8192 in 16 slices read 49 MB for 17.)
    // Returns the tile's position in the walk, which numbers the tiles 0 .. tiles - 1.
    __host__ __device__ int locate_cut(int wg, int &slice, int &tm, int &tn) const
    {
        const uint32_t logical = regroup(wg, cut_per_xcd, cut_extra);
        slice = (int)tiles.div(logical);
        const uint32_t tile = logical - (uint32_t)slice * tiles.divisor;
        walk(tile, tm, tn);
        return (int)tile;
    }
};

// The same walk with general divisions (host side, and the definition the fast form is tested against).
__host__ __device__ inline void map_tile(int wg, int tiles_m, int tiles_n, int group_m, int &tm, int &tn)
{
    const int nt = tiles_m * tiles_n;
    const int q = nt / kXcds, rem = nt % kXcds;
    const int xcd = wg % kXcds, idx = wg / kXcds;
    const int logical = xcd * q + (xcd < rem ? xcd : rem) + idx;
    const int band = group_m * tiles_n;
    const int g = logical / band, in_band = logical % band;
    const int first_m = g * group_m;
    const int gm = (tiles_m - first_m) < group_m ? (tiles_m - first_m) : group_m;
    tm = first_m + in_band % gm;
    tn = in_band / gm;
}

// Static shape of one kernel variant.  B_KMAJOR = true: the B operand reaches LDS as
// [BK][BN] (n contiguous, as a row-major K x N matrix is stored); false: as [BN][BK]
// (k contiguous, as the KRSC filter is stored).
template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_, bool B_KMAJOR_>
struct TileShape {
    static constexpr int BM = BM_, BN = BN_, BK = BK_;
    static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
    static constexpr bool B_KMAJOR = B_KMAJOR_;
    static constexpr int NT = 64 * WAVES_M * WAVES_N;
    static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;  // wave tile
    static constexpr int TM = WTM / 32, TN = WTN / 32;            // 32x32 blocks per wave
    static constexpr int A_LD = BK + 4;                            // floats per LDS row of A
    static constexpr int B_LD = B_KMAJOR ? BN + 8 : BK + 4;        // floats per LDS row of B
    static constexpr int A_STAGE = BM * A_LD;
    static constexpr int B_STAGE = (B_KMAJOR ? BK : BN) * B_LD;
    static constexpr int LDS_FLOATS = 2 * (A_STAGE + B_STAGE);
    static constexpr int A_SLOTS = BM * BK / 4 / NT;  // 16-byte slots per thread and chunk
    static constexpr int B_SLOTS = BK * BN / 4 / NT;
    static_assert(BM % (32 * WAVES_M) == 0 && BN % (32 * WAVES_N) == 0, "wave tiles are 32-multiples");
    static_assert(BK % 8 == 0, "a chunk is consumed in groups of eight k");
    static_assert((BM * BK / 4) % NT == 0 && (BK * BN / 4) % NT == 0, "loads divide evenly");
    static_assert(TN == 1 || TN == 2 || TN == 4, "B fragment is read as 1, 2 or 4 floats");
    static_assert(LDS_FLOATS * 4 <= 160 * 1024, "LDS budget");
};

// The accumulators of one wave and the LDS -> MFMA inner product over one staged chunk.
template <class T>
struct WaveTile {
    f32x16 acc[T::TM][T::TN];

    __device__ inline void clear()
    {
#pragma unroll
        for (int a = 0; a < T::TM; ++a)
#pragma unroll
            for (int b = 0; b < T::TN; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    }

    // as, bs: start of the chunk's A and B stage; wrow / wcol: first row / column of this
    // wave inside the workgroup tile; li = lane % 32, half = lane / 32.
    __device__ inline void consume_chunk(const float *as, const float *bs, int wrow, int wcol,
                                         int li, int half)
    {
#pragma unroll
        for (int u = 0; u < T::BK / 8; ++u) {
            const int kk = 8 * u + 4 * half;
            f32x4 af[T::TM];
#pragma unroll
            for (int a = 0; a < T::TM; ++a)
                af[a] = *reinterpret_cast<const f32x4 *>(as + (wrow + 32 * a + li) * T::A_LD + kk);
            if constexpr (T::B_KMAJOR) {
                // column of block b in this wave is TN*li + b: one vector read serves all blocks
                typename FVec<T::TN>::type bf[4];
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    bf[t] = *reinterpret_cast<const typename FVec<T::TN>::type *>(
                        bs + (kk + t) * T::B_LD + wcol + T::TN * li);
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int a = 0; a < T::TM; ++a)
#pragma unroll
                        for (int b = 0; b < T::TN; ++b)
                            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                                af[a][t], vec_get<T::TN>(bf[t], b), acc[a][b], 0, 0, 0);
            } else {
                // column of block b is 32*b + li; B rows are k-contiguous like A
                f32x4 bf[T::TN];
#pragma unroll
                for (int b = 0; b < T::TN; ++b)
                    bf[b] = *reinterpret_cast<const f32x4 *>(bs + (wcol + 32 * b + li) * T::B_LD + kk);
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int a = 0; a < T::TM; ++a)
#pragma unroll
                        for (int b = 0; b < T::TN; ++b)
                            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[a][t], bf[b][t],
                                                                            acc[a][b], 0, 0, 0);
            }
        }
    }

    // Row (inside the wave tile) of accumulator register v of block row a.
    __device__ static inline int acc_row(int a, int v, int half)
    {
        return 32 * a + 8 * (v >> 2) + 4 * half + (v & 3);
    }
};

}  // namespace lsmi
