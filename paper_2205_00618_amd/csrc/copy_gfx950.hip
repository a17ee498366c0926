// Single-operand contraction (Section 5.2, "Single Operand LoopNest"; the transpositions and
// broadcasts in Section 2.1's list): no reduction index and one input,
//   out[i0,i1,i2,i3] = in[i0*s0 + i1*s1 + i2*s2 + i3*s3],
// out dense row-major.  Permuted strides transpose (NCHW <-> NHWC, a matrix transpose, the
// k-contiguous packing of an int8 B operand), the strides of an enclosing tensor extract a
// sub-tensor, a stride of 0 broadcasts.  Pure data movement, bound by HBM: what matters is
// that both the reads and the writes of a wave are contiguous.  Three kernels:
//   rows      the input's innermost stride is 1: both sides are contiguous along i3; 16-byte
//             accesses when extents, strides and bases allow, element accesses otherwise;
//   transpose another index j has input stride 1: 64 x 64 element tiles (128 x 128 for bytes) of
//             the (ij, i3) plane go through LDS, read along ij, written along i3; 16-byte
//             accesses when extents, strides and bases allow, element or dword ones otherwise;
//   narrow    a transpose one of whose two extents is at most 16 (NCHW <-> NHWC with 3 channels):
//             a 64 x 64 tile would be mostly empty, so a workgroup moves 256 positions of the
//             long index times the whole short one through LDS, reading runs along the
//             input's unit stride and writing runs along the output's;
//   gather    anything else (broadcast along i3, strided slices): one lane per output
//             element, contiguous writes.
#include "common.hpp"

namespace lsmi {
namespace {

struct CopyGeom {
    long long d[4], s[4];
    long long total;  // d0*d1*d2*d3
};

template <class E, int VEC>
struct Pack;
template <> struct Pack<float, 4> { typedef float type __attribute__((ext_vector_type(4))); };
template <> struct Pack<signed char, 16> { typedef int type __attribute__((ext_vector_type(4))); };

// rows, vectorised: one lane per VEC consecutive i3
template <class E, int VEC>
__global__ __launch_bounds__(256) void copy_rows_vec_kernel(CopyGeom g, const E *__restrict__ in, E *__restrict__ out)
{
    typedef typename Pack<E, VEC>::type pack;
    const long long item = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long per_row = g.d[3] / VEC;
    if (item >= g.total / VEC) return;
    const long long i3 = (item % per_row) * VEC;
    long long rest = item / per_row;
    const long long i2 = rest % g.d[2];
    rest /= g.d[2];
    const long long i1 = rest % g.d[1], i0 = rest / g.d[1];
    const pack v = *reinterpret_cast<const pack *>(in + i0 * g.s[0] + i1 * g.s[1] + i2 * g.s[2] + i3);
    *reinterpret_cast<pack *>(out + item * VEC) = v;
}

// gather (also rows without alignment): one lane per output element
template <class E>
__global__ __launch_bounds__(256) void copy_gather_kernel(CopyGeom g, const E *__restrict__ in, E *__restrict__ out)
{
    const long long item = (long long)blockIdx.x * 256 + threadIdx.x;
    if (item >= g.total) return;
    const long long i3 = item % g.d[3];
    long long rest = item / g.d[3];
    const long long i2 = rest % g.d[2];
    rest /= g.d[2];
    const long long i1 = rest % g.d[1], i0 = rest / g.d[1];
    out[item] = in[i0 * g.s[0] + i1 * g.s[1] + i2 * g.s[2] + i3 * g.s[3]];
}

// Which tile of the (iJ, i3) plane a workgroup moves; `t` is left holding the index over the
// other two extents.  Consecutive workgroups step along both tile indices at once, so that
// the workgroups in flight together read from many different columns of the input and write
// to many different columns of the output: with a row-by-row order one of the two sides
// marches down a single column, and on a matrix whose pitch is a power of two that column
// lives in a few memory channels.
__device__ inline void take_tile(long long &t, long long tiles_j, long long tiles_3, long long &tj, long long &t3)
{
    tj = t % tiles_j;
    t /= tiles_j;
    t3 = (t % tiles_3 + tj) % tiles_3;
    t /= tiles_3;
}

// transpose: index J (0..2) has input stride 1.  A workgroup moves one 64 x 64 tile of the
// (iJ, i3) plane for fixed values of the other two indices: 256 lanes read 64 rows (fixed
// i3) of 64 consecutive iJ, store them to LDS with one element of row padding, and write 64
// rows (fixed iJ) of 64 consecutive i3.
template <class E, int J>
__global__ __launch_bounds__(256) void copy_transpose_kernel(CopyGeom g, const E *__restrict__ in, E *__restrict__ out,
                                                             long long tiles_j, long long tiles_3)
{
    __shared__ E tile[64][64 + 4 / sizeof(E)];
    constexpr int A = J == 0 ? 1 : 0, B = J == 2 ? 1 : 2;  // the two other indices, A before B
    long long t = blockIdx.x, tj, t3;
    take_tile(t, tiles_j, tiles_3, tj, t3);
    const long long ib = t % g.d[B], ia = t / g.d[B];
    const long long j0 = tj * 64, c0 = t3 * 64;
    const int lane_x = threadIdx.x & 63, lane_y = threadIdx.x >> 6;
    const long long in_base = ia * g.s[A] + ib * g.s[B];
    // read: row r of the tile is i3 = c0 + r, lane_x runs along iJ (contiguous in the input);
    // a lane's sixteen loads are all requested before the first is stored (64 KiB in flight per CU)
    E held[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const long long i3 = c0 + lane_y + 4 * k, ij = j0 + lane_x;
        held[k] = (i3 < g.d[3] && ij < g.d[J]) ? in[in_base + ij + i3 * g.s[3]] : E(0);
    }
#pragma unroll
    for (int k = 0; k < 16; ++k) tile[lane_y + 4 * k][lane_x] = held[k];
    __syncthreads();
    // write: row r is iJ = j0 + r, lane_x runs along i3 (contiguous in the output)
    long long idx[4];
    idx[A] = ia;
    idx[B] = ib;
#pragma unroll 4
    for (int r = lane_y; r < 64; r += 4) {
        const long long ij = j0 + r, i3 = c0 + lane_x;
        if (ij < g.d[J] && i3 < g.d[3]) {
            idx[J] = ij;
            out[((idx[0] * g.d[1] + idx[1]) * g.d[2] + idx[2]) * g.d[3] + i3] = tile[lane_x][r];
        }
    }
}

// narrow: the plane (iJ, i3) with one short extent S <= 16.  The tile is 256 positions of the
// long index by S, kept in LDS in the order of the side that is contiguous as a whole: element
// (l, c) at l * S + c (one more word every 32 keeps the strided side off a single bank).
//   SHORT3 (i3 is the short index, J == 2 the long one with input stride 1): reads run along
//   iJ for each i3, and the tile is one contiguous run of the dense output.
//   !SHORT3 (iJ is the short index, stride 1 in the input, i3 the long one): the tile is read
//   as it lies in the input (contiguous when the input is dense in these two indices) and
//   written as S runs along i3.
template <class E, int J, bool SHORT3>
__global__ __launch_bounds__(256) void copy_narrow_kernel(CopyGeom g, const E *__restrict__ in, E *__restrict__ out,
                                                          long long tiles)
{
    __shared__ E tile[256 * 16 + 256 * 16 / 32];
    auto slot = [](int idx) { return idx + (idx >> 5); };
    constexpr int A = J == 0 ? 1 : 0, B = J == 2 ? 1 : 2;  // the two other indices, A before B
    long long t = blockIdx.x;
    const long long tl = t % tiles;
    t /= tiles;
    const long long ib = t % g.d[B], ia = t / g.d[B];
    const long long in_base = ia * g.s[A] + ib * g.s[B];
    const int lane = threadIdx.x;
    long long idx[4];
    idx[A] = ia;
    idx[B] = ib;
    if constexpr (SHORT3) {
        static_assert(J == 2 || !SHORT3, "the long index is the one next to i3");
        const int S = (int)g.d[3];
        const long long j0 = tl * 256;
        const int count = (int)(g.d[2] - j0 < 256 ? g.d[2] - j0 : 256);
        if (lane < count)
            for (int c = 0; c < S; ++c) tile[slot(lane * S + c)] = in[in_base + j0 + lane + c * g.s[3]];
        __syncthreads();
        E *const dst = out + (((idx[0] * g.d[1] + idx[1]) * g.d[2]) + j0) * S;
        for (int e = lane; e < count * S; e += 256) dst[e] = tile[slot(e)];
    } else {
        const int S = (int)g.d[J];
        const long long c0 = tl * 256;
        const int count = (int)(g.d[3] - c0 < 256 ? g.d[3] - c0 : 256);
        for (int e = lane; e < count * S; e += 256) {
            const int l = e / S, j = e - l * S;
            tile[slot(e)] = in[in_base + (c0 + l) * g.s[3] + j];
        }
        __syncthreads();
        if (lane < count)
            for (int j = 0; j < S; ++j) {
                idx[J] = j;
                out[((idx[0] * g.d[1] + idx[1]) * g.d[2] + idx[2]) * g.d[3] + c0 + lane] = tile[slot(lane * S + j)];
            }
    }
}

// narrow, fp32, short extent up to 4 (RGB and RGBA images), 16-byte accesses on both sides: the
// tile is 1024 positions of the long index; a lane moves four consecutive positions of a run.
// Needs the long extent a multiple of 4 and every address a lane forms a multiple of 16 bytes;
// !SHORT3 also an input that is dense in the two indices (s3 == S), so that the tile is one run.
template <int J, bool SHORT3>
__global__ __launch_bounds__(256) void copy_narrow_f32_wide_kernel(CopyGeom g, const float *__restrict__ in,
                                                                   float *__restrict__ out, long long tiles)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    __shared__ float tile[1024 * 4 + 1024 * 4 / 32];
    auto slot = [](int idx) { return idx + (idx >> 5); };
    constexpr int A = J == 0 ? 1 : 0, B = J == 2 ? 1 : 2;
    long long t = blockIdx.x;
    const long long tl = t % tiles;
    t /= tiles;
    const long long ib = t % g.d[B], ia = t / g.d[B];
    const long long in_base = ia * g.s[A] + ib * g.s[B];
    const int lane = threadIdx.x;
    long long idx[4];
    idx[A] = ia;
    idx[B] = ib;
    if constexpr (SHORT3) {
        const int S = (int)g.d[3];
        const long long j0 = tl * 1024;
        const int count = (int)(g.d[2] - j0 < 1024 ? g.d[2] - j0 : 1024);  // a multiple of 4
        if (4 * lane < count)
            for (int c = 0; c < S; ++c) {
                const f4 v = *reinterpret_cast<const f4 *>(in + in_base + j0 + 4 * lane + c * g.s[3]);
#pragma unroll
                for (int u = 0; u < 4; ++u) tile[slot((4 * lane + u) * S + c)] = v[u];
            }
        __syncthreads();
        float *const dst = out + (((idx[0] * g.d[1] + idx[1]) * g.d[2]) + j0) * S;
        for (int e = lane; 4 * e < count * S; e += 256) {
            f4 w;
#pragma unroll
            for (int u = 0; u < 4; ++u) w[u] = tile[slot(4 * e + u)];
            *reinterpret_cast<f4 *>(dst + 4 * e) = w;
        }
    } else {
        const int S = (int)g.d[J];
        const long long c0 = tl * 1024;
        const int count = (int)(g.d[3] - c0 < 1024 ? g.d[3] - c0 : 1024);  // a multiple of 4
        const float *const src = in + in_base + c0 * S;
        for (int e = lane; 4 * e < count * S; e += 256) {
            const f4 v = *reinterpret_cast<const f4 *>(src + 4 * e);
#pragma unroll
            for (int u = 0; u < 4; ++u) tile[slot(4 * e + u)] = v[u];
        }
        __syncthreads();
        if (4 * lane < count)
            for (int j = 0; j < S; ++j) {
                idx[J] = j;
                f4 w;
#pragma unroll
                for (int u = 0; u < 4; ++u) w[u] = tile[slot((4 * lane + u) * S + j)];
                *reinterpret_cast<f4 *>(out + ((idx[0] * g.d[1] + idx[1]) * g.d[2] + idx[2]) * g.d[3] + c0 + 4 * lane) = w;
            }
    }
}

// The same for 1-byte elements with 128 x 128 tiles: a lane moves four consecutive bytes at
// a time on both sides (whole dwords when `in_dwords` / `out_dwords` say the addresses are
// 4-byte aligned), so that a wave still touches 128 contiguous bytes per row.
template <int J>
__global__ __launch_bounds__(256) void copy_transpose_bytes_kernel(CopyGeom g, const signed char *__restrict__ in,
                                                                   signed char *__restrict__ out, long long tiles_j,
                                                                   long long tiles_3, bool in_dwords, bool out_dwords)
{
    __shared__ __attribute__((aligned(4))) unsigned char tile[128][128 + 4];
    constexpr int A = J == 0 ? 1 : 0, B = J == 2 ? 1 : 2;
    long long t = blockIdx.x, tj, t3;
    take_tile(t, tiles_j, tiles_3, tj, t3);
    const long long ib = t % g.d[B], ia = t / g.d[B];
    const long long j0 = tj * 128, c0 = t3 * 128;
    const int lx = threadIdx.x & 31, ly = threadIdx.x >> 5;
    const long long in_base = ia * g.s[A] + ib * g.s[B];
    // read: row r of the tile is i3 = c0 + r, the lane covers iJ = j0 + 4 lx .. + 3
    for (int r = ly; r < 128; r += 8) {
        const long long i3 = c0 + r, ij = j0 + 4 * lx;
        if (i3 >= g.d[3] || ij >= g.d[J]) continue;
        const signed char *src = in + in_base + ij + i3 * g.s[3];
        if (in_dwords && ij + 3 < g.d[J]) {
            *reinterpret_cast<unsigned *>(&tile[r][4 * lx]) = *reinterpret_cast<const unsigned *>(src);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (ij + e < g.d[J]) tile[r][4 * lx + e] = (unsigned char)src[e];
        }
    }
    __syncthreads();
    // write: row r is iJ = j0 + r, the lane covers i3 = c0 + 4 lx .. + 3
    long long idx[4];
    idx[A] = ia;
    idx[B] = ib;
    for (int r = ly; r < 128; r += 8) {
        const long long ij = j0 + r, i3 = c0 + 4 * lx;
        if (ij >= g.d[J] || i3 >= g.d[3]) continue;
        idx[J] = ij;
        signed char *dst = out + ((idx[0] * g.d[1] + idx[1]) * g.d[2] + idx[2]) * g.d[3] + i3;
        if (out_dwords && i3 + 3 < g.d[3]) {
            const unsigned w = (unsigned)tile[4 * lx][r] | ((unsigned)tile[4 * lx + 1][r] << 8) |
                               ((unsigned)tile[4 * lx + 2][r] << 16) | ((unsigned)tile[4 * lx + 3][r] << 24);
            *reinterpret_cast<unsigned *>(dst) = w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (i3 + e < g.d[3]) dst[e] = (signed char)tile[4 * lx + e][r];
        }
    }
}

// The tiled transposes again for operands whose extents, strides and bases are multiples of
// 16 bytes: every global access is 16 bytes per lane, four of them in flight per lane on the
// reading side (64 KiB per compute unit at full occupancy, what the HBM latency asks for).
// fp32: lanes load four consecutive iJ of four rows, scatter them to the padded tile, gather
// four consecutive i3 of one output row back (both LDS patterns touch 64 different banks).
template <int J>
__global__ __launch_bounds__(256) void copy_transpose_f32_wide_kernel(CopyGeom g, const float *__restrict__ in,
                                                                      float *__restrict__ out, long long tiles_j,
                                                                      long long tiles_3)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    __shared__ float tile[64][65];
    constexpr int A = J == 0 ? 1 : 0, B = J == 2 ? 1 : 2;
    long long t = blockIdx.x, tj, t3;
    take_tile(t, tiles_j, tiles_3, tj, t3);
    const long long ib = t % g.d[B], ia = t / g.d[B];
    const long long j0 = tj * 64, c0 = t3 * 64;
    const int cx = threadIdx.x & 15, ry = threadIdx.x >> 4;
    const long long in_base = ia * g.s[A] + ib * g.s[B];
    f4 v[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const long long i3 = c0 + ry + 16 * p, ij = j0 + 4 * cx;
        v[p] = f4{0.f, 0.f, 0.f, 0.f};
        if (i3 < g.d[3] && ij < g.d[J]) v[p] = *reinterpret_cast<const f4 *>(in + in_base + ij + i3 * g.s[3]);
    }
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int e = 0; e < 4; ++e) tile[ry + 16 * p][4 * cx + e] = v[p][e];
    __syncthreads();
    long long idx[4];
    idx[A] = ia;
    idx[B] = ib;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int r = ry + 16 * p;
        const long long ij = j0 + r, i3 = c0 + 4 * cx;
        if (ij < g.d[J] && i3 < g.d[3]) {
            const f4 w = {tile[4 * cx][r], tile[4 * cx + 1][r], tile[4 * cx + 2][r], tile[4 * cx + 3][r]};
            idx[J] = ij;
            *reinterpret_cast<f4 *>(out + ((idx[0] * g.d[1] + idx[1]) * g.d[2] + idx[2]) * g.d[3] + i3) = w;
        }
    }
}

// bytes: a lane loads 16 consecutive iJ of four consecutive i3, transposes each 4 x 4 byte
// block in registers (byte permutes) and stores dwords that hold four consecutive i3 of one
// iJ; the tile in LDS is therefore already the output's layout and is read back 16 bytes a lane.
template <int J>
__global__ __launch_bounds__(256) void copy_transpose_bytes_wide_kernel(CopyGeom g, const signed char *__restrict__ in,
                                                                        signed char *__restrict__ out,
                                                                        long long tiles_j, long long tiles_3)
{
    typedef unsigned u4 __attribute__((ext_vector_type(4)));
    __shared__ __attribute__((aligned(8))) unsigned tile[128][34];  // [iJ][i3 / 4], rows of 136 bytes
    constexpr int A = J == 0 ? 1 : 0, B = J == 2 ? 1 : 2;
    long long t = blockIdx.x, tj, t3;
    take_tile(t, tiles_j, tiles_3, tj, t3);
    const long long ib = t % g.d[B], ia = t / g.d[B];
    const long long j0 = tj * 128, c0 = t3 * 128;
    // eight neighbouring lanes cover the 128 bytes of one input row: a load instruction of a
    // wave then touches 8 whole rows of the tile rather than 32 bytes of each of 32 rows
    const int bq = threadIdx.x & 7, a = threadIdx.x >> 3;
    const long long in_base = ia * g.s[A] + ib * g.s[B];
    u4 row[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const long long i3 = c0 + 4 * a + e, ij = j0 + 16 * bq;
        row[e] = u4{0u, 0u, 0u, 0u};
        if (i3 < g.d[3] && ij < g.d[J]) row[e] = *reinterpret_cast<const u4 *>(in + in_base + ij + i3 * g.s[3]);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        // bytes 0..3 of the selector's source pair are the second operand, 4..7 the first
        const unsigned x_lo = __builtin_amdgcn_perm(row[1][q], row[0][q], 0x05010400u);
        const unsigned x_hi = __builtin_amdgcn_perm(row[1][q], row[0][q], 0x07030602u);
        const unsigned y_lo = __builtin_amdgcn_perm(row[3][q], row[2][q], 0x05010400u);
        const unsigned y_hi = __builtin_amdgcn_perm(row[3][q], row[2][q], 0x07030602u);
        tile[16 * bq + 4 * q + 0][a] = __builtin_amdgcn_perm(y_lo, x_lo, 0x05040100u);
        tile[16 * bq + 4 * q + 1][a] = __builtin_amdgcn_perm(y_lo, x_lo, 0x07060302u);
        tile[16 * bq + 4 * q + 2][a] = __builtin_amdgcn_perm(y_hi, x_hi, 0x05040100u);
        tile[16 * bq + 4 * q + 3][a] = __builtin_amdgcn_perm(y_hi, x_hi, 0x07060302u);
    }
    __syncthreads();
    long long idx[4];
    idx[A] = ia;
    idx[B] = ib;
    const int c = threadIdx.x & 7, rr = threadIdx.x >> 3;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int r = rr + 32 * p;
        const long long ij = j0 + r, i3 = c0 + 16 * c;
        if (ij < g.d[J] && i3 < g.d[3]) {
            const u4 w = {tile[r][4 * c], tile[r][4 * c + 1], tile[r][4 * c + 2], tile[r][4 * c + 3]};
            idx[J] = ij;
            *reinterpret_cast<u4 *>(out + ((idx[0] * g.d[1] + idx[1]) * g.d[2] + idx[2]) * g.d[3] + i3) = w;
        }
    }
}

template <class E, int VEC>
int launch_copy_typed(const CopyGeom &g, const E *in, E *out, ThreadState &st, const char *const names[6])
{
    auto blocks_for = [](long long items) { return (unsigned)((items + 255) / 256); };
    // a unit-stride index with more than one element; i3 first
    int unit = -1;
    for (int a : {3, 2, 1, 0})
        if (g.d[a] > 1 && g.s[a] == 1) {
            unit = a;
            break;
        }
    if (g.d[3] == 1 && unit < 0) unit = 3;
    if (unit == 3 || g.d[3] == 1) {
        const uintptr_t mask = VEC * sizeof(E) - 1;
        const bool vec = g.s[3] == 1 && g.d[3] % VEC == 0 && (((uintptr_t)in | (uintptr_t)out) & mask) == 0 &&
                         (g.d[2] == 1 || g.s[2] % VEC == 0) && (g.d[1] == 1 || g.s[1] % VEC == 0) &&
                         (g.d[0] == 1 || g.s[0] % VEC == 0);
        if (vec) {
            copy_rows_vec_kernel<E, VEC><<<dim3(blocks_for(g.total / VEC)), dim3(256), 0, st.stream>>>(g, in, out);
            st.last_variant = names[0];
        } else {
            copy_gather_kernel<E><<<dim3(blocks_for(g.total)), dim3(256), 0, st.stream>>>(g, in, out);
            st.last_variant = names[2];
        }
        return check_launch();
    }
    // one of the two extents of the transposed plane at most 16, the other long
    // (16-byte accesses: fp32, a short extent of at most 4, every lane address a multiple of 16 bytes)
    auto others_aligned = [&](int skip) {
        for (int a = 0; a < 3; ++a)
            if (a != skip && g.d[a] > 1 && g.s[a] % 4 != 0) return false;
        return (((uintptr_t)in | (uintptr_t)out) & 15) == 0;
    };
    if (unit == 2 && g.d[3] <= 16 && g.d[2] >= 64) {
        if constexpr (sizeof(E) == 4) {
            const long long tiles = (g.d[2] + 1023) / 1024, blocks = tiles * g.d[0] * g.d[1];
            if (g.d[3] <= 4 && g.d[2] % 4 == 0 && g.s[3] % 4 == 0 && others_aligned(2) && blocks <= INT32_MAX) {
                copy_narrow_f32_wide_kernel<2, true><<<dim3((unsigned)blocks), dim3(256), 0, st.stream>>>(g, in, out, tiles);
                st.last_variant = names[5];
                return check_launch();
            }
        }
        const long long tiles = (g.d[2] + 255) / 256, blocks = tiles * g.d[0] * g.d[1];
        if (blocks <= INT32_MAX) {
            copy_narrow_kernel<E, 2, true><<<dim3((unsigned)blocks), dim3(256), 0, st.stream>>>(g, in, out, tiles);
            st.last_variant = names[4];
            return check_launch();
        }
    }
    if (unit >= 0 && g.d[unit] <= 16 && g.d[3] >= 64) {
        long long others = 1;
        for (int a = 0; a < 3; ++a)
            if (a != unit) others *= g.d[a];
        if constexpr (sizeof(E) == 4) {
            const long long tiles = (g.d[3] + 1023) / 1024, blocks = tiles * others;
            if (g.d[unit] <= 4 && g.d[3] % 4 == 0 && g.s[3] == g.d[unit] && others_aligned(unit) && blocks <= INT32_MAX) {
                const dim3 grid((unsigned)blocks), block(256);
                if (unit == 0) copy_narrow_f32_wide_kernel<0, false><<<grid, block, 0, st.stream>>>(g, in, out, tiles);
                else if (unit == 1) copy_narrow_f32_wide_kernel<1, false><<<grid, block, 0, st.stream>>>(g, in, out, tiles);
                else copy_narrow_f32_wide_kernel<2, false><<<grid, block, 0, st.stream>>>(g, in, out, tiles);
                st.last_variant = names[5];
                return check_launch();
            }
        }
        const long long tiles = (g.d[3] + 255) / 256, blocks = tiles * others;
        if (blocks <= INT32_MAX) {
            const dim3 grid((unsigned)blocks), block(256);
            if (unit == 0) copy_narrow_kernel<E, 0, false><<<grid, block, 0, st.stream>>>(g, in, out, tiles);
            else if (unit == 1) copy_narrow_kernel<E, 1, false><<<grid, block, 0, st.stream>>>(g, in, out, tiles);
            else copy_narrow_kernel<E, 2, false><<<grid, block, 0, st.stream>>>(g, in, out, tiles);
            st.last_variant = names[4];
            return check_launch();
        }
    }
    if (unit >= 0 && g.d[unit] >= 8 && g.d[3] >= 8) {
        constexpr int TILE = sizeof(E) == 1 ? 128 : 64;
        const long long tiles_j = (g.d[unit] + TILE - 1) / TILE, tiles_3 = (g.d[3] + TILE - 1) / TILE;
        long long others = 1;
        for (int a = 0; a < 3; ++a)
            if (a != unit) others *= g.d[a];
        const long long blocks = others * tiles_j * tiles_3;
        if (blocks <= INT32_MAX) {
            const dim3 grid((unsigned)blocks), block(256);
            // 16-byte accesses on both sides: every address a lane forms is a multiple of 16 bytes
            bool wide = (((uintptr_t)in | (uintptr_t)out) & 15) == 0 && g.d[unit] % VEC == 0 && g.d[3] % VEC == 0 &&
                        g.s[3] % VEC == 0;
            for (int a = 0; a < 3; ++a)
                if (a != unit && g.d[a] > 1 && g.s[a] % VEC != 0) wide = false;
            if (wide) {
                if constexpr (sizeof(E) == 1) {
                    if (unit == 0) copy_transpose_bytes_wide_kernel<0><<<grid, block, 0, st.stream>>>(g, in, out, tiles_j, tiles_3);
                    else if (unit == 1) copy_transpose_bytes_wide_kernel<1><<<grid, block, 0, st.stream>>>(g, in, out, tiles_j, tiles_3);
                    else copy_transpose_bytes_wide_kernel<2><<<grid, block, 0, st.stream>>>(g, in, out, tiles_j, tiles_3);
                } else {
                    if (unit == 0) copy_transpose_f32_wide_kernel<0><<<grid, block, 0, st.stream>>>(g, in, out, tiles_j, tiles_3);
                    else if (unit == 1) copy_transpose_f32_wide_kernel<1><<<grid, block, 0, st.stream>>>(g, in, out, tiles_j, tiles_3);
                    else copy_transpose_f32_wide_kernel<2><<<grid, block, 0, st.stream>>>(g, in, out, tiles_j, tiles_3);
                }
                st.last_variant = names[3];
                return check_launch();
            }
            if constexpr (sizeof(E) == 1) {
                // dword accesses need every address a lane forms to be a multiple of four
                bool in_dw = ((uintptr_t)in & 3) == 0 && (g.d[3] == 1 || g.s[3] % 4 == 0);
                for (int a = 0; a < 3; ++a)
                    if (a != unit && g.d[a] > 1 && g.s[a] % 4 != 0) in_dw = false;
                const bool out_dw = ((uintptr_t)out & 3) == 0 && g.d[3] % 4 == 0;
                if (unit == 0)
                    copy_transpose_bytes_kernel<0><<<grid, block, 0, st.stream>>>(g, in, out, tiles_j, tiles_3, in_dw, out_dw);
                else if (unit == 1)
                    copy_transpose_bytes_kernel<1><<<grid, block, 0, st.stream>>>(g, in, out, tiles_j, tiles_3, in_dw, out_dw);
                else
                    copy_transpose_bytes_kernel<2><<<grid, block, 0, st.stream>>>(g, in, out, tiles_j, tiles_3, in_dw, out_dw);
                st.last_variant = names[1];
                return check_launch();
            }
            if (unit == 0) copy_transpose_kernel<E, 0><<<grid, block, 0, st.stream>>>(g, in, out, tiles_j, tiles_3);
            else if (unit == 1) copy_transpose_kernel<E, 1><<<grid, block, 0, st.stream>>>(g, in, out, tiles_j, tiles_3);
            else copy_transpose_kernel<E, 2><<<grid, block, 0, st.stream>>>(g, in, out, tiles_j, tiles_3);
            st.last_variant = names[1];
            return check_launch();
        }
    }
    copy_gather_kernel<E><<<dim3(blocks_for(g.total)), dim3(256), 0, st.stream>>>(g, in, out);
    st.last_variant = names[2];
    return check_launch();
}

const char *const kCopyNamesF32[6] = {"copy_f32_rows_vec4", "copy_f32_transpose_64x64", "copy_f32_gather",
                                      "copy_f32_transpose_64x64_vec4", "copy_f32_narrow_256", "copy_f32_narrow_1024_vec4"};
const char *const kCopyNamesS8[6] = {"copy_s8_rows_vec16", "copy_s8_transpose_128x128", "copy_s8_gather",
                                     "copy_s8_transpose_128x128_vec16", "copy_s8_narrow_256", ""};

}  // namespace

int launch_tensor_copy(int esize, const int64_t d[4], const int64_t s[4], const void *in, void *out)
{
    // The output is dense, so two neighbouring indices whose input strides nest (s[a] =
    // d[a+1] * s[a+1]) are one index, and an extent of 1 is none: NCHW -> NHWC becomes the
    // transpose of H*W x C planes, a dense tensor one long row.  Fewer, longer indices give
    // the tiled kernels full tiles and the row kernel long rows.
    CopyGeom g;
    int n = 0;
    g.total = 1;
    for (int a = 0; a < 4; ++a) {
        g.total *= d[a];
        if (d[a] == 1) continue;
        if (n > 0 && g.s[n - 1] == d[a] * s[a]) {
            g.d[n - 1] *= d[a];
            g.s[n - 1] = s[a];
        } else {
            g.d[n] = d[a];
            g.s[n] = s[a];
            ++n;
        }
    }
    for (int a = n - 1, b = 3; b >= 0; --a, --b) {  // right-align, pad with extent 1 in front
        g.d[b] = a >= 0 ? g.d[a] : 1;
        g.s[b] = a >= 0 ? g.s[a] : 0;
    }
    ThreadState &st = tls();
    if (esize == 4)
        return launch_copy_typed<float, 4>(g, static_cast<const float *>(in), static_cast<float *>(out), st,
                                           kCopyNamesF32);
    return launch_copy_typed<signed char, 16>(g, static_cast<const signed char *>(in),
                                              static_cast<signed char *>(out), st, kCopyNamesS8);
}

}  // namespace lsmi
