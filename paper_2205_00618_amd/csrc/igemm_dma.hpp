// Signed 8-bit GEMM for aligned shapes (gfx950): both operand tiles stream global -> LDS
// with direct-to-LDS loads into a ring of chunk buffers, as in the aligned fp32 kernel, and
// the n-contiguous B operand is turned into the k-contiguous MFMA operand by the LDS
// transpose read DS_READ_B64_TR_B8 instead of a transpose in registers.
//
// V_MFMA_I32_32X32X32_I8 wants from lane l sixteen consecutive-k bytes of A row l%32 and of
// B column l%32, lanes 0..31 the first sixteen k of a 32-k group, lanes 32..63 the second.
//
//   A (k-contiguous in memory): tile rows are BK = 128 (or 64) bytes; the 16-byte k-groups
//     of row r sit at slot g ^ ((r >> 1) & 7) (g ^ ((r >> 2) & 3) for 64-byte rows).  A
//     16-byte read is served sixteen lanes at a time; with these slots the sixteen
//     consecutive rows of such a group cover all 64 banks once (g ^ (r & 7) made rows r and
//     r + 8 collide: half of the LDS cycles were bank conflicts).  One ds_read_b128 per
//     32x32x32 block operand.
//   B (n-contiguous): the tile is stored as it is in memory, [k][n] bytes, rows of 128 bytes
//     (BN = 128), the 16-byte n-groups of row k at slot g ^ (k & 7).  The transpose read
//     works on groups of 16 lanes: lane j of a group supplies the address of 8 bytes, and
//     lane i receives byte i%8 of the rows supplied by lanes i/8, i/8 + 2, ..., i/8 + 14
//     (checked on the hardware).  With lane j pointing at row k0 + j/2, bytes 8*(j&1)..+7
//     of a 16-byte n-group, lane i receives column i of that group for k0..k0+7: eight
//     consecutive k of its own column.  Two such reads give the sixteen bytes of an operand.
//
// Sums are exact and wrap modulo 2^32; slices of a split reduction are combined with
// integer atomic adds, so every dispatch gives the same bits.
#pragma once

#include <type_traits>

#include "sgemm_dma.hpp"

namespace lsmi {

typedef int i32x2v __attribute__((ext_vector_type(2)));
typedef int i32x16v __attribute__((ext_vector_type(16)));

// B_KMAJOR: the second operand is given transposed (N x K, k-contiguous like A); its tile is
// then staged and read exactly like A's, one 16-byte read per block operand.
//
// EDGE: M, N and K need not be multiples of the tile.  The loads go through raw buffer
// descriptors, and a lane whose 16 bytes lie in a row past M, a column group past N or a
// k-group past K passes an out-of-range offset and gets zeros (as in the fp32 kernel);
// the epilogue tests every element.  Needs 16-byte aligned rows (bases and row pitches
// multiples of 16) and K a multiple of 16: a 16-byte group never straddles the end of a row;
// the group of B that holds column N - 1 is loaded whole, its columns past N feed accumulator
// columns that are never stored.
//
// DWORD (an EDGE form): every load instruction moves 4 bytes per lane instead of 16, so bases,
// row pitches and K need only be multiples of 4 (a dense B with N = 1000, K = 1000): the same
// image of the chunk in LDS from four times the load instructions, and the test against K is
// per 4-byte group.
template <int BM_, int WAVES_M_, int WAVES_N_, int NSTAGE_, int BK_ = 128, bool B_KMAJOR_ = false,
          bool EDGE_ = false, bool DWORD_ = false>
struct IDmaShape {
    static constexpr bool B_KMAJOR = B_KMAJOR_, EDGE = EDGE_, DWORD = DWORD_;
    static constexpr int BM = BM_, BN = 128, BK = BK_, NSTAGE = NSTAGE_;
    static constexpr int A_GROUPS = BK / 16;            // 16-byte k-groups per A row
    static constexpr int A_ROWS_PER_INSTR = 1024 / BK;  // A rows one load instruction moves
    static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, NWAVES = WAVES_M * WAVES_N;
    static constexpr int NT = 64 * NWAVES;
    static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    static constexpr int TM = WTM / 32, TN = WTN / 32;
    static constexpr int A_BYTES = BM * BK, B_BYTES = BK * BN;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;
    static constexpr int INSTR_BYTES = DWORD ? 256 : 1024;  // LDS bytes one load instruction fills
    static constexpr int A_PER_WAVE = A_BYTES / INSTR_BYTES / NWAVES;  // load instructions per wave and chunk
    static constexpr int B_PER_WAVE = B_BYTES / INSTR_BYTES / NWAVES;
    static constexpr int LOADS = A_PER_WAVE + B_PER_WAVE;
    static_assert(!DWORD || EDGE, "the 4-byte loads are a form of the buffer-load kernel");
    static constexpr int WGS_PER_CU = (160 * 1024) / LDS_BYTES < 4 ? (160 * 1024) / LDS_BYTES : 4;
    static constexpr int WAVES_PER_SIMD = (WGS_PER_CU * NWAVES + 3) / 4;
    static_assert(A_BYTES % (INSTR_BYTES * NWAVES) == 0 && B_BYTES % (INSTR_BYTES * NWAVES) == 0, "even DMA split");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && TM >= 1 && TN >= 1, "wave tiles are 32-multiples");
    static_assert(BK == 64 || BK == 128, "chunk depth in bytes");
    static_assert(NSTAGE >= 2 && NSTAGE <= 6 && LOADS * (NSTAGE - 2) <= 63, "ring depth");

    // slot of A k-group g in row r: the 16-byte reads of consecutive rows spread over all banks
    __host__ __device__ static constexpr int a_slot(int g, int r)
    {
        return BK == 128 ? (g ^ ((r >> 1) & 7)) : (g ^ ((r >> 2) & 3));
    }
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

template <bool DWORD>
__device__ __forceinline__ void idma_load(i32x4 buffer, uint32_t voff, uint32_t lds_addr)
{
    if constexpr (DWORD) dma4_buf(buffer, voff, lds_addr); else dma16_buf(buffer, voff, lds_addr);
}

template <class T>
__global__ __launch_bounds__(T::NT)
__attribute__((amdgpu_waves_per_eu(1, T::WAVES_PER_SIMD))) void igemm_dma_kernel(
    int M, int N, int K, const int8_t *__restrict__ A, int64_t lda, const int8_t *__restrict__ B, int64_t ldb,
    int32_t *__restrict__ C, int64_t ldc, TileMap tmap, int chunks_per_slice)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char ilds[];
    const uint32_t lds_base = (uint32_t)(uintptr_t)ilds;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, half = lane >> 5;
    const int wrow = (wave / T::WAVES_N) * T::WTM;
    const int wcol = (wave % T::WAVES_N) * T::WTN;

    int tm, tn;
    tmap.locate(blockIdx.x, tm, tn);
    const int m0 = tm * T::BM, n0 = tn * T::BN;
    const bool sliced = gridDim.y > 1;
    const int first = (int)blockIdx.y * chunks_per_slice;
    const int nk = min((T::EDGE ? (K + T::BK - 1) / T::BK : K / T::BK) - first, chunks_per_slice);

    // ---- DMA sources: one instruction moves 1 KiB, i.e. 1024/BK rows of A or eight 128-byte
    // rows of B; lane -> (row, slot) ----
    const int r8 = lane >> 3, slot = lane & 7;
    uint32_t voff_a[T::A_PER_WAVE], voff_b[T::B_PER_WAVE];
    // EDGE: first k (relative to the chunk) of the 16 bytes a lane moves, for the test against
    // K in the last chunk; rows past M and columns past N are out of range from the start
    int a_k[T::EDGE ? T::A_PER_WAVE : 1], b_k[T::EDGE ? T::B_PER_WAVE : 1];
    // a k-contiguous operand (A, a k-major B): instruction `idx` of the tile -> this lane's row
    // and the offset of its bytes inside the row's chunk
    auto k_major = [&](int idx, int &row, int &koff) __attribute__((always_inline)) {
        if constexpr (T::DWORD) {
            constexpr int LANES_PER_ROW = T::BK / 4;
            row = idx * (256 / T::BK) + lane / LANES_PER_ROW;
            const int u = lane % LANES_PER_ROW;  // 4-byte unit inside the row's image: slot u / 4, word u % 4
            koff = T::a_slot(u >> 2, row) * 16 + (u & 3) * 4;
        } else {
            row = idx * T::A_ROWS_PER_INSTR + lane / T::A_GROUPS;
            koff = T::a_slot(lane % T::A_GROUPS, row) * 16;  // the group g with a_slot(g, row) == lane's slot
        }
    };
    // (compile-time indices: the 4-byte form's 16 to 32 entries per array stay in registers)
    static_for<T::A_PER_WAVE>([&](auto q_c) {
        constexpr int q = decltype(q_c)::value;
        int row, koff;
        k_major(wave * T::A_PER_WAVE + q, row, koff);
        voff_a[q] = (uint32_t)((int64_t)row * lda + koff);
        if constexpr (T::EDGE) {
            a_k[q] = koff;
            if (m0 + row >= M) voff_a[q] = kOutOfRange;
        }
    });
    static_for<T::B_PER_WAVE>([&](auto q_c) {
        constexpr int q = decltype(q_c)::value;
        if constexpr (T::B_KMAJOR) {
            int row, koff;
            k_major(wave * T::B_PER_WAVE + q, row, koff);
            voff_b[q] = (uint32_t)((int64_t)row * ldb + koff);
            if constexpr (T::EDGE) {
                b_k[q] = koff;
                if (n0 + row >= N) voff_b[q] = kOutOfRange;
            }
        } else {
            int krow, noff;
            if constexpr (T::DWORD) {
                krow = (wave * T::B_PER_WAVE + q) * 2 + (lane >> 5);
                const int u = lane & 31;
                noff = ((u >> 2) ^ (krow & 7)) * 16 + (u & 3) * 4;
            } else {
                krow = (wave * T::B_PER_WAVE + q) * 8 + r8;
                noff = (slot ^ (krow & 7)) * 16;
            }
            voff_b[q] = (uint32_t)((int64_t)krow * ldb + noff);
            if constexpr (T::EDGE) {
                b_k[q] = krow;
                if (n0 + noff >= N) voff_b[q] = kOutOfRange;
            }
        }
    });
    int kcur = first * T::BK;  // first k of the next chunk to request (EDGE)
    uint64_t sbase_a = (uint64_t)(uintptr_t)(A + (int64_t)m0 * lda + (int64_t)first * T::BK);
    uint64_t sbase_b = T::B_KMAJOR ? (uint64_t)(uintptr_t)(B + (int64_t)n0 * ldb + (int64_t)first * T::BK)
                                   : (uint64_t)(uintptr_t)(B + (int64_t)first * T::BK * ldb + n0);
    const uint64_t bstep = T::B_KMAJOR ? (uint64_t)T::BK : (uint64_t)ldb * T::BK;

    auto issue = [&](int stage) __attribute__((always_inline)) {
        const uint32_t dst = lds_base + stage * T::STAGE_BYTES;
        if constexpr (T::EDGE) {
            const i32x4 buf_a = make_buffer((const void *)sbase_a), buf_b = make_buffer((const void *)sbase_b);
            const uint32_t dst_a = dst + wave * (T::A_PER_WAVE * T::INSTR_BYTES);
            const uint32_t dst_b = dst + T::A_BYTES + wave * (T::B_PER_WAVE * T::INSTR_BYTES);
            if (kcur + T::BK <= K) {  // only the chunk that crosses K tests its lanes against it
                static_for<T::A_PER_WAVE>([&](auto q_c) {
                    constexpr int q = decltype(q_c)::value;
                    idma_load<T::DWORD>(buf_a, voff_a[q], dst_a + q * T::INSTR_BYTES);
                });
                static_for<T::B_PER_WAVE>([&](auto q_c) {
                    constexpr int q = decltype(q_c)::value;
                    idma_load<T::DWORD>(buf_b, voff_b[q], dst_b + q * T::INSTR_BYTES);
                });
            } else {
                static_for<T::A_PER_WAVE>([&](auto q_c) {
                    constexpr int q = decltype(q_c)::value;
                    idma_load<T::DWORD>(buf_a, kcur + a_k[q] < K ? voff_a[q] : kOutOfRange, dst_a + q * T::INSTR_BYTES);
                });
                static_for<T::B_PER_WAVE>([&](auto q_c) {
                    constexpr int q = decltype(q_c)::value;
                    idma_load<T::DWORD>(buf_b, kcur + b_k[q] < K ? voff_b[q] : kOutOfRange, dst_b + q * T::INSTR_BYTES);
                });
            }
            kcur += T::BK;
        } else {
#pragma unroll
            for (int q = 0; q < T::A_PER_WAVE; ++q)
                dma16(sbase_a, voff_a[q], dst + (wave * T::A_PER_WAVE + q) * 1024);
#pragma unroll
            for (int q = 0; q < T::B_PER_WAVE; ++q)
                dma16(sbase_b, voff_b[q], dst + T::A_BYTES + (wave * T::B_PER_WAVE + q) * 1024);
        }
        sbase_a += T::BK;
        sbase_b += bstep;
    };

    // ---- fragment read offsets inside a stage ----
    // A, block row a, 32-k group u: row wrow + 32a + li, k-group 2u + half
    // rows of a block differ from li by multiples of 32, which the slot function ignores
    const uint32_t a_row = (uint32_t)((wrow + li) * T::BK);
    // B, block column b, 32-k group u, read j: the 16-lane group of this lane covers columns
    // 16*(li/16) .. +15 of the block, i.e. n-group (wcol + 32b)/16 + li/16; this lane points at
    // k row 32u + 16half + 8j + (lane%16)/2, bytes 8*(lane&1) of that group
    const int jl = lane & 15;
    const int b_krow = 16 * half + (jl >> 1);                      // + 32u + 8j
    const int b_group = (wcol >> 4) + ((lane >> 4) & 1);           // + 2b
    const uint32_t b_byte = (uint32_t)(8 * (jl & 1));

    i32x16v acc[T::TM][T::TN];
#pragma unroll
    for (int a = 0; a < T::TM; ++a)
#pragma unroll
        for (int b = 0; b < T::TN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0;

    typedef __attribute__((address_space(3))) i32x2v lds_i32x2;
    auto compute = [&](int stage, auto between) __attribute__((always_inline)) {
        const unsigned char *st = ilds + stage * T::STAGE_BYTES;
        const unsigned char *stb = st + T::A_BYTES;
        constexpr int U = T::BK / 32;
        // all fragment reads of the chunk are issued before its first MFMA: an int8 MFMA is
        // short (32 cycles for 32 k), so the LDS latency has to be paid once per chunk, not
        // once per k-group
        i32x4 af[U][T::TM], bf[U][T::TN];
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int a = 0; a < T::TM; ++a)
                af[u][a] = *reinterpret_cast<const i32x4 *>(st + a_row + a * 32 * T::BK +
                                                            T::a_slot(2 * u + half, li) * 16);
#pragma unroll
            for (int b = 0; b < T::TN; ++b) {
                if constexpr (T::B_KMAJOR) {
                    bf[u][b] = *reinterpret_cast<const i32x4 *>(stb + (wcol + 32 * b + li) * T::BK +
                                                                T::a_slot(2 * u + half, li) * 16);
                    continue;
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int krow = 32 * u + 8 * j + b_krow;
                    const uint32_t off = (uint32_t)(krow * T::BN) +
                                         (uint32_t)((((b_group + 2 * b) ^ (krow & 7)) * 16)) + b_byte;
                    const i32x2v two = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2 *)(stb + off));
                    bf[u][b][2 * j] = two[0];
                    bf[u][b][2 * j + 1] = two[1];
                }
            }
        }
        between();
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int a = 0; a < T::TM; ++a)
#pragma unroll
                for (int b = 0; b < T::TN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[u][a], bf[u][b], acc[a][b], 0, 0, 0);
    };

    // wait until at most `chunks` later chunks' loads are outstanding, then the barrier
    auto wait_for = [&](int chunks) {
        switch (chunks) {
        case 0: wait_vmcnt_and_barrier<0>(); break;
        case 1: wait_vmcnt_and_barrier<T::LOADS>(); break;
        case 2: wait_vmcnt_and_barrier<(T::NSTAGE > 3 ? 2 : 0) * T::LOADS>(); break;
        case 3: wait_vmcnt_and_barrier<(T::NSTAGE > 4 ? 3 : 0) * T::LOADS>(); break;
        default: wait_vmcnt_and_barrier<(T::NSTAGE > 5 ? 4 : 0) * T::LOADS>(); break;
        }
    };
    auto step = [&](int it, auto stage_tag) __attribute__((always_inline)) {
        constexpr int stage = decltype(stage_tag)::value;
        const int ahead = nk - 1 - it;  // later chunks whose loads may stay in flight
        wait_for(ahead < T::NSTAGE - 2 ? ahead : T::NSTAGE - 2);
        compute(stage, [&]() {
            if (it + T::NSTAGE - 1 < nk) issue((stage + T::NSTAGE - 1) % T::NSTAGE);
        });
    };

#pragma unroll
    for (int p = 0; p < T::NSTAGE - 1; ++p)
        if (p < nk) issue(p);
    for (int it = 0; it < nk; it += T::NSTAGE)
        static_for<T::NSTAGE>([&](auto s_c) {
            if (it + decltype(s_c)::value < nk) step(it + decltype(s_c)::value, s_c);
        });

    // ---- epilogue: register v of block (a, b) is row 32a + 8(v/4) + 4half + v%4, column 32b + li ----
    // The old values of a block row are requested together, before the first store: a load
    // behind a store to C would wait for that store, one memory round trip per register.
    if constexpr (T::EDGE) {
        if (m0 + T::BM > M || n0 + T::BN > N) {
            // A tile on the edge of C: through a buffer descriptor over the tile's part of C.  An
            // element past M or N gets an out-of-range offset, for which a load returns zero and a
            // store does nothing: every lane issues the same instructions, and a block row of old
            // values is in flight before the first is used.  (With a test around every plain load
            // each element became a branch and a round trip to memory of its own, and the edge
            // tiles ended long after the others.)  32-bit offsets: BM rows of ldc words stay below
            // 2^31 bytes (host check).
            const __amdgpu_buffer_rsrc_t cbuf = __builtin_amdgcn_make_buffer_rsrc(
                C + (int64_t)m0 * ldc + n0, 0, (int)kOutOfRange, 0x00020000);
            const int rows_in = M - m0, cols_in = N - n0;
#pragma unroll
            for (int a = 0; a < T::TM; ++a) {
                const int r0 = wrow + 32 * a + 4 * half, c0 = wcol + li;  // inside the tile
                uint32_t off[16][T::TN];
#pragma unroll
                for (int v = 0; v < 16; ++v)
#pragma unroll
                    for (int b = 0; b < T::TN; ++b) {
                        const int r = r0 + 8 * (v >> 2) + (v & 3), c = c0 + 32 * b;
                        off[v][b] = (r < rows_in && c < cols_in) ? (uint32_t)r * (uint32_t)(ldc * 4) + (uint32_t)(c * 4) : kOutOfRange;
                    }
                if (sliced) {
                    int32_t *const dst = C + (int64_t)m0 * ldc + n0;
#pragma unroll
                    for (int v = 0; v < 16; ++v)
#pragma unroll
                        for (int b = 0; b < T::TN; ++b)
                            if (off[v][b] != kOutOfRange) atomicAdd(dst + off[v][b] / 4, acc[a][b][v]);
                } else {
                    uint32_t old[16][T::TN];
#pragma unroll
                    for (int v = 0; v < 16; ++v)
#pragma unroll
                        for (int b = 0; b < T::TN; ++b)
                            old[v][b] = __builtin_amdgcn_raw_buffer_load_b32(cbuf, (int)off[v][b], 0, 0);
#pragma unroll
                    for (int v = 0; v < 16; ++v)
#pragma unroll
                        for (int b = 0; b < T::TN; ++b)
                            __builtin_amdgcn_raw_buffer_store_b32(old[v][b] + (uint32_t)acc[a][b][v], cbuf, (int)off[v][b], 0, 0);
                }
            }
            return;
        }
    }
#pragma unroll
    for (int a = 0; a < T::TM; ++a) {
        int32_t *const dst = C + (int64_t)(m0 + wrow + 32 * a + 4 * half) * ldc + n0 + wcol + li;
        auto at = [&](int v, int b) { return dst + (int64_t)(8 * (v >> 2) + (v & 3)) * ldc + 32 * b; };
        if (sliced) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
#pragma unroll
                for (int b = 0; b < T::TN; ++b) atomicAdd(at(v, b), acc[a][b][v]);
        } else {
            uint32_t old[16][T::TN];
#pragma unroll
            for (int v = 0; v < 16; ++v)
#pragma unroll
                for (int b = 0; b < T::TN; ++b) old[v][b] = (uint32_t)*at(v, b);
#pragma unroll
            for (int v = 0; v < 16; ++v)
#pragma unroll
                for (int b = 0; b < T::TN; ++b) *at(v, b) = (int32_t)(old[v][b] + (uint32_t)acc[a][b][v]);
        }
    }
}

}  // namespace lsmi
