// Aligned-shape fp32 GEMM kernel for gfx950: C += A.B with the operand tiles streamed
// global -> LDS by the load unit itself (GLOBAL_LOAD_LDS_DWORDX4), never passing through
// registers, in a ring of NSTAGE chunk buffers that keeps the loads two chunks ahead of
// the matrix cores.
//
// Preconditions (checked by the host before this kernel is chosen).  Plain form: M % BM == 0,
// N % BN == 0, K % 16 == 0, A and B 16-byte aligned with lda, ldb multiples of 4, C
// 8-byte aligned with even ldc, BM*lda*4 and 16*ldb*4 + BN*4 below 2^32.  EDGE form: only
// A and B 16-byte aligned with lda, ldb and K multiples of 4 and BM*lda*4, 16*ldb*4 + BN*4
// below 2^31; M, N and the K remainder are free.  There the loads go through buffer
// descriptors and 16-byte groups that lie past M, past the slice's last k or past N are
// given an out-of-range offset, which yields zeros; tiles on the matrix edge store element-wise, and the reduction may be split over blockIdx.y (partial sums
// are then added to C with atomics).
//
// LDS image of one chunk (BK = 16):
//   A: BM rows x 64 bytes.  The four 16-byte k-groups of a row are stored at slot
//      g ^ f(row), f(r) = ((r >> 1) ^ (r >> 2)) & 3, so that the 16-byte fragment reads of
//      32 consecutive rows fall into distinct banks without padding (a DMA write is
//      always 64 lanes x 16 contiguous bytes, so padding is not available).
//   B: 16 rows x BN floats, as in memory.
// A wave instruction moves 1 KiB: 16 rows of A, or 1024/(4*BN) rows of B; each lane
// picks the global 16 bytes that belong in its LDS slot.
//
// Per chunk `it`:  wait until this wave's loads of chunk `it` have landed, barrier (all
// waves' parts are there, and everyone is done reading chunk it-1), issue the loads of
// chunk it+2 into the buffer chunk it-1 used, then LDS -> MFMA for chunk `it`.
// The loads are issued from inline assembly: the compiler would otherwise wait for all
// outstanding LDS-writing loads before every LDS read.  The counter waits are explicit.
#pragma once

#include <type_traits>

#include "tile_f32.hpp"

namespace lsmi {

// PREFETCH_C: the old contents of the C tile are requested before the first chunk and wait in
// registers, so the epilogue does not pay their latency; the registers that takes leave room
// for MAX_WGS = 2 workgroups per CU only.
//
// KPAIR: a step brings in two chunks, and the waves come in two sets of WAVES_M x WAVES_N, each
// of which loads and multiplies one of the two over the whole tile; the two partial tiles are
// added through LDS before the epilogue.  A 64 x 64 tile then occupies all four SIMDs with
// 32 x 64 wave tiles: the form for outputs with about one tile per CU.
//
// DWORD (an EDGE form): every load instruction moves 4 bytes per lane instead of 16, so nothing
// about A, B, lda, ldb or K has to be a multiple of four elements: rows may start at any
// element, and the test against the end of the reduction is per element.  Four times the load
// instructions for the same image of the chunk in LDS.
template <int BM_, int BN_, int WAVES_M_, int WAVES_N_, int NSTAGE_, bool PREFETCH_C_, bool EDGE_ = false,
          int MAX_WGS_ = 4, bool KPAIR_ = false, bool DWORD_ = false>
struct DmaShape {
    static constexpr bool PREFETCH_C = PREFETCH_C_, EDGE = EDGE_, KPAIR = KPAIR_, DWORD = DWORD_;
    static constexpr int BM = BM_, BN = BN_, BK = 16, NSTAGE = NSTAGE_;
    static constexpr int KSETS = KPAIR ? 2 : 1;       // chunks per step = wave sets
    static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, SET_WAVES = WAVES_M * WAVES_N;
    static constexpr int NWAVES = SET_WAVES * KSETS;
    static constexpr int NT = 64 * NWAVES;
    static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    static constexpr int TM = WTM / 32, TN = WTN / 32;
    static constexpr int A_BYTES = BM * BK * 4, B_BYTES = BK * BN * 4;
    static constexpr int CHUNK_BYTES = A_BYTES + B_BYTES;
    static constexpr int STAGE_BYTES = KSETS * CHUNK_BYTES;
    static constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;
    static constexpr int A_PER_WAVE = A_BYTES / 1024 / SET_WAVES;  // DMA instructions per wave and step
    static constexpr int B_PER_WAVE = B_BYTES / 1024 / SET_WAVES;
    static constexpr int INSTR_BYTES = DWORD ? 256 : 1024;  // LDS bytes one load instruction fills
    static constexpr int A_INSTR = A_PER_WAVE * (1024 / INSTR_BYTES);  // load instructions per wave and step
    static constexpr int B_INSTR = B_PER_WAVE * (1024 / INSTR_BYTES);
    static constexpr int LOADS = A_INSTR + B_INSTR;
    static constexpr int B_ROWS_PER_INSTR = 1024 / (4 * BN);
    // waves per SIMD the register allocation must allow: as many workgroups as LDS holds
    static constexpr int WGS_PER_CU = (160 * 1024) / LDS_BYTES < MAX_WGS_ ? (160 * 1024) / LDS_BYTES : MAX_WGS_;
    static constexpr int WAVES_PER_SIMD = WGS_PER_CU * NWAVES / 4;
    static_assert(TN == 2, "B fragments are read as float2, C is accessed as float2");
    static_assert(A_BYTES % (1024 * SET_WAVES) == 0 && B_BYTES % (1024 * SET_WAVES) == 0, "even DMA split");
    static_assert(BN == 64 || BN == 128 || BN == 256, "a DMA instruction covers whole B rows");
    static_assert(!KPAIR || (!PREFETCH_C && TM * TN * 16 * 256 * SET_WAVES <= LDS_BYTES),
                  "the second set's partial tile passes through the ring's LDS");
    static_assert(LDS_BYTES <= 160 * 1024 && NSTAGE * STAGE_BYTES < 65536 + STAGE_BYTES, "LDS budget");
    static_assert(LOADS * (NSTAGE - 2) <= 63, "vmcnt range");
    static_assert(NSTAGE >= 2 && NSTAGE <= 8, "the step loop is unrolled NSTAGE times");
    static_assert(!(EDGE && PREFETCH_C), "the early C request assumes a full tile");
    static_assert(!DWORD || EDGE, "the 4-byte loads are a form of the buffer-load kernel");
};

// 16 bytes per lane, global (scalar base + 32-bit lane offset) -> LDS at lds_addr + lane*16.
__device__ __forceinline__ void dma16(uint64_t sbase, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(sbase)
                 : "memory", "m0");
}

// The same through a buffer descriptor: 16 bytes per lane from base + voff -> LDS at
// lds_addr + lane*16, and a lane whose offset is kOutOfRange gets sixteen zero bytes (the
// buffer range check), which is how padding and ragged edges are filled without a branch.
// (A full 64-bit address per lane would also do, but GLOBAL_LOAD_LDS with a vector address
// pair runs at about two thirds of the rate of the scalar-base forms here.)
typedef int i32x4 __attribute__((ext_vector_type(4)));
constexpr uint32_t kOutOfRange = 0x80000000u;

__device__ __forceinline__ i32x4 make_buffer(const void *base)
{
    const uint64_t addr = (uint64_t)(uintptr_t)base;
    i32x4 r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(addr & 0xffffffffu));
    r[1] = __builtin_amdgcn_readfirstlane((int)((addr >> 32) & 0xffffu));  // stride 0: raw buffer
    r[2] = (int)kOutOfRange;  // bytes in range: every offset below kOutOfRange
    r[3] = 0x00020000;        // 32-bit data format
    return r;
}

__device__ __forceinline__ void dma16_buf(i32x4 buffer, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(buffer)
                 : "memory", "m0");
}

// The same with a scalar byte offset added to every lane's address after the range check of
// the lane offset: a lane that is out of range stays so, the others move together, and the
// loop that walks along a row needs no vector arithmetic.
__device__ __forceinline__ void dma16_buf_s(i32x4 buffer, uint32_t voff, uint32_t soff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(buffer), "s"(soff)
                 : "memory", "m0");
}

// Four bytes per lane: base + voff -> LDS at lds_addr + lane*4, zeros for kOutOfRange.
__device__ __forceinline__ void dma4_buf(i32x4 buffer, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dword %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(buffer)
                 : "memory", "m0");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt_and_barrier()
{
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" : : "n"(N) : "memory");
}

// Waits until at most `chunks` (0 .. MAX) chunks of LOADS load instructions each are still
// outstanding, then the barrier.  The wait count is an immediate, hence the dispatch.
template <int LOADS, int MAX>
__device__ __forceinline__ void wait_chunks_and_barrier(int chunks)
{
    static_assert(MAX >= 0 && MAX <= 6 && LOADS * MAX <= 63, "vmcnt range");
    switch (chunks) {
    case 0: wait_vmcnt_and_barrier<0>(); break;
    case 1: wait_vmcnt_and_barrier<(MAX >= 1 ? 1 : 0) * LOADS>(); break;
    case 2: wait_vmcnt_and_barrier<(MAX >= 2 ? 2 : 0) * LOADS>(); break;
    case 3: wait_vmcnt_and_barrier<(MAX >= 3 ? 3 : 0) * LOADS>(); break;
    case 4: wait_vmcnt_and_barrier<(MAX >= 4 ? 4 : 0) * LOADS>(); break;
    case 5: wait_vmcnt_and_barrier<(MAX >= 5 ? 5 : 0) * LOADS>(); break;
    default: wait_vmcnt_and_barrier<(MAX >= 6 ? 6 : 0) * LOADS>(); break;
    }
}

template <class T>
__global__ __launch_bounds__(T::NT)
__attribute__((amdgpu_waves_per_eu(T::WAVES_PER_SIMD, T::WAVES_PER_SIMD))) void sgemm_dma_kernel(
    int M, int N, int K, const float *__restrict__ A, int64_t lda, const float *__restrict__ B,
    int64_t ldb, float *__restrict__ C, int64_t ldc, int tiles_m, int tiles_n, int group_m,
    int k_per_split, int split_k, int tail_first, int tail_split, Epilogue ep)
{
    __shared__ __attribute__((aligned(1024))) unsigned char lds[T::LDS_BYTES];
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, half = lane >> 5;
    // KPAIR: wave set kset takes chunk kset of every step; sw is the wave's index in its set
    const int kset = wave / T::SET_WAVES, sw = wave % T::SET_WAVES;
    const int wrow = (sw / T::WAVES_N) * T::WTM;
    const int wcol = (sw % T::WAVES_N) * T::WTN;

    // Which tile, and which slice of its reduction (the whole of it unless EDGE splits K).
    // Uniform split: blockIdx.y is the slice.  Tail split (tail_split > 1, a one-dimensional
    // grid): the first tail_first workgroups take whole tiles, and each tile after those is
    // cut into tail_split slices whose partial sums are added atomically -- the tiles left
    // over after the last whole round of the CUs then keep every CU busy for a fraction of a
    // tile's time instead of a few CUs for all of it.
    // (without a tail split, tail_first is the index of the launch's first tile: a large
    // output is computed by several launches of one generation of resident workgroups each)
    int wg = (int)blockIdx.x + ((!T::EDGE || tail_split <= 1) ? tail_first : 0), slice = T::EDGE ? (int)blockIdx.y : 0,
        slices = T::EDGE ? split_k : 1;
    int kper = k_per_split;
    if (T::EDGE && tail_split > 1) {
        if (wg >= tail_first) {
            const int r = wg - tail_first;
            wg = tail_first + r / tail_split;
            slice = r % tail_split;
            slices = tail_split;
        } else {
            kper = K;
        }
    }
    int tm, tn;
    map_tile(wg, tiles_m, tiles_n, group_m, tm, tn);
    const int m0 = tm * T::BM, n0 = tn * T::BN;
    const int kbeg = T::EDGE ? slice * kper : 0;
    const int kend = T::EDGE ? (kbeg + kper < K ? kbeg + kper : K) : K;
    constexpr int STEP_K = T::BK * T::KSETS;  // reduction elements per step
    const int nk = (kend - kbeg + STEP_K - 1) / STEP_K;

    // ---- DMA sources ----
    // plain form: 32-bit lane offsets (constant over the reduction) from two scalar bases
    uint32_t voff_a[T::A_INSTR], voff_b[T::B_INSTR];
    // EDGE form: the same offsets, kOutOfRange for a row past M or a column group past N,
    // and the k-group / k-row of the lane inside a chunk for the test against the slice end
    int a_k[T::A_INSTR], b_k[T::B_INSTR];
    if constexpr (T::DWORD) {
        // instruction i of the wave set fills bytes 256 i .. 256 i + 255 of the chunk's image:
        // A, four rows of 64 bytes, the lane's dword at slot (lane & 15) >> 2 of its row, which
        // holds k-group slot ^ f(row); B, 64 consecutive floats of the row-major 16 x BN image
#pragma unroll
        for (int q = 0; q < T::A_INSTR; ++q) {
            const int row = (sw * T::A_INSTR + q) * 4 + (lane >> 4);
            const int r16 = row & 15;
            const int g = ((lane & 15) >> 2) ^ (((r16 >> 1) ^ (r16 >> 2)) & 3);
            a_k[q] = g * 4 + (lane & 3);
            voff_a[q] = m0 + row < M ? (uint32_t)(((int64_t)row * lda + a_k[q]) * 4) : kOutOfRange;
        }
#pragma unroll
        for (int q = 0; q < T::B_INSTR; ++q) {
            const int e = (sw * T::B_INSTR + q) * 64 + lane;
            b_k[q] = e / T::BN;
            const int col = e % T::BN;
            voff_b[q] = n0 + col < N ? (uint32_t)(((int64_t)b_k[q] * ldb + col) * 4) : kOutOfRange;
        }
    } else if constexpr (T::EDGE) {
        const int r16 = lane >> 2;
        const int g = (lane & 3) ^ (((r16 >> 1) ^ (r16 >> 2)) & 3);
#pragma unroll
        for (int q = 0; q < T::A_PER_WAVE; ++q) {
            const int row = (sw * T::A_PER_WAVE + q) * 16 + r16;
            a_k[q] = g * 4;
            voff_a[q] = m0 + row < M ? (uint32_t)(((int64_t)row * lda + g * 4) * 4) : kOutOfRange;
        }
        const int lanes_per_row = T::BN / 4;
#pragma unroll
        for (int q = 0; q < T::B_PER_WAVE; ++q) {
            b_k[q] = (sw * T::B_PER_WAVE + q) * T::B_ROWS_PER_INSTR + lane / lanes_per_row;
            const int col4 = (lane % lanes_per_row) * 4;
            voff_b[q] = n0 + col4 < N ? (uint32_t)(((int64_t)b_k[q] * ldb + col4) * 4) : kOutOfRange;
        }
    } else {
        const int r16 = lane >> 2;  // row inside the 16-row block of one instruction
        const int g = (lane & 3) ^ (((r16 >> 1) ^ (r16 >> 2)) & 3);  // k-group stored in this slot
#pragma unroll
        for (int q = 0; q < T::A_PER_WAVE; ++q) {
            const int row = (sw * T::A_PER_WAVE + q) * 16 + r16;
            voff_a[q] = (uint32_t)(((int64_t)row * lda + g * 4) * 4);
        }
        const int lanes_per_row = T::BN / 4;
#pragma unroll
        for (int q = 0; q < T::B_PER_WAVE; ++q) {
            const int kk = (sw * T::B_PER_WAVE + q) * T::B_ROWS_PER_INSTR + lane / lanes_per_row;
            voff_b[q] = (uint32_t)(((int64_t)kk * ldb + (lane % lanes_per_row) * 4) * 4);
        }
    }
    const int kfirst = kbeg + kset * T::BK;  // this wave set's chunk of the first step
    uint64_t sbase_a = (uint64_t)(uintptr_t)(A + (int64_t)m0 * lda + kfirst);
    uint64_t sbase_b = (uint64_t)(uintptr_t)(B + (int64_t)kfirst * ldb + n0);
    const uint64_t bstep = (uint64_t)ldb * (STEP_K * 4);
    int kcur = kfirst;  // first k of the next chunk to request (EDGE form)

    auto issue = [&](int stage) {
        const uint32_t dst = lds_base + stage * T::STAGE_BYTES + kset * T::CHUNK_BYTES;
        if constexpr (T::DWORD) {
            const i32x4 buf_a = make_buffer((const void *)sbase_a), buf_b = make_buffer((const void *)sbase_b);
            if (kcur + T::BK <= kend) {
#pragma unroll
                for (int q = 0; q < T::A_INSTR; ++q) dma4_buf(buf_a, voff_a[q], dst + (sw * T::A_INSTR + q) * 256);
#pragma unroll
                for (int q = 0; q < T::B_INSTR; ++q)
                    dma4_buf(buf_b, voff_b[q], dst + T::A_BYTES + (sw * T::B_INSTR + q) * 256);
            } else {
#pragma unroll
                for (int q = 0; q < T::A_INSTR; ++q)
                    dma4_buf(buf_a, kcur + a_k[q] < kend ? voff_a[q] : kOutOfRange, dst + (sw * T::A_INSTR + q) * 256);
#pragma unroll
                for (int q = 0; q < T::B_INSTR; ++q)
                    dma4_buf(buf_b, kcur + b_k[q] < kend ? voff_b[q] : kOutOfRange,
                             dst + T::A_BYTES + (sw * T::B_INSTR + q) * 256);
            }
            kcur += STEP_K;
            sbase_a += STEP_K * 4;
            sbase_b += bstep;
        } else if constexpr (T::EDGE) {
            const i32x4 buf_a = make_buffer((const void *)sbase_a), buf_b = make_buffer((const void *)sbase_b);
            // only the chunk that crosses the end of the slice tests its lanes against it
            // (vector instructions take matrix-pipe time; a whole chunk needs none)
            if (kcur + T::BK <= kend) {
#pragma unroll
                for (int q = 0; q < T::A_PER_WAVE; ++q)
                    dma16_buf(buf_a, voff_a[q], dst + (sw * T::A_PER_WAVE + q) * 1024);
#pragma unroll
                for (int q = 0; q < T::B_PER_WAVE; ++q)
                    dma16_buf(buf_b, voff_b[q], dst + T::A_BYTES + (sw * T::B_PER_WAVE + q) * 1024);
            } else {
#pragma unroll
                for (int q = 0; q < T::A_PER_WAVE; ++q)
                    dma16_buf(buf_a, kcur + a_k[q] < kend ? voff_a[q] : kOutOfRange,
                              dst + (sw * T::A_PER_WAVE + q) * 1024);
#pragma unroll
                for (int q = 0; q < T::B_PER_WAVE; ++q)
                    dma16_buf(buf_b, kcur + b_k[q] < kend ? voff_b[q] : kOutOfRange,
                              dst + T::A_BYTES + (sw * T::B_PER_WAVE + q) * 1024);
            }
            kcur += STEP_K;
            sbase_a += STEP_K * 4;
            sbase_b += bstep;
        } else {
#pragma unroll
            for (int q = 0; q < T::A_PER_WAVE; ++q)
                dma16(sbase_a, voff_a[q], dst + (sw * T::A_PER_WAVE + q) * 1024);
#pragma unroll
            for (int q = 0; q < T::B_PER_WAVE; ++q)
                dma16(sbase_b, voff_b[q], dst + T::A_BYTES + (sw * T::B_PER_WAVE + q) * 1024);
            sbase_a += STEP_K * 4;
            sbase_b += bstep;
        }
    };

    // ---- fragment read offsets inside a stage ----
    const int fsw = ((li >> 1) ^ (li >> 2)) & 3;  // f(row): rows of a block differ from li by multiples of 32
    const uint32_t a_off0 = (uint32_t)((wrow + li) * 64 + ((half ^ fsw) * 16));        // k-groups 0/1
    const uint32_t a_off1 = (uint32_t)((wrow + li) * 64 + (((2 + half) ^ fsw) * 16));  // k-groups 2/3
    const uint32_t b_off = (uint32_t)(T::A_BYTES + half * 4 * T::BN * 4 + (wcol + 2 * li) * 4);

    f32x16 acc[T::TM][T::TN];
#pragma unroll
    for (int a = 0; a < T::TM; ++a)
#pragma unroll
        for (int b = 0; b < T::TN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // `between` runs after the fragment reads are issued and before the first MFMA: the
    // next chunk's global loads are issued there, under the LDS latency.
    auto compute = [&](int stage, auto between) {
        const unsigned char *st = lds + stage * T::STAGE_BYTES + kset * T::CHUNK_BYTES;
        // all fragment reads of the chunk are issued before its first MFMA, so the reads of
        // the second k-half are in flight while the first half is being multiplied
        f32x4 af[2][T::TM];
        f32x2 bf[2][4];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
#pragma unroll
            for (int a = 0; a < T::TM; ++a)
                af[u][a] = *reinterpret_cast<const f32x4 *>(st + (u ? a_off1 : a_off0) + a * 32 * 64);
#pragma unroll
            for (int t = 0; t < 4; ++t)
                bf[u][t] = *reinterpret_cast<const f32x2 *>(st + b_off + (8 * u + t) * T::BN * 4);
        }
        between();
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int a = 0; a < T::TM; ++a)
#pragma unroll
                    for (int b = 0; b < T::TN; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[u][a][t], bf[u][t][b],
                                                                        acc[a][b], 0, 0, 0);
    };

    // C tile of this lane: two adjacent columns per (block row a, register v).
    const int col = n0 + wcol + 2 * li;
    auto c_ptr = [&](int a, int v) {
        const int row = m0 + wrow + 32 * a + 8 * (v >> 2) + 4 * half + (v & 3);
        return reinterpret_cast<f32x2 *>(C + (int64_t)row * ldc + col);
    };
    f32x2 cin[T::PREFETCH_C ? T::TM * 16 : 1];
    auto prefetch_c = [&]() {
        if constexpr (T::PREFETCH_C) {
            if (ep.pre != kPreAccumulate) return;
#pragma unroll
            for (int a = 0; a < T::TM; ++a)
#pragma unroll
                for (int v = 0; v < 16; ++v) cin[a * 16 + v] = *c_ptr(a, v);
        }
    };

    // One pipeline step with a compile-time stage index.
    auto step = [&](int it, auto stage_tag, auto first_tag) {
        constexpr int stage = decltype(stage_tag)::value;
        // chunks after `it` whose loads may stay in flight: at most NSTAGE-2, fewer at the end
        const int ahead = nk - 1 - it;
        wait_chunks_and_barrier<T::LOADS, T::NSTAGE - 2>(ahead < T::NSTAGE - 2 ? ahead : T::NSTAGE - 2);
        // the old contents of C are requested once the first chunk has landed, so the request
        // is not in the way of the first wait and arrives under the MFMAs
        if constexpr (decltype(first_tag)::value) prefetch_c();
        compute(stage, [&]() {
            if (it + T::NSTAGE - 1 < nk) issue((stage + T::NSTAGE - 1) % T::NSTAGE);
        });
    };

    // Prologue: NSTAGE-1 chunks in flight.  Then the steps, the first one peeled off (it alone
    // requests C), the rest unrolled NSTAGE times so that the stage index (and with it every
    // LDS offset) is a compile-time constant.
#pragma unroll
    for (int p = 0; p < T::NSTAGE - 1; ++p)
        if (p < nk) issue(p);
    if (nk > 0) step(0, std::integral_constant<int, 0>{}, std::true_type{});
    for (int it = 1; it < nk; it += T::NSTAGE)
        static_for<T::NSTAGE>([&](auto s_c) {
            constexpr int s = decltype(s_c)::value;
            if (it + s < nk) step(it + s, std::integral_constant<int, (s + 1) % T::NSTAGE>{}, std::false_type{});
        });

    if constexpr (T::KPAIR) {
        // the second wave set hands its partial tile to the first through the ring's LDS
        // ([wave][register][lane], conflict-free), then only the first set has an epilogue
        __syncthreads();  // every wave is through with the last chunks
        float *part = reinterpret_cast<float *>(lds) + sw * (T::TM * T::TN * 16 * 64);
        if (kset == 1) {
#pragma unroll
            for (int a = 0; a < T::TM; ++a)
#pragma unroll
                for (int b = 0; b < T::TN; ++b)
#pragma unroll
                    for (int v = 0; v < 16; ++v) part[((a * T::TN + b) * 16 + v) * 64 + lane] = acc[a][b][v];
        }
        __syncthreads();
        if (kset == 1) return;
#pragma unroll
        for (int a = 0; a < T::TM; ++a)
#pragma unroll
            for (int b = 0; b < T::TN; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[a][b][v] += part[((a * T::TN + b) * 16 + v) * 64 + lane];
    }

    // ---- epilogue: C = post(pre(C) + acc) ----
    bool vec = true;  // whole tile inside the matrix, C accessible as float2, no partial sums
    if constexpr (T::EDGE)
        vec = slices == 1 && m0 + T::BM <= M && n0 + T::BN <= N &&
              (((uintptr_t)C | (uintptr_t)(ldc * 4)) & 7) == 0 &&
              (ep.pre != kPreBias || ((uintptr_t)ep.bias & 7) == 0);
    if (vec) {
        // Old values are requested eight registers at a time before the first of them is used:
        // a load placed behind a store to C would have to wait for that store (they may
        // overlap as far as the compiler can tell), one memory round trip per register.
        if (ep.pre == kPreAccumulate) {
            constexpr int BATCH = 8;  // registers of a block row requested together
#pragma unroll
            for (int a = 0; a < T::TM; ++a)
#pragma unroll
                for (int v0 = 0; v0 < 16; v0 += BATCH) {
                    f32x2 c[BATCH];
#pragma unroll
                    for (int v = 0; v < BATCH; ++v) {
                        if constexpr (T::PREFETCH_C) c[v] = cin[a * 16 + v0 + v]; else c[v] = *c_ptr(a, v0 + v);
                    }
#pragma unroll
                    for (int v = 0; v < BATCH; ++v) {
                        c[v][0] = apply_post(c[v][0] + acc[a][0][v0 + v], ep.post);
                        c[v][1] = apply_post(c[v][1] + acc[a][1][v0 + v], ep.post);
                        *c_ptr(a, v0 + v) = c[v];
                    }
                }
        } else {
            f32x2 init{0.f, 0.f};
            if (ep.pre == kPreBias) init = *reinterpret_cast<const f32x2 *>(ep.bias + col);  // col is even, bias 8-byte aligned
#pragma unroll
            for (int a = 0; a < T::TM; ++a)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    f32x2 c;
                    c[0] = apply_post(init[0] + acc[a][0][v], ep.post);
                    c[1] = apply_post(init[1] + acc[a][1][v], ep.post);
                    *c_ptr(a, v) = c;
                }
        }
    } else if (slices > 1) {
#pragma unroll
        for (int a = 0; a < T::TM; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wrow + 32 * a + 8 * (v >> 2) + 4 * half + (v & 3);
                float *dst = C + (int64_t)row * ldc + col;
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    if (row < M && col + b < N) atomicAdd(dst + b, acc[a][b][v]);  // plain accumulate form only
            }
    } else {
        // edge tiles, element by element; the old values again half a block row ahead of the stores
#pragma unroll
        for (int a = 0; a < T::TM; ++a)
#pragma unroll
            for (int v0 = 0; v0 < 16; v0 += 8) {
                float c[8][2];
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    const int row = m0 + wrow + 32 * a + 8 * ((v0 + v) >> 2) + 4 * half + (v & 3);
                    const float *src = C + (int64_t)row * ldc + col;
#pragma unroll
                    for (int b = 0; b < 2; ++b) {
                        c[v][b] = 0.f;
                        if (row < M && col + b < N)
                            c[v][b] = ep.pre == kPreAccumulate ? src[b] : ep.pre == kPreBias ? ep.bias[col + b] : 0.f;
                    }
                }
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    const int row = m0 + wrow + 32 * a + 8 * ((v0 + v) >> 2) + 4 * half + (v & 3);
                    float *dst = C + (int64_t)row * ldc + col;
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        if (row < M && col + b < N) dst[b] = apply_post(c[v][b] + acc[a][b][v0 + v], ep.post);
                }
            }
    }
}

}  // namespace lsmi
