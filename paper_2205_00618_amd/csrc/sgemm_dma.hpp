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
// KSETS > 1: a step brings in KSETS chunks, and the waves come in KSETS sets of WAVES_M x WAVES_N,
// each of which loads and multiplies one of them over the whole tile; the partial tiles are
// added through LDS, in set order, before the epilogue.  A 64 x 64 tile then occupies all four
// SIMDs with 32 x 64 wave tiles, once (KSETS = 2) or twice over (KSETS = 4, two waves per SIMD
// that cover each other's waits): the forms for outputs with about one tile per CU, where the
// reduction has to be cut inside the workgroup because nothing else shares the CU.
//
// DWORD (an EDGE form): every load instruction moves 4 bytes per lane instead of 16, so nothing
// about A, B, lda, ldb or K has to be a multiple of four elements: rows may start at any
// element, and the test against the end of the reduction is per element.  Four times the load
// instructions for the same image of the chunk in LDS.
//
// A_T: the array A holds the left operand transposed, K x M with row stride lda (Section 2.1
// lists the transposition among the contractions; here it is the affine index map of an operand,
// applied on the way into LDS, not a pass of its own).  Its chunk is then stored like B's, 16
// rows of BM floats, and block row a of a wave takes the rows wrow + TM i + a, so that one
// read fetches the lane's operands of all TM blocks.
// B_T: the array B holds the right operand transposed, N x K with row stride ldb.  Its chunk is
// stored like A's, BN rows of 64 bytes with the same XOR of the k-groups, and since every lane of
// a load picks the global 16 bytes that belong in its LDS slot, the rows are stored permuted:
// LDS row 32 b + i of a wave's 64 columns holds column 2 i + b, which keeps the wave's two
// blocks on adjacent columns (C as float2) while the fragment reads stay the 16-byte reads of A.
template <int BM_, int BN_, int WAVES_M_, int WAVES_N_, int NSTAGE_, bool PREFETCH_C_, bool EDGE_ = false,
          int MAX_WGS_ = 4, int KSETS_ = 1, bool DWORD_ = false, bool A_T_ = false, bool B_T_ = false>
struct DmaShape {
    static constexpr bool PREFETCH_C = PREFETCH_C_, EDGE = EDGE_, DWORD = DWORD_, A_T = A_T_, B_T = B_T_;
    static constexpr int BM = BM_, BN = BN_, BK = 16, NSTAGE = NSTAGE_;
    static constexpr int KSETS = KSETS_;              // chunks per step = wave sets
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
    static constexpr int A_ROWS_PER_INSTR = 1024 / (4 * BM);  // k-rows of a transposed A per 1 KiB
    static constexpr int B_ROWS_PER_INSTR = 1024 / (4 * BN);
    // waves per SIMD the register allocation must allow: as many workgroups as LDS holds
    static constexpr int WGS_PER_CU = (160 * 1024) / LDS_BYTES < MAX_WGS_ ? (160 * 1024) / LDS_BYTES : MAX_WGS_;
    static constexpr int WAVES_PER_SIMD = WGS_PER_CU * NWAVES / 4;
    static constexpr int TILE = BM * BN;  // floats of a tile: one partial sum in the workspace
    static_assert(TN == 2, "B fragments are read as float2, C is accessed as float2");
    static_assert(TM == 1 || TM == 2 || TM == 4, "a transposed A fragment is read as 1, 2 or 4 floats");
    static_assert(KSETS == 1 || KSETS == 2 || KSETS == 4, "wave sets");
    static_assert(A_BYTES % (1024 * SET_WAVES) == 0 && B_BYTES % (1024 * SET_WAVES) == 0, "even DMA split");
    static_assert(BN == 64 || BN == 128 || BN == 256, "a DMA instruction covers whole B rows");
    static_assert(!A_T || BM == 64 || BM == 128 || BM == 256, "a DMA instruction covers whole rows of a transposed A");
    static_assert(KSETS == 1 || (!PREFETCH_C && KSETS * TM * TN * 16 * 256 * SET_WAVES <= LDS_BYTES),
                  "the sets' partial tiles pass through the ring's LDS");
    static_assert(LDS_BYTES + 16 <= 160 * 1024, "LDS budget");
    static_assert(LOADS * (NSTAGE - 2) <= 63, "vmcnt range");
    static_assert(NSTAGE >= 2 && NSTAGE <= 8, "the step loop is unrolled NSTAGE times");
    static_assert(!(EDGE && PREFETCH_C), "the early C request assumes a full tile");
    static_assert(!DWORD || EDGE, "the 4-byte loads are a form of the buffer-load kernel");
    static_assert((TILE / 4) % NT == 0, "the fix-up walks the tile in 16-byte groups");
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

// The workgroup's barrier alone, behind this wave's LDS operations.  (__syncthreads() also waits
// for the wave's outstanding global loads: where a request is meant to stay in flight across
// the barrier, this is the one to use.)
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
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

// Where the partial sums of a cut reduction meet when the caller provides memory for them
// instead of letting them meet in atomic adds onto C.  `partials` holds one BM x BN tile
// (row-major floats) per slice of every cut tile; `counters` one word per cut tile, zero when
// the kernel starts and zero again when it ends.  Every workgroup stores its partial tile,
// and the one that finds itself the last of its tile's slices to arrive adds all of them in
// slice order and runs the epilogue: no atomic arithmetic, the result does not depend on
// which workgroup came last, and any pre- and post-operation applies.
struct Meeting {
    float *partials;
    unsigned *counters;
};

// Device-coherent accesses to the partial tiles: relaxed atomics at device scope, 8 bytes each.
__device__ __forceinline__ void store_coherent(float *p, f32x2 v)
{
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), __builtin_bit_cast(unsigned long long, v),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ f32x4 load_coherent(const float *p)
{
    const unsigned long long lo = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED,
                                                    __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long hi = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p) + 1,
                                                    __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const f32x2 a = __builtin_bit_cast(f32x2, lo), b = __builtin_bit_cast(f32x2, hi);
    return f32x4{a[0], a[1], b[0], b[1]};
}

template <class T>
__global__ __launch_bounds__(T::NT)
__attribute__((amdgpu_waves_per_eu(T::WAVES_PER_SIMD, T::WAVES_PER_SIMD))) void sgemm_dma_kernel(
    int M, int N, int K, const float *__restrict__ A, int64_t lda, const float *__restrict__ B,
    int64_t ldb, float *__restrict__ C, int64_t ldc, TileMap tmap,
    int k_per_split, int split_k, int tail_first, int tail_split, Epilogue ep, Meeting meet)
{
    __shared__ __attribute__((aligned(1024))) unsigned char lds[T::LDS_BYTES];
    __shared__ unsigned ticket;
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;

    // 128 x 128 tiles, four workgroups per CU, long reductions: the quarter of the grid a workgroup
    // belongs to sets its waves' priority, so that a CU's four (placed one per quarter) finish
    // one after the other by design rather than by the age of their waves, each epilogue under
    // the others' matrix work (4096^3 946.5 -> 942.4 us, 4000^3 933.2 -> 928.8; with 16 chunks per
    // tile the order costs more than it hides: 4096 x 4096 x 256 78.6 -> 80.8, so not there).
    if constexpr (T::BM == 128 && T::BN == 128 && T::KSETS == 1) {
        if (K >= 2048) {
            const unsigned quarter = gridDim.x / 4, rank = quarter ? blockIdx.x / quarter : 3;
            if (rank == 0) __builtin_amdgcn_s_setprio(3);
            else if (rank == 1) __builtin_amdgcn_s_setprio(2);
            else if (rank == 2) __builtin_amdgcn_s_setprio(1);
        }
    }
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, half = lane >> 5;
    // KSETS > 1: wave set kset takes chunk kset of every step; sw is the wave's index in its set
    const int kset = wave / T::SET_WAVES, sw = wave % T::SET_WAVES;
    const int wrow = (sw / T::WAVES_N) * T::WTM;
    const int wcol = (sw % T::WAVES_N) * T::WTN;

    // Which tile, and which slice of its reduction (the whole of it unless EDGE splits K).
    // Uniform split: tiles x slices workgroups, slice-major (TileMap::locate_cut).  Tail split (tail_split > 1, a one-dimensional
    // grid): the first tail_first workgroups take whole tiles, and each tile after those is
    // cut into tail_split slices whose partial sums are added atomically -- the tiles left
    // over after the last whole round of the CUs then keep every CU busy for a fraction of a
    // tile's time instead of a few CUs for all of it.
    // (without a tail split, tail_first is the index of the launch's first tile: a large
    // output is computed by several launches of one generation of resident workgroups each)
    int wg = (int)blockIdx.x + ((!T::EDGE || tail_split <= 1) ? tail_first : 0), slice = 0,
        slices = T::EDGE ? split_k : 1;
    int kper = k_per_split;
    int cut_tile = wg;  // index of the tile among those whose reduction is cut
    int tm, tn;
    if (T::EDGE && tail_split > 1) {
        if (wg >= tail_first) {
            const int r = wg - tail_first;
            cut_tile = r / tail_split;
            wg = tail_first + cut_tile;
            slice = r % tail_split;
            slices = tail_split;
        } else {
            kper = K;
        }
        tmap.locate(wg, tm, tn);
    } else if (T::EDGE && split_k > 1) {
        cut_tile = tmap.locate_cut(wg, slice, tm, tn);  // uniform split: a one-dimensional grid, slice-major
    } else {
        tmap.locate(wg, tm, tn);
    }
    const int m0 = tm * T::BM, n0 = tn * T::BN;
    const int kbeg = T::EDGE ? slice * kper : 0;
    const int kend = T::EDGE ? (kbeg + kper < K ? kbeg + kper : K) : K;
    constexpr int STEP_K = T::BK * T::KSETS;  // reduction elements per step
    const int nk = (kend - kbeg + STEP_K - 1) / STEP_K;

    // ---- DMA sources ----
    // Every load instruction fills 1 KiB (DWORD: 256 bytes) of the chunk's LDS image, and each
    // lane fetches the global bytes that belong in its slot of it: a 32-bit offset from a scalar
    // base that moves along the reduction.  EDGE forms: kOutOfRange for a row past M or a column
    // past N, and the reduction index of the lane's first element inside a chunk (kin_*) for the
    // test against the end of the slice.
    // LDS images: an operand whose reduction index is contiguous in memory (A, a transposed B)
    // is kept as rows of 64 bytes with the four 16-byte k-groups XOR-swizzled; the other kind
    // (B, a transposed A) as 16 rows of the tile's width.
    uint32_t voff_a[T::A_INSTR], voff_b[T::B_INSTR];
    // (for an operand with the reduction index contiguous kin depends on the instruction only
    // through its row modulo 16: one value with 16-byte loads, four with 4-byte loads)
    constexpr int KIN_C = T::DWORD ? 4 : 1;
    int kin_a[T::A_T ? T::A_INSTR : KIN_C], kin_b[T::B_T ? KIN_C : T::B_INSTR];
    auto ka = [](int q) { return T::A_T ? q : q % KIN_C; };
    auto kb = [](int q) { return T::B_T ? q % KIN_C : q; };
    auto swizzle = [](int r) { return ((r >> 1) ^ (r >> 2)) & 3; };
    // column held by LDS row rho of a transposed B: rows 32 b + i of a wave's 64 hold column 2 i + b
    auto perm = [](int rho) { return (rho & ~63) + 2 * (rho & 31) + ((rho >> 5) & 1); };
    // an operand stored with the reduction index contiguous: row (or permuted column) `line` of the tile
    static_assert(!T::DWORD || (T::A_INSTR % 4 == 0 && T::B_INSTR % 4 == 0), "a wave's 4-byte loads start on a 16-row block");
    auto k_contiguous = [&](int instr, int64_t ld, int extent0, int extent, bool permuted, uint32_t &voff, int &kin) {
        int line, g;
        if constexpr (T::DWORD) {
            line = instr * 4 + (lane >> 4);
            g = ((lane & 15) >> 2) ^ swizzle(line & 15);
            kin = g * 4 + (lane & 3);
        } else {
            line = instr * 16 + (lane >> 2);
            g = (lane & 3) ^ swizzle(line & 15);
            kin = g * 4;
        }
        if (permuted) line = perm(line);
        voff = (uint32_t)(((int64_t)line * ld + kin) * 4);
        if (T::EDGE && extent0 + line >= extent) voff = kOutOfRange;
    };
    // an operand stored with the tile's other index contiguous: 16 rows of `width` floats
    auto k_strided = [&](int instr, int width, int64_t ld, int extent0, int extent, uint32_t &voff, int &kin) {
        int x;
        if constexpr (T::DWORD) {
            const int e = instr * 64 + lane;
            kin = e / width;
            x = e % width;
        } else {
            const int lanes_per_row = width / 4;
            kin = instr * (256 / width) + lane / lanes_per_row;
            x = (lane % lanes_per_row) * 4;
        }
        voff = (uint32_t)(((int64_t)kin * ld + x) * 4);
        if (T::EDGE && extent0 + x >= extent) voff = kOutOfRange;
    };
#pragma unroll
    for (int q = 0; q < T::A_INSTR; ++q) {
        if constexpr (T::A_T) k_strided(sw * T::A_INSTR + q, T::BM, lda, m0, M, voff_a[q], kin_a[ka(q)]);
        else k_contiguous(sw * T::A_INSTR + q, lda, m0, M, false, voff_a[q], kin_a[ka(q)]);
    }
#pragma unroll
    for (int q = 0; q < T::B_INSTR; ++q) {
        if constexpr (T::B_T) k_contiguous(sw * T::B_INSTR + q, ldb, n0, N, true, voff_b[q], kin_b[kb(q)]);
        else k_strided(sw * T::B_INSTR + q, T::BN, ldb, n0, N, voff_b[q], kin_b[kb(q)]);
    }
    const int kfirst = kbeg + kset * T::BK;  // this wave set's chunk of the first step
    uint64_t sbase_a = (uint64_t)(uintptr_t)(T::A_T ? A + (int64_t)kfirst * lda + m0 : A + (int64_t)m0 * lda + kfirst);
    uint64_t sbase_b = (uint64_t)(uintptr_t)(T::B_T ? B + (int64_t)n0 * ldb + kfirst : B + (int64_t)kfirst * ldb + n0);
    const uint64_t astep = T::A_T ? (uint64_t)lda * (STEP_K * 4) : (uint64_t)(STEP_K * 4);
    const uint64_t bstep = T::B_T ? (uint64_t)(STEP_K * 4) : (uint64_t)ldb * (STEP_K * 4);
    int kcur = kfirst;  // first k of the next chunk to request (EDGE form)

    auto issue = [&](int stage) {
        const uint32_t dst_a = lds_base + stage * T::STAGE_BYTES + kset * T::CHUNK_BYTES + sw * T::A_INSTR * T::INSTR_BYTES;
        const uint32_t dst_b = lds_base + stage * T::STAGE_BYTES + kset * T::CHUNK_BYTES + T::A_BYTES +
                               sw * T::B_INSTR * T::INSTR_BYTES;
        if constexpr (T::EDGE) {
            const i32x4 buf_a = make_buffer((const void *)sbase_a), buf_b = make_buffer((const void *)sbase_b);
            auto load = [](i32x4 buf, uint32_t voff, uint32_t dst) {
                if constexpr (T::DWORD) dma4_buf(buf, voff, dst); else dma16_buf(buf, voff, dst);
            };
            // only the chunk that crosses the end of the slice tests its lanes against it
            // (vector instructions take matrix-pipe time; a whole chunk needs none)
            if (kcur + T::BK <= kend) {
#pragma unroll
                for (int q = 0; q < T::A_INSTR; ++q) load(buf_a, voff_a[q], dst_a + q * T::INSTR_BYTES);
#pragma unroll
                for (int q = 0; q < T::B_INSTR; ++q) load(buf_b, voff_b[q], dst_b + q * T::INSTR_BYTES);
            } else {
#pragma unroll
                for (int q = 0; q < T::A_INSTR; ++q)
                    load(buf_a, kcur + kin_a[ka(q)] < kend ? voff_a[q] : kOutOfRange, dst_a + q * T::INSTR_BYTES);
#pragma unroll
                for (int q = 0; q < T::B_INSTR; ++q)
                    load(buf_b, kcur + kin_b[kb(q)] < kend ? voff_b[q] : kOutOfRange, dst_b + q * T::INSTR_BYTES);
            }
            kcur += STEP_K;
        } else {
#pragma unroll
            for (int q = 0; q < T::A_INSTR; ++q) dma16(sbase_a, voff_a[q], dst_a + q * 1024);
#pragma unroll
            for (int q = 0; q < T::B_INSTR; ++q) dma16(sbase_b, voff_b[q], dst_b + q * 1024);
        }
        sbase_a += astep;
        sbase_b += bstep;
    };

    // ---- fragment read offsets inside a stage ----
    const int fsw = swizzle(li);  // rows of a block differ from li by multiples of 32
    // k-contiguous images: the lane's row, k-groups half (k 0..7) and 2 + half (k 8..15)
    const uint32_t a_off0 = (uint32_t)((wrow + li) * 64 + ((half ^ fsw) * 16));
    const uint32_t a_off1 = (uint32_t)((wrow + li) * 64 + (((2 + half) ^ fsw) * 16));
    const uint32_t bt_off0 = (uint32_t)(T::A_BYTES + (wcol + li) * 64 + ((half ^ fsw) * 16));
    const uint32_t bt_off1 = (uint32_t)(T::A_BYTES + (wcol + li) * 64 + (((2 + half) ^ fsw) * 16));
    // k-strided images: row 4 half of the chunk, the lane's TM rows / TN columns of the tile
    const uint32_t at_off = (uint32_t)(half * 4 * T::BM * 4 + (wrow + T::TM * li) * 4);
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
        f32x4 af[2][T::A_T ? 1 : T::TM];                        // [u][block row], element t
        typename FVec<T::TM>::type aft[2][T::A_T ? 4 : 1];     // [u][t], element = block row
        f32x2 bf[2][T::B_T ? 1 : 4];                            // [u][t], element = block column
        f32x4 bft[2][T::B_T ? T::TN : 1];                       // [u][block column], element t
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if constexpr (T::A_T) {
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    aft[u][t] = *reinterpret_cast<const typename FVec<T::TM>::type *>(st + at_off + (8 * u + t) * T::BM * 4);
            } else {
#pragma unroll
                for (int a = 0; a < T::TM; ++a)
                    af[u][a] = *reinterpret_cast<const f32x4 *>(st + (u ? a_off1 : a_off0) + a * 32 * 64);
            }
            if constexpr (T::B_T) {
#pragma unroll
                for (int b = 0; b < T::TN; ++b)
                    bft[u][b] = *reinterpret_cast<const f32x4 *>(st + (u ? bt_off1 : bt_off0) + b * 32 * 64);
            } else {
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    bf[u][t] = *reinterpret_cast<const f32x2 *>(st + b_off + (8 * u + t) * T::BN * 4);
            }
        }
        between();
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int a = 0; a < T::TM; ++a)
#pragma unroll
                    for (int b = 0; b < T::TN; ++b) {
                        float x, y;
                        if constexpr (T::A_T) x = vec_get<T::TM>(aft[u][t], a); else x = af[u][a][t];
                        if constexpr (T::B_T) y = bft[u][b][t]; else y = bf[u][t][b];
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(x, y, acc[a][b], 0, 0, 0);
                    }
    };

    // C tile of this lane: two adjacent columns per (block row a, register v).  Row inside the
    // workgroup tile: block rows are 32 apart, or interleaved when A arrives transposed.
    const int col = n0 + wcol + 2 * li;
    auto tile_row = [&](int a, int v) {
        const int i = 8 * (v >> 2) + 4 * half + (v & 3);  // row inside the 32 x 32 block
        return T::A_T ? wrow + T::TM * i + a : wrow + 32 * a + i;
    };
    auto c_ptr = [&](int a, int v) {
        return reinterpret_cast<f32x2 *>(C + (int64_t)(m0 + tile_row(a, v)) * ldc + col);
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

    // partial sums of several workgroups meet in the caller's memory (uniform over the workgroup)
    const bool meeting = T::EDGE && slices > 1 && meet.partials != nullptr;

    // KSETS > 1, tiles whose epilogue all waves share: wave w owns rows w ROWS .. of the tile,
    // one column per lane (see there).  When the call accumulates, the old values of those
    // elements are requested ahead of the first chunks and arrive with them; rows past M and
    // columns past N are clamped rather than skipped (no divergence at the head of the kernel).
    constexpr int ROWS = T::KSETS > 1 ? T::BM / T::NWAVES : 1;
    const int row0 = m0 + wave * ROWS, ccol = n0 + lane;
    // whole tile inside the matrix, C accessible as float2, no partial sums
    const bool whole = m0 + T::BM <= M && n0 + T::BN <= N && (((uintptr_t)C | (uintptr_t)(ldc * 4)) & 7) == 0 &&
                       (ep.pre != kPreBias || ((uintptr_t)ep.bias & 7) == 0);
    // the epilogue with all waves: atomic adds and tiles on the matrix edge, and with four wave
    // sets (outputs of a tile or two per CU, where nothing else covers the epilogue) every tile
    // (1000^3 21.4 -> 20.8 us, 896^3 18.8 -> 18.3; with two sets and nine tiles per CU the first
    // set alone is ahead: 3072^3 425 against 435 us)
    const bool by_rows = T::KSETS > 1 && !meeting && (slices > 1 || !whole || T::KSETS == 4);
    const bool late_c = by_rows && slices == 1 && ep.pre == kPreAccumulate;
    float init[ROWS];
    auto request_c = [&]() {
        if constexpr (T::KSETS > 1) {
            if (!late_c) return;
            const float *src = C + (ccol < N ? ccol : N - 1);
#pragma unroll
            for (int rr = 0; rr < ROWS; ++rr) init[rr] = src[(int64_t)(row0 + rr < M ? row0 + rr : M - 1) * ldc];
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
    request_c();  // (ahead of the first chunks: the first wait covers it)
#pragma unroll
    for (int p = 0; p < T::NSTAGE - 1; ++p)
        if (p < nk) issue(p);
    if (nk > 0) step(0, std::integral_constant<int, 0>{}, std::true_type{});
    for (int it = 1; it < nk; it += T::NSTAGE)
        static_for<T::NSTAGE>([&](auto s_c) {
            constexpr int s = decltype(s_c)::value;
            if (it + s < nk) step(it + s, std::integral_constant<int, (s + 1) % T::NSTAGE>{}, std::false_type{});
        });

    float *const tile_parts = meeting ? meet.partials + (int64_t)cut_tile * slices * T::TILE : nullptr;

    if constexpr (T::KSETS > 1) {
        // ---- the wave sets' partial tiles meet in LDS ----
        static_assert(T::BN == 64 && T::TM == 1 && T::WAVES_N == 1, "one column per lane, 32 rows per wave of a set");
        static_assert(ROWS == 8 || ROWS == 16, "a wave's rows lie in one block row and start on a multiple of eight");
        constexpr int WAVE_UNITS = T::TN * 4 * 64;  // 16-byte units of a wave's partial tile
        f32x4 *const part = reinterpret_cast<f32x4 *>(lds);
        lds_barrier();  // every wave is through with the last chunks
        if (by_rows) {
            // Atomic adds, tiles on the matrix edge, every tile of the four-set kernels: every wave
            // takes part in the epilogue.
            // All waves put their accumulators into the ring's LDS; then wave w owns rows
            // w ROWS .. w ROWS + ROWS - 1 of the tile with one column per lane, adds the sets'
            // values for them in set order (deterministic) and adds them to C atomically, or to
            // the old values requested during the last steps.  Every global access is then a whole
            // row of the tile, 256 contiguous bytes per instruction, from all waves at once: the
            // atomic adds touch each line once instead of twice, and an edge tile pays no round
            // trip to memory at all.  (Left to the first set alone, with its two columns per lane
            // and element-wise tests, the atomic adds of 256 x 256 x 8192 took 8 of 21 us and the
            // edge tiles of 1000^3 held the kernel 6 us beyond its interior tiles.)
            // Layout, in 16-byte units: [wave][q][half][block column b][position], a unit holding
            // the registers 4 q .. 4 q + 3 of one lane, i.e. the rows 8 q + 4 half + 0..3 of one
            // column; the lane that holds column 2 j + b writes to position (j + 8 b) mod 32, so
            // that the 16 lanes of a pass, reading consecutive columns, fall into distinct banks.
            {
                f32x4 *mine = part + wave * WAVE_UNITS + half * 64;
#pragma unroll
                for (int b = 0; b < T::TN; ++b)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        mine[q * 128 + b * 32 + ((li + 8 * b) & 31)] =
                            f32x4{acc[0][b][4 * q], acc[0][b][4 * q + 1], acc[0][b][4 * q + 2], acc[0][b][4 * q + 3]};
            }
            lds_barrier();
            float val[ROWS];
            {
                const int cb = lane & 1, cj = lane >> 1;
                const int r0 = wave * ROWS;  // first row; r0 % 8 == 0
                const f32x4 *src = part + (r0 / 32) * WAVE_UNITS + ((r0 % 32) >> 3) * 128 + cb * 32 + ((cj + 8 * cb) & 31);
#pragma unroll
                for (int g = 0; g < ROWS / 4; ++g) {
                    // rows 4 g .. 4 g + 3 of the wave's: q advances every eight rows, half every four
                    const int off = (g >> 1) * 128 + (g & 1) * 64;
                    f32x4 sum = src[off];
#pragma unroll
                    for (int s = 1; s < T::KSETS; ++s) sum += src[s * T::SET_WAVES * WAVE_UNITS + off];
#pragma unroll
                    for (int e = 0; e < 4; ++e) val[4 * g + e] = sum[e];
                }
            }
            float *const dst = C + (int64_t)row0 * ldc + ccol;
            if (slices > 1) {
#pragma unroll
                for (int rr = 0; rr < ROWS; ++rr)
                    if (row0 + rr < M && ccol < N) atomicAdd(dst + rr * ldc, val[rr]);  // plain accumulate form only
            } else {
                if (!late_c) {
                    const float bias = (ep.pre == kPreBias && ccol < N) ? ep.bias[ccol] : 0.f;
#pragma unroll
                    for (int rr = 0; rr < ROWS; ++rr) init[rr] = bias;
                }
#pragma unroll
                for (int rr = 0; rr < ROWS; ++rr)
                    if (row0 + rr < M && ccol < N) dst[rr * ldc] = apply_post(init[rr] + val[rr], ep.post);
            }
            return;
        }
        // Whole tiles of the two-set kernels, and partial tiles on their way to the workspace: the
        // other sets hand their accumulators to the first ([set][wave][register][lane],
        // conflict-free), which goes on alone with its two columns per lane.
        constexpr int WAVE_FLOATS = T::TM * T::TN * 16 * 64;
        float *const fpart = reinterpret_cast<float *>(lds) + sw * WAVE_FLOATS;
        if (kset > 0) {
            float *mine = fpart + (kset - 1) * T::SET_WAVES * WAVE_FLOATS;
#pragma unroll
            for (int b = 0; b < T::TN; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) mine[(b * 16 + v) * 64 + lane] = acc[0][b][v];
        }
        lds_barrier();
        if (kset > 0 && !meeting) return;
        if (kset == 0) {
#pragma unroll
            for (int s = 1; s < T::KSETS; ++s)
#pragma unroll
                for (int b = 0; b < T::TN; ++b)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        acc[0][b][v] += fpart[(s - 1) * T::SET_WAVES * WAVE_FLOATS + (b * 16 + v) * 64 + lane];
        }
    }

    if (meeting) {
        // ---- the slices of a cut tile meet in memory ----
        // The workgroups of a tile run on different XCDs, each with an L2 of its own, so the
        // partial tiles are written and read with device-coherent accesses (relaxed atomic
        // stores and loads at device scope: they go through to memory and are not served from
        // a stale line), 8 bytes each.  A fence at device scope would do as well, but it writes
        // back and invalidates the whole L2 for every wave that executes it: measured, the
        // kernel then took 0.1 us longer per workgroup in the grid.  Order: every wave waits for
        // its own stores to be acknowledged, the barrier joins the waves, then one thread counts
        // the workgroup's arrival; whoever draws the last ticket reads only after that.
        if (kset == 0) {
            float *mine = tile_parts + (int64_t)slice * T::TILE + wcol + 2 * li;
#pragma unroll
            for (int a = 0; a < T::TM; ++a)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    store_coherent(mine + tile_row(a, v) * T::BN, f32x2{acc[a][0][v], acc[a][1][v]});
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) ticket = atomicAdd(meet.counters + cut_tile, 1u);
        __syncthreads();
        if (ticket != (unsigned)(slices - 1)) return;
        if (tid == 0) meet.counters[cut_tile] = 0;  // as the next launch expects it
        const bool c16 = (((uintptr_t)C | (uintptr_t)(ldc * 4)) & 15) == 0;
        constexpr int GROUPS = T::TILE / 4 / T::NT;  // 16-byte groups per thread
        // All loads of a batch of slices are in flight before the first is used: the partial
        // tiles come from memory, a round trip each, and the workgroups that still wait for
        // this one's tile have nothing else to do.  Sixteen slices at a time, of two groups for
        // kernels with the registers of two waves per SIMD, of one for the others.
        constexpr int JB = (T::WAVES_PER_SIMD <= 2 && GROUPS % 2 == 0) ? 2 : 1;
        constexpr int SB = T::WAVES_PER_SIMD <= 2 ? 16 : 8;
#pragma unroll 1
        for (int j0 = 0; j0 < GROUPS; j0 += JB) {
            // the old values of C (or the bias) are requested with the first batch
            float *dst[JB];
            bool wide[JB];
            f32x4 init[JB];
            int cols[JB];  // columns of the group inside the matrix, 0 when its row is past M
#pragma unroll
            for (int jj = 0; jj < JB; ++jj) {
                const int e = (tid + (j0 + jj) * T::NT) * 4;  // first element of the group inside the tile
                const int row = m0 + e / T::BN, c0 = n0 + e % T::BN;
                cols[jj] = row < M ? (N - c0 < 4 ? (N - c0 > 0 ? N - c0 : 0) : 4) : 0;
                dst[jj] = C + (int64_t)row * ldc + c0;
                wide[jj] = c16 && cols[jj] == 4;
                init[jj] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (wide[jj] && ep.pre == kPreAccumulate) {
                    init[jj] = *reinterpret_cast<const f32x4 *>(dst[jj]);
                } else {
#pragma unroll
                    for (int x = 0; x < 4; ++x)
                        if (x < cols[jj])
                            init[jj][x] = ep.pre == kPreAccumulate ? dst[jj][x] : ep.pre == kPreBias ? ep.bias[c0 + x] : 0.f;
                }
            }
            f32x4 sums[JB];
            for (int s0 = 0; s0 < slices; s0 += SB) {
                f32x4 p[JB][SB];
#pragma unroll
                for (int jj = 0; jj < JB; ++jj)
#pragma unroll
                    for (int u = 0; u < SB; ++u)
                        if (s0 + u < slices)
                            p[jj][u] = load_coherent(tile_parts + (tid + (j0 + jj) * T::NT) * 4 + (int64_t)(s0 + u) * T::TILE);
#pragma unroll
                for (int jj = 0; jj < JB; ++jj)
#pragma unroll
                    for (int u = 0; u < SB; ++u)
                        if (s0 + u < slices) sums[jj] = (s0 + u == 0) ? p[jj][u] : sums[jj] + p[jj][u];
            }
#pragma unroll
            for (int jj = 0; jj < JB; ++jj) {
                f32x4 out;
#pragma unroll
                for (int x = 0; x < 4; ++x) out[x] = apply_post(init[jj][x] + sums[jj][x], ep.post);
                if (wide[jj]) {
                    *reinterpret_cast<f32x4 *>(dst[jj]) = out;
                } else {
#pragma unroll
                    for (int x = 0; x < 4; ++x)
                        if (x < cols[jj]) dst[jj][x] = out[x];
                }
            }
        }
        return;
    }

    // ---- epilogue: C = post(pre(C) + acc) ----
    bool vec = true;
    if constexpr (T::EDGE) vec = slices == 1 && whole;
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
                const int row = m0 + tile_row(a, v);
                float *dst = C + (int64_t)row * ldc + col;
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    if (row < M && col + b < N) atomicAdd(dst + b, acc[a][b][v]);  // plain accumulate form only
            }
    } else {
        // Tiles on the matrix edge: element by element through a buffer descriptor over the
        // tile's part of C.  An element past M or N gets an out-of-range offset, for which a load
        // returns zero and a store does nothing, so every lane issues the same instructions and
        // the old values of a batch are all in flight before the first is used.  (Written as
        // tests around plain loads and stores, every element became a branch with a round trip
        // to memory of its own: the 63 edge tiles of 4000 x 4000 x 64 ended 15 us after the other
        // 961.)  Offsets are 32-bit: BM rows of ldc floats stay below 2^31 bytes (host check).
        const __amdgpu_buffer_rsrc_t cbuf = __builtin_amdgcn_make_buffer_rsrc(
            C + (int64_t)m0 * ldc + n0, 0, (int)kOutOfRange, 0x00020000);
        const int rows_in = M - m0, lc = wcol + 2 * li, cols_in = N - n0 - lc;  // rows of the tile, columns from this lane's on
        float bias[2] = {0.f, 0.f};
        if (ep.pre == kPreBias) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
                if (b < cols_in) bias[b] = ep.bias[n0 + lc + b];
        }
        constexpr int BATCH = 8;
#pragma unroll
        for (int a = 0; a < T::TM; ++a)
#pragma unroll
            for (int v0 = 0; v0 < 16; v0 += BATCH) {
                uint32_t off[BATCH][2];
                float c[BATCH][2];
#pragma unroll
                for (int v = 0; v < BATCH; ++v) {
                    const int r = tile_row(a, v0 + v);
                    const uint32_t o = (uint32_t)r * (uint32_t)(ldc * 4) + (uint32_t)(lc * 4);
#pragma unroll
                    for (int b = 0; b < 2; ++b) {
                        off[v][b] = (r < rows_in && b < cols_in) ? o + 4 * b : kOutOfRange;
                        c[v][b] = bias[b];
                        if (ep.pre == kPreAccumulate)
                            c[v][b] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(cbuf, (int)off[v][b], 0, 0));
                    }
                }
#pragma unroll
                for (int v = 0; v < BATCH; ++v)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        __builtin_amdgcn_raw_buffer_store_b32(
                            __builtin_bit_cast(unsigned, apply_post(c[v][b] + acc[a][b][v0 + v], ep.post)), cbuf,
                            (int)off[v][b], 0, 0);
            }
    }
}

}  // namespace lsmi
