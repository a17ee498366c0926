// Signed 8-bit GEMM for large aligned outputs (gfx950): 256 x 256 tiles, four waves of
// 128 x 128, one workgroup per CU, one wave per SIMD.
//
// V_MFMA_I32_32X32X32_I8 takes 32 cycles for 65536 operations, eight times the rate of the
// fp32 instruction, so everything around it has to shrink by as much per instruction.  A
// 64 x 64 wave tile reads 1 KiB from LDS per matrix instruction and a 128-row tile brings
// 1.5 - 2 KiB per instruction in from L2; with 128 x 128 per wave (256 accumulator registers,
// which is why a SIMD holds one wave) both halve.  With one wave per SIMD nothing hides a
// wave's latencies but its own instruction order, so the loop is scheduled by hand and pinned
// with scheduling barriers:
//   * a chunk is 64 reduction bytes = two groups of 32; each group is 16 matrix instructions
//     on fragments that were read from LDS while the previous group was multiplied;
//   * the LDS reads of the next group and the direct-to-LDS loads of the chunks NSTAGE - 1 and
//     NSTAGE ahead are placed one by one between the matrix instructions, which issue in 4
//     of their 32 cycles and leave the rest to them; the loads are spread over the whole step;
//   * the wait for the next chunk's loads and the workgroup barrier sit behind the first four
//     matrix instructions of a chunk's second group, whose operands are in registers already,
//     so the matrix pipe has work queued while the waves meet.
// Every step issues the same eight loads per wave (past the end of the reduction the last
// chunk is requested again into a stage nobody reads), so the load counter is uniform and the
// loop has no branches but its own.
//
// LDS image of a stage: A as 256 rows of 64 bytes with the 16-byte k-groups of row r at slot
// g ^ ((r >> 2) & 3) (the conflict-free layout of the 64-byte chunks of igemm_dma.hpp); B given
// k-contiguous (N x K) likewise; B given n-contiguous (K x N) as two panels of 64 rows x 128
// bytes in the transpose-read layout of igemm_dma.hpp.
#pragma once

#include "igemm_dma.hpp"

namespace lsmi {

// BN = 128: the same loop on 256 x 128 tiles, four waves of 128 x 64 with 128 accumulator
// registers each, so that two workgroups share a CU (three stages of 24 KiB each) and one
// multiplies while the other reads and writes its C tile: with 256 accumulator registers a
// SIMD holds one wave, and at 4096^3 a third of the kernel's time was that epilogue with the
// matrix pipes idle.
template <int NSTAGE_, bool B_KMAJOR_, int BN_ = 256>
struct IBigShape {
    static constexpr bool B_KMAJOR = B_KMAJOR_;
    static constexpr int BM = 256, BN = BN_, BK = 64, NSTAGE = NSTAGE_;
    static constexpr int NWAVES = 4, NT = 256, TM = 4, TN = BN / 64;
    static constexpr int WAVES_PER_SIMD = BN == 256 ? 1 : 2;
    static_assert(BN == 256 || BN == 128, "two or one panel of 128 columns");
    static constexpr int A_BYTES = BM * BK, B_BYTES = BN * BK, STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;
    static constexpr int A_PER_WAVE = A_BYTES / 1024 / NWAVES, B_PER_WAVE = B_BYTES / 1024 / NWAVES;
    static constexpr int LOADS = A_PER_WAVE + B_PER_WAVE;
    // LDS read instructions per group of 32: four A fragments, four B fragments (two transpose
    // reads each when B is n-contiguous)
    static constexpr int READS = TM + (B_KMAJOR ? TN : 2 * TN);
    static_assert(NSTAGE >= 2 && LDS_BYTES <= 160 * 1024 && LOADS * (NSTAGE - 1) <= 63, "ring depth");

    __host__ __device__ static constexpr int a_slot(int g, int r) { return g ^ ((r >> 2) & 3); }
};

template <class T>
__global__ __launch_bounds__(T::NT) __attribute__((amdgpu_waves_per_eu(T::WAVES_PER_SIMD, T::WAVES_PER_SIMD))) void igemm_big_kernel(
    int K, const int8_t *__restrict__ A, int64_t lda, const int8_t *__restrict__ B, int64_t ldb,
    int32_t *__restrict__ C, int64_t ldc, TileMap tmap)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char blds[];
    const uint32_t lds_base = (uint32_t)(uintptr_t)blds;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, half = lane >> 5;
    const int wrow = (wave >> 1) * 128, wcol = (wave & 1) * (T::BN / 2);

    int tm, tn;
    tmap.locate(blockIdx.x, tm, tn);
    const int m0 = tm * T::BM, n0 = tn * T::BN;
    const int nk = K / T::BK;
    // Two workgroups per CU (the 256 x 128 tiles): the first half of the grid gets the matrix
    // pipe whenever it can use it, so that the two workgroups of a CU do not end together --
    // one is in its epilogue, the memory system busy and the matrix pipe free, while the other
    // multiplies.  (Workgroups are placed one per CU in grid order, then the second ones.)
    if constexpr (T::WAVES_PER_SIMD == 2) {
        if (2 * blockIdx.x < gridDim.x) __builtin_amdgcn_s_setprio(3);
    }

    // ---- direct-to-LDS sources: an instruction moves 1 KiB = 16 rows of 64 bytes (A, k-major B)
    // or 8 rows of 128 bytes (one panel of n-major B); lane -> (row, slot) ----
    uint32_t voff_a[T::A_PER_WAVE], voff_b[T::B_PER_WAVE];
#pragma unroll
    for (int q = 0; q < T::A_PER_WAVE; ++q) {
        const int row = (wave * T::A_PER_WAVE + q) * 16 + (lane >> 2);
        voff_a[q] = (uint32_t)((int64_t)row * lda + T::a_slot(lane & 3, row) * 16);
    }
#pragma unroll
    for (int q = 0; q < T::B_PER_WAVE; ++q) {
        const int t = wave * T::B_PER_WAVE + q;
        if constexpr (T::B_KMAJOR) {
            const int row = t * 16 + (lane >> 2);
            voff_b[q] = (uint32_t)((int64_t)row * ldb + T::a_slot(lane & 3, row) * 16);
        } else {
            const int panel = t >> 3, krow = (t & 7) * 8 + (lane >> 3);
            voff_b[q] = (uint32_t)((int64_t)krow * ldb + 128 * panel + (((lane & 7) ^ (krow & 7)) * 16));
        }
    }
    const uint64_t base_a = (uint64_t)(uintptr_t)(A + (int64_t)m0 * lda);
    const uint64_t base_b =
        T::B_KMAJOR ? (uint64_t)(uintptr_t)(B + (int64_t)n0 * ldb) : (uint64_t)(uintptr_t)(B + n0);
    const uint64_t step_b = T::B_KMAJOR ? (uint64_t)T::BK : (uint64_t)ldb * T::BK;

    // load q (0 .. LOADS-1) of chunk `chunk` (clamped to the last one) into `stage`
    auto issue_one = [&](int chunk, int stage, auto q_c) {
        constexpr int q = decltype(q_c)::value;
        const int cc = chunk < nk ? chunk : nk - 1;
        const uint32_t dst = lds_base + stage * T::STAGE_BYTES;
        if constexpr (q < T::A_PER_WAVE)
            dma16(base_a + (uint64_t)cc * T::BK, voff_a[q], dst + (wave * T::A_PER_WAVE + q) * 1024);
        else
            dma16(base_b + (uint64_t)cc * step_b, voff_b[q - T::A_PER_WAVE],
                  dst + T::A_BYTES + (wave * T::B_PER_WAVE + (q - T::A_PER_WAVE)) * 1024);
    };

    // ---- fragment reads ----
    struct Frags {
        i32x4 a[T::TM], b[T::TN];
    };
    typedef __attribute__((address_space(3))) i32x2v lds_i32x2;
    const int jl = lane & 15;
    const uint32_t a_lane = (uint32_t)((wrow + li) * T::BK);
    const uint32_t bk_lane = (uint32_t)(T::A_BYTES + (wcol + li) * T::BK);           // k-major B
    const uint32_t bn_panel = (uint32_t)(T::A_BYTES + (wcol >> 7) * (T::BK * 128));   // n-major B
    // read r (0 .. READS-1) of the fragments of 32-group u of `stage`
    auto read_one = [&](Frags &f, int stage, auto u_c, auto r_c) {
        constexpr int u = decltype(u_c)::value, r = decltype(r_c)::value;
        const unsigned char *st = blds + stage * T::STAGE_BYTES;
        if constexpr (r < T::TM) {
            f.a[r] = *reinterpret_cast<const i32x4 *>(st + a_lane + r * 32 * T::BK + T::a_slot(2 * u + half, li) * 16);
        } else if constexpr (T::B_KMAJOR) {
            constexpr int b = r - T::TM;
            f.b[b] = *reinterpret_cast<const i32x4 *>(st + bk_lane + b * 32 * T::BK + T::a_slot(2 * u + half, li) * 16);
        } else {
            // block column b, part j: this lane points at k row 32u + 8j + 16half + (lane%16)/2,
            // bytes 8*(lane&1) of the 16-byte column group 2b + (lane/16)%2 of its panel
            constexpr int b = (r - T::TM) >> 1, j = (r - T::TM) & 1;
            const int krow = 32 * u + 8 * j + 16 * half + (jl >> 1);
            const int group = ((wcol & 127) >> 4) + 2 * b + ((lane >> 4) & 1);
            const uint32_t off = bn_panel + (uint32_t)(krow * 128) + (uint32_t)(((group ^ (krow & 7)) * 16)) +
                                 (uint32_t)(8 * (jl & 1));
            const i32x2v two = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2 *)(st + off));
            f.b[b][2 * j] = two[0];
            f.b[b][2 * j + 1] = two[1];
        }
    };

    i32x16v acc[T::TM][T::TN];
#pragma unroll
    for (int a = 0; a < T::TM; ++a)
#pragma unroll
        for (int b = 0; b < T::TN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0;
    auto multiply_one = [&](const Frags &f, auto i_c) {
        constexpr int i = decltype(i_c)::value, a = i / T::TN, b = i % T::TN;
        acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.a[a], f.b[b], acc[a][b], 0, 0, 0);
    };

    // ---- prologue: fill the ring but for the late loads of its last stage, which the first
    // step issues; wait for chunk 0, read its first group ----
    // A chunk's loads are spread over a whole step, EARLY of them right behind the barrier
    // that frees their stage and the rest over the next step up to its barrier: the four
    // waves share one address unit that takes about 16 cycles per load, and a burst of 32
    // loads would hold back the matrix instructions queued behind them.
    constexpr int EARLY = 3;
    static_for<T::NSTAGE>([&](auto p_c) {
        constexpr int p = decltype(p_c)::value;
        static_for<(p < T::NSTAGE - 1 ? T::LOADS : EARLY)>([&](auto q_c) { issue_one(p, p, q_c); });
    });
    wait_vmcnt_and_barrier<T::LOADS *(T::NSTAGE - 2) + EARLY>();
    Frags x0, x1;
    static_for<T::READS>([&](auto r_c) { read_one(x0, 0, std::integral_constant<int, 0>{}, r_c); });

    // ---- main loop: chunk c lives in stage c % NSTAGE; x0 holds its first group on entry ----
    constexpr int MM = T::TM * T::TN;  // matrix instructions per group
    constexpr int LATE = T::LOADS - EARLY;
    // behind the barrier MM - 4 matrix instructions are left: the next group's reads and the
    // EARLY loads are spread evenly over them
    constexpr int RPS = (T::READS + MM - 5) / (MM - 4), ISTEP = (MM - 4) / EARLY;
    static_assert(T::READS <= MM && (MM + 1) / 3 >= LATE && ISTEP >= 1, "the schedule's slots");
    for (int c0 = 0; c0 < nk; c0 += T::NSTAGE)
        static_for<T::NSTAGE>([&](auto s_c) {
            constexpr int stage = decltype(s_c)::value;
            const int c = c0 + stage;
            if (c < nk) {
                // first group: multiply x0, read the second group into x1, and finish the loads
                // of chunk c + NSTAGE - 1 (one behind every third matrix instruction)
                static_for<MM>([&](auto i_c) {
                    constexpr int i = decltype(i_c)::value;
                    multiply_one(x0, i_c);
                    if constexpr (i < T::READS)
                        read_one(x1, stage, std::integral_constant<int, 1>{}, std::integral_constant<int, i>{});
                    if constexpr (i % 3 == 1 && i / 3 < LATE)
                        issue_one(c + T::NSTAGE - 1, (stage + T::NSTAGE - 1) % T::NSTAGE,
                                  std::integral_constant<int, EARLY + i / 3>{});
                    __builtin_amdgcn_sched_barrier(0);
                });
                // second group: four matrix instructions queued, then the waves meet: chunk
                // c + 1 has landed and nobody reads this stage any more
                static_for<4>([&](auto i_c) { multiply_one(x1, i_c); });
                __builtin_amdgcn_sched_barrier(0);
                wait_vmcnt_and_barrier<T::LOADS *(T::NSTAGE - 2)>();
                __builtin_amdgcn_sched_barrier(0);
                // the rest of the second group: read the next chunk's first group into x0 and
                // start the loads of chunk c + NSTAGE into the stage just freed
                static_for<MM - 4>([&](auto k_c) {
                    constexpr int k = decltype(k_c)::value;
                    multiply_one(x1, std::integral_constant<int, k + 4>{});
                    static_for<RPS>([&](auto j_c) {
                        constexpr int r = k * RPS + decltype(j_c)::value;
                        if constexpr (r < T::READS)
                            read_one(x0, (stage + 1) % T::NSTAGE, std::integral_constant<int, 0>{},
                                     std::integral_constant<int, r>{});
                    });
                    if constexpr (k % ISTEP == ISTEP - 1 && k / ISTEP < EARLY)
                        issue_one(c + T::NSTAGE, stage, std::integral_constant<int, k / ISTEP>{});
                    __builtin_amdgcn_sched_barrier(0);
                });
            }
        });
    // the ring still receives the repeated last chunk: drain before the LDS is given back
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // ---- epilogue: register v of block (a, b) is row 32a + 8(v/4) + 4half + v%4, column 32b + li ----
    // In batches of half a block row (8 registers x TN block columns).  The old values of a batch
    // are requested before the batch ahead of it is stored: a wait for loads then leaves those
    // stores in flight (the counter retires in order, and they are younger), so the kernel pays
    // one load round trip per batch and the stores drain behind.  Written batch by batch -- load,
    // add, store -- every batch waited for its predecessor's stores as well, and the eight
    // batches of this tile took a third of the kernel's time at 4096^3 with the matrix pipes idle.
    constexpr int BATCHES = 2 * T::TM;
    auto at = [&](int t, int v, int b) {  // batch t = (block row a, half h)
        return C + (int64_t)(m0 + wrow + 32 * (t >> 1) + 16 * (t & 1) + 4 * half + 8 * (v >> 2) + (v & 3)) * ldc + n0 +
               wcol + li + 32 * b;
    };
    uint32_t old[2][8][T::TN];
    auto request = [&](auto t_c) {
        constexpr int t = decltype(t_c)::value;
#pragma unroll
        for (int v = 0; v < 8; ++v)
#pragma unroll
            for (int b = 0; b < T::TN; ++b) old[t & 1][v][b] = (uint32_t)*at(t, v, b);
    };
    request(std::integral_constant<int, 0>{});
    static_for<BATCHES>([&](auto t_c) {
        constexpr int t = decltype(t_c)::value;
        if constexpr (t + 1 < BATCHES) request(std::integral_constant<int, t + 1>{});
#pragma unroll
        for (int v = 0; v < 8; ++v)
#pragma unroll
            for (int b = 0; b < T::TN; ++b)
                *at(t, v, b) = (int32_t)(old[t & 1][v][b] + (uint32_t)acc[t >> 1][b][8 * (t & 1) + v]);
    });
}

}  // namespace lsmi
