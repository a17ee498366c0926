// fp32 GEMM, C += op(A).op(B) (Section 2.1, Fig. 1 with alpha = beta = 1; either operand may be
// stored transposed, the transposition of Section 2.1 taken as the operand's index map), for
// gfx950: the choice of a kernel variant, of the reduction split and of where partial sums
// meet, and the launch.  The kernels are in sgemm_variants.hpp, sgemm_dma.hpp and
// sgemm_rows.hpp; this translation unit also holds the table for the plain layouts.
#include <cmath>
#include <mutex>

#include "sgemm_variants.hpp"

namespace lsmi {

LSMI_DEFINE_SGEMM_TABLE(sgemm_table_nn, false, false, "")

namespace {

constexpr int kNumVariants = kNumSgemmVariants;
constexpr int64_t kCounterBytes = kSgemmCounterBytes;

const Variant *table_of(bool ta, bool tb)
{
    return ta ? (tb ? sgemm_table_tt() : sgemm_table_tn()) : (tb ? sgemm_table_nt() : sgemm_table_nn());
}

// Shapes the direct-to-LDS kernels accept (see sgemm_dma.hpp).  ta / tb: the operand is stored
// transposed, i.e. A is K x M, B is N x K.
bool dma_supported(const Variant &v, bool ta, bool tb, int M, int N, int K, const float *A, int64_t lda,
                   const float *B, int64_t ldb, const float *C, int64_t ldc, const Epilogue &ep)
{
    if (v.launch == nullptr) return false;
    if (v.cols) {
        // a few columns against A as given: A is streamed in 16-byte groups along k; B is read by
        // the element (stored K x N) or in 16-byte groups along k (stored N x K); 32-bit offsets
        const bool b_ok = !tb || ((((uintptr_t)B) & 15) == 0 && ldb % 4 == 0);
        const int64_t span_b = tb ? 16 * ldb * 4 + (int64_t)K * 4 : (int64_t)K * ldb * 4 + 64;
        return !ta && N <= 16 && ep.pre == kPreAccumulate && ep.post == kPostNone && K % 4 == 0 && K >= 4 &&
               (((uintptr_t)A) & 15) == 0 && lda % 4 == 0 && b_ok &&
               64 * lda * 4 + (int64_t)K * 4 < (int64_t)INT32_MAX && span_b < (int64_t)INT32_MAX;
    }
    // (the few-row kernels combine their slices with atomic adds: plain accumulate form only)
    // (32-bit offsets: k rows of B, or with the transposed B a tile's 64 rows and k along them)
    if (v.rows && (ep.pre != kPreAccumulate || ep.post != kPostNone ||
                   (tb ? 64 * ldb * 4 + (int64_t)K * 4 : (int64_t)K * ldb * 4) >= (int64_t)INT32_MAX))
        return false;
    // 32-bit lane offsets: an operand with the reduction index contiguous spans the tile's
    // rows, the other kind the sixteen k-rows of a chunk
    const int64_t span_a = ta ? 16 * lda * 4 + v.bm * 4 : (int64_t)v.bm * lda * 4 + 64;
    const int64_t span_b = tb ? (int64_t)v.bn * ldb * 4 + 64 : 16 * ldb * 4 + v.bn * 4;
    // (a tile on the matrix edge reaches its part of C through 32-bit offsets as well)
    if (v.edge && (int64_t)v.bm * ldc * 4 >= (int64_t)INT32_MAX) return false;
    if (v.dword) return K >= 1 && span_a < (int64_t)INT32_MAX && span_b < (int64_t)INT32_MAX;
    const bool aligned = (((uintptr_t)A | (uintptr_t)B) & 15) == 0 && lda % 4 == 0 && ldb % 4 == 0;
    // a 16-byte group of an operand whose reduction index is contiguous must not straddle K
    const bool k_groups = !ta || tb;
    if (v.edge)
        return aligned && K >= 1 && (!k_groups || K % 4 == 0) && span_a < (int64_t)INT32_MAX &&
               span_b < (int64_t)INT32_MAX;
    if (ep.pre == kPreBias && ((uintptr_t)ep.bias & 7) != 0) return false;
    return M % v.bm == 0 && N % v.bn == 0 && K % 16 == 0 && K >= 16 && aligned &&
           ((uintptr_t)C & 7) == 0 && ldc % 2 == 0 && span_a < (int64_t)UINT32_MAX && span_b < (int64_t)UINT32_MAX;
}

// Slices for the tiles of an incomplete last round (0: none).  `gain_us` is the estimated
// time saved against running those tiles whole.
struct TailPlan {
    int split = 0;
    double gain_us = 0;
    int64_t tiles = 0;  // how many of the last tiles are cut
};

TailPlan plan_tail(const Variant &v, int64_t nt, int chunks, int cus, bool in_workspace)
{
    TailPlan p;
    const int64_t rem = nt % cus, per_cu = nt / cus;
    if (nt <= cus) return p;
    int64_t tiles = rem;
    int s = rem > 0 ? (int)(cus / rem) : 0;
    const int cap = chunks / 4 < 64 ? chunks / 4 : 64;  // at least four chunks per slice
    if (s > cap) s = cap;
    // 128 x 128 tiles, four workgroups resident per CU: tiles beyond a multiple of four per CU start
    // when the others are about to end, and a workgroup of theirs that has its CU to itself runs at
    // half the rate; two half-length ones side by side do not.  So such tiles are cut in two also
    // when they are more than half a round (4992 x 4096 x 2060, 1248 tiles: 712 us whole, 609 so)
    // or a whole one (5120 x 4096 x 2060, five per CU: 716 us, 622 so; 4736 x 4544 x 5352, 5.2 per CU).
    bool pairs = false;
    // (not the eight-wave form, two per CU: a workgroup of eight waves that has its CU to itself keeps
    // two waves on every SIMD)
    if (v.bm >= 128 && v.per_cu == 4 && cap >= 2) {
        if (rem > 0 && s < 2 && per_cu % 4 == 0) pairs = true;
        if (per_cu % 4 == 1 && per_cu > 1) {  // (and what is left over beyond the fifth with it)
            pairs = true;
            tiles = cus + rem;
        }
    }
    if (pairs) s = 2;
    if (s < 2 || tiles == 0) return p;
    const double chunk_us = 2.0 * v.bm * v.bn * v.bk / 0.47e6;
    // the slices' partial sums meet in atomic adds at about 0.7 TB/s (1.5 where all waves of a
    // workgroup add whole rows), or in the caller's workspace
    const double bytes = 4.0 * v.bm * v.bn * tiles * s;
    const double meet_us = in_workspace ? 1.0 + 0.5 * s + bytes / 6.0e6 : bytes / (v.ksets > 1 ? 1.5e6 : 0.7e6);
    const int per = (chunks + s - 1) / s;
    const double gain = (pairs ? 0.6 * chunk_us * chunks : chunk_us * (chunks - per)) - meet_us;
    if (gain <= 0) return p;
    p.split = s;
    p.gain_us = gain;
    p.tiles = tiles;
    return p;
}

}  // namespace

int sgemm_variant_count() { return kNumVariants; }

const char *sgemm_variant_name(int index)
{
    return (index >= 0 && index < kNumVariants) ? sgemm_table_nn()[index].name : nullptr;
}

uint32_t fast_divide(uint32_t n, uint32_t d) { return FastDiv(d).div(n); }

void tile_of_workgroup(int wg, int tiles_m, int tiles_n, int group_m, int *tm, int *tn)
{
    TileMap(tiles_m, tiles_n, group_m).locate(wg, *tm, *tn);  // the kernels' form of the walk
}

namespace {

// What a call would do, for a caller that first asks and launches nothing: the uniform cut of
// the reduction, and for the 64 x 64 kernels with wave sets the fitted time of the call with
// that cut and with the reduction whole (0 for the other kernels).
struct CutPlan {
    int slices = 1;
    double cut_us = 0, whole_us = 0;
};

// C[i, j] = bias[j] (or 0 without a bias) for i < M, j < N: pre(C) ahead of a cut reduction
// whose slices then add onto it.
__global__ __launch_bounds__(256) void sgemm_init_kernel(float *__restrict__ C, int64_t ldc, int M, int N,
                                                         const float *__restrict__ bias)
{
    const int j = (int)blockIdx.x * 256 + (int)threadIdx.x;
    if (j >= N) return;
    const float v = bias ? bias[j] : 0.f;
    for (int i = (int)blockIdx.y; i < M; i += (int)gridDim.y) C[(int64_t)i * ldc + j] = v;
}

// C = max(C, 0) in place: the post-operation behind a cut reduction.
__global__ __launch_bounds__(256) void sgemm_relu_kernel(float *__restrict__ C, int64_t ldc, int M, int N)
{
    const int j = (int)blockIdx.x * 256 + (int)threadIdx.x;
    if (j >= N) return;
    for (int i = (int)blockIdx.y; i < M; i += (int)gridDim.y) {
        float *const c = C + (int64_t)i * ldc + j;
        *c = fmaxf(*c, 0.f);
    }
}

int launch_sgemm_planned(int M, int N, int K, const float *A, int64_t lda, const float *B, int64_t ldb,
                         float *C, int64_t ldc, const float *bias, int pre, int post, bool ta, bool tb,
                         void *workspace, int64_t workspace_bytes, bool no_atomics, int64_t *plan_bytes,
                         CutPlan *plan_only);

}  // namespace

int launch_sgemm(int M, int N, int K, const float *A, int64_t lda, const float *B, int64_t ldb,
                 float *C, int64_t ldc, const float *bias, int pre, int post, bool ta, bool tb,
                 void *workspace, int64_t workspace_bytes, bool no_atomics, int64_t *plan_bytes)
{
    // A pre- or post-operation on a small output with a long reduction (a fully connected layer
    // with bias and ReLU at a small batch: 64 x 1024 x 4096, 16 tiles).  In one kernel every
    // element's reduction would have to stay in one workgroup, on a sixteenth of the CUs (66.7 us
    // against 10.6 for the plain product, 256 x 256 x 8192 130 against 14.5).  Where the plain
    // form would cut the reduction and gain more than the two small launches cost, the call runs
    // as pre(C) written out, the plain product with its slices added onto that, and post in
    // place (as the convolution's cut reduction does).  Not when the caller keeps reductions
    // whole (split 1), has ruled atomic adds out, or provides a workspace for the slices to meet in.
    const bool fused = pre != kPreAccumulate || post != kPostNone;
    if (fused && K > 0 && workspace == nullptr && !no_atomics && plan_bytes == nullptr && tls().forced_split_k != 1) {
        CutPlan plan;
        int rc = launch_sgemm_planned(M, N, K, A, lda, B, ldb, C, ldc, nullptr, kPreAccumulate, kPostNone, ta, tb,
                                      nullptr, 0, false, nullptr, &plan);
        if (rc != LSMI_OK) return rc;
        const double extra_us = (pre != kPreAccumulate ? 2.5 : 0.0) + (post != kPostNone ? 2.5 : 0.0) +
                                4.0 * M * N / 2.0e6;  // (and the output through memory once more each way)
        if (plan.slices > 1 && plan.whole_us - plan.cut_us > extra_us) {
            ThreadState &st = tls();
            const dim3 grid((unsigned)((N + 255) / 256), (unsigned)(M < 1024 ? M : 1024));
            if (pre != kPreAccumulate)
                hipLaunchKernelGGL(sgemm_init_kernel, grid, dim3(256), 0, st.stream, C, ldc, M, N,
                                   pre == kPreBias ? bias : nullptr);
            rc = launch_sgemm_planned(M, N, K, A, lda, B, ldb, C, ldc, nullptr, kPreAccumulate, kPostNone, ta, tb,
                                      nullptr, 0, false, nullptr, nullptr);
            if (rc != LSMI_OK) return rc;
            if (post == kPostRelu) {
                hipLaunchKernelGGL(sgemm_relu_kernel, grid, dim3(256), 0, st.stream, C, ldc, M, N);
                rc = check_launch();
            }
            return rc;
        }
    }
    return launch_sgemm_planned(M, N, K, A, lda, B, ldb, C, ldc, bias, pre, post, ta, tb, workspace, workspace_bytes,
                                no_atomics, plan_bytes, nullptr);
}

namespace {

int launch_sgemm_planned(int M, int N, int K, const float *A, int64_t lda, const float *B, int64_t ldb,
                         float *C, int64_t ldc, const float *bias, int pre, int post, bool ta, bool tb,
                         void *workspace, int64_t workspace_bytes, bool no_atomics, int64_t *plan_bytes,
                         CutPlan *plan_only)
{
    const Epilogue ep{bias, pre, post};
    const Variant *const kVariants = table_of(ta, tb);
    // Where the partial sums of a cut reduction meet.  In the caller's workspace (the buffer-load
    // kernels only): any pre/post form may be cut, the result is deterministic.  Otherwise in
    // atomic adds onto the old C, which is only possible when nothing else happens to the
    // element (the plain accumulate form) and when the caller has not ruled atomics out.
    // The workspace starts with kCounterBytes of arrival counters, then the partial tiles.
    const int64_t part_bytes = workspace != nullptr ? workspace_bytes - kCounterBytes : 0;
    const bool can_meet = part_bytes > 0;
    const bool may_split = can_meet || (!no_atomics && pre == kPreAccumulate && post == kPostNone);
    ThreadState &st = tls();
    const int cus = device_cu_count();
    auto tiles = [&](const Variant &v) {
        return (int64_t)((M + v.bm - 1) / v.bm) * ((N + v.bn - 1) / v.bn);
    };
    // a kernel that cannot take this problem's shape or alignment, or one whose slices always
    // meet in atomic adds when the caller has ruled them out
    auto usable = [&](int index) {
        const Variant &c = kVariants[index];
        if (c.rows && (no_atomics || can_meet)) return false;
        return !c.dma || dma_supported(c, ta, tb, M, N, K, A, lda, B, ldb, C, ldc, ep);
    };
    // what the partial sums of s slices of `bytes` of output cost where they meet: through the
    // floating-point atomic units at about 0.7 TB/s (1.5 from the kernels with wave sets, whose
    // waves all add whole rows); or written through to memory, counted and
    // read back by the last workgroup to arrive, three dependent round trips to memory that
    // grow with the number of slices it has to wait for and read (256 x 256 x 8192 in 16
    // slices: 9 us of 21; 1024^3 in 2: 2.3 us)
    auto meeting_us = [&](double bytes, int s, bool by_rows = false) {
        return can_meet ? 1.0 + 0.5 * s + bytes * s / 6.0e6 : bytes * s / (by_rows ? 1.5e6 : 0.7e6);
    };
    // Time of a 64 x 64 kernel with wave sets on an output of fewer than two tiles per CU, its
    // reduction in s slices, and the s that minimises it.  Fitted (6.5 % rms) to sweeps of 57
    // shapes x 2 kernels x 11 cuts, aligned and not: a step of a workgroup that has its CU to
    // itself takes `lone` us; w workgroups resident on a CU take w steps' worth of matrix
    // instructions (0.864 us for 64 x 64 x 64) over `eff` when that is longer; workgroups beyond
    // what a CU holds (two with four wave sets, three with two) follow in further rounds; the
    // slices' partial sums go through the atomic units at about 1.5 TB/s (all waves adding whole
    // rows), or meet in the workspace.
    struct SmallPlan {
        int split;
        double us;
    };
    auto plan_small = [&](const Variant &c, bool cut_allowed) {
        const bool k4 = c.ksets == 4;
        const double lone = c.dword ? (k4 ? 0.90 : 0.65) : (k4 ? 0.987 : 0.548);
        const double eff = c.dword ? (k4 ? 0.82 : 0.90) : (k4 ? 0.97 : 1.035);
        const double start_us = c.dword ? 5.4 : 4.4, rate = c.dword ? 1.46e6 : 1.57e6, cut_us = c.dword ? -2.55 : -1.16;
        const double mfma_us = 2.0 * 64 * 64 * c.bk / 0.607e6;  // a step's matrix instructions on one CU (256 flop/clk at 2.37 GHz)
        const int hold = k4 ? 2 : 3;
        const int64_t t = tiles(c);
        const int chunks = K > 0 ? (K + c.bk - 1) / c.bk : 1;
        const int min_steps = 64 / c.bk > 1 ? 64 / c.bk : 1;  // at least 64 reduction indices per slice
        const int cap = !cut_allowed ? 1 : chunks / min_steps > 1 ? (chunks / min_steps < 64 ? chunks / min_steps : 64) : 1;
        SmallPlan best{1, 0.0};
        for (int s = 1; s <= cap; ++s) {
            const int per = (chunks + s - 1) / s;
            const int slices = (chunks + per - 1) / per;
            if (slices != s) continue;  // the same cut as a smaller s
            const int64_t per_cu = (t * s + cus - 1) / cus;
            auto together = [&](int64_t w) { return w == 0 ? 0.0 : (w * mfma_us / eff > lone ? w * mfma_us / eff : lone); };
            double us = start_us + per * ((double)(per_cu / hold) * together(hold) + together(per_cu % hold));
            if (s > 1) us += can_meet ? meeting_us(4.0 * 4096 * t, s) : 4.0 * 4096 * t * s / rate + cut_us;
            if (s == 1 || us < best.us) best = SmallPlan{s, us};
        }
        return best;
    };
    int vi = st.forced_variant;
    bool keep_whole = false;  // the choice below was made for one workgroup per tile
    if (vi >= 0 && !usable(vi)) vi = -1;  // a forced kernel that cannot take this call: use the built-in choice
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
            const TailPlan tp = tail_ok && c.edge ? plan_tail(c, t, chunks, cus, can_meet) : TailPlan{};
            if (tp.split > 1)
                return chunk_us * chunks * (double)((t - tp.tiles) / cus) +
                       chunk_us * ((chunks + tp.split - 1) / tp.split) +
                       meeting_us(4.0 * c.bm * c.bn * (double)tp.tiles, tp.split, c.ksets > 1);
            return chunk_us * chunks * (double)(t / cus + (t % cus != 0 ? 1 : 0));
        };
        const bool tail_ok = may_split && st.forced_split_k <= 0;
        // 64 x 64 tiles: four wave sets (two workgroups per CU) for outputs of at most two tiles
        // per CU, two wave sets (three per CU) beyond -- 1024^3 22.0 -> 20.4 us, 2048 x 2048 x 512
        // 47.1 -> 41.6, but 1536^3 62 -> 64, 3500 x 1000 x 2000 118 -> 129 with four sets
        const int64_t t64 = (int64_t)((M + 63) / 64) * ((N + 63) / 64);
        // (two tiles per CU with a last round that is full, or nearly, or a long reduction -- an
        // incomplete round cut into slices goes better with three smaller workgroups per CU: 3296 x
        // 284 x 684 21.2 -> 18.3 us -- and whole rounds of up to four)
        const bool full_rounds = t64 % cus == 0 || 10 * (t64 % cus) >= 9 * cus;
        const bool few64 = t64 <= cus || (t64 <= 2 * cus && (full_rounds || K >= 1024)) || (t64 <= 4 * cus && full_rounds);
        // (short reductions: the two-set kernel's 32-deep steps and three-stage ring, 640 x 2368 x 148
        // 12.6 -> 9.6 us, 1408 x 768 x 224 13.4 -> 11.0, 2688 x 768 x 260 16.5 -> 14.5)
        const bool quad = few64 && K >= 512;
        const int kEdgeSmall = quad ? kEdgeQuad : kEdgePair, kEdgeSmallDword = quad ? kEdgeQuadDword : kEdgeDword;
        const double small_rate = quad ? 0.55e6 : 0.53e6, small_dword_rate = quad ? 0.52e6 : 0.51e6;
        const bool edge_ok = dma_supported(kVariants[kEdgeBig], ta, tb, M, N, K, A, lda, B, ldb, C, ldc, ep);
        // Below this the register-staged kernel is as quick or quicker (192^3 5.3 against 5.6 us,
        // 320^3 5.6 / 5.8, 512 x 512 x 128 5.6 / 5.9); above, the wave-set kernels lead, by more
        // when rows are unaligned (256 x 256 x 512 5.6 against 6.0, 384^3 5.9 / 6.7, 4096 x 64 x 256
        // 6.0 / 7.8, 512^3 7.5 / 9.0, 64 x 64 x 8192 6.5 / 8.1; 385^3 7.1 / 9.6, 513^3 9.4 / 14.0).
        // Multiply-adds are counted over whole tiles.
        // That holds for whole 64 x 64 tiles only: on ragged ones the register-staged kernel loads
        // element by element under tests and is twice as slow as the buffer loads' zero fill
        // (528 x 246 x 111 13.3 against 6.7 us, 96 x 48 x 96 9.2 / 5.4, 32 x 599 x 74 11.3 / 6.3).
        auto small_pays = [&](int64_t t, bool unaligned) {
            // (a handful of reduction indices: all epilogue, the register-staged kernel's is as good --
            // unless one side of C is a fraction of its tile: 132552 x 8 x 24 41.0 us against 14.0)
            if (K < 32) return M <= 32 || N <= 32;
            if (M % 64 != 0 || N % 64 != 0 || K % 16 != 0) return true;
            // (a transposed A costs the register-staged kernel strided loads: 448 x 64 x 592 with both
            // operands transposed 7.4 us against 5.3, 64 x 576 x 464 5.9 / 5.2)
            if (ta) return true;
            if (K < 64) return false;
            if (2 * t >= cus) return true;
            if (K >= 256 && 4 * t >= cus) return true;
            return t * 4096 * K >= (1LL << 25) && K >= (unaligned ? 256 : 384);
        };
        const int rows = kRows16;
        // (not with a reduction so short that the call is its atomic adds, which in the plain layout
        // go out 16 bytes per row and lane group: 16 x 401408 x 32 83.7 us against 34.4 on 64 x 64 tiles,
        // 16 x 200000 x 128 46.7 / 40.7; 4 x 100000 x 64 9.7 / 14.2 and 8 x 65536 x 256 17.1 / 21.5 stay; with a
        // transposed B they are 64 bytes per row: 29.0 and 27.0 us on the first two)
        if (M <= 16 && (tb || K >= 16 * M) && (int64_t)N * K >= (1 << 20) && st.forced_split_k != 1 && usable(rows)) {
            // a few rows against a B of 4 MB or more: the kernel that streams B straight into
            // registers (a caller who keeps the reduction in one workgroup does not get it:
            // its slices always meet in atomic adds).  N = K = 4096, B from HBM: M = 1
            // 24.1 -> 14.9 us, M = 8 22.9 -> 15.8, M = 16 23.7 -> 19.0.  With two row blocks (M up
            // to 32) the wave-set kernels are level or ahead since their epilogue is shared by all
            // waves (32 x 944 x 3592 10.0 against 8.0 us, 32 x 11008 x 4096 58.2 / 51.2, 32 x 4096 x
            // 4096 18.8 / 20.4)
            vi = rows;
        } else if (N <= 16 && (K >= 32 + 12 * N || (!tb && ldb % 4 != 0)) && (int64_t)M * K >= (1 << 20) &&
                   st.forced_split_k != 1 && usable(kCols16)) {
            // a few columns against an A of 4 MB or more (a matrix-vector product): the same kernel
            // on the transposed problem (4096 x 1 x 4096 22.1 us on 64 x 64 tiles, 4096 x 8 x 4096 19.8).
            // With a short reduction its workgroups are all epilogue, atomic adds scattered into
            // the transposed C, the more so the more columns: per row of A it costs about 0.08 +
            // 0.01 N + 0.0003 K ns against 0.05 + 0.0012 K on 64 x 64 tiles (401408 x 16 x 32: 86.8 us
            // against 35.5, 200000 x 16 x 128 48.3 / 41.3, 109824 x 12 x 228 31.4 / 41.7, 65536 x 8 x 256
            // 17.4 / 22.0) -- unless B's rows are not 16-byte aligned, which this kernel does not
            // mind and the tiles do (81480 x 1 x 20: 6.8 against 20.7)
            vi = kCols16;
        } else if (st.forced_split_k <= 1 && (tiles(d) == cus ? K <= 2048 : 5 * tiles(d) >= 4 * cus && tiles(d) < cus && K <= 1024) &&
                   (usable(kLoneDma) ||
                    // (ragged: when 128-row and -column tiles cover little more than 64 x 64 tiles would, and to
                    // K = 512: 428 x 6532 x 304 24.8 us against 22.5 on 64 x 64 tiles, 3108 x 1144 x 820 59.6 / 54.8)
                    (edge_ok && K <= 512 &&
                     25 * ((int64_t)(M + 127) / 128 * 128) * ((int64_t)(N + 127) / 128 * 128) <=
                         26 * ((int64_t)(M + 63) / 64 * 64) * ((int64_t)(N + 63) / 64 * 64)))) {
            // one 128 x 128 tile per CU, or nearly, and a reduction short enough that the start and the
            // end of a workgroup count: one round of whole tiles on eight waves of 32 x 64, two per SIMD,
            // instead of four rounds of 64 x 64 tiles (2048 x 2048 x 256 27.8 -> 21.4 us, x 1024 71.8 -> 67.4,
            // x 2048 129.2 -> 128.4, 4096 x 1024 x 512 41.2 -> 37.9, 1792 x 2048 x 256 27.0 -> 21.1, 1920 x 2048 x
            // 1024 70.2 -> 67.4; the same tile on four waves: 22.1, 69.5, 131.1; from K = 3072 the wave sets
            // lead, 187.3 against 189.6, and with three quarters of the CUs at any K: 1536 x 2048 x 512 31.4 / 36.2);
            // ragged shapes on the buffer-load form of the same tile (596 x 6260 x 128 18.0 -> 15.5, 2944 x 1152 x
            // 188 19.6 -> 18.0)
            vi = usable(kLoneDma) ? kLoneDma : kEdgeBig;
            keep_whole = true;
        } else if (st.forced_split_k <= 1 && tiles(d) >= cus && K >= 64 &&
            dma_supported(d, ta, tb, M, N, K, A, lda, B, ldb, C, ldc, ep)) {
            // with one workgroup per CU (2048^3: 256 tiles) nothing else hides the latency of
            // the C tile in the epilogue: request it up front (5 %); with two or more per CU
            // the plain kernel is as fast or faster
            vi = (tiles(d) < 2 * cus && ep.pre == kPreAccumulate) ? kOneRoundDma : kDefaultDma;
            double best = estimate(kDefaultDma, 0.57e6, false);
            if (edge_ok) {
                // with four or more tiles per CU and a reduction of 128 .. 1024 the buffer-load form
                // of the same tile is ahead (4096 x 4096 x 256: 77.6 against 87.5 us, x 1024: 251
                // against 259; at 4096 and with two tiles per CU the full-tile form leads)
                const bool short_k = tiles(d) >= 4 * cus && K >= 64 && K <= 1024;  // (7808 x 3200 x 96: 70.4 against 60.8 us)
                const double big = estimate(kEdgeBig, short_k ? 0.65e6 : 0.565e6, tail_ok);
                if (big < best) {
                    best = big;
                    vi = kEdgeBig;
                }
                if (estimate(kEdgeSmall, small_rate, tail_ok) < best) vi = kEdgeSmall;
            }
            // Whole generations of 256 x 128 tiles on eight waves, two workgroups per CU: a
            // chunk brought into LDS costs its SIMD about 31 cycles of matrix-instruction issue
            // per KB, whatever the width or the source of the load, and the larger tile brings
            // in 96 bytes per matrix instruction where 128 x 128 brings 128 (4096^3 941.9 ->
            // 932.3 us, 8192 x 4096 x 4096 1877 -> 1845, 4096 x 4096 x 1024 252.0 -> 248.4; 256 x 256
            // tiles on sixteen waves, one barrier for the whole CU: 936, 1870, 254)
            // -- when every CU gets the same number of them, two or more, in one launch: the two
            // slots of a CU refill one at a time (16384 x 4096 x 4096 3780 -> 3672 us, 10240 x 4096 x 4096,
            // five per CU, 2375 -> 2309; a CU with a tile more than the others holds everyone up:
            // 5120 x 4096 x 2048, 2.5 per CU, 616 -> 705)
            // The same holds for 128 x 128 tiles on eight waves of 32 x 64, two workgroups per CU, and
            // with a short reduction they are ahead of every other form, their waves' epilogues
            // being half as long: whenever every CU gets the same number of 128 x 128 tiles, in one
            // launch (6144 x 6144 x 512, nine per CU, 320.5 -> 290.2 us, x 4096 2143 -> 2091; 5120 x 4096 x
            // 1024 369 -> 308; 8192 x 4096 x 128 103.0 -> 90.3; 3072 x 4096 x 256 66.9 -> 58.1; 8192 x 8192 x 256:
            // 293.6 against 306.9 on 256 x 128 tiles, x 2048 1860 / 1877, x 4096 3698 / 3687; 8192 x 4096 x 2048 944.8 /
            // 949.6, 16384 x 4096 x 4096 3689 / 3678), the 256 x 128 tiles from K = 4096
            // -- and, tile counts aside, wherever whole tiles of the four-wave form would have run:
            // 4992 x 4096 x 4096 1237 us in generations of the four-wave tile, 1161 in one launch of this
            // one; 7936 x 4096 x 2048 971 -> 945
            if (((K >= 128 || tiles(d) >= 5 * cus) && tiles(d) >= 2 * cus && tiles(d) % cus == 0) || vi == kDefaultDma ||
                vi == kOneRoundDma)
                if (usable(kLoneDma)) vi = kLoneDma;
            const int64_t wide_tiles = tiles(kVariants[kWideDma]);
            if (vi == kLoneDma && K >= 4096 && wide_tiles >= 2 * cus && wide_tiles % cus == 0 && usable(kWideDma))
                vi = kWideDma;
        } else if (edge_ok && (can_meet || small_pays(t64, false))) {
            // ragged shapes with aligned rows, and whole-tile shapes too small for the 128 x 128
            // tiles: the buffer-load kernels, 128 x 128 tiles or the form in which four sets of
            // waves share a 64 x 64 tile, each taking every fourth chunk (1024^3: 31 us on plain
            // 64 x 64 tiles, 22 with two sets, 20.4 with four; 1000^3 28.8 -> 27.0), by the same
            // estimate.  A caller whose partial sums meet in a workspace always comes here: the
            // register-staged kernel could only keep every reduction whole.  Problems with fewer than 2^28 multiply-adds (counted over
            // whole tiles: a few rows against a large B cost what 64 rows do, 8 x 4096 x 4096
            // 42 -> 23 us) and 64 x 64 tiles for less than half the CUs stay with the
            // register-staged kernel, which is as quick there (with more tiles and a short
            // reduction it is not: 1024 x 1024 x 128 10.8 -> 6.1 us)
            vi = kEdgeSmall;
            if (t64 <= cus && st.forced_split_k <= 0 &&
                plan_small(kVariants[kEdgePair], may_split).us < plan_small(kVariants[kEdgeQuad], may_split).us)
                vi = kEdgePair;
            // a handful of chunks on many tiles: one set of waves, 16-deep steps (868 x 4436 x 68
            // 15.8 -> 11.9 us, 2048 x 2048 x 64 13.3 -> 10.1)
            if (K < 128 && t64 >= 2 * cus && st.forced_split_k <= 1 && usable(kEdgeSingle)) vi = kEdgeSingle;
            if (st.forced_split_k <= 1 && tiles(kVariants[kEdgeBig]) >= cus &&
                estimate(kEdgeBig, 0.565e6, tail_ok) < estimate(kEdgeSmall, small_rate, tail_ok))
                vi = kEdgeBig;
        } else if ((can_meet || small_pays(t64, true)) &&
                   dma_supported(kVariants[kEdgeSmallDword], ta, tb, M, N, K, A, lda, B, ldb, C, ldc, ep)) {
            // rows that start at any element (lda, ldb or K not multiples of four, or bases not
            // 16-byte aligned): the same kernels with 4-byte loads, by the same estimate (rates
            // 0.544 and 0.51 TFLOP/s per CU; 4001^3: 965 us on 128 x 128 tiles, 1029 on 64 x 64)
            vi = kEdgeSmallDword;
            if (t64 <= cus && st.forced_split_k <= 0 &&
                plan_small(kVariants[kEdgeDword], may_split).us < plan_small(kVariants[kEdgeQuadDword], may_split).us)
                vi = kEdgeDword;
            if (st.forced_split_k <= 1 && tiles(kVariants[kEdgeBigDword]) >= cus &&
                estimate(kEdgeBigDword, 0.544e6, tail_ok) < estimate(kEdgeSmallDword, small_dword_rate, tail_ok))
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
    // the buffer-load kernels can let the slices meet in the workspace; everything else that is
    // cut adds its partial sums to C atomically
    const bool meets = can_meet && v.edge && !v.rows;
    const bool cut_ok = meets || (!can_meet && !no_atomics && pre == kPreAccumulate && post == kPostNone);
    const int64_t part_tiles = meets ? part_bytes / ((int64_t)v.bm * v.bn * 4) : 0;  // partial tiles the workspace holds
    int split = ((v.dma && !v.edge) || !cut_ok || keep_whole) ? 1 : st.forced_split_k;
    auto rows_cost = [&](int s) {  // the few-row kernel in s slices, see below
        // (on a few columns the streamed operand is A, in panels of 64 of its rows)
        const double stream_us = 4.0 * (v.cols ? M : N) * K / 6.3e6, share_us = 4.0 * 64 * K / 38.5e3;
        // (a slice's adds: 3.7 us per MB of C; scattered into the transposed C 15: 32052 x 4 x 1204
        // 30.4 us whole, 38.4 in two slices)
        const double slice_us = (v.cols ? 15e-6 : 3.7e-6) * 4.0 * M * N + 0.15;
        const double wgs = (double)(v.cols ? tiles_m : tiles_n) * s;
        double us = stream_us + share_us / s * (wgs < cus ? cus / wgs : 1.0) + slice_us * s;
        if (tb || v.cols) {
            // A transposed B is read a 128-byte line of 64 rows per step: the time follows the
            // rounds of workgroups over the CUs (8 x 4096 x 4096, 64 column tiles: 14.6 us in 4 or 8
            // slices, 19.1 in 5, 16.9 in 6 or 7, 17.6 in 11), and a wave whose share starts inside a line reads
            // every line twice.
            const double r = wgs / cus;
            if (r > 1.0 && std::ceil(r) != r) us *= 1.15 * (0.5 + 0.5 * std::ceil(r) / r);
            if (((chunks + s - 1) / s) % 2 != 0) us *= 1.1;
        }
        return us;
    };
    if (split <= 0 && v.rows) {
        // fitted to sweeps of M = 1 .. 32 against 16 to 180 MB of B read from HBM (several
        // copies of B in rotation): B streams at 6.3 TB/s, plus the time one workgroup needs
        // for its own share at 38.5 GB/s (what it keeps in flight; longer when there are fewer
        // workgroups than CUs), plus, per slice, the output through the atomic units at 3.7 us
        // per MB and 0.15 us; at least two 64-deep chunks per slice.  Three steps in flight
        // per wave instead of one changed nothing.
        const int cap = chunks / 2 > 1 ? (chunks / 2 < 256 ? chunks / 2 : 256) : 1;
        double best = 0;
        split = 1;
        for (int s = 1; s <= cap; ++s) {
            const double cost = rows_cost(s);
            if (s == 1 || cost < best) {
                best = cost;
                split = s;
            }
        }
    }
    // the tiles of an incomplete last round as slices, see below
    TailPlan tail;
    if (v.edge && !v.rows && cut_ok && st.forced_split_k <= 0) tail = plan_tail(v, nt, chunks, cus, meets);
    if (meets && tail.split > 1 && (tail.tiles * tail.split > part_tiles || tail.tiles > kCounterBytes / 4))
        tail = TailPlan{};  // the workspace does not hold the tail's partial tiles
    if (split <= 0 && v.edge && v.bm == 64 && v.ksets > 1) {
        // (outputs of more than a tile per CU keep their reductions whole when the tiles of the
        // incomplete last round can be cut instead -- 1152^3, 324 tiles: 29.1 us against 32.9 in two
        // uniform slices -- and those of two tiles per CU or more in any case)
        split = (nt >= 2 * cus || (nt > cus && tail.split > 1)) ? 1 : plan_small(v, true).split;
    } else if (split <= 0 && v.edge && v.bm == 64) {
        // one set of waves, three-stage ring (a tuner's candidate): a 16-deep chunk costs a lone
        // workgroup 0.29 us, workgroups beyond one per CU share it
        const int cap = nt >= 2 * cus ? 1 : chunks / 4 > 1 ? (chunks / 4 < 64 ? chunks / 4 : 64) : 1;
        double best = 0;
        split = 1;
        for (int s = 1; s <= cap; ++s) {
            const int per = (chunks + s - 1) / s;
            const int64_t rounds = (nt * s + cus - 1) / cus;
            const double cost = 0.29 * per * rounds + (s > 1 ? meeting_us(4.0 * M * N, s) : 0.0);
            if (s == 1 || cost < best) {
                best = cost;
                split = s;
            }
        }
    }
    if (split <= 0) {
        split = 1;
        if (nt < 2 * cus && tail.split <= 1) {
            int64_t want = (3 * (int64_t)cus + 2 * nt - 1) / (2 * nt);
            // (a workgroup of eight waves fills its CU by itself, and two slices of a 128 x 128 tile
            // meeting in atomic adds cost more than they save: 2000 x 2000 x 256 61.8 us in two, 22.9 whole)
            if (v.per_cu == 2) want = cus / nt > 1 ? cus / nt : 1;
            int64_t cap = chunks / 4 > 1 ? chunks / 4 : 1;
            split = (int)(want < cap ? want : cap);
        }
    }
    if (split > chunks) split = chunks;
    if (split > 65535) split = 65535;
    if (meets && split > 1) {
        // as many slices as the workspace has partial tiles and counters for
        if (nt > kCounterBytes / 4) split = 1;
        else if (nt * split > part_tiles) split = (int)(part_tiles / nt > 1 ? part_tiles / nt : 1);
    }
    const int chunks_per_split = (chunks + split - 1) / split;
    const int k_per_split = chunks_per_split * v.bk;
    split = (chunks + chunks_per_split - 1) / chunks_per_split;
    if (plan_only != nullptr) {
        plan_only->slices = split;
        if (v.edge && v.bm == 64 && v.ksets > 1 && split > 1 && st.forced_split_k <= 0) {
            plan_only->cut_us = plan_small(v, true).us;
            plan_only->whole_us = plan_small(v, false).us;
        } else if (v.rows && split > 1 && st.forced_split_k <= 0) {
            plan_only->cut_us = rows_cost(split);
            plan_only->whole_us = rows_cost(1);
        } else if (split > 1 && st.forced_split_k <= 0) {
            // the other kernels are cut only on outputs of less than two tiles per CU, where a
            // workgroup's chunk is bound by the latency of its loads: 0.5 us for 16 reduction indices
            // on the register-staged kernels (64 x 256 x 1024, 4 tiles, whole: 33.5 us), 0.29 on the
            // direct-to-LDS ones
            const double per_chunk = v.dma ? 0.29 * v.bk / 16.0 : 0.5;
            plan_only->whole_us = per_chunk * chunks * (double)((nt + cus - 1) / cus);
            plan_only->cut_us = per_chunk * chunks_per_split * (double)((nt * split + cus - 1) / cus) +
                                meeting_us(4.0 * M * N, split);
        }
        return LSMI_OK;
    }
    if (plan_bytes != nullptr) {
        // what this call's partial sums occupy in a workspace that does not limit them; nothing is launched
        int64_t parts = split > 1 ? nt * split : 0;
        if (tail.split > 1 && split == 1) parts = tail.tiles * tail.split;
        *plan_bytes = meets && parts > 0 ? kCounterBytes + parts * (int64_t)v.bm * v.bn * 4 : 0;
        return LSMI_OK;
    }
    Meeting meet{nullptr, nullptr};
    if (meets) {
        meet.counters = static_cast<unsigned *>(workspace);
        meet.partials = reinterpret_cast<float *>(static_cast<char *>(workspace) + kCounterBytes);
    }

    // tile rows per band of the walk: 1024 rows of C either way (4096^3 on 256 x 128 tiles: 813 MB
    // between the L2s and the fabric in bands of eight tile rows, 669 MB in bands of four, the time the same)
    const int group_m = st.forced_group_m > 0 ? st.forced_group_m : v.bm >= 256 ? 4 : 8;
    // Tail split (buffer-load kernels, plain accumulate form): the tiles left over after the
    // last whole round of the CUs are cut into as many slices as fill one more round, so that
    // round lasts a slice's time instead of a tile's.  Taken when the time saved (at the rate
    // of one tile per CU, 0.47 TFLOP/s) exceeds what the slices' atomic adds cost.
    if (tail.split > 1 && split == 1) {
        const int per = (chunks + tail.split - 1) / tail.split;
        const int slices = (chunks + per - 1) / per;
        const int64_t rem = tail.tiles;
        v.launch(dim3((unsigned)(nt - rem + rem * slices), 1u), st.stream, M, N, K, A, lda, B, ldb, C, ldc,
                 tiles_m, tiles_n, group_m, per * v.bk, 1, (int)(nt - rem), slices, ep, meet);
        int rc = check_launch();
        if (rc == LSMI_OK) {
            st.last_variant = v.tail_name;
            st.last_split = slices;
        }
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
    const bool whole_tiles = vi == kDefaultDma || ((vi == kEdgeBigFour || vi == kEdgeBigDword) && tail.split <= 1 &&
                                                   K >= 2048 && (M % 128 != 0 || N % 128 != 0));
    // The full-tile kernel's last generation, when it is one or two tiles per CU or less, goes to
    // the form of the same tile that requests its C tile at the start (two workgroups per CU): a
    // workgroup of the plain form that has its CU to itself runs at half the rate (4992 x 4096 x
    // 4096, 1248 tiles: 1387 us in one launch, the last 224 tiles alone on their CUs; 5120 x 4096 x
    // 2060, five per CU: 718 us).
    const bool last_alone = vi == kDefaultDma && ep.pre == kPreAccumulate && usable(kOneRoundDma);
    if (whole_tiles && split == 1 && (nt >= generation + cus || (last_alone && nt > generation))) {
        for (int64_t first = 0; first < nt;) {
            const int64_t left = nt - first;
            const int64_t count = last_alone ? (left < generation ? left : generation)
                                             : (left < generation + cus ? left : generation);
            const Variant &g = last_alone && first > 0 && count <= 2 * (int64_t)cus ? kVariants[kOneRoundDma] : v;
            g.launch(dim3((unsigned)count, 1u), st.stream, M, N, K, A, lda, B, ldb, C, ldc, tiles_m, tiles_n,
                     group_m, k_per_split, 1, (int)first, 0, ep, meet);
            first += count;
        }
    } else {
        v.launch(dim3((unsigned)nt, (unsigned)split), st.stream, M, N, K, A, lda, B, ldb, C, ldc,
                 tiles_m, tiles_n, group_m, k_per_split, split, 0, 0, ep, meet);
    }
    int rc = check_launch();
    if (rc == LSMI_OK) {
        st.last_variant = v.name;
        st.last_split = split;
    }
    return rc;
}

}  // namespace

// ---- the entry point that allocates nothing ----
//
// sgemm_ws with the workspace in a file-scope device array instead of the caller's memory, for
// callers that cannot provide one because they cannot allocate.  The array's name is only a
// host-side handle: the device address comes from hipGetSymbolAddress, once per device, and
// is what the kernels get.
}  // namespace lsmi

static __device__ __align__(256) unsigned char scratch[lsmi::kSgemmCounterBytes + lsmi::kSgemmStaticPartialBytes];

namespace lsmi {

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};
}  // namespace

int sgemm_static_scratch(void **ptr)
{
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err == hipSuccess && (dev < 0 || dev >= kMaxDevices)) err = hipErrorInvalidDevice;
    if (err == hipSuccess) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (g_scratch_ptr[dev] == nullptr) {
            void *p = nullptr;
            err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));  // this device's copy of the array
            if (err == hipSuccess && p == nullptr) err = hipErrorInvalidSymbol;
            if (err == hipSuccess) g_scratch_ptr[dev] = p;
        }
        *ptr = g_scratch_ptr[dev];
    }
    if (err != hipSuccess) {
        tls().last_hip_error = static_cast<int>(err);
        (void)hipGetLastError();
        return LSMI_ERR_LAUNCH;
    }
    return LSMI_OK;
}

}  // namespace lsmi
