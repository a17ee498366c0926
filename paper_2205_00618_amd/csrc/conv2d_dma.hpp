// Direct convolution kernel for channel counts that are a multiple of the chunk depth
// (C % BK == 0, 16-byte aligned tensors): both operand tiles stream global -> LDS with
// GLOBAL_LOAD_LDS_DWORDX4 into a ring of NSTAGE chunk buffers, like the aligned GEMM kernel.
//
// The contraction is the one of Section 2.1 ("convolution as a contraction" with an affine
// operand index): rows of the A tile are output pixels m = (n, p, q), its columns the
// reduction index (r, s, c); a BK chunk lies inside one filter tap (r, s), so per chunk a
// lane only adds a scalar tap offset to its pixel's base address and tests whether the tap
// falls inside the image.  The loads go through buffer descriptors over the input and the
// filter (both below 2^31 bytes); taps in the zero padding, pixel rows past N*P*Q and filter
// rows past K are given an out-of-range offset, for which the hardware writes zeros, so every
// lane always issues its load and the load counter stays uniform.  B rows are output channels, k-contiguous in the KRSC
// filter, and use the same LDS image as A.
//
// LDS image of one operand chunk: rows x (BK*4) bytes; the 16-byte k-groups of row r sit at
// slot g ^ f(r), with f chosen so that the 16-byte fragment reads of 32 consecutive rows
// are bank-conflict free without padding:
//   BK = 16 (4 groups): f(r) = ((r >> 1) ^ (r >> 2)) & 3
//   BK = 32 (8 groups): f(r) = (r & 7) ^ ((r >> 3) & 1)
// (both depend on r mod 16 only, so a lane's value holds for every 32-row block it reads)
#pragma once

#include <type_traits>

#include "sgemm_dma.hpp"
#include "tile_f32.hpp"

namespace lsmi {

// AHEAD: the fragments of chunk c + 1 are read from LDS into a second set of registers while
// the matrix instructions of chunk c run, so a workgroup hides its LDS latency by itself
// (the ring then needs one stage more for the same distance between request and use).
//
// GROUP_TAP: the channel count is a multiple of 4 only (24, 40, 72, ... channels, or a stem
// padded to 4).  A lane's 16 bytes, four consecutive channels, still lie inside one tap, but
// the k-groups of a chunk may belong to different taps and the reduction need not end on a
// chunk: every lane keeps the position of its own k-group in the walk, as a filter row r and
// an offset x = s*C + c inside that row (in NHWC the taps of one filter row are contiguous
// for a pixel, so x is also the address offset), moves them by one chunk per request, and
// asks for zeros when the group lies in the padding or past the last filter row.
//
// ELEM (a GROUP_TAP form): any channel count (a stem of 3 channels).  Every load instruction
// moves 4 bytes per lane, one element of the reduction, so neither a pixel's channels nor a
// filter's R*S*C elements need to start on a 16-byte boundary: the same walk per lane with
// (r, x) of its own element, the same range tests, four times the load instructions for the
// same image of the chunk in LDS.  An instruction fills four 64-byte rows of the image; the
// instructions are dealt to the waves round-robin, so that a lane's rows lie 16 apart and its
// slot in the row (which depends on the row modulo 16) is the same for all of them.
template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_, int NSTAGE_, bool AHEAD_ = false,
          bool GROUP_TAP_ = false, bool ELEM_ = false>
struct ConvDmaShape {
    static constexpr bool AHEAD = AHEAD_, GROUP_TAP = GROUP_TAP_, ELEM = ELEM_;
    static constexpr int BM = BM_, BN = BN_, BK = BK_, NSTAGE = NSTAGE_;
    static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, NWAVES = WAVES_M * WAVES_N;
    static constexpr int NT = 64 * NWAVES;
    static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    static constexpr int TM = WTM / 32, TN = WTN / 32;
    static constexpr int ROW_BYTES = BK * 4, GROUPS = BK / 4;
    static constexpr int INSTR_BYTES = ELEM ? 256 : 1024;  // LDS bytes one load instruction fills
    static constexpr int ROWS_PER_INSTR = INSTR_BYTES / ROW_BYTES;
    static constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;
    static constexpr int A_PER_WAVE = A_BYTES / INSTR_BYTES / NWAVES;  // load instructions per wave and chunk
    static constexpr int B_PER_WAVE = B_BYTES / INSTR_BYTES / NWAVES;
    static constexpr int LOADS = A_PER_WAVE + B_PER_WAVE;
    static constexpr int WGS_PER_CU = (160 * 1024) / LDS_BYTES < 8 ? (160 * 1024) / LDS_BYTES : 8;
    static constexpr int WAVES_PER_SIMD = WGS_PER_CU * NWAVES / 4 < 8 ? WGS_PER_CU * NWAVES / 4 : 8;
    static_assert(BK == 16 || BK == 32, "chunk depth");
    static_assert(A_BYTES % (1024 * NWAVES) == 0 && B_BYTES % (1024 * NWAVES) == 0, "even DMA split");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && TM >= 1 && TN >= 1, "wave tiles are 32-multiples");
    static_assert(NSTAGE >= 2 && NSTAGE <= 6 && LOADS * (NSTAGE - 2) <= 63, "ring depth");
    static_assert(!AHEAD || NSTAGE >= 3, "reading a chunk ahead takes a third stage");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
    // one k-group per lane for all of its requests: the slot swizzle repeats every 16 rows
    static_assert(!GROUP_TAP || (BK == 16 && !AHEAD), "per-lane taps: 16-deep chunks");
    static_assert(!ELEM || (GROUP_TAP && NWAVES == 4), "per-lane elements: a lane's rows 16 apart");

    __host__ __device__ static constexpr int swizzle(int r)
    {
        return BK == 16 ? (((r >> 1) ^ (r >> 2)) & 3) : ((r & 7) ^ ((r >> 3) & 1));
    }
};

// Four bytes per lane with a scalar byte offset added after the range check of the lane offset
// (dma16_buf_s with a quarter of the bytes).
__device__ __forceinline__ void dma4_buf_s(i32x4 buffer, uint32_t voff, uint32_t soff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dword %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(buffer), "s"(soff)
                 : "memory", "m0");
}

struct ConvDmaGeom {
    int H, W, C, K, S, stride, pad, P, Q;
    int pixels;  // N*P*Q
    int red;     // R*S*C
    int hwc;     // H*W*C
    int R;
    FastDiv by_pq, by_q;  // pixel index -> image, row, column without general divisions
    FastDiv by_c, by_s;   // reduction index -> tap and channel (start of a slice)
    TileMap tmap;         // the walk over (channel tile, pixel tile): channel tiles are neighbours

    ConvDmaGeom(int H_, int W_, int C_, int K_, int R_, int S_, int stride_, int pad_, int P_, int Q_, int pixels_,
                int tiles_m, int tiles_n)
        : H(H_), W(W_), C(C_), K(K_), S(S_), stride(stride_), pad(pad_), P(P_), Q(Q_), pixels(pixels_),
          red(R_ * S_ * C_), hwc(H_ * W_ * C_), R(R_), by_pq((uint32_t)(P_ * Q_)), by_q((uint32_t)Q_),
          by_c((uint32_t)C_), by_s((uint32_t)S_), tmap(tiles_n, tiles_m, tiles_n)
    {
    }
};


// Quarter-tile pieces for the last tile rows.  When the tile count is a little over a whole
// number of rounds of the machine, the few tiles of the last round would each occupy a CU
// alone while the others idle.  Instead the pixel rows past m_cut are cut into 32 x 32 pieces,
// one workgroup each, dispatched ahead of the whole tiles: a piece is a quarter of a 64 x 64
// tile's work, so the surplus spreads over four times as many CUs.  Inside a piece the four
// waves split the reduction (wave w takes the w-th quarter of the 8-element groups), fetch
// their fragments straight from global memory through the same zero-filling buffer
// descriptors (16 bytes per lane: four consecutive reduction elements of the lane's pixel /
// output channel, no LDS staging, the latency is covered by the whole tiles sharing the CU),
// and add their partial sums through LDS in a fixed order, so the result does not depend on
// the dispatch.  The epilogue is the whole tiles' one.
template <class T>
__device__ __forceinline__ void conv2d_piece(const ConvDmaGeom &g, const float *__restrict__ in,
                                             const float *__restrict__ w, float *__restrict__ out,
                                             int piece, int pieces_n, int m_cut, const Epilogue &ep,
                                             unsigned char *lds)
{
    static_assert(T::NWAVES == 4 && T::LDS_BYTES >= 4 * 16 * 64 * 4, "four waves, 16 KiB for the partial sums");
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int li = lane & 31, half = lane >> 5;
    const int m0 = m_cut + 32 * (piece / pieces_n), n0 = 32 * (piece % pieces_n);
    const __amdgpu_buffer_rsrc_t buf_in =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(in), 0, (int)kOutOfRange, 0x00020000);
    const __amdgpu_buffer_rsrc_t buf_w =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(w), 0, (int)kOutOfRange, 0x00020000);

    // this lane's pixel (A row) and output channel (B row); its four elements of a group of
    // eight are 4*half .. 4*half + 3, the same for both operands
    const int m = m0 + li;
    int a_h0 = INT32_MIN / 2, a_w0 = 0, a_off = 0;  // a row past the last pixel fails every range test
    if (m < g.pixels) {
        const int n = (int)g.by_pq.div((uint32_t)m), pq = m - n * g.P * g.Q, p = (int)g.by_q.div((uint32_t)pq);
        a_h0 = p * g.stride - g.pad;
        a_w0 = (pq - p * g.Q) * g.stride - g.pad;
        a_off = (n * g.hwc + (a_h0 * g.W + a_w0) * g.C + 4 * half) * 4;
    }
    const uint32_t b_off = n0 + li < g.K ? (uint32_t)(((n0 + li) * g.red + 4 * half) * 4) : kOutOfRange;

    const int groups = g.red / 8, per_wave = (groups + 3) / 4;
    int gi = wave * per_wave;
    const int gend = min(groups, gi + per_wave);
    int k0 = gi * 8;
    const int k0_tap = (int)g.by_c.div((uint32_t)k0);
    int tap_c = k0 - k0_tap * g.C, tap_r = (int)g.by_s.div((uint32_t)k0_tap), tap_s = k0_tap - tap_r * g.S;

    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    constexpr int BATCH = 4;  // groups requested together: eight 16-byte loads in flight per lane
    // as in the whole tiles' loop, the per-lane offset is worked out once per tap and the walk
    // along the channels is a scalar offset
    uint32_t a_cur = kOutOfRange;
    bool new_tap = true;
    while (gi < gend) {
        f32x4 af[BATCH], bf[BATCH];
#pragma unroll
        for (int j = 0; j < BATCH; ++j) {
            if (new_tap) {
                const bool ok = (unsigned)(a_h0 + tap_r) < (unsigned)g.H && (unsigned)(a_w0 + tap_s) < (unsigned)g.W;
                a_cur = ok ? (uint32_t)(a_off + ((tap_r * g.W + tap_s) * g.C) * 4) : kOutOfRange;
                new_tap = false;
            }
            // groups past the wave's share are requested out of range: zeros, which add nothing
            const bool live = gi + j < gend;
            af[j] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                                                  buf_in, live ? (int)a_cur : (int)kOutOfRange, tap_c * 4, 0));
            bf[j] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                                                  buf_w, live ? (int)b_off : (int)kOutOfRange, k0 * 4, 0));
            k0 += 8;
            tap_c += 8;
            if (tap_c == g.C) {
                tap_c = 0;
                new_tap = true;
                if (++tap_s == g.S) {
                    tap_s = 0;
                    ++tap_r;
                }
            }
        }
#pragma unroll
        for (int j = 0; j < BATCH; ++j)
#pragma unroll
            for (int t = 0; t < 4; ++t)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[j][t], bf[j][t], acc, 0, 0, 0);
        gi += BATCH;
    }

    // partial sums [wave][register][lane]; wave x then adds up registers 4x .. 4x + 3 in wave
    // order, i.e. rows 8x + 4*half + (0..3) of the piece, and stores them
    float *part = reinterpret_cast<float *>(lds);
#pragma unroll
    for (int v = 0; v < 16; ++v) part[(wave * 16 + v) * 64 + lane] = acc[v];
    __syncthreads();
    const int k = n0 + li;
    const float init = (ep.pre == kPreBias && k < g.K) ? ep.bias[k] : 0.f;
    float sum[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int v = 4 * wave + j;
        sum[j] = part[v * 64 + lane];
#pragma unroll
        for (int x = 1; x < 4; ++x) sum[j] += part[(x * 16 + v) * 64 + lane];
        sum[j] = apply_post(init + sum[j], ep.post);
    }
    const int row0 = m0 + 8 * wave + 4 * half;
    if (m0 + 32 <= g.pixels && n0 + 32 <= g.K) {  // untested stores, see the whole tiles' epilogue
#pragma unroll
        for (int j = 0; j < 4; ++j) out[(int64_t)(row0 + j) * g.K + k] = sum[j];
        return;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (row0 + j < g.pixels && k < g.K) out[(int64_t)(row0 + j) * g.K + k] = sum[j];
}

// Workgroups [0, pieces) of the grid compute quarter-tile pieces of the pixel rows from m_cut
// on (pieces_n pieces per 32 pixel rows); the others the whole tiles of the rows before m_cut.
template <class T>
__global__ __launch_bounds__(T::NT)
__attribute__((amdgpu_waves_per_eu(1, T::WAVES_PER_SIMD))) void conv2d_dma_kernel(
    ConvDmaGeom g, const float *__restrict__ in, const float *__restrict__ w,
    float *__restrict__ out, int tiles_m, int tiles_n, int chunks_per_slice, int pieces, int pieces_n,
    int m_cut, Epilogue ep)
{
    __shared__ __attribute__((aligned(1024))) unsigned char lds[T::LDS_BYTES];
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
    if constexpr (T::NWAVES == 4 && T::LDS_BYTES >= 16384) {
        if ((int)blockIdx.x < pieces) {
            conv2d_piece<T>(g, in, w, out, (int)blockIdx.x, pieces_n, m_cut, ep, lds);
            return;
        }
    }

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, half = lane >> 5;
    const int wrow = (wave / T::WAVES_N) * T::WTM;
    const int wcol = (wave % T::WAVES_N) * T::WTN;

    // channel tiles of one pixel tile are neighbours in the walk: they share the input patch
    int tn, tm;
    g.tmap.locate((int)blockIdx.x - pieces, tn, tm);
    const int m0 = tm * T::BM, n0 = tn * T::BN;
    // the slice of the reduction this workgroup owns: all of it, or, when the output has too
    // few tiles to fill the machine, chunks [first, first + nk) with the partial sums of the
    // slices added atomically into an output that the caller has set to its initial value
    const bool sliced = gridDim.y > 1;
    const int first = (int)blockIdx.y * chunks_per_slice;
    const int nk = min((T::GROUP_TAP ? (g.red + T::BK - 1) / T::BK : g.red / T::BK) - first, chunks_per_slice);
    const i32x4 buf_in = make_buffer(in), buf_w = make_buffer(w);

    // ---- per-lane DMA sources (byte offsets into the two buffers) ----
    // A: the pixel of this lane's row; offset of in[n, h0, w0, 4*group] (may lie outside the
    // image: it is only used for taps that pass the range test)
    int a_off[T::A_PER_WAVE], a_h0[T::A_PER_WAVE], a_w0[T::A_PER_WAVE];
    // GROUP_TAP: the filter rows [r_lo, r_lo + r_span) and the row offsets [x_lo, x_lo + x_span)
    // whose taps fall inside the image for this pixel (empty for a row past the last pixel)
    int r_lo[T::GROUP_TAP ? T::A_PER_WAVE : 1], x_lo[T::GROUP_TAP ? T::A_PER_WAVE : 1];
    uint32_t r_span[T::GROUP_TAP ? T::A_PER_WAVE : 1], x_span[T::GROUP_TAP ? T::A_PER_WAVE : 1];
    const int filter_rows = g.R;
    // instruction q of this wave: its index among the operand's instructions (= its 1 KiB or
    // 256 B of the image), this lane's row of the tile and the first element of the row's chunk
    // that the lane moves
    auto instr_index = [&](int q, int per_wave) __attribute__((always_inline)) {
        return T::ELEM ? q * T::NWAVES + wave : wave * per_wave + q;
    };
    auto lane_row = [&](int index) __attribute__((always_inline)) {
        return index * T::ROWS_PER_INSTR + lane / (T::ROW_BYTES / (T::ELEM ? 4 : 16));
    };
    auto lane_kin = [&](int row) __attribute__((always_inline)) {
        if constexpr (T::ELEM) return 4 * (((lane & 15) >> 2) ^ T::swizzle(row)) + (lane & 3);
        else return 4 * ((lane % T::GROUPS) ^ T::swizzle(row));
    };
#pragma unroll
    for (int q = 0; q < T::A_PER_WAVE; ++q) {
        const int row = lane_row(instr_index(q, T::A_PER_WAVE));
        const int grp = lane_kin(row) >> 2;
        const int m = m0 + row;
        if (m < g.pixels) {
            const int n = (int)g.by_pq.div((uint32_t)m), pq = m - n * g.P * g.Q, p = (int)g.by_q.div((uint32_t)pq);
            a_h0[q] = p * g.stride - g.pad;
            a_w0[q] = (pq - p * g.Q) * g.stride - g.pad;
            a_off[q] = (n * g.hwc + (a_h0[q] * g.W + a_w0[q]) * g.C + (T::GROUP_TAP ? 0 : grp * 4)) * 4;
        } else {
            a_h0[q] = INT32_MIN / 2;  // fails every range test
            a_w0[q] = 0;
            a_off[q] = 0;
        }
        if constexpr (T::GROUP_TAP) {
            const int r_first = max(0, -a_h0[q]), r_end = m < g.pixels ? min(filter_rows, g.H - a_h0[q]) : 0;
            const int s_first = max(0, -a_w0[q]), s_end = min(g.S, g.W - a_w0[q]);
            r_lo[q] = r_first;
            r_span[q] = (uint32_t)max(0, r_end - r_first);
            x_lo[q] = s_first * g.C;
            x_span[q] = (uint32_t)max(0, s_end - s_first) * (uint32_t)g.C;
        }
    }
    // B: filter row of this lane's output channel (out of range past the last channel)
    uint32_t b_off[T::B_PER_WAVE];
#pragma unroll
    for (int q = 0; q < T::B_PER_WAVE; ++q) {
        const int row = lane_row(instr_index(q, T::B_PER_WAVE));
        b_off[q] = n0 + row < g.K ? (uint32_t)(((n0 + row) * g.red + lane_kin(row)) * 4) : kOutOfRange;
    }

    // scalar walk over the reduction, starting at the slice's first chunk.  Vector
    // instructions other than the matrix ones are not free here (each takes about five cycles
    // of the SIMD's matrix pipe), so the per-lane part of an address, the pixel's tap offset or
    // "out of range" when the tap falls into the padding, is worked out once per tap, and the
    // walk along the channels inside a tap is a scalar offset on the load.
    int k0 = first * T::BK;
    const int k0_tap = (int)g.by_c.div((uint32_t)k0);
    int tap_c = k0 - k0_tap * g.C, tap_r = (int)g.by_s.div((uint32_t)k0_tap), tap_s = k0_tap - tap_r * g.S;
    uint32_t a_cur[T::A_PER_WAVE];
    bool new_tap = true;
    // GROUP_TAP: filter row and offset inside it of this lane's k-group in the next chunk to
    // request, and the byte offset (r*W*C + x) * 4 from the pixel's base that goes with them
    int lane_r = 0, lane_x = 0, lane_off = 0;
    const int row_len = g.S * g.C;                    // reduction elements of one filter row
    const int row_jump = (g.W * g.C - row_len) * 4;   // extra bytes from the end of one to the next
    if constexpr (T::GROUP_TAP) {
        const int lane_k = k0 + lane_kin(lane_row(instr_index(0, T::A_PER_WAVE)));  // the same for every q
        lane_r = lane_k / row_len;
        lane_x = lane_k - lane_r * row_len;
        lane_off = (lane_r * g.W * g.C + lane_x) * 4;
    }
    auto issue = [&](int stage) {
        const uint32_t dst = lds_base + stage * T::STAGE_BYTES;
        if constexpr (T::GROUP_TAP) {
#pragma unroll
            for (int q = 0; q < T::A_PER_WAVE; ++q) {
                const bool ok = (uint32_t)(lane_r - r_lo[q]) < r_span[q] && (uint32_t)(lane_x - x_lo[q]) < x_span[q];
                const uint32_t voff = ok ? (uint32_t)(a_off[q] + lane_off) : kOutOfRange;
                const uint32_t to = dst + instr_index(q, T::A_PER_WAVE) * T::INSTR_BYTES;
                if constexpr (T::ELEM) dma4_buf(buf_in, voff, to); else dma16_buf(buf_in, voff, to);
            }
            const bool live = lane_r < filter_rows;
#pragma unroll
            for (int q = 0; q < T::B_PER_WAVE; ++q) {
                const uint32_t voff = live ? b_off[q] : kOutOfRange;
                const uint32_t to = dst + T::A_BYTES + instr_index(q, T::B_PER_WAVE) * T::INSTR_BYTES;
                if constexpr (T::ELEM) dma4_buf_s(buf_w, voff, (uint32_t)k0 * 4, to);
                else dma16_buf_s(buf_w, voff, (uint32_t)k0 * 4, to);
            }
            k0 += T::BK;
            lane_x += T::BK;
            lane_off += T::BK * 4;
            while (lane_x >= row_len) {  // at most once unless a filter row is shorter than a chunk
                lane_x -= row_len;
                lane_off += row_jump;
                ++lane_r;
            }
            return;
        }
        if (new_tap) {
            const int tap_off = ((tap_r * g.W + tap_s) * g.C) * 4;
#pragma unroll
            for (int q = 0; q < T::A_PER_WAVE; ++q) {
                const bool ok = (unsigned)(a_h0[q] + tap_r) < (unsigned)g.H &&
                                (unsigned)(a_w0[q] + tap_s) < (unsigned)g.W;
                a_cur[q] = ok ? (uint32_t)(a_off[q] + tap_off) : kOutOfRange;
            }
            new_tap = false;
        }
#pragma unroll
        for (int q = 0; q < T::A_PER_WAVE; ++q)
            dma16_buf_s(buf_in, a_cur[q], (uint32_t)tap_c * 4, dst + (wave * T::A_PER_WAVE + q) * 1024);
#pragma unroll
        for (int q = 0; q < T::B_PER_WAVE; ++q)
            dma16_buf_s(buf_w, b_off[q], (uint32_t)k0 * 4, dst + T::A_BYTES + (wave * T::B_PER_WAVE + q) * 1024);
        k0 += T::BK;
        tap_c += T::BK;
        if (tap_c == g.C) {
            tap_c = 0;
            new_tap = true;
            if (++tap_s == g.S) {
                tap_s = 0;
                ++tap_r;
            }
        }
    };

    // ---- fragment read offsets inside a stage (rows of a block differ from li by 32s) ----
    const int fsw = T::swizzle(li);
    const uint32_t a_row = (uint32_t)((wrow + li) * T::ROW_BYTES);
    const uint32_t b_row = (uint32_t)(T::A_BYTES + (wcol + li) * T::ROW_BYTES);

    f32x16 acc[T::TM][T::TN];
#pragma unroll
    for (int a = 0; a < T::TM; ++a)
#pragma unroll
        for (int b = 0; b < T::TN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    constexpr int U = T::BK / 8;
    struct Frags {
        f32x4 a[U][T::TM], b[U][T::TN];
    };
    auto read_frags = [&](int stage, Frags &f) {
        const unsigned char *st = lds + stage * T::STAGE_BYTES;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t goff = (uint32_t)(((2 * u + half) ^ fsw) * 16);
#pragma unroll
            for (int a = 0; a < T::TM; ++a)
                f.a[u][a] = *reinterpret_cast<const f32x4 *>(st + a_row + a * 32 * T::ROW_BYTES + goff);
#pragma unroll
            for (int b = 0; b < T::TN; ++b)
                f.b[u][b] = *reinterpret_cast<const f32x4 *>(st + b_row + b * 32 * T::ROW_BYTES + goff);
        }
    };
    auto multiply = [&](const Frags &f) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int a = 0; a < T::TM; ++a)
#pragma unroll
                    for (int b = 0; b < T::TN; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a[u][a][t], f.b[u][b][t],
                                                                        acc[a][b], 0, 0, 0);
    };

#pragma unroll
    for (int p = 0; p < T::NSTAGE - 1; ++p)
        if (p < nk) issue(p);

    if constexpr (T::AHEAD) {
        // Chunk c's fragments wait in registers x[c & 1].  Step c: once chunk c + 1 has landed
        // for every wave (at most NSTAGE - 3 later chunks stay in flight) and every wave is
        // through with chunk c - 1, request chunk c + NSTAGE - 1 into the stage chunk c - 1
        // leaves, start reading chunk c + 1 into the other registers, and multiply chunk c.
        Frags x[2];
        wait_chunks_and_barrier<T::LOADS, T::NSTAGE - 2>(min(T::NSTAGE - 2, nk - 1));
        read_frags(0, x[0]);
        constexpr int UNROLL = T::NSTAGE % 2 == 0 ? T::NSTAGE : 2 * T::NSTAGE;
        for (int it = 0; it < nk; it += UNROLL)
            static_for<UNROLL>([&](auto j_c) {
                constexpr int j = decltype(j_c)::value, stage = j % T::NSTAGE, buf = j % 2;
                const int c = it + j;
                if (c < nk) {
                    if (c + 1 < nk) {
                        wait_chunks_and_barrier<T::LOADS, T::NSTAGE - 3>(min(T::NSTAGE - 3, nk - 2 - c));
                        if (c + T::NSTAGE - 1 < nk) issue((stage + T::NSTAGE - 1) % T::NSTAGE);
                        read_frags((stage + 1) % T::NSTAGE, x[buf ^ 1]);
                    }
                    multiply(x[buf]);
                }
            });
    } else {
        // The next chunk's global loads are issued after the fragment reads and before the
        // first MFMA, under the LDS latency.
        auto step = [&](int it, auto stage_tag) {
            constexpr int stage = decltype(stage_tag)::value;
            const int ahead = nk - 1 - it;  // later chunks whose loads may stay in flight
            wait_chunks_and_barrier<T::LOADS, T::NSTAGE - 2>(min(T::NSTAGE - 2, ahead));
            Frags f;
            read_frags(stage, f);
            if (it + T::NSTAGE - 1 < nk) issue((stage + T::NSTAGE - 1) % T::NSTAGE);
            multiply(f);
        };
        for (int it = 0; it < nk; it += T::NSTAGE)
            static_for<T::NSTAGE>([&](auto s_c) {
                if (it + decltype(s_c)::value < nk) step(it + decltype(s_c)::value, s_c);
            });
    }

    // ---- epilogue: out = post(bias + acc); 32 lanes write 128 contiguous bytes of one pixel ----
    if (sliced) {
#pragma unroll
        for (int a = 0; a < T::TM; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wrow + 32 * a + 8 * (v >> 2) + 4 * half + (v & 3);
#pragma unroll
                for (int b = 0; b < T::TN; ++b) {
                    const int k = n0 + wcol + 32 * b + li;
                    if (m < g.pixels && k < g.K) atomicAdd(&out[(int64_t)m * g.K + k], acc[a][b][v]);
                }
            }
        return;
    }
    float init[T::TN];
#pragma unroll
    for (int b = 0; b < T::TN; ++b) {
        const int k = n0 + wcol + 32 * b + li;
        init[b] = (ep.pre == kPreBias && k < g.K) ? ep.bias[k] : 0.f;
    }
    // A tile that lies wholly inside the output stores without per-element tests: tested
    // stores sit in basic blocks of their own, and there each one would first wait for the
    // store before it to be acknowledged.
    if (m0 + T::BM <= g.pixels && n0 + T::BN <= g.K) {
        float *const dst = out + (int64_t)(m0 + wrow + 4 * half) * g.K + n0 + wcol + li;
#pragma unroll
        for (int a = 0; a < T::TM; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v)
#pragma unroll
                for (int b = 0; b < T::TN; ++b)
                    dst[(int64_t)(32 * a + 8 * (v >> 2) + (v & 3)) * g.K + 32 * b] =
                        apply_post(init[b] + acc[a][b][v], ep.post);
        return;
    }
#pragma unroll
    for (int a = 0; a < T::TM; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = m0 + wrow + 32 * a + 8 * (v >> 2) + 4 * half + (v & 3);
#pragma unroll
            for (int b = 0; b < T::TN; ++b) {
                const int k = n0 + wcol + 32 * b + li;
                if (m < g.pixels && k < g.K)
                    out[(int64_t)m * g.K + k] = apply_post(init[b] + acc[a][b][v], ep.post);
            }
        }
}

// The same tiles computed by workgroups that stay: the grid has a fixed number of workgroups
// per CU, workgroup w takes the tiles w, w + W, w + 2W, ... of the walk, and the ring of chunk
// buffers runs on across tile boundaries -- the first chunks of the next tile are requested
// while the last chunks of the current one are multiplied, its per-lane addresses are worked out
// half a tile ahead, and a finished tile's stores drain under the next tile's matrix
// instructions.  With one workgroup per tile every tile pays its own start (address arithmetic,
// the first loads' latency with nothing to multiply) and its own end (stores with nothing else
// to issue); here only the first and the last tile of a workgroup do.
// (The outstanding-load count of a wait never under-waits because of the stores in between:
// at most N operations outstanding means every load older than the newest N operations is back.)
template <class T>
__global__ __launch_bounds__(T::NT)
__attribute__((amdgpu_waves_per_eu(1, T::WAVES_PER_SIMD))) void conv2d_stream_kernel(
    ConvDmaGeom g, const float *__restrict__ in, const float *__restrict__ w,
    float *__restrict__ out, int tiles_m, int tiles_n, int pieces, int pieces_n, int m_cut, Epilogue ep)
{
    static_assert(!T::AHEAD && !T::GROUP_TAP, "chunks inside one tap, fragments read in step");
    __shared__ __attribute__((aligned(1024))) unsigned char lds[T::LDS_BYTES];
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
    if constexpr (T::NWAVES == 4 && T::LDS_BYTES >= 16384) {
        if ((int)blockIdx.x < pieces) {
            conv2d_piece<T>(g, in, w, out, (int)blockIdx.x, pieces_n, m_cut, ep, lds);
            return;
        }
    }

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, half = lane >> 5;
    const int wrow = (wave / T::WAVES_N) * T::WTM;
    const int wcol = (wave % T::WAVES_N) * T::WTN;

    const int wg = (int)blockIdx.x - pieces, stride_w = (int)gridDim.x - pieces;
    const int tiles = tiles_m * tiles_n;
    const int mine = (tiles - wg + stride_w - 1) / stride_w;  // tiles of this workgroup (the host launches W <= tiles)
    const int nk = g.red / T::BK;                             // chunks of a tile
    const int total = mine * nk;
    const i32x4 buf_in = make_buffer(in), buf_w = make_buffer(w);

    // per-lane DMA sources of one tile (byte offsets into the two buffers), as in conv2d_dma_kernel
    struct Source {
        int a_off[T::A_PER_WAVE], a_h0[T::A_PER_WAVE], a_w0[T::A_PER_WAVE];
        uint32_t b_off[T::B_PER_WAVE];
    };
    auto setup = [&](int tile, Source &s) __attribute__((always_inline)) {
        int tn, tm;
        g.tmap.locate(tile, tn, tm);
        const int m0 = tm * T::BM, n0 = tn * T::BN;
#pragma unroll
        for (int q = 0; q < T::A_PER_WAVE; ++q) {
            const int row = (wave * T::A_PER_WAVE + q) * T::ROWS_PER_INSTR + lane / T::GROUPS;
            const int grp = (lane % T::GROUPS) ^ T::swizzle(row);
            const int m = m0 + row;
            if (m < g.pixels) {
                const int n = (int)g.by_pq.div((uint32_t)m), pq = m - n * g.P * g.Q, p = (int)g.by_q.div((uint32_t)pq);
                s.a_h0[q] = p * g.stride - g.pad;
                s.a_w0[q] = (pq - p * g.Q) * g.stride - g.pad;
                s.a_off[q] = (n * g.hwc + (s.a_h0[q] * g.W + s.a_w0[q]) * g.C + grp * 4) * 4;
            } else {
                s.a_h0[q] = INT32_MIN / 2;  // fails every range test
                s.a_w0[q] = 0;
                s.a_off[q] = 0;
            }
        }
#pragma unroll
        for (int q = 0; q < T::B_PER_WAVE; ++q) {
            const int row = (wave * T::B_PER_WAVE + q) * T::ROWS_PER_INSTR + lane / T::GROUPS;
            const int grp = (lane % T::GROUPS) ^ T::swizzle(row);
            s.b_off[q] = n0 + row < g.K ? (uint32_t)(((n0 + row) * g.red + grp * 4) * 4) : kOutOfRange;
        }
    };
    Source src, nxt;
    setup(wg, src);
    nxt = src;

    // the walk of the requests: tile, chunk inside it, tap and channel of that chunk
    int lc = 0, k0 = 0, tap_c = 0, tap_s = 0, tap_r = 0;
    uint32_t a_cur[T::A_PER_WAVE];
    bool new_tap = true;
    auto issue = [&](int stage) __attribute__((always_inline)) {
        const uint32_t dst = lds_base + stage * T::STAGE_BYTES;
        if (new_tap) {
            const int tap_off = ((tap_r * g.W + tap_s) * g.C) * 4;
#pragma unroll
            for (int q = 0; q < T::A_PER_WAVE; ++q) {
                const bool ok = (unsigned)(src.a_h0[q] + tap_r) < (unsigned)g.H &&
                                (unsigned)(src.a_w0[q] + tap_s) < (unsigned)g.W;
                a_cur[q] = ok ? (uint32_t)(src.a_off[q] + tap_off) : kOutOfRange;
            }
            new_tap = false;
        }
#pragma unroll
        for (int q = 0; q < T::A_PER_WAVE; ++q)
            dma16_buf_s(buf_in, a_cur[q], (uint32_t)tap_c * 4, dst + (wave * T::A_PER_WAVE + q) * 1024);
#pragma unroll
        for (int q = 0; q < T::B_PER_WAVE; ++q)
            dma16_buf_s(buf_w, src.b_off[q], (uint32_t)k0 * 4, dst + T::A_BYTES + (wave * T::B_PER_WAVE + q) * 1024);
        k0 += T::BK;
        tap_c += T::BK;
        if (tap_c == g.C) {
            tap_c = 0;
            new_tap = true;
            if (++tap_s == g.S) {
                tap_s = 0;
                ++tap_r;
            }
        }
        // at the end of a tile's chunks the walk moves on to the next tile's sources, which the
        // tile loop below has worked out in the meantime
        if (++lc == nk) {
            lc = 0;
            k0 = tap_c = tap_s = tap_r = 0;
            new_tap = true;
            src = nxt;
        }
    };

    const int fsw = T::swizzle(li);
    const uint32_t a_row = (uint32_t)((wrow + li) * T::ROW_BYTES);
    const uint32_t b_row = (uint32_t)(T::A_BYTES + (wcol + li) * T::ROW_BYTES);

    f32x16 acc[T::TM][T::TN];
    auto clear = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int a = 0; a < T::TM; ++a)
#pragma unroll
            for (int b = 0; b < T::TN; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    };
    clear();

    constexpr int U = T::BK / 8;
    struct Frags {
        f32x4 a[U][T::TM], b[U][T::TN];
    };
    auto read_frags = [&](int stage, Frags &f) __attribute__((always_inline)) {
        const unsigned char *st = lds + stage * T::STAGE_BYTES;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t goff = (uint32_t)(((2 * u + half) ^ fsw) * 16);
#pragma unroll
            for (int a = 0; a < T::TM; ++a)
                f.a[u][a] = *reinterpret_cast<const f32x4 *>(st + a_row + a * 32 * T::ROW_BYTES + goff);
#pragma unroll
            for (int b = 0; b < T::TN; ++b)
                f.b[u][b] = *reinterpret_cast<const f32x4 *>(st + b_row + b * 32 * T::ROW_BYTES + goff);
        }
    };
    auto multiply = [&](const Frags &f) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int a = 0; a < T::TM; ++a)
#pragma unroll
                    for (int b = 0; b < T::TN; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a[u][a][t], f.b[u][b][t],
                                                                        acc[a][b], 0, 0, 0);
    };

    // out = post(bias + acc) for the tile just finished; 32 lanes write 128 contiguous bytes of one pixel
    auto store_tile = [&](int tile) __attribute__((always_inline)) {
        int tn, tm;
        g.tmap.locate(tile, tn, tm);
        const int m0 = tm * T::BM, n0 = tn * T::BN;
        float init[T::TN];
#pragma unroll
        for (int b = 0; b < T::TN; ++b) {
            const int k = n0 + wcol + 32 * b + li;
            init[b] = (ep.pre == kPreBias && k < g.K) ? ep.bias[k] : 0.f;
        }
        if (m0 + T::BM <= g.pixels && n0 + T::BN <= g.K) {
            float *const dst = out + (int64_t)(m0 + wrow + 4 * half) * g.K + n0 + wcol + li;
#pragma unroll
            for (int a = 0; a < T::TM; ++a)
#pragma unroll
                for (int v = 0; v < 16; ++v)
#pragma unroll
                    for (int b = 0; b < T::TN; ++b)
                        dst[(int64_t)(32 * a + 8 * (v >> 2) + (v & 3)) * g.K + 32 * b] =
                            apply_post(init[b] + acc[a][b][v], ep.post);
            return;
        }
#pragma unroll
        for (int a = 0; a < T::TM; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wrow + 32 * a + 8 * (v >> 2) + 4 * half + (v & 3);
#pragma unroll
                for (int b = 0; b < T::TN; ++b) {
                    const int k = n0 + wcol + 32 * b + li;
                    if (m < g.pixels && k < g.K)
                        out[(int64_t)m * g.K + k] = apply_post(init[b] + acc[a][b][v], ep.post);
                }
            }
    };

#pragma unroll
    for (int p = 0; p < T::NSTAGE - 1; ++p)
        if (p < total) issue(p);

    // The host launches this kernel only when nk is a multiple of NSTAGE, so that a tile starts
    // at stage 0 and the stage of a step is a compile-time constant inside the unrolled loop.
    for (int t = 0; t < mine; ++t) {
        const int tile = wg + t * stride_w;
        // sources of the tile after this one: its first requests come NSTAGE - 1 steps before
        // this tile's last multiply
        if (t + 1 < mine) setup(tile + stride_w, nxt);
        const int base = t * nk;
        for (int it = 0; it < nk; it += T::NSTAGE)
            static_for<T::NSTAGE>([&](auto s_c) __attribute__((always_inline)) {
                constexpr int stage = decltype(s_c)::value;
                const int step = base + it + stage;
                const int ahead = total - 1 - step;  // later chunks whose loads may stay in flight
                wait_chunks_and_barrier<T::LOADS, T::NSTAGE - 2>(min(T::NSTAGE - 2, ahead));
                Frags f;
                read_frags(stage, f);
                if (step + T::NSTAGE - 1 < total) issue((stage + T::NSTAGE - 1) % T::NSTAGE);
                multiply(f);
            });
        store_tile(tile);
        clear();
    }
}

}  // namespace lsmi
