// Depth-wise 2-D convolution, NHWC, fp32 (gfx950): the DWCONV rows of Table 1, i.e. the
// convolution of Section 2.1 with the channel kept as an output index,
//   out[n,p,q,c] = post(bias[c] + sum_{r,s} in[n, p*stride-pad+r, q*stride-pad+s, c] * w[r,s,c]).
//
// Per output element there are only R*S multiply-adds against one read and one write, so
// the operation is bound by HBM traffic, not by arithmetic, and has no use for the matrix
// cores.  What matters is that every input byte leaves HBM once and that all accesses are
// wide and coalesced:
//   - channels are innermost in memory, so a lane owns four consecutive channels (one
//     16-byte access) of one output column and consecutive lanes own consecutive channel
//     groups, then consecutive columns: loads and stores of a wave are contiguous;
//   - a lane walks down a strip of output rows and keeps the R x S input window of its
//     column in registers, so each step loads only the rows that enter the window
//     (`stride` of them); the S-fold reuse between neighbouring columns is served by the
//     vector L1;
//   - the rows for the next step are requested before the current step's arithmetic;
//   - the row loop is unrolled R times so that the rotating window is indexed statically
//     (no register moves, no scratch).
#include <mutex>

#include "common.hpp"
#include "tile_f32.hpp"
#include "sgemm_dma.hpp"

namespace lsmi {
namespace {

struct DwGeom {
    int N, H, W, C, R, S, stride, pad, P, Q;
    int cgroups;      // C / channels per lane
    int strip;        // output rows per lane
    int strips;       // ceil(P / strip)
    unsigned items;   // lanes with work: N * strips * Q * cgroups (below 2^31)
};

// Workgroup ids are dealt round-robin to the XCDs; regroup them so that each XCD works on
// one contiguous range of the item space (neighbouring strips share halo rows in its L2).
__device__ inline unsigned regrouped_block(unsigned blocks)
{
    const unsigned b = blockIdx.x;
    const unsigned q = blocks / kXcds, rem = blocks % kXcds;
    const unsigned xcd = b % kXcds, idx = b / kXcds;
    return xcd * q + (xcd < rem ? xcd : rem) + idx;
}

template <int VEC>
__device__ inline typename FVec<VEC>::type zero_vec()
{
    typename FVec<VEC>::type v;
#pragma unroll
    for (int e = 0; e < VEC; ++e) v[e] = 0.f;
    return v;
}

// f(0), f(1), ... as compile-time constants until one call returns false; true if none did.
template <class F, int... I>
__device__ __forceinline__ bool static_for_while_impl(F &&f, std::integer_sequence<int, I...>)
{
    return (f(std::integral_constant<int, I>{}) && ...);
}
template <int N, class F>
__device__ __forceinline__ bool static_for_while(F &&f)
{
    return static_for_while_impl(f, std::make_integer_sequence<int, N>{});
}

// VEC channels per lane (4, or 2 where the window of a larger filter would not leave
// enough registers for several waves per SIMD).  The rows that enter the window at the next
// step are requested before the current step's arithmetic and held in `next`.  (Requesting
// them two or three steps ahead was tried: the compiler's wait counts at the loop head
// then wait for every outstanding load anyway, and the extra registers cost a wave per SIMD.)
// FILTER_IN_LDS: the taps are read from a copy of the filter in LDS instead of being held
// in registers.
template <int R, int S, int STRIDE, int VEC, bool FILTER_IN_LDS>
__global__ __launch_bounds__(256) void dwconv_window_kernel(DwGeom g, const float *__restrict__ in,
                                                             const float *__restrict__ w,
                                                             float *__restrict__ out, Epilogue ep)
{
    typedef typename FVec<VEC>::type vec;
    constexpr int NEW = STRIDE < R ? STRIDE : R;          // rows entering the window per step
    constexpr int PERIOD = R;  // steps after which the window's slot indices repeat
    extern __shared__ float w_lds[];                      // [R*S][C] when FILTER_IN_LDS
    if constexpr (FILTER_IN_LDS) {
        for (int t = threadIdx.x; t < R * S * g.cgroups; t += 256)
            *reinterpret_cast<vec *>(w_lds + VEC * t) = *reinterpret_cast<const vec *>(w + VEC * (long long)t);
        __syncthreads();
    }
    const unsigned blocks = (g.items + 255u) / 256u;
    const unsigned item = regrouped_block(blocks) * 256u + threadIdx.x;
    if (item >= g.items) return;
    const unsigned ucg = (unsigned)g.cgroups, uq = (unsigned)g.Q, us = (unsigned)g.strips;
    const int cg = (int)(item % ucg);
    unsigned rest = item / ucg;
    const int q = (int)(rest % uq);
    rest /= uq;
    const int sb = (int)(rest % us);
    const int n = (int)(rest / us);
    const int p0 = sb * g.strip;
    const int rows = min(g.strip, g.P - p0);
    const int c = VEC * cg;

    // filter taps of this lane's channels
    vec f[FILTER_IN_LDS ? 1 : R * S];
    if constexpr (!FILTER_IN_LDS) {
#pragma unroll
        for (int t = 0; t < R * S; ++t) f[t] = *reinterpret_cast<const vec *>(w + (long long)t * g.C + c);
    }
    vec bias_v = zero_vec<VEC>();
    if (ep.bias) bias_v = *reinterpret_cast<const vec *>(ep.bias + c);

    // columns of the window: fixed for the whole strip
    const int x0 = q * STRIDE - g.pad;
    bool col_ok[S];
    int col_off[S];  // element offset of column s inside an image row (clamped when outside)
#pragma unroll
    for (int s = 0; s < S; ++s) {
        col_ok[s] = (unsigned)(x0 + s) < (unsigned)g.W;
        col_off[s] = (col_ok[s] ? x0 + s : 0) * g.C + c;
    }
    const float *img = in + (long long)n * g.H * g.W * g.C;
    const int h0 = p0 * STRIDE - g.pad;  // input row of window row 0 at step 0
    const int row_elems = g.W * g.C;

    // Every lane always issues its load: a row outside the image, or one that belongs to a
    // step past the end of the strip, is read from the image's first row, so addresses stay
    // valid and the body stays free of branches.  The loaded value is replaced by zero only
    // where it is consumed (mask_row), so that a request can stay in flight until then.
    auto row_wanted = [&](int h, bool wanted) { return wanted && (unsigned)h < (unsigned)g.H; };
    auto load_row = [&](int h, bool wanted, vec(&dst)[S]) {
        const float *row = img + (long long)(row_wanted(h, wanted) ? h : 0) * row_elems;
#pragma unroll
        for (int s = 0; s < S; ++s) dst[s] = *reinterpret_cast<const vec *>(row + col_off[s]);
    };
    auto mask_row = [&](int h, bool wanted, const vec(&src)[S], vec(&dst)[S]) {
        const bool row_ok = row_wanted(h, wanted);
#pragma unroll
        for (int s = 0; s < S; ++s) dst[s] = (row_ok && col_ok[s]) ? src[s] : zero_vec<VEC>();
    };
    // rows that enter the window at `step` >= 1: relative rows step*STRIDE + R-NEW .. + R-1
    auto load_step = [&](int step, vec(&dst)[NEW][S]) {
#pragma unroll
        for (int a = 0; a < NEW; ++a) load_row(h0 + step * STRIDE + R - NEW + a, step < rows, dst[a]);
    };

    vec win[R][S];             // window row j (relative input row) lives in slot j % R
    vec next[NEW][S];          // rows entering at the next step
#pragma unroll
    for (int r = 0; r < R; ++r) load_row(h0 + r, true, win[r]);
#pragma unroll
    for (int r = 0; r < R; ++r) mask_row(h0 + r, true, win[r], win[r]);

    float *dst = out + (((long long)n * g.P + p0) * g.Q + q) * g.C + c;
    const long long out_row = (long long)g.Q * g.C;

    for (int i0 = 0;; i0 += PERIOD) {
        const bool go_on = static_for_while<PERIOD>([&](auto phase_c) {
            constexpr int phase = decltype(phase_c)::value;
            const int i = i0 + phase;
            if (i >= rows) return false;
            load_step(i + 1, next);
            vec acc = bias_v;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int slot = (phase * STRIDE + r) % R;
#pragma unroll
                for (int s = 0; s < S; ++s) {
                    vec tap;
                    if constexpr (FILTER_IN_LDS)
                        tap = *reinterpret_cast<const vec *>(w_lds + (r * S + s) * g.C + c);
                    else
                        tap = f[r * S + s];
                    acc += win[slot][s] * tap;
                }
            }
            if (ep.post == kPostRelu) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] = fmaxf(acc[e], 0.f);
            }
            *reinterpret_cast<vec *>(dst + i * out_row) = acc;
#pragma unroll
            for (int a = 0; a < NEW; ++a) {
                const int slot = ((phase + 1) * STRIDE + R - NEW + a) % R;
                mask_row(h0 + (i + 1) * STRIDE + R - NEW + a, i + 1 < rows, next[a], win[slot]);
            }
            return true;
        });
        if (!go_on) break;
    }
}

// Any filter size, stride and channel count: one lane per output element (VEC = 1) or per
// four channels (VEC = 4), taps walked in a run-time loop.  The window is not kept, the
// R*S-fold reuse is left to the caches.
template <int VEC>
__global__ __launch_bounds__(256) void dwconv_direct_kernel(DwGeom g, const float *__restrict__ in,
                                                             const float *__restrict__ w,
                                                             float *__restrict__ out, Epilogue ep)
{
    typedef typename FVec<VEC>::type vec;
    const unsigned blocks = (g.items + 255u) / 256u;
    const unsigned item = regrouped_block(blocks) * 256u + threadIdx.x;
    if (item >= g.items) return;
    const int cg = (int)(item % (unsigned)g.cgroups);
    unsigned rest = item / (unsigned)g.cgroups;
    const int q = (int)(rest % (unsigned)g.Q);
    rest /= (unsigned)g.Q;
    const int p = (int)(rest % (unsigned)g.P);
    const int n = (int)(rest / (unsigned)g.P);
    const int c = VEC * cg;
    vec acc;
    if constexpr (VEC == 1) acc = ep.bias ? ep.bias[c] : 0.f;
    else acc = ep.bias ? *reinterpret_cast<const vec *>(ep.bias + c) : vec{0.f, 0.f, 0.f, 0.f};
    const float *img = in + (long long)n * g.H * g.W * g.C;
    for (int r = 0; r < g.R; ++r) {
        const int h = p * g.stride - g.pad + r;
        if ((unsigned)h >= (unsigned)g.H) continue;
        for (int s = 0; s < g.S; ++s) {
            const int x = q * g.stride - g.pad + s;
            if ((unsigned)x >= (unsigned)g.W) continue;
            const vec a = *reinterpret_cast<const vec *>(img + ((long long)h * g.W + x) * g.C + c);
            const vec b = *reinterpret_cast<const vec *>(w + (long long)(r * g.S + s) * g.C + c);
            acc += a * b;
        }
    }
    if (ep.post == kPostRelu) {
        if constexpr (VEC == 1) acc = fmaxf(acc, 0.f);
        else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] = fmaxf(acc[e], 0.f);
        }
    }
    *reinterpret_cast<vec *>(out + (((long long)n * g.P + p) * g.Q + q) * g.C + c) = acc;
}

// ---------------------------------------------------------------------------------------
// LDS-staged kernel.  The vector L1 is the narrow point of the register-window kernels: it
// sees every input element S times.  Here each input row segment travels HBM -> LDS once,
// as plain contiguous direct-to-LDS loads, and the R*S-fold reuse is served by LDS reads.
//
// A workgroup owns a tile of TQB output columns x CB channels of one image and walks down a
// band of output rows, TP rows per step.  Input rows live in a ring of NR row slots in LDS
// (slot = zero-padded row segment, [in_cols][CB] floats; padding and rows outside the image
// are loads with an out-of-range buffer offset, which write zeros, so the arithmetic needs
// no masks).  Wave 4 does nothing but issue the loads, PD steps ahead; because it issues no
// other memory operation, "the rows of step b have landed" is exactly "at most the loads of
// the younger steps are outstanding", a plain s_waitcnt.  Waves 0..3 compute: one barrier
// per step hands a step's rows over and releases the slots of the step before.
struct DwLdsGeom {
    int N, H, W, C, stride, pad, P, Q;
    int tqb, cb;         // output columns and channels per tile
    int in_cols;         // (tqb-1)*stride + S input columns per slot
    int cbg;             // cb / 4
    int slot_bytes;      // in_cols*cb*4 rounded up to a multiple of 1024
    int chr;             // slot_bytes / 1024: load instructions per row
    int nr;              // row slots in the ring
    int pd;              // steps the loads run ahead (1 or 2)
    int band_rows;       // output rows per workgroup
    int bands, qtiles, ctiles;
    int taps_bytes;      // R*S*cb*4
    unsigned tiles;      // N*bands*qtiles*ctiles
};

constexpr int kDwMaxChunks = 16;  // a row slot is at most 16 KiB
constexpr int kDwMaxPasses = 4;   // a tile has at most 1024 (column, channel group) items

__device__ __forceinline__ void wait_vmcnt_dynamic(int n)
{
#define LSMI_WAIT_CASE(k) case k: asm volatile("s_waitcnt vmcnt(" #k ")" ::: "memory"); break;
    switch (n) {
        LSMI_WAIT_CASE(0) LSMI_WAIT_CASE(1) LSMI_WAIT_CASE(2) LSMI_WAIT_CASE(3) LSMI_WAIT_CASE(4)
        LSMI_WAIT_CASE(5) LSMI_WAIT_CASE(6) LSMI_WAIT_CASE(7) LSMI_WAIT_CASE(8) LSMI_WAIT_CASE(9)
        LSMI_WAIT_CASE(10) LSMI_WAIT_CASE(11) LSMI_WAIT_CASE(12) LSMI_WAIT_CASE(13) LSMI_WAIT_CASE(14)
        LSMI_WAIT_CASE(15) LSMI_WAIT_CASE(16) LSMI_WAIT_CASE(17) LSMI_WAIT_CASE(18) LSMI_WAIT_CASE(19)
        LSMI_WAIT_CASE(20) LSMI_WAIT_CASE(21) LSMI_WAIT_CASE(22) LSMI_WAIT_CASE(23) LSMI_WAIT_CASE(24)
        LSMI_WAIT_CASE(25) LSMI_WAIT_CASE(26) LSMI_WAIT_CASE(27) LSMI_WAIT_CASE(28) LSMI_WAIT_CASE(29)
        LSMI_WAIT_CASE(30) LSMI_WAIT_CASE(31) LSMI_WAIT_CASE(32) LSMI_WAIT_CASE(33) LSMI_WAIT_CASE(34)
        LSMI_WAIT_CASE(35) LSMI_WAIT_CASE(36) LSMI_WAIT_CASE(37) LSMI_WAIT_CASE(38) LSMI_WAIT_CASE(39)
        LSMI_WAIT_CASE(40) LSMI_WAIT_CASE(41) LSMI_WAIT_CASE(42) LSMI_WAIT_CASE(43) LSMI_WAIT_CASE(44)
        LSMI_WAIT_CASE(45) LSMI_WAIT_CASE(46) LSMI_WAIT_CASE(47) LSMI_WAIT_CASE(48)
    default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    }
#undef LSMI_WAIT_CASE
}

// Loader wave: requests input rows first .. first+count-1 (relative to h_begin) into their
// ring slots, chr load instructions per row; coff[j] is the lane's byte offset inside an
// image row for chunk j, or kOutOfRange.
__device__ __forceinline__ void dw_issue_rows(i32x4 rsrc, const uint32_t (&coff)[kDwMaxChunks], int first,
                                              int count, int h_begin, int H, uint32_t img_bytes,
                                              uint32_t row_bytes, uint32_t ring_addr, int nr, int slot_bytes,
                                              int chr)
{
    for (int rel = first; rel < first + count; ++rel) {
        const int h = h_begin + rel;
        const bool row_ok = (unsigned)h < (unsigned)H;
        const uint32_t base = img_bytes + (uint32_t)(row_ok ? h : 0) * row_bytes;
        const uint32_t slot_addr = ring_addr + (uint32_t)(rel % nr) * slot_bytes;
#pragma unroll
        for (int j = 0; j < kDwMaxChunks; ++j) {
            if (j < chr) {
                const uint32_t voff = (row_ok && coff[j] != kOutOfRange) ? base + coff[j] : kOutOfRange;
                dma16_buf(rsrc, voff, (uint32_t)__builtin_amdgcn_readfirstlane((int)(slot_addr + 1024u * j)));
            }
        }
    }
}

// TAPS_IN_REGS: a tile has at most 256 items (one pass) and each lane keeps the R*S taps of
// its channel group in registers instead of reading them from LDS at every step.
// QP: neighbouring output columns per lane.  Their windows overlap, so a lane reads
// (QP-1)*STRIDE + S window columns and S taps per window row for QP outputs instead of S and
// S for one: with a 5x5 filter, where the LDS reads are what bounds the kernel, 27.5 (QP = 2)
// or 16.25 (QP = 4) reads per output instead of 50.  The planner keeps the tile's column
// count a multiple of QP, so the extra columns a lane reads are inside the slot.
template <int R, int S, int STRIDE, int TP, bool TAPS_IN_REGS, int QP = 1>
__global__ __launch_bounds__(320, 3) void dwconv_lds_kernel(DwLdsGeom g, const float *__restrict__ in,
                                                         const float *__restrict__ w,
                                                         float *__restrict__ out, Epilogue ep)
{
    static_assert(STRIDE <= R, "a step's window overlaps the next one");
    constexpr int TPS = TP * STRIDE;            // input rows that enter per step
    constexpr int WIN = (TP - 1) * STRIDE + R;  // input rows one step reads
    constexpr int WS = (QP - 1) * STRIDE + S;   // window columns one lane reads
    extern __shared__ __attribute__((aligned(1024))) unsigned char dw_lds[];
    unsigned char *ring = dw_lds;                                                  // nr slots
    float *taps = reinterpret_cast<float *>(dw_lds + (size_t)g.nr * g.slot_bytes);  // [cb/4][R*S] float4

    // tile of this workgroup: channel tile fastest, then column tile, band, image
    unsigned t = regrouped_block(g.tiles);
    const int ct = (int)(t % (unsigned)g.ctiles);
    t /= (unsigned)g.ctiles;
    const int qt = (int)(t % (unsigned)g.qtiles);
    t /= (unsigned)g.qtiles;
    const int band = (int)(t % (unsigned)g.bands);
    const int n = (int)(t / (unsigned)g.bands);
    const int c0 = ct * g.cb;
    const int cbg = min(g.cbg, (g.C - c0) / 4);  // channel groups of this tile
    const int q0 = qt * g.tqb;
    const int nq = min(g.tqb, g.Q - q0);
    const int p_begin = band * g.band_rows;
    const int p_end = min(g.P, p_begin + g.band_rows);
    const int nsteps = (p_end - p_begin + TP - 1) / TP;
    const int h_begin = p_begin * STRIDE - g.pad;
    const int x_begin = q0 * STRIDE - g.pad;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: the role branch is uniform

    // filter taps of the tile's channels -> LDS, [channel group][tap] float4: a lane's taps
    // are then at compile-time offsets from one address
    for (int i = tid; i < R * S * cbg; i += 320) {
        const int tap = i / cbg, cg = i % cbg;
        *reinterpret_cast<f32x4 *>(taps + (cg * R * S + tap) * 4) =
            *reinterpret_cast<const f32x4 *>(w + (long long)tap * g.C + c0 + 4 * cg);
    }
    __syncthreads();

    if (wave == 4) {
        // ---- loader wave ----
        // It shares a SIMD with a compute wave and issues a handful of instructions per step:
        // at the default priority the arbiter prefers the older compute wave whenever that
        // one is ready, and the loads of the next steps go out late.
        __builtin_amdgcn_s_setprio(3);
        const int lane = tid - 256;
        const uint32_t ring_addr = (uint32_t)(uintptr_t)ring;
        // byte offset, inside an image row, of the 16 bytes this lane moves for chunk j of a
        // row (chunk = lane + 64 j, laid out [column][channel group]); out of range for
        // columns outside the image, channel groups past C and chunks past the slot
        uint32_t coff[kDwMaxChunks];
#pragma unroll
        for (int j = 0; j < kDwMaxChunks; ++j) {
            const int k = lane + 64 * j;
            const int px = k / g.cbg, cg = k % g.cbg;
            const int x = x_begin + px;
            const bool ok = px < g.in_cols && cg < cbg && (unsigned)x < (unsigned)g.W;
            coff[j] = ok ? (uint32_t)(x * g.C + c0 + 4 * cg) * 4u : kOutOfRange;
        }
        const uint32_t row_bytes = (uint32_t)g.W * g.C * 4u;
        const uint32_t img_bytes = (uint32_t)n * g.H * row_bytes;
        // group 0 = the WIN rows of step 0, group j >= 1 = the TPS rows that enter at step j
        auto issue_group = [&](int j) {
            const int first = j == 0 ? 0 : WIN + (j - 1) * TPS;
            const int count = j == 0 ? WIN : TPS;
            dw_issue_rows(make_buffer(in), coff, first, count, h_begin, g.H, img_bytes, row_bytes, ring_addr,
                          g.nr, g.slot_bytes, g.chr);
        };
        for (int j = 0; j < g.pd; ++j)
            if (j < nsteps) issue_group(j);
        for (int b = 0; b < nsteps; ++b) {
            // groups younger than b that have been issued: b+1 .. min(b+pd-1, nsteps-1)
            const int younger = min(b + g.pd - 1, nsteps - 1) - b;
            wait_vmcnt_dynamic(younger * TPS * g.chr);
            asm volatile("s_barrier" ::: "memory");
            if (b + g.pd < nsteps) issue_group(b + g.pd);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        return;
    }

    // ---- compute waves ----
    const int items = (nq + QP - 1) / QP * cbg;
    constexpr int NPASS = TAPS_IN_REGS ? 1 : kDwMaxPasses;
    int lds_col[NPASS];         // float offset of (first window column, channel group) in a slot
    long long out_off[NPASS];   // float offset of (first column, channel) in an output row
    int tap_off[NPASS];         // channel group of the item inside the tile
    int ncol[NPASS];            // columns of the item inside the tile (QP, fewer at its right edge)
#pragma unroll
    for (int ps = 0; ps < NPASS; ++ps) {
        const int it = tid + 256 * ps;
        const int q = it / cbg * QP, cg = it % cbg;
        lds_col[ps] = it < items ? (q * STRIDE * g.cbg + cg) * 4 : -1;
        out_off[ps] = (long long)(q0 + q) * g.C + c0 + 4 * cg;
        tap_off[ps] = cg;
        ncol[ps] = min(QP, nq - q);
    }
    const f32x4 zero = zero_vec<4>();
    float *out_img = out + (long long)n * g.P * g.Q * g.C;
    const long long out_row = (long long)g.Q * g.C;
    const int slot_floats = g.slot_bytes / 4;
    const float *ringf = reinterpret_cast<const float *>(ring);
    f32x4 tapreg[TAPS_IN_REGS ? R * S : 1];
    if constexpr (TAPS_IN_REGS) {
#pragma unroll
        for (int k = 0; k < R * S; ++k)
            tapreg[k] = lds_col[0] < 0 ? zero : reinterpret_cast<const f32x4 *>(taps)[tap_off[0] * (R * S) + k];
    }

    // The bias is loaded once, ahead of the steps: a global load inside the step loop makes
    // the compiler wait for the vector-memory counter to reach zero there, and that counter
    // also holds the previous step's output stores, so every step would wait for its
    // predecessor's stores to be acknowledged by the memory (2 - 3 us a step under load).
    f32x4 bias_of[NPASS];
#pragma unroll
    for (int ps = 0; ps < NPASS; ++ps) {
        bias_of[ps] = zero;
        if (ep.bias && lds_col[ps] >= 0) bias_of[ps] = *reinterpret_cast<const f32x4 *>(ep.bias + c0 + 4 * tap_off[ps]);
    }
    int slot0 = 0;  // ring slot of the step's first window row
    for (int b = 0; b < nsteps; ++b) {
        asm volatile("s_barrier" ::: "memory");
        // ring slot of window row rr: one conditional subtraction, WIN <= nr
        auto slot_of = [&](int rr) {
            const int sl = slot0 + rr;
            return sl >= g.nr ? sl - g.nr : sl;
        };
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) {
            if (lds_col[ps] < 0) continue;
            f32x4 acc[TP][QP];
            const f32x4 bias4 = bias_of[ps];
            const f32x4 *my_taps = reinterpret_cast<const f32x4 *>(taps) + tap_off[ps] * (R * S);
#pragma unroll
            for (int ti = 0; ti < TP; ++ti)
#pragma unroll
                for (int j = 0; j < QP; ++j) acc[ti][j] = bias4;
#pragma unroll
            for (int rr = 0; rr < WIN; ++rr) {
                const float *row = ringf + slot_of(rr) * slot_floats + lds_col[ps];
                f32x4 v[WS];
#pragma unroll
                for (int ss = 0; ss < WS; ++ss) v[ss] = *reinterpret_cast<const f32x4 *>(row + ss * g.cbg * 4);
#pragma unroll
                for (int ti = 0; ti < TP; ++ti) {
                    const int r = rr - ti * STRIDE;  // filter row that meets window row rr in output ti
                    if (r >= 0 && r < R) {
#pragma unroll
                        for (int ss = 0; ss < S; ++ss) {
                            const f32x4 tap = TAPS_IN_REGS ? tapreg[r * S + ss] : my_taps[r * S + ss];
#pragma unroll
                            for (int j = 0; j < QP; ++j) acc[ti][j] += v[j * STRIDE + ss] * tap;
                        }
                    }
                }
                // A 5x5 filter: finish this row's multiply-adds here and keep the LDS reads of
                // later rows below.  Without the tie to `acc` the compiler sinks every
                // multiply-add into the `p < p_end` block of the store, below all R*S window
                // and tap reads, and spills most of what they returned.  (Requesting row rr+1
                // ahead of row rr's arithmetic was measured too: 20 to 40 % slower.)
                if constexpr (R * S > 9) {
#pragma unroll
                    for (int ti = 0; ti < TP; ++ti)
#pragma unroll
                        for (int j = 0; j < QP; ++j) asm volatile("" : "+v"(acc[ti][j])::"memory");
                }
            }
#pragma unroll
            for (int ti = 0; ti < TP; ++ti) {
                const int p = p_begin + b * TP + ti;
                if (p < p_end) {
#pragma unroll
                    for (int j = 0; j < QP; ++j) {
                        if (j >= ncol[ps]) break;
                        f32x4 o = acc[ti][j];
                        if (ep.post == kPostRelu) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) o[e] = fmaxf(o[e], 0.f);
                        }
                        *reinterpret_cast<f32x4 *>(out_img + p * out_row + out_off[ps] + (long long)j * g.C) = o;
                    }
                }
            }
        }
        slot0 += TPS;  // TPS <= nr
        if (slot0 >= g.nr) slot0 -= g.nr;
    }
}

typedef void (*DwLdsKernel)(DwLdsGeom, const float *, const float *, float *, Epilogue);

typedef void (*DwKernel)(DwGeom, const float *, const float *, float *, Epilogue);

struct DwVariant {
    const char *name;
    int R, S, stride;  // 0 = any
    int vec;           // channels per lane
    bool lds_filter;
    DwKernel kernel;
    int tp;            // LDS-staged kernels: output rows per step (else 0)
    bool one_pass;     // LDS-staged kernels: taps in registers, at most 256 items per tile
    DwLdsKernel lds_kernel;
    int qp = 1;        // LDS-staged kernels: output columns per lane
};

const DwVariant kDwVariants[] = {
    {"dwconv_window_3x3_s1_v4", 3, 3, 1, 4, false, dwconv_window_kernel<3, 3, 1, 4, false>, 0, false, nullptr},
    {"dwconv_window_3x3_s2_v4", 3, 3, 2, 4, false, dwconv_window_kernel<3, 3, 2, 4, false>, 0, false, nullptr},
    {"dwconv_window_5x5_s1_v2", 5, 5, 1, 2, true, dwconv_window_kernel<5, 5, 1, 2, true>, 0, false, nullptr},
    {"dwconv_window_5x5_s2_v2", 5, 5, 2, 2, true, dwconv_window_kernel<5, 5, 2, 2, true>, 0, false, nullptr},
    {"dwconv_direct_vec4", 0, 0, 0, 4, false, dwconv_direct_kernel<4>, 0, false, nullptr},
    {"dwconv_direct_scalar", 0, 0, 0, 1, false, dwconv_direct_kernel<1>, 0, false, nullptr},
    {"dwconv_lds_3x3_s1_tp2", 3, 3, 1, 4, false, nullptr, 2, false, dwconv_lds_kernel<3, 3, 1, 2, false>},
    {"dwconv_lds_3x3_s1_tp2_regs", 3, 3, 1, 4, false, nullptr, 2, true, dwconv_lds_kernel<3, 3, 1, 2, true>},
    {"dwconv_lds_3x3_s1_tp4", 3, 3, 1, 4, false, nullptr, 4, false, dwconv_lds_kernel<3, 3, 1, 4, false>},
    {"dwconv_lds_3x3_s1_tp4_regs", 3, 3, 1, 4, false, nullptr, 4, true, dwconv_lds_kernel<3, 3, 1, 4, true>},
    {"dwconv_lds_3x3_s2_tp1", 3, 3, 2, 4, false, nullptr, 1, false, dwconv_lds_kernel<3, 3, 2, 1, false>},
    {"dwconv_lds_3x3_s2_tp1_regs", 3, 3, 2, 4, false, nullptr, 1, true, dwconv_lds_kernel<3, 3, 2, 1, true>},
    {"dwconv_lds_3x3_s2_tp2", 3, 3, 2, 4, false, nullptr, 2, false, dwconv_lds_kernel<3, 3, 2, 2, false>},
    {"dwconv_lds_3x3_s2_tp2_regs", 3, 3, 2, 4, false, nullptr, 2, true, dwconv_lds_kernel<3, 3, 2, 2, true>},
    {"dwconv_lds_5x5_s1_tp1", 5, 5, 1, 4, false, nullptr, 1, false, dwconv_lds_kernel<5, 5, 1, 1, false>},
    {"dwconv_lds_5x5_s1_tp1_regs", 5, 5, 1, 4, false, nullptr, 1, true, dwconv_lds_kernel<5, 5, 1, 1, true>},
    {"dwconv_lds_5x5_s2_tp1", 5, 5, 2, 4, false, nullptr, 1, false, dwconv_lds_kernel<5, 5, 2, 1, false>},
    {"dwconv_lds_5x5_s2_tp1_regs", 5, 5, 2, 4, false, nullptr, 1, true, dwconv_lds_kernel<5, 5, 2, 1, true>},
    {"dwconv_lds_5x5_s1_tp1_q2", 5, 5, 1, 4, false, nullptr, 1, false, dwconv_lds_kernel<5, 5, 1, 1, false, 2>, 2},
    {"dwconv_lds_5x5_s1_tp1_q2_regs", 5, 5, 1, 4, false, nullptr, 1, true, dwconv_lds_kernel<5, 5, 1, 1, true, 2>, 2},
    {"dwconv_lds_3x3_s1_tp2_q2", 3, 3, 1, 4, false, nullptr, 2, false, dwconv_lds_kernel<3, 3, 1, 2, false, 2>, 2},
    {"dwconv_lds_3x3_s1_tp2_q2_regs", 3, 3, 1, 4, false, nullptr, 2, true, dwconv_lds_kernel<3, 3, 1, 2, true, 2>, 2},
    {"dwconv_lds_3x3_s2_tp1_q2_regs", 3, 3, 2, 4, false, nullptr, 1, true, dwconv_lds_kernel<3, 3, 2, 1, true, 2>, 2},
    // 7x7 (the depth-wise layers of recent convolutional networks): 49 taps do not fit in registers,
    // and with taps and window both read from LDS the reads per output decide: 98 with one column
    // per lane, 52 with two, 30 with four
    {"dwconv_lds_7x7_s1_tp1", 7, 7, 1, 4, false, nullptr, 1, false, dwconv_lds_kernel<7, 7, 1, 1, false>},
    {"dwconv_lds_7x7_s1_tp1_q2", 7, 7, 1, 4, false, nullptr, 1, false, dwconv_lds_kernel<7, 7, 1, 1, false, 2>, 2},
    {"dwconv_lds_7x7_s1_tp1_q4", 7, 7, 1, 4, false, nullptr, 1, false, dwconv_lds_kernel<7, 7, 1, 1, false, 4>, 4},
    {"dwconv_lds_7x7_s2_tp1", 7, 7, 2, 4, false, nullptr, 1, false, dwconv_lds_kernel<7, 7, 2, 1, false>},
    {"dwconv_lds_7x7_s2_tp1_q2", 7, 7, 2, 4, false, nullptr, 1, false, dwconv_lds_kernel<7, 7, 2, 1, false, 2>, 2},
};
constexpr int kDwDirectVec = 4, kDwDirectScalar = 5, kDwLds3x3S1Regs = 7, kDwLds5x5S1 = 14, kDwLds5x5S2 = 16;
constexpr int kDwLds5x5S2Regs = 17, kDwLds5x5S1Pair = 18, kDwLds5x5S1PairRegs = 19, kDwLds3x3S1PairRegs = 21;
constexpr int kDwLds7x7S1 = 23, kDwLds7x7S1Pair = 24, kDwLds7x7S2 = 26, kDwLds7x7S2Pair = 27;  // (25: four columns per lane, a tuner's candidate)
constexpr int kDwVariantCount = sizeof(kDwVariants) / sizeof(kDwVariants[0]);
constexpr int kDwLdsBudget = 78 * 1024;  // two workgroups per CU

// Tile shape of an LDS-staged kernel for one call: searches channels per tile, columns per
// tile and prefetch depth under the limits of the kernel (slot size, item count, wait
// count, LDS) and keeps the cheapest by a traffic / lane-use estimate.  Returns false when
// nothing fits.
bool plan_lds(const DwVariant &v, int N, int H, int W, int C, int stride, int pad, int P, int Q, int cus,
              const ThreadState &ts, DwLdsGeom &best)
{
    const int R = v.R, S = v.S, tp = v.tp;
    const int tps = tp * stride, win = (tp - 1) * stride + R;
    double best_cost = 1e30;
    bool found = false;
    for (int ck = 1; ck <= 16; ++ck) {
        if (C % ck != 0 || (C / ck) % 4 != 0) continue;
        const int cb = C / ck;
        if (ts.forced_dwconv_channels > 0 && cb != ts.forced_dwconv_channels) continue;
        for (int qk = 1; qk <= Q && qk <= 64; ++qk) {
            const int tqb = ((Q + qk - 1) / qk + v.qp - 1) / v.qp * v.qp;
            if (qk > 1 && tqb == ((Q + qk - 2) / (qk - 1) + v.qp - 1) / v.qp * v.qp) continue;  // same tile as the previous split
            if (ts.forced_dwconv_cols > 0 && tqb != (ts.forced_dwconv_cols + v.qp - 1) / v.qp * v.qp) continue;
            const int in_cols = (tqb - 1) * stride + S;
            const long long raw = (long long)in_cols * cb * 4;
            const int slot = (int)((raw + 1023) / 1024 * 1024);
            const int chr = slot / 1024;
            const int items = tqb / v.qp * (cb / 4);
            if (chr > kDwMaxChunks || items > 256 * (v.one_pass ? 1 : kDwMaxPasses)) continue;
            for (int pd = 2; pd >= 1; --pd) {
                if (ts.forced_dwconv_depth > 0 && pd != ts.forced_dwconv_depth) continue;
                const int nr = win + pd * tps;
                const long long lds = (long long)nr * slot + (long long)R * S * cb * 4;
                if (lds > kDwLdsBudget || (pd - 1) * tps * chr > 48) continue;
                const double halo_x = (double)in_cols / (tqb * stride);
                const double lane_eff = (double)items / (256.0 * ((items + 255) / 256));
                const double pad_eff = (double)raw / slot;
                double cost = halo_x / (lane_eff * pad_eff);
                if (pd == 1) cost *= 1.1;
                if (cb * 4 < 128) cost *= 1.3;  // short runs per pixel
                if (cost < best_cost) {
                    best_cost = cost;
                    found = true;
                    best = DwLdsGeom{N, H, W, C, stride, pad, P, Q, tqb, cb, in_cols, cb / 4, slot, chr, nr, pd,
                                     0, 0, (Q + tqb - 1) / tqb, ck, R * S * cb * 4, 0};
                }
            }
        }
    }
    if (!found) return false;
    // a workgroup walks a whole image column (long bands amortise the pipeline fill) unless
    // that leaves fewer than two workgroups per CU; bands are at least two steps long
    const long long base = (long long)N * best.qtiles * best.ctiles;
    long long bands = (2LL * cus + base - 1) / base;
    const int max_bands = (P + 2 * tp - 1) / (2 * tp);
    if (bands > max_bands) bands = max_bands;
    if (bands < 1) bands = 1;
    int band_rows = (int)((P + bands - 1) / bands);
    band_rows = (band_rows + tp - 1) / tp * tp;
    if (ts.forced_dwconv_strip > 0) band_rows = (ts.forced_dwconv_strip + tp - 1) / tp * tp;
    best.band_rows = band_rows;
    best.bands = (P + band_rows - 1) / band_rows;
    const long long tiles = (long long)N * best.bands * best.qtiles * best.ctiles;
    if (tiles > INT32_MAX) return false;
    best.tiles = (unsigned)tiles;
    return true;
}

}  // namespace

int dwconv_variant_count() { return kDwVariantCount; }

const char *dwconv_variant_name(int index)
{
    return index >= 0 && index < kDwVariantCount ? kDwVariants[index].name : nullptr;
}

int launch_dwconv2d(int N, int H, int W, int C, int R, int S, int stride, int pad, int P, int Q,
                    const float *in, const float *w, float *out, const float *bias, int post)
{
    ThreadState &ts = tls();
    const int cus = device_cu_count();
    DwLdsGeom lg{};
    // max_halo: an LDS-staged kernel is taken only if its tile's input columns per output
    // column (times the stride) stay below it, a channel split leaves runs of at least 256
    // contiguous bytes per pixel, and at least 80 % of the lanes of its passes have an item
    auto fits = [&](int i, double max_halo = 1e9) {
        const DwVariant &v = kDwVariants[i];
        const uintptr_t mask = 4 * v.vec - 1;
        auto aligned = [&](const void *p) { return (reinterpret_cast<uintptr_t>(p) & mask) == 0; };
        if (C % v.vec != 0 || !aligned(in) || !aligned(w) || !aligned(out) || !aligned(bias)) return false;
        if (v.R == 0) return true;
        if (H == 0 || W == 0) return false;  // the window kernels read clamped addresses
        if (v.R != R || v.S != S || v.stride != stride) return false;
        if (v.lds_kernel != nullptr) {
            // buffer offsets of the loader are 31-bit
            if ((long long)N * H * W * C * 4 >= (1LL << 31)) return false;
            if (!plan_lds(v, N, H, W, C, stride, pad, P, Q, cus, ts, lg)) return false;
            if (max_halo >= 1e9) return true;
            const int items = lg.tqb / v.qp * lg.cbg;
            return (double)lg.in_cols <= max_halo * lg.tqb * stride && (lg.ctiles == 1 || lg.cb * 4 >= 256) &&
                   items * 5 >= (items + 255) / 256 * 256 * 4;
        }
        // the LDS copy of the filter stays within the 64 KiB a kernel gets without opting in
        return !v.lds_filter || (size_t)R * S * C * 4 <= 64 * 1024;
    };
    // built-in choice: the first kernel of the list that fits.  Measured on the Table 1 shapes
    // and six more (batch 32 - 256): for 5x5 the LDS-staged kernels lead, at stride 1 with two
    // output columns per lane (the register window of a 5x5 filter does not fit four waves
    // per SIMD); for 3x3 stride 1 the LDS-staged kernels with the taps in registers (4.4
    // against 3.9 TB/s on DWCONV-3) unless the 256 items of their single pass force narrow
    // column tiles with a wide halo, short channel runs or many idle lanes: then two columns
    // per lane under the same conditions, else the register-window kernel, which also serves
    // 3x3 stride 2 (4.8 against 4.7 TB/s).  7x7 (batch 32): the LDS-staged kernels with two columns
    // per lane at stride 1 (56x56x96 115 us on the direct kernel, 52.5 here; 28x28x192 58.8 -> 24.3;
    // four columns per lane: 58.0 and 29.0) and one at stride 2 (112x112x96 131 -> 80.6).
    struct Choice {
        int index;
        double max_halo;
    };
    const Choice order[] = {{kDwLds5x5S1PairRegs, 1e9}, {kDwLds5x5S1Pair, 1e9}, {kDwLds5x5S1, 1e9},
                            {kDwLds5x5S2Regs, 1e9},     {kDwLds5x5S2, 1e9},     {kDwLds3x3S1Regs, 1.25},
                            {kDwLds3x3S1PairRegs, 1.25}, {kDwLds7x7S1Pair, 1e9}, {kDwLds7x7S1, 1e9},
                            {kDwLds7x7S2, 1e9},         {kDwLds7x7S2Pair, 1e9},   {0, 1e9},
                            {1, 1e9},                   {2, 1e9},               {3, 1e9},
                            {kDwDirectVec, 1e9}};
    int vi = kDwDirectScalar;
    const bool large = (long long)N * P * Q * C >= (1LL << 21);  // below that a call is launch-bound
    for (const Choice &c : order) {
        if (kDwVariants[c.index].lds_kernel != nullptr && !large) continue;
        if (fits(c.index, c.max_halo)) {
            vi = c.index;
            break;
        }
    }
    if (ts.forced_dwconv_variant >= 0 && fits(ts.forced_dwconv_variant)) vi = ts.forced_dwconv_variant;
    const DwVariant &v = kDwVariants[vi];
    Epilogue ep{bias, bias ? kPreBias : kPreZero, post};

    if (v.lds_kernel != nullptr) {
        if (!plan_lds(v, N, H, W, C, stride, pad, P, Q, cus, ts, lg)) return LSMI_ERR_LAUNCH;
        const size_t lds = (size_t)lg.nr * lg.slot_bytes + lg.taps_bytes;
        static std::once_flag raised[kDwVariantCount];
        static hipError_t raise_status[kDwVariantCount];
        std::call_once(raised[vi], [&] {
            raise_status[vi] = hipFuncSetAttribute(reinterpret_cast<const void *>(v.lds_kernel),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, kDwLdsBudget);
        });
        if (raise_status[vi] != hipSuccess) {
            ts.last_hip_error = (int)raise_status[vi];
            return LSMI_ERR_LAUNCH;
        }
        v.lds_kernel<<<dim3(lg.tiles), dim3(320), lds, ts.stream>>>(lg, in, w, out, ep);
        int rc = check_launch();
        if (rc == LSMI_OK) ts.last_variant = v.name;
        return rc;
    }

    DwGeom g{N, H, W, C, R, S, stride, pad, P, Q, 0, 1, 0, 0};
    g.cgroups = C / v.vec;
    if (v.R != 0) {
        // longest strip that still leaves about forty waves per CU (the strips' tails then
        // cost little); short strips re-read more halo rows, so stride 1 starts at four rows
        const long long want = (long long)cus * 40 * 64;
        const long long per_row = (long long)N * Q * g.cgroups;
        g.strip = stride >= 2 ? 2 : 4;
        for (int cand : {4, 8, 12, 16}) {
            const int use = cand < P ? cand : P;
            if (use > g.strip && per_row * ((P + use - 1) / use) >= want) g.strip = use;
        }
        if (ts.forced_dwconv_strip > 0) g.strip = ts.forced_dwconv_strip;
        if (g.strip > P) g.strip = P;
        g.strips = (P + g.strip - 1) / g.strip;
        g.items = (unsigned)(per_row * g.strips);
    } else {
        g.strip = 1;
        g.strips = P;
        g.items = (unsigned)((long long)N * P * Q * g.cgroups);
    }
    const unsigned blocks = (g.items + 255u) / 256u;
    const size_t lds = v.lds_filter ? (size_t)R * S * C * 4 : 0;
    v.kernel<<<dim3(blocks), dim3(256), lds, ts.stream>>>(g, in, w, out, ep);
    int rc = check_launch();
    if (rc == LSMI_OK) ts.last_variant = v.name;
    return rc;
}

}  // namespace lsmi
