// Direct 2-D convolution, NHWC input, KRSC filter, NPQK output, fp32, for gfx950.
//
// out[n,p,q,k] = sum_{r,s,c} in[n, p*stride-pad+r, q*stride-pad+s, c] * w[k,r,s,c]
// (Section 2.1: convolution as a contraction whose operand index is an affine function
// of the loop indices).  The kernel never materialises the unfolded input: a workgroup
// owns BM consecutive output pixels (n,p,q flattened) x BN output channels and walks the
// reduction index kk = (r*S + s)*C + c in BK chunks.  For each chunk every thread
// evaluates the affine map for its pixel rows, loads the c-contiguous run (or zeros
// where the tap falls in the padding) and stages it in LDS; the filter chunk, which is
// kk-contiguous per output channel, is staged the same way.  From there on the wave-level
// inner product is the one the GEMM uses.
#include "common.hpp"
#include "conv2d_dma.hpp"
#include "tile_f32.hpp"

namespace lsmi {
namespace {

struct ConvGeom {
    int N, H, W, C, K, R, S, stride, pad, P, Q;
    int pixels;  // N*P*Q
    int red;     // R*S*C
};

// CHUNK_IN_TAP: C % BK == 0 and 16-byte aligned tensors, so a BK chunk lies inside one
// filter tap (r, s): the reduction is walked tap by tap with scalar (r, s, c0) counters and
// the only per-lane work per chunk is one address add and one range test.  Otherwise each
// element's (r, s, c) is decoded from the flat reduction index.
template <class T, bool CHUNK_IN_TAP>
__global__ __launch_bounds__(T::NT) void conv2d_kernel(ConvGeom g, const float *__restrict__ in,
                                                       const float *__restrict__ w,
                                                       float *__restrict__ out, int tiles_m,
                                                       int tiles_n, Epilogue ep)
{
    __shared__ __attribute__((aligned(16))) float lds[T::LDS_FLOATS];
    float *const a_lds = lds;
    float *const b_lds = lds + 2 * T::A_STAGE;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, half = lane >> 5;
    const int wrow = (wave / T::WAVES_N) * T::WTM;
    const int wcol = (wave % T::WAVES_N) * T::WTN;

    // all channel tiles of one pixel tile are adjacent in the logical order, so the
    // input patch they share is fetched from HBM once
    int tn, tm;
    map_tile(blockIdx.x, tiles_n, tiles_m, tiles_n, tn, tm);
    const int m0 = tm * T::BM, n0 = tn * T::BN;

    // 16-byte loads need every c-run start to be aligned: base pointers and C % 4 == 0
    const bool in_vec = (((uintptr_t)in) & 15) == 0 && (g.C & 3) == 0;
    const bool w_vec = (((uintptr_t)w) & 15) == 0 && (g.red & 3) == 0;

    // Per-thread pixel rows are the same for every chunk: decode them once.
    int pix_base[T::A_SLOTS];  // offset of in[n, h0, w0, 4*kq] (may point before the image)
    int pix_h0[T::A_SLOTS];    // p*stride - pad, or a large negative value for rows past the end
    int pix_w0[T::A_SLOTS];
#pragma unroll
    for (int v = 0; v < T::A_SLOTS; ++v) {
        const int slot = tid + v * T::NT;
        const int m = m0 + slot / (T::BK / 4);
        if (m < g.pixels) {
            const int n = m / (g.P * g.Q), pq = m % (g.P * g.Q);
            pix_h0[v] = (pq / g.Q) * g.stride - g.pad;
            pix_w0[v] = (pq % g.Q) * g.stride - g.pad;
            pix_base[v] = n * g.H * g.W * g.C;
            if (CHUNK_IN_TAP)
                pix_base[v] += (pix_h0[v] * g.W + pix_w0[v]) * g.C + (slot % (T::BK / 4)) * 4;
        } else {
            pix_base[v] = 0;
            pix_h0[v] = INT32_MIN / 2;  // every tap fails the range test
            pix_w0[v] = 0;
        }
    }
    int w_off[T::B_SLOTS];  // offset of w[n0 + row, 0, 0, 4*kq], or -1 past the last channel
#pragma unroll
    for (int v = 0; v < T::B_SLOTS; ++v) {
        const int slot = tid + v * T::NT;
        const int row = slot / (T::BK / 4);
        w_off[v] = n0 + row < g.K ? (n0 + row) * g.red + (slot % (T::BK / 4)) * 4 : -1;
    }

    f32x4 ra[T::A_SLOTS], rb[T::B_SLOTS];
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};

    auto in_at = [&](int v, int kk) -> const float * {
        // address of the input element that reduction index kk multiplies, or nullptr
        // when it lies in the zero padding / past the reduction / past the last pixel
        if (kk >= g.red) return nullptr;
        const int rs = kk / g.C, c = kk % g.C;
        const int h = pix_h0[v] + rs / g.S, x = pix_w0[v] + rs % g.S;
        if ((unsigned)h >= (unsigned)g.H || (unsigned)x >= (unsigned)g.W) return nullptr;
        return in + pix_base[v] + (h * g.W + x) * g.C + c;
    };

    // Scalar walk over the reduction for the CHUNK_IN_TAP path.
    int tap_r = 0, tap_s = 0, tap_c = 0;
    auto gload_tap = [&](int k0) {
        const int tap_off = (tap_r * g.W + tap_s) * g.C + tap_c;
#pragma unroll
        for (int v = 0; v < T::A_SLOTS; ++v) {
            const bool ok = (unsigned)(pix_h0[v] + tap_r) < (unsigned)g.H &&
                            (unsigned)(pix_w0[v] + tap_s) < (unsigned)g.W;
            ra[v] = ok ? *reinterpret_cast<const f32x4 *>(in + pix_base[v] + tap_off) : zero4;
        }
#pragma unroll
        for (int v = 0; v < T::B_SLOTS; ++v)
            rb[v] = w_off[v] >= 0 ? *reinterpret_cast<const f32x4 *>(w + w_off[v] + k0) : zero4;
        tap_c += T::BK;
        if (tap_c == g.C) {
            tap_c = 0;
            if (++tap_s == g.S) {
                tap_s = 0;
                ++tap_r;
            }
        }
    };

    auto gload_flat = [&](int k0) {
#pragma unroll
        for (int v = 0; v < T::A_SLOTS; ++v) {
            const int slot = tid + v * T::NT;
            const int kk = k0 + (slot % (T::BK / 4)) * 4;
            if (in_vec) {
                // C % 4 == 0: the four elements share one tap and are contiguous
                const float *src = in_at(v, kk);
                ra[v] = src ? *reinterpret_cast<const f32x4 *>(src) : zero4;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float *src = in_at(v, kk + e);
                    ra[v][e] = src ? *src : 0.f;
                }
            }
        }
#pragma unroll
        for (int v = 0; v < T::B_SLOTS; ++v) {
            const int slot = tid + v * T::NT;
            const int kk = k0 + (slot % (T::BK / 4)) * 4;
            const float *src = w + w_off[v] + k0;
            if (w_vec) {
                rb[v] = (w_off[v] >= 0 && kk < g.red) ? *reinterpret_cast<const f32x4 *>(src) : zero4;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) rb[v][e] = (w_off[v] >= 0 && kk + e < g.red) ? src[e] : 0.f;
            }
        }
    };

    auto gload = [&](int k0) {
        if constexpr (CHUNK_IN_TAP) gload_tap(k0); else gload_flat(k0);
    };

    auto sstore = [&](int buf) {
        float *as = a_lds + buf * T::A_STAGE;
        float *bs = b_lds + buf * T::B_STAGE;
#pragma unroll
        for (int v = 0; v < T::A_SLOTS; ++v) {
            const int slot = tid + v * T::NT;
            *reinterpret_cast<f32x4 *>(as + (slot / (T::BK / 4)) * T::A_LD + (slot % (T::BK / 4)) * 4) = ra[v];
        }
#pragma unroll
        for (int v = 0; v < T::B_SLOTS; ++v) {
            const int slot = tid + v * T::NT;
            *reinterpret_cast<f32x4 *>(bs + (slot / (T::BK / 4)) * T::B_LD + (slot % (T::BK / 4)) * 4) = rb[v];
        }
    };

    WaveTile<T> wt;
    wt.clear();

    gload(0);
    sstore(0);
    __syncthreads();
    int buf = 0;
    for (int k0 = 0; k0 < g.red; k0 += T::BK) {
        const bool has_next = k0 + T::BK < g.red;
        if (has_next) gload(k0 + T::BK);
        wt.consume_chunk(a_lds + buf * T::A_STAGE, b_lds + buf * T::B_STAGE, wrow, wcol, li, half);
        if (has_next) sstore(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }

    // Epilogue: out = post(bias + acc).  Register v of block (a, b) is pixel m0 + wrow +
    // acc_row and channel n0 + wcol + 32*b + li: 32 lanes write 128 contiguous bytes.
    float init[T::TN];
#pragma unroll
    for (int b = 0; b < T::TN; ++b) {
        const int k = n0 + wcol + 32 * b + li;
        init[b] = (ep.pre == kPreBias && k < g.K) ? ep.bias[k] : 0.f;
    }
#pragma unroll
    for (int a = 0; a < T::TM; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = m0 + wrow + WaveTile<T>::acc_row(a, v, half);
#pragma unroll
            for (int b = 0; b < T::TN; ++b) {
                const int k = n0 + wcol + 32 * b + li;
                if (m < g.pixels && k < g.K) out[m * g.K + k] = apply_post(init[b] + wt.acc[a][b][v], ep.post);
            }
        }
}

// out[m, k] = bias[k] (or 0): the initial value that the slices of a split reduction add to.
__global__ __launch_bounds__(256) void conv_init_kernel(float *__restrict__ out, const float *__restrict__ bias,
                                                        int K, int64_t total)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < total) out[i] = bias ? bias[i % K] : 0.f;
}

// out = max(out, 0) in place: the post-operation after a split reduction.
__global__ __launch_bounds__(256) void conv_relu_kernel(float *__restrict__ out, int64_t total)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < total) out[i] = fmaxf(out[i], 0.f);
}

struct ConvVariant {
    const char *name;
    const char *split_name;
    const char *pieces_name;  // when the last tile rows were computed as quarter-tile pieces
    int bm, bn;
    // 0: register-staged kernel for any shape; 16/32: direct-to-LDS kernel, needs C % dma_bk == 0
    // (C % 4 == 0 when group_tap, any C when elem) and 16-byte aligned tensors (4-byte when elem)
    int dma_bk;
    // tail: tile rows at the end of the pixel range to compute as quarter-tile pieces;
    // returns 0 for the plain launch, 1 for a split reduction, 2 with pieces
    int (*launch)(hipStream_t s, bool chunk_in_tap, const ConvGeom &g, const float *in,
                  const float *w, float *out, Epilogue ep, int slices, int tail, int cus);
    bool group_tap = false;  // every lane follows the tap of its own four channels
    bool elem = false;       // ... of its own element: any channel count
};

template <class T>
int launch_conv_variant(hipStream_t s, bool chunk_in_tap, const ConvGeom &g, const float *in,
                        const float *w, float *out, Epilogue ep, int, int, int)
{
    const int tiles_m = (g.pixels + T::BM - 1) / T::BM, tiles_n = (g.K + T::BN - 1) / T::BN;
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(T::NT);
    if (chunk_in_tap)
        hipLaunchKernelGGL((conv2d_kernel<T, true>), grid, block, 0, s, g, in, w, out, tiles_m, tiles_n, ep);
    else
        hipLaunchKernelGGL((conv2d_kernel<T, false>), grid, block, 0, s, g, in, w, out, tiles_m, tiles_n, ep);
    return 0;
}

template <class T>
int launch_conv_dma_variant(hipStream_t s, bool, const ConvGeom &g, const float *in, const float *w,
                            float *out, Epilogue ep, int slices, int tail, int)
{
    const int tiles_m = (g.pixels + T::BM - 1) / T::BM, tiles_n = (g.K + T::BN - 1) / T::BN;
    auto geom = [&](int tile_rows) {
        return ConvDmaGeom(g.H, g.W, g.C, g.K, g.R, g.S, g.stride, g.pad, g.P, g.Q, g.pixels, tile_rows, tiles_n);
    };
    const int nk = T::GROUP_TAP ? (g.red + T::BK - 1) / T::BK : g.red / T::BK;
    const int per = (nk + slices - 1) / slices;
    const int used = (nk + per - 1) / per;  // no empty slice
    if (used <= 1) {
        int tail_rows = 0;  // the caller's plan (conv_plan) or the forced value
        if constexpr (T::NWAVES == 4 && T::LDS_BYTES >= 16384) {
            if (tail > 0 && g.C % 8 == 0) tail_rows = tail < tiles_m ? tail : tiles_m;
        }
        const int big_m = tiles_m - tail_rows, m_cut = big_m * T::BM;
        const int pieces_n = (g.K + 31) / 32;
        const int pieces = tail_rows > 0 ? ((g.pixels - m_cut + 31) / 32) * pieces_n : 0;
        hipLaunchKernelGGL(conv2d_dma_kernel<T>, dim3((unsigned)(pieces + big_m * tiles_n)), dim3(T::NT), 0, s,
                           geom(big_m), in, w, out, big_m, tiles_n, nk, pieces, pieces_n, m_cut, ep);
        return pieces > 0 ? 2 : 0;
    }
    // split reduction: initial value, partial sums added atomically, then the post-operation
    const int64_t total = (int64_t)g.pixels * g.K;
    const dim3 egrid((unsigned)((total + 255) / 256));
    hipLaunchKernelGGL(conv_init_kernel, egrid, dim3(256), 0, s, out, ep.pre == kPreBias ? ep.bias : nullptr,
                       g.K, total);
    hipLaunchKernelGGL(conv2d_dma_kernel<T>, dim3((unsigned)(tiles_m * tiles_n), (unsigned)used), dim3(T::NT), 0,
                       s, geom(tiles_m), in, w, out, tiles_m, tiles_n, per, 0, 1, 0, Epilogue{nullptr, kPreZero, kPostNone});
    if (ep.post == kPostRelu) hipLaunchKernelGGL(conv_relu_kernel, egrid, dim3(256), 0, s, out, total);
    return 1;
}

// The workgroups that stay (conv2d_stream_kernel): G per CU, each walking its share of the whole
// tiles; a split reduction goes to the one-tile-per-workgroup kernel of the same tile.
template <class T, int G>
int launch_conv_stream_variant(hipStream_t s, bool chunk_in_tap, const ConvGeom &g, const float *in, const float *w,
                               float *out, Epilogue ep, int slices, int tail, int cus)
{
    // (also when a tile's chunks do not fill whole turns of the ring: the kernel's stage indices
    // are compile-time constants that assume a tile starts at stage 0)
    if (slices > 1 || (g.red / T::BK) % T::NSTAGE != 0)
        return launch_conv_dma_variant<T>(s, chunk_in_tap, g, in, w, out, ep, slices, tail, cus);
    const int tiles_m = (g.pixels + T::BM - 1) / T::BM, tiles_n = (g.K + T::BN - 1) / T::BN;
    int tail_rows = 0;
    if (tail > 0 && g.C % 8 == 0) tail_rows = tail < tiles_m ? tail : tiles_m;
    const int big_m = tiles_m - tail_rows, m_cut = big_m * T::BM;
    const int pieces_n = (g.K + 31) / 32;
    const int pieces = tail_rows > 0 ? ((g.pixels - m_cut + 31) / 32) * pieces_n : 0;
    const int64_t tiles = (int64_t)big_m * tiles_n;
    const int64_t wgs = tiles < (int64_t)cus * G ? tiles : (int64_t)cus * G;
    if (pieces + wgs == 0) return 0;
    const ConvDmaGeom d(g.H, g.W, g.C, g.K, g.R, g.S, g.stride, g.pad, g.P, g.Q, g.pixels, big_m, tiles_n);
    hipLaunchKernelGGL(conv2d_stream_kernel<T>, dim3((unsigned)(pieces + wgs)), dim3(T::NT), 0, s, d, in, w, out,
                       big_m, tiles_n, pieces, pieces_n, m_cut, ep);
    return pieces > 0 ? 2 : 0;
}

#define LSMI_CONV_VARIANT(BM, BN, WM, WN)                                                    \
    {"conv2d_" #BM "x" #BN "x16_w" #WM "x" #WN, "", "", BM, BN, 0,                            \
     &launch_conv_variant<TileShape<BM, BN, 16, WM, WN, false>>}
#define LSMI_CONV_AHEAD_VARIANT(BM, BN, BK, WM, WN, NS)                                      \
    {"conv2d_dma_" #BM "x" #BN "x" #BK "_w" #WM "x" #WN "_s" #NS "_ahead",                    \
     "conv2d_dma_" #BM "x" #BN "x" #BK "_w" #WM "x" #WN "_s" #NS "_ahead_splitk",             \
     "conv2d_dma_" #BM "x" #BN "x" #BK "_w" #WM "x" #WN "_s" #NS "_ahead_pieces", BM, BN, BK, \
     &launch_conv_dma_variant<ConvDmaShape<BM, BN, BK, WM, WN, NS, true>>}
#define LSMI_CONV_DMA_VARIANT(BM, BN, BK, WM, WN, NS)                                        \
    {"conv2d_dma_" #BM "x" #BN "x" #BK "_w" #WM "x" #WN "_s" #NS,                             \
     "conv2d_dma_" #BM "x" #BN "x" #BK "_w" #WM "x" #WN "_s" #NS "_splitk",                    \
     "conv2d_dma_" #BM "x" #BN "x" #BK "_w" #WM "x" #WN "_s" #NS "_pieces", BM, BN, BK,        \
     &launch_conv_dma_variant<ConvDmaShape<BM, BN, BK, WM, WN, NS>>}

#define LSMI_CONV_STREAM_VARIANT(BM, BN, WM, WN, NS, G)                                      \
    {"conv2d_stream_" #BM "x" #BN "x16_w" #WM "x" #WN "_s" #NS "_g" #G,                       \
     "conv2d_dma_" #BM "x" #BN "x16_w" #WM "x" #WN "_s" #NS "_splitk",                        \
     "conv2d_stream_" #BM "x" #BN "x16_w" #WM "x" #WN "_s" #NS "_g" #G "_pieces", BM, BN, 16,  \
     &launch_conv_stream_variant<ConvDmaShape<BM, BN, 16, WM, WN, NS>, G>}

#define LSMI_CONV_GROUP_TAP_VARIANT(BM, BN, WM, WN, NS)                                      \
    {"conv2d_dma_c4_" #BM "x" #BN "x16_w" #WM "x" #WN "_s" #NS,                               \
     "conv2d_dma_c4_" #BM "x" #BN "x16_w" #WM "x" #WN "_s" #NS "_splitk",                      \
     "conv2d_dma_c4_" #BM "x" #BN "x16_w" #WM "x" #WN "_s" #NS "_pieces", BM, BN, 16,          \
     &launch_conv_dma_variant<ConvDmaShape<BM, BN, 16, WM, WN, NS, false, true>>, true}

#define LSMI_CONV_ELEM_VARIANT(BM, BN, WM, WN, NS)                                           \
    {"conv2d_dma_c1_" #BM "x" #BN "x16_w" #WM "x" #WN "_s" #NS,                               \
     "conv2d_dma_c1_" #BM "x" #BN "x16_w" #WM "x" #WN "_s" #NS "_splitk",                      \
     "conv2d_dma_c1_" #BM "x" #BN "x16_w" #WM "x" #WN "_s" #NS "_pieces", BM, BN, 16,          \
     &launch_conv_dma_variant<ConvDmaShape<BM, BN, 16, WM, WN, NS, false, true, true>>, true, true}

const ConvVariant kConvVariants[] = {
    LSMI_CONV_VARIANT(128, 64, 2, 2),              // 0: 64 x 32 wave tiles
    LSMI_CONV_VARIANT(64, 64, 2, 2),               // 1: 32 x 32 wave tiles
    LSMI_CONV_VARIANT(64, 32, 2, 1),               // 2: few pixels or few channels
    LSMI_CONV_VARIANT(128, 128, 2, 2),             // 3: 64 x 64 wave tiles, many channels
    LSMI_CONV_DMA_VARIANT(64, 64, 32, 2, 2, 2),    // 4: C % 32 == 0
    LSMI_CONV_DMA_VARIANT(128, 64, 32, 2, 2, 2),   // 5
    LSMI_CONV_DMA_VARIANT(64, 64, 16, 2, 2, 3),    // 6: C % 16 == 0
    LSMI_CONV_DMA_VARIANT(128, 64, 16, 2, 2, 3),   // 7
    LSMI_CONV_DMA_VARIANT(128, 128, 16, 2, 2, 3),  // 8
    LSMI_CONV_DMA_VARIANT(32, 64, 16, 1, 2, 3),    // 9: two waves; finer tiles waste less of the last round
    LSMI_CONV_DMA_VARIANT(32, 64, 16, 1, 2, 4),    // 10
    LSMI_CONV_DMA_VARIANT(64, 32, 16, 2, 1, 3),    // 11
    LSMI_CONV_AHEAD_VARIANT(64, 64, 16, 2, 2, 3),  // 12: fragments read a chunk ahead (no faster in sweeps)
    LSMI_CONV_DMA_VARIANT(256, 64, 16, 4, 1, 3),   // 13: four waves of 64 x 64 (no faster either)
    LSMI_CONV_GROUP_TAP_VARIANT(64, 64, 2, 2, 3),  // 14: C % 4 == 0
    LSMI_CONV_GROUP_TAP_VARIANT(128, 64, 2, 2, 3), // 15
    LSMI_CONV_GROUP_TAP_VARIANT(64, 32, 2, 1, 3),  // 16
    LSMI_CONV_STREAM_VARIANT(64, 64, 2, 2, 3, 3),  // 17: workgroups that stay, three per CU
    LSMI_CONV_STREAM_VARIANT(128, 64, 2, 2, 3, 2), // 18: 128 x 64 tiles, two per CU
    LSMI_CONV_STREAM_VARIANT(128, 64, 2, 2, 3, 3), // 19
    LSMI_CONV_ELEM_VARIANT(64, 64, 2, 2, 3),       // 20: any C (a stem of 3 channels), 4-byte loads
    LSMI_CONV_ELEM_VARIANT(128, 64, 2, 2, 3),      // 21
};
constexpr int kNumConvVariants = sizeof(kConvVariants) / sizeof(kConvVariants[0]);
constexpr int kConvDmaDefault = 6;  // conv2d_dma_64x64x16_w2x2_s3
constexpr int kConvDmaTall = 7;     // conv2d_dma_128x64x16_w2x2_s3
constexpr int kConvStreamTall = 18;  // conv2d_stream_128x64x16_w2x2_s3_g2
constexpr int kConvGroupTap = 14;   // conv2d_dma_c4_64x64x16_w2x2_s3
constexpr int kConvGroupTapTall = 15;
constexpr int kConvElem = 20, kConvElemTall = 21;
constexpr int kConvDmaNarrow = 11;       // conv2d_dma_64x32x16_w2x1_s3
constexpr int kConvGroupTapNarrow = 16;  // conv2d_dma_c4_64x32x16_w2x1_s3

}  // namespace

int conv_variant_count() { return kNumConvVariants; }

const char *conv_variant_name(int index)
{
    return index >= 0 && index < kNumConvVariants ? kConvVariants[index].name : nullptr;
}

namespace {

// Work of the busiest CU, in 64 x 64 tiles, for bm x 64 tiles of which `slots` fit a CU at a
// time; with_pieces: the tile rows of the last, partly filled round are cut into 32 x 32
// pieces (a quarter of a 64 x 64 tile each, at most one per CU) that are dispatched first.
// The constants are fitted to sweeps of the 56 x 56 and 64 x 64 workloads at 3 .. 13 tiles per
// CU: pieces cost a third of a tile when they fit beside the whole tiles of a single round,
// most of a tile when whole tiles already fill every slot (the tiles that start after the
// pieces then finish alone), half a tile otherwise.  Returns a negative value when the plan
// does not apply; *tail_rows receives the tile rows to hand to the pieces.
double conv_plan(int bm, int slots, int pixels, int K, int cus, bool with_pieces, int *tail_rows)
{
    const int tiles_m = (pixels + bm - 1) / bm, tiles_n = (K + 63) / 64;
    const int64_t tiles = (int64_t)tiles_m * tiles_n;
    const double unit = bm / 64.0;
    *tail_rows = 0;
    if (!with_pieces) return (double)((tiles + cus - 1) / cus) * unit;
    const int64_t rounds = tiles / cus, rem = tiles % cus;
    if (rounds < 1 || rem == 0) return -1.0;
    const int rows = (int)((rem + tiles_n - 1) / tiles_n);
    const int64_t big = (int64_t)(tiles_m - rows) * tiles_n;
    const int64_t pieces = (int64_t)((pixels - (tiles_m - rows) * bm + 31) / 32) * ((K + 31) / 32);
    if (pieces > cus || big > rounds * cus) return -1.0;
    const double penalty = rounds + 1 <= slots ? 0.35 : rounds == slots ? 0.9 : 0.5;
    *tail_rows = rows;
    return rounds * unit + 0.25 + penalty;
}

}  // namespace

int launch_conv2d(int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int P,
                  int Q, const float *in, const float *w, float *out, const float *bias, int post)
{
    const Epilogue ep{bias, bias ? kPreBias : kPreZero, post};
    ThreadState &st = tls();
    ConvGeom g{N, H, W, C, K, R, S, stride, pad, P, Q, N * P * Q, R * S * C};
    const int cus = device_cu_count();
    const bool aligned = (((uintptr_t)in | (uintptr_t)w) & 15) == 0;
    auto dma_ok = [&](const ConvVariant &v) {
        if (v.dma_bk == 0) return true;
        // the buffer descriptors of the direct-to-LDS kernels address less than 2^31 bytes
        return (v.elem || (aligned && C % (v.group_tap ? 4 : v.dma_bk) == 0)) &&
               (int64_t)N * H * W * C < (1 << 29) && (int64_t)K * g.red < (1 << 29);
    };
    int vi = st.forced_conv_variant;
    int planned_tail = 0;  // tile rows for the quarter-tile pieces, when the variant is chosen here
    if (vi >= 0 && !dma_ok(kConvVariants[vi])) vi = -1;  // forced kernel cannot take this shape
    const bool planned = vi < 0;
    if (vi < 0) {
        // Direct-to-LDS kernels where the shape allows them, and among those the 64 x 64 tile
        // with the 16-deep three-stage ring: in sweeps over batch 16 .. 256 and 64 .. 256 output
        // channels of the 56 x 56 x 64 workload it led every larger tile by 7 - 12 % (the larger
        // tiles' lower LDS traffic does not pay here, their coarser last round does cost).
        // Otherwise the register-staged tile whose workgroup count spreads best over the CUs:
        // cost = rounds of the busiest CU x work per tile, weighted by how often a small tile
        // re-reads its operands.
        // (channel counts that are multiples of 4 only: the per-lane-tap form of the same tiles)
        // (any other channel count, or tensors off a 16-byte boundary: the per-lane-element form)
        const bool by_elem = C % 4 != 0 || !aligned;
        const int wide = by_elem ? kConvElem : C % 16 == 0 ? kConvDmaDefault : kConvGroupTap;
        const int tall = by_elem ? kConvElemTall : C % 16 == 0 ? kConvDmaTall : kConvGroupTapTall;
        if (K > 32 && dma_ok(kConvVariants[wide])) {
            // 64 x 64 or 128 x 64 tiles, whole or with the last round as pieces: the plan with
            // the least work on the busiest CU (ties go to whole 64 x 64 tiles)
            vi = wide;
            double best = conv_plan(64, 6, g.pixels, K, cus, false, &planned_tail);
            const int cand_bm[3] = {64, 128, 128};
            const bool cand_pieces[3] = {true, false, true};
            for (int c = 0; c < 3; ++c) {
                if (cand_pieces[c] && st.forced_conv_tail >= 0) continue;  // the caller decides about pieces
                int rows = 0;
                const double cost = conv_plan(cand_bm[c], cand_bm[c] == 64 ? 6 : 4, g.pixels, K, cus,
                                              cand_pieces[c], &rows);
                if (cost >= 0 && cost < best - 1e-9 && C % 8 == 0) {
                    best = cost;
                    vi = cand_bm[c] == 64 ? wide : tall;
                    planned_tail = rows;
                }
            }
        }
        // The 128 x 64 tiles are taken when three or four of them make a CU's whole share; then two
        // workgroups per CU that stay and walk the tiles (the next tile's first chunks requested
        // under the current tile's last, its stores draining under the next tile's multiplies)
        // are ahead of one workgroup per tile: 32 x 56 x 56 x 64 -> 64 63.2 -> 60.8 us,
        // 32 x 28 x 28 x 128 -> 256 116.3 -> 113.0.  With six 64 x 64 workgroups per CU the two forms
        // are level, with fewer workgroups of that tile the loop itself is slower (67 -> 70 us).
        if (vi == kConvDmaTall && (g.red / 16) % 3 == 0) vi = kConvStreamTall;
        // Output channels that fill the last 64-wide tile column less than half (K <= 32, 96,
        // 160): 32-wide tiles compute a sixth to a half fewer columns.  Measured at batch 32:
        // 56x56x64 -> 96, 3x3: 119.5 -> 100.8 us; -> 32: 55.3 (register-staged) -> 40.4;
        // 28x28x128 -> 160: 92.0 -> 78.7; from 224 channels on (an eighth saved) the wide tiles win.
        const int cols32 = (K + 31) / 32 * 32, cols64 = (K + 63) / 64 * 64;
        // (a caller who asks for pieces keeps the 64-wide tiles that have them)
        // (with a reduction shorter than 256 only when a quarter is saved: 112x112x24 -> 144, 1x1,
        // a sixth saved, runs 81.7 us on the wide tiles and 88.1 on the narrow ones)
        // (and not with a long reduction, where a 32-wide tile's three operand bytes per two of a
        // 64-wide one decide: 64x28x28x512 -> 96, 5x5, stride 2, 12800 deep: 399 us narrow, 307 wide)
        if (cols32 * 100 <= cols64 * (g.red >= 256 ? 84 : 76) && (g.red <= 2048 || K <= 32) && st.forced_conv_tail <= 0) {
            const int narrow = C % 16 == 0 ? kConvDmaNarrow : kConvGroupTapNarrow;
            // (the per-lane-tap form on two waves when its tiles fill the CUs twice over, or up to 32
            // channels: 8x56x56x24 -> 80, 5x5, stride 2, 294 tiles: 26.4 us on 64 x 32 tiles, 17.9 on
            // 64 x 64; 16x56x56x24 -> 160, 980 tiles: 26.8 against 35.9)
            const int64_t narrow_tiles = (int64_t)((g.pixels + 63) / 64) * ((K + 31) / 32);
            if (dma_ok(kConvVariants[narrow]) && (narrow == kConvDmaNarrow || K <= 32 || narrow_tiles >= 2 * (int64_t)cus)) {
                vi = narrow;
                planned_tail = 0;
            }
        }
        // (the per-lane-element form also for few output channels: 16x112x112x3 -> 32, 3x3, stride 2:
        // 10.6 us on the register-staged 64 x 32 tile, 9.2 here)
        if (vi < 0 && by_elem && dma_ok(kConvVariants[kConvElem])) vi = kConvElem;
        if (vi < 0) {
            double best = 0;
            for (int i = 0; i < kNumConvVariants; ++i) {
                const ConvVariant &v = kConvVariants[i];
                if (v.dma_bk != 0) continue;
                if (v.bn > 32 && K <= 32) continue;
                if (v.bn > 64 && K <= 64) continue;
                const int64_t tiles = (int64_t)((g.pixels + v.bm - 1) / v.bm) * ((K + v.bn - 1) / v.bn);
                const double cost = (double)((tiles + cus - 1) / cus) * v.bm * v.bn *
                                    (1.0 + 16.0 / v.bm + 16.0 / v.bn);
                if (vi < 0 || cost < best) {
                    vi = i;
                    best = cost;
                }
            }
        }
        if (vi < 0) vi = 2;
    }
    const ConvVariant &v = kConvVariants[vi];
    const bool chunk_in_tap = C % 16 == 0 && aligned;
    // Few output tiles and a long reduction (the single-image CONV rows of Table 1, 14 x 14 and
    // 7 x 7 images at batch 32): split the reduction over gridDim.y, each slice at least 128
    // reduction elements long.  The number of slices minimises a cost fitted to sweeps of 8 to
    // 392 tiles: the CU with the most workgroups runs ceil(tiles * s / CUs) of them, each
    // ceil(chunks / s) chunks long at 0.256 us per 64 x 64 x 16 chunk; s > 1 slices cost two
    // more launches (2.5 us) and send s times the output through the atomic units (0.2 us per
    // MB).  What matters is how evenly tiles * s divides over the CUs: 392 tiles run 74 us
    // whole, 77 us in two slices and 65 us in three.  Only the direct-to-LDS kernels split.
    int slices = 1;
    if (v.dma_bk != 0) {
        const int64_t tiles = (int64_t)((g.pixels + v.bm - 1) / v.bm) * ((K + v.bn - 1) / v.bn);
        const int nk = v.group_tap ? (g.red + v.dma_bk - 1) / v.dma_bk : g.red / v.dma_bk;
        // (a caller who asks for pieces gets them: pieces and slices do not combine)
        if (tiles < 2 * cus && g.red >= 256 && st.forced_conv_tail <= 0) {
            const int longest = g.red / 128;
            const double unit = 0.256 * (v.bm * v.bn / 4096.0) * (v.dma_bk / 16.0);
            const double out_mb = 4.0 * g.pixels * K / 1e6;
            double best = 0;
            for (int s = 1; s <= longest; ++s) {
                const int per = (nk + s - 1) / s;
                const int64_t rounds = (tiles * s + cus - 1) / cus;
                // (a workgroup that has its CU to itself is bound by the latency of a chunk's loads,
                // whatever the tile: 32x7x7x48 -> 16, 3x3, 25 tiles of 64 x 32: 12.7 us whole, 7.5 cut)
                const double chunk = tiles * s <= cus && unit < 0.256 ? 0.256 : unit;
                const double cost = chunk * rounds * per + (s > 1 ? 2.5 + 0.2 * out_mb * s : 0.0);
                if (s == 1 || cost < best) {
                    best = cost;
                    slices = s;
                }
            }
        }
        if (st.forced_conv_slices > 0) slices = st.forced_conv_slices < nk ? st.forced_conv_slices : nk;
        if (slices < 1) slices = 1;
    }
    // pieces: forced by the caller, or the plan's; a forced tile configuration gets the plan of
    // its own tile height
    int tail = st.forced_conv_tail;
    if (tail < 0) {
        tail = planned ? planned_tail : 0;
        if (!planned && v.dma_bk != 0 && v.bn == 64 && (v.bm == 64 || v.bm == 128) && C % 8 == 0) {
            int rows = 0;
            const int slots = v.bm == 64 ? 6 : 4;
            const double with = conv_plan(v.bm, slots, g.pixels, K, cus, true, &rows);
            int none = 0;
            if (with >= 0 && with < conv_plan(v.bm, slots, g.pixels, K, cus, false, &none)) tail = rows;
        }
    }
    const int how = v.launch(st.stream, chunk_in_tap, g, in, w, out, ep, slices, tail, cus);
    int rc = check_launch();
    if (rc == LSMI_OK) st.last_variant = how == 1 ? v.split_name : how == 2 ? v.pieces_name : v.name;
    return rc;
}

}  // namespace lsmi
