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
#include "tile_f32.hpp"

namespace lsmi {
namespace {

struct ConvGeom {
    int N, H, W, C, K, R, S, stride, pad, P, Q;
    int pixels;  // N*P*Q
    int red;     // R*S*C
};

template <class T>
__global__ __launch_bounds__(T::NT) void conv2d_kernel(ConvGeom g, const float *__restrict__ in,
                                                       const float *__restrict__ w,
                                                       float *__restrict__ out, int tiles_m,
                                                       int tiles_n)
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
    int pix_base[T::A_SLOTS];  // offset of in[n, 0, 0, 0]
    int pix_h0[T::A_SLOTS];    // p*stride - pad, or a large negative value for rows past the end
    int pix_w0[T::A_SLOTS];
#pragma unroll
    for (int v = 0; v < T::A_SLOTS; ++v) {
        const int slot = tid + v * T::NT;
        const int m = m0 + slot / (T::BK / 4);
        if (m < g.pixels) {
            const int n = m / (g.P * g.Q), pq = m % (g.P * g.Q);
            pix_base[v] = n * g.H * g.W * g.C;
            pix_h0[v] = (pq / g.Q) * g.stride - g.pad;
            pix_w0[v] = (pq % g.Q) * g.stride - g.pad;
        } else {
            pix_base[v] = 0;
            pix_h0[v] = INT32_MIN / 2;  // every tap fails the range test
            pix_w0[v] = 0;
        }
    }

    f32x4 ra[T::A_SLOTS], rb[T::B_SLOTS];

    auto in_at = [&](int v, int kk) -> const float * {
        // address of the input element that reduction index kk multiplies, or nullptr
        // when it lies in the zero padding / past the reduction / past the last pixel
        if (kk >= g.red) return nullptr;
        const int rs = kk / g.C, c = kk % g.C;
        const int h = pix_h0[v] + rs / g.S, x = pix_w0[v] + rs % g.S;
        if ((unsigned)h >= (unsigned)g.H || (unsigned)x >= (unsigned)g.W) return nullptr;
        return in + pix_base[v] + (h * g.W + x) * g.C + c;
    };

    auto gload = [&](int k0) {
#pragma unroll
        for (int v = 0; v < T::A_SLOTS; ++v) {
            const int slot = tid + v * T::NT;
            const int kk = k0 + (slot % (T::BK / 4)) * 4;
            if (in_vec) {
                // C % 4 == 0: the four elements share one tap and are contiguous
                const float *src = in_at(v, kk);
                ra[v] = src ? *reinterpret_cast<const f32x4 *>(src) : f32x4{0.f, 0.f, 0.f, 0.f};
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
            const int row = slot / (T::BK / 4), kk = k0 + (slot % (T::BK / 4)) * 4;
            const bool row_ok = n0 + row < g.K;
            const float *src = w + (n0 + row) * g.red + kk;
            if (w_vec) {
                rb[v] = (row_ok && kk < g.red) ? *reinterpret_cast<const f32x4 *>(src)
                                                : f32x4{0.f, 0.f, 0.f, 0.f};
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) rb[v][e] = (row_ok && kk + e < g.red) ? src[e] : 0.f;
            }
        }
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

    // Epilogue: out = acc.  Register v of block (a, b) is pixel m0 + wrow + acc_row and
    // channel n0 + wcol + 32*b + li: 32 lanes write 128 contiguous bytes.
#pragma unroll
    for (int a = 0; a < T::TM; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = m0 + wrow + WaveTile<T>::acc_row(a, v, half);
#pragma unroll
            for (int b = 0; b < T::TN; ++b) {
                const int k = n0 + wcol + 32 * b + li;
                if (m < g.pixels && k < g.K) out[m * g.K + k] = wt.acc[a][b][v];
            }
        }
}

typedef TileShape<128, 64, 16, 2, 2, false> ConvWide;   // 64 x 32 wave tiles
typedef TileShape<64, 32, 16, 2, 1, false> ConvSmall;   // few pixels or few channels

}  // namespace

int launch_conv2d(int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int P,
                  int Q, const float *in, const float *w, float *out)
{
    ThreadState &st = tls();
    ConvGeom g{N, H, W, C, K, R, S, stride, pad, P, Q, N * P * Q, R * S * C};
    const int cus = device_cu_count();
    const int64_t wide_tiles = (int64_t)((g.pixels + 127) / 128) * ((K + 63) / 64);
    if (wide_tiles >= cus || K > 32) {
        const int tiles_m = (g.pixels + 127) / 128, tiles_n = (K + 63) / 64;
        hipLaunchKernelGGL(conv2d_kernel<ConvWide>, dim3((unsigned)(tiles_m * tiles_n)),
                           dim3(ConvWide::NT), 0, st.stream, g, in, w, out, tiles_m, tiles_n);
        st.last_variant = "conv2d_128x64x16";
    } else {
        const int tiles_m = (g.pixels + 63) / 64, tiles_n = (K + 31) / 32;
        hipLaunchKernelGGL(conv2d_kernel<ConvSmall>, dim3((unsigned)(tiles_m * tiles_n)),
                           dim3(ConvSmall::NT), 0, st.stream, g, in, w, out, tiles_m, tiles_n);
        st.last_variant = "conv2d_64x32x16";
    }
    return check_launch();
}

}  // namespace lsmi
