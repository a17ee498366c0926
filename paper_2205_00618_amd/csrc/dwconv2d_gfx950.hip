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
#include "common.hpp"
#include "tile_f32.hpp"

namespace lsmi {
namespace {

struct DwGeom {
    int N, H, W, C, R, S, stride, pad, P, Q;
    int cgroups;      // C / channels per lane
    int strip;        // output rows per lane
    int strips;       // ceil(P / strip)
    long long items;  // lanes with work: N * strips * Q * cgroups
};

__device__ inline f32x4 zero4() { return f32x4{0.f, 0.f, 0.f, 0.f}; }

// Workgroup ids are dealt round-robin to the XCDs; regroup them so that each XCD works on
// one contiguous range of the item space (neighbouring strips share halo rows in its L2).
__device__ inline long long regrouped_block(long long blocks)
{
    const long long b = blockIdx.x;
    const long long q = blocks / kXcds, rem = blocks % kXcds;
    const long long xcd = b % kXcds, idx = b / kXcds;
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

// VEC channels per lane (4, or 2 where the window of a larger filter would not leave
// enough registers for several waves per SIMD).  FILTER_IN_LDS: the taps are read from a
// copy of the filter in LDS instead of being held in registers.
template <int R, int S, int STRIDE, int VEC, bool FILTER_IN_LDS>
__global__ __launch_bounds__(256) void dwconv_window_kernel(DwGeom g, const float *__restrict__ in,
                                                             const float *__restrict__ w,
                                                             float *__restrict__ out, Epilogue ep)
{
    typedef typename FVec<VEC>::type vec;
    constexpr int NEW = STRIDE < R ? STRIDE : R;  // rows entering the window per step
    extern __shared__ float w_lds[];              // [R*S][C] when FILTER_IN_LDS
    if constexpr (FILTER_IN_LDS) {
        for (int t = threadIdx.x; t < R * S * g.cgroups; t += 256)
            *reinterpret_cast<vec *>(w_lds + VEC * t) = *reinterpret_cast<const vec *>(w + VEC * (long long)t);
        __syncthreads();
    }
    const long long blocks = (g.items + 255) / 256;
    const long long item = regrouped_block(blocks) * 256 + threadIdx.x;
    if (item >= g.items) return;
    const int cg = (int)(item % g.cgroups);
    long long rest = item / g.cgroups;
    const int q = (int)(rest % g.Q);
    rest /= g.Q;
    const int sb = (int)(rest % g.strips);
    const int n = (int)(rest / g.strips);
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

    auto load_row = [&](int h, vec(&dst)[S]) {
        const bool row_ok = (unsigned)h < (unsigned)g.H;
        const float *row = img + (long long)(row_ok ? h : 0) * g.W * g.C;
#pragma unroll
        for (int s = 0; s < S; ++s) {
            vec v = *reinterpret_cast<const vec *>(row + col_off[s]);
            dst[s] = (row_ok && col_ok[s]) ? v : zero_vec<VEC>();
        }
    };

    vec win[R][S];  // window row j (relative input row) lives in slot j % R
#pragma unroll
    for (int r = 0; r < R; ++r) load_row(h0 + r, win[r]);

    float *dst = out + (((long long)n * g.P + p0) * g.Q + q) * g.C + c;
    const long long out_row = (long long)g.Q * g.C;

    for (int i0 = 0; i0 < rows; i0 += R) {
        static_for<R>([&](auto phase_c) {
            constexpr int phase = decltype(phase_c)::value;
            const int i = i0 + phase;
            if (i < rows) {
                // rows that enter the window at step i+1: relative rows (i+1)*STRIDE + R-NEW .. + R-1
                vec nxt[NEW][S];
                const bool more = i + 1 < rows;
                if (more) {
#pragma unroll
                    for (int a = 0; a < NEW; ++a) load_row(h0 + (i + 1) * STRIDE + R - NEW + a, nxt[a]);
                }
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
                if (more) {
#pragma unroll
                    for (int a = 0; a < NEW; ++a) {
                        const int slot = ((phase + 1) * STRIDE + R - NEW + a) % R;
#pragma unroll
                        for (int s = 0; s < S; ++s) win[slot][s] = nxt[a][s];
                    }
                }
            }
        });
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
    const long long blocks = (g.items + 255) / 256;
    const long long item = regrouped_block(blocks) * 256 + threadIdx.x;
    if (item >= g.items) return;
    const int cg = (int)(item % g.cgroups);
    long long rest = item / g.cgroups;
    const int q = (int)(rest % g.Q);
    rest /= g.Q;
    const int p = (int)(rest % g.P);
    const int n = (int)(rest / g.P);
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

typedef void (*DwKernel)(DwGeom, const float *, const float *, float *, Epilogue);

struct DwVariant {
    const char *name;
    int R, S, stride;  // 0 = any
    int vec;           // channels per lane
    bool lds_filter;
    DwKernel kernel;
};

const DwVariant kDwVariants[] = {
    {"dwconv_window_3x3_s1_v4", 3, 3, 1, 4, false, dwconv_window_kernel<3, 3, 1, 4, false>},
    {"dwconv_window_3x3_s2_v4", 3, 3, 2, 4, false, dwconv_window_kernel<3, 3, 2, 4, false>},
    {"dwconv_window_5x5_s1_v2", 5, 5, 1, 2, true, dwconv_window_kernel<5, 5, 1, 2, true>},
    {"dwconv_window_5x5_s2_v2", 5, 5, 2, 2, true, dwconv_window_kernel<5, 5, 2, 2, true>},
    {"dwconv_direct_vec4", 0, 0, 0, 4, false, dwconv_direct_kernel<4>},
    {"dwconv_direct_scalar", 0, 0, 0, 1, false, dwconv_direct_kernel<1>},
};
constexpr int kDwDirectVec = 4, kDwDirectScalar = 5;
constexpr int kDwVariantCount = sizeof(kDwVariants) / sizeof(kDwVariants[0]);

}  // namespace

int dwconv_variant_count() { return kDwVariantCount; }

int launch_dwconv2d(int N, int H, int W, int C, int R, int S, int stride, int pad, int P, int Q,
                    const float *in, const float *w, float *out, const float *bias, int post)
{
    ThreadState &ts = tls();
    auto fits = [&](int i) {
        const DwVariant &v = kDwVariants[i];
        const uintptr_t mask = 4 * v.vec - 1;
        auto aligned = [&](const void *p) { return (reinterpret_cast<uintptr_t>(p) & mask) == 0; };
        if (C % v.vec != 0 || !aligned(in) || !aligned(w) || !aligned(out) || !aligned(bias)) return false;
        if (v.R == 0) return true;
        if (H == 0 || W == 0) return false;  // the window kernels read clamped addresses
        // the LDS copy of the filter stays within the 64 KiB a kernel gets without opting in
        return v.R == R && v.S == S && v.stride == stride && (!v.lds_filter || (size_t)R * S * C * 4 <= 64 * 1024);
    };
    int vi = kDwDirectScalar;
    for (int i = kDwDirectVec; i >= 0; --i)
        if (fits(i)) vi = i;
    if (ts.forced_dwconv_variant >= 0 && fits(ts.forced_dwconv_variant)) vi = ts.forced_dwconv_variant;
    const DwVariant &v = kDwVariants[vi];

    DwGeom g{N, H, W, C, R, S, stride, pad, P, Q, 0, 1, 0, 0};
    g.cgroups = C / v.vec;
    if (v.R != 0) {
        // longest strip that still leaves about sixteen waves per SIMD-quad of every CU
        const long long want = (long long)device_cu_count() * 16 * 64;
        const long long per_row = (long long)N * Q * g.cgroups;
        g.strip = 4;
        for (int cand : {8, 16, 32}) {
            const int use = cand < P ? cand : P;
            if (per_row * ((P + use - 1) / use) >= want) g.strip = use;
        }
        if (ts.forced_dwconv_strip > 0) g.strip = ts.forced_dwconv_strip;
        if (g.strip > P) g.strip = P;
        g.strips = (P + g.strip - 1) / g.strip;
        g.items = per_row * g.strips;
    } else {
        g.strip = 1;
        g.strips = P;
        g.items = (long long)N * P * Q * g.cgroups;
    }
    const long long blocks = (g.items + 255) / 256;
    if (blocks > INT32_MAX) return LSMI_ERR_TOO_LARGE;
    const size_t lds = v.lds_filter ? (size_t)R * S * C * 4 : 0;
    Epilogue ep{bias, bias ? kPreBias : kPreZero, post};
    v.kernel<<<dim3((unsigned)blocks), dim3(256), lds, ts.stream>>>(g, in, w, out, ep);
    int rc = check_launch();
    if (rc == LSMI_OK) ts.last_variant = v.name;
    return rc;
}

}  // namespace lsmi
