// Convolution of any geometry as a multi-branch binary product (paper Eq. (8) with the layer's
// "Op" of Sec. 3.2 a strided, dilated, KH x KW or transposed convolution, as the networks of
// Sec. 5 need them: 7x7 stride-2 stems, strided 3x3 and 1x1 convolutions, atrous convolutions,
// deconvolutions).  Compiled once per activation bit width, -DQNN_AB=<1..8>.
//
// Same mapping as the 3x3 kernels (lane = filter, a wavefront owns 64 filters and a run of
// output pixels, weight words of the current chunk in VGPRs, the pixel's activation words
// wave-uniform through scalar loads), but everything about the window is a run-time value:
// a chunk is TT taps x CWT channel words, every tap of every pixel is tested against the image,
// taps outside contribute nothing and the constant term counts the taps that are inside.
// Partial sums of the chunks round-trip through the output buffer (same lane, same address).
// This is the general path: the 3x3 / stride 1 / pad 1 case has its own, faster kernels.
#include <type_traits>
#include "qnn_internal.h"
#include "qnn_device_util.h"

#ifndef QNN_AB
#error "compile with -DQNN_AB=<activation bits>"
#endif

namespace qnn {
namespace {

// Input coordinate of one tap along one axis.  Forward: i = o*stride + off (off = k*dil - pad).
// Transposed: o = i*stride - pad + k*dil, so i = (o + off) / stride with off = pad - k*dil, if
// that division is exact.  Returns false if the tap does not touch the image.
__device__ __forceinline__ bool tap_coord(bool transposed, int o, int stride, int off, int size, int &i) {
    if (!transposed) {
        i = o * stride + off;
    } else {
        const int num = o + off;
        if (num < 0) return false;
        i = num / stride;
        if (i * stride != num) return false;
    }
    return (unsigned)i < (unsigned)size;
}

template <int AB, int WB, int CWT, int TT, bool EMIT>
__global__ __launch_bounds__(256) void conv_general_kernel(const BranchArgs g) {
    typedef typename std::conditional<EMIT, OutViewEmit, OutView>::type OV;
    const int wave = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
    const int ct = wave % g.col_tiles;
    const int rb = wave / g.col_tiles;
    if ((int64_t)rb * g.rows_per_wave >= g.rows) return;
    const int r0 = rb * g.rows_per_wave;
    const int r1 = min(g.rows, r0 + g.rows_per_wave);
    const int lane = (int)(threadIdx.x & 63);
    const int n = ct * 64 + lane;
    const int nload = (n < g.N) ? n : g.N - 1;         // lanes past N redo column N-1 (same value, same address)
    const float sc = (g.scale != nullptr) ? g.scale[nload] : 1.0f;
    const OV ov = make_out_view<OV>(g, r0, r1, nload, sc, ct);
    uniform_words As = as_uniform(g.A);
    const ConvGeom &q = g.geo;
    const int T = q.KH * q.KW, Cw = g.Cw;
    const bool transposed = q.transposed != 0;
    if (Cw == 0 || T == 0) {                            // empty sum
        for (int r = r0; r < r1; ++r) finish_row<true>(ov, r - r0, 0, true, true);
        return;
    }
    // position of the first output pixel (integer division runs on the vector ALU)
    const int ow0 = __builtin_amdgcn_readfirstlane(r0 % q.Wo);
    const int oh0 = __builtin_amdgcn_readfirstlane((r0 / q.Wo) % q.Ho);
    const int n0 = __builtin_amdgcn_readfirstlane(r0 / (q.Wo * q.Ho));

    for (int c0 = 0; c0 < Cw; c0 += CWT) {
        for (int t0 = 0; t0 < T; t0 += TT) {
            const bool first = (c0 == 0 && t0 == 0);
            const bool last = (c0 + CWT >= Cw && t0 + TT >= T);
            uint32_t w[TT][WB][CWT];
            int offh[TT], offw[TT];
#pragma unroll
            for (int i = 0; i < TT; ++i) {
                const int t = t0 + i;
                const int kh = t / q.KW, kw = t - kh * q.KW;
                offh[i] = transposed ? q.ph - kh * q.dh : kh * q.dh - q.ph;
                offw[i] = transposed ? q.pw - kw * q.dw : kw * q.dw - q.pw;
#pragma unroll
                for (int qq = 0; qq < WB; ++qq)
#pragma unroll
                    for (int j = 0; j < CWT; ++j)
                        w[i][qq][j] = (t < T && c0 + j < Cw) ? g.Wt[((nload * T + t) * WB + qq) * Cw + c0 + j] : 0u;
            }
            int ow = ow0, oh = oh0, img = n0;
            for (int r = r0; r < r1; ++r) {
                int prev = 0;
                if (!first)
                    prev = __builtin_amdgcn_raw_buffer_load_b32(ov.d0, ov.col_bytes, (int)((uint32_t)(r - r0) * ov.row_bytes), 0);
                int part[AB + WB - 1];
#pragma unroll
                for (int s = 0; s < AB + WB - 1; ++s) part[s] = 0;
                int nvalid = 0;
#pragma unroll
                for (int i = 0; i < TT; ++i) {
                    int ih, iw;
                    const bool ok = (t0 + i < T) && tap_coord(transposed, oh, q.sh, offh[i], g.H, ih) &&
                                    tap_coord(transposed, ow, q.sw, offw[i], g.W, iw);
                    if (ok) {                           // uniform
                        const int pix = (img * g.H + ih) * g.W + iw;
                        uint32_t a[AB][CWT];
#pragma unroll
                        for (int p = 0; p < AB; ++p)
#pragma unroll
                            for (int j = 0; j < CWT; ++j)
                                a[p][j] = (CWT == 1 || c0 + j < Cw) ? As[(pix * AB + p) * Cw + c0 + j] : 0u;
#pragma unroll
                        for (int qq = 0; qq < WB; ++qq)
#pragma unroll
                            for (int p = 0; p < AB; ++p)
#pragma unroll
                                for (int j = 0; j < CWT; ++j) popc_acc(part[p + qq], a[p][j] ^ w[i][qq][j]);
                        ++nvalid;
                    }
                }
                int s = part[AB + WB - 2];
#pragma unroll
                for (int i = AB + WB - 3; i >= 0; --i) s = (s << 1) + part[i];
                int val = prev - 2 * s;
                if (c0 == 0) val += nvalid * g.kconst;  // kconst = C * (2^AB-1) * (2^WB-1), once per tap
                finish_row<false>(ov, r - r0, val, /*first=*/true, last);   // the earlier part is already added
                if (++ow == q.Wo) {
                    ow = 0;
                    if (++oh == q.Ho) { oh = 0; ++img; }
                }
            }
        }
    }
}

template <int AB, int WB>
hipError_t launch_general_t(const BranchArgs &g, hipStream_t s) {
    // taps per chunk so that TT * WB * CWT weight words stay at or below 64
    constexpr int TT = (WB <= 2) ? 8 : (WB <= 4) ? 4 : 2;
    const int64_t row_blocks = ((int64_t)g.rows + g.rows_per_wave - 1) / g.rows_per_wave;
    const dim3 grid((unsigned)((row_blocks * g.col_tiles + 3) / 4));
    const bool emit = g.planes_out != nullptr;
    if (g.Cw <= 1 || AB > 4) {
        if (emit) hipLaunchKernelGGL((conv_general_kernel<AB, WB, 1, TT, true>), grid, dim3(256), 0, s, g);
        else hipLaunchKernelGGL((conv_general_kernel<AB, WB, 1, TT, false>), grid, dim3(256), 0, s, g);
    } else if constexpr (AB <= 4) {
        constexpr int CWT = (AB <= 2) ? 4 : 2;
        constexpr int TT4 = (TT * CWT > 16) ? 16 / CWT : TT;
        if (emit) hipLaunchKernelGGL((conv_general_kernel<AB, WB, CWT, TT4, true>), grid, dim3(256), 0, s, g);
        else hipLaunchKernelGGL((conv_general_kernel<AB, WB, CWT, TT4, false>), grid, dim3(256), 0, s, g);
    }
    return hipGetLastError();
}

}  // namespace

#define QNN_CAT2(a, b) a##b
#define QNN_CAT(a, b) QNN_CAT2(a, b)

hipError_t QNN_CAT(launch_conv_general_ab, QNN_AB)(const BranchArgs &g, int wb, hipStream_t s) {
    switch (wb) {
        case 1: return launch_general_t<QNN_AB, 1>(g, s);
        case 2: return launch_general_t<QNN_AB, 2>(g, s);
        case 3: return launch_general_t<QNN_AB, 3>(g, s);
        case 4: return launch_general_t<QNN_AB, 4>(g, s);
        case 5: return launch_general_t<QNN_AB, 5>(g, s);
        case 6: return launch_general_t<QNN_AB, 6>(g, s);
        case 7: return launch_general_t<QNN_AB, 7>(g, s);
        case 8: return launch_general_t<QNN_AB, 8>(g, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace qnn
