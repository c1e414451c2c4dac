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

// offset of kernel element k along one axis: see tap_coord
__device__ __forceinline__ int tap_off(bool transposed, int k, int dil, int pad) {
    return transposed ? pad - k * dil : k * dil - pad;
}

// State of one chunk (TT taps x CWT channel words) on the fast path: the taps whose kernel row
// exists (okmask) are inside the image for every pixel of the run, so nothing is tested.
template <int AB, int WB, int CWT, int TT>
struct GenCtx {
    uint64_t base;                   // byte address of the activation planes
    uint32_t plane_bytes;            // Cw * 4
    uint32_t toff[TT];               // byte offset of tap i relative to the window origin (a tap that is
                                     // not used points at a used one: in bounds, skipped when consumed)
    uint32_t okmask;                 // bit i: tap i is used
    uint32_t w[TT][WB][CWT];
};

// CWT consecutive words at a wave-uniform byte address (4-byte aligned): one scalar load
template <int CWT>
__device__ __forceinline__ void load_words(uint64_t addr, uint32_t (&out)[CWT]) {
    typedef uint32_t vec_t __attribute__((ext_vector_type(CWT), aligned(4)));
    typedef const vec_t __attribute__((address_space(4))) *ptr_t;
    if constexpr (CWT == 1) {
        out[0] = *(uniform_words)addr;
    } else {
        const vec_t v = *(ptr_t)addr;
#pragma unroll
        for (int j = 0; j < CWT; ++j) out[j] = v[j];
    }
}

// Output pixels ra .. rb-1 (one output row, every used tap inside the image).  off_a: byte offset
// of the window origin of pixel ra (plane 0, word c0); step: bytes between the origins of
// neighbouring output pixels; kadd: constant term of this chunk.  All words of a pixel are
// requested before any is used; other wavefronts of the SIMD cover the latency.
template <int AB, int WB, int CWT, int TT, class OV>
__device__ __forceinline__ void gen_run_fast(const GenCtx<AB, WB, CWT, TT> &c, const OV &ov, int r0, int ra, int rb,
                                             uint32_t off_a, uint32_t step, int kadd, bool first, bool last) {
    uint32_t off = off_a;
    for (int r = ra; r < rb; ++r) {
        int prev = 0;
        if (!first)
            prev = __builtin_amdgcn_raw_buffer_load_b32(ov.d0, ov.col_bytes, (int)((uint32_t)(r - r0) * ov.row_bytes), 0);
        uint32_t a[TT][AB][CWT];
#pragma unroll
        for (int i = 0; i < TT; ++i)
#pragma unroll
            for (int p = 0; p < AB; ++p)
                load_words<CWT>(c.base + (uint32_t)(off + c.toff[i] + (uint32_t)p * c.plane_bytes), a[i][p]);
        int part[AB + WB - 1];
#pragma unroll
        for (int s = 0; s < AB + WB - 1; ++s) part[s] = 0;
#pragma unroll
        for (int i = 0; i < TT; ++i)
            if (c.okmask & (1u << i)) {
#pragma unroll
                for (int qq = 0; qq < WB; ++qq)
#pragma unroll
                    for (int p = 0; p < AB; ++p)
#pragma unroll
                        for (int j = 0; j < CWT; ++j) popc_acc(part[p + qq], a[i][p][j] ^ c.w[i][qq][j]);
            }
        int s = part[AB + WB - 2];
#pragma unroll
        for (int i = AB + WB - 3; i >= 0; --i) s = (s << 1) + part[i];
        finish_row<false>(ov, r - r0, prev + kadd - 2 * s, /*first=*/true, last);   // earlier part already added
        off += step;
    }
}

// One output pixel of one chunk with every tap tested (image borders, transposed convolution,
// chunks with padding words).
template <int AB, int WB, int CWT, int TT, class OV>
__device__ __forceinline__ void gen_pixel_checked(const BranchArgs &g, const OV &ov, uniform_words As,
                                                  const uint32_t (&w)[TT][WB][CWT], const int (&offh)[TT],
                                                  const int (&offw)[TT], int r0, int r, int img, int oh, int ow,
                                                  int c0, int t0, bool first, bool last) {
    const ConvGeom &q = g.geo;
    const int T = q.KH * q.KW, Cw = g.Cw;
    const bool transposed = q.transposed != 0;
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
}

__device__ __forceinline__ int floor_div(int a, int b) {       // b > 0
    const int qd = a / b;
    return (a % b != 0 && a < 0) ? qd - 1 : qd;
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
    const uint32_t pixel_bytes = (uint32_t)(AB * Cw) * 4u;

    GenCtx<AB, WB, CWT, TT> c;
    c.base = (uint64_t)g.A;
    c.plane_bytes = (uint32_t)Cw * 4u;
    for (int c0 = 0; c0 < Cw; c0 += CWT) {
        for (int t0 = 0; t0 < T; t0 += TT) {
            const bool first = (c0 == 0 && t0 == 0);
            const bool last = (c0 + CWT >= Cw && t0 + TT >= T);
            int offh[TT], offw[TT];         // offsets of the chunk's taps along both axes (see tap_coord)
            // output columns for which every tap of the chunk is inside the image: [lo, hi)
            int lo = 0, hi = q.Wo;
#pragma unroll
            for (int i = 0; i < TT; ++i) {
                const int t = t0 + i;
                const int kh = t / q.KW, kw = t - kh * q.KW;
                offh[i] = tap_off(transposed, kh, q.dh, q.ph);
                offw[i] = tap_off(transposed, kw, q.dw, q.pw);
                if (t < T) {
                    lo = max(lo, -floor_div(offw[i], q.sw));                  // ceil(-off / s)
                    hi = min(hi, floor_div(g.W - 1 - offw[i], q.sw) + 1);
                }
#pragma unroll
                for (int qq = 0; qq < WB; ++qq)
#pragma unroll
                    for (int j = 0; j < CWT; ++j)
                        c.w[i][qq][j] = (t < T && c0 + j < Cw) ? g.Wt[((nload * T + t) * WB + qq) * Cw + c0 + j] : 0u;
            }
            lo = __builtin_amdgcn_readfirstlane(lo);
            hi = __builtin_amdgcn_readfirstlane(hi);
            const bool fast_chunk = !transposed && (c0 + CWT <= Cw);
            int ow = ow0, oh = oh0, img = n0;
            int r = r0;
            while (r < r1) {
                const int row_end = min(r1, r - ow + q.Wo);                   // end of this output row within the range
                // fast interval of this row in pixel numbers
                int fa = r, fb = r;
                if (fast_chunk) {
                    // taps of the chunk whose kernel row exists for this output row; their offsets
                    uint32_t okmask = 0u, safe_off = 0u;
#pragma unroll
                    for (int i = 0; i < TT; ++i) {
                        const bool ok = (t0 + i < T) && (unsigned)(oh * q.sh + offh[i]) < (unsigned)g.H;
                        c.toff[i] = (uint32_t)(offh[i] * g.W + offw[i]) * pixel_bytes;
                        if (ok) {
                            if (okmask == 0u) safe_off = c.toff[i];
                            okmask |= 1u << i;
                        }
                    }
                    if (okmask != 0u) {
                        fa = max(r, r - ow + lo);
                        fb = min(row_end, r - ow + hi);
                        if (fb <= fa) { fa = r; fb = r; }
                        else {
                            c.okmask = okmask;
#pragma unroll
                            for (int i = 0; i < TT; ++i)
                                if (!(okmask & (1u << i))) c.toff[i] = safe_off;   // in bounds, skipped when consumed
                        }
                    }
                }
                // [r, fa) tested, [fa, fb) fast, [fb, row_end) tested
                for (int x = r; x < fa; ++x)
                    gen_pixel_checked<AB, WB, CWT, TT>(g, ov, As, c.w, offh, offw, r0, x, img, oh, ow + (x - r), c0, t0, first, last);
                if (fb > fa) {
                    const int owa = ow + (fa - r);
                    const uint32_t off_a = (uint32_t)((img * g.H + oh * q.sh) * g.W + owa * q.sw) * pixel_bytes + (uint32_t)c0 * 4u;
                    const int kadd = (c0 == 0) ? __builtin_popcount(c.okmask) * g.kconst : 0;
                    gen_run_fast<AB, WB, CWT, TT>(c, ov, r0, fa, fb, off_a, (uint32_t)q.sw * pixel_bytes, kadd, first, last);
                }
                for (int x = max(fb, fa); x < row_end; ++x)
                    gen_pixel_checked<AB, WB, CWT, TT>(g, ov, As, c.w, offh, offw, r0, x, img, oh, ow + (x - r), c0, t0, first, last);
                ow += row_end - r;
                r = row_end;
                if (ow == q.Wo) {
                    ow = 0;
                    if (++oh == q.Ho) { oh = 0; ++img; }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Few input channels (C <= 32) and a window of at most 256 bits (KH*KW*C): the K axis of an
// output pixel is materialised as a packed im2col row of KWP words per plane (bit t*C + c =
// tap t, channel c; see window_pack_kernel), so a 7x7x3 stem costs 5 words per plane instead
// of 49.  The row carries one more "plane": the mask of bits whose tap lies inside the image.
// Bits of taps outside are zero in the activation words, and the weights are and-ed with the
// mask, so such taps contribute nothing; the constant term counts the mask bits.
// ---------------------------------------------------------------------------------------
template <int AB, int WB, int KWP, bool EMIT>
__global__ __launch_bounds__(256) void conv_window_kernel(const BranchArgs g) {
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
    const int T = g.geo.KH * g.geo.KW, C = g.C;

    // the filter's window bits per weight plane, assembled from its per-tap words (C bits each)
    uint32_t w[WB][KWP];
#pragma unroll
    for (int qq = 0; qq < WB; ++qq)
#pragma unroll
        for (int k = 0; k < KWP; ++k) w[qq][k] = 0u;
    for (int t = 0; t < T; ++t) {
        const int bit = t * C, wi = bit >> 5, sh = bit & 31;
#pragma unroll
        for (int qq = 0; qq < WB; ++qq) {
            const uint32_t x = g.Wt[(nload * T + t) * WB + qq];
            const uint32_t lo = x << sh, hi = sh ? x >> (32 - sh) : 0u;      // hi: the part that spills into the next word
#pragma unroll
            for (int k = 0; k < KWP; ++k) {
                if (k == wi) w[qq][k] |= lo;
                if (k == wi + 1) w[qq][k] |= hi;
            }
        }
    }
    const uint64_t base = (uint64_t)g.A;
    constexpr uint32_t kRowBytes = (uint32_t)((AB + 1) * KWP) * 4u;
    for (int r = r0; r < r1; ++r) {
        const uint64_t row = base + (uint64_t)((uint32_t)r * kRowBytes);     // < 4 GiB, checked on the host
        uint32_t m[KWP], a[AB][KWP];
        load_words<KWP>(row + (uint32_t)(AB * KWP) * 4u, m);
#pragma unroll
        for (int p = 0; p < AB; ++p) load_words<KWP>(row + (uint32_t)(p * KWP) * 4u, a[p]);
        int nvalid = 0;
#pragma unroll
        for (int k = 0; k < KWP; ++k) nvalid += __builtin_popcount(m[k]);
        int part[AB + WB - 1];
#pragma unroll
        for (int s = 0; s < AB + WB - 1; ++s) part[s] = 0;
#pragma unroll
        for (int qq = 0; qq < WB; ++qq)
#pragma unroll
            for (int k = 0; k < KWP; ++k) {
                const uint32_t wm = w[qq][k] & m[k];
#pragma unroll
                for (int p = 0; p < AB; ++p) popc_acc(part[p + qq], a[p][k] ^ wm);
            }
        int s = part[AB + WB - 2];
#pragma unroll
        for (int i = AB + WB - 3; i >= 0; --i) s = (s << 1) + part[i];
        finish_row<true>(ov, r - r0, nvalid * g.kconst - 2 * s, true, true);   // kconst = (2^AB-1)(2^WB-1) per element
    }
}

template <int AB, int WB, int KWP>
void launch_window_shape(const BranchArgs &g, dim3 grid, hipStream_t s) {
    if (g.planes_out != nullptr) hipLaunchKernelGGL((conv_window_kernel<AB, WB, KWP, true>), grid, dim3(256), 0, s, g);
    else hipLaunchKernelGGL((conv_window_kernel<AB, WB, KWP, false>), grid, dim3(256), 0, s, g);
}

template <int AB, int WB>
hipError_t launch_window_t(const BranchArgs &g, hipStream_t s) {
    const int64_t row_blocks = ((int64_t)g.rows + g.rows_per_wave - 1) / g.rows_per_wave;
    const dim3 grid((unsigned)((row_blocks * g.col_tiles + 3) / 4));
    switch (g.Cw) {                                    // words per plane of the packed window
        case 1: launch_window_shape<AB, WB, 1>(g, grid, s); break;
        case 2: launch_window_shape<AB, WB, 2>(g, grid, s); break;
        case 3: launch_window_shape<AB, WB, 3>(g, grid, s); break;
        case 5: launch_window_shape<AB, WB, 5>(g, grid, s); break;
        case 8: launch_window_shape<AB, WB, 8>(g, grid, s); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

constexpr int imin3(int a, int b, int c) { return a < b ? (a < c ? a : c) : (b < c ? b : c); }

template <int AB, int WB, int CWT>
void launch_general_shape(const BranchArgs &g, dim3 grid, bool emit, hipStream_t s) {
    constexpr int TT = imin3(6, 64 / (WB * CWT), 24 / (AB * CWT));
    if (emit) hipLaunchKernelGGL((conv_general_kernel<AB, WB, CWT, TT, true>), grid, dim3(256), 0, s, g);
    else hipLaunchKernelGGL((conv_general_kernel<AB, WB, CWT, TT, false>), grid, dim3(256), 0, s, g);
}

template <int AB, int WB>
hipError_t launch_general_t(const BranchArgs &g, hipStream_t s) {
    const int64_t row_blocks = ((int64_t)g.rows + g.rows_per_wave - 1) / g.rows_per_wave;
    const dim3 grid((unsigned)((row_blocks * g.col_tiles + 3) / 4));
    const bool emit = g.planes_out != nullptr;
    // channel words per chunk (at most AB*CWT = 8 and no more than there are), then taps per chunk
    // such that the chunk's weight words (TT*WB*CWT) stay at or below 64 VGPRs and one pixel's
    // activation words (TT*AB*CWT) at or below 24 SGPRs
    constexpr int CMAX = (AB <= 2) ? 4 : (AB <= 4) ? 2 : 1;
    if (g.Cw >= 4 && CMAX >= 4) launch_general_shape<AB, WB, (CMAX >= 4 ? 4 : 1)>(g, grid, emit, s);
    else if (g.Cw >= 2 && CMAX >= 2) launch_general_shape<AB, WB, (CMAX >= 2 ? 2 : 1)>(g, grid, emit, s);
    else launch_general_shape<AB, WB, 1>(g, grid, emit, s);
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

hipError_t QNN_CAT(launch_conv_window_ab, QNN_AB)(const BranchArgs &g, int wb, hipStream_t s) {
    switch (wb) {
        case 1: return launch_window_t<QNN_AB, 1>(g, s);
        case 2: return launch_window_t<QNN_AB, 2>(g, s);
        case 3: return launch_window_t<QNN_AB, 3>(g, s);
        case 4: return launch_window_t<QNN_AB, 4>(g, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace qnn
