// Convolution of any geometry as a multi-branch binary product (paper Eq. (8) with the layer's
// "Op" of Sec. 3.2 a strided, dilated, KH x KW or transposed convolution, as the networks of
// Sec. 5 need them: 7x7 stride-2 stems, strided 3x3 and 1x1 convolutions, atrous convolutions,
// deconvolutions).  Compiled once per activation bit width, -DQNN_AB=<1..8>.
//
// Same mapping as the 3x3 kernels (lane = filter, a wavefront owns 64 filters and a run of
// output pixels, weight words of the current chunk in VGPRs, the pixel's activation words
// wave-uniform through scalar loads), but everything about the window is a run-time value.
// A chunk is TT taps x CWT channel words.  Per output row the pixels for which every tap of the
// chunk lies inside the image run without any test (gen_run_fast); the others (borders, chunks
// with padding words) test every tap, taps outside contribute nothing and the constant term
// counts the taps that are inside (gen_pixel_checked).  Partial sums of the chunks round-trip
// through the output buffer (same lane, same address).  The transposed form walks the output
// by phase (transposed_phases).  Few input channels take the packed-window kernel at the end of
// the file.  This is the general path: the 3x3 / stride 1 / pad 1 case has its own, faster
// kernels, and single-tap convolutions without padding run on the GEMM kernels.
#include <type_traits>
#include "qnn_internal.h"
#include "qnn_device_util.h"

#ifndef QNN_AB
#error "compile with -DQNN_AB=<activation bits>"
#endif

namespace qnn {
namespace {

// Transposed convolution, one axis.  Output o gets a contribution of kernel element k from the
// input i with o = i*stride - pad + k*dil, i.e. i = (o + off) / stride with off = pad - k*dil, if
// that division is exact.  With o = oq*stride + om and off = fq*stride + fm (0 <= om, fm < stride)
// it is exact iff om + fm is 0 or stride, and then i = oq + fq + (om + fm == stride): no division
// per tap.
struct AxisSplit {
    int q, m;             // value = q * stride + m, 0 <= m < stride
};
__device__ __forceinline__ int floor_div(int a, int b) {       // b > 0
    const int qd = a / b;
    return (a % b != 0 && a < 0) ? qd - 1 : qd;
}
__device__ __forceinline__ AxisSplit split(int v, int stride) {
    AxisSplit s;
    s.q = floor_div(v, stride);
    s.m = v - s.q * stride;
    return s;
}
__device__ __forceinline__ bool transposed_coord(AxisSplit o, AxisSplit f, int stride, int size, int &i) {
    const int sum = o.m + f.m;
    i = o.q + f.q + (sum == stride ? 1 : 0);
    return (sum == 0 || sum == stride) && (unsigned)i < (unsigned)size;
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

// `count` output pixels of one output row, every used tap inside the image; pixel x has output
// number r0 + rel0 + x * rel_step.  off_a: byte offset of the window origin of the first pixel
// (plane 0, word c0); step: bytes between the origins of successive pixels; kadd: constant term
// of this chunk.  All words of a pixel are requested before any is used; other wavefronts of
// the SIMD cover the latency.
// The chunk's taps are taken in groups of LG (LG divides TT): the words of a group are requested
// together, which bounds the scalar registers a pixel needs while the chunk's weights (TT taps)
// stay in vector registers; a group without a used tap is skipped.
// ALL: every tap of the chunk is used (the usual case away from the top and bottom image rows):
// no test per tap or group.
template <int AB, int WB, int CWT, int TT, int LG, bool ALL, class OV>
__device__ __forceinline__ void gen_run_fast_t(const GenCtx<AB, WB, CWT, TT> &c, const OV &ov, int rel0, int count,
                                               int rel_step, uint32_t off_a, uint32_t step, int kadd, bool first,
                                               bool last) {
    static_assert(TT % LG == 0, "whole load groups");
    uint32_t off = off_a;
    int rel = rel0;
    for (int x = 0; x < count; ++x) {
        int prev = 0;
        if (!first)
            prev = __builtin_amdgcn_raw_buffer_load_b32(ov.d0, ov.col_bytes, (int)((uint32_t)rel * ov.row_bytes), 0);
        int part[AB + WB - 1];
#pragma unroll
        for (int s = 0; s < AB + WB - 1; ++s) part[s] = 0;
#pragma unroll
        for (int g0 = 0; g0 < TT; g0 += LG) {
            if (!ALL && TT > LG && !(c.okmask & (((1u << LG) - 1u) << g0))) continue;
            uint32_t a[LG][AB][CWT];
#pragma unroll
            for (int i = 0; i < LG; ++i)
#pragma unroll
                for (int p = 0; p < AB; ++p)
                    load_words<CWT>(c.base + (uint32_t)(off + c.toff[g0 + i] + (uint32_t)p * c.plane_bytes), a[i][p]);
#pragma unroll
            for (int i = 0; i < LG; ++i)
                if (ALL || (c.okmask & (1u << (g0 + i)))) {
#pragma unroll
                    for (int qq = 0; qq < WB; ++qq)
#pragma unroll
                        for (int p = 0; p < AB; ++p)
#pragma unroll
                            for (int j = 0; j < CWT; ++j) popc_acc(part[p + qq], a[i][p][j] ^ c.w[g0 + i][qq][j]);
                }
        }
        int s = part[AB + WB - 2];
#pragma unroll
        for (int i = AB + WB - 3; i >= 0; --i) s = (s << 1) + part[i];
        finish_row<false>(ov, rel, prev + kadd - 2 * s, /*first=*/true, last);   // earlier part already added
        off += step;
        rel += rel_step;
    }
}

template <int AB, int WB, int CWT, int TT, int LG, class OV>
__device__ __forceinline__ void gen_run_fast(const GenCtx<AB, WB, CWT, TT> &c, const OV &ov, int rel0, int count,
                                             int rel_step, uint32_t off_a, uint32_t step, int kadd, bool first,
                                             bool last) {
    if (c.okmask == (1u << TT) - 1u) gen_run_fast_t<AB, WB, CWT, TT, LG, true>(c, ov, rel0, count, rel_step, off_a, step, kadd, first, last);
    else gen_run_fast_t<AB, WB, CWT, TT, LG, false>(c, ov, rel0, count, rel_step, off_a, step, kadd, first, last);
}

// One output pixel of one chunk with every tap tested (image borders, transposed convolution,
// chunks with padding words).
// `tap(i, ih, iw)` says whether tap i of the chunk touches the image for this output pixel and
// where.
template <int AB, int WB, int CWT, int TT, class OV, class TapFn>
__device__ __forceinline__ void gen_pixel_checked(const BranchArgs &g, const OV &ov, uniform_words As,
                                                  const uint32_t (&w)[TT][WB][CWT], TapFn tap, int rel, int img,
                                                  int c0, bool first, bool last) {
    const int Cw = g.Cw;
    int prev = 0;
    if (!first)
        prev = __builtin_amdgcn_raw_buffer_load_b32(ov.d0, ov.col_bytes, (int)((uint32_t)rel * ov.row_bytes), 0);
    int part[AB + WB - 1];
#pragma unroll
    for (int s = 0; s < AB + WB - 1; ++s) part[s] = 0;
    int nvalid = 0;
#pragma unroll
    for (int i = 0; i < TT; ++i) {
        int ih, iw;
        if (tap(i, ih, iw)) {               // uniform
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
    finish_row<false>(ov, rel, val, /*first=*/true, last);      // the earlier part is already added
}

// Transposed convolution by output phase.  Output pixel (oh, ow) receives kernel element (kh, kw)
// only if oh + ph - kh*dh is a multiple of the stride (likewise in w), so the pixels of one phase
// (pa, pb) = ((oh + ph) mod sh, (ow + pw) mod sw) all use the same sub-kernel, and along a row the
// input column of a tap advances by one per phase pixel: a stride-1 run in the input, written to
// every sw-th output pixel.  Per phase the sub-kernel is taken in chunks of TT taps like the
// forward kernel's; interior phase pixels go through the untested run, the others are tested.
// k*dil written as Q*stride + res (0 <= res < stride), stepped from one kernel element to the next
// without a division
struct TapWalk {
    int Q, res;
};
__device__ __forceinline__ void step(TapWalk &w, AxisSplit dil, int stride) {   // dil = dil_q*stride + dil_m
    w.Q += dil.q;
    w.res += dil.m;
    if (w.res >= stride) { w.res -= stride; ++w.Q; }
}

// The launch is phase-major: blockIdx.y walks the sh*sw phases, and within a phase the wavefronts
// split its pixels (all images, sub-rows and sub-columns of that phase, in this order) into runs
// of rows_per_wave, so a wavefront has ONE sub-kernel and every SIMD gets its share whatever the
// stride.  Sub-row i, sub-column j of phase (pa, pb) is output pixel (a0 + i*sh, b0 + j*sw), with
// a0 the first row of the phase, and reads input pixel (i + qa, j + qb) shifted by the tap.
template <int AB, int WB, int CWT, int TT, int LG, class OV>
__device__ __forceinline__ void transposed_phases(const BranchArgs &g, uniform_words As, int nload, float sc, int ct,
                                                  int wave_x) {
    const ConvGeom &q = g.geo;
    const int T = q.KH * q.KW, Cw = g.Cw;
    const uint32_t pixel_bytes = (uint32_t)(AB * Cw) * 4u;
    const int Nb = __builtin_amdgcn_readfirstlane(g.rows / (q.Ho * q.Wo));
    // the divisions of this function are per wavefront (or per phase), never per tap or pixel
    AxisSplit dh_s = split(q.dh, q.sh), dw_s = split(q.dw, q.sw);
    dh_s.q = __builtin_amdgcn_readfirstlane(dh_s.q); dh_s.m = __builtin_amdgcn_readfirstlane(dh_s.m);
    dw_s.q = __builtin_amdgcn_readfirstlane(dw_s.q); dw_s.m = __builtin_amdgcn_readfirstlane(dw_s.m);
    const int ph_m = __builtin_amdgcn_readfirstlane(q.ph % q.sh), pw_m = __builtin_amdgcn_readfirstlane(q.pw % q.sw);
    GenCtx<AB, WB, CWT, TT> c;
    c.base = (uint64_t)g.A;
    c.plane_bytes = (uint32_t)Cw * 4u;
    for (int phase = (int)blockIdx.y; phase < q.sh * q.sw; phase += (int)gridDim.y) {
        const int pa = __builtin_amdgcn_readfirstlane(phase / q.sw), pb = phase - pa * q.sw;
        // first output row / column of the phase: the smallest o >= 0 with (o + pad) mod s == p
        const int a0 = (pa >= ph_m) ? pa - ph_m : pa - ph_m + q.sh;
        const int b0 = (pb >= pw_m) ? pb - pw_m : pb - pw_m + q.sw;
        if (a0 >= q.Ho || b0 >= q.Wo) continue;                           // no pixel has this phase
        const int Hp = __builtin_amdgcn_readfirstlane((q.Ho - a0 + q.sh - 1) / q.sh);
        const int Wp = __builtin_amdgcn_readfirstlane((q.Wo - b0 + q.sw - 1) / q.sw);
        const int items = Nb * Hp * Wp;
        const int it0 = wave_x * g.rows_per_wave;
        if (wave_x >= (items + g.rows_per_wave - 1) / g.rows_per_wave) continue;
        const int it1 = min(items, it0 + g.rows_per_wave);
        const int qa = __builtin_amdgcn_readfirstlane((a0 + q.ph - pa) / q.sh);   // exact by construction
        const int qb = __builtin_amdgcn_readfirstlane((b0 + q.pw - pb) / q.sw);
        auto decode = [&](int it, int &n, int &i, int &j) {
            n = __builtin_amdgcn_readfirstlane(it / (Hp * Wp));
            const int rem = it - n * Hp * Wp;
            i = __builtin_amdgcn_readfirstlane(rem / Wp);
            j = rem - i * Wp;
        };
        auto out_pixel = [&](int n, int i, int j) { return (n * q.Ho + a0 + i * q.sh) * q.Wo + b0 + j * q.sw; };
        int n0, i0, j0, n9, i9, j9;
        decode(it0, n0, i0, j0);
        decode(it1 - 1, n9, i9, j9);
        const int first_pix = out_pixel(n0, i0, j0);
        const OV ov = make_out_view<OV>(g, first_pix, out_pixel(n9, i9, j9) + 1, nload, sc, ct);

        // taps of this phase: kh*dh = pa and kw*dw = pb modulo the stride
        int ntaps = 0;
        {
            TapWalk wh = {0, 0}, ww = {0, 0};
            int kw = 0;
            for (int t = 0; t < T; ++t) {
                if (wh.res == pa && ww.res == pb) ++ntaps;
                step(ww, dw_s, q.sw);
                if (++kw == q.KW) { kw = 0; ww.Q = 0; ww.res = 0; step(wh, dh_s, q.sh); }
            }
        }
        const int nchunks = (ntaps + TT - 1) / TT;             // 0: the phase's pixels are plain zeros
        for (int c0 = 0; c0 < ((nchunks == 0) ? 1 : Cw); c0 += CWT)
            for (int lc = 0; lc < ((nchunks == 0) ? 1 : nchunks); ++lc) {
                const bool first = (c0 == 0 && lc == 0);
                const bool last = (nchunks == 0) || (c0 + CWT >= Cw && lc + 1 >= nchunks);
                // taps lc*TT .. of the phase's list: weight index and input offset in input pixels
                // relative to (i + qa, j + qb); for a tap of the phase (pa - kh*dh) / sh = -Q exactly
                int dqh[TT], dqw[TT];
                uint32_t used = 0u;                             // bit i: slot i holds a tap
#pragma unroll
                for (int i = 0; i < TT; ++i) {
                    dqh[i] = 0; dqw[i] = 0;
#pragma unroll
                    for (int qq = 0; qq < WB; ++qq)
#pragma unroll
                        for (int j = 0; j < CWT; ++j) c.w[i][qq][j] = 0u;
                }
                {
                    TapWalk wh = {0, 0}, ww = {0, 0};
                    int kw = 0, seen = 0, slot = 0;
                    for (int t = 0; t < T && slot < TT && nchunks > 0; ++t) {
                        if (wh.res == pa && ww.res == pb) {
                            if (seen >= lc * TT) {
#pragma unroll
                                for (int i = 0; i < TT; ++i)
                                    if (i == slot) {
                                        dqh[i] = -wh.Q;
                                        dqw[i] = -ww.Q;
#pragma unroll
                                        for (int qq = 0; qq < WB; ++qq) {
                                            if (c0 + CWT <= Cw) {
                                                load_run<CWT>(g.Wt + ((nload * T + t) * WB + qq) * Cw + c0, c.w[i][qq]);
                                            } else {
#pragma unroll
                                                for (int j = 0; j < CWT; ++j)
                                                    c.w[i][qq][j] = (c0 + j < Cw) ? g.Wt[((nload * T + t) * WB + qq) * Cw + c0 + j] : 0u;
                                            }
                                        }
                                    }
                                used |= 1u << slot;
                                ++slot;
                            }
                            ++seen;
                        }
                        step(ww, dw_s, q.sw);
                        if (++kw == q.KW) { kw = 0; ww.Q = 0; ww.res = 0; step(wh, dh_s, q.sh); }
                    }
                }
                // sub-columns of the phase whose taps are all inside the image: j + qb in [jlo, jhi)
                int jlo = 0, jhi = g.W;
#pragma unroll
                for (int i = 0; i < TT; ++i)
                    if (used & (1u << i)) {
                        jlo = max(jlo, -dqw[i]);
                        jhi = min(jhi, g.W - dqw[i]);
                    }
                const bool fast_chunk = (c0 + CWT <= Cw) && used != 0u;
                int n = n0, i = i0, j = j0, it = it0;
                while (it < it1) {
                    const int seg_end = min(it1, it - j + Wp);        // end of this sub-row within the range
                    const int count = seg_end - it;
                    const int Iq = i + qa, Jq0 = j + qb;
                    const int rel0 = out_pixel(n, i, j) - first_pix;
                    // phase pixels x in [xa, xb) run untested
                    int xa = 0, xb = 0;
                    if (fast_chunk) {
                        uint32_t okmask = 0u, safe_off = 0u;
#pragma unroll
                        for (int k = 0; k < TT; ++k) {
                            const bool ok = (used & (1u << k)) && (unsigned)(Iq + dqh[k]) < (unsigned)g.H;
                            c.toff[k] = (uint32_t)(dqh[k] * g.W + dqw[k]) * pixel_bytes;
                            if (ok) {
                                if (okmask == 0u) safe_off = c.toff[k];
                                okmask |= 1u << k;
                            }
                        }
                        if (okmask != 0u) {
                            xa = max(0, jlo - Jq0);
                            xb = min(count, jhi - Jq0);
                            if (xb <= xa) { xa = 0; xb = 0; }
                            else {
                                c.okmask = okmask;
#pragma unroll
                                for (int k = 0; k < TT; ++k)
                                    if (!(okmask & (1u << k))) c.toff[k] = safe_off;
                            }
                        }
                    }
                    auto checked = [&](int x) {
                        auto tap = [&](int k, int &ih, int &iw) {
                            ih = Iq + dqh[k];
                            iw = Jq0 + x + dqw[k];
                            return (used & (1u << k)) && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W;
                        };
                        gen_pixel_checked<AB, WB, CWT, TT>(g, ov, As, c.w, tap, rel0 + x * q.sw, n, c0, first, last);
                    };
                    for (int x = 0; x < xa; ++x) checked(x);
                    if (xb > xa) {
                        const uint32_t off_a = (uint32_t)((n * g.H + Iq) * g.W + Jq0 + xa) * pixel_bytes + (uint32_t)c0 * 4u;
                        const int kadd = (c0 == 0) ? __builtin_popcount(c.okmask) * g.kconst : 0;
                        gen_run_fast<AB, WB, CWT, TT, LG>(c, ov, rel0 + xa * q.sw, xb - xa, q.sw, off_a, pixel_bytes, kadd, first, last);
                    }
                    for (int x = max(xb, xa); x < count; ++x) checked(x);
                    it = seg_end;
                    j = 0;
                    if (++i == Hp) { i = 0; ++n; }
                }
            }
    }
}

template <int AB, int WB, int CWT, int TT, int LG, bool TR, bool EMIT>
__global__ __launch_bounds__(256) void conv_general_kernel(const BranchArgs g) {
    typedef typename std::conditional<EMIT, OutViewEmit, OutView>::type OV;
    // forward: blocks numbered per XCD; the transposed launch is two-dimensional and keeps blockIdx
    const uint32_t block = TR ? blockIdx.x : xcd_block(g.xcd_ranges, g.grid_blocks);
    const int wave = __builtin_amdgcn_readfirstlane((int)(block * 4 + (threadIdx.x >> 6)));
    int ct, rb;
    fast_divmod((uint32_t)wave, g.div_tiles, rb, ct);
    const int lane = (int)(threadIdx.x & 63);
    const int n = ct * 64 + lane;
    const int nload = (n < g.N) ? n : g.N - 1;         // lanes past N redo column N-1 (same value, same address)
    const float sc = (g.scale != nullptr) ? g.scale[nload] : 1.0f;
    uniform_words As = as_uniform(g.A);
    const ConvGeom &q = g.geo;
    const int T = q.KH * q.KW, Cw = g.Cw;
    if constexpr (TR) {
        if (Cw != 0 && T != 0) {                        // (the empty sum takes the plain row split below)
            transposed_phases<AB, WB, CWT, TT, LG, OV>(g, As, nload, sc, ct, rb);
            return;
        }
    }
    if ((int64_t)rb * g.rows_per_wave >= g.rows) return;
    const int r0 = rb * g.rows_per_wave;
    const int r1 = min(g.rows, r0 + g.rows_per_wave);
    const OV ov = make_out_view<OV>(g, r0, r1, nload, sc, ct);
    if (Cw == 0 || T == 0) {                            // empty sum
        for (int r = r0; r < r1; ++r) finish_row<true>(ov, r - r0, 0, true, true);
        return;
    }
    // position of the first output pixel (integer division runs on the vector ALU)
    int ow0, oh0, n0, line0;                            // divisions by the output image size: scalar unit
    fast_divmod((uint32_t)r0, g.div_w, line0, ow0);
    fast_divmod((uint32_t)line0, g.div_h, n0, oh0);
    const uint32_t pixel_bytes = (uint32_t)(AB * Cw) * 4u;

    GenCtx<AB, WB, CWT, TT> c;
    c.base = (uint64_t)g.A;
    c.plane_bytes = (uint32_t)Cw * 4u;
    for (int c0 = 0; c0 < Cw; c0 += CWT) {
        int kh_next = 0, kw_next = 0;                    // kernel element of tap t0: counted, never divided
        for (int t0 = 0; t0 < T; t0 += TT) {
            const bool first = (c0 == 0 && t0 == 0);
            const bool last = (c0 + CWT >= Cw && t0 + TT >= T);
            // offsets of the chunk's taps along both axes: input = output*stride + off, off = k*dil - pad
            // (all on the scalar unit, so that tap tests and addresses stay there too)
            int offh[TT], offw[TT];
            int kw_min = q.KW, kw_max = -1;
#pragma unroll
            for (int i = 0; i < TT; ++i) {
                const int t = t0 + i;
                offh[i] = kh_next * q.dh - q.ph;
                offw[i] = kw_next * q.dw - q.pw;
                if (t < T) {
                    kw_min = min(kw_min, kw_next);
                    kw_max = max(kw_max, kw_next);
                }
                if (++kw_next == q.KW) { kw_next = 0; ++kh_next; }
            }
            // output columns for which every tap of the chunk is inside the image, [lo, hi): the
            // left end is set by the leftmost kernel column of the chunk, the right end by the rightmost
            const int lo = max(0, __builtin_amdgcn_readfirstlane(-floor_div(kw_min * q.dw - q.pw, q.sw)));   // ceil(-off / s)
            const int hi = min(q.Wo, __builtin_amdgcn_readfirstlane(floor_div(g.W - 1 - (kw_max * q.dw - q.pw), q.sw) + 1));
#pragma unroll
            for (int i = 0; i < TT; ++i) {
                const int t = t0 + i;
#pragma unroll
                for (int qq = 0; qq < WB; ++qq) {
                    if (t < T && c0 + CWT <= Cw) {
                        load_run<CWT>(g.Wt + ((nload * T + t) * WB + qq) * Cw + c0, c.w[i][qq]);
                    } else {
#pragma unroll
                        for (int j = 0; j < CWT; ++j)
                            c.w[i][qq][j] = (t < T && c0 + j < Cw) ? g.Wt[((nload * T + t) * WB + qq) * Cw + c0 + j] : 0u;
                    }
                }
            }
            int ow = ow0, oh = oh0, img = n0;
            int r = r0;
            {
                const bool fast_chunk = (c0 + CWT <= Cw);
                auto checked = [&](int x, int oh_x, int ow_x) {
                    auto tap = [&](int i, int &ih, int &iw) {
                        ih = oh_x * q.sh + offh[i];
                        iw = ow_x * q.sw + offw[i];
                        return (t0 + i < T) && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W;
                    };
                    gen_pixel_checked<AB, WB, CWT, TT>(g, ov, As, c.w, tap, x - r0, img, c0, first, last);
                };
                while (r < r1) {
                    const int row_end = min(r1, r - ow + q.Wo);               // end of this output row within the range
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
                    for (int x = r; x < fa; ++x) checked(x, oh, ow + (x - r));
                    if (fb > fa) {
                        const int owa = ow + (fa - r);
                        const uint32_t off_a = (uint32_t)((img * g.H + oh * q.sh) * g.W + owa * q.sw) * pixel_bytes + (uint32_t)c0 * 4u;
                        const int kadd = (c0 == 0) ? __builtin_popcount(c.okmask) * g.kconst : 0;
                        gen_run_fast<AB, WB, CWT, TT, LG>(c, ov, fa - r0, fb - fa, 1, off_a, (uint32_t)q.sw * pixel_bytes, kadd, first, last);
                    }
                    for (int x = max(fb, fa); x < row_end; ++x) checked(x, oh, ow + (x - r));
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
    const int wave = __builtin_amdgcn_readfirstlane((int)(xcd_block(g.xcd_ranges, g.grid_blocks) * 4 + (threadIdx.x >> 6)));
    int ct, rb;
    fast_divmod((uint32_t)wave, g.div_tiles, rb, ct);
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
    auto place = [&](int t, const uint32_t *x) {       // tap t: C bits per plane at window bit t*C
        const int bit = t * C, wi = bit >> 5, sh = bit & 31;
#pragma unroll
        for (int qq = 0; qq < WB; ++qq) {
            const uint32_t lo = x[qq] << sh, hi = sh ? x[qq] >> (32 - sh) : 0u;   // hi: the part that spills into the next word
#pragma unroll
            for (int k = 0; k < KWP; ++k) {
                if (k == wi) w[qq][k] |= lo;
                if (k == wi + 1) w[qq][k] |= hi;
            }
        }
    };
    int t = 0;
    for (; t + 2 <= T; t += 2) {                       // the filter's words are contiguous: two taps per load run
        uint32_t x[2 * WB];
        load_run<2 * WB>(g.Wt + (nload * T + t) * WB, x);
        place(t, x);
        place(t + 1, x + WB);
    }
    if (t < T) {
        uint32_t x[WB];
        load_run<WB>(g.Wt + (nload * T + t) * WB, x);
        place(t, x);
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
    if (g.planes_out != nullptr) launch_kernel((conv_window_kernel<AB, WB, KWP, true>), grid, dim3(256), 0, s, g);
    else launch_kernel((conv_window_kernel<AB, WB, KWP, false>), grid, dim3(256), 0, s, g);
}

template <int AB, int WB>
hipError_t launch_window_t(const BranchArgs &g, hipStream_t s) {
    const int64_t row_blocks = ((int64_t)g.rows + g.rows_per_wave - 1) / g.rows_per_wave;
    const dim3 grid((unsigned)((row_blocks * g.col_tiles + 3) / 4));
    if (g.xcd_ranges && g.grid_blocks != grid.x) return hipErrorInvalidValue;             // host bug
    switch (g.Cw) {                                    // words per plane of the packed window
        case 1: launch_window_shape<AB, WB, 1>(g, grid, s); break;
        case 2: launch_window_shape<AB, WB, 2>(g, grid, s); break;
        case 3: launch_window_shape<AB, WB, 3>(g, grid, s); break;
        case 5: launch_window_shape<AB, WB, 5>(g, grid, s); break;
        case 8: launch_window_shape<AB, WB, 8>(g, grid, s); break;
        default: return hipErrorInvalidValue;
    }
    return launch_status();
}

constexpr int imin3(int a, int b, int c) { return a < b ? (a < c ? a : c) : (b < c ? b : c); }

// Largest number of kernel elements any phase of a transposed convolution uses (see transposed_phases)
inline int transposed_phase_taps(const ConvGeom &q) {
    int most = 0;
    for (int pa = 0; pa < q.sh; ++pa)
        for (int pb = 0; pb < q.sw; ++pb) {
            int nh = 0, nw = 0;
            for (int kh = 0; kh < q.KH; ++kh) nh += ((kh * q.dh) % q.sh == pa);
            for (int kw = 0; kw < q.KW; ++kw) nw += ((kw * q.dw) % q.sw == pb);
            most = nh * nw > most ? nh * nw : most;
        }
    return most;
}

template <int AB, int WB, int CWT>
void launch_general_shape(const BranchArgs &g, dim3 grid, bool emit, hipStream_t s) {
    // taps whose activation words are requested together (scalar registers), also the weight chunk
    // of the plain variant
    constexpr int TT = CWT > 4 ? 1 : imin3(6, 64 / (WB * CWT), 24 / (AB * CWT));
    // wide variant for kernels with more taps than that: up to three groups of (at most 3) taps per
    // weight chunk while the chunk stays below 96 vector registers; fewer passes over the output
    // and fewer weight reloads (forward convolution, up to four activation bits: measured 15 %
    // faster on 3x3 and 5x5 layers with 64..96 channels and one or two bits, 0..6 % with four)
    constexpr int LGW = TT < 3 ? TT : 3;
    constexpr int NGW = imin3(3, 96 / (WB * CWT * LGW), 3);
    if (g.geo.transposed) {
        // phase-major grid: y walks the phases, x the wavefronts of the largest phase (all images)
        const ConvGeom &q = g.geo;
        const int64_t nb = (int64_t)g.rows / ((int64_t)q.Ho * q.Wo);
        const int64_t hp = (q.Ho + q.sh - 1) / q.sh, wp = (q.Wo + q.sw - 1) / q.sw;
        const int64_t waves = ((nb * hp * wp + g.rows_per_wave - 1) / g.rows_per_wave) * g.col_tiles;
        const int64_t phases = (int64_t)q.sh * q.sw;
        const dim3 tgrid((unsigned)((waves + 3) / 4), (unsigned)(phases < 65535 ? phases : 65535));
        // A phase of the usual deconvolutions (4x4 or 3x3 kernel, stride 2) has at most four taps:
        // with one or two activation bits all four fit one chunk (4 x WB x CWT weight registers),
        // taken as two groups of two taps (one group of one with eight channel words and two bits),
        // instead of a chunk of TT taps and a second one for the rest.
        if constexpr (AB <= 2 && WB * CWT <= 16 && TT < 4) {
            if (transposed_phase_taps(q) == 4) {
                if (emit) launch_kernel((conv_general_kernel<AB, WB, CWT, 4, (AB * CWT <= 8 ? 2 : 1), true, true>), tgrid, dim3(256), 0, s, g);
                else launch_kernel((conv_general_kernel<AB, WB, CWT, 4, (AB * CWT <= 8 ? 2 : 1), true, false>), tgrid, dim3(256), 0, s, g);
                return;
            }
        }
        if constexpr (CWT <= 4) {
            if (emit) launch_kernel((conv_general_kernel<AB, WB, CWT, TT, TT, true, true>), tgrid, dim3(256), 0, s, g);
            else launch_kernel((conv_general_kernel<AB, WB, CWT, TT, TT, true, false>), tgrid, dim3(256), 0, s, g);
        }
        return;
    }
    // (eight-word chunks exist for the four-tap deconvolution alone)
    if constexpr (CWT <= 4) {
        // measured with four activation bits: 5x5, 64 -> 64 channels, 56x56: 135 -> 127 us; 3x3 dilation 4,
        // 512 -> 512, 17x17: 357 -> 340 us; 3x3 dilation 2, 256 -> 256, 33x33, three weight bits: equal
        if constexpr (AB <= 4 && WB <= 4 && NGW >= 2) {
            if (g.geo.KH * g.geo.KW > TT) {
                if (emit) launch_kernel((conv_general_kernel<AB, WB, CWT, NGW * LGW, LGW, false, true>), grid, dim3(256), 0, s, g);
                else launch_kernel((conv_general_kernel<AB, WB, CWT, NGW * LGW, LGW, false, false>), grid, dim3(256), 0, s, g);
                return;
            }
        }
        if (emit) launch_kernel((conv_general_kernel<AB, WB, CWT, TT, TT, false, true>), grid, dim3(256), 0, s, g);
        else launch_kernel((conv_general_kernel<AB, WB, CWT, TT, TT, false, false>), grid, dim3(256), 0, s, g);
    }
}

template <int AB, int WB>
hipError_t launch_general_t(const BranchArgs &g, hipStream_t s) {
    const int64_t row_blocks = ((int64_t)g.rows + g.rows_per_wave - 1) / g.rows_per_wave;
    const dim3 grid((unsigned)((row_blocks * g.col_tiles + 3) / 4));
    if (g.xcd_ranges && g.grid_blocks != grid.x) return hipErrorInvalidValue;             // host bug
    const bool emit = g.planes_out != nullptr;
    // channel words per chunk (at most AB*CWT = 8 and no more than there are), then taps per chunk
    // such that the chunk's weight words (TT*WB*CWT) stay at or below 64 VGPRs and one pixel's
    // activation words (TT*AB*CWT) at or below 24 SGPRs
    // A chunk that runs past the last channel word takes the tested path for every pixel, so the
    // chunk width divides the word count where a width of 4, 2 or 1 does (C = 96: three chunks of
    // one word); only beyond 16 words is a ragged last chunk the smaller cost.
    constexpr int CMAX = (AB <= 2) ? 4 : (AB <= 4) ? 2 : 1;
    const bool any = g.Cw > 16;
    if constexpr (AB <= 2 && WB <= 2) {
        if (g.geo.transposed && g.Cw % 8 == 0 && transposed_phase_taps(g.geo) == 4) {
            launch_general_shape<AB, WB, 8>(g, grid, emit, s);
            return launch_status();
        }
    }
    if (CMAX >= 4 && g.Cw >= 4 && (any || g.Cw % 4 == 0)) launch_general_shape<AB, WB, (CMAX >= 4 ? 4 : 1)>(g, grid, emit, s);
    else if (CMAX >= 4 && g.Cw % 3 == 0) launch_general_shape<AB, WB, (CMAX >= 4 ? 3 : 1)>(g, grid, emit, s);   // C = 96, 192, 288
    else if (CMAX >= 2 && g.Cw >= 2 && (any || g.Cw % 2 == 0)) launch_general_shape<AB, WB, (CMAX >= 2 ? 2 : 1)>(g, grid, emit, s);
    else launch_general_shape<AB, WB, 1>(g, grid, emit, s);
    return launch_status();
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
        case 5: return launch_window_t<QNN_AB, 5>(g, s);
        case 6: return launch_window_t<QNN_AB, 6>(g, s);
        case 7: return launch_window_t<QNN_AB, 7>(g, s);
        case 8: return launch_window_t<QNN_AB, 8>(g, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace qnn
