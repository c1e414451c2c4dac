// 3x3 convolution with very few input channels (9*C <= 32, e.g. the 3-channel first layer of a
// VGG-shaped stack): the whole K axis of an output pixel fits ONE 32-bit word per bit plane, so
// the im2col row is materialised after all — it is as small as the per-pixel planes — and the
// branch product (paper Eq. (8)) is a GEMM with a single word per plane.  Compiled once per
// activation bit width, -DQNN_AB=<1..8>.
//
//   im2col_pack_kernel   codes NHWC -> words [pixel][AB]: bit t*C + c of word p is digit p of
//                        u = (v + 2^AB - 1)/2 of tap t = (kh, kw), channel c; bits of taps
//                        outside the image are 0.
//   conv_small_kernel    lane = filter; a pixel's AB words arrive through scalar loads (two
//                        buffers, hand-placed wait, as in qnn_branch.hip), two pixels per load;
//                        per branch one v_xor_b32 + v_bcnt_u32_b32 and nothing else.  Zero padding
//                        costs the inner loop nothing: the bits of a padded tap are 0 in every
//                        activation word, so the unmasked sum is too large by exactly
//                        (2^AB - 1) * sum_q 2^q popcount(w_q at the padded taps), a per-filter
//                        number that depends only on WHICH taps are padded.  It is folded into the
//                        constant term, worked out once per image row (and once more for each of
//                        the row's two end pixels).
#include "qnn_internal.h"
#include "qnn_device_util.h"

#ifndef QNN_AB
#error "compile with -DQNN_AB=<activation bits>"
#endif

namespace qnn {
namespace {

// ---------------------------------------------------------------------------------------
// im2col words.  Two steps per block of 256 output pixels, through LDS:
//   1. every input pixel the block's windows touch gets a "pixel word": digit p of channel c
//      at bit p*C + c (C*BITS <= 24 bits), each channel's digits spread by a 256-entry table;
//   2. the thread of output pixel r gathers its nine neighbours' pixel words (zero where the
//      neighbour is outside the image) and regroups them by plane: word p = the C bits of plane
//      p of tap t at bit t*C.
// One thread writes its pixel's BITS consecutive words; a wavefront writes one contiguous piece.
// ---------------------------------------------------------------------------------------
constexpr int kIm2colBlock = 256;
constexpr int kIm2colMaxW = 3072;          // LDS: (block + 2*W + 2) pixel words; wider images take the simple kernel

template <typename CodeT, int BITS>
__global__ __launch_bounds__(kIm2colBlock) void im2col_pack_kernel(const CodeT *__restrict__ codes, int64_t pixels,
                                                                    int H, int W, int C, FastDiv div_w, FastDiv div_h,
                                                                    uint32_t *__restrict__ words) {
    constexpr int VMAX = (1 << BITS) - 1;
    extern __shared__ uint32_t lds[];
    uint32_t *spread = lds;                          // [256]: digits of u at stride C
    uint32_t *pw = lds + 256;                        // pixel words of input pixels lo .. lo + span - 1
    const int tid = (int)threadIdx.x;
    {
        uint32_t e = 0u;
#pragma unroll
        for (int p = 0; p < BITS; ++p) e |= (uint32_t)((tid >> p) & 1) << (p * C);
        spread[tid] = e;
    }
    const int64_t b0 = (int64_t)blockIdx.x * kIm2colBlock;
    const int64_t lo = (b0 - W - 1 > 0) ? b0 - W - 1 : 0;
    const int64_t hi = (b0 + kIm2colBlock + W + 1 < pixels) ? b0 + kIm2colBlock + W + 1 : pixels;
    const int span = (int)(hi - lo);
    __syncthreads();
    for (int i = tid; i < span; i += kIm2colBlock) {
        const CodeT *src = codes + (lo + i) * C;
        uint32_t v = 0u;
        for (int c = 0; c < C; ++c) v |= spread[(((int)src[c] + VMAX) >> 1) & 255] << c;
        pw[i] = v;
    }
    __syncthreads();
    const int64_t r = b0 + tid;
    if (r >= pixels) return;
    int line, ow, img, oh;
    fast_divmod((uint32_t)r, div_w, line, ow);
    fast_divmod((uint32_t)line, div_h, img, oh);
    uint32_t nb[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        const int dh = t / 3 - 1, dw = t % 3 - 1;
        const bool ok = (unsigned)(oh + dh) < (unsigned)H && (unsigned)(ow + dw) < (unsigned)W;
        const int idx = ok ? (int)(r - lo) + dh * W + dw : 0;     // inside [0, span) whenever the tap is in the image
        const uint32_t v = pw[idx];
        nb[t] = ok ? v : 0u;
    }
    const uint32_t cmask = (1u << C) - 1u;
    uint32_t out[BITS];
#pragma unroll
    for (int p = 0; p < BITS; ++p) {
        uint32_t wv = 0u;
#pragma unroll
        for (int t = 0; t < 9; ++t) wv |= ((nb[t] >> (p * C)) & cmask) << (t * C);
        out[p] = wv;
    }
    uint32_t *dst = words + r * BITS;                // 16-byte aligned where BITS is a multiple of 4
    if constexpr (BITS % 4 == 0) {
        typedef uint32_t w4 __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int p = 0; p < BITS; p += 4) {
            w4 v;
            v.x = out[p]; v.y = out[p + 1]; v.z = out[p + 2]; v.w = out[p + 3];
            *reinterpret_cast<w4 *>(dst + p) = v;
        }
    } else {
#pragma unroll
        for (int p = 0; p < BITS; ++p) dst[p] = out[p];
    }
}

// the same, one thread per pixel straight from global memory (images too wide for the LDS variant)
template <typename CodeT, int BITS>
__global__ __launch_bounds__(256) void im2col_pack_simple_kernel(const CodeT *__restrict__ codes, int64_t pixels,
                                                                 int H, int W, int C, uint32_t *__restrict__ words) {
    constexpr int VMAX = (1 << BITS) - 1;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < pixels;
         r += (int64_t)gridDim.x * blockDim.x) {
        const int ow = (int)(r % W);
        const int oh = (int)((r / W) % H);
        uint32_t word[BITS];
#pragma unroll
        for (int p = 0; p < BITS; ++p) word[p] = 0u;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const int dh = t / 3 - 1, dw = t % 3 - 1;
            if ((unsigned)(oh + dh) < (unsigned)H && (unsigned)(ow + dw) < (unsigned)W) {
                const CodeT *src = codes + (r + (int64_t)dh * W + dw) * C;
                for (int c = 0; c < C; ++c) {
                    const int u = ((int)src[c] + VMAX) >> 1;
#pragma unroll
                    for (int p = 0; p < BITS; ++p) word[p] |= (uint32_t)((u >> p) & 1) << (t * C + c);
                }
            }
        }
#pragma unroll
        for (int p = 0; p < BITS; ++p) words[r * BITS + p] = word[p];
    }
}

// ---------------------------------------------------------------------------------------
// The product.  State of one wavefront: its filter's window word per weight plane, the valid-tap
// masks, where the im2col words are.
// ---------------------------------------------------------------------------------------
template <int AB, int WB, class OV>
struct SmallCtx {
    uint32_t wq[WB];                 // the lane's filter: bit t*C + c of plane q
    uint32_t rowmask[3], colmask[3]; // window bits of kernel row / column k
    uint32_t full;                   // all 9*C window bits
    int kelem;                       // (2^AB - 1)(2^WB - 1): constant term per window bit
    uint64_t base;                   // byte address of the im2col words
    int r0;                          // first pixel of the wavefront (output rows are relative to it)

    // Constant term of a pixel whose valid window bits are m:  kelem * popcount(m), plus the
    // correction for the padded taps (see the head of the file).
    __device__ __forceinline__ int class_const(uint32_t m) const {
        const uint32_t pad = full & ~m;
        int wpad = 0;
#pragma unroll
        for (int q = WB - 1; q >= 0; --q) wpad = (wpad << 1) + __builtin_popcount(wq[q] & pad);
        return __builtin_popcount(m) * kelem + 2 * ((1 << AB) - 1) * wpad;
    }

    // all AB*WB branches of one pixel whose words are a[first_word .. first_word + AB):
    // S' = sum_s 2^s part[s], parts shared by the branches with equal p + q
    template <class Words>
    __device__ __forceinline__ int branch_sum(const Words &a, int first_word) const {
        int part[AB + WB - 1];
#pragma unroll
        for (int q = 0; q < WB; ++q)
#pragma unroll
            for (int p = 0; p < AB; ++p) {
                const uint32_t x = a.get(first_word + p) ^ wq[q];
                if (q == 0 || p == AB - 1) popc_set(part[p + q], x);      // first branch of its sum
                else popc_acc(part[p + q], x);
            }
        int sum = part[AB + WB - 2];
#pragma unroll
        for (int i = AB + WB - 3; i >= 0; --i) sum = (sum << 1) + part[i];
        return sum;
    }

    // one pixel on its own (row ends, one-pixel leftovers): load, wait, compute
    __device__ __forceinline__ void single(const OV &ov, int r, uint32_t m) const {
        SRun<AB> a;
        a.template request<0>(base, (uint32_t)r * (uint32_t)(AB * 4));
        a.template arrive<true>();
        finish_row<true>(ov, r - r0, class_const(m) - 2 * branch_sum(a, 0), true, true);
    }

    // pixels ra .. rb-1 (rb - ra >= 2), all with the same valid mask (constant term kvec), two per
    // load.  An odd count ends with a pair placed at rb-2 that redoes one pixel (same value, same
    // address).  Two buffers: the next pair is in flight while this one is consumed.
    __device__ __forceinline__ void pairs(const OV &ov, int ra, int rb, int kvec) const {
        constexpr uint32_t kPixelBytes = AB * 4u;
        SRun<2 * AB> bufA, bufB;
        const int r_last = rb - 2;
        int r = ra;
        bufA.template request<0>(base, (uint32_t)ra * kPixelBytes);
        auto one_pair = [&](SRun<2 * AB> &cur, SRun<2 * AB> &nxt) {
            cur.template arrive<true>();
            const int rn = (r < r_last) ? min(r + 2, r_last) : r;      // the last pair prefetches itself (unused)
            nxt.template request<0>(base, (uint32_t)rn * kPixelBytes);
            const int s0 = branch_sum(cur, 0), s1 = branch_sum(cur, AB);
            finish_row<true>(ov, r - r0, kvec - 2 * s0, true, true);
            finish_row<true>(ov, r - r0 + 1, kvec - 2 * s1, true, true);
            r = rn;
        };
        const int npairs = (rb - ra + 1) / 2;
        int done = 0;
        while (done + 1 < npairs) {
            one_pair(bufA, bufB);
            one_pair(bufB, bufA);
            done += 2;
        }
        if (done < npairs) one_pair(bufA, bufB);
        bufA.template arrive<true>();                  // drain the last prefetch
        bufB.template arrive<false>();
    }
};

template <int AB, int WB, bool EMIT>
__global__ __launch_bounds__(256) void conv_small_kernel(const BranchArgs g) {
    typedef typename std::conditional<EMIT, OutViewEmit, OutView>::type OV;
    const int wave = __builtin_amdgcn_readfirstlane((int)(xcd_block(g.xcd_ranges, g.grid_blocks) * 4 + (threadIdx.x >> 6)));
    int ct, rb;
    fast_divmod((uint32_t)wave, g.div_tiles, rb, ct);
    const bool active = (int64_t)rb * g.rows_per_wave < g.rows;
    if (!active) return;
    const int r0 = rb * g.rows_per_wave;
    const int r1 = min(g.rows, r0 + g.rows_per_wave);
    const int lane = (int)(threadIdx.x & 63);
    const int n = ct * 64 + lane;
    const int nload = (n < g.N) ? n : g.N - 1;         // lanes past N redo column N-1 (same value, same address)
    const float sc = (g.scale != nullptr) ? g.scale[nload] : 1.0f;
    const int C = g.C, H = g.H, W = g.W;

    SmallCtx<AB, WB, OV> c;
    {
        // the filter's 9*C-bit word per weight plane, assembled from the per-tap words
        uint32_t taps[9 * WB];                         // the filter's words are contiguous: [tap][plane]
        load_run<9 * WB>(g.Wt + nload * 9 * WB, taps);
#pragma unroll
        for (int q = 0; q < WB; ++q) {
            c.wq[q] = 0u;
#pragma unroll
            for (int t = 0; t < 9; ++t) c.wq[q] |= taps[t * WB + q] << (t * C);
        }
    }
    const uint32_t tapbits = (1u << C) - 1u;
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        c.rowmask[k] = (tapbits << ((3 * k) * C)) | (tapbits << ((3 * k + 1) * C)) | (tapbits << ((3 * k + 2) * C));
        c.colmask[k] = (tapbits << (k * C)) | (tapbits << ((k + 3) * C)) | (tapbits << ((k + 6) * C));
    }
    c.full = c.rowmask[0] | c.rowmask[1] | c.rowmask[2];
    c.kelem = g.kconst;
    c.base = (uint64_t)g.A;
    c.r0 = r0;
    const OV ov = make_out_view<OV>(g, r0, r1, nload, sc, ct);

    int ow, oh, line0, img0;
    fast_divmod((uint32_t)r0, g.div_w, line0, ow);
    fast_divmod((uint32_t)line0, g.div_h, img0, oh);
    int r = r0;
    while (r < r1) {
        // the part of this image row that belongs to the wavefront: pixels r .. stop-1
        const int row_end = r - ow + W;
        const int stop = min(r1, row_end);
        uint32_t mrow = c.full;
        if (oh == 0) mrow &= ~c.rowmask[0];
        if (oh == H - 1) mrow &= ~c.rowmask[2];
        int a = r, b = stop;
        if (ow == 0) {                                  // column 0 (in a one-column image also the last one)
            c.single(ov, a, mrow & ~c.colmask[0] & (W == 1 ? ~c.colmask[2] : ~0u));
            ++a;
        }
        const bool ends_row = (stop == row_end) && (b > a);
        if (ends_row) --b;                              // column W-1 is taken on its own below
        if (b - a >= 2) c.pairs(ov, a, b, c.class_const(mrow));
        else if (b - a == 1) c.single(ov, a, mrow);
        if (ends_row) c.single(ov, b, mrow & ~c.colmask[2]);
        ow += stop - r;
        r = stop;
        if (ow == W) {
            ow = 0;
            if (++oh == H) oh = 0;
        }
    }
}

template <int AB, int WB>
hipError_t launch_small_t(const BranchArgs &g, hipStream_t s) {
    const int64_t row_blocks = ((int64_t)g.rows + g.rows_per_wave - 1) / g.rows_per_wave;
    const int64_t waves = row_blocks * g.col_tiles;
    const dim3 grid((unsigned)((waves + 3) / 4));
    if (g.xcd_ranges && g.grid_blocks != grid.x) return hipErrorInvalidValue;             // host bug
    if (g.planes_out != nullptr) launch_kernel((conv_small_kernel<AB, WB, true>), grid, dim3(256), 0, s, g);
    else launch_kernel((conv_small_kernel<AB, WB, false>), grid, dim3(256), 0, s, g);
    return launch_status();
}

}  // namespace

#define QNN_CAT2(a, b) a##b
#define QNN_CAT(a, b) QNN_CAT2(a, b)

hipError_t QNN_CAT(launch_conv_small_ab, QNN_AB)(const BranchArgs &g, int wb, hipStream_t s) {
    switch (wb) {
        case 1: return launch_small_t<QNN_AB, 1>(g, s);
        case 2: return launch_small_t<QNN_AB, 2>(g, s);
        case 3: return launch_small_t<QNN_AB, 3>(g, s);
        case 4: return launch_small_t<QNN_AB, 4>(g, s);
        case 5: return launch_small_t<QNN_AB, 5>(g, s);
        case 6: return launch_small_t<QNN_AB, 6>(g, s);
        case 7: return launch_small_t<QNN_AB, 7>(g, s);
        case 8: return launch_small_t<QNN_AB, 8>(g, s);
    }
    return hipErrorInvalidValue;
}

hipError_t QNN_CAT(launch_im2col_pack_ab, QNN_AB)(const void *codes, int code_bytes, int64_t pixels, int H, int W,
                                                  int C, uint32_t *words, hipStream_t s) {
    if (pixels == 0) return hipSuccess;
    if (W <= kIm2colMaxW) {
        const unsigned blocks = (unsigned)((pixels + kIm2colBlock - 1) / kIm2colBlock);
        const size_t lds = (size_t)(256 + kIm2colBlock + 2 * W + 2) * 4u;
        const FastDiv dw = fast_div_for(W), dh = fast_div_for(H);
        if (code_bytes == 1)
            launch_kernel((im2col_pack_kernel<int8_t, QNN_AB>), dim3(blocks), dim3(kIm2colBlock), lds, s,
                               (const int8_t *)codes, pixels, H, W, C, dw, dh, words);
        else
            launch_kernel((im2col_pack_kernel<int16_t, QNN_AB>), dim3(blocks), dim3(kIm2colBlock), lds, s,
                               (const int16_t *)codes, pixels, H, W, C, dw, dh, words);
        return launch_status();
    }
    const int64_t want = (pixels + 255) / 256;
    const unsigned blocks = (unsigned)(want < (int64_t)1 << 20 ? want : (int64_t)1 << 20);
    if (code_bytes == 1)
        launch_kernel((im2col_pack_simple_kernel<int8_t, QNN_AB>), dim3(blocks), dim3(256), 0, s,
                           (const int8_t *)codes, pixels, H, W, C, words);
    else
        launch_kernel((im2col_pack_simple_kernel<int16_t, QNN_AB>), dim3(blocks), dim3(256), 0, s,
                           (const int16_t *)codes, pixels, H, W, C, words);
    return launch_status();
}

}  // namespace qnn
