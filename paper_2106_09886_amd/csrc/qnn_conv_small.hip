// 3x3 convolution with very few input channels (9*C <= 32, e.g. the 3-channel first layer of a
// VGG-shaped stack): the whole K axis of an output pixel fits ONE 32-bit word per bit plane, so
// the im2col row is materialised after all — it is as small as the per-pixel planes — and the
// branch product (paper Eq. (8)) is a GEMM with a single word per plane.  Compiled once per
// activation bit width, -DQNN_AB=<1..8>.
//
//   im2col_pack_kernel   codes NHWC -> words [pixel][AB]: bit t*C + c of word p is digit p of
//                        u = (v + 2^AB - 1)/2 of tap t = (kh, kw), channel c; bits of taps
//                        outside the image are 0.
//   conv_small_kernel    lane = filter; the pixel's AB words arrive through scalar loads (two
//                        buffers, hand-placed wait, as in qnn_branch.hip); per branch one
//                        v_xor_b32 + v_bcnt_u32_b32.  Zero padding: for a border pixel the xor is
//                        masked with the pixel's valid-tap mask (one extra v_and_b32 per branch)
//                        and the constant term uses the number of valid bits.
#include "qnn_internal.h"
#include "qnn_device_util.h"

#ifndef QNN_AB
#error "compile with -DQNN_AB=<activation bits>"
#endif

namespace qnn {
namespace {

template <typename CodeT, int BITS>
__global__ __launch_bounds__(256) void im2col_pack_kernel(const CodeT *__restrict__ codes, int64_t pixels,
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
    const int C = g.C;

    // the filter's 9*C-bit word per weight plane, assembled from the per-tap words
    uint32_t wq[WB];
    {
        uint32_t taps[9 * WB];                         // the filter's words are contiguous: [tap][plane]
        load_run<9 * WB>(g.Wt + nload * 9 * WB, taps);
#pragma unroll
        for (int q = 0; q < WB; ++q) {
            wq[q] = 0u;
#pragma unroll
            for (int t = 0; t < 9; ++t) wq[q] |= taps[t * WB + q] << (t * C);
        }
    }
    // valid-tap masks
    const uint32_t tapbits = (1u << C) - 1u;
    uint32_t rowmask[3], colmask[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        rowmask[k] = (tapbits << ((3 * k) * C)) | (tapbits << ((3 * k + 1) * C)) | (tapbits << ((3 * k + 2) * C));
        colmask[k] = (tapbits << (k * C)) | (tapbits << ((k + 3) * C)) | (tapbits << ((k + 6) * C));
    }
    const uint32_t full = rowmask[0] | rowmask[1] | rowmask[2];

    const OV ov = make_out_view<OV>(g, r0, r1, nload, sc, ct);

    int ow, oh, line0, img0;
    fast_divmod((uint32_t)r0, g.div_w, line0, ow);
    fast_divmod((uint32_t)line0, g.div_h, img0, oh);
    const uint64_t base = (uint64_t)g.A;
    constexpr uint32_t kPixelBytes = AB * 4u;
    SRun<AB> bufA, bufB;                                   // the pixel's AB consecutive words, in SGPRs
    bufA.template request<0>(base, (uint32_t)r0 * kPixelBytes);

    int r = r0;
    // Pixels from here on that are known to see all nine taps: in an image row that is neither the
    // first nor the last, everything between the first and the last column.  While the count runs,
    // a pixel costs no mask work at all; at 0 the masks are worked out from (oh, ow).
    int full_left = 0;
    const int kfull = __builtin_popcount(full) * g.kconst;
    auto one_pixel = [&](SRun<AB> &cur, SRun<AB> &nxt) {
        cur.template arrive<true>();
        const int rn = (r + 1 < r1) ? r + 1 : r;           // the last pixel prefetches itself (unused)
        nxt.template request<0>(base, (uint32_t)rn * kPixelBytes);
        int part[AB + WB - 1];                             // part[s]: branches with p + q = s
        uint32_t m = full;
        auto add_branches = [&](auto masked) {
#pragma unroll
            for (int q = 0; q < WB; ++q)
#pragma unroll
                for (int p = 0; p < AB; ++p) {
                    uint32_t x = cur.get(p) ^ wq[q];
                    if constexpr (decltype(masked)::value) x &= m;
                    if (q == 0 || p == AB - 1) popc_set(part[p + q], x);   // first branch of its sum
                    else popc_acc(part[p + q], x);
                }
        };
        int konst = kfull;
        if (full_left > 0) {
            --full_left;
            ++ow;                                          // stays below W - 1 while the count runs
            add_branches(std::false_type());
        } else {
            if (oh == 0) m &= ~rowmask[0];
            if (oh == g.H - 1) m &= ~rowmask[2];
            if (ow == 0) m &= ~colmask[0];
            if (ow == g.W - 1) m &= ~colmask[2];
            if (m == full) {
                add_branches(std::false_type());
            } else {
                add_branches(std::true_type());
                konst = __builtin_popcount(m) * g.kconst;   // kconst = (2^AB-1)(2^WB-1) per element
            }
            if (++ow == g.W) {
                ow = 0;
                if (++oh == g.H) oh = 0;
            }
            if (oh > 0 && oh < g.H - 1 && ow >= 1 && ow < g.W - 1) full_left = g.W - 1 - ow;   // columns ow .. W-2
        }
        int sum = part[AB + WB - 2];
#pragma unroll
        for (int i = AB + WB - 3; i >= 0; --i) sum = (sum << 1) + part[i];
        finish_row<true>(ov, r - r0, konst - 2 * sum, true, true);
        ++r;
    };
    while (r + 1 < r1) {
        one_pixel(bufA, bufB);
        one_pixel(bufB, bufA);
    }
    if (r < r1) one_pixel(bufA, bufB);
    bufA.template arrive<true>();                          // drain the last prefetch
    bufB.template arrive<false>();
}

template <int AB, int WB>
hipError_t launch_small_t(const BranchArgs &g, hipStream_t s) {
    const int64_t row_blocks = ((int64_t)g.rows + g.rows_per_wave - 1) / g.rows_per_wave;
    const int64_t waves = row_blocks * g.col_tiles;
    const dim3 grid((unsigned)((waves + 3) / 4));
    if (g.xcd_ranges && g.grid_blocks != grid.x) return hipErrorInvalidValue;             // host bug
    if (g.planes_out != nullptr) hipLaunchKernelGGL((conv_small_kernel<AB, WB, true>), grid, dim3(256), 0, s, g);
    else hipLaunchKernelGGL((conv_small_kernel<AB, WB, false>), grid, dim3(256), 0, s, g);
    return hipGetLastError();
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
    const int64_t want = (pixels + 255) / 256;
    const unsigned blocks = (unsigned)(want < (int64_t)1 << 20 ? want : (int64_t)1 << 20);
    if (code_bytes == 1)
        hipLaunchKernelGGL((im2col_pack_kernel<int8_t, QNN_AB>), dim3(blocks), dim3(256), 0, s,
                           (const int8_t *)codes, pixels, H, W, C, words);
    else
        hipLaunchKernelGGL((im2col_pack_kernel<int16_t, QNN_AB>), dim3(blocks), dim3(256), 0, s,
                           (const int16_t *)codes, pixels, H, W, C, words);
    return hipGetLastError();
}

}  // namespace qnn
