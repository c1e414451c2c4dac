// Multi-branch binary product kernels (paper Eq. (8)): GEMM and implicit-im2col 3x3
// convolution.  Compiled once per activation bit width, -DQNN_AB=<1..8>.
//
// Mapping (gfx950, 64-lane wavefronts).  A wavefront owns 64 output columns (lane = column
// / filter) and a contiguous run of rows (GEMM rows or output pixels):
//   * the weight words of the lane's column for the current K chunk stay in VGPRs;
//   * the activation words of the current row are the same for all 64 lanes, so they are
//     fetched with scalar loads and used as the SGPR operand of v_xor_b32;
//   * per 32 binary products and branch the loop issues exactly v_xor_b32 +
//     v_bcnt_u32_b32 (popcount with fused accumulate);
//   * branches with equal p+q share an accumulator; the 2^(p+q) weights are applied once
//     per row and chunk with AB+WB-2 shift-adds (Eq. (8) regrouped by p+q);
//   * stores are lane-contiguous: one 256-byte segment per row and wavefront.
// A product whose K extent does not fit the VGPR chunk is done in several chunk passes by
// the same wavefront; partial sums round-trip through the output buffer (same lane, same
// address, program order).
#include "qnn_internal.h"

#ifndef QNN_AB
#error "compile with -DQNN_AB=<activation bits>"
#endif

namespace qnn {
namespace {

// Scalar (wave-uniform) read-only view of global memory: loads through this pointer type
// with a uniform index are selected as s_load_dword*.
typedef const uint32_t __attribute__((address_space(4))) *uniform_words;

__device__ __forceinline__ uniform_words as_uniform(const uint32_t *p) {
    return (uniform_words)(uint64_t)p;
}

// part += popcount(x): v_bcnt_u32_b32 with its add operand.  Written as asm so that the
// accumulate chain is not re-associated into separate popcounts and three-input adds.
__device__ __forceinline__ void popc_acc(int &part, uint32_t x) {
    asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(part) : "v"(x));
}

// One segment of CWT words: all AB*WB plane pairs; pairs with equal p+q share part[p+q].
template <int AB, int WB, int CWT>
__device__ __forceinline__ void seg_accum(const uint32_t (&a)[AB][CWT],
                                          const uint32_t (&w)[WB][CWT],
                                          int (&part)[AB + WB - 1]) {
#pragma unroll
    for (int q = 0; q < WB; ++q)
#pragma unroll
        for (int p = 0; p < AB; ++p)
#pragma unroll
            for (int j = 0; j < CWT; ++j) popc_acc(part[p + q], a[p][j] ^ w[q][j]);
}

// S = sum_s 2^s part[s]  (Eq. (8) weights, grouped by s = p + q)
template <int NP>
__device__ __forceinline__ int weighted_sum(const int (&part)[NP]) {
    int s = part[NP - 1];
#pragma unroll
    for (int i = NP - 2; i >= 0; --i) s = (s << 1) + part[i];
    return s;
}

// Finish one row of one chunk pass for this lane's column.
__device__ __forceinline__ void finish_row(const BranchArgs &g, int64_t row, int n, bool n_ok,
                                           int val, bool first, bool last, float sc) {
    const int64_t base = row * (int64_t)g.N;
    if (!n_ok) return;
    if (!first) val += (g.partial + base)[n];
    if (!last) {
        (g.partial + base)[n] = val;
    } else {
        if (g.acc) (g.acc + base)[n] = val;
        if (g.out) (g.out + base)[n] = (float)val * sc;
    }
}

__device__ __forceinline__ int wave_index() {
    return __builtin_amdgcn_readfirstlane((int)(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)));
}

// ---------------------------------------------------------------------------------------
// GEMM: acc[i][n] = sum_{p,q} 2^(p+q) (K - 2 popc(A[i][p] ^ Wt[n][q]))
// Chunk = SEGS segments of CWT words.  GUARD = the chunk may run past Kw (tail chunk).
// ---------------------------------------------------------------------------------------
template <int AB, int WB, int SEGS, int CWT, bool GUARD>
__device__ __forceinline__ void gemm_chunk(const BranchArgs &g, uniform_words As, int n, int nload,
                                           bool n_ok, int r0, int r1, int k0, bool first,
                                           bool last, float sc) {
    const int Kw = g.Cw;
    uint32_t w[SEGS][WB][CWT];
#pragma unroll
    for (int t = 0; t < SEGS; ++t)
#pragma unroll
        for (int q = 0; q < WB; ++q)
#pragma unroll
            for (int j = 0; j < CWT; ++j) {
                const int k = k0 + t * CWT + j;
                if (!GUARD || k < Kw) w[t][q][j] = g.Wt[(nload * WB + q) * Kw + k];
                else w[t][q][j] = 0u;
            }
    for (int r = r0; r < r1; ++r) {
        int part[AB + WB - 1];
#pragma unroll
        for (int s = 0; s < AB + WB - 1; ++s) part[s] = 0;
#pragma unroll
        for (int t = 0; t < SEGS; ++t) {
            uint32_t a[AB][CWT];
#pragma unroll
            for (int p = 0; p < AB; ++p)
#pragma unroll
                for (int j = 0; j < CWT; ++j) {
                    const int k = k0 + t * CWT + j;
                    if (!GUARD || k < Kw) a[p][j] = As[(r * AB + p) * Kw + k];
                    else a[p][j] = 0u;
                }
            seg_accum<AB, WB, CWT>(a, w[t], part);
        }
        int val = -2 * weighted_sum(part);
        if (first) val += g.kconst;
        finish_row(g, r, n, n_ok, val, first, last, sc);
    }
}

template <int AB, int WB, int SEGS, int CWT>
__global__ __launch_bounds__(256) void gemm_kernel(const BranchArgs g) {
    const int wave = wave_index();
    const int ct = wave % g.col_tiles;
    const int rb = wave / g.col_tiles;
    const int r0 = rb * g.rows_per_wave;
    if (r0 >= g.rows) return;
    const int r1 = min(g.rows, r0 + g.rows_per_wave);
    const int n = ct * 64 + (int)(threadIdx.x & 63);
    const bool n_ok = n < g.N;
    const int nload = n_ok ? n : g.N - 1;
    const float sc = (g.scale != nullptr) ? g.scale[nload] : 1.0f;
    uniform_words As = as_uniform(g.A);
    constexpr int KC = SEGS * CWT;
    const int Kw = g.Cw;
    if (Kw == 0) {  // K == 0: every product is the empty sum
        for (int r = r0; r < r1; ++r) finish_row(g, r, n, n_ok, 0, true, true, sc);
        return;
    }
    for (int k0 = 0; k0 < Kw; k0 += KC) {
        const bool first = (k0 == 0);
        const bool last = (k0 + KC >= Kw);
        if (k0 + KC <= Kw)
            gemm_chunk<AB, WB, SEGS, CWT, false>(g, As, n, nload, n_ok, r0, r1, k0, first, last, sc);
        else
            gemm_chunk<AB, WB, SEGS, CWT, true>(g, As, n, nload, n_ok, r0, r1, k0, first, last, sc);
    }
}

// ---------------------------------------------------------------------------------------
// 3x3 convolution, stride 1, pad 1.  Rows are output pixels in NHWC order; the K axis of a
// pixel is the nine neighbouring pixels' plane words, never materialised.  A chunk is a block
// of CWT channel words of all nine taps.  Taps outside the image are skipped (the pixel is
// wave-uniform, so this is a scalar branch) and the constant term uses the count of valid taps.
// ---------------------------------------------------------------------------------------
template <int AB, int WB, int CWT, bool GUARD>
__device__ __forceinline__ void conv_chunk(const BranchArgs &g, uniform_words As, int n, int nload,
                                           bool n_ok, int r0, int r1, int c0, bool first,
                                           bool last, float sc) {
    const int Cw = g.Cw;
    uint32_t w[9][WB][CWT];
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int q = 0; q < WB; ++q)
#pragma unroll
            for (int j = 0; j < CWT; ++j) {
                if (!GUARD || c0 + j < Cw) w[t][q][j] = g.Wt[((nload * 9 + t) * WB + q) * Cw + c0 + j];
                else w[t][q][j] = 0u;
            }
    // position of the first pixel inside its image
    int ow = r0 % g.W;
    int oh = (r0 / g.W) % g.H;
    for (int r = r0; r < r1; ++r) {
        int part[AB + WB - 1];
#pragma unroll
        for (int s = 0; s < AB + WB - 1; ++s) part[s] = 0;
        int nvalid = 0;
#pragma unroll
        for (int kh = 0; kh < 3; ++kh) {
            const bool row_ok = (kh == 0) ? (oh > 0) : (kh == 2) ? (oh < g.H - 1) : true;
            uint32_t a[3][AB][CWT];
            bool ok[3];
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                const bool col_ok = (kw == 0) ? (ow > 0) : (kw == 2) ? (ow < g.W - 1) : true;
                ok[kw] = row_ok && col_ok;
                // an invalid tap reads the centre pixel instead (always in bounds) and is skipped
                const int pix = ok[kw] ? r + (kh - 1) * g.W + (kw - 1) : r;
#pragma unroll
                for (int p = 0; p < AB; ++p)
#pragma unroll
                    for (int j = 0; j < CWT; ++j) {
                        if (!GUARD || c0 + j < Cw) a[kw][p][j] = As[(pix * AB + p) * Cw + c0 + j];
                        else a[kw][p][j] = 0u;
                    }
            }
#pragma unroll
            for (int kw = 0; kw < 3; ++kw)
                if (ok[kw]) {
                    seg_accum<AB, WB, CWT>(a[kw], w[kh * 3 + kw], part);
                    ++nvalid;
                }
        }
        int val = -2 * weighted_sum(part);
        if (first) val += nvalid * g.kconst;
        finish_row(g, r, n, n_ok, val, first, last, sc);
        if (++ow == g.W) {
            ow = 0;
            if (++oh == g.H) oh = 0;
        }
    }
}

template <int AB, int WB, int CWT>
__global__ __launch_bounds__(256) void conv_kernel(const BranchArgs g) {
    const int wave = wave_index();
    const int ct = wave % g.col_tiles;
    const int rb = wave / g.col_tiles;
    const int r0 = rb * g.rows_per_wave;
    if (r0 >= g.rows) return;
    const int r1 = min(g.rows, r0 + g.rows_per_wave);
    const int n = ct * 64 + (int)(threadIdx.x & 63);
    const bool n_ok = n < g.N;
    const int nload = n_ok ? n : g.N - 1;
    const float sc = (g.scale != nullptr) ? g.scale[nload] : 1.0f;
    uniform_words As = as_uniform(g.A);
    const int Cw = g.Cw;
    if (Cw == 0) {  // no input channels: every product is the empty sum
        for (int r = r0; r < r1; ++r) finish_row(g, r, n, n_ok, 0, true, true, sc);
        return;
    }
    for (int c0 = 0; c0 < Cw; c0 += CWT) {
        const bool first = (c0 == 0);
        const bool last = (c0 + CWT >= Cw);
        if (CWT == 1 || c0 + CWT <= Cw)
            conv_chunk<AB, WB, CWT, false>(g, As, n, nload, n_ok, r0, r1, c0, first, last, sc);
        else
            conv_chunk<AB, WB, CWT, true>(g, As, n, nload, n_ok, r0, r1, c0, first, last, sc);
    }
}

// Chunk shapes.  GEMM: the activation words of one segment (AB*CWT) must fit comfortably in
// SGPRs, the weight words of one chunk (WB*KC) in VGPRs.
template <int AB> struct GemmShape {
    static constexpr int CWT = (AB <= 2) ? 8 : (AB <= 4) ? 4 : 2;
};
template <int WB> struct GemmChunk {
    static constexpr int KC = (WB <= 2) ? 32 : (WB <= 4) ? 16 : 8;
};

inline dim3 grid_for(const BranchArgs &g) {
    const int64_t row_blocks = ((int64_t)g.rows + g.rows_per_wave - 1) / g.rows_per_wave;
    const int64_t waves = row_blocks * g.col_tiles;
    return dim3((unsigned)((waves + 3) / 4));
}

template <int AB, int WB>
hipError_t launch_gemm_t(const BranchArgs &g, hipStream_t s) {
    constexpr int CWT = GemmShape<AB>::CWT;
    constexpr int SEGS = GemmChunk<WB>::KC / CWT;
    hipLaunchKernelGGL((gemm_kernel<AB, WB, SEGS, CWT>), grid_for(g), dim3(256), 0, s, g);
    return hipGetLastError();
}

template <int AB, int WB>
hipError_t launch_conv_t(const BranchArgs &g, hipStream_t s) {
    if (g.Cw == 1)
        hipLaunchKernelGGL((conv_kernel<AB, WB, 1>), grid_for(g), dim3(256), 0, s, g);
    else
        hipLaunchKernelGGL((conv_kernel<AB, WB, 2>), grid_for(g), dim3(256), 0, s, g);
    return hipGetLastError();
}

}  // namespace

#define QNN_CAT2(a, b) a##b
#define QNN_CAT(a, b) QNN_CAT2(a, b)

hipError_t QNN_CAT(launch_gemm_ab, QNN_AB)(const BranchArgs &g, int wb, hipStream_t s) {
    switch (wb) {
        case 1: return launch_gemm_t<QNN_AB, 1>(g, s);
        case 2: return launch_gemm_t<QNN_AB, 2>(g, s);
        case 3: return launch_gemm_t<QNN_AB, 3>(g, s);
        case 4: return launch_gemm_t<QNN_AB, 4>(g, s);
        case 5: return launch_gemm_t<QNN_AB, 5>(g, s);
        case 6: return launch_gemm_t<QNN_AB, 6>(g, s);
        case 7: return launch_gemm_t<QNN_AB, 7>(g, s);
        case 8: return launch_gemm_t<QNN_AB, 8>(g, s);
    }
    return hipErrorInvalidValue;
}

hipError_t QNN_CAT(launch_conv_ab, QNN_AB)(const BranchArgs &g, int wb, hipStream_t s) {
    switch (wb) {
        case 1: return launch_conv_t<QNN_AB, 1>(g, s);
        case 2: return launch_conv_t<QNN_AB, 2>(g, s);
        case 3: return launch_conv_t<QNN_AB, 3>(g, s);
        case 4: return launch_conv_t<QNN_AB, 4>(g, s);
        case 5: return launch_conv_t<QNN_AB, 5>(g, s);
        case 6: return launch_conv_t<QNN_AB, 6>(g, s);
        case 7: return launch_conv_t<QNN_AB, 7>(g, s);
        case 8: return launch_conv_t<QNN_AB, 8>(g, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace qnn
