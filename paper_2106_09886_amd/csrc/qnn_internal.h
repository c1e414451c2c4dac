// Internal declarations shared by the translation units of libqnn (not installed).
#pragma once
#include <atomic>
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <tuple>
#include <type_traits>
#include <utility>
#include "qnn.h"

namespace qnn {

// Kernel launches.  launch_kernel starts `kernel` on `stream` and keeps the status that the launch
// call itself returned (the first failure since the last launch_status()); launch_status() hands
// it out and clears it.  The runtime's per-thread "last error" is not consulted: an error left
// there by an unrelated call of the host program would otherwise be reported as this library's.
inline thread_local hipError_t t_launch_error = hipSuccess;

template <typename... KArgs, size_t... I>
inline hipError_t launch_held(const void *kernel, dim3 grid, dim3 block, unsigned lds_bytes, hipStream_t stream,
                              std::tuple<KArgs...> &held, std::index_sequence<I...>) {
    void *ptrs[sizeof...(KArgs) + 1] = {static_cast<void *>(&std::get<I>(held))..., nullptr};
    return hipLaunchKernel(kernel, grid, block, ptrs, lds_bytes, stream);
}

template <typename... KArgs, typename... Args>
inline void launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, unsigned lds_bytes, hipStream_t stream,
                          const Args &...args) {
    static_assert(sizeof...(KArgs) == sizeof...(Args), "one value per kernel parameter");
    std::tuple<std::remove_cv_t<KArgs>...> held(args...);   // values of exactly the parameters' types
    const hipError_t e = launch_held(reinterpret_cast<const void *>(kernel), grid, block, lds_bytes, stream, held,
                                     std::index_sequence_for<KArgs...>{});
    if (e != hipSuccess && t_launch_error == hipSuccess) t_launch_error = e;
}

inline hipError_t launch_status() {
    const hipError_t e = t_launch_error;
    t_launch_error = hipSuccess;
    return e;
}

// Window geometry of the general convolution kernel (all run-time values).
struct ConvGeom {
    int KH, KW;           // kernel size
    int sh, sw;           // stride
    int ph, pw;           // zero padding
    int dh, dw;           // dilation
    int Ho, Wo;           // output image size
    int transposed;       // 0: convolution, 1: transposed convolution
};

// Division of a wave-uniform number n < 2^31 by a launch constant d >= 1 without the vector ALU
// (there is no integer divide instruction; the compiler's expansion is some 25 vector
// instructions per division, and a wavefront's set-up has four of them).  The host prepares
// m = ceil(2^(31+L) / d), L = ceil(log2 d); then n / d = (n * m) >> (31 + L) exactly, because the
// error n * (m*d - 2^(31+L)) stays below 2^(31+L) for n < 2^31.  The kernel needs one
// s_mul_hi_u32 and a shift.  d = 1 is coded as m = 0.
struct FastDiv {
    uint32_t d, m, sh;
};
inline FastDiv fast_div_for(int64_t d_in) {
    FastDiv f;
    const uint64_t d = d_in < 1 ? 1 : (uint64_t)d_in;
    f.d = (uint32_t)d;
    if (d == 1) { f.m = 0; f.sh = 0; return f; }
    int L = 0;
    while (((uint64_t)1 << L) < d) ++L;                        // L = ceil(log2 d) >= 1
    const uint64_t two_k = (uint64_t)1 << (31 + L);            // d < 2^31, so L <= 31
    f.m = (uint32_t)((two_k + d - 1) / d);                     // < 2^32 (= 2^31 for a power of two)
    f.sh = (uint32_t)(L - 1);                                  // after taking the high word
    return f;
}

// Arguments of the branch kernels (GEMM and 3x3 convolution).  All sizes were range
// checked on the host; index arithmetic inside the kernels is 32-bit except for the
// row base of the outputs.
struct BranchArgs {
    const uint32_t *A;    // activation planes [rows][AB][Cw]
    const uint32_t *Wt;   // weight planes     [N][taps][WB][Cw]   (taps = 1 for GEMM)
    int32_t *acc;         // int32 out [rows][N] or nullptr
    const float *scale;   // fp32 [N] or nullptr
    float *out;           // fp32 out [rows][N] or nullptr
    int32_t *partial;     // where partial sums of a multi-chunk product live (acc, else out)
    uint32_t out_flags;   // bit 0: acc != nullptr, bit 1: out != nullptr (the kernels test this word on the
                          // scalar unit instead of comparing the pointers)
    int rows;             // GEMM rows / output pixels
    int N;                // output columns / filters
    int Cw;               // words per (row, plane)
    int H, W;             // image height and width in pixels (convolution only)
    int C;                // input channels (small-channel convolution only)
    int kconst;           // (true K of one tap) * (2^AB - 1) * (2^WB - 1)
    int rows_per_wave;    // contiguous rows handled by one wavefront
    int col_tiles;        // ceil(N / 64)
    int split_k;          // K (GEMM) or channel (3x3 convolution) chunks split over the four wavefronts of a
                          // block; then rows_per_wave is the number of rows per BLOCK
    int gather_rows;      // GEMM only: row r is output pixel r of a single-tap strided convolution (geo, H, W);
                          // bit widths up to 4, not with split_k
    int lds_partials;     // GEMM only: partial sums between chunk passes stay in LDS (rows_per_wave <=
                          // kLdsPartialRows, bit widths up to 4, not with split_k or gather_rows)
    int xcd_ranges;       // convolution kernels: number the blocks so that each XCD takes one contiguous range
    unsigned grid_blocks; // blocks of the launch (wave_grid_blocks), read by the kernels when xcd_ranges is set
    uint64_t *trace;      // optional per-wavefront trace records (4 x uint64 each), or nullptr
    uint32_t trace_waves; // capacity of `trace` in wavefronts
    uint32_t *planes_out; // optional: the scaled result re-encoded with out_bits bits, as bit planes
                          // uint32 [rows][out_bits][ceil(N/32)] (the next layer's activations)
    int out_bits;
    ConvGeom geo;         // general convolution only
    FastDiv div_tiles;    // col_tiles
    FastDiv div_w, div_h; // W and H (3x3 convolution), Wo and Ho (general convolution, strided rows)
};
// fills the division constants from the fields they belong to (call last, before the launch)
inline void set_divisors(BranchArgs &g, bool output_image = false) {
    g.div_tiles = fast_div_for(g.col_tiles);
    g.div_w = fast_div_for(output_image ? g.geo.Wo : g.W);
    g.div_h = fast_div_for(output_image ? g.geo.Ho : g.H);
}

constexpr int kLdsPartialRows = 24;   // rows per wavefront whose partial sums the GEMM kernel keeps in LDS

// Blocks of four wavefronts in a launch that gives one wavefront to every (row block, column tile).
inline unsigned wave_grid_blocks(const BranchArgs &g) {
    const int64_t row_blocks = ((int64_t)g.rows + g.rows_per_wave - 1) / g.rows_per_wave;
    return (unsigned)((row_blocks * g.col_tiles + 3) / 4);
}

// Process-wide knobs behind qnn_tune and qnn_set_trace.  Each is an atomic of its own: a launch reads
// every knob it uses once, while it sizes its grid, so a change made from another thread takes
// effect at a call boundary of the calls that start later and never tears a value.
struct Tuning {
    std::atomic<int> waves_per_simd{0};   // target resident wavefronts per SIMD when sizing rows_per_wave
    std::atomic<int> rows_per_wave{0};    // > 0 overrides the automatic choice
    std::atomic<uint64_t *> trace{nullptr};  // device buffer for per-wavefront trace records, or nullptr
    std::atomic<uint32_t> trace_waves{0};
    std::atomic<int> general_only{0};     // qnn_conv2d_general hands no 3x3 pad-1 window to the 3x3 kernel
    std::atomic<int> block_order{0};      // 0: automatic, 1: plain block numbers, 2: a contiguous range per XCD
    std::atomic<int> lds_partials{0};     // 0: automatic, 1: GEMM partial sums through the output buffer, 2: in LDS where possible
    std::atomic<int> split_channels{0};   // 3x3 convolution: 0 automatic, 1 never split the channel chunks over a block, 2 wherever possible
};
Tuning &tuning();

int device_simd_count();  // 4 * number of compute units of the current device (cached)
// K words per weight chunk of the GEMM kernels (GemmShape::KC in qnn_branch.hip)
inline int gemm_chunk_words(int wb) { return (wb == 1) ? 64 : (wb == 2) ? 32 : (wb <= 4) ? 16 : 8; }

// Chunk shape of the convolution kernels with a compile-time plane stride cws (a power of two
// up to 16; bit widths up to 4).  A chunk is cwt channel words x tpc taps; its weight words
// (tpc*wb*cwt) must leave room in the VGPR file for several wavefronts per SIMD (<= 80), one
// pipeline stage gt*ab*cwt must fit the SGPR budget twice (<= 32), and among the shapes that fit
// the one with the most work per chunk pass (cwt*tpc) wins, so that the round trip of partial
// sums is paid least often.  gt: taps per pipeline stage; p: output pixels per loop iteration.
struct ConvShapeV {
    int cwt, tpc, gt, p;
};
constexpr int conv_pow2_floor(int x) { return x >= 16 ? 16 : x >= 8 ? 8 : x >= 4 ? 4 : x >= 2 ? 2 : 1; }
constexpr int conv_shape_score(int ab, int wb, int cws, int cwt, int tpc) {
    const int cmax = cws < conv_pow2_floor(32 / ab) ? cws : conv_pow2_floor(32 / ab);
    return (cwt <= cmax && tpc * wb * cwt <= (wb >= 5 ? 96 : 80)) ? cwt * tpc : 0;
}
constexpr ConvShapeV conv_shape(int ab, int wb, int cws) {
    int bc = 1, bs = 0;
    for (int cwt = 1; cwt <= cws; cwt *= 2)
        for (int tpc = 1; tpc <= 9; tpc *= 3) {
            const int sc = conv_shape_score(ab, wb, cws, cwt, tpc);
            if (sc > bs || (sc == bs && bs > 0 && cwt > bc)) { bs = sc; bc = cwt; }
        }
    int bt = 1;
    bs = 0;
    for (int tpc = 1; tpc <= 9; tpc *= 3) {
        const int sc = conv_shape_score(ab, wb, cws, bc, tpc);
        if (sc > bs) { bs = sc; bt = tpc; }
    }
    const int gt = (bt >= 3 && bc == cws && 3 * ab * bc <= 24) ? 3 : 1;
    const bool groups = (gt == 3 && bt == 9 && bc == cws);
    // pixels per iteration: as many as keep one stage ((p+2) pixels) within 16 SGPRs
    const int p = !groups ? 1 : (6 * ab * bc <= 16) ? 4 : (4 * ab * bc <= 16) ? 2 : 1;
    return ConvShapeV{bc, bt, gt, p};
}
static_assert(conv_shape(2, 2, 2).cwt == 2 && conv_shape(2, 2, 2).tpc == 9 && conv_shape(2, 2, 2).gt == 3 &&
              conv_shape(2, 2, 2).p == 2, "ResNet-18 stage-1 shape: whole product in one pass, pixel pairs");
static_assert(conv_shape(4, 3, 8).cwt == 8 && conv_shape(4, 3, 8).tpc == 3, "ResNet-50 stage-3 shape: one kernel row per pass");
static_assert(conv_shape(4, 2, 16).cwt == 4 && conv_shape(4, 2, 16).tpc == 9, "512-channel W2A4: four passes of nine taps");
// Does the convolution launcher have an instantiation with this compile-time plane stride?  Bit
// widths up to 4 x 4, plus the wider pairs of the paper's mixed-precision tables (Table 4: 4-bit
// activations with 5- and 6-bit weights; 8-bit activations with 6- to 8-bit weights): a bounded
// list, to bound build time.  (Weight widths from 5 bits on may use 96 instead of 80 weight
// registers per chunk, so that a 64-channel layer with 5-bit weights keeps all nine taps.)
constexpr bool conv_has_fixed_widths(int ab, int wb) {
    return (ab <= 4 && wb <= 6) || (ab == 8 && wb >= 6);
}
constexpr bool conv_has_fixed_shape(int ab, int wb, int cw) {
    return conv_has_fixed_widths(ab, wb) && (cw == 1 || cw == 2 || cw == 4 || cw == 8 || cw == 16);
}
// chunk passes a wavefront makes over its pixels
constexpr int conv_passes(int ab, int wb, int cw) {
    if (cw <= 0) return 1;
    if (conv_has_fixed_shape(ab, wb, cw)) {
        const ConvShapeV v = conv_shape(ab, wb, cw);
        return (cw / v.cwt) * (9 / v.tpc);
    }
    // the runtime-stride kernels: chunks of four words where they divide the plane (up to W2A4), else two, else one
    const int cwt = (ab <= 4 && wb <= 2 && cw % 4 == 0) ? 4 : (cw == 1 || ab > 4) ? 1 : 2;
    return (cw + cwt - 1) / cwt;
}

// output pixels the convolution kernel takes per loop iteration
constexpr int conv_group(int ab, int wb, int cw) {
    return conv_has_fixed_shape(ab, wb, cw) ? conv_shape(ab, wb, cw).p : 1;
}

// Chunk shape of the variant of the 3x3 kernel whose four wavefronts per block split the channel
// chunks: all nine taps per chunk, and channel words per chunk such that the chunks divide evenly
// among the four wavefronts (a quarter of the plane, or less if nine taps of that many words do not
// fit the weight registers).  It exists for the fixed shapes with at least four channel words whose
// plain kernel makes more than one pass.
constexpr ConvShapeV conv_split_shape(int ab, int wb, int cws) {
    int cwt = cws / 4;
    while (cwt >= 1 && conv_shape_score(ab, wb, cws, cwt, 9) == 0) cwt /= 2;
    return ConvShapeV{cwt, 9, 1, 1};
}
constexpr bool conv_can_split(int ab, int wb, int cw) {
    return conv_has_fixed_shape(ab, wb, cw) && cw >= 4 && conv_split_shape(ab, wb, cw).cwt >= 1 &&
           (cw / conv_shape(ab, wb, cw).cwt) * (9 / conv_shape(ab, wb, cw).tpc) >= 2;
}
static_assert(conv_split_shape(4, 2, 16).cwt == 4 && conv_split_shape(4, 2, 8).cwt == 2 && conv_split_shape(4, 3, 8).cwt == 2,
              "512- and 256-channel W2A4 and the ResNet-50 stage-3 shape: four chunks of nine taps");
constexpr int kConvSplitRows = 16;
// Fixed shapes of the 3x3 kernel that also serve other odd windows with "same" padding at stride 1
// (atrous 3x3, 5x5, 7x7, 1x3 ...): one tap per pipeline stage, one pixel per iteration, and a stage
// of at most 16 scalar registers -- with 32 the second copy of the chunk loop leaves the compiler
// too few scalar registers and it spills stage registers whose load is in flight (the static check
// of the generated code finds exactly those).  Separately for the plain variant and for the one
// whose four wavefronts per block split the channel chunks; the host takes whichever exists.
constexpr bool conv_wide_stage_ok(int ab, int cwt) { return ab * cwt <= 16; }
constexpr bool conv_wide_plain_ok(int ab, int wb, int cw) {
    return conv_has_fixed_shape(ab, wb, cw) && conv_shape(ab, wb, cw).gt == 1 && conv_shape(ab, wb, cw).p == 1 &&
           conv_wide_stage_ok(ab, conv_shape(ab, wb, cw).cwt);
}
constexpr bool conv_wide_split_ok(int ab, int wb, int cw) {
    return conv_can_split(ab, wb, cw) && conv_wide_stage_ok(ab, conv_split_shape(ab, wb, cw).cwt);
}
// Shapes (64 to 256 channels) whose 3x3 kernel holds several taps or pixels per stage, and no split
// variant either: other windows get an instantiation of their own there, with one tap of as many
// channel words per stage as fit it (bit widths up to 4 x 4, to bound build time)
constexpr ConvShapeV conv_wide_extra_shape(int ab, int wb, int cws) {
    int cwt = cws;
    while (cwt >= 1 && (!conv_wide_stage_ok(ab, cwt) || conv_shape_score(ab, wb, cws, cwt, 9) == 0)) cwt /= 2;
    return ConvShapeV{cwt, 9, 1, 1};
}
constexpr bool conv_wide_extra_ok(int ab, int wb, int cw) {
    return (cw == 2 || cw == 4 || cw == 8) && ab <= 4 && wb <= 4 && conv_has_fixed_shape(ab, wb, cw) &&
           !conv_wide_plain_ok(ab, wb, cw) && !conv_wide_split_ok(ab, wb, cw) && conv_wide_extra_shape(ab, wb, cw).cwt >= 1;
}
constexpr int conv_wide_extra_passes(int ab, int wb, int cw) { return cw / conv_wide_extra_shape(ab, wb, cw).cwt; }

// the same for the stride-2 variant of the 3x3 kernel: two output pixels share a stage of five input
// pixels where those fit the scalar registers of a stage, else one pixel per iteration
constexpr int conv_group_strided(int ab, int wb, int cw) {
    return (conv_has_fixed_shape(ab, wb, cw) && conv_shape(ab, wb, cw).p >= 2 && 5 * ab * conv_shape(ab, wb, cw).cwt <= 20) ? 2 : 1;
}

// Launchers, one translation unit per activation bit width AB (1..8).
typedef hipError_t (*branch_launch_fn)(const BranchArgs &, int wb, hipStream_t);
hipError_t launch_gemm_ab1(const BranchArgs &, int, hipStream_t);
hipError_t launch_gemm_ab2(const BranchArgs &, int, hipStream_t);
hipError_t launch_gemm_ab3(const BranchArgs &, int, hipStream_t);
hipError_t launch_gemm_ab4(const BranchArgs &, int, hipStream_t);
hipError_t launch_gemm_ab5(const BranchArgs &, int, hipStream_t);
hipError_t launch_gemm_ab6(const BranchArgs &, int, hipStream_t);
hipError_t launch_gemm_ab7(const BranchArgs &, int, hipStream_t);
hipError_t launch_gemm_ab8(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_ab1(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_ab2(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_ab3(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_ab4(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_ab5(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_ab6(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_ab7(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_ab8(const BranchArgs &, int, hipStream_t);

hipError_t launch_conv_general_ab1(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_general_ab2(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_general_ab3(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_general_ab4(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_general_ab5(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_general_ab6(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_general_ab7(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_general_ab8(const BranchArgs &, int, hipStream_t);

hipError_t launch_conv_window_ab1(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_window_ab2(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_window_ab3(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_window_ab4(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_window_ab5(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_window_ab6(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_window_ab7(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_window_ab8(const BranchArgs &, int, hipStream_t);
hipError_t launch_window_pack(const uint32_t *planes, int64_t out_pixels, const ConvGeom &q, int H, int W, int C,
                              int ab, int kwp, bool dense_rows, uint32_t *out, hipStream_t s);
// words per plane of a packed window of `bits` = KH*KW*C bits (the instantiated sizes), 0 if none fits
inline int window_words(int64_t bits) {
    return bits <= 32 ? 1 : bits <= 64 ? 2 : bits <= 96 ? 3 : bits <= 160 ? 5 : bits <= 256 ? 8 : 0;
}

hipError_t launch_conv_small_ab1(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_small_ab2(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_small_ab3(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_small_ab4(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_small_ab5(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_small_ab6(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_small_ab7(const BranchArgs &, int, hipStream_t);
hipError_t launch_conv_small_ab8(const BranchArgs &, int, hipStream_t);
hipError_t launch_im2col_pack_ab1(const void *, int, int64_t, int, int, int, uint32_t *, hipStream_t);
hipError_t launch_im2col_pack_ab2(const void *, int, int64_t, int, int, int, uint32_t *, hipStream_t);
hipError_t launch_im2col_pack_ab3(const void *, int, int64_t, int, int, int, uint32_t *, hipStream_t);
hipError_t launch_im2col_pack_ab4(const void *, int, int64_t, int, int, int, uint32_t *, hipStream_t);
hipError_t launch_im2col_pack_ab5(const void *, int, int64_t, int, int, int, uint32_t *, hipStream_t);
hipError_t launch_im2col_pack_ab6(const void *, int, int64_t, int, int, int, uint32_t *, hipStream_t);
hipError_t launch_im2col_pack_ab7(const void *, int, int64_t, int, int, int, uint32_t *, hipStream_t);
hipError_t launch_im2col_pack_ab8(const void *, int, int64_t, int, int, int, uint32_t *, hipStream_t);
typedef hipError_t (*im2col_launch_fn)(const void *, int, int64_t, int, int, int, uint32_t *, hipStream_t);

hipError_t launch_pack(const void *codes, int code_bytes, int64_t rows, int64_t K, int bits,
                       uint32_t *planes, int32_t *bad_count, bool validate, hipStream_t);
hipError_t launch_requant(const float *y, int64_t Nb, int64_t H, int64_t W, int64_t C, bool pool, int bits,
                          float premul, int clip, void *codes, uint32_t *planes, hipStream_t);
hipError_t launch_encoder_backward(const float *x, const float *g, int64_t n, int bits, float *gx, hipStream_t);
hipError_t launch_binarize(const float *w, int64_t rows, int64_t K, int8_t *codes, uint32_t *planes, hipStream_t);
hipError_t launch_binarize_backward(const float *w, const float *g_wb, int64_t n, float *g_w, hipStream_t);
hipError_t launch_quantize_k(const float *x, int64_t n, int bits, float t, float *q, int32_t *levels, hipStream_t);
hipError_t launch_quantize_k_backward(const float *x, const float *g_q, int64_t n, float t, float *g_x, hipStream_t);
// backward lines of Alg. 1 through the product: out[p][r][c] = 2^p sum_j G(r, j) code[j][c] (qnn_backward.hip)
hipError_t launch_backward_gemm(const float *g, int64_t ldg, const float *scale, const uint32_t *planes, int code_bits,
                                int R, int J, int C, int P, bool towards_weights, float *out, hipStream_t);
// the same through a 3x3 / stride 1 / pad 1 convolution; the weight gradient goes through a workspace of
// conv_backward_splits() partial results
int conv_backward_splits(int64_t pixels, int64_t O, int64_t C);
hipError_t launch_conv_backward_input(const float *g, const float *scale, const uint32_t *Wt, int wb, int64_t Nb, int H, int W,
                                      int C, int O, int P, float *out, hipStream_t);
hipError_t launch_conv_backward_weight(const float *g, const float *scale, const uint32_t *x_planes, int ab, int64_t Nb, int H,
                                       int W, int C, int O, int P, float *out, float *workspace, hipStream_t);
hipError_t launch_update_sgd(float *w, const float *g, int64_t n, float lr, hipStream_t);
hipError_t launch_update_adam(float *w, const float *g, float *m, float *v, int64_t n, float lr, float b1, float b2,
                              float omb1, float omb2, float bc1, float bc2, float eps, hipStream_t);
hipError_t launch_pool_planes(const uint32_t *planes, int64_t Nb, int64_t Ho, int64_t Wo, int64_t Cw, int bits,
                              uint32_t *out, hipStream_t);
hipError_t launch_mfma_arrange(const int8_t *codes, int64_t rows, int64_t K, void *out, hipStream_t);
hipError_t launch_mfma_gemm(const void *A, const void *B, int64_t M, int64_t N, int64_t K, int32_t *C, hipStream_t);
hipError_t launch_dot4_gemm(const int8_t *A, const int8_t *Wt, int64_t M, int64_t N, int64_t K, int32_t *C,
                            hipStream_t s);
hipError_t launch_scale(const int32_t *acc, int64_t total, int64_t N, const float *scale,
                        float *out, hipStream_t);

}  // namespace qnn
