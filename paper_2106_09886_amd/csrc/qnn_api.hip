// C ABI of libqnn: argument checks on the host, then launches.  See include/qnn.h.
#include <atomic>
#include <cmath>
#include "qnn_internal.h"

// Scratch of qnn_conv2d_im2col_static: the per-pixel activation planes between its two kernels.
// One copy per GPU, held until the process ends.  In host code the array's name is only a handle
// for hipGetSymbolAddress; the kernels get the device address that call returns.
static __device__ __align__(256) unsigned char scratch[QNN_STATIC_SCRATCH_BYTES];

namespace qnn {

Tuning &tuning() {
    static Tuning t;
    return t;
}

int device_simd_count() {
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 1024;
    int v = cached[dev].load(std::memory_order_relaxed);
    if (v == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        v = 4 * cus;
        cached[dev].store(v, std::memory_order_relaxed);
    }
    return v;
}

namespace {

thread_local int g_last_hip_error = 0;

constexpr size_t kStaticScratchBytes = QNN_STATIC_SCRATCH_BYTES;
std::atomic<void *> g_scratch_ptr[64];       // per device: address of `scratch` on that GPU, once resolved

qnn_status from_hip(hipError_t e) {
    if (e == hipSuccess) return QNN_OK;
    g_last_hip_error = (int)e;
    return QNN_EHIP;
}

bool aligned16(const void *p) { return (((uintptr_t)p) & 15u) == 0; }
bool aligned4(const void *p) { return (((uintptr_t)p) & 3u) == 0; }
bool bits_ok(int b) { return b >= 1 && b <= 8; }

const branch_launch_fn k_gemm[8] = {launch_gemm_ab1, launch_gemm_ab2, launch_gemm_ab3, launch_gemm_ab4,
                                    launch_gemm_ab5, launch_gemm_ab6, launch_gemm_ab7, launch_gemm_ab8};
const branch_launch_fn k_conv[8] = {launch_conv_ab1, launch_conv_ab2, launch_conv_ab3, launch_conv_ab4,
                                    launch_conv_ab5, launch_conv_ab6, launch_conv_ab7, launch_conv_ab8};

const branch_launch_fn k_conv_general[8] = {launch_conv_general_ab1, launch_conv_general_ab2, launch_conv_general_ab3,
                                            launch_conv_general_ab4, launch_conv_general_ab5, launch_conv_general_ab6,
                                            launch_conv_general_ab7, launch_conv_general_ab8};
const branch_launch_fn k_conv_window[8] = {launch_conv_window_ab1, launch_conv_window_ab2, launch_conv_window_ab3,
                                           launch_conv_window_ab4, launch_conv_window_ab5, launch_conv_window_ab6,
                                           launch_conv_window_ab7, launch_conv_window_ab8};
const branch_launch_fn k_conv_small[8] = {launch_conv_small_ab1, launch_conv_small_ab2, launch_conv_small_ab3,
                                          launch_conv_small_ab4, launch_conv_small_ab5, launch_conv_small_ab6,
                                          launch_conv_small_ab7, launch_conv_small_ab8};
const im2col_launch_fn k_im2col[8] = {launch_im2col_pack_ab1, launch_im2col_pack_ab2, launch_im2col_pack_ab3,
                                      launch_im2col_pack_ab4, launch_im2col_pack_ab5, launch_im2col_pack_ab6,
                                      launch_im2col_pack_ab7, launch_im2col_pack_ab8};

const int64_t kInt31 = ((int64_t)1 << 31) - 1;

// Rows handled by one wavefront: enough wavefronts to give every SIMD of the chip
// `waves_per_simd` of them, but never fewer than `min_rows` rows each (the weight chunk a
// wavefront loads is reused for all of its rows).
int pick_rows_per_wave(int64_t rows, int col_tiles, int min_rows, int default_waves_per_simd = 4) {
    const int knob_rows = tuning().rows_per_wave, knob_waves = tuning().waves_per_simd;
    if (knob_rows > 0) return knob_rows;
    const int64_t target_waves = (int64_t)device_simd_count() * (knob_waves > 0 ? knob_waves : default_waves_per_simd);
    int64_t row_blocks = target_waves / col_tiles;
    if (row_blocks < 1) row_blocks = 1;
    int64_t rpw = (rows + row_blocks - 1) / row_blocks;
    if (rpw < min_rows) rpw = min_rows;
    if (rpw > rows) rpw = rows;
    if (rpw < 1) rpw = 1;
    return (int)rpw;
}

// Convolution: how many pixels one wavefront takes.  Candidates: every count up to one image
// row, and whole image rows.  Cost model, in units of one pixel of one wavefront:
//   a wavefront costs rows_per_wave + 0.22 per chunk pass (weight loads, run set-up), plus 0.3
//   per pass for the second run if it straddles two image rows, plus the pixels its last pixel
//   group redoes when the count is not a multiple of the group size;
//   a SIMD works through its wavefronts one after the other in effect.  If all wavefronts are
//   resident at once the busiest SIMD has ceil(wavefronts / SIMDs) of them and the kernel ends
//   with the slowest SIMD (about 4 % behind the mean); with more than fit, the hardware hands
//   out new wavefronts as old ones finish, which evens the load out to the average plus about
//   half a wavefront;
//   fewer than four wavefronts per SIMD hide latencies badly.
// The constants were fitted to measured times of the VGG- and ResNet-shaped layers.
int pick_conv_rows_per_wave(int64_t rows, int64_t W, int col_tiles, int passes, int group) {
    const int knob_rows = tuning().rows_per_wave, knob_waves = tuning().waves_per_simd;
    if (knob_rows > 0) return knob_rows;
    const double simds = (double)device_simd_count();
    const int resident = knob_waves > 0 ? knob_waves : 8;   // wavefronts a SIMD holds at once
    int64_t best = 0;
    double best_cost = 0.0;
    auto consider = [&](int64_t rpw) {
        if (rpw < 1 || rpw > rows) return;
        const double waves = (double)(((rows + rpw - 1) / rpw) * col_tiles);
        const double avg = waves / simds;
        if (avg > 64.0) return;                                            // launch overhead, no further gain
        const double rounds = (avg <= (double)resident) ? 1.04 * std::ceil(avg) : avg + 0.5;
        double wave_cost = (double)rpw + 0.22 * (double)passes;
        if (rpw % W != 0 && W % rpw != 0)                                  // may straddle two image rows
            wave_cost += 0.3 * (double)passes * (double)((rpw - 1) % W) / (double)W;
        if (rpw % group != 0) wave_cost += (double)(group - rpw % group);
        double cost = rounds * wave_cost;
        if (rounds < 4.0) cost *= 1.0 + 0.1 * (4.0 - rounds);
        if (best == 0 || cost < best_cost) { best = rpw; best_cost = cost; }
    };
    for (int64_t d = 1; d <= W; ++d) consider(d);
    for (int64_t k = 2; k <= 64; ++k) consider(k * W);
    if (best == 0) best = pick_rows_per_wave(rows, col_tiles, 4);
    return (int)best;
}

// Block numbering of a convolution launch (xcd_block() in the kernels): one contiguous range of
// blocks per XCD keeps each XCD's L2 to its own part of the activation planes (on the
// ResNet-18-shaped layer the kernel then fetches 3.5 MB instead of 10.2 MB).  Measured effect on
// the time: the general and window kernels gain up to 8 %, the 3x3 kernel gains 1-2 % from four
// column tiles on and loses 0.2-0.4 % below, the few-channel 3x3 kernel loses 3 %.  (The 3x3
// kernel has the numbering as a compile-time variant for channel counts of 64, 128, 256 and 512
// and ignores the request otherwise.)
int xcd_ranges_for(bool automatic) {
    const int o = tuning().block_order;
    return (o == 2 || (o == 0 && automatic)) ? 1 : 0;
}

// One wavefront's output slice (rows_per_wave * N * 4 bytes) must stay below 2^31 bytes.
int clamp_rows_per_wave(int rpw, int64_t N) {
    const int64_t cap = (((int64_t)1 << 29) - 1) / (N > 0 ? N : 1);
    if (rpw > cap) rpw = (int)(cap < 1 ? 1 : cap);
    return rpw;
}

// Checks shared by the GEMM and convolution entry points.  k_tap = true inner length of one
// tap (K for GEMM, C for conv), taps = 1 or 9.
// The re-encoded output of a chained layer: planes of out_bits bits, or nothing (planes == nullptr).
// Without an int32 / fp32 result buffer the partial sums of a multi-pass product need a workspace.
struct Emit {
    uint32_t *planes;
    int bits;
    void *workspace;
    size_t workspace_bytes;
};
const Emit kNoEmit = {nullptr, 0, nullptr, 0};

qnn_status check_branch(const void *A, int ab, const void *Wt, int wb, int64_t rows, int64_t N,
                        int64_t k_tap, int taps, const void *acc, const void *scale, const void *out,
                        const Emit &e = kNoEmit) {
    if (!bits_ok(ab) || !bits_ok(wb)) return QNN_EINVAL;
    if (rows < 0 || N < 0 || k_tap < 0) return QNN_EINVAL;
    const bool emit = e.bits != 0;                     // a *_requant entry point
    if (emit) {
        if (!bits_ok(e.bits)) return QNN_EINVAL;
        if (out != nullptr && scale == nullptr) return QNN_EINVAL;
    } else if ((scale == nullptr) != (out == nullptr)) {
        return QNN_EINVAL;
    }
    if (rows == 0 || N == 0) return QNN_OK;            // empty output: nothing is dereferenced
    if (emit) {
        if (e.planes == nullptr) return QNN_EINVAL;
        if (!aligned16(e.planes)) return QNN_EALIGN;
        if (acc == nullptr && out == nullptr) {
            if (e.workspace == nullptr) return QNN_EINVAL;
            if (!aligned16(e.workspace)) return QNN_EALIGN;
        }
    } else if (acc == nullptr && out == nullptr) {
        return QNN_EINVAL;
    }
    if ((A == nullptr || Wt == nullptr) && k_tap > 0) return QNN_EINVAL;
    if (!aligned16(A) || !aligned16(Wt)) return QNN_EALIGN;
    if (!aligned4(acc) || !aligned4(scale) || !aligned4(out)) return QNN_EALIGN;
    const int64_t fa = ((int64_t)1 << ab) - 1, fw = ((int64_t)1 << wb) - 1;
    if (k_tap > kInt31 / (fa * fw * taps)) return QNN_EUNSUPPORTED;       // int32 result range
    const int64_t cw = (k_tap + 31) / 32;
    // the kernels address the packed operands with 32-bit byte offsets and one output row with
    // a 32-bit byte offset inside a wavefront's slice
    const int64_t kWords30 = ((int64_t)1 << 30) - 1;
    if (rows > kInt31 || N > ((int64_t)1 << 24)) return QNN_EUNSUPPORTED;
    if (cw > 0 && (rows > kWords30 / (ab * cw) || N > kWords30 / (wb * cw * taps))) return QNN_EUNSUPPORTED;
    if (emit) {
        if (rows > kWords30 / (e.bits * ((N + 31) / 32))) return QNN_EUNSUPPORTED;
        if (acc == nullptr && out == nullptr && e.workspace_bytes < (size_t)(rows * N * 4)) return QNN_EWORKSPACE;
    }
    return QNN_OK;
}

// where the partial sums of a multi-pass product live
int32_t *partial_buffer(int32_t *acc, float *out, const Emit &e) {
    return acc ? acc : out ? reinterpret_cast<int32_t *>(out) : static_cast<int32_t *>(e.workspace);
}

// A wavefront's slice of the emitted planes (rows_per_wave * out_bits * Nw * 4 bytes) must stay
// below 2^31 bytes as well.
int clamp_rows_for_emit(int rpw, int64_t N, const Emit &e) {
    if (e.bits == 0) return rpw;
    const int64_t cap = (((int64_t)1 << 29) - 1) / (e.bits * ((N + 31) / 32));
    if (rpw > cap) rpw = (int)(cap < 1 ? 1 : cap);
    return rpw;
}

// `gather` (with the input image size H x W): row r of A is not row r of the buffer but the input
// pixel that output pixel r of a single-tap strided convolution reads (bit widths up to 4).
qnn_status run_gemm(const uint32_t *A, int ab, const uint32_t *Wt, int wb, int64_t M, int64_t N, int64_t K,
                    int32_t *acc, const float *scale, float *out_f32, const Emit &e, void *stream,
                    const ConvGeom *gather = nullptr, int H = 1, int W = 1) {
    qnn_status st = check_branch(A, ab, Wt, wb, M, N, K, 1, acc, scale, out_f32, e);
    if (st != QNN_OK || M == 0 || N == 0) return st;
    BranchArgs g;
    g.A = A; g.Wt = Wt; g.acc = acc; g.scale = scale; g.out = out_f32;
    g.partial = partial_buffer(acc, out_f32, e);
    g.out_flags = (acc != nullptr ? 1u : 0u) | (out_f32 != nullptr ? 2u : 0u);
    g.planes_out = e.planes; g.out_bits = e.bits;
    g.rows = (int)M; g.N = (int)N; g.Cw = (int)((K + 31) / 32); g.H = H; g.W = W; g.C = 0;
    g.gather_rows = (gather != nullptr) ? 1 : 0;
    g.xcd_ranges = 0; g.grid_blocks = 0;
    g.lds_partials = 0;
    if (gather != nullptr) g.geo = *gather;
    g.kconst = (int)(K * (((int64_t)1 << ab) - 1) * (((int64_t)1 << wb) - 1));
    g.col_tiles = (int)((N + 63) / 64);
    g.trace = tuning().trace; g.trace_waves = tuning().trace_waves;
    // Rows per wavefront.  Many short wavefronts (about 32 per SIMD over the launch) balance the
    // load and hide the latency of the partial sums that pass through the output between chunks;
    // the floor keeps a wavefront's products per weight chunk at about 1500 vector instructions or
    // more, below which reloading the weights costs more than the balance gains.  Measured on
    // products from 100352 x 64 x 256 to 8192^3 at one to four bits: 0.90-0.96 of the lane-op peak
    // at 16-32 wavefronts per SIMD against 0.82-0.87 at four.  The floor never leaves fewer than ten
    // wavefronts per SIMD: with four, one SIMD in ten gets a fifth and the launch waits for it
    // (measured with the floor at four per SIMD -> ten: 100352 x 64 x 256 at W2A2 20.2 -> 16.0 us,
    // 25088 x 512 x 256 31.0 -> 28.6 us, 100352 x 256 x 64 42.6 -> 33 us).
    {
        const int kc = gemm_chunk_words(wb);
        const int64_t per_row = 2 * (int64_t)ab * wb * (g.Cw < kc ? (g.Cw > 0 ? g.Cw : 1) : kc);
        int min_rows = (int)((1536 + per_row - 1) / per_row);
        const int at_ten = pick_rows_per_wave(M, g.col_tiles, 4, 10);
        if (min_rows > at_ten) min_rows = at_ten;
        if (min_rows > 20) min_rows = 20;      // very short rows (100352 x 256 x 64: 38.2 us at 39 rows, 32.5 at 20)
        const int rpw = pick_rows_per_wave(M, g.col_tiles, min_rows < 4 ? 4 : min_rows, 32);
        g.rows_per_wave = clamp_rows_for_emit(clamp_rows_per_wave(rpw, N), N, e);
    }
    g.split_k = 0;
    // Long K and too few rows (under 16 per wavefront at four wavefronts per SIMD) for every
    // wavefront to amortise its weight chunks: let the four wavefronts of a block share rows and
    // split the chunks instead.
    const int chunks = (g.Cw + gemm_chunk_words(wb) - 1) / gemm_chunk_words(wb);
    if (chunks >= 4 && pick_rows_per_wave(M, g.col_tiles, 4) < 16 && tuning().rows_per_wave == 0 && !g.gather_rows) {
        const int64_t target_blocks = (int64_t)device_simd_count();          // 4 blocks (16 wavefronts) per CU
        int64_t rows_per_block = (M * g.col_tiles + target_blocks - 1) / target_blocks;
        if (rows_per_block < 8) rows_per_block = 8;
        if (rows_per_block > 32) rows_per_block = 32;
        if (rows_per_block > M) rows_per_block = M;
        g.split_k = 1;
        g.rows_per_wave = (int)rows_per_block;
    }
    // Several chunk passes per wavefront: keep the partial sums of its rows in LDS rather than
    // sending them through the output buffer (at 8192^3 the partials of the resident wavefronts
    // do not stay in the L2s, and the kernel moved 2 GB per launch for 0.3 GB of operands and result).
    // Measured at 8192^3: 1 bit 1042 -> 949 us, 2 bits equal, 3 and 4 bits 1 % slower (fewer rows per
    // wavefront, and their round trip is small against the products of a chunk), hence the limit
    // of 256 vector instructions per row and chunk for the automatic choice.
    const bool lds_auto = 2 * ab * wb * gemm_chunk_words(wb) <= 256;
    const int knob_lds = tuning().lds_partials, knob_rows = tuning().rows_per_wave;
    if (!g.split_k && !g.gather_rows && chunks >= 2 && ab <= 4 && wb <= 4 &&
        (knob_lds == 2 || (knob_lds == 0 && lds_auto)) && (knob_rows == 0 || knob_rows <= kLdsPartialRows)) {
        g.lds_partials = 1;
        if (g.rows_per_wave > kLdsPartialRows) g.rows_per_wave = kLdsPartialRows;
    }
    set_divisors(g, /*output_image=*/g.gather_rows != 0);
    return from_hip(k_gemm[ab - 1](g, wb, (hipStream_t)stream));
}

// bytes of the packed im2col rows [rows][ab + 1][kwp]
size_t window_workspace_bytes(int64_t rows, int ab, int kwp) { return (size_t)rows * (size_t)(ab + 1) * (size_t)kwp * 4u; }

qnn_status check_image(int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Cout) {
    if (Nb < 0 || H < 0 || W < 0 || C < 0 || Cout < 0) return QNN_EINVAL;
    if (H > kInt31 || W > kInt31 || Nb > kInt31) return QNN_EUNSUPPORTED;
    if (H > 0 && W > 0 && Nb > kInt31 / H / W) return QNN_EUNSUPPORTED;
    return QNN_OK;
}

// stride: 1, or 2 where the 3x3 kernel has a fixed-shape instantiation (conv_has_fixed_shape).
// Other windows than 3x3 / dilation 1 (odd kh x kw, taps `dilation` pixels apart, "same" padding
// (k/2)*dilation): only at stride 1 and for the shapes conv_wide_plain_ok() / conv_wide_split_ok() /
// conv_wide_extra_ok() name.
qnn_status run_conv_packed(const uint32_t *x_planes, int ab, const uint32_t *Wt, int wb, int64_t Nb, int64_t H,
                           int64_t W, int64_t C, int64_t Cout, int32_t *acc, const float *scale,
                           float *out_f32, const Emit &e, void *stream, int stride = 1, int dilation = 1,
                           int kh = 3, int kw = 3) {
    qnn_status st = check_image(Nb, H, W, C, Cout);
    if (st != QNN_OK) return st;
    const int64_t Ho = (H > 0) ? (H - 1) / stride + 1 : 0, Wo = (W > 0) ? (W - 1) / stride + 1 : 0;
    const int64_t rows = Nb * Ho * Wo;
    st = check_branch(x_planes, ab, Wt, wb, rows, Cout, C, kh * kw, acc, scale, out_f32, e);
    if (st != QNN_OK || rows == 0 || Cout == 0) return st;
    const int64_t cw = (C + 31) / 32;
    if (cw > 0 && Nb * H * W > ((((int64_t)1 << 30) - 1) / (ab * cw))) return QNN_EUNSUPPORTED;      // input planes
    BranchArgs g;
    g.A = x_planes; g.Wt = Wt; g.acc = acc; g.scale = scale; g.out = out_f32;
    g.partial = partial_buffer(acc, out_f32, e);
    g.out_flags = (acc != nullptr ? 1u : 0u) | (out_f32 != nullptr ? 2u : 0u);
    g.planes_out = e.planes; g.out_bits = e.bits;
    g.rows = (int)rows; g.N = (int)Cout; g.Cw = (int)cw; g.H = (int)H; g.W = (int)W; g.C = (int)C;
    g.kconst = (int)(C * (((int64_t)1 << ab) - 1) * (((int64_t)1 << wb) - 1));
    g.col_tiles = (int)((Cout + 63) / 64);
    g.split_k = 0; g.gather_rows = 0; g.lds_partials = 0;
    g.xcd_ranges = (stride == 1) ? xcd_ranges_for(g.col_tiles >= 4) : 0;        // the strided variant keeps plain numbers
    g.trace = tuning().trace; g.trace_waves = tuning().trace_waves;
    g.geo.KH = kh; g.geo.KW = kw; g.geo.sh = stride; g.geo.sw = stride;
    g.geo.ph = (kh / 2) * dilation; g.geo.pw = (kw / 2) * dilation; g.geo.dh = dilation; g.geo.dw = dilation;
    g.geo.Ho = (int)Ho; g.geo.Wo = (int)Wo; g.geo.transposed = 0;
    const bool other_window = kh != 3 || kw != 3 || dilation != 1;
    // shapes without a one-tap-per-stage 3x3 kernel: another window has an instantiation of its own there
    const bool wide_extra = other_window && conv_wide_extra_ok(ab, wb, g.Cw);
    if (other_window) g.xcd_ranges = 0;          // those kernels exist with plain block numbers only
    const int group = wide_extra ? 1 : (stride == 1) ? conv_group(ab, wb, g.Cw) : conv_group_strided(ab, wb, g.Cw);
    // chunk passes per pixel: for a window of more than nine taps, so many times more tap chunks
    const int tap_factor = (kh * kw + 8) / 9;
    const int passes = wide_extra ? conv_wide_extra_passes(ab, wb, g.Cw) : conv_passes(ab, wb, g.Cw);
    g.rows_per_wave = clamp_rows_for_emit(clamp_rows_per_wave(pick_conv_rows_per_wave(rows, Wo, g.col_tiles, passes * tap_factor, group), Cout),
                                          Cout, e);
    // Few pixels and many channels: fewer than four wavefronts per SIMD would each make several
    // chunk passes.  The variant whose four wavefronts per block split the channel chunks gives four
    // times the wavefronts (measured on 32 x 7 x 7 x 512 -> 512, W2A4: 70.7 -> 50.6 us).  Its chunks
    // are a quarter of the plane where nine taps of that fit the weight registers, so they divide
    // evenly among the four wavefronts, no partial sum passes through the output buffer and every
    // wavefront loads one chunk of weights: with chunks of at least two words it is the faster
    // variant at any size (measured, W2A4: 512 -> 512 at 16 x 14 x 14: 115.6 -> 103.1 us, at
    // 16 x 28 x 28: 414.3 -> 382.1 us; 256 -> 256 at 16 x 56 x 56: 417.3 -> 394.5 us; W3A4
    // 256 -> 256 at 64 x 14 x 14: 161.4 -> 155.1 us; W4A4 256 -> 256 at 32 x 14 x 14: 145.2 ->
    // 103.9 us).  One-word chunks (128 channels, W3A4) gain at 56 x 56 (325.8 -> 299.3 us) and lose
    // at 28 x 28 (87.5 -> 91.7 us): those keep the plain variant unless the pixels are few.
    // (24 instead of 16 rows per block: equal for W2A4, 6-11 % slower for W3A4.)
    const int64_t plain_waves = ((rows + g.rows_per_wave - 1) / g.rows_per_wave) * g.col_tiles;
    const int knob_split = tuning().split_channels;
    const int split_words = conv_can_split(ab, wb, g.Cw) ? conv_split_shape(ab, wb, g.Cw).cwt : 0;
    const int split_chunks = split_words ? g.Cw / split_words : 0;
    // another window than the plain 3x3 on a shape whose plain variant does not take it: the split variant does
    const bool wide_needs_split = other_window && !conv_wide_plain_ok(ab, wb, g.Cw) && !wide_extra;
    const bool wide_needs_plain = other_window && !conv_wide_split_ok(ab, wb, g.Cw);
    if (split_chunks != 0 && !wide_needs_plain && ((tuning().rows_per_wave == 0 && knob_split != 1 &&
        (plain_waves < 4 * (int64_t)device_simd_count() || (split_chunks % 4 == 0 && split_words >= 2) || knob_split == 2)) ||
        wide_needs_split)) {
        const int chunks = split_chunks;
        int rpb = pick_conv_rows_per_wave(rows, Wo, g.col_tiles * 4, ((chunks + 3) / 4) * tap_factor, 1);
        if (rpb > kConvSplitRows) rpb = kConvSplitRows;
        g.rows_per_wave = clamp_rows_for_emit(clamp_rows_per_wave(rpb, Cout), Cout, e);
        g.split_k = 1;
        g.xcd_ranges = 0;
    }
    g.grid_blocks = wave_grid_blocks(g);
    set_divisors(g, /*output_image=*/true);
    return from_hip(k_conv[ab - 1](g, wb, (hipStream_t)stream));
}

qnn_status run_conv_im2col(const void *x_codes, int code_bytes, int ab, const uint32_t *Wt, int wb, int64_t Nb,
                           int64_t H, int64_t W, int64_t C, int64_t Cout, int32_t *acc, const float *scale,
                           float *out_f32, void *workspace, size_t workspace_bytes, const Emit &e,
                           void *stream, bool *dry_run = nullptr) {
    // dry_run: only the host-side checks; *dry_run says whether the call would launch anything
    if (dry_run) *dry_run = false;
    qnn_status st = check_image(Nb, H, W, C, Cout);
    if (st != QNN_OK) return st;
    if (code_bytes != 1 && code_bytes != 2) return QNN_EINVAL;
    if (code_bytes == 1 && ab == 8) return QNN_EINVAL;
    const int64_t rows = Nb * H * W;
    uint32_t *planes = static_cast<uint32_t *>(workspace);
    // validate everything before the first launch, so that an error launches nothing
    const bool have_k = C > 0;
    if (have_k && rows > 0 && Cout > 0) {
        if (x_codes == nullptr || workspace == nullptr) return QNN_EINVAL;
        if (!aligned16(workspace)) return QNN_EALIGN;
        if (code_bytes == 2 && (((uintptr_t)x_codes) & 1u)) return QNN_EALIGN;
    }
    st = check_branch(planes, ab, Wt, wb, rows, Cout, C, 9, acc, scale, out_f32, e);
    if (st != QNN_OK) return st;
    if (rows == 0 || Cout == 0) return QNN_OK;
    if (have_k) {
        if (workspace_bytes < qnn_conv2d_im2col_workspace_bytes(Nb, H, W, C, ab)) return QNN_EWORKSPACE;
    }
    if (dry_run) {
        *dry_run = true;
        return QNN_OK;
    }
    if (have_k) {
        if (9 * C <= 32) {
            // few input channels: one im2col word per plane and pixel (same workspace size as the
            // per-pixel planes, Cw == 1), then the single-word branch kernel
            st = from_hip(k_im2col[ab - 1](x_codes, code_bytes, rows, (int)H, (int)W, (int)C, planes,
                                           (hipStream_t)stream));
            if (st != QNN_OK) return st;
            BranchArgs g;
            g.A = planes; g.Wt = Wt; g.acc = acc; g.scale = scale; g.out = out_f32;
            g.partial = partial_buffer(acc, out_f32, e);
    g.out_flags = (acc != nullptr ? 1u : 0u) | (out_f32 != nullptr ? 2u : 0u);
            g.planes_out = e.planes; g.out_bits = e.bits;
            g.rows = (int)rows; g.N = (int)Cout; g.Cw = 1; g.H = (int)H; g.W = (int)W; g.C = (int)C;
            g.kconst = (int)((((int64_t)1 << ab) - 1) * (((int64_t)1 << wb) - 1));
            g.col_tiles = (int)((Cout + 63) / 64);
            g.split_k = 0; g.gather_rows = 0; g.lds_partials = 0; g.xcd_ranges = xcd_ranges_for(false);
            g.trace = nullptr; g.trace_waves = 0;
            // Short wavefronts that stream through the SIMDs: measured on the 16 x 224 x 224 x 3 -> 64
            // layer, 16 pixels each are best with int32 + fp32 outputs (95 us; 123 us at 196 pixels, where
            // four wavefronts per SIMD are all there is) and 28 with emitted planes only (99.5 us).
            const int knob_rows = tuning().rows_per_wave;
            const int small_rpw = knob_rows > 0 ? knob_rows : (e.bits != 0 ? 28 : 16);
            g.rows_per_wave = clamp_rows_for_emit(clamp_rows_per_wave(small_rpw, Cout), Cout, e);
            g.grid_blocks = wave_grid_blocks(g);
            set_divisors(g);
            return from_hip(k_conv_small[ab - 1](g, wb, (hipStream_t)stream));
        }
        st = qnn_encode_pack(x_codes, code_bytes, rows, C, ab, planes, nullptr, 0, stream);
        if (st != QNN_OK) return st;
    }
    return run_conv_packed(planes, ab, Wt, wb, Nb, H, W, C, Cout, acc, scale, out_f32, e, stream);
}

}  // namespace
}  // namespace qnn

using namespace qnn;

extern "C" {

const char *qnn_status_string(int status) {
    switch (status) {
        case QNN_OK: return "ok";
        case QNN_EINVAL: return "invalid argument";
        case QNN_EALIGN: return "buffer not aligned as documented";
        case QNN_EUNSUPPORTED: return "size beyond the documented limits";
        case QNN_EWORKSPACE: return "workspace too small";
        case QNN_EHIP: return "HIP runtime error at launch";
    }
    return "unknown status";
}

int qnn_last_hip_error(void) { return g_last_hip_error; }

int qnn_version(void) { return 101; }

qnn_status qnn_device_info(int *h_compute_units, int *h_clock_khz) {
    if (h_compute_units == nullptr || h_clock_khz == nullptr) return QNN_EINVAL;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(h_compute_units, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(h_clock_khz, hipDeviceAttributeClockRate, dev);
    return from_hip(e);
}

int qnn_set_wave_trace(void *buffer, size_t bytes) {
    if (buffer != nullptr && ((((uintptr_t)buffer) & 7u) || bytes < 32)) return QNN_EINVAL;
    tuning().trace = static_cast<uint64_t *>(buffer);
    tuning().trace_waves = buffer ? (uint32_t)(bytes / 32 > 0xffffffffu ? 0xffffffffu : bytes / 32) : 0;
    return QNN_OK;
}

int qnn_tune(int key, int value) {
    if (value < 0) return QNN_EINVAL;
    switch (key) {
        case QNN_TUNE_WAVES_PER_SIMD: tuning().waves_per_simd = value; return QNN_OK;
        case QNN_TUNE_ROWS_PER_WAVE: tuning().rows_per_wave = value; return QNN_OK;
        case QNN_TUNE_GENERAL_ONLY: tuning().general_only = value; return QNN_OK;
        case QNN_TUNE_LDS_PARTIALS:
            if (value > 2) return QNN_EINVAL;
            tuning().lds_partials = value;
            return QNN_OK;
        case QNN_TUNE_SPLIT_CHANNELS:
            if (value > 2) return QNN_EINVAL;
            tuning().split_channels = value;
            return QNN_OK;
        case QNN_TUNE_BLOCK_ORDER:
            if (value > 2) return QNN_EINVAL;
            tuning().block_order = value;
            return QNN_OK;
    }
    return QNN_EINVAL;
}

qnn_status qnn_encode_pack(const void *codes, int code_bytes, int64_t rows, int64_t K, int bits,
                           uint32_t *planes, int32_t *bad_count, unsigned flags, void *stream) {
    if (!bits_ok(bits) || rows < 0 || K < 0) return QNN_EINVAL;
    if (code_bytes != 1 && code_bytes != 2) return QNN_EINVAL;
    if (code_bytes == 1 && bits == 8) return QNN_EINVAL;          // 8-bit codes need int16
    if (flags & ~QNN_PACK_VALIDATE) return QNN_EINVAL;
    if (rows == 0 || K == 0) return QNN_OK;
    if (codes == nullptr || planes == nullptr) return QNN_EINVAL;
    if (!aligned16(planes)) return QNN_EALIGN;
    if (code_bytes == 2 && (((uintptr_t)codes) & 1u)) return QNN_EALIGN;
    if (!aligned4(bad_count)) return QNN_EALIGN;
    if (K > kInt31) return QNN_EUNSUPPORTED;
    const int64_t Kw = (K + 31) / 32;
    if (rows > (((int64_t)1 << 40) - 1) / (bits * Kw)) return QNN_EUNSUPPORTED;
    const bool validate = (flags & QNN_PACK_VALIDATE) && bad_count != nullptr;
    return from_hip(launch_pack(codes, code_bytes, rows, K, bits, planes, bad_count, validate,
                                (hipStream_t)stream));
}

qnn_status qnn_branch_gemm(const uint32_t *A, int ab, const uint32_t *Wt, int wb, int64_t M, int64_t N,
                           int64_t K, int32_t *acc, const float *scale, float *out_f32, void *stream) {
    return run_gemm(A, ab, Wt, wb, M, N, K, acc, scale, out_f32, kNoEmit, stream);
}

size_t qnn_conv2d_im2col_workspace_bytes(int64_t Nb, int64_t H, int64_t W, int64_t C, int ab) {
    if (Nb <= 0 || H <= 0 || W <= 0 || C <= 0 || !bits_ok(ab)) return 0;
    const int64_t cw = (C + 31) / 32;
    return (size_t)(Nb * H * W * ab * cw * 4);
}

qnn_status qnn_conv2d_packed(const uint32_t *x_planes, int ab, const uint32_t *Wt, int wb, int64_t Nb,
                             int64_t H, int64_t W, int64_t C, int64_t Cout, int32_t *acc,
                             const float *scale, float *out_f32, void *stream) {
    return run_conv_packed(x_planes, ab, Wt, wb, Nb, H, W, C, Cout, acc, scale, out_f32, kNoEmit, stream);
}

qnn_status qnn_conv2d_im2col(const void *x_codes, int code_bytes, int ab, const uint32_t *Wt, int wb,
                             int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Cout, int32_t *acc,
                             const float *scale, float *out_f32, void *workspace,
                             size_t workspace_bytes, void *stream) {
    return run_conv_im2col(x_codes, code_bytes, ab, Wt, wb, Nb, H, W, C, Cout, acc, scale, out_f32, workspace,
                           workspace_bytes, kNoEmit, stream);
}

qnn_status qnn_conv2d_im2col_static(const void *x_codes, int code_bytes, int ab, const uint32_t *Wt, int wb,
                                    int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Cout, int32_t *acc,
                                    const float *scale, float *out_f32, void *stream) {
    // Every host-side check first, with a stand-in for the scratch address: they need no GPU, and
    // nothing may be looked up or launched for a call that fails them.
    alignas(16) static char stand_in;
    bool launches = false;
    const qnn_status st = run_conv_im2col(x_codes, code_bytes, ab, Wt, wb, Nb, H, W, C, Cout, acc, scale, out_f32,
                                          &stand_in, kStaticScratchBytes, kNoEmit, stream, &launches);
    if (st == QNN_EWORKSPACE) return QNN_EUNSUPPORTED;          // the planes do not fit the static scratch
    if (st != QNN_OK || !launches) return st;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return from_hip(hipErrorInvalidDevice);
    void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        // first call on this GPU (it is the current device): every GPU has its own copy of the array
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || ptr == nullptr) return from_hip(e != hipSuccess ? e : hipErrorInvalidSymbol);
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    // Both kernels overwrite every word of the planes they use (tail bits included), so the
    // contents a previous call left behind need no clearing.
    return run_conv_im2col(x_codes, code_bytes, ab, Wt, wb, Nb, H, W, C, Cout, acc, scale, out_f32, ptr,
                           kStaticScratchBytes, kNoEmit, stream);
}

size_t qnn_requant_workspace_bytes(int64_t rows, int64_t N) {
    if (rows <= 0 || N <= 0) return 0;
    return (size_t)(rows * N * 4);
}

qnn_status qnn_branch_gemm_requant(const uint32_t *A, int ab, const uint32_t *Wt, int wb, int64_t M, int64_t N,
                                   int64_t K, const float *scale, int out_bits, uint32_t *out_planes,
                                   int32_t *acc, float *out_f32, void *workspace, size_t workspace_bytes,
                                   void *stream) {
    if (!bits_ok(out_bits)) return QNN_EINVAL;
    const Emit e = {out_planes, out_bits, workspace, workspace_bytes};
    return run_gemm(A, ab, Wt, wb, M, N, K, acc, scale, out_f32, e, stream);
}

qnn_status qnn_conv2d_packed_requant(const uint32_t *x_planes, int ab, const uint32_t *Wt, int wb, int64_t Nb,
                                     int64_t H, int64_t W, int64_t C, int64_t Cout, const float *scale,
                                     int out_bits, uint32_t *out_planes, int32_t *acc, float *out_f32,
                                     void *workspace, size_t workspace_bytes, void *stream) {
    if (!bits_ok(out_bits)) return QNN_EINVAL;
    const Emit e = {out_planes, out_bits, workspace, workspace_bytes};
    return run_conv_packed(x_planes, ab, Wt, wb, Nb, H, W, C, Cout, acc, scale, out_f32, e, stream);
}

size_t qnn_conv2d_im2col_requant_workspace_bytes(int64_t Nb, int64_t H, int64_t W, int64_t C, int ab,
                                                 int64_t Cout) {
    const size_t a = (qnn_conv2d_im2col_workspace_bytes(Nb, H, W, C, ab) + 15) & ~(size_t)15;
    return a + qnn_requant_workspace_bytes(Nb * H * W, Cout);
}

qnn_status qnn_conv2d_im2col_requant(const void *x_codes, int code_bytes, int ab, const uint32_t *Wt, int wb,
                                     int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Cout,
                                     const float *scale, int out_bits, uint32_t *out_planes, int32_t *acc,
                                     float *out_f32, void *workspace, size_t workspace_bytes, void *stream) {
    if (!bits_ok(out_bits)) return QNN_EINVAL;
    if (check_image(Nb, H, W, C, Cout) != QNN_OK || !bits_ok(ab)) return QNN_EINVAL;
    // the workspace holds the packed activations first, then (16-byte aligned) the partial sums
    const size_t first = (qnn_conv2d_im2col_workspace_bytes(Nb, H, W, C, ab) + 15) & ~(size_t)15;
    Emit e = {out_planes, out_bits, nullptr, 0};
    if (workspace != nullptr) {
        e.workspace = static_cast<char *>(workspace) + first;
        e.workspace_bytes = workspace_bytes > first ? workspace_bytes - first : 0;
    }
    return run_conv_im2col(x_codes, code_bytes, ab, Wt, wb, Nb, H, W, C, Cout, acc, scale, out_f32, workspace,
                           workspace_bytes < first ? workspace_bytes : first, e, stream);
}

qnn_status qnn_requant_pack(const float *y, int64_t Nb, int64_t H, int64_t W, int64_t C, int pool2x2, int bits,
                            void *codes, uint32_t *planes, void *stream) {
    if (!bits_ok(bits) || Nb < 0 || H < 0 || W < 0 || C < 0) return QNN_EINVAL;
    if (pool2x2 != 0 && pool2x2 != 1) return QNN_EINVAL;
    if (pool2x2 && ((H & 1) || (W & 1))) return QNN_EINVAL;
    if (H > kInt31 || W > kInt31 || Nb > kInt31 || C > kInt31) return QNN_EUNSUPPORTED;
    if (Nb == 0 || H == 0 || W == 0 || C == 0) return QNN_OK;
    if (Nb > kInt31 / H / W) return QNN_EUNSUPPORTED;
    if (y == nullptr || (codes == nullptr && planes == nullptr)) return QNN_EINVAL;
    if (!aligned4(y) || !aligned16(planes)) return QNN_EALIGN;
    if (bits == 8 && (((uintptr_t)codes) & 1u)) return QNN_EALIGN;
    return from_hip(launch_requant(y, Nb, H, W, C, pool2x2 != 0, bits, 1.0f, 0, codes, planes, (hipStream_t)stream));
}

qnn_status qnn_encode_real(const float *x, int64_t rows, int64_t K, int bits, int clip, void *codes,
                           uint32_t *planes, void *stream) {
    if (!bits_ok(bits) || rows < 0 || K < 0 || clip < QNN_CLIP_HTANH || clip > QNN_CLIP_SIGMOID) return QNN_EINVAL;
    if (rows > kInt31 || K > kInt31) return QNN_EUNSUPPORTED;
    if (rows == 0 || K == 0) return QNN_OK;
    if (x == nullptr || (codes == nullptr && planes == nullptr)) return QNN_EINVAL;
    if (!aligned4(x) || !aligned16(planes)) return QNN_EALIGN;
    if (bits == 8 && (((uintptr_t)codes) & 1u)) return QNN_EALIGN;
    const float alpha = (float)((1 << bits) - 1);
    return from_hip(launch_requant(x, 1, 1, rows, K, false, bits, alpha, clip, codes, planes, (hipStream_t)stream));
}

qnn_status qnn_encoder_backward(const float *x, const float *g_bits, int64_t n, int bits, float *g_x, void *stream) {
    if (!bits_ok(bits) || n < 0) return QNN_EINVAL;
    if (n == 0) return QNN_OK;
    if (x == nullptr || g_bits == nullptr || g_x == nullptr) return QNN_EINVAL;
    if (!aligned4(x) || !aligned4(g_bits) || !aligned4(g_x)) return QNN_EALIGN;
    if (n > (((int64_t)1 << 40) - 1) / bits) return QNN_EUNSUPPORTED;
    return from_hip(launch_encoder_backward(x, g_bits, n, bits, g_x, (hipStream_t)stream));
}

qnn_status qnn_binarize(const float *w, int64_t rows, int64_t K, int8_t *codes, uint32_t *planes, void *stream) {
    if (rows < 0 || K < 0) return QNN_EINVAL;
    if (K > kInt31 || rows > kInt31) return QNN_EUNSUPPORTED;
    if (rows == 0 || K == 0) return QNN_OK;
    if (w == nullptr || (codes == nullptr && planes == nullptr)) return QNN_EINVAL;
    if (!aligned4(w) || !aligned16(planes)) return QNN_EALIGN;
    return from_hip(launch_binarize(w, rows, K, codes, planes, (hipStream_t)stream));
}

qnn_status qnn_binarize_backward(const float *w, const float *g_wb, int64_t n, float *g_w, void *stream) {
    if (n < 0) return QNN_EINVAL;
    if (n == 0) return QNN_OK;
    if (w == nullptr || g_wb == nullptr || g_w == nullptr) return QNN_EINVAL;
    if (!aligned4(w) || !aligned4(g_wb) || !aligned4(g_w)) return QNN_EALIGN;
    return from_hip(launch_binarize_backward(w, g_wb, n, g_w, (hipStream_t)stream));
}

qnn_status qnn_quantize_k(const float *x, int64_t n, int bits, float t, float *q, int32_t *levels, void *stream) {
    if (bits < 2 || bits > 24 || n < 0 || !(t > 0.0f) || !(t <= 3.0e38f)) return QNN_EINVAL;   // one bit has no state besides 0
    if (n == 0) return QNN_OK;
    if (x == nullptr || (q == nullptr && levels == nullptr)) return QNN_EINVAL;
    if (!aligned4(x) || !aligned4(q) || !aligned4(levels)) return QNN_EALIGN;
    return from_hip(launch_quantize_k(x, n, bits, t, q, levels, (hipStream_t)stream));
}

qnn_status qnn_quantize_k_backward(const float *x, const float *g_q, int64_t n, float t, float *g_x, void *stream) {
    if (n < 0 || !(t > 0.0f) || !(t <= 3.0e38f)) return QNN_EINVAL;
    if (n == 0) return QNN_OK;
    if (x == nullptr || g_q == nullptr || g_x == nullptr) return QNN_EINVAL;
    if (!aligned4(x) || !aligned4(g_q) || !aligned4(g_x)) return QNN_EALIGN;
    return from_hip(launch_quantize_k_backward(x, g_q, n, t, g_x, (hipStream_t)stream));
}

qnn_status qnn_branch_gemm_backward_input(const float *g_out, const float *scale, const uint32_t *Wt, int wb,
                                          int64_t M, int64_t N, int64_t K, int ab, float *g_bits, void *stream) {
    if (!bits_ok(ab) || !bits_ok(wb) || M < 0 || N < 0 || K < 0) return QNN_EINVAL;
    if (M > kInt31 || N > kInt31 || K > kInt31) return QNN_EUNSUPPORTED;
    if (M == 0 || K == 0) return QNN_OK;
    if (g_bits == nullptr || (N > 0 && (g_out == nullptr || Wt == nullptr))) return QNN_EINVAL;
    if (!aligned4(g_out) || !aligned4(scale) || !aligned4(g_bits) || !aligned16(Wt)) return QNN_EALIGN;
    return from_hip(launch_backward_gemm(g_out, N, scale, Wt, wb, (int)M, (int)N, (int)K, ab, /*towards_weights=*/false,
                                         g_bits, (hipStream_t)stream));
}

qnn_status qnn_branch_gemm_backward_weight(const float *g_out, const float *scale, const uint32_t *A, int ab,
                                           int64_t M, int64_t N, int64_t K, int wb, float *g_wb, void *stream) {
    if (!bits_ok(ab) || !bits_ok(wb) || M < 0 || N < 0 || K < 0) return QNN_EINVAL;
    if (M > kInt31 || N > kInt31 || K > kInt31) return QNN_EUNSUPPORTED;
    if (N == 0 || K == 0) return QNN_OK;
    if (g_wb == nullptr || (M > 0 && (g_out == nullptr || A == nullptr))) return QNN_EINVAL;
    if (!aligned4(g_out) || !aligned4(scale) || !aligned4(g_wb) || !aligned16(A)) return QNN_EALIGN;
    return from_hip(launch_backward_gemm(g_out, N, scale, A, ab, (int)N, (int)M, (int)K, wb, /*towards_weights=*/true,
                                         g_wb, (hipStream_t)stream));
}

namespace {
qnn_status check_conv_backward(int ab, int wb, int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Cout) {
    if (!bits_ok(ab) || !bits_ok(wb) || Nb < 0 || H < 0 || W < 0 || C < 0 || Cout < 0) return QNN_EINVAL;
    if (H > kInt31 || W > kInt31 || Nb > kInt31 || C >= ((int64_t)1 << 20) || Cout >= ((int64_t)1 << 20)) return QNN_EUNSUPPORTED;
    if (H > 0 && W > 0 && Nb > ((((int64_t)1 << 30) - 1) / H) / W) return QNN_EUNSUPPORTED;
    return QNN_OK;
}
}  // namespace

qnn_status qnn_conv2d_backward_input(const float *g_out, const float *scale, const uint32_t *Wt, int wb, int64_t Nb,
                                     int64_t H, int64_t W, int64_t C, int64_t Cout, int ab, float *g_bits, void *stream) {
    const qnn_status st = check_conv_backward(ab, wb, Nb, H, W, C, Cout);
    if (st != QNN_OK) return st;
    if (Nb * H * W == 0 || C == 0) return QNN_OK;
    if (g_bits == nullptr || (Cout > 0 && (g_out == nullptr || Wt == nullptr))) return QNN_EINVAL;
    if (!aligned4(g_out) || !aligned4(scale) || !aligned4(g_bits) || !aligned16(Wt)) return QNN_EALIGN;
    return from_hip(launch_conv_backward_input(g_out, scale, Wt, wb, Nb, (int)H, (int)W, (int)C, (int)Cout, ab, g_bits,
                                               (hipStream_t)stream));
}

size_t qnn_conv2d_backward_weight_workspace_bytes(int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Cout) {
    if (check_conv_backward(1, 1, Nb, H, W, C, Cout) != QNN_OK || C == 0 || Cout == 0) return 0;
    return (size_t)conv_backward_splits(Nb * H * W, Cout, C) * (size_t)Cout * 9u * (size_t)C * 4u;
}

qnn_status qnn_conv2d_backward_weight(const float *g_out, const float *scale, const uint32_t *x_planes, int ab, int64_t Nb,
                                      int64_t H, int64_t W, int64_t C, int64_t Cout, int wb, float *g_wb, void *workspace,
                                      size_t workspace_bytes, void *stream) {
    const qnn_status st = check_conv_backward(ab, wb, Nb, H, W, C, Cout);
    if (st != QNN_OK) return st;
    if (Cout == 0 || C == 0) return QNN_OK;
    const int64_t pixels = Nb * H * W;
    if (g_wb == nullptr || workspace == nullptr || (pixels > 0 && (g_out == nullptr || x_planes == nullptr))) return QNN_EINVAL;
    if (!aligned4(g_out) || !aligned4(scale) || !aligned4(g_wb) || !aligned16(x_planes) || !aligned16(workspace)) return QNN_EALIGN;
    if (workspace_bytes < qnn_conv2d_backward_weight_workspace_bytes(Nb, H, W, C, Cout)) return QNN_EWORKSPACE;
    return from_hip(launch_conv_backward_weight(g_out, scale, x_planes, ab, Nb, (int)H, (int)W, (int)C, (int)Cout, wb, g_wb,
                                                static_cast<float *>(workspace), (hipStream_t)stream));
}

qnn_status qnn_update_adam(float *w, const float *g, float *m, float *v, int64_t n, float lr, float beta1, float beta2,
                           float eps, int step, void *stream) {
    if (n < 0 || step < 1 || !(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f) || !(eps >= 0.0f))
        return QNN_EINVAL;
    if (n == 0) return QNN_OK;
    if (w == nullptr || g == nullptr || m == nullptr || v == nullptr) return QNN_EINVAL;
    if (!aligned4(w) || !aligned4(g) || !aligned4(m) || !aligned4(v)) return QNN_EALIGN;
    const float omb1 = (float)(1.0 - (double)beta1), omb2 = (float)(1.0 - (double)beta2);
    const float bc1 = (float)(1.0 - std::pow((double)beta1, (double)step));
    const float bc2 = (float)(1.0 - std::pow((double)beta2, (double)step));
    return from_hip(launch_update_adam(w, g, m, v, n, lr, beta1, beta2, omb1, omb2, bc1, bc2, eps, (hipStream_t)stream));
}

qnn_status qnn_update_sgd(float *w, const float *g, int64_t n, float lr, void *stream) {
    if (n < 0) return QNN_EINVAL;
    if (n == 0) return QNN_OK;
    if (w == nullptr || g == nullptr) return QNN_EINVAL;
    if (!aligned4(w) || !aligned4(g)) return QNN_EALIGN;
    return from_hip(launch_update_sgd(w, g, n, lr, (hipStream_t)stream));
}

qnn_status qnn_conv2d_general_output_size(int64_t H, int64_t W, const qnn_conv_geometry *q, int64_t *h_Ho,
                                          int64_t *h_Wo) {
    if (q == nullptr || h_Ho == nullptr || h_Wo == nullptr || H < 0 || W < 0) return QNN_EINVAL;
    if (q->kh < 1 || q->kw < 1 || q->stride_h < 1 || q->stride_w < 1 || q->dil_h < 1 || q->dil_w < 1) return QNN_EINVAL;
    if (q->pad_h < 0 || q->pad_w < 0 || (q->transposed != 0 && q->transposed != 1)) return QNN_EINVAL;
    if (q->dense_rows != 0 && q->dense_rows != 1) return QNN_EINVAL;
    const int lim = 1 << 12;                               // keeps every coordinate sum and product inside int32
    if (q->kh > lim || q->kw > lim || q->stride_h > lim || q->stride_w > lim || q->dil_h > lim || q->dil_w > lim ||
        q->pad_h > lim || q->pad_w > lim)
        return QNN_EUNSUPPORTED;
    if (H > ((int64_t)1 << 30) || W > ((int64_t)1 << 30)) return QNN_EUNSUPPORTED;
    int64_t Ho, Wo;
    if (q->transposed) {
        const int mh = q->stride_h > q->dil_h ? q->stride_h : q->dil_h, mw = q->stride_w > q->dil_w ? q->stride_w : q->dil_w;
        if (q->out_pad_h < 0 || q->out_pad_w < 0 || q->out_pad_h >= mh || q->out_pad_w >= mw) return QNN_EINVAL;
        Ho = (H - 1) * q->stride_h - 2 * (int64_t)q->pad_h + (int64_t)q->dil_h * (q->kh - 1) + q->out_pad_h + 1;
        Wo = (W - 1) * q->stride_w - 2 * (int64_t)q->pad_w + (int64_t)q->dil_w * (q->kw - 1) + q->out_pad_w + 1;
    } else {
        if (q->out_pad_h != 0 || q->out_pad_w != 0) return QNN_EINVAL;
        const int64_t nh = H + 2 * (int64_t)q->pad_h - (int64_t)q->dil_h * (q->kh - 1) - 1;
        const int64_t nw = W + 2 * (int64_t)q->pad_w - (int64_t)q->dil_w * (q->kw - 1) - 1;
        if (nh < 0 || nw < 0) return QNN_EINVAL;
        Ho = nh / q->stride_h + 1;
        Wo = nw / q->stride_w + 1;
    }
    if (H == 0 || W == 0) { Ho = 0; Wo = 0; }
    if ((H > 0 && W > 0) && (Ho < 1 || Wo < 1)) return QNN_EINVAL;
    if (Ho > ((int64_t)1 << 30) || Wo > ((int64_t)1 << 30)) return QNN_EUNSUPPORTED;
    *h_Ho = Ho;
    *h_Wo = Wo;
    return QNN_OK;
}

size_t qnn_conv2d_general_workspace_bytes(int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Cout, int ab,
                                          int wb, const qnn_conv_geometry *q) {
    int64_t Ho = 0, Wo = 0;
    if (!bits_ok(ab) || !bits_ok(wb) || Nb <= 0 || C <= 0 || Cout <= 0) return 0;
    if (qnn_conv2d_general_output_size(H, W, q, &Ho, &Wo) != QNN_OK) return 0;
    const int64_t rows = Nb * Ho * Wo, taps = (int64_t)q->kh * q->kw;
    const int kwp = (!q->transposed && C <= 32 && taps >= 2) ? window_words(taps * C) : 0;
    const size_t win = kwp > 0 ? window_workspace_bytes(rows, ab, kwp) : 0;
    const size_t part = (size_t)(rows * Cout * 4);
    return win > part ? win : part;
}

qnn_status qnn_conv2d_general(const uint32_t *x_planes, int ab, const uint32_t *Wt, int wb, int64_t Nb, int64_t H,
                              int64_t W, int64_t C, int64_t Cout, const qnn_conv_geometry *q, int32_t *acc,
                              const float *scale, float *out_f32, int out_bits, uint32_t *out_planes,
                              void *workspace, size_t workspace_bytes, void *stream) {
    if (out_bits != 0 && !bits_ok(out_bits)) return QNN_EINVAL;
    qnn_status st = check_image(Nb, H, W, C, Cout);
    if (st != QNN_OK) return st;
    int64_t Ho = 0, Wo = 0;
    st = qnn_conv2d_general_output_size(H, W, q, &Ho, &Wo);
    if (st != QNN_OK) return st;
    if (Ho > 0 && Wo > 0 && Nb > kInt31 / Ho / Wo) return QNN_EUNSUPPORTED;
    const int64_t rows = Nb * Ho * Wo, taps = (int64_t)q->kh * q->kw;
    if (taps > (1 << 20)) return QNN_EUNSUPPORTED;
    const Emit e = (out_bits != 0) ? Emit{out_planes, out_bits, workspace, workspace_bytes} : kNoEmit;
    st = check_branch(x_planes, ab, Wt, wb, rows, Cout, C, (int)taps, acc, scale, out_f32, e);
    if (st != QNN_OK || rows == 0 || Cout == 0) return st;
    // row-dense input exists for the packed-window path only
    if (q->dense_rows && (q->transposed || C > 32 || taps < 2 || window_words(taps * C) == 0))
        return QNN_EUNSUPPORTED;
    // A single tap at stride 1 without padding reads pixel r for output pixel r: the product of the
    // [pixels][C] matrix with the [Cout][C] weights, whichever way the transposed flag is set.
    if (taps == 1 && q->stride_h == 1 && q->stride_w == 1 && q->pad_h == 0 && q->pad_w == 0)
        return run_gemm(x_planes, ab, Wt, wb, rows, Cout, C, acc, scale, out_f32, e, stream);
    const int64_t cw = (C + 31) / 32;
    if (cw > 0 && Nb * H * W > ((((int64_t)1 << 30) - 1) / (ab * cw))) return QNN_EUNSUPPORTED;   // input planes
    // A single tap with a stride (the shortcut convolutions of the residual networks): the same
    // product over a strided selection of the pixels.
    if (taps == 1 && !q->transposed && q->pad_h == 0 && q->pad_w == 0 && ab <= 4 && wb <= 4 && cw > 0) {
        ConvGeom cg;
        cg.KH = 1; cg.KW = 1; cg.sh = q->stride_h; cg.sw = q->stride_w; cg.ph = 0; cg.pw = 0; cg.dh = 1; cg.dw = 1;
        cg.Ho = (int)Ho; cg.Wo = (int)Wo; cg.transposed = 0;
        return run_gemm(x_planes, ab, Wt, wb, rows, Cout, C, acc, scale, out_f32, e, stream, &cg, (int)H, (int)W);
    }
    BranchArgs g;
    g.A = x_planes; g.Wt = Wt; g.acc = acc; g.scale = scale; g.out = out_f32;
    g.partial = partial_buffer(acc, out_f32, e);
    g.out_flags = (acc != nullptr ? 1u : 0u) | (out_f32 != nullptr ? 2u : 0u);
    g.planes_out = e.planes; g.out_bits = e.bits;
    g.rows = (int)rows; g.N = (int)Cout; g.Cw = (int)cw; g.H = (int)H; g.W = (int)W; g.C = (int)C;
    g.kconst = (int)(C * (((int64_t)1 << ab) - 1) * (((int64_t)1 << wb) - 1));
    g.col_tiles = (int)((Cout + 63) / 64);
    g.split_k = 0; g.gather_rows = 0; g.lds_partials = 0; g.xcd_ranges = xcd_ranges_for(true);
    g.trace = nullptr; g.trace_waves = 0;
    g.geo.KH = q->kh; g.geo.KW = q->kw; g.geo.sh = q->stride_h; g.geo.sw = q->stride_w;
    g.geo.ph = q->pad_h; g.geo.pw = q->pad_w; g.geo.dh = q->dil_h; g.geo.dw = q->dil_w;
    g.geo.Ho = (int)Ho; g.geo.Wo = (int)Wo;
    g.geo.transposed = (q->transposed && cw > 0) ? 1 : 0;      // an empty sum needs no phases
    // Few input channels and a window of at most 256 bits: packed im2col rows, if the caller gave
    // the workspace for them (else the general kernel below does the same, a word per tap).
    const int kwp = (!q->transposed && C <= 32 && taps >= 2) ? window_words(taps * C) : 0;
    if (kwp > 0) {
        const size_t need = window_workspace_bytes(rows, ab, kwp);
        if (workspace != nullptr && aligned16(workspace) && workspace_bytes >= need && need < ((size_t)1 << 32)) {
            uint32_t *win = static_cast<uint32_t *>(workspace);
            st = from_hip(launch_window_pack(x_planes, rows, g.geo, (int)H, (int)W, (int)C, ab, kwp,
                                             q->dense_rows != 0, win, (hipStream_t)stream));
            if (st != QNN_OK) return st;
            g.A = win;
            g.Cw = kwp;
            g.kconst = (int)((((int64_t)1 << ab) - 1) * (((int64_t)1 << wb) - 1));
            int64_t rpw2 = tuning().rows_per_wave;
            if (rpw2 <= 0) {
                rpw2 = rows * g.col_tiles / ((int64_t)device_simd_count() * 8);
                if (rpw2 < 16) rpw2 = 16;
            }
            if (rpw2 > rows) rpw2 = rows;
            g.rows_per_wave = clamp_rows_for_emit(clamp_rows_per_wave((int)rpw2, Cout), Cout, e);
            g.grid_blocks = wave_grid_blocks(g);
            set_divisors(g, true);
            return from_hip(k_conv_window[ab - 1](g, wb, (hipStream_t)stream));
        }
    }
    if (q->dense_rows) return (kwp > 0) ? QNN_EWORKSPACE : QNN_EUNSUPPORTED;   // only the window path reads row-dense input
    // The 3x3 window at stride 1 with one pixel of padding has a kernel of its own (the same
    // operands, the same outputs; about 1.5x faster on a ResNet-18-shaped layer).
    // At stride 2 the same kernel serves the channel counts it is instantiated for with a compile-time
    // plane stride (the strided layers of the residual networks: 64 ... 512 channels).
    const bool s1 = q->stride_h == 1 && q->stride_w == 1;
    const bool s2 = q->stride_h == 2 && q->stride_w == 2 && conv_has_fixed_shape(ab, wb, (int)cw);
    if (!q->transposed && q->kh == 3 && q->kw == 3 && (s1 || s2) && q->pad_h == 1 &&
        q->pad_w == 1 && q->dil_h == 1 && q->dil_w == 1 && cw > 0 && !tuning().general_only)
        return run_conv_packed(x_planes, ab, Wt, wb, Nb, H, W, C, Cout, acc, scale, out_f32, e, stream, s1 ? 1 : 2);
    // Other odd windows with "same" padding at stride 1 -- the atrous 3x3 convolution, 5x5, 7x7, 1x3 ...
    // -- run on that kernel too where its shape takes one tap per pipeline stage (128 channels and
    // more): only the tap offsets, their number and the border tests depend on the window there.
    if (!q->transposed && s1 && (q->kh & 1) && (q->kw & 1) && q->kh * q->kw > 1 && q->kh * q->kw <= 49 &&
        q->dil_h == q->dil_w && q->dil_h >= 1 && q->dil_h <= 64 && q->pad_h == (q->kh / 2) * q->dil_h &&
        q->pad_w == (q->kw / 2) * q->dil_w && !tuning().general_only &&
        (conv_wide_plain_ok(ab, wb, (int)cw) || conv_wide_extra_ok(ab, wb, (int)cw) ||
         (conv_wide_split_ok(ab, wb, (int)cw) && tuning().split_channels != 1)))
        return run_conv_packed(x_planes, ab, Wt, wb, Nb, H, W, C, Cout, acc, scale, out_f32, e, stream, 1, q->dil_h,
                               q->kh, q->kw);
    // about six wavefronts per SIMD, but at least 14 pixels each: every chunk pass reloads the
    // wavefront's weight words, which has to be spread over enough pixels (measured optimum 14-16
    // on layers of 25 k to 100 k pixels)
    int64_t rpw = tuning().rows_per_wave;
    if (rpw <= 0) {
        rpw = rows * g.col_tiles / ((int64_t)device_simd_count() * 6);
        if (rpw < 14) rpw = 14;
        // With only a few wavefronts per SIMD the kernel lasts as long as the SIMDs that got one
        // more than the others: around that count (down to 10 pixels) take the one that fills the
        // last round best (3.5 wavefronts per SIMD at 14 pixels cost 12 % on a strided ResNet layer).
        if (!g.geo.transposed) {
            const int64_t base = rpw;
            double best = -1.0;
            for (int64_t cand = (base - 4 < 10 ? 10 : base - 4); cand <= base + 2; ++cand) {
                const double avg = (double)(((rows + cand - 1) / cand) * g.col_tiles) / (double)device_simd_count();
                const double score = avg / std::ceil(avg) - 0.01 * (double)(cand > base ? cand - base : base - cand);
                if (score > best) { best = score; rpw = cand; }
            }
        }
    }
    if (g.geo.transposed && tuning().rows_per_wave <= 0) {
        // pixels of one phase per wavefront: a divisor of the phase's row length near 16, so that
        // runs do not straddle phase rows (measured on 2x2, 3x3 and 4x4 stride-2 layers), else 20
        const int64_t wp = (Wo + q->stride_w - 1) / q->stride_w;
        rpw = 20;
        int64_t best = 1 << 30;
        for (int64_t cand = 12; cand <= 32; ++cand)
            if (wp % cand == 0 && (cand > 16 ? cand - 16 : 16 - cand) < best) {
                best = cand > 16 ? cand - 16 : 16 - cand;
                rpw = cand;
            }
    }
    if (rpw > rows) rpw = rows;
    if (g.geo.transposed) {
        // The launch is phase-major: rows_per_wave counts pixels of ONE output phase, which lie
        // stride_w apart in a row and stride_h rows apart.  The output slice a wavefront addresses
        // spans at most (rpw + 3) * stride_h + 1 output rows; it has to stay below 2^31 bytes like
        // any other wavefront's slice.
        const int64_t span_rows = (rpw + 3) * (int64_t)q->stride_h + 1;
        if (span_rows > kInt31 / Wo) return QNN_EUNSUPPORTED;
        const int64_t span = span_rows * Wo;
        if (span > kInt31 || clamp_rows_for_emit(clamp_rows_per_wave((int)span, Cout), Cout, e) != (int)span)
            return QNN_EUNSUPPORTED;
        g.rows_per_wave = (int)rpw;
        g.xcd_ranges = 0; g.grid_blocks = 0;          // two-dimensional launch: plain block numbers
        set_divisors(g, true);
        return from_hip(k_conv_general[ab - 1](g, wb, (hipStream_t)stream));
    }
    g.rows_per_wave = clamp_rows_for_emit(clamp_rows_per_wave((int)rpw, Cout), Cout, e);
    g.grid_blocks = wave_grid_blocks(g);
    set_divisors(g, true);
    return from_hip(k_conv_general[ab - 1](g, wb, (hipStream_t)stream));
}

qnn_status qnn_maxpool2x2_planes(const uint32_t *planes, int64_t Nb, int64_t H, int64_t W, int64_t C, int bits,
                                 uint32_t *out_planes, void *stream) {
    if (!bits_ok(bits) || Nb < 0 || H < 0 || W < 0 || C < 0) return QNN_EINVAL;
    if ((H & 1) || (W & 1)) return QNN_EINVAL;
    if (H > kInt31 || W > kInt31 || Nb > kInt31 || C > kInt31) return QNN_EUNSUPPORTED;
    if (Nb == 0 || H == 0 || W == 0 || C == 0) return QNN_OK;
    if (Nb > kInt31 / H / W) return QNN_EUNSUPPORTED;
    if (planes == nullptr || out_planes == nullptr) return QNN_EINVAL;
    if (!aligned16(planes) || !aligned16(out_planes)) return QNN_EALIGN;
    const int64_t cw = (C + 31) / 32;
    if (Nb * H * W > (((int64_t)1 << 40) - 1) / (bits * cw)) return QNN_EUNSUPPORTED;
    return from_hip(launch_pool_planes(planes, Nb, H / 2, W / 2, cw, bits, out_planes, (hipStream_t)stream));
}

size_t qnn_compare_mfma_arranged_bytes(int64_t rows, int64_t K) {
    if (rows <= 0 || K <= 0) return 0;
    return (size_t)(((rows + 31) / 32) * ((K + 31) / 32) * 1024);
}

qnn_status qnn_compare_mfma_arrange(const int8_t *codes, int64_t rows, int64_t K, void *arranged, void *stream) {
    if (rows < 0 || K < 0) return QNN_EINVAL;
    if (rows == 0 || K == 0) return QNN_OK;
    if (codes == nullptr || arranged == nullptr) return QNN_EINVAL;
    if (!aligned16(arranged)) return QNN_EALIGN;
    if (rows > kInt31 || K > kInt31 / (127 * 127)) return QNN_EUNSUPPORTED;
    return from_hip(launch_mfma_arrange(codes, rows, K, arranged, (hipStream_t)stream));
}

qnn_status qnn_compare_mfma_gemm(const void *A_arranged, const void *Wt_arranged, int64_t M, int64_t N, int64_t K,
                                 int32_t *acc, void *stream) {
    if (M < 0 || N < 0 || K < 0) return QNN_EINVAL;
    if (M == 0 || N == 0) return QNN_OK;
    if (acc == nullptr || ((A_arranged == nullptr || Wt_arranged == nullptr) && K > 0)) return QNN_EINVAL;
    if (!aligned16(A_arranged) || !aligned16(Wt_arranged) || !aligned4(acc)) return QNN_EALIGN;
    if (M > kInt31 || N > kInt31 || K > kInt31 / (127 * 127)) return QNN_EUNSUPPORTED;
    return from_hip(launch_mfma_gemm(A_arranged, Wt_arranged, M, N, K, acc, (hipStream_t)stream));
}

qnn_status qnn_compare_dot4_gemm(const int8_t *A_codes, const int8_t *Wt_codes, int64_t M, int64_t N, int64_t K,
                                 int32_t *acc, void *stream) {
    if (M < 0 || N < 0 || K < 0) return QNN_EINVAL;
    if (M == 0 || N == 0) return QNN_OK;
    if (acc == nullptr || ((A_codes == nullptr || Wt_codes == nullptr) && K > 0)) return QNN_EINVAL;
    if (!aligned4(A_codes) || !aligned4(Wt_codes) || !aligned4(acc)) return QNN_EALIGN;
    if ((K & 3) != 0) return QNN_EUNSUPPORTED;
    if (M > kInt31 || N > kInt31 || K > kInt31 / (127 * 127)) return QNN_EUNSUPPORTED;
    return from_hip(launch_dot4_gemm(A_codes, Wt_codes, M, N, K, acc, (hipStream_t)stream));
}

qnn_status qnn_scale_epilogue(const int32_t *acc, int64_t M, int64_t N, const float *scale,
                              float *out_f32, void *stream) {
    if (M < 0 || N < 0) return QNN_EINVAL;
    if (M == 0 || N == 0) return QNN_OK;
    if (acc == nullptr || scale == nullptr || out_f32 == nullptr) return QNN_EINVAL;
    if (!aligned4(acc) || !aligned4(scale) || !aligned4(out_f32)) return QNN_EALIGN;
    if (M > (((int64_t)1 << 40) - 1) / N) return QNN_EUNSUPPORTED;
    return from_hip(launch_scale(acc, M * N, N, scale, out_f32, (hipStream_t)stream));
}

}  // extern "C"
