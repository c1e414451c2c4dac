// Internal declarations shared by the translation units of libqnn (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "qnn.h"

namespace qnn {

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
    int rows;             // GEMM rows / output pixels
    int N;                // output columns / filters
    int Cw;               // words per (row, plane)
    int H, W;             // image height and width in pixels (convolution only)
    int C;                // input channels (small-channel convolution only)
    int kconst;           // (true K of one tap) * (2^AB - 1) * (2^WB - 1)
    int rows_per_wave;    // contiguous rows handled by one wavefront
    int col_tiles;        // ceil(N / 64)
    int split_k;          // GEMM only: K chunks split over the wavefronts of a block; then
                          // rows_per_wave is the number of rows per BLOCK
    uint64_t *trace;      // optional per-wavefront trace records (4 x uint64 each), or nullptr
    uint32_t trace_waves; // capacity of `trace` in wavefronts
    uint32_t *planes_out; // optional: the scaled result re-encoded with out_bits bits, as bit planes
                          // uint32 [rows][out_bits][ceil(N/32)] (the next layer's activations)
    int out_bits;
};

struct Tuning {
    int waves_per_simd;   // target resident wavefronts per SIMD when sizing rows_per_wave
    int rows_per_wave;    // > 0 overrides the automatic choice
    uint64_t *trace;      // device buffer for per-wavefront trace records, or nullptr
    uint32_t trace_waves;
};
Tuning &tuning();

int device_simd_count();  // 4 * number of compute units of the current device (cached)
// K words per weight chunk of the GEMM kernels (GemmShape::KC in qnn_branch.hip)
inline int gemm_chunk_words(int wb) { return (wb == 1) ? 64 : (wb == 2) ? 32 : (wb <= 4) ? 16 : 8; }

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
                          void *codes, uint32_t *planes, hipStream_t);
hipError_t launch_pool_planes(const uint32_t *planes, int64_t Nb, int64_t Ho, int64_t Wo, int64_t Cw, int bits,
                              uint32_t *out, hipStream_t);
hipError_t launch_scale(const int32_t *acc, int64_t total, int64_t N, const float *scale,
                        float *out, hipStream_t);

}  // namespace qnn
