// Comparison line only: the SAME integer product of decoded codes evaluated with the packed
// int8 dot-product instruction of the vector ALU (v_dot4_i32_i8: four multiply-adds per lane and
// instruction) instead of through the {-1,+1} decomposition.  Nothing of the method's path uses
// this file; bench.py reports its rate next to the branch GEMM.  Same mapping as the branch
// GEMM: lane = output column, the chunk's weight words (four codes each) in vector registers,
// the row's activation words wave-uniform through scalar loads, partial sums of a group of rows
// in LDS while the chunks go by.  Written for clarity, not tuned (the scalar loads of a row are
// not overlapped with the previous row's products).  A xor/popcount pair covers 32 elements of
// ONE branch, so the decomposition needs ab*wb/16 instructions per element where this needs 1/4:
// equal instruction counts at ab*wb = 4, a fourfold advantage for the decomposition at one bit each.
#include "qnn_internal.h"
#include "qnn_device_util.h"

namespace qnn {
namespace {

constexpr int kDotChunk = 32;      // words (4 codes each) per weight chunk
constexpr int kDotGroupRows = 32;  // rows whose partial sums stay in LDS

__global__ __launch_bounds__(256) void dot4_gemm_kernel(const uint32_t *__restrict__ A, const uint32_t *__restrict__ Wt,
                                                        int M, int N, int K4, int rows_per_wave, int col_tiles,
                                                        int32_t *__restrict__ C) {
    __shared__ int slab[4][kDotGroupRows][64];
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    const int wave = __builtin_amdgcn_readfirstlane((int)blockIdx.x * 4 + wv);
    const int ct = wave % col_tiles, rb = wave / col_tiles;
    if ((int64_t)rb * rows_per_wave >= M) return;
    const int r0 = rb * rows_per_wave, r1 = min(M, r0 + rows_per_wave);
    const int n = ct * 64 + lane;
    const int nload = (n < N) ? n : N - 1;             // lanes past N redo column N-1 and store nothing
    uniform_words As = as_uniform(A);
    for (int g0 = r0; g0 < r1; g0 += kDotGroupRows) {
        const int g1 = min(r1, g0 + kDotGroupRows);
        for (int k0 = 0; k0 < K4; k0 += kDotChunk) {
            const bool first = (k0 == 0), last = (k0 + kDotChunk >= K4), full = (k0 + kDotChunk <= K4);
            uint32_t w[kDotChunk];
            if (full) {
                load_run<kDotChunk>(Wt + (int64_t)nload * K4 + k0, w);
            } else {
#pragma unroll
                for (int j = 0; j < kDotChunk; ++j) w[j] = (k0 + j < K4) ? Wt[(int64_t)nload * K4 + k0 + j] : 0u;
            }
            for (int r = g0; r < g1; ++r) {
                // four independent accumulators: a dot product waits for the one it accumulates onto
                int part[4] = {first ? 0 : slab[wv][r - g0][lane], 0, 0, 0};
                const int64_t row = (int64_t)r * K4 + k0;
                if (full) {
                    // the row's 32 words as two 16-word scalar loads (4-byte alignment suffices)
                    typedef uint32_t w16 __attribute__((ext_vector_type(16), aligned(4)));
                    typedef const w16 __attribute__((address_space(4))) *w16_ptr;
                    const w16 lo = *(w16_ptr)(As + row), hi = *(w16_ptr)(As + row + 16);
#pragma unroll
                    for (int j = 0; j < kDotChunk; ++j)
                        part[j & 3] = __builtin_amdgcn_sdot4((int)(j < 16 ? lo[j] : hi[j - 16]), (int)w[j], part[j & 3], false);
                } else {
#pragma unroll
                    for (int j = 0; j < kDotChunk; ++j)
                        if (k0 + j < K4) part[j & 3] = __builtin_amdgcn_sdot4((int)As[row + j], (int)w[j], part[j & 3], false);
                }
                const int acc = (part[0] + part[1]) + (part[2] + part[3]);
                if (!last) slab[wv][r - g0][lane] = acc;
                else if (n < N) C[(int64_t)r * N + n] = acc;
            }
        }
    }
}

}  // namespace

hipError_t launch_dot4_gemm(const int8_t *A, const int8_t *Wt, int64_t M, int64_t N, int64_t K, int32_t *C,
                            hipStream_t s) {
    const int col_tiles = (int)((N + 63) / 64);
    // about four wavefronts per SIMD; whole row groups once there are that many rows
    int64_t rpw = (M * col_tiles + (int64_t)device_simd_count() * 4 - 1) / ((int64_t)device_simd_count() * 4);
    if (rpw > kDotGroupRows) rpw = (rpw + kDotGroupRows - 1) / kDotGroupRows * kDotGroupRows;
    if (rpw < 8) rpw = 8;
    if (rpw > M) rpw = M;
    const int64_t row_blocks = (M + rpw - 1) / rpw;
    const int64_t waves = row_blocks * col_tiles;
    launch_kernel(dot4_gemm_kernel, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, s,
                       reinterpret_cast<const uint32_t *>(A), reinterpret_cast<const uint32_t *>(Wt), (int)M, (int)N,
                       (int)(K / 4), (int)rpw, col_tiles, C);
    return launch_status();
}

}  // namespace qnn
