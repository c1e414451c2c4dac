// Comparison line only: the SAME integer product of decoded codes evaluated on the int8 matrix
// cores (v_mfma_i32_32x32x32_i8) instead of through the {-1,+1} decomposition.  Nothing of the
// method's path uses this file; bench.py reports its rate next to the branch GEMM so that the
// cost of the decomposition on this chip can be read off.  Written for clarity, not tuned:
// operands are pre-arranged into matrix-core fragment order so that every fragment is one
// coalesced 1 KiB load, there is no LDS stage, and a wavefront owns a 128 x 64 output tile
// (8 accumulator tiles).
//
// Fragment order.  A 32-row x 32-k block of int8 is stored as 64 x 16 bytes: entry l holds
// row (l % 32), k = 16*(l / 32) .. +15 of the block.  Both operands use the same arrangement, so
// whatever order the instruction assigns to the 16 bytes of a lane inside the k axis, the two
// operands agree on it and the sum over k is the same.  The 32 x 32 int32 result tile has the
// usual layout: lane l holds column l % 32, rows 8*(v / 4) + 4*(l / 32) + (v % 4), v = 0..15.
#include "qnn_internal.h"

namespace qnn {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// codes int8 [rows][K] -> fragments [ceil(rows/32)][ceil(K/32)][64][16 bytes], zero padded
__global__ __launch_bounds__(256) void mfma_arrange_kernel(const int8_t *__restrict__ codes, int64_t rows, int64_t K,
                                                           int64_t row_blocks, int64_t k_blocks,
                                                           v4i *__restrict__ out) {
    const int64_t total = row_blocks * k_blocks * 64;
    for (int64_t it = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; it < total;
         it += (int64_t)gridDim.x * blockDim.x) {
        const int l = (int)(it & 63);
        const int64_t blk = it >> 6;
        const int64_t kb = blk % k_blocks, rb = blk / k_blocks;
        const int64_t row = rb * 32 + (l & 31);
        const int64_t k0 = kb * 32 + 16 * (l >> 5);
        union { int8_t b[16]; v4i v; } u;
#pragma unroll
        for (int j = 0; j < 16; ++j) u.b[j] = (row < rows && k0 + j < K) ? codes[row * K + k0 + j] : (int8_t)0;
        out[it] = u.v;
    }
}

constexpr int kTilesM = 4, kTilesN = 2;      // 32x32 tiles per wavefront: 128 rows x 64 columns

// A, B in fragment order; C int32 [M][N] row-major.  Grid: one wavefront per 128 x 64 tile.
__global__ __launch_bounds__(256) void mfma_gemm_kernel(const v4i *__restrict__ A, const v4i *__restrict__ B,
                                                        int M, int N, int64_t k_blocks, int64_t tiles_n,
                                                        int64_t wave_tiles, int32_t *__restrict__ C) {
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wave >= wave_tiles) return;
    const int lane = (int)(threadIdx.x & 63);
    // the four wavefronts of a block sit 2 x 2, so that each A and B fragment is used twice per block
    const int64_t blocks_n = (tiles_n + 1) / 2;
    const int64_t blk = wave >> 2;
    const int64_t tm = (blk / blocks_n) * 2 + ((wave >> 1) & 1);
    const int64_t tn = (blk % blocks_n) * 2 + (wave & 1);
    if (tn >= tiles_n) return;
    v16i acc[kTilesM][kTilesN];
#pragma unroll
    for (int i = 0; i < kTilesM; ++i)
#pragma unroll
        for (int j = 0; j < kTilesN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
    const int64_t rbm = (int64_t)((M + 31) / 32), rbn = (int64_t)((N + 31) / 32);
    const v4i zero = {0, 0, 0, 0};
    for (int64_t kb = 0; kb < k_blocks; ++kb) {
        v4i a[kTilesM], b[kTilesN];
#pragma unroll
        for (int i = 0; i < kTilesM; ++i) {
            const int64_t rb = tm * kTilesM + i;
            a[i] = (rb < rbm) ? A[(rb * k_blocks + kb) * 64 + lane] : zero;
        }
#pragma unroll
        for (int j = 0; j < kTilesN; ++j) {
            const int64_t cb = tn * kTilesN + j;
            b[j] = (cb < rbn) ? B[(cb * k_blocks + kb) * 64 + lane] : zero;
        }
#pragma unroll
        for (int i = 0; i < kTilesM; ++i)
#pragma unroll
            for (int j = 0; j < kTilesN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < kTilesM; ++i)
#pragma unroll
        for (int j = 0; j < kTilesN; ++j) {
            const int64_t col = (tn * kTilesN + j) * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = (tm * kTilesM + i) * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
                if (row < M && col < N) C[row * N + col] = acc[i][j][v];
            }
        }
}

}  // namespace

hipError_t launch_mfma_arrange(const int8_t *codes, int64_t rows, int64_t K, void *out, hipStream_t s) {
    const int64_t rb = (rows + 31) / 32, kb = (K + 31) / 32;
    const int64_t total = rb * kb * 64;
    if (total == 0) return hipSuccess;
    const int64_t want = (total + 255) / 256;
    const unsigned blocks = (unsigned)(want < (int64_t)1 << 20 ? want : (int64_t)1 << 20);
    launch_kernel(mfma_arrange_kernel, dim3(blocks), dim3(256), 0, s, codes, rows, K, rb, kb, (v4i *)out);
    return launch_status();
}

hipError_t launch_mfma_gemm(const void *A, const void *B, int64_t M, int64_t N, int64_t K, int32_t *C,
                            hipStream_t s) {
    const int64_t kb = (K + 31) / 32;
    const int64_t tiles_m = (M + 32 * kTilesM - 1) / (32 * kTilesM), tiles_n = (N + 32 * kTilesN - 1) / (32 * kTilesN);
    const int64_t blocks_m = (tiles_m + 1) / 2, blocks_n = (tiles_n + 1) / 2;
    const int64_t blocks = blocks_m * blocks_n;
    if (blocks == 0) return hipSuccess;
    launch_kernel(mfma_gemm_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (const v4i *)A, (const v4i *)B, (int)M,
                       (int)N, kb, tiles_n, blocks * 4, C);
    return launch_status();
}

}  // namespace qnn
