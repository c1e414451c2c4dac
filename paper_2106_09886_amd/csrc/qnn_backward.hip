// Backward propagation through the multi-branch product of a fully connected layer (Alg. 1,
// backward lines) and the SGD form of Update().  Not on the inference path.
//
// With g_ahat[i][n] = scale[n] * g_a[i][n] (Alg. 1 scales the incoming gradient first), the
// gradient of the encoded activation element m and of the binary weight element k are
//     g_{a^{mb}}[i][c] = sum_k 2^(m+k-2) sum_n g_ahat[i][n] W^{kb}[n][c] = 2^(m-1) sum_n g_ahat[i][n] w[n][c]
//     g_{W^{kb}}[n][c] = sum_m 2^(m+k-2) sum_i g_ahat[i][n] a^{mb}[i][c] = 2^(k-1) sum_i g_ahat[i][n] a[i][c]
// with w, a the odd-integer codes the elements add up to (Eq. (7)).  Both are one real matrix
// times one code matrix that is stored as bit planes, so one kernel serves both:
//     out[p][r][c] = 2^p * sum_j G(r, j) * code[j][c],    code[j][c] = sum_q 2^q (2 bit_q(j, c) - 1),
// G(r, j) = g[r][j] * scale[j] (towards the activations: r = i, j = n) or g[j][r] * scale[r]
// (towards the weights: r = n, j = i).  The contraction is dense and real-valued: it runs on the
// matrix cores in binary32 (v_mfma_f32_32x32x2_f32); the codes are decoded from the planes in
// registers (exact in binary32), 1/32 of the bytes a real operand would take.
#include "qnn_internal.h"
#include "qnn_device_util.h"

namespace qnn {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct BackArgs {
    const float *g;          // incoming gradient, row stride ldg
    const float *scale;      // per output channel n of the layer, or nullptr
    const uint32_t *planes;  // [J][CB][Cw]
    float *out;              // [P][R][C]
    int R, J, C, Cw, P, col_blocks;
    int64_t ldg;
};

// A block of four wavefronts takes 32*RT rows x 128 columns of the output; wavefront v the 32
// columns of plane word 4*cb + v.  One iteration takes eight reduction indices: lanes 0..31 hold
// j0..j0+3, lanes 32..63 j0+4..j0+7, and the u-th of four matrix instructions pairs j0+u with
// j0+4+u (any pairing is right as long as both operands use it).
//   A operand (32 x 2): lane l supplies row l % 32, reduction index l / 32.
//   B operand (2 x 32): lane l supplies column l % 32, reduction index l / 32.
//   D (32 x 32, 16 registers): register v of lane l is row 8 * (v / 4) + 4 * (l / 32) + v % 4, column l % 32.
// GT: g is indexed [j][r] (gradient of the weights) instead of [r][j].
// VEC (only without GT): J is a multiple of 8, ldg of 4 and g, scale are 16-byte aligned: the four
// values of a lane are one 16-byte load.
template <int CB, int RT, bool GT, bool VEC>
__global__ __launch_bounds__(256) void backward_gemm_kernel(const BackArgs a) {
    const int wave = (int)(threadIdx.x >> 6), lane = (int)(threadIdx.x & 63);
    const int half = lane >> 5, l5 = lane & 31;
    const int rb = (int)(blockIdx.x / (unsigned)a.col_blocks);
    const int cb = (int)(blockIdx.x - (unsigned)rb * (unsigned)a.col_blocks);
    const int r0 = rb * (32 * RT);
    const int cw = cb * 4 + wave;
    if (cw >= a.Cw) return;                              // no barrier in this kernel
    f32x16 acc[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;
    int rowc[RT];                                        // the lane's A row, clamped for the loads
    float srow[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        const int row = r0 + t * 32 + l5;
        rowc[t] = row < a.R ? row : a.R - 1;
        srow[t] = (GT && a.scale != nullptr) ? a.scale[rowc[t]] : 1.0f;
    }
    constexpr int kOffset = (1 << CB) - 1;
    for (int j0 = 0; j0 < a.J; j0 += 8) {
        const int jb = j0 + 4 * half;
        float av[RT][4], bv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int j = jb + u;
            const int jc = j < a.J ? j : a.J - 1;
            uint32_t bits = 0;
#pragma unroll
            for (int q = 0; q < CB; ++q) {
                const uint32_t w = a.planes[((int64_t)jc * CB + q) * a.Cw + cw];
                bits |= ((w >> l5) & 1u) << q;
            }
            bv[u] = (float)(2 * (int)bits - kOffset);
        }
        if constexpr (VEC) {
            f32x4 sv = {1.0f, 1.0f, 1.0f, 1.0f};
            if (a.scale != nullptr) sv = *reinterpret_cast<const f32x4 *>(a.scale + jb);
#pragma unroll
            for (int t = 0; t < RT; ++t) {
                const f32x4 gv = *reinterpret_cast<const f32x4 *>(a.g + (int64_t)rowc[t] * a.ldg + jb);
#pragma unroll
                for (int u = 0; u < 4; ++u) av[t][u] = gv[u] * sv[u];
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = jb + u;
                const bool jok = j < a.J;
                const int jc = jok ? j : a.J - 1;
                const float sj = (!GT && a.scale != nullptr) ? a.scale[jc] : 1.0f;
#pragma unroll
                for (int t = 0; t < RT; ++t) {
                    const float gv = GT ? a.g[(int64_t)jc * a.ldg + rowc[t]] : a.g[(int64_t)rowc[t] * a.ldg + jc];
                    const float val = GT ? gv * srow[t] : gv * sj;
                    av[t][u] = jok ? val : 0.0f;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int t = 0; t < RT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[t][u], bv[u], acc[t], 0, 0, 0);
    }
    const int col = cw * 32 + l5;
    if (col >= a.C) return;
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = r0 + t * 32 + 8 * (v / 4) + 4 * half + (v % 4);
            if (row < a.R) {
                float val = acc[t][v];
                for (int p = 0; p < a.P; ++p) {
                    a.out[((int64_t)p * a.R + row) * a.C + col] = val;
                    val *= 2.0f;                          // exact
                }
            }
        }
}

template <int CB, int RT, bool GT>
void launch_one(const BackArgs &a, bool vec, dim3 grid, hipStream_t s) {
    if constexpr (!GT) {
        if (vec) {
            launch_kernel((backward_gemm_kernel<CB, RT, false, true>), grid, dim3(256), 0, s, a);
            return;
        }
    }
    launch_kernel((backward_gemm_kernel<CB, RT, GT, false>), grid, dim3(256), 0, s, a);
}

template <int CB, bool GT>
hipError_t launch_cb(BackArgs a, bool vec, hipStream_t s) {
    // rows per block: 128 where that still gives two blocks per compute unit, else 64 or 32
    a.col_blocks = (a.Cw + 3) / 4;
    const int64_t want = 2 * (int64_t)device_simd_count() / 4;
    auto blocks = [&](int rt) { return ((int64_t)a.R + 32 * rt - 1) / (32 * rt) * a.col_blocks; };
    const int rt = blocks(4) >= want ? 4 : blocks(2) >= want ? 2 : 1;
    const int64_t nb = blocks(rt);
    if (nb > 0x7fffffff) return hipErrorInvalidValue;
    const dim3 grid((unsigned)nb);
    if (rt == 4) launch_one<CB, 4, GT>(a, vec, grid, s);
    else if (rt == 2) launch_one<CB, 2, GT>(a, vec, grid, s);
    else launch_one<CB, 1, GT>(a, vec, grid, s);
    return launch_status();
}

template <bool GT>
hipError_t launch_form(int cb, const BackArgs &a, bool vec, hipStream_t s) {
    switch (cb) {
        case 1: return launch_cb<1, GT>(a, vec, s);
        case 2: return launch_cb<2, GT>(a, vec, s);
        case 3: return launch_cb<3, GT>(a, vec, s);
        case 4: return launch_cb<4, GT>(a, vec, s);
        case 5: return launch_cb<5, GT>(a, vec, s);
        case 6: return launch_cb<6, GT>(a, vec, s);
        case 7: return launch_cb<7, GT>(a, vec, s);
        case 8: return launch_cb<8, GT>(a, vec, s);
    }
    return hipErrorInvalidValue;
}

// w <- w - lr * g: one binary32 multiply, one subtraction (no fused multiply-add)
__global__ __launch_bounds__(256) void update_sgd_kernel(float *__restrict__ w, const float *__restrict__ g, int64_t n, float lr) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
        w[i] = __fsub_rn(w[i], __fmul_rn(lr, g[i]));
}

}  // namespace

// out[p][r][c] = 2^p sum_j G(r, j) code[j][c]; towards_weights selects G(r, j) = g[j][r] scale[r],
// else g[r][j] scale[j].  R, C >= 1; J may be 0 (the output is then zero).
hipError_t launch_backward_gemm(const float *g, int64_t ldg, const float *scale, const uint32_t *planes, int code_bits,
                                int R, int J, int C, int P, bool towards_weights, float *out, hipStream_t s) {
    BackArgs a;
    a.g = g; a.scale = scale; a.planes = planes; a.out = out;
    a.R = R; a.J = J; a.C = C; a.Cw = (C + 31) / 32; a.P = P; a.col_blocks = 0; a.ldg = ldg;
    const bool vec = !towards_weights && J % 8 == 0 && ldg % 4 == 0 && ((((uintptr_t)g) & 15u) == 0) &&
                     (scale == nullptr || (((uintptr_t)scale) & 15u) == 0);
    return towards_weights ? launch_form<true>(code_bits, a, vec, s) : launch_form<false>(code_bits, a, vec, s);
}

hipError_t launch_update_sgd(float *w, const float *g, int64_t n, float lr, hipStream_t s) {
    const int64_t want = (n + 255) / 256;
    const int64_t cap = (int64_t)device_simd_count() * 16;
    launch_kernel(update_sgd_kernel, dim3((unsigned)(want < cap ? want : cap)), dim3(256), 0, s, w, g, n, lr);
    return launch_status();
}

}  // namespace qnn
