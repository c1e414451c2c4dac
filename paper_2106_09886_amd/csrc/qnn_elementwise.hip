// Element-wise pieces of the paper's training procedures (Sec. 4): the derivative of the M-bit
// encoder (Eq. (12), Alg. 1's BackMBitEncoder), the weight binarisation of Eq. (14) with its
// gradient, and the linear quantiser of Eq. (15) with its straight-through gradient.  All of them
// stream through memory once; none is part of the inference path.
#include "qnn_internal.h"
#include "qnn_device_util.h"

namespace qnn {
namespace {

constexpr int kBlock = 256;

inline unsigned blocks_for(int64_t n, int per_thread = 1) {
    const int64_t want = (n + (int64_t)kBlock * per_thread - 1) / ((int64_t)kBlock * per_thread);
    const int64_t cap = (int64_t)device_simd_count() * 16;           // grid-stride beyond that
    return (unsigned)(want < cap ? (want < 1 ? 1 : want) : cap);
}

// g_x[i] = sum_m g[m-1][i] * d phi_M^m / dx (x[i]);  d phi_M^m / dx = +-c_m pi cos(c_m pi x) on
// [-1, 1] (+ for the high bit m = M), 0 outside, c_m = (2^M - 1) / 2^m.  The cosine is taken in
// double precision of the exactly representable product c_m * x (cospi reduces the period exactly),
// so the result is the correctly rounded sum up to a few units of the last binary32 place.
template <int M>
__global__ __launch_bounds__(kBlock) void encoder_backward_kernel(const float *__restrict__ x, const float *__restrict__ g,
                                                                   int64_t n, float *__restrict__ gx) {
    constexpr double kPi = 3.14159265358979323846;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock) {
        const float xv = x[i];
        double acc = 0.0;
        if (xv >= -1.0f && xv <= 1.0f) {
#pragma unroll
            for (int m = 1; m <= M; ++m) {
                constexpr double scale = (double)((1 << M) - 1);
                const double c = scale / (double)(1 << m);
                const double d = c * kPi * cospi(c * (double)xv);
                const double gm = (double)g[(int64_t)(m - 1) * n + i];
                acc += (m == M) ? gm * d : -(gm * d);
            }
        }
        gx[i] = (float)acc;
    }
}

// Binarize(w) = sign(HTanh(w)), sign(0) = +1.  One wavefront per 64 consecutive weights of a row:
// the plane words are the ballot of w >= 0 (bit 1 <=> +1), columns past K contribute 0.
__global__ __launch_bounds__(kBlock) void binarize_kernel(const float *__restrict__ w, int64_t rows, int K, int groups,
                                                           int8_t *__restrict__ codes, uint32_t *__restrict__ planes) {
    const int lane = (int)(threadIdx.x & 63);
    const int Kw = (K + 31) >> 5;
    const int64_t items = rows * groups;
    for (int64_t it = (int64_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6); it < items;
         it += (int64_t)gridDim.x * (kBlock / 64)) {
        const int64_t row = it / groups;
        const int gidx = (int)(it - row * groups);
        const int col = gidx * 64 + lane;
        const bool ok = col < K;
        const float v = ok ? w[row * K + col] : -1.0f;
        const bool plus = ok && (v >= 0.0f);
        const uint64_t mask = __ballot(plus);
        if (codes != nullptr && ok) codes[row * K + col] = plus ? (int8_t)1 : (int8_t)-1;
        if (planes != nullptr && lane < 2 && 2 * gidx + lane < Kw)
            planes[row * Kw + 2 * gidx + lane] = (uint32_t)(mask >> (32 * lane));
    }
}

__global__ __launch_bounds__(kBlock) void binarize_backward_kernel(const float *__restrict__ w, const float *__restrict__ g_wb,
                                                                    int64_t n, float *__restrict__ g_w) {
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock) {
        const float v = w[i];
        g_w[i] = (v >= -1.0f && v <= 1.0f) ? g_wb[i] : 0.0f;
    }
}

// Quantize_K: round(clamp(x / t, 1) * nlev) * d, nlev = 2^(K-1) - 1, d = t / nlev; each step one
// binary32 operation (IEEE division, clamp, multiply, round to nearest even, multiply).
__global__ __launch_bounds__(kBlock) void quantize_k_kernel(const float *__restrict__ x, int64_t n, float t, float nlev, float d,
                                                             float *__restrict__ q, int32_t *__restrict__ levels) {
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock) {
        float c = __fdiv_rn(x[i], t);
        if (!(c <= 1.0f)) c = 1.0f;                  // a NaN clamps to +1 as well
        if (c < -1.0f) c = -1.0f;
        const float k = rintf(__fmul_rn(c, nlev));
        if (q != nullptr) q[i] = __fmul_rn(k, d);
        if (levels != nullptr) levels[i] = (int32_t)k;
    }
}

__global__ __launch_bounds__(kBlock) void quantize_k_backward_kernel(const float *__restrict__ x, const float *__restrict__ g_q,
                                                                      int64_t n, float t, float *__restrict__ g_x) {
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock) {
        const float r = __fdiv_rn(x[i], t);
        g_x[i] = (r >= -1.0f && r <= 1.0f) ? g_q[i] : 0.0f;
    }
}

}  // namespace

hipError_t launch_encoder_backward(const float *x, const float *g, int64_t n, int bits, float *gx, hipStream_t s) {
    const unsigned blocks = blocks_for(n);
#define QNN_EB(M) case M: launch_kernel((encoder_backward_kernel<M>), dim3(blocks), dim3(kBlock), 0, s, x, g, n, gx); break
    switch (bits) {
        QNN_EB(1); QNN_EB(2); QNN_EB(3); QNN_EB(4); QNN_EB(5); QNN_EB(6); QNN_EB(7); QNN_EB(8);
        default: return hipErrorInvalidValue;
    }
#undef QNN_EB
    return launch_status();
}

hipError_t launch_binarize(const float *w, int64_t rows, int64_t K, int8_t *codes, uint32_t *planes, hipStream_t s) {
    const int groups = (int)((K + 63) / 64);
    launch_kernel(binarize_kernel, dim3(blocks_for(rows * groups * 64)), dim3(kBlock), 0, s, w, rows, (int)K, groups, codes,
                       planes);
    return launch_status();
}

hipError_t launch_binarize_backward(const float *w, const float *g_wb, int64_t n, float *g_w, hipStream_t s) {
    launch_kernel(binarize_backward_kernel, dim3(blocks_for(n)), dim3(kBlock), 0, s, w, g_wb, n, g_w);
    return launch_status();
}

hipError_t launch_quantize_k(const float *x, int64_t n, int bits, float t, float *q, int32_t *levels, hipStream_t s) {
    const float nlev = (float)((1 << (bits - 1)) - 1);
    const float d = t / nlev;                        // one binary32 division on the host, as in the definition
    launch_kernel(quantize_k_kernel, dim3(blocks_for(n)), dim3(kBlock), 0, s, x, n, t, nlev, d, q, levels);
    return launch_status();
}

hipError_t launch_quantize_k_backward(const float *x, const float *g_q, int64_t n, float t, float *g_x, hipStream_t s) {
    launch_kernel(quantize_k_backward_kernel, dim3(blocks_for(n)), dim3(kBlock), 0, s, x, g_q, n, t, g_x);
    return launch_status();
}

}  // namespace qnn
