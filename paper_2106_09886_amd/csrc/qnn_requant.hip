// Re-encoding between layers (paper Alg. 1 forward: a_l -> MBitEncoder(a_l); Table 2 as a
// look-up rule): optional 2x2 max-pool of the scaled fp32 activations, mapping of each real
// value to the odd code grid, and direct emission of the next layer's per-pixel bit planes.
//
//   a = |y|;  c = min(2*floor(a/2) + 1, 2^bits - 1);  code = (y > 0) ? +c : -c
// reproduces the four intervals of Table 2 (scaled by 2^bits - 1) with their printed
// closures; zero maps to -1.  All steps are exact in binary32 (halving, floor, doubling of
// values below 2^24; larger magnitudes clamp), so the decision equals the one taken in
// double precision on the same binary32 input.
//
// One wavefront handles one output pixel and 64 channels (lane = channel): the loads are
// contiguous 256-byte rows, and plane p of the 64 codes is the 64-bit ballot of "digit p of
// u = (code + 2^bits - 1)/2 is set", i.e. two packed words at once.  HBM-bound: 4 (16 with
// pooling) bytes in and bits/8 (+1 with codes) bytes out per output element.
#include "qnn_internal.h"

namespace qnn {
namespace {

template <int BITS>
__device__ __forceinline__ int round_odd(float y) {
    constexpr float CMAX = (float)((1 << BITS) - 1);
    const float a = fabsf(y);
    float c = 2.0f * floorf(a * 0.5f) + 1.0f;
    c = (c <= CMAX) ? c : CMAX;                 // also catches inf / nan
    return (y > 0.0f) ? (int)c : -(int)c;
}

template <typename CodeT, int BITS, bool POOL>
__global__ __launch_bounds__(256) void requant_pack_kernel(const float *__restrict__ y, int64_t out_pixels,
                                                           int Ho, int Wo, int C,
                                                           CodeT *__restrict__ codes,
                                                           uint32_t *__restrict__ planes) {
    constexpr int VMAX = (1 << BITS) - 1;
    const int lane = (int)(threadIdx.x & 63);
    const int cgroups = (C + 63) / 64;
    const int Cw = (C + 31) / 32;
    const int64_t items = out_pixels * cgroups;
    const int64_t wave0 = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x >> 6);
    for (int64_t it = wave0; it < items; it += nwaves) {
        const int64_t pix = it / cgroups;
        const int cg = (int)(it - pix * cgroups);
        const int c = cg * 64 + lane;
        const bool valid = c < C;
        float v = 0.0f;
        if (valid) {
            if (POOL) {
                const int64_t n = pix / ((int64_t)Ho * Wo);
                const int64_t rem = pix - n * (int64_t)Ho * Wo;
                const int oh = (int)(rem / Wo), ow = (int)(rem - (int64_t)oh * Wo);
                const int W = 2 * Wo;
                const float *p00 = y + (((n * 2 * Ho + 2 * oh) * W) + 2 * ow) * (int64_t)C + c;
                v = p00[0];
                const float v01 = p00[C], v10 = p00[(int64_t)W * C], v11 = p00[(int64_t)W * C + C];
                if (v01 > v) v = v01;
                if (v10 > v) v = v10;
                if (v11 > v) v = v11;
            } else {
                v = y[pix * (int64_t)C + c];
            }
        }
        const int code = round_odd<BITS>(v);
        if (codes != nullptr && valid) codes[pix * (int64_t)C + c] = (CodeT)code;
        if (planes != nullptr) {
            const int u = (code + VMAX) >> 1;
            uint32_t *dst = planes + pix * (int64_t)BITS * Cw + 2 * cg;
#pragma unroll
            for (int p = 0; p < BITS; ++p) {
                const uint64_t mask = __ballot(valid && ((u >> p) & 1));
                if (lane == 0) {
                    dst[(int64_t)p * Cw] = (uint32_t)mask;
                    if (2 * cg + 1 < Cw) dst[(int64_t)p * Cw + 1] = (uint32_t)(mask >> 32);
                }
            }
        }
    }
}

template <typename CodeT, int BITS>
hipError_t launch_rq(const float *y, int64_t out_pixels, int Ho, int Wo, int C, bool pool, void *codes,
                     uint32_t *planes, unsigned blocks, hipStream_t s) {
    if (pool)
        hipLaunchKernelGGL((requant_pack_kernel<CodeT, BITS, true>), dim3(blocks), dim3(256), 0, s, y,
                           out_pixels, Ho, Wo, C, (CodeT *)codes, planes);
    else
        hipLaunchKernelGGL((requant_pack_kernel<CodeT, BITS, false>), dim3(blocks), dim3(256), 0, s, y,
                           out_pixels, Ho, Wo, C, (CodeT *)codes, planes);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_requant(const float *y, int64_t Nb, int64_t H, int64_t W, int64_t C, bool pool, int bits,
                          void *codes, uint32_t *planes, hipStream_t s) {
    const int Ho = (int)(pool ? H / 2 : H), Wo = (int)(pool ? W / 2 : W);
    const int64_t out_pixels = Nb * Ho * (int64_t)Wo;
    const int64_t items = out_pixels * ((C + 63) / 64);
    if (items == 0) return hipSuccess;
    const int64_t want = (items + 3) / 4;
    const unsigned blocks = (unsigned)(want < (int64_t)1 << 18 ? want : (int64_t)1 << 18);
#define QNN_RQ(B, T) case B: return launch_rq<T, B>(y, out_pixels, Ho, Wo, (int)C, pool, codes, planes, blocks, s)
    switch (bits) {
        QNN_RQ(1, int8_t); QNN_RQ(2, int8_t); QNN_RQ(3, int8_t); QNN_RQ(4, int8_t);
        QNN_RQ(5, int8_t); QNN_RQ(6, int8_t); QNN_RQ(7, int8_t); QNN_RQ(8, int16_t);
    }
#undef QNN_RQ
    return hipErrorInvalidValue;
}

}  // namespace qnn
