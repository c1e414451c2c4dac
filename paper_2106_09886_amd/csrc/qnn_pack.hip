// Encode + pack kernel (paper Eq. (7); "store those numbers by bits", Sec. 5.4).
//
// A code v = sum_m 2^(m-1) c_m with c_m = +-1 has c_m = +1 exactly where binary digit m-1 of
// u = (v + 2^bits - 1) / 2 is set, so plane p of the output is digit p of u.  One thread
// produces the `bits` words of one (row, 32-element group): it reads its 32 codes (two 16-byte
// loads on the aligned fast path) and writes one word per plane.  HBM-bound: 1 (or 2) bytes in
// and bits/8 bytes out per code.
#include "qnn_internal.h"

namespace qnn {
namespace {

template <typename CodeT>
__device__ __forceinline__ void pack_one(int v, int bits, int vmax, int k, bool validate,
                                         uint32_t (&word)[8], int &bad) {
    const int u = (v + vmax) >> 1;
    bool ok = true;
    if (validate) ok = ((v & 1) != 0) && (v >= -vmax) && (v <= vmax);
    if (validate && !ok) { ++bad; return; }
#pragma unroll
    for (int p = 0; p < 8; ++p)
        if (p < bits) word[p] |= (uint32_t)((u >> p) & 1) << k;
}

template <typename CodeT, bool VALIDATE>
__global__ __launch_bounds__(256) void pack_kernel(const CodeT *__restrict__ codes, int64_t rows,
                                                   int K, int Kw, int bits,
                                                   uint32_t *__restrict__ planes,
                                                   int32_t *__restrict__ bad_count) {
    const int64_t total = rows * (int64_t)Kw;
    const int vmax = (1 << bits) - 1;
    int bad = 0;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = idx / Kw;
        const int wi = (int)(idx - row * Kw);
        const int kbeg = wi * 32;
        const int cnt = min(32, K - kbeg);
        const CodeT *src = codes + row * (int64_t)K + kbeg;
        uint32_t word[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
        const bool aligned = (cnt == 32) && ((((uintptr_t)src) & 15u) == 0);
        if (aligned) {
            constexpr int PER = 16 / (int)sizeof(CodeT);     // codes per 16-byte load
            constexpr int NLD = 32 / PER;
            const uint4 *s4 = reinterpret_cast<const uint4 *>(src);
#pragma unroll
            for (int l = 0; l < NLD; ++l) {
                const uint4 q = s4[l];
                const uint32_t lanes[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int e = 0; e < PER; ++e) {
                    int v;
                    if (sizeof(CodeT) == 1) v = (int)(int8_t)(lanes[e >> 2] >> (8 * (e & 3)));
                    else v = (int)(int16_t)(lanes[e >> 1] >> (16 * (e & 1)));
                    pack_one<CodeT>(v, bits, vmax, l * PER + e, VALIDATE, word, bad);
                }
            }
        } else {
            for (int k = 0; k < cnt; ++k) pack_one<CodeT>((int)src[k], bits, vmax, k, VALIDATE, word, bad);
        }
        uint32_t *dst = planes + (row * bits) * (int64_t)Kw + wi;
#pragma unroll
        for (int p = 0; p < 8; ++p)
            if (p < bits) dst[(int64_t)p * Kw] = word[p];
    }
    if (VALIDATE) {
        // wavefront sum, one atomic per wavefront that saw something
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) bad += __shfl_down(bad, off, 64);
        if ((threadIdx.x & 63) == 0 && bad != 0) atomicAdd(bad_count, bad);
    }
}

}  // namespace

hipError_t launch_pack(const void *codes, int code_bytes, int64_t rows, int64_t K, int bits,
                       uint32_t *planes, int32_t *bad_count, bool validate, hipStream_t s) {
    const int Kw = (int)((K + 31) / 32);
    const int64_t total = rows * (int64_t)Kw;
    if (total == 0) return hipSuccess;
    const int64_t want = (total + 255) / 256;
    const unsigned blocks = (unsigned)(want < (int64_t)1 << 20 ? want : (int64_t)1 << 20);
    if (code_bytes == 1) {
        if (validate)
            hipLaunchKernelGGL((pack_kernel<int8_t, true>), dim3(blocks), dim3(256), 0, s,
                               (const int8_t *)codes, rows, (int)K, Kw, bits, planes, bad_count);
        else
            hipLaunchKernelGGL((pack_kernel<int8_t, false>), dim3(blocks), dim3(256), 0, s,
                               (const int8_t *)codes, rows, (int)K, Kw, bits, planes, bad_count);
    } else {
        if (validate)
            hipLaunchKernelGGL((pack_kernel<int16_t, true>), dim3(blocks), dim3(256), 0, s,
                               (const int16_t *)codes, rows, (int)K, Kw, bits, planes, bad_count);
        else
            hipLaunchKernelGGL((pack_kernel<int16_t, false>), dim3(blocks), dim3(256), 0, s,
                               (const int16_t *)codes, rows, (int)K, Kw, bits, planes, bad_count);
    }
    return hipGetLastError();
}

}  // namespace qnn
