// Stand-alone scale epilogue (paper Eq. (9)): out[i][j] = (float)acc[i][j] * scale[j].
// HBM-bound: 4 bytes in, 4 bytes out per element; 16-byte accesses where N allows.
#include "qnn_internal.h"

namespace qnn {
namespace {

__global__ __launch_bounds__(256) void scale_kernel_v4(const int4 *__restrict__ acc, int64_t total4,
                                                       int N4, const float4 *__restrict__ scale,
                                                       float4 *__restrict__ out) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total4;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int4 a = acc[i];
        const float4 s = scale[i % N4];
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        f32x4 o;
        o.x = (float)a.x * s.x;
        o.y = (float)a.y * s.y;
        o.z = (float)a.z * s.z;
        o.w = (float)a.w * s.w;
        __builtin_nontemporal_store(o, reinterpret_cast<f32x4 *>(out + i));   // streamed: nothing reads it back here
    }
}

__global__ __launch_bounds__(256) void scale_kernel(const int32_t *__restrict__ acc, int64_t total,
                                                    int64_t N, const float *__restrict__ scale,
                                                    float *__restrict__ out) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x)
        __builtin_nontemporal_store((float)acc[i] * scale[i % N], &out[i]);
}

}  // namespace

hipError_t launch_scale(const int32_t *acc, int64_t total, int64_t N, const float *scale,
                        float *out, hipStream_t s) {
    if (total == 0) return hipSuccess;
    const bool v4 = (N % 4 == 0) && ((((uintptr_t)acc) | ((uintptr_t)scale) | ((uintptr_t)out)) & 15u) == 0;
    const int64_t work = v4 ? total / 4 : total;
    const int64_t want = (work + 255) / 256;
    const unsigned blocks = (unsigned)(want < 65536 ? want : 65536);
    if (v4)
        launch_kernel(scale_kernel_v4, dim3(blocks), dim3(256), 0, s, (const int4 *)acc, work,
                           (int)(N / 4), (const float4 *)scale, (float4 *)out);
    else
        launch_kernel(scale_kernel, dim3(blocks), dim3(256), 0, s, acc, total, N, scale, out);
    return launch_status();
}

}  // namespace qnn
