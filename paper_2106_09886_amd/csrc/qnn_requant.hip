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
// One work item is one output pixel and 64 channels (lane = channel): the loads are
// contiguous 256-byte rows, and plane p of the 64 codes is the 64-bit ballot of "digit p of
// u = (code + 2^bits - 1)/2 is set", i.e. two packed words at once.  A wavefront keeps several
// items in flight.  HBM-bound: 4 (16 with pooling) bytes in and bits/8 (+1 with codes) bytes
// out per output element.  The same kernel serves the real-valued front end (qnn_encode_real):
// an optional clip to [0,1] and one binary32 multiply by 2^bits - 1 before the rule.
#include <type_traits>
#include <utility>
#include "qnn_internal.h"
#include "qnn_device_util.h"

namespace qnn {
namespace {

template <class F, int... I>
__device__ __forceinline__ void static_for_items_impl(F &&f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop whose index is a constant
template <int N, class F>
__device__ __forceinline__ void static_for_items(F &&f) {
    static_for_items_impl(f, std::make_integer_sequence<int, N>{});
}

// Stored index u = (code + 2^BITS - 1) / 2 of the rule above: with H = 2^(BITS-1) and
// f = min(floor(|y|/2), H-1),  u = f xor (y > 0 ? H : H-1)  (and code = 2u - (2^BITS - 1)).
// The range limiters of Table 1 in front of the encoder: 0 HTanh (the clamp of the rule itself),
// 1 HReLU (x <= 0 and NaN -> 0), 2 Tanh, 3 Sigmoid (binary32, device math library).
__device__ __forceinline__ float limit_range(float v, int clip) {
    if (clip == 1) return (v > 0.0f) ? v : 0.0f;
    if (clip == 2) return tanhf(v);
    if (clip == 3) return 1.0f / (1.0f + expf(-v));
    return v;
}

template <int BITS>
__device__ __forceinline__ uint32_t round_odd_index(float y) {
    constexpr uint32_t H = 1u << (BITS - 1);
    constexpr float FMAX = (float)(H - 1u) + 0.5f;
    // floor(min(|y|/2, H - 1/2)): the minimum clamps, and returns its second operand for inf / nan
    const int f = floor_to_int(__builtin_fminf(__builtin_fabsf(y) * 0.5f, FMAX));
    return (uint32_t)f ^ ((y > 0.0f) ? H : H - 1u);
}

// U work items (pixel, 64-channel group) per loop trip: all their loads are issued before any
// is consumed, so that a wavefront keeps U (4U with pooling) 256-byte rows in flight.
template <typename CodeT, int BITS, bool POOL, int U>
__global__ __launch_bounds__(256) void requant_pack_kernel(const float *__restrict__ y, int64_t out_pixels,
                                                           int Ho, int Wo, int C, float premul, int clip,
                                                           CodeT *__restrict__ codes,
                                                           uint32_t *__restrict__ planes) {
    constexpr int VMAX = (1 << BITS) - 1;
    const int lane = (int)(threadIdx.x & 63);
    const int cgroups = (C + 63) / 64;
    const int Cw = (C + 31) / 32;
    const int64_t items = out_pixels * cgroups;
    const int64_t wave0 = (int64_t)blockIdx.x * (blockDim.x >> 6) +
                          __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));      // wave-uniform
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x >> 6);
    for (int64_t it0 = wave0 * U; it0 < items; it0 += nwaves * U) {
        float v[U];
        int64_t pix[U];
        int cg[U];
        bool valid[U];
        // position of the first item, by division once per trip; the following items step from it
        int64_t cur_pix = it0 / cgroups;
        int cur_cg = (int)(it0 - cur_pix * cgroups);
        int64_t cur_n = 0;
        int cur_oh = 0, cur_ow = 0;
        if (POOL) {
            cur_n = cur_pix / ((int64_t)Ho * Wo);
            const int64_t rem = cur_pix - cur_n * (int64_t)Ho * Wo;
            cur_oh = (int)(rem / Wo);
            cur_ow = (int)(rem - (int64_t)cur_oh * Wo);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool item_ok = it0 + u < items;
            pix[u] = cur_pix;
            cg[u] = cur_cg;
            const int c = cur_cg * 64 + lane;
            valid[u] = item_ok && c < C;
            v[u] = 0.0f;
            if (valid[u]) {
                if (POOL) {
                    const int W = 2 * Wo;
                    const float *p00 = y + (((cur_n * 2 * Ho + 2 * cur_oh) * W) + 2 * cur_ow) * (int64_t)C + c;
                    float m = p00[0];
                    const float v01 = p00[C], v10 = p00[(int64_t)W * C], v11 = p00[(int64_t)W * C + C];
                    if (v01 > m) m = v01;
                    if (v10 > m) m = v10;
                    if (v11 > m) m = v11;
                    v[u] = m;
                } else {
                    v[u] = y[cur_pix * (int64_t)C + c];
                }
            }
            if (++cur_cg == cgroups) {                       // next item
                cur_cg = 0;
                ++cur_pix;
                if (POOL && ++cur_ow == Wo) {
                    cur_ow = 0;
                    if (++cur_oh == Ho) { cur_oh = 0; ++cur_n; }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (it0 + u >= items) break;                    // wave-uniform
            // real-valued front end (Table 1, Table 2): clip to [0,1] if asked, then one binary32
            // multiply by 2^bits - 1 brings the number space onto the code grid (re-encoding: x 1)
            const float val = limit_range(v[u], clip);
            const uint32_t uidx = valid[u] ? round_odd_index<BITS>(val * premul) : 0u;   // 0: all plane bits clear
            const int c = cg[u] * 64 + lane;
            if (codes != nullptr && valid[u]) codes[pix[u] * (int64_t)C + c] = (CodeT)(2 * (int)uidx - VMAX);
            if (planes != nullptr) {
                // index at the top of the register; each doubling shifts out one plane, high plane
                // first, as the carry mask of the wavefront = the plane's two packed words
                const int mine = emit_planes<BITS>(uidx << (32 - BITS));
                const int p = BITS - 1 - (lane >> 1), h = lane & 1;
                if (lane < 2 * BITS && 2 * cg[u] + h < Cw)
                    planes[(pix[u] * BITS + p) * (int64_t)Cw + 2 * cg[u] + h] = (uint32_t)mine;
            }
        }
    }
}

// Planes of one item into lanes 2*ITEM and 2*ITEM+1 of P[k] (step k carries plane BITS-1-k, as in
// emit_planes): after the U items of a trip, lane 2u+h of P[k] holds half h of that plane of item u,
// and one store per plane writes the trip's words of the plane, which are consecutive in memory
// wherever the items are consecutive channel groups of one pixel.  One asm statement for the
// doublings and one per (at most) four planes for the lane writes, as in emit_planes.
template <int BITS, int ITEM>
struct PlanesAt;

template <int ITEM>
struct PlanesAt<1, ITEM> {
    static __device__ __forceinline__ void put(uint32_t top, int (&P)[1]) {
        uint64_t m0;
        asm volatile("v_add_co_u32 %0, %1, %0, %0" : "+v"(top), "=&s"(m0));
        asm volatile("v_writelane_b32 %0, %1, %c3\n\tv_writelane_b32 %0, %2, %c4" : "+v"(P[0]) : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)), "n"(2 * ITEM), "n"(2 * ITEM + 1));
    }
};
template <int ITEM>
struct PlanesAt<2, ITEM> {
    static __device__ __forceinline__ void put(uint32_t top, int (&P)[2]) {
        uint64_t m0, m1;
        asm volatile("v_add_co_u32 %0, %1, %0, %0\n\tv_add_co_u32 %0, %2, %0, %0" : "+v"(top), "=&s"(m0), "=&s"(m1));
        asm volatile("v_writelane_b32 %0, %2, %c6\n\tv_writelane_b32 %0, %3, %c7\n\tv_writelane_b32 %1, %4, %c6\n\tv_writelane_b32 %1, %5, %c7" : "+v"(P[0]), "+v"(P[1]) : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)), "s"((uint32_t)m1), "s"((uint32_t)(m1 >> 32)), "n"(2 * ITEM), "n"(2 * ITEM + 1));
    }
};
template <int ITEM>
struct PlanesAt<3, ITEM> {
    static __device__ __forceinline__ void put(uint32_t top, int (&P)[3]) {
        uint64_t m0, m1, m2;
        asm volatile("v_add_co_u32 %0, %1, %0, %0\n\tv_add_co_u32 %0, %2, %0, %0\n\tv_add_co_u32 %0, %3, %0, %0" : "+v"(top), "=&s"(m0), "=&s"(m1), "=&s"(m2));
        asm volatile("v_writelane_b32 %0, %3, %c9\n\tv_writelane_b32 %0, %4, %c10\n\tv_writelane_b32 %1, %5, %c9\n\tv_writelane_b32 %1, %6, %c10\n\tv_writelane_b32 %2, %7, %c9\n\tv_writelane_b32 %2, %8, %c10" : "+v"(P[0]), "+v"(P[1]), "+v"(P[2]) : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)), "s"((uint32_t)m1), "s"((uint32_t)(m1 >> 32)), "s"((uint32_t)m2), "s"((uint32_t)(m2 >> 32)), "n"(2 * ITEM), "n"(2 * ITEM + 1));
    }
};
template <int ITEM>
struct PlanesAt<4, ITEM> {
    static __device__ __forceinline__ void put(uint32_t top, int (&P)[4]) {
        uint64_t m0, m1, m2, m3;
        asm volatile("v_add_co_u32 %0, %1, %0, %0\n\tv_add_co_u32 %0, %2, %0, %0\n\tv_add_co_u32 %0, %3, %0, %0\n\tv_add_co_u32 %0, %4, %0, %0" : "+v"(top), "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3));
        asm volatile("v_writelane_b32 %0, %4, %c12\n\tv_writelane_b32 %0, %5, %c13\n\tv_writelane_b32 %1, %6, %c12\n\tv_writelane_b32 %1, %7, %c13\n\tv_writelane_b32 %2, %8, %c12\n\tv_writelane_b32 %2, %9, %c13\n\tv_writelane_b32 %3, %10, %c12\n\tv_writelane_b32 %3, %11, %c13" : "+v"(P[0]), "+v"(P[1]), "+v"(P[2]), "+v"(P[3]) : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)), "s"((uint32_t)m1), "s"((uint32_t)(m1 >> 32)), "s"((uint32_t)m2), "s"((uint32_t)(m2 >> 32)), "s"((uint32_t)m3), "s"((uint32_t)(m3 >> 32)), "n"(2 * ITEM), "n"(2 * ITEM + 1));
    }
};
template <int ITEM>
struct PlanesAt<5, ITEM> {
    static __device__ __forceinline__ void put(uint32_t top, int (&P)[5]) {
        uint64_t m0, m1, m2, m3, m4;
        asm volatile("v_add_co_u32 %0, %1, %0, %0\n\tv_add_co_u32 %0, %2, %0, %0\n\tv_add_co_u32 %0, %3, %0, %0\n\tv_add_co_u32 %0, %4, %0, %0\n\tv_add_co_u32 %0, %5, %0, %0" : "+v"(top), "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3), "=&s"(m4));
        asm volatile("v_writelane_b32 %0, %4, %c12\n\tv_writelane_b32 %0, %5, %c13\n\tv_writelane_b32 %1, %6, %c12\n\tv_writelane_b32 %1, %7, %c13\n\tv_writelane_b32 %2, %8, %c12\n\tv_writelane_b32 %2, %9, %c13\n\tv_writelane_b32 %3, %10, %c12\n\tv_writelane_b32 %3, %11, %c13" : "+v"(P[0]), "+v"(P[1]), "+v"(P[2]), "+v"(P[3]) : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)), "s"((uint32_t)m1), "s"((uint32_t)(m1 >> 32)), "s"((uint32_t)m2), "s"((uint32_t)(m2 >> 32)), "s"((uint32_t)m3), "s"((uint32_t)(m3 >> 32)), "n"(2 * ITEM), "n"(2 * ITEM + 1));
        asm volatile("v_writelane_b32 %0, %1, %c3\n\tv_writelane_b32 %0, %2, %c4" : "+v"(P[4]) : "s"((uint32_t)m4), "s"((uint32_t)(m4 >> 32)), "n"(2 * ITEM), "n"(2 * ITEM + 1));
    }
};
template <int ITEM>
struct PlanesAt<6, ITEM> {
    static __device__ __forceinline__ void put(uint32_t top, int (&P)[6]) {
        uint64_t m0, m1, m2, m3, m4, m5;
        asm volatile("v_add_co_u32 %0, %1, %0, %0\n\tv_add_co_u32 %0, %2, %0, %0\n\tv_add_co_u32 %0, %3, %0, %0\n\tv_add_co_u32 %0, %4, %0, %0\n\tv_add_co_u32 %0, %5, %0, %0\n\tv_add_co_u32 %0, %6, %0, %0" : "+v"(top), "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3), "=&s"(m4), "=&s"(m5));
        asm volatile("v_writelane_b32 %0, %4, %c12\n\tv_writelane_b32 %0, %5, %c13\n\tv_writelane_b32 %1, %6, %c12\n\tv_writelane_b32 %1, %7, %c13\n\tv_writelane_b32 %2, %8, %c12\n\tv_writelane_b32 %2, %9, %c13\n\tv_writelane_b32 %3, %10, %c12\n\tv_writelane_b32 %3, %11, %c13" : "+v"(P[0]), "+v"(P[1]), "+v"(P[2]), "+v"(P[3]) : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)), "s"((uint32_t)m1), "s"((uint32_t)(m1 >> 32)), "s"((uint32_t)m2), "s"((uint32_t)(m2 >> 32)), "s"((uint32_t)m3), "s"((uint32_t)(m3 >> 32)), "n"(2 * ITEM), "n"(2 * ITEM + 1));
        asm volatile("v_writelane_b32 %0, %2, %c6\n\tv_writelane_b32 %0, %3, %c7\n\tv_writelane_b32 %1, %4, %c6\n\tv_writelane_b32 %1, %5, %c7" : "+v"(P[4]), "+v"(P[5]) : "s"((uint32_t)m4), "s"((uint32_t)(m4 >> 32)), "s"((uint32_t)m5), "s"((uint32_t)(m5 >> 32)), "n"(2 * ITEM), "n"(2 * ITEM + 1));
    }
};
template <int ITEM>
struct PlanesAt<7, ITEM> {
    static __device__ __forceinline__ void put(uint32_t top, int (&P)[7]) {
        uint64_t m0, m1, m2, m3, m4, m5, m6;
        asm volatile("v_add_co_u32 %0, %1, %0, %0\n\tv_add_co_u32 %0, %2, %0, %0\n\tv_add_co_u32 %0, %3, %0, %0\n\tv_add_co_u32 %0, %4, %0, %0\n\tv_add_co_u32 %0, %5, %0, %0\n\tv_add_co_u32 %0, %6, %0, %0\n\tv_add_co_u32 %0, %7, %0, %0" : "+v"(top), "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3), "=&s"(m4), "=&s"(m5), "=&s"(m6));
        asm volatile("v_writelane_b32 %0, %4, %c12\n\tv_writelane_b32 %0, %5, %c13\n\tv_writelane_b32 %1, %6, %c12\n\tv_writelane_b32 %1, %7, %c13\n\tv_writelane_b32 %2, %8, %c12\n\tv_writelane_b32 %2, %9, %c13\n\tv_writelane_b32 %3, %10, %c12\n\tv_writelane_b32 %3, %11, %c13" : "+v"(P[0]), "+v"(P[1]), "+v"(P[2]), "+v"(P[3]) : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)), "s"((uint32_t)m1), "s"((uint32_t)(m1 >> 32)), "s"((uint32_t)m2), "s"((uint32_t)(m2 >> 32)), "s"((uint32_t)m3), "s"((uint32_t)(m3 >> 32)), "n"(2 * ITEM), "n"(2 * ITEM + 1));
        asm volatile("v_writelane_b32 %0, %3, %c9\n\tv_writelane_b32 %0, %4, %c10\n\tv_writelane_b32 %1, %5, %c9\n\tv_writelane_b32 %1, %6, %c10\n\tv_writelane_b32 %2, %7, %c9\n\tv_writelane_b32 %2, %8, %c10" : "+v"(P[4]), "+v"(P[5]), "+v"(P[6]) : "s"((uint32_t)m4), "s"((uint32_t)(m4 >> 32)), "s"((uint32_t)m5), "s"((uint32_t)(m5 >> 32)), "s"((uint32_t)m6), "s"((uint32_t)(m6 >> 32)), "n"(2 * ITEM), "n"(2 * ITEM + 1));
    }
};
template <int ITEM>
struct PlanesAt<8, ITEM> {
    static __device__ __forceinline__ void put(uint32_t top, int (&P)[8]) {
        uint64_t m0, m1, m2, m3, m4, m5, m6, m7;
        asm volatile("v_add_co_u32 %0, %1, %0, %0\n\tv_add_co_u32 %0, %2, %0, %0\n\tv_add_co_u32 %0, %3, %0, %0\n\tv_add_co_u32 %0, %4, %0, %0\n\tv_add_co_u32 %0, %5, %0, %0\n\tv_add_co_u32 %0, %6, %0, %0\n\tv_add_co_u32 %0, %7, %0, %0\n\tv_add_co_u32 %0, %8, %0, %0" : "+v"(top), "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3), "=&s"(m4), "=&s"(m5), "=&s"(m6), "=&s"(m7));
        asm volatile("v_writelane_b32 %0, %4, %c12\n\tv_writelane_b32 %0, %5, %c13\n\tv_writelane_b32 %1, %6, %c12\n\tv_writelane_b32 %1, %7, %c13\n\tv_writelane_b32 %2, %8, %c12\n\tv_writelane_b32 %2, %9, %c13\n\tv_writelane_b32 %3, %10, %c12\n\tv_writelane_b32 %3, %11, %c13" : "+v"(P[0]), "+v"(P[1]), "+v"(P[2]), "+v"(P[3]) : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)), "s"((uint32_t)m1), "s"((uint32_t)(m1 >> 32)), "s"((uint32_t)m2), "s"((uint32_t)(m2 >> 32)), "s"((uint32_t)m3), "s"((uint32_t)(m3 >> 32)), "n"(2 * ITEM), "n"(2 * ITEM + 1));
        asm volatile("v_writelane_b32 %0, %4, %c12\n\tv_writelane_b32 %0, %5, %c13\n\tv_writelane_b32 %1, %6, %c12\n\tv_writelane_b32 %1, %7, %c13\n\tv_writelane_b32 %2, %8, %c12\n\tv_writelane_b32 %2, %9, %c13\n\tv_writelane_b32 %3, %10, %c12\n\tv_writelane_b32 %3, %11, %c13" : "+v"(P[4]), "+v"(P[5]), "+v"(P[6]), "+v"(P[7]) : "s"((uint32_t)m4), "s"((uint32_t)(m4 >> 32)), "s"((uint32_t)m5), "s"((uint32_t)(m5 >> 32)), "s"((uint32_t)m6), "s"((uint32_t)(m6 >> 32)), "s"((uint32_t)m7), "s"((uint32_t)(m7 >> 32)), "n"(2 * ITEM), "n"(2 * ITEM + 1));
    }
};

// The same without pooling when C is a multiple of 64: item i is the 64 consecutive floats
// y[64 i ..], i.e. (pixel i / (C/64), channel group i % (C/64)), and its plane words are
// planes[(pixel*BITS + p)*Cw + 2*group + h].  All addressing is wave-uniform (scalar unit) plus
// a per-lane constant, through buffer descriptors; the vector ALU only sees the rule itself.
// FRONT: the real-valued front end (clip, multiply) before the rule; the plain re-encoder skips it.
// CODES / PLANES: which outputs are written (compile-time, so a trip carries no test for them).
// Everything but the rule itself is kept on the scalar unit: item numbers are 32-bit (the host sends
// larger problems to the general kernel), a full trip of U items has no per-item tests, and the
// pixel / channel-group position is divided out once per trip with the host's constants.  Per item
// the vector ALU sees 7 instructions for the rule and 3 per plane.  GATHER: the plane words of a trip
// are collected (PlanesAt) and stored once per plane and trip, for rows of many channels: 8-byte
// stores per item and plane held a stream of 4096-channel rows at 4.1 TB/s where the same kernel
// writing codes reached 5.2.
// POOL: the item's value is the maximum over the 2x2 input pixels of its output pixel (four loads per
// item; the input is addressed through one descriptor with byte offsets below 2^32, which the host
// checks), taken in the order (0,0), (0,1), (1,0), (1,1) with "greater than" as the plain kernel does.
struct PoolArgs {
    FastDiv div_wo, div_howo;       // output pixel -> (image, row, column)
    int Wo, Ho;
    uint32_t pix_bytes, row_bytes, img_bytes, total_bytes;      // of the input: C*4, W*C*4, H*W*C*4, Nb*H*W*C*4
};

template <typename CodeT, int BITS, int U, bool FRONT, bool CODES, bool PLANES, bool GATHER, bool POOL = false>
__global__ __launch_bounds__(256) void requant_flat_kernel(const float *__restrict__ y, int items, int cgroups,
                                                           FastDiv div_groups, float premul, int clip,
                                                           CodeT *__restrict__ codes, uint32_t *__restrict__ planes,
                                                           PoolArgs pg) {
    constexpr int VMAX = (1 << BITS) - 1;
    const int lane = (int)(threadIdx.x & 63);
    const int Cw = 2 * cgroups;
    const int wave0 = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4u + (threadIdx.x >> 6)));
    const int nwaves = (int)gridDim.x * 4;
    const uint32_t plane_bytes = (uint32_t)Cw * 4u;
    const uint32_t pixel_bytes = (uint32_t)BITS * plane_bytes;             // plane words of one pixel
    const int lane_item = lane >> 1, lane_half = lane & 1;               // lane 2u+h: item u of a trip, half h
    const int store_off = ((BITS - 1 - (lane >> 1)) * Cw + (lane & 1)) * 4;   // !GATHER
    const bool stores = lane < 2 * BITS;
    // trips of U items; a wavefront takes every nwaves-th trip
    for (int it0 = wave0 * U; it0 < items; it0 += nwaves * U) {
        const int n = __builtin_amdgcn_readfirstlane(min(items - it0, U));
        int pix, cg;
        fast_divmod((uint32_t)it0, div_groups, pix, cg);
        float v[U];
        if constexpr (!POOL) {
            const __amdgpu_buffer_rsrc_t src = make_rsrc((void *)(y + (int64_t)it0 * 64), (uint32_t)n * 256u);
#pragma unroll
            for (int u = 0; u < U; ++u)         // reads past the descriptor's n*256 bytes return 0
                v[u] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(src, lane * 4, u * 256, 0));
        } else {
            const __amdgpu_buffer_rsrc_t src = make_rsrc((void *)y, pg.total_bytes);
            int img, rem, oh, ow;
            fast_divmod((uint32_t)pix, pg.div_howo, img, rem);
            fast_divmod((uint32_t)rem, pg.div_wo, oh, ow);
            int cgl = cg;
            float w4[U][4];
#pragma unroll
            for (int u = 0; u < U; ++u) {       // (an item past the last one reads zeros or valid memory, and is not used)
                const uint32_t base = (uint32_t)img * pg.img_bytes + (uint32_t)(2 * oh) * pg.row_bytes +
                                      (uint32_t)(2 * ow) * pg.pix_bytes + (uint32_t)cgl * 256u;
                w4[u][0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(src, lane * 4, (int)base, 0));
                w4[u][1] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(src, lane * 4, (int)(base + pg.pix_bytes), 0));
                w4[u][2] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(src, lane * 4, (int)(base + pg.row_bytes), 0));
                w4[u][3] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(src, lane * 4, (int)(base + pg.row_bytes + pg.pix_bytes), 0));
                if (++cgl == cgroups) {
                    cgl = 0;
                    if (++ow == pg.Wo) {
                        ow = 0;
                        if (++oh == pg.Ho) { oh = 0; ++img; }
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float m = w4[u][0];
                if (w4[u][1] > m) m = w4[u][1];
                if (w4[u][2] > m) m = w4[u][2];
                if (w4[u][3] > m) m = w4[u][3];
                v[u] = m;
            }
        }
        // outputs of the trip through descriptors based at its first item
        __amdgpu_buffer_rsrc_t dc, dp;
        if constexpr (CODES) dc = make_rsrc((void *)(codes + (int64_t)it0 * 64), (uint32_t)n * 64u * (uint32_t)sizeof(CodeT));
        int P[BITS];
        int lane_off = 0;                   // bytes from the first item's plane-0 words to this lane's item and half
        uint32_t poff = 0u;                 // !GATHER: bytes from the first item's plane words to the current item's
        int cgi = cg;
        if constexpr (PLANES && !GATHER) dp = make_rsrc((void *)(planes + ((int64_t)pix * BITS) * Cw + 2 * cg), 0xffffffffu);
        if constexpr (PLANES && GATHER) {
            // the trip spans at most U/cgroups + 2 pixels
            dp = make_rsrc((void *)(planes + ((int64_t)pix * BITS) * Cw + 2 * cg), 0xffffffffu);
#pragma unroll
            for (int k = 0; k < BITS; ++k) P[k] = 0;
            // item u of the trip is channel group (cg + u) mod cgroups of pixel pix + (cg + u) / cgroups
            const int t = cg + lane_item;
            const int dpix = (int)fast_div((uint32_t)t, div_groups);
            lane_off = dpix * (int)pixel_bytes + (2 * (t - dpix * cgroups - cg) + lane_half) * 4;
        }
        auto item = [&](auto UC) {
            constexpr int u = decltype(UC)::value;
            float val = v[u];
            if constexpr (FRONT) val = limit_range(val, clip) * premul;
            const uint32_t uidx = round_odd_index<BITS>(val);
            if constexpr (CODES) {
                const int code = 2 * (int)uidx - VMAX;
                if (sizeof(CodeT) == 1) __builtin_amdgcn_raw_buffer_store_b8((char)code, dc, lane, u * 64, 0);
                else __builtin_amdgcn_raw_buffer_store_b16((short)code, dc, lane * 2, u * 128, 0);
            }
            if constexpr (PLANES && GATHER) PlanesAt<BITS, u>::put(uidx << (32 - BITS), P);
            if constexpr (PLANES && !GATHER) {
                // lane 2k+h stores half h of plane BITS-1-k (see emit_planes)
                const int mine = emit_planes<BITS>(uidx << (32 - BITS));
                if (stores) __builtin_amdgcn_raw_buffer_store_b32(mine, dp, store_off, (int)poff, 0);
                poff += 8u;                                              // next channel group: two words on
                if (++cgi == cgroups) {                                  // next pixel
                    cgi = 0;
                    poff += pixel_bytes - 8u * (uint32_t)cgroups;
                }
            }
        };
        if (n == U) {                                                    // a full trip: no test per item
            static_for_items<U>(item);
        } else {                                                         // the short last trip
            static_for_items<U>([&](auto UC) {
                if (decltype(UC)::value < n) item(UC);
            });
        }
        if constexpr (PLANES && GATHER) {
            if (lane_item < n && lane < 2 * U) {
#pragma unroll
                for (int k = 0; k < BITS; ++k)
                    __builtin_amdgcn_raw_buffer_store_b32(P[k], dp, lane_off, (int)((uint32_t)(BITS - 1 - k) * plane_bytes), 0);
            }
        }
    }
}

template <typename CodeT, int BITS>
hipError_t launch_rq(const float *y, int64_t Nb, int64_t H, int64_t W, int64_t out_pixels, int Ho, int Wo, int C, bool pool,
                     float premul, int clip, void *codes, uint32_t *planes, unsigned blocks, hipStream_t s) {
    const int64_t in_bytes = (int64_t)Nb * H * W * C * 4;
    const bool flat_ok = C % 64 == 0 && out_pixels * (C / 64) < ((int64_t)1 << 30);
    if (pool && flat_ok && in_bytes < ((int64_t)1 << 32) && Ho > 0 && Wo > 0) {
        const int items = (int)(out_pixels * (C / 64)), groups = C / 64;
        const FastDiv dg = fast_div_for(groups);
        PoolArgs pg;
        pg.div_wo = fast_div_for(Wo);
        pg.div_howo = fast_div_for(Ho * Wo);
        pg.Wo = Wo; pg.Ho = Ho;
        pg.pix_bytes = (uint32_t)C * 4u;
        pg.row_bytes = (uint32_t)(W * C * 4);
        pg.img_bytes = (uint32_t)(H * W * C * 4);
        pg.total_bytes = (uint32_t)in_bytes;
        const bool front = clip || premul != 1.0f;
        CodeT *cp = (CodeT *)codes;
        // four items (sixteen 256-byte rows) in flight per wavefront
#define QNN_POOL(F, CO, PL) launch_kernel((requant_flat_kernel<CodeT, BITS, 4, F, CO, PL, false, true>), dim3(blocks), dim3(256), 0, \
                                          s, y, items, groups, dg, premul, clip, cp, planes, pg)
        if (front) {
            if (cp && planes) QNN_POOL(true, true, true);
            else if (planes) QNN_POOL(true, false, true);
            else QNN_POOL(true, true, false);
        } else {
            if (cp && planes) QNN_POOL(false, true, true);
            else if (planes) QNN_POOL(false, false, true);
            else QNN_POOL(false, true, false);
        }
#undef QNN_POOL
    } else if (pool)
        launch_kernel((requant_pack_kernel<CodeT, BITS, true, 2>), dim3(blocks), dim3(256), 0, s, y,
                           out_pixels, Ho, Wo, C, premul, clip, (CodeT *)codes, planes);
    else if (flat_ok) {
        const int items = (int)(out_pixels * (C / 64)), groups = C / 64;
        const FastDiv dg = fast_div_for(groups);
        const bool front = clip || premul != 1.0f;
        CodeT *cp = (CodeT *)codes;
        const PoolArgs pg = {};
        // plane words gathered per trip (one store per plane) from 1024 channels on; measured, 4-bit planes
        // out of fp32: 65536 x 4096: 289 -> 251 us, 65536 x 1024: 67 -> 49 us; up to 512 channels the
        // per-item stores are as fast or 3 % faster (the words of a pixel's planes lie close together)
        const bool gather = groups >= 16;
#define QNN_FLAT(F, CO, PL)                                                                                            \
    do {                                                                                                               \
        if (PL && gather)                                                                                              \
            launch_kernel((requant_flat_kernel<CodeT, BITS, 16, F, CO, PL, PL>), dim3(blocks), dim3(256), 0, s, y, items, \
                          groups, dg, premul, clip, cp, planes, pg);                                                   \
        else                                                                                                           \
            launch_kernel((requant_flat_kernel<CodeT, BITS, 16, F, CO, PL, false>), dim3(blocks), dim3(256), 0, s, y,  \
                          items, groups, dg, premul, clip, cp, planes, pg);                                            \
    } while (0)
        if (front) {
            if (cp && planes) QNN_FLAT(true, true, true);
            else if (planes) QNN_FLAT(true, false, true);
            else QNN_FLAT(true, true, false);
        } else {
            if (cp && planes) QNN_FLAT(false, true, true);
            else if (planes) QNN_FLAT(false, false, true);
            else QNN_FLAT(false, true, false);
        }
#undef QNN_FLAT
    }
    else
        launch_kernel((requant_pack_kernel<CodeT, BITS, false, 8>), dim3(blocks), dim3(256), 0, s, y,
                           out_pixels, Ho, Wo, C, premul, clip, (CodeT *)codes, planes);
    return launch_status();
}

// ---------------------------------------------------------------------------------------
// 2x2 max-pool of codes that are already stored as bit planes.  The stored index
// u = (code + 2^bits - 1)/2 is monotone in the code, so the maximum code is the maximum u, and
// the maximum of bit-sliced numbers is a bitwise comparator run from the high plane down: one
// thread handles 32 channels of one output pixel.
// ---------------------------------------------------------------------------------------

// Keeps a value opaque to the optimiser.  The comparator below is a chain of three-input
// boolean steps; folded across steps into v_bitop3_b32 truth tables by this compiler version
// it gave wrong results for three planes and more, step by step it is correct.
__device__ __forceinline__ uint32_t opaque(uint32_t x) {
    asm volatile("" : "+v"(x));
    return x;
}

template <int BITS>
__device__ __forceinline__ void planes_max(uint32_t (&a)[BITS], const uint32_t (&b)[BITS]) {
    uint32_t gt = 0u, lt = 0u;                       // channels where a > b / a < b is already decided
#pragma unroll
    for (int p = BITS - 1; p >= 0; --p) {
        const uint32_t undecided = opaque(~(gt | lt) & (a[p] ^ b[p]));
        gt = opaque(gt | (undecided & a[p]));
        lt = opaque(lt | (undecided & b[p]));
    }
#pragma unroll
    for (int p = 0; p < BITS; ++p) a[p] = opaque((a[p] & ~lt) | (b[p] & lt));
}

template <int BITS>
__global__ __launch_bounds__(256) void pool_planes_kernel(const uint32_t *__restrict__ in, int64_t items, int Ho,
                                                          int Wo, int Cw, uint32_t *__restrict__ out) {
    for (int64_t it = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; it < items;
         it += (int64_t)gridDim.x * blockDim.x) {
        const int64_t opix = it / Cw;
        const int j = (int)(it - opix * Cw);
        const int64_t n = opix / ((int64_t)Ho * Wo);
        const int64_t rem = opix - n * (int64_t)Ho * Wo;
        const int oh = (int)(rem / Wo), ow = (int)(rem - (int64_t)oh * Wo);
        const int64_t p00 = (n * 2 * Ho + 2 * oh) * (2 * (int64_t)Wo) + 2 * ow;       // top-left input pixel
        const int64_t src[4] = {p00, p00 + 1, p00 + 2 * (int64_t)Wo, p00 + 2 * (int64_t)Wo + 1};
        uint32_t m[BITS], v[BITS];
#pragma unroll
        for (int p = 0; p < BITS; ++p) m[p] = in[(src[0] * BITS + p) * Cw + j];
#pragma unroll
        for (int k = 1; k < 4; ++k) {
#pragma unroll
            for (int p = 0; p < BITS; ++p) v[p] = in[(src[k] * BITS + p) * Cw + j];
            planes_max<BITS>(m, v);
        }
#pragma unroll
        for (int p = 0; p < BITS; ++p) out[(opix * BITS + p) * Cw + j] = m[p];
    }
}

template <int BITS>
hipError_t launch_pool_planes_t(const uint32_t *in, int64_t items, int Ho, int Wo, int Cw, uint32_t *out,
                                hipStream_t s) {
    const int64_t want = (items + 255) / 256;
    const int64_t cap = (int64_t)device_simd_count() * 8;
    launch_kernel((pool_planes_kernel<BITS>), dim3((unsigned)(want < cap ? want : cap)), dim3(256), 0, s, in,
                       items, Ho, Wo, Cw, out);
    return launch_status();
}

}  // namespace

hipError_t launch_requant(const float *y, int64_t Nb, int64_t H, int64_t W, int64_t C, bool pool, int bits,
                          float premul, int clip, void *codes, uint32_t *planes, hipStream_t s) {
    const int Ho = (int)(pool ? H / 2 : H), Wo = (int)(pool ? W / 2 : W);
    const int64_t out_pixels = Nb * Ho * (int64_t)Wo;
    const int64_t items = out_pixels * ((C + 63) / 64);
    if (items == 0) return hipSuccess;
    // about 8 wavefronts per SIMD, each looping over its share of the items
    const int64_t want = (items + 3) / 4;
    const int64_t cap = (int64_t)device_simd_count() * 2;
    const unsigned blocks = (unsigned)(want < cap ? want : cap);
#define QNN_RQ(B, T) case B: return launch_rq<T, B>(y, Nb, H, W, out_pixels, Ho, Wo, (int)C, pool, premul, clip, codes, planes, blocks, s)
    switch (bits) {
        QNN_RQ(1, int8_t); QNN_RQ(2, int8_t); QNN_RQ(3, int8_t); QNN_RQ(4, int8_t);
        QNN_RQ(5, int8_t); QNN_RQ(6, int8_t); QNN_RQ(7, int8_t); QNN_RQ(8, int16_t);
    }
#undef QNN_RQ
    return hipErrorInvalidValue;
}

hipError_t launch_pool_planes(const uint32_t *planes, int64_t Nb, int64_t Ho, int64_t Wo, int64_t Cw, int bits,
                              uint32_t *out, hipStream_t s) {
    const int64_t items = Nb * Ho * Wo * Cw;
    if (items == 0) return hipSuccess;
    switch (bits) {
        case 1: return launch_pool_planes_t<1>(planes, items, (int)Ho, (int)Wo, (int)Cw, out, s);
        case 2: return launch_pool_planes_t<2>(planes, items, (int)Ho, (int)Wo, (int)Cw, out, s);
        case 3: return launch_pool_planes_t<3>(planes, items, (int)Ho, (int)Wo, (int)Cw, out, s);
        case 4: return launch_pool_planes_t<4>(planes, items, (int)Ho, (int)Wo, (int)Cw, out, s);
        case 5: return launch_pool_planes_t<5>(planes, items, (int)Ho, (int)Wo, (int)Cw, out, s);
        case 6: return launch_pool_planes_t<6>(planes, items, (int)Ho, (int)Wo, (int)Cw, out, s);
        case 7: return launch_pool_planes_t<7>(planes, items, (int)Ho, (int)Wo, (int)Cw, out, s);
        case 8: return launch_pool_planes_t<8>(planes, items, (int)Ho, (int)Wo, (int)Cw, out, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace qnn
