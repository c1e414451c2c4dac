// Device-side helpers shared by the branch kernels (qnn_branch.hip, qnn_conv_small.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include "qnn_internal.h"

namespace qnn {
namespace {

// Scalar (wave-uniform) read-only view of global memory: loads through this pointer type
// with a uniform index are selected as s_load_dword*.
typedef const uint32_t __attribute__((address_space(4))) *uniform_words;

__device__ __forceinline__ uniform_words as_uniform(const uint32_t *p) {
    return (uniform_words)(uint64_t)p;
}

// part += popcount(x): v_bcnt_u32_b32 with its add operand.  Written as asm so that the
// accumulate chain is not re-associated into separate popcounts and three-input adds;
// volatile so that it keeps its place between the scalar-load requests and waits below.
__device__ __forceinline__ void popc_acc(int &part, uint32_t x) {
    asm volatile("v_bcnt_u32_b32 %0, %1, %0" : "+v"(part) : "v"(x));
}

// part = popcount(x): first contribution to an accumulator (saves zeroing it).
__device__ __forceinline__ void popc_set(int &part, uint32_t x) {
    asm volatile("v_bcnt_u32_b32 %0, %1, 0" : "=v"(part) : "v"(x));
}

// A wave-uniform flag test that stays on the scalar unit.  The word is pinned to an SGPR at the
// point of use (an empty asm the optimiser cannot look through), so the comparison is neither
// hoisted out of the loop nor kept as a lane mask across basic blocks -- testing such a mask again
// costs two VECTOR instructions (a select and a compare) every time.
__device__ __forceinline__ bool sflag(uint32_t word_in, uint32_t mask) {
    uint32_t word = (uint32_t)__builtin_amdgcn_readfirstlane((int)word_in);   // no code if it is in an SGPR already
    asm volatile("" : "+s"(word));
    return (word & mask) != 0u;
}
// The other half of the same trick: a flag word built from comparisons is pinned right where it is
// built, so that later tests see an opaque integer and not the comparisons behind it.
__device__ __forceinline__ uint32_t spin(uint32_t word_in) {
    uint32_t word = (uint32_t)__builtin_amdgcn_readfirstlane((int)word_in);
    asm volatile("" : "+s"(word));
    return word;
}

// n / f.d and n % f.d for a wave-uniform n < 2^31 (see FastDiv): scalar-unit instructions only.
__device__ __forceinline__ uint32_t fast_div(uint32_t n, const FastDiv &f) {
    const uint32_t q = __umulhi(n, f.m) >> f.sh;
    return f.m != 0u ? q : n;
}
__device__ __forceinline__ void fast_divmod(uint32_t n, const FastDiv &f, int &quot, int &rem) {
    const uint32_t q = fast_div(n, f);
    quot = (int)q;
    rem = (int)(n - q * f.d);
}

// N consecutive words at a per-lane address (4-byte aligned only): 16- and 8-byte vector loads
// where N allows.  A lane's weight words are contiguous in memory while different lanes are a
// whole filter apart, so every load instruction touches 64 cache lines whatever its width:
// wide loads cut the number of such instructions (and of tag look-ups) fourfold.
template <int N>
__device__ __forceinline__ void load_run(const uint32_t *__restrict__ p, uint32_t *out) {
    typedef uint32_t w4 __attribute__((ext_vector_type(4), aligned(4)));
    typedef uint32_t w2 __attribute__((ext_vector_type(2), aligned(4)));
    constexpr int N4 = N / 4 * 4;
#pragma unroll
    for (int k = 0; k < N4; k += 4) {
        const w4 v = *reinterpret_cast<const w4 *>(p + k);
        out[k] = v.x; out[k + 1] = v.y; out[k + 2] = v.z; out[k + 3] = v.w;
    }
    if constexpr (N - N4 >= 2) {
        const w2 v = *reinterpret_cast<const w2 *>(p + N4);
        out[N4] = v.x; out[N4 + 1] = v.y;
    }
    if constexpr ((N - N4) & 1) out[N - 1] = p[N - 1];
}

// Re-encoding of a real value on the odd code grid of 2^bits states (Table 2 gives the four
// intervals for 2 bits, with their closures): a = |y|; c = min(2*floor(a/2) + 1, vmax);
// code = (y > 0) ? +c : -c, so zero goes to -1 and NaN to -vmax.  The stored index is
// u = (code + vmax) / 2, whose binary digits are the plane bits.  With H = 2^(bits-1) and
// f = min(floor(a/2), H-1):  c = 2f+1,  u = H + f for y > 0 and u = H-1-f = f xor (H-1)
// otherwise, i.e. u = f xor (y > 0 ? H : H-1).  All steps are exact in binary32 (halving,
// floor; larger magnitudes clamp; a NaN fails the comparison and clamps too).

// ---------------------------------------------------------------------------------------
// Output addressing: buffer descriptors (base in SGPRs, wave-uniform byte offset in an SGPR,
// the lane's column offset in a VGPR).  A descriptor covers the rows of one wavefront.
// ---------------------------------------------------------------------------------------
struct OutView {
    __amdgpu_buffer_rsrc_t d0;   // int32 result if requested, else the fp32 result; also holds partial sums
    __amdgpu_buffer_rsrc_t d1;   // the fp32 result when both outputs are requested
    uint32_t flags;              // bit 0: int32 result requested, bit 1: fp32 result requested
    uint32_t row_bytes;          // N * 4
    int col_bytes;               // lane's column * 4.  Lanes past N compute column N-1 again (same
                                 // weights, same scale) and store the identical value to it, so
                                 // the epilogue needs no lane mask
    float sc;
};

// The same plus the re-encoded result as bit planes of the next layer (Alg. 1 forward: the scaled
// output is encoded again).  Row r of the product becomes out_bits * Nw words, Nw = ceil(N/32);
// a wavefront owns columns 64*ct .. 64*ct+63, i.e. words 2*ct and 2*ct+1 of every plane.
struct OutViewEmit : OutView {
    __amdgpu_buffer_rsrc_t dp;   // plane words of the wavefront's rows
    uint32_t prow_bytes;         // out_bits * Nw * 4
    int bits;                    // out_bits
    int shift;                   // 32 - out_bits: the index is handled at the top of a register
    // per-lane constants; a lane whose column does not exist (it repeats column N-1) has all
    // three zero, which makes its index zero = all plane bits zero
    float fmax;                  // H - 1/2: floor(min(|y|/2, fmax)) is the clamped magnitude index
    uint32_t sel_pos, sel_neg;   // H and H - 1, shifted to the top
    int word_off;                // byte offset inside a row of the word this lane stores (lane 2k+h:
                                 // half h of plane out_bits-1-k), or -1 if the lane stores nothing
};

// Partial sums of one wavefront kept in LDS (rows x 64 lanes of int32, the lane's own column):
// used where the four wavefronts of a block each form a part of the same outputs and one pass
// over LDS combines them.  `slab` already points at the lane's slot of row 0.
struct OutViewSlab {
    int *slab;
    bool with_const;             // this wavefront's first part carries the product's constant term
};
template <class OV> struct is_slab { static constexpr bool value = false; };
template <> struct is_slab<OutViewSlab> { static constexpr bool value = true; };
template <class OV>
__device__ __forceinline__ bool adds_const(const OV &v) {
    if constexpr (is_slab<OV>::value) return v.with_const;
    else return true;
}
// what earlier chunk passes of this wavefront left for a row (multi-pass products)
template <class OV>
__device__ __forceinline__ int partial_load(const OV &v, int rel_row) {
    if constexpr (is_slab<OV>::value) return v.slab[rel_row * 64];
    else return __builtin_amdgcn_raw_buffer_load_b32(v.d0, v.col_bytes, (int)((uint32_t)rel_row * v.row_bytes), 0);
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(void *p, uint32_t bytes) {
    // raw dword buffer: stride 0, num_records in bytes, 32-bit data format word for gfx9
    return __builtin_amdgcn_make_buffer_rsrc(p, 0, bytes, 0x00020000);
}

// Plane emission.  The index of every lane sits at the top of `top`; doubling it shifts out one
// plane per step, high plane first, and the carry-out of the 64 lanes IS that plane's two packed
// words (one vector op per plane).  All N doublings are issued first, each carry mask into its own
// SGPR pair, then lanes 2k and 2k+1 of the result receive the low and high word of step k's plane
// (plane out_bits-1-k): the writes no longer wait on the mask just produced, and the register that
// held the indices is dead by then and takes the words itself.
// The same one step at a time, for code that is short of scalar registers (the branch kernels'
// epilogue: holding all masks at once cost them 1 %): step K of the emission, lanes 2K and 2K+1 of
// `mine` receive the two words of plane out_bits-1-K.
template <int K>
__device__ __forceinline__ void emit_step(uint32_t &top, int &mine) {
    uint64_t m;
    asm volatile("v_add_co_u32 %0, %1, %0, %0" : "+v"(top), "=s"(m));
    asm volatile("v_writelane_b32 %0, %1, %2\n\tv_writelane_b32 %0, %3, %4"
                 : "+v"(mine) : "s"((uint32_t)m), "n"(2 * K), "s"((uint32_t)(m >> 32)), "n"(2 * K + 1));
}

template <int N>
__device__ __forceinline__ int emit_planes(uint32_t top);
// One asm statement for the N doublings and one for the 2N lane writes: between separate asm
// statements the compiler pads with a wait state each, which costs the wavefront an issue slot per
// instruction.  (No wait state is required here: the masks are read as data, not as lane selects.)
template <>
__device__ __forceinline__ int emit_planes<1>(uint32_t top) {
    uint64_t m0;
    asm volatile("v_add_co_u32 %0, %1, %0, %0" : "+v"(top), "=&s"(m0));
    int mine = (int)top;
    asm volatile("v_writelane_b32 %0, %1, 0\n\tv_writelane_b32 %0, %2, 1" : "+v"(mine) : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)));
    return mine;
}
template <>
__device__ __forceinline__ int emit_planes<2>(uint32_t top) {
    uint64_t m0, m1;
    asm volatile("v_add_co_u32 %0, %1, %0, %0\n\tv_add_co_u32 %0, %2, %0, %0" : "+v"(top), "=&s"(m0), "=&s"(m1));
    int mine = (int)top;
    asm volatile("v_writelane_b32 %0, %1, 0\n\tv_writelane_b32 %0, %2, 1\n\tv_writelane_b32 %0, %3, 2\n\tv_writelane_b32 %0, %4, 3" : "+v"(mine) : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)), "s"((uint32_t)m1), "s"((uint32_t)(m1 >> 32)));
    return mine;
}
template <>
__device__ __forceinline__ int emit_planes<3>(uint32_t top) {
    uint64_t m0, m1, m2;
    asm volatile("v_add_co_u32 %0, %1, %0, %0\n\tv_add_co_u32 %0, %2, %0, %0\n\tv_add_co_u32 %0, %3, %0, %0" : "+v"(top), "=&s"(m0), "=&s"(m1), "=&s"(m2));
    int mine = (int)top;
    asm volatile("v_writelane_b32 %0, %1, 0\n\tv_writelane_b32 %0, %2, 1\n\tv_writelane_b32 %0, %3, 2\n\tv_writelane_b32 %0, %4, 3\n\tv_writelane_b32 %0, %5, 4\n\tv_writelane_b32 %0, %6, 5" : "+v"(mine) : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)), "s"((uint32_t)m1), "s"((uint32_t)(m1 >> 32)), "s"((uint32_t)m2), "s"((uint32_t)(m2 >> 32)));
    return mine;
}
template <>
__device__ __forceinline__ int emit_planes<4>(uint32_t top) {
    uint64_t m0, m1, m2, m3;
    asm volatile("v_add_co_u32 %0, %1, %0, %0\n\tv_add_co_u32 %0, %2, %0, %0\n\tv_add_co_u32 %0, %3, %0, %0\n\tv_add_co_u32 %0, %4, %0, %0" : "+v"(top), "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3));
    int mine = (int)top;
    asm volatile("v_writelane_b32 %0, %1, 0\n\tv_writelane_b32 %0, %2, 1\n\tv_writelane_b32 %0, %3, 2\n\tv_writelane_b32 %0, %4, 3\n\tv_writelane_b32 %0, %5, 4\n\tv_writelane_b32 %0, %6, 5\n\tv_writelane_b32 %0, %7, 6\n\tv_writelane_b32 %0, %8, 7" : "+v"(mine) : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)), "s"((uint32_t)m1), "s"((uint32_t)(m1 >> 32)), "s"((uint32_t)m2), "s"((uint32_t)(m2 >> 32)), "s"((uint32_t)m3), "s"((uint32_t)(m3 >> 32)));
    return mine;
}
template <>
__device__ __forceinline__ int emit_planes<5>(uint32_t top) {
    uint64_t m0, m1, m2, m3, m4;
    asm volatile("v_add_co_u32 %0, %1, %0, %0\n\tv_add_co_u32 %0, %2, %0, %0\n\tv_add_co_u32 %0, %3, %0, %0\n\tv_add_co_u32 %0, %4, %0, %0\n\tv_add_co_u32 %0, %5, %0, %0" : "+v"(top), "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3), "=&s"(m4));
    int mine = (int)top;
    asm volatile("v_writelane_b32 %0, %1, 0\n\tv_writelane_b32 %0, %2, 1\n\tv_writelane_b32 %0, %3, 2\n\tv_writelane_b32 %0, %4, 3\n\tv_writelane_b32 %0, %5, 4\n\tv_writelane_b32 %0, %6, 5\n\tv_writelane_b32 %0, %7, 6\n\tv_writelane_b32 %0, %8, 7\n\tv_writelane_b32 %0, %9, 8\n\tv_writelane_b32 %0, %10, 9" : "+v"(mine) : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)), "s"((uint32_t)m1), "s"((uint32_t)(m1 >> 32)), "s"((uint32_t)m2), "s"((uint32_t)(m2 >> 32)), "s"((uint32_t)m3), "s"((uint32_t)(m3 >> 32)), "s"((uint32_t)m4), "s"((uint32_t)(m4 >> 32)));
    return mine;
}
template <>
__device__ __forceinline__ int emit_planes<6>(uint32_t top) {
    uint64_t m0, m1, m2, m3, m4, m5;
    asm volatile("v_add_co_u32 %0, %1, %0, %0\n\tv_add_co_u32 %0, %2, %0, %0\n\tv_add_co_u32 %0, %3, %0, %0\n\tv_add_co_u32 %0, %4, %0, %0\n\tv_add_co_u32 %0, %5, %0, %0\n\tv_add_co_u32 %0, %6, %0, %0" : "+v"(top), "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3), "=&s"(m4), "=&s"(m5));
    int mine = (int)top;
    asm volatile("v_writelane_b32 %0, %1, 0\n\tv_writelane_b32 %0, %2, 1\n\tv_writelane_b32 %0, %3, 2\n\tv_writelane_b32 %0, %4, 3\n\tv_writelane_b32 %0, %5, 4\n\tv_writelane_b32 %0, %6, 5\n\tv_writelane_b32 %0, %7, 6\n\tv_writelane_b32 %0, %8, 7\n\tv_writelane_b32 %0, %9, 8\n\tv_writelane_b32 %0, %10, 9\n\tv_writelane_b32 %0, %11, 10\n\tv_writelane_b32 %0, %12, 11" : "+v"(mine) : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)), "s"((uint32_t)m1), "s"((uint32_t)(m1 >> 32)), "s"((uint32_t)m2), "s"((uint32_t)(m2 >> 32)), "s"((uint32_t)m3), "s"((uint32_t)(m3 >> 32)), "s"((uint32_t)m4), "s"((uint32_t)(m4 >> 32)), "s"((uint32_t)m5), "s"((uint32_t)(m5 >> 32)));
    return mine;
}
template <>
__device__ __forceinline__ int emit_planes<7>(uint32_t top) {
    uint64_t m0, m1, m2, m3, m4, m5, m6;
    asm volatile("v_add_co_u32 %0, %1, %0, %0\n\tv_add_co_u32 %0, %2, %0, %0\n\tv_add_co_u32 %0, %3, %0, %0\n\tv_add_co_u32 %0, %4, %0, %0\n\tv_add_co_u32 %0, %5, %0, %0\n\tv_add_co_u32 %0, %6, %0, %0\n\tv_add_co_u32 %0, %7, %0, %0" : "+v"(top), "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3), "=&s"(m4), "=&s"(m5), "=&s"(m6));
    int mine = (int)top;
    asm volatile("v_writelane_b32 %0, %1, 0\n\tv_writelane_b32 %0, %2, 1\n\tv_writelane_b32 %0, %3, 2\n\tv_writelane_b32 %0, %4, 3\n\tv_writelane_b32 %0, %5, 4\n\tv_writelane_b32 %0, %6, 5\n\tv_writelane_b32 %0, %7, 6\n\tv_writelane_b32 %0, %8, 7\n\tv_writelane_b32 %0, %9, 8\n\tv_writelane_b32 %0, %10, 9\n\tv_writelane_b32 %0, %11, 10\n\tv_writelane_b32 %0, %12, 11\n\tv_writelane_b32 %0, %13, 12\n\tv_writelane_b32 %0, %14, 13" : "+v"(mine) : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)), "s"((uint32_t)m1), "s"((uint32_t)(m1 >> 32)), "s"((uint32_t)m2), "s"((uint32_t)(m2 >> 32)), "s"((uint32_t)m3), "s"((uint32_t)(m3 >> 32)), "s"((uint32_t)m4), "s"((uint32_t)(m4 >> 32)), "s"((uint32_t)m5), "s"((uint32_t)(m5 >> 32)), "s"((uint32_t)m6), "s"((uint32_t)(m6 >> 32)));
    return mine;
}
template <>
__device__ __forceinline__ int emit_planes<8>(uint32_t top) {
    uint64_t m0, m1, m2, m3, m4, m5, m6, m7;
    asm volatile("v_add_co_u32 %0, %1, %0, %0\n\tv_add_co_u32 %0, %2, %0, %0\n\tv_add_co_u32 %0, %3, %0, %0\n\tv_add_co_u32 %0, %4, %0, %0\n\tv_add_co_u32 %0, %5, %0, %0\n\tv_add_co_u32 %0, %6, %0, %0\n\tv_add_co_u32 %0, %7, %0, %0\n\tv_add_co_u32 %0, %8, %0, %0" : "+v"(top), "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3), "=&s"(m4), "=&s"(m5), "=&s"(m6), "=&s"(m7));
    int mine = (int)top;
    asm volatile("v_writelane_b32 %0, %1, 0\n\tv_writelane_b32 %0, %2, 1\n\tv_writelane_b32 %0, %3, 2\n\tv_writelane_b32 %0, %4, 3\n\tv_writelane_b32 %0, %5, 4\n\tv_writelane_b32 %0, %6, 5\n\tv_writelane_b32 %0, %7, 6\n\tv_writelane_b32 %0, %8, 7\n\tv_writelane_b32 %0, %9, 8\n\tv_writelane_b32 %0, %10, 9\n\tv_writelane_b32 %0, %11, 10\n\tv_writelane_b32 %0, %12, 11\n\tv_writelane_b32 %0, %13, 12\n\tv_writelane_b32 %0, %14, 13\n\tv_writelane_b32 %0, %15, 14\n\tv_writelane_b32 %0, %16, 15" : "+v"(mine) : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)), "s"((uint32_t)m1), "s"((uint32_t)(m1 >> 32)), "s"((uint32_t)m2), "s"((uint32_t)(m2 >> 32)), "s"((uint32_t)m3), "s"((uint32_t)(m3 >> 32)), "s"((uint32_t)m4), "s"((uint32_t)(m4 >> 32)), "s"((uint32_t)m5), "s"((uint32_t)(m5 >> 32)), "s"((uint32_t)m6), "s"((uint32_t)(m6 >> 32)), "s"((uint32_t)m7), "s"((uint32_t)(m7 >> 32)));
    return mine;
}

// floor of a non-negative binary32 value as an integer, one instruction
__device__ __forceinline__ int floor_to_int(float t) {
    int f;
    asm("v_cvt_flr_i32_f32 %0, %1" : "=v"(f) : "v"(t));
    return f;
}

template <class OV>
__device__ __forceinline__ OV make_out_view(const BranchArgs &g, int r0, int r1, int nload, float sc, int ct) {
    OV v;
    if constexpr (std::is_same<OV, OutViewEmit>::value) {
        const int lane = (int)(threadIdx.x & 63);
        const int Nw = (g.N + 31) >> 5;
        const bool n_ok = ct * 64 + lane < g.N;
        const uint32_t H = 1u << (g.out_bits - 1);
        v.bits = g.out_bits;
        v.shift = 32 - g.out_bits;
        v.fmax = n_ok ? (float)(H - 1u) + 0.5f : 0.0f;
        v.sel_pos = n_ok ? 0x80000000u : 0u;
        v.sel_neg = n_ok ? (H - 1u) << (32 - g.out_bits) : 0u;
        v.prow_bytes = (uint32_t)(g.out_bits * Nw) * 4u;
        v.dp = make_rsrc((void *)(g.planes_out + (int64_t)r0 * g.out_bits * Nw), (uint32_t)(r1 - r0) * v.prow_bytes);
        const int word = 2 * ct + (lane & 1);
        const int step = lane >> 1;                  // see emit_planes: step k carries plane out_bits-1-k
        v.word_off = (step < g.out_bits && word < Nw) ? ((g.out_bits - 1 - step) * Nw + word) * 4 : -1;
    }
    const int64_t first = (int64_t)r0 * g.N;
    const uint32_t bytes = (uint32_t)(r1 - r0) * (uint32_t)g.N * 4u;    // < 2^31, checked on the host
    v.flags = g.out_flags;                                              // set by the host: a plain kernel argument
    v.d0 = make_rsrc((void *)(g.partial + first), bytes);               // partial == acc if present, else out
    v.d1 = make_rsrc((g.out != nullptr) ? (void *)(g.out + first) : (void *)(g.partial + first), bytes);
    v.row_bytes = (uint32_t)g.N * 4u;
    v.col_bytes = nload * 4;
    v.sc = sc;
    return v;
}

// Finish one row of one chunk pass for this lane's column.  rel_row = row - r0.  SINGLE: the
// product has a single chunk pass (first and last are both true at compile time).
template <bool SINGLE>
__device__ __forceinline__ void finish_row(const OutViewSlab &v, int rel_row, int val, bool first, bool) {
    if (!first) val += v.slab[rel_row * 64];
    v.slab[rel_row * 64] = val;
}

// Cache policy of the stores of results (not of partial sums, which the same wavefront reads back):
// device scope (the sc1 bit of the gfx94x/gfx950 buffer stores), i.e. written through the XCD's L2
// as the kernel runs.  With the default policy the results stay dirty in the L2s and are written back
// when the kernel ends, before the next one may start: on the ResNet-18-shaped layer (51 MB of
// results per launch) that write-back was 2.4 us of every 30.9 us launch (28.5 us with sc1; the
// non-temporal bit alone gives 29.2, the workgroup-scope bit nothing).  Only for the branch kernels'
// row stores (256 contiguous bytes per wavefront): on the re-encoder's 8-byte plane pieces the same
// bit costs 10-45 % (the L2 no longer merges them into whole lines), and on the pack and pooling
// kernels' word stores it changed nothing or cost 1 %.
constexpr int kResultStore = 16;
template <bool SINGLE, class OV>
__device__ __forceinline__ void finish_row(const OV &v, int rel_row, int val, bool first, bool last) {
    const int soff = (int)((uint32_t)rel_row * v.row_bytes);
    if constexpr (!SINGLE) {
        if (!first) val += __builtin_amdgcn_raw_buffer_load_b32(v.d0, v.col_bytes, soff, 0);
        if (!last) {
            __builtin_amdgcn_raw_buffer_store_b32(val, v.d0, v.col_bytes, soff, 0);
            return;
        }
    }
    const float y = (float)val * v.sc;
    if (sflag(v.flags, 1u)) {
        __builtin_amdgcn_raw_buffer_store_b32(val, v.d0, v.col_bytes, soff, kResultStore);
        if (sflag(v.flags, 2u)) __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, y), v.d1, v.col_bytes, soff, kResultStore);
    } else if (sflag(v.flags, 2u)) {
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, y), v.d0, v.col_bytes, soff, kResultStore);
    }
    if constexpr (std::is_same<OV, OutViewEmit>::value) {
        // Table 2 rule on y (see the top of this file), index at the top of the register:
        // f = floor(min(|y|/2, H - 1/2)) (the minimum also catches inf and NaN), u = f xor (H or H-1)
        const int f = floor_to_int(__builtin_fminf(__builtin_fabsf(y) * 0.5f, v.fmax));
        uint32_t top = ((uint32_t)f << v.shift) ^ ((y > 0.0f) ? v.sel_pos : v.sel_neg);
        int mine = (int)top;                         // every lane that stores is overwritten below
        int b = v.bits;
        asm volatile("" : "+s"(b));                  // decided here, per call, on the scalar unit
        // steps 0 .. bits-1, rounded up to 1, 2, 4 or 8 of them: a step past the last plane
        // shifts out zeros into lanes that store nothing
        emit_step<0>(top, mine);
        if (b > 1) {
            emit_step<1>(top, mine);
            if (b > 2) {
                emit_step<2>(top, mine);
                emit_step<3>(top, mine);
                if (b > 4) {
                    emit_step<4>(top, mine);
                    emit_step<5>(top, mine);
                    emit_step<6>(top, mine);
                    emit_step<7>(top, mine);
                }
            }
        }
        if (v.word_off >= 0)
            __builtin_amdgcn_raw_buffer_store_b32(mine, v.dp, v.word_off, (int)((uint32_t)rel_row * v.prow_bytes), kResultStore);
    }
}

// ---------------------------------------------------------------------------------------
// Block numbering for the convolution kernels.  The blocks of a launch are handed to the chip's
// eight XCDs in turn (block b runs on XCD b % 8), and every XCD has an L2 of its own.  With the
// plain numbering each XCD works on pixels from all over the batch and its L2 fetches the whole
// set of activation planes; numbered as below, XCD x works on one contiguous part of the blocks,
// i.e. of the pixels, and fetches that part only.  With q = gridDim.x / 8 and r = gridDim.x % 8,
// XCD x receives q + (x < r) blocks, and they are given the numbers x*q + min(x, r) + (b / 8):
// consecutive ranges that tile [0, gridDim.x) exactly.  (1-D grids only.)  The grid size comes in
// with the kernel arguments (nb; the launchers check it against the grid they launch): reading
// gridDim.x costs a vector load and a wait at the start of every wavefront.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t xcd_block(int on, uint32_t nb) {
    const uint32_t b = blockIdx.x;
    if (!on) return b;
    const uint32_t q = nb >> 3, r = nb & 7u, x = b & 7u;
    return x * q + (x < r ? x : r) + (b >> 3);
}

// ---------------------------------------------------------------------------------------
// Scalar loads under manual control.
//
// Scalar loads return out of order, so the only wait a wavefront has is "all of them".  The
// compiler places that wait before the first use of any loaded register and is free to sink
// the loads towards their use, which serialises fetch and compute.  The activation words
// are therefore requested with s_load_dword* written as asm (the compiler does not know the
// destination registers are still in flight) and the wait is written explicitly: arrive()
// is s_waitcnt lgkmcnt(0) with the registers as in/out operands, so every use of the words
// is ordered after it.  Invariant, checked on the generated code: between a request and its
// arrive nothing reads or moves the requested registers.
// ---------------------------------------------------------------------------------------
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
template <int N> struct SVec;
template <> struct SVec<1> { typedef uint32_t type; };
template <> struct SVec<2> { typedef u32x2 type; };
template <> struct SVec<4> { typedef u32x4 type; };
template <> struct SVec<8> { typedef u32x8 type; };
template <> struct SVec<16> { typedef u32x16 type; };

// N consecutive words, fetched as the binary decomposition of N (x16, x8, x4, x2, x1).
template <int N>
struct SRun {
    static constexpr int HEAD = N >= 16 ? 16 : N >= 8 ? 8 : N >= 4 ? 4 : N >= 2 ? 2 : 1;
    typename SVec<HEAD>::type head;
    SRun<N - HEAD> tail;

    // words at byte address base + off + IMM ...
    template <int IMM>
    __device__ __forceinline__ void request(uint64_t base, uint32_t off_in) {
        // wave-uniform by construction; this pins the value to an SGPR (no code if it already is)
        const uint32_t off = (uint32_t)__builtin_amdgcn_readfirstlane((int)off_in);
        if constexpr (HEAD == 16)
            asm volatile("s_load_dwordx16 %0, %1, %2 offset:%3" : "=s"(head) : "s"(base), "s"(off), "n"(IMM));
        else if constexpr (HEAD == 8)
            asm volatile("s_load_dwordx8 %0, %1, %2 offset:%3" : "=s"(head) : "s"(base), "s"(off), "n"(IMM));
        else if constexpr (HEAD == 4)
            asm volatile("s_load_dwordx4 %0, %1, %2 offset:%3" : "=s"(head) : "s"(base), "s"(off), "n"(IMM));
        else if constexpr (HEAD == 2)
            asm volatile("s_load_dwordx2 %0, %1, %2 offset:%3" : "=s"(head) : "s"(base), "s"(off), "n"(IMM));
        else
            asm volatile("s_load_dword %0, %1, %2 offset:%3" : "=s"(head) : "s"(base), "s"(off), "n"(IMM));
        tail.template request<IMM + HEAD * 4>(base, off_in);
    }
    // WAIT: emit the s_waitcnt (first piece of a stage only); later pieces are just ordered
    // after it.
    template <bool WAIT>
    __device__ __forceinline__ void arrive() {
        if constexpr (WAIT) asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(head));
        else asm volatile("" : "+s"(head));
        tail.template arrive<false>();
    }
    __device__ __forceinline__ uint32_t get(int i) const {
        if constexpr (HEAD == 1) return i == 0 ? head : tail.get(i - 1);
        else return i < HEAD ? head[i] : tail.get(i - HEAD);
    }
};
template <>
struct SRun<0> {
    template <int IMM> __device__ __forceinline__ void request(uint64_t, uint32_t) {}
    template <bool WAIT> __device__ __forceinline__ void arrive() {}
    __device__ __forceinline__ uint32_t get(int) const { return 0u; }
};

// NR runs of LEN words each (one pipeline stage).
template <int NR, int LEN>
struct SStage {
    SRun<LEN> run[NR];
    template <bool WAIT>
    __device__ __forceinline__ void arrive() {
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            if (i == 0) run[i].template arrive<WAIT>();
            else run[i].template arrive<false>();
        }
    }
};

}  // namespace
}  // namespace qnn
