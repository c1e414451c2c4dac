// Device-side helpers shared by the branch kernels (qnn_branch.hip, qnn_conv_small.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

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
