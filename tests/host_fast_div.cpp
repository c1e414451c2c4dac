// Host test of the division constants the kernels use on the scalar unit (FastDiv in
// qnn_internal.h): n / d from one 32x32 -> high word multiply and a shift must equal the true
// quotient for every n < 2^31.  Compiled and run by tests/test_host_logic.py.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include "qnn_internal.h"

static uint32_t quotient(uint32_t n, const qnn::FastDiv &f) {      // what fast_div() computes on the GPU
    const uint32_t q = (uint32_t)(((uint64_t)n * f.m) >> 32) >> f.sh;
    return f.m != 0u ? q : n;
}

int main() {
    unsigned long long bad = 0, checked = 0;
    const uint32_t ds[] = {1, 2, 3, 5, 7, 9, 14, 27, 56, 64, 100, 224, 255, 256, 257, 1000, 3136, 65535, 65536, 65537,
                           1000003, 1u << 30, (1u << 30) + 1, 0x7ffffffeu, 0x7fffffffu};
    for (uint32_t d : ds) {
        const qnn::FastDiv f = qnn::fast_div_for(d);
        for (uint64_t n = 0; n < (1ull << 31); n += (n < 100000 ? 1 : 1 + rand() % 9973)) {
            ++checked;
            if (quotient((uint32_t)n, f) != (uint32_t)n / d) ++bad;
        }
        for (uint64_t k = 1; k * d < (1ull << 31); k += (k < 1000 ? 1 : rand() % 100000 + 1)) {   // around multiples of d
            const uint32_t n = (uint32_t)(k * d);
            checked += 2;
            if (quotient(n, f) != n / d || quotient(n - 1, f) != (n - 1) / d) ++bad;
        }
        if (quotient(0x7fffffffu, f) != 0x7fffffffu / d) ++bad;
    }
    for (int t = 0; t < 2000000; ++t) {
        uint32_t d = (uint32_t)(rand() % 0x7fffffff) + 1;
        if (t & 1) d = d % 5000 + 1;
        const qnn::FastDiv f = qnn::fast_div_for(d);
        const uint32_t n = (((uint32_t)rand() << 1) ^ (uint32_t)rand()) & 0x7fffffffu;
        ++checked;
        if (quotient(n, f) != n / d) ++bad;
    }
    printf("checked %llu bad %llu\n", checked, bad);
    return bad != 0;
}
