// Encode + pack kernel (paper Eq. (7); the bit-wise storage of the encoded matrices, Sec. 5.4).
//
// A code v = sum_m 2^(m-1) c_m with c_m = +-1 has c_m = +1 exactly where binary digit m-1 of
// u = (v + 2^bits - 1) / 2 is set, so plane p of the output is digit p of u, i.e. digit p+1
// of t = v + 2^bits - 1 (which fits the code's own byte / halfword: 0 <= t <= 2^(bits+1) - 2).
//
// One thread produces the `bits` words of one (row, 32-element group).  On the fast path it
// reads its 32 codes as 16-byte vectors and works on four (int8) or two (int16) codes per
// 32-bit register: a carry-free per-field add of 2^bits - 1, then per plane one shift+mask
// that leaves one bit per field and two shift-ors that gather the fields' bits.  HBM-bound:
// 1 (or 2) bytes in and bits/8 bytes out per code.
#include "qnn_internal.h"

namespace qnn {
namespace {

// per-byte add without carries between bytes: fields of x plus the constant c in every byte
__device__ __forceinline__ uint32_t add_bytes(uint32_t x, uint32_t c) {
    return ((x & 0x7f7f7f7fu) + (c & 0x7f7f7f7fu)) ^ ((x ^ c) & 0x80808080u);
}
__device__ __forceinline__ uint32_t add_halves(uint32_t x, uint32_t c) {
    return ((x & 0x7fff7fffu) + (c & 0x7fff7fffu)) ^ ((x ^ c) & 0x80008000u);
}
// bits 0, 8, 16, 24 of t -> bits 0..3
__device__ __forceinline__ uint32_t gather4(uint32_t t) {
    t |= t >> 7;
    t |= t >> 14;
    return t & 0xfu;
}
// bits 0, 16 of t -> bits 0..1
__device__ __forceinline__ uint32_t gather2(uint32_t t) { return (t | (t >> 15)) & 0x3u; }

// Validity of the four byte codes in x: odd and |v| <= vmax.  Returns the number of bad ones.
__device__ __forceinline__ int count_bad(int v, int vmax) {
    return (((v & 1) == 0) || v < -vmax || v > vmax) ? 1 : 0;
}

template <typename CodeT, int BITS, bool VALIDATE>
__global__ __launch_bounds__(256) void pack_kernel(const CodeT *__restrict__ codes, int64_t rows,
                                                   int K, int Kw, uint32_t *__restrict__ planes,
                                                   int32_t *__restrict__ bad_count) {
    constexpr int VMAX = (1 << BITS) - 1;
    const int64_t total = rows * (int64_t)Kw;
    int bad = 0;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (int64_t)gridDim.x * blockDim.x) {
        int64_t row;
        int wi;
        if (Kw == 2) { row = idx >> 1; wi = (int)(idx & 1); }         // common small cases without a divide
        else if (Kw == 1) { row = idx; wi = 0; }
        else { row = idx / Kw; wi = (int)(idx - row * Kw); }
        const int kbeg = wi * 32;
        const int cnt = min(32, K - kbeg);
        const CodeT *src = codes + row * (int64_t)K + kbeg;
        uint32_t word[BITS];
#pragma unroll
        for (int p = 0; p < BITS; ++p) word[p] = 0u;
        const bool fast = (cnt == 32) && ((((uintptr_t)src) & 15u) == 0);
        if (fast) {
            int bad_here = 0;                                          // of this group of 32 alone
            constexpr int NLD = (int)sizeof(CodeT) * 2;                // 16-byte loads per 32 codes
            const uint4 *s4 = reinterpret_cast<const uint4 *>(src);
#pragma unroll
            for (int l = 0; l < NLD; ++l) {
                const uint4 q = s4[l];
                const uint32_t lanes[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    uint32_t x = lanes[d];
                    if (sizeof(CodeT) == 1) {
                        if (VALIDATE) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) bad_here += count_bad((int)(int8_t)(x >> (8 * e)), VMAX);
                        }
                        const uint32_t t = add_bytes(x, 0x01010101u * (uint32_t)VMAX);
#pragma unroll
                        for (int p = 0; p < BITS; ++p)
                            word[p] |= gather4((t >> (p + 1)) & 0x01010101u) << (l * 16 + d * 4);
                    } else {
                        if (VALIDATE) {
#pragma unroll
                            for (int e = 0; e < 2; ++e) bad_here += count_bad((int)(int16_t)(x >> (16 * e)), VMAX);
                        }
                        const uint32_t t = add_halves(x, 0x00010001u * (uint32_t)VMAX);
#pragma unroll
                        for (int p = 0; p < BITS; ++p)
                            word[p] |= gather2((t >> (p + 1)) & 0x00010001u) << (l * 8 + d * 2);
                    }
                }
            }
            if (VALIDATE && bad_here) {
                // a bad entry packs as the lowest code: redo this group element by element
                bad += bad_here;
#pragma unroll
                for (int p = 0; p < BITS; ++p) word[p] = 0u;
                for (int k = 0; k < 32; ++k) {
                    const int v = (int)src[k];
                    if (count_bad(v, VMAX)) continue;
                    const int u = (v + VMAX) >> 1;
#pragma unroll
                    for (int p = 0; p < BITS; ++p) word[p] |= (uint32_t)((u >> p) & 1) << k;
                }
            }
        } else {
            for (int k = 0; k < cnt; ++k) {
                const int v = (int)src[k];
                if (VALIDATE && count_bad(v, VMAX)) { ++bad; continue; }
                const int u = (v + VMAX) >> 1;
#pragma unroll
                for (int p = 0; p < BITS; ++p) word[p] |= (uint32_t)((u >> p) & 1) << k;
            }
        }
        uint32_t *dst = planes + (row * BITS) * (int64_t)Kw + wi;
#pragma unroll
        for (int p = 0; p < BITS; ++p) dst[(int64_t)p * Kw] = word[p];
    }
    if (VALIDATE) {
        // wavefront sum, one atomic per wavefront that saw something
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) bad += __shfl_down(bad, off, 64);
        if ((threadIdx.x & 63) == 0 && bad != 0) atomicAdd(bad_count, bad);
    }
}

template <typename CodeT, int BITS>
hipError_t launch_bits(const void *codes, int64_t rows, int K, int Kw, uint32_t *planes,
                       int32_t *bad_count, bool validate, unsigned blocks, hipStream_t s) {
    if (validate)
        launch_kernel((pack_kernel<CodeT, BITS, true>), dim3(blocks), dim3(256), 0, s,
                           (const CodeT *)codes, rows, K, Kw, planes, bad_count);
    else
        launch_kernel((pack_kernel<CodeT, BITS, false>), dim3(blocks), dim3(256), 0, s,
                           (const CodeT *)codes, rows, K, Kw, planes, bad_count);
    return launch_status();
}

template <typename CodeT>
hipError_t launch_type(const void *codes, int64_t rows, int K, int Kw, int bits, uint32_t *planes,
                       int32_t *bad_count, bool validate, unsigned blocks, hipStream_t s) {
    switch (bits) {
        case 1: return launch_bits<CodeT, 1>(codes, rows, K, Kw, planes, bad_count, validate, blocks, s);
        case 2: return launch_bits<CodeT, 2>(codes, rows, K, Kw, planes, bad_count, validate, blocks, s);
        case 3: return launch_bits<CodeT, 3>(codes, rows, K, Kw, planes, bad_count, validate, blocks, s);
        case 4: return launch_bits<CodeT, 4>(codes, rows, K, Kw, planes, bad_count, validate, blocks, s);
        case 5: return launch_bits<CodeT, 5>(codes, rows, K, Kw, planes, bad_count, validate, blocks, s);
        case 6: return launch_bits<CodeT, 6>(codes, rows, K, Kw, planes, bad_count, validate, blocks, s);
        case 7: return launch_bits<CodeT, 7>(codes, rows, K, Kw, planes, bad_count, validate, blocks, s);
        case 8: return launch_bits<CodeT, 8>(codes, rows, K, Kw, planes, bad_count, validate, blocks, s);
    }
    return hipErrorInvalidValue;
}

// Packed im2col rows for convolutions with few input channels (C <= 32, window of at most 256
// bits): from per-pixel planes [pix_in][AB] (one word per plane) to [pix_out][AB+1][KWP], where
// bit t*C + c of plane p is the plane bit of tap t = (kh, kw), channel c, zero if the tap lies
// outside the image, and "plane" AB is the mask of the bits whose tap lies inside.
// One thread = one (output pixel, plane).
__global__ __launch_bounds__(256) void window_pack_kernel(const uint32_t *__restrict__ planes, int64_t items,
                                                          ConvGeom q, int H, int W, int C, int AB, int KWP,
                                                          uint32_t *__restrict__ out) {
    const uint32_t cmask = (C >= 32) ? 0xffffffffu : ((1u << C) - 1u);
    for (int64_t it = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; it < items;
         it += (int64_t)gridDim.x * blockDim.x) {
        const int64_t opix = it / (AB + 1);
        const int p = (int)(it - opix * (AB + 1));
        const int ow = (int)(opix % q.Wo);
        const int oh = (int)((opix / q.Wo) % q.Ho);
        const int64_t img = opix / ((int64_t)q.Wo * q.Ho);
        // The bit position t*C grows with the tap number, so the row is built as a stream: a 64-bit
        // window collects taps and its low word is written out whenever it is complete.
        uint32_t *dst = out + it * KWP;
        uint64_t win = 0;                                // bits [32*wcur, 32*wcur + 64) of the row
        int wcur = 0, t = 0;
        for (int kh = 0; kh < q.KH; ++kh) {
            const int ih = oh * q.sh - q.ph + kh * q.dh;
            const bool row_ok = (unsigned)ih < (unsigned)H;
            for (int kw = 0; kw < q.KW; ++kw, ++t) {
                const int iw = ow * q.sw - q.pw + kw * q.dw;
                const int bit = t * C - 32 * wcur;       // < 32 on entry: completed words were flushed
                if (row_ok && (unsigned)iw < (unsigned)W) {
                    const int64_t ipix = (img * H + ih) * W + iw;
                    const uint32_t x = (p < AB) ? (planes[ipix * AB + p] & cmask) : cmask;
                    win |= (uint64_t)x << bit;
                }
                if (bit + C >= 32) {                     // the low word is complete
                    dst[wcur++] = (uint32_t)win;
                    win >>= 32;
                }
            }
        }
        for (; wcur < KWP; ++wcur) {                     // the partly filled word, then padding words
            dst[wcur] = (uint32_t)win;
            win >>= 32;
        }
    }
}

// The same rows from a ROW-DENSE input: planes [Nb*H][AB][Rw], Rw = ceil(W*C/32), bit w*C + c of
// a row's plane word stream = channel c of pixel w (qnn_encode_pack of the codes viewed as
// [Nb*H][W*C]).  With dilation 1 along w the taps kw = 0..KW-1 of a kernel row are KW*C
// consecutive bits of that stream, so a kernel row costs two loads and a funnel shift per 32 bits
// instead of a load per tap: 14 loads instead of 49 for a 7x7 window of 3 channels.
__global__ __launch_bounds__(256) void window_pack_dense_kernel(const uint32_t *__restrict__ planes, int64_t items,
                                                                ConvGeom q, int H, int W, int C, int AB, int KWP,
                                                                uint32_t *__restrict__ out) {
    const int Rw = (W * C + 31) >> 5;
    const int per = (q.dw == 1) ? max(1, 32 / C) : 1;            // taps fetched together (<= 32 bits)
    for (int64_t it = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; it < items;
         it += (int64_t)gridDim.x * blockDim.x) {
        const int64_t opix = it / (AB + 1);
        const int p = (int)(it - opix * (AB + 1));
        const int ow = (int)(opix % q.Wo);
        const int oh = (int)((opix / q.Wo) % q.Ho);
        const int64_t img = opix / ((int64_t)q.Wo * q.Ho);
        uint32_t *dst = out + it * KWP;
        uint64_t win = 0;                                // bits [32*wcur, 32*wcur + 64) of the row
        int wcur = 0, t = 0;
        for (int kh = 0; kh < q.KH; ++kh) {
            const int ih = oh * q.sh - q.ph + kh * q.dh;
            const bool row_ok = (unsigned)ih < (unsigned)H;
            const uint32_t *row = planes + ((img * H + (row_ok ? ih : 0)) * AB + (p < AB ? p : 0)) * Rw;
            for (int kw0 = 0; kw0 < q.KW; kw0 += per) {
                const int ntap = min(per, q.KW - kw0);
                // taps kw0 .. kw0+ntap-1 read pixels iw0, iw0+1, ... (dilation 1 when ntap > 1);
                // those inside the image are the taps [lo, hi) of the group
                const int iw0 = ow * q.sw - q.pw + kw0 * q.dw;
                const int lo = row_ok ? min(ntap, max(0, -iw0)) : ntap;
                const int hi = row_ok ? max(lo, min(ntap, W - iw0)) : ntap;
                uint32_t x = 0u;
                if (hi > lo) {
                    const int nbits = (hi - lo) * C;                      // 1..32
                    const uint32_t m = (nbits >= 32) ? 0xffffffffu : ((1u << nbits) - 1u);
                    if (p < AB) {
                        const int pos = (iw0 + lo) * C, wi = pos >> 5, sh = pos & 31;
                        uint32_t v = row[wi] >> sh;
                        if (sh != 0 && sh + nbits > 32) v |= row[wi + 1] << (32 - sh);   // wi + 1 < Rw: the bits exist
                        x = (v & m) << (lo * C);
                    } else {
                        x = m << (lo * C);
                    }
                }
                const int nb = ntap * C;                                  // bits this group adds to the window
                const int bit = t * C - 32 * wcur;                        // < 32 on entry: completed words were flushed
                win |= (uint64_t)x << bit;
                if (bit + nb >= 32) {                                     // the low word is complete (nb <= 32: one at most)
                    dst[wcur++] = (uint32_t)win;
                    win >>= 32;
                }
                t += ntap;
            }
        }
        for (; wcur < KWP; ++wcur) {                     // the partly filled word, then padding words
            dst[wcur] = (uint32_t)win;
            win >>= 32;
        }
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
    if (code_bytes == 1)
        return launch_type<int8_t>(codes, rows, (int)K, Kw, bits, planes, bad_count, validate, blocks, s);
    return launch_type<int16_t>(codes, rows, (int)K, Kw, bits, planes, bad_count, validate, blocks, s);
}

hipError_t launch_window_pack(const uint32_t *planes, int64_t out_pixels, const ConvGeom &q, int H, int W, int C,
                              int ab, int kwp, bool dense_rows, uint32_t *out, hipStream_t s) {
    const int64_t items = out_pixels * (ab + 1);
    if (items == 0) return hipSuccess;
    const int64_t want = (items + 255) / 256;
    const unsigned blocks = (unsigned)(want < (int64_t)1 << 20 ? want : (int64_t)1 << 20);
    if (dense_rows)
        launch_kernel(window_pack_dense_kernel, dim3(blocks), dim3(256), 0, s, planes, items, q, H, W, C, ab, kwp, out);
    else
        launch_kernel(window_pack_kernel, dim3(blocks), dim3(256), 0, s, planes, items, q, H, W, C, ab, kwp, out);
    return launch_status();
}

}  // namespace qnn
