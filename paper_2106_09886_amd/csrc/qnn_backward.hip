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
    int lds_vec;             // 16-byte loads are possible in the LDS-staged kernel
    int64_t ldg;
};

// Small outputs with short sums (fewer than 512 tiles of 128 x 128 and sums under 256 terms; the
// others take the two LDS-staged kernels below).
// A block of four wavefronts takes 32*RT rows (RT = 1, 2) x 128 columns of the output; wavefront v
// all rows and the 32 columns of plane word 4*cb + v, so a decoded code feeds RT matrix instructions.
// One iteration takes eight reduction indices: lanes 0..31 hold j0..j0+3, lanes 32..63
// j0+4..j0+7, and the u-th of four matrix instructions pairs j0+u with j0+4+u (any pairing is
// right as long as both operands use it).
//   A operand (32 x 2): lane l supplies row l % 32, reduction index l / 32.
//   B operand (2 x 32): lane l supplies column l % 32, reduction index l / 32.
//   D (32 x 32, 16 registers): register v of lane l is row 8 * (v / 4) + 4 * (l / 32) + v % 4, column l % 32.
// The loads of the next eight indices are issued before the matrix instructions of the current ones
// (two stage buffers, the loop unrolled by two).
// GT: g is indexed [j][r] (gradient of the weights) instead of [r][j].
// VEC (only without GT): J is a multiple of 8, ldg of 4 and g, scale are 16-byte aligned: the four
// values of a lane are one 16-byte load.
// (Left to itself the compiler sizes the kernel for one wavefront per SIMD; two to four resident
// wavefronts are asked for instead.)
template <int CB, int RT, bool GT, bool VEC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(RT == 2 ? (CB >= 7 ? 2 : 3) : (CB >= 7 ? 3 : 4))))
void backward_gemm_kernel(const BackArgs a) {
    constexpr int NT = RT;                               // row tiles per wavefront
    constexpr int CT = 1;                                // plane words (32 columns each) per wavefront
    static_assert(RT == 1 || RT == 2, "larger tiles belong to the LDS-staged kernel");
    const int wave = (int)(threadIdx.x >> 6), lane = (int)(threadIdx.x & 63);
    const int half = lane >> 5, l5 = lane & 31;
    const int rb = (int)(blockIdx.x / (unsigned)a.col_blocks);
    const int cb = (int)(blockIdx.x - (unsigned)rb * (unsigned)a.col_blocks);
    const int r0 = rb * (32 * RT);
    const int cw0 = cb * 4 + wave;
    if (cw0 >= a.Cw || r0 >= a.R) return;                // (no barrier in this kernel)
    const int jbeg = 0, jend = a.J;
    f32x16 acc[NT][CT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int c = 0; c < CT; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][c][v] = 0.0f;
    int rowc[NT];                                        // the lane's A row, clamped for the loads
    float srow[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int row = r0 + t * 32 + l5;
        rowc[t] = row < a.R ? row : a.R - 1;
        srow[t] = (GT && a.scale != nullptr) ? a.scale[rowc[t]] : 1.0f;
    }
    int cwc[CT];                                         // plane words, clamped for the loads
#pragma unroll
    for (int c = 0; c < CT; ++c) cwc[c] = min(cw0 + c, a.Cw - 1);
    constexpr int kOffset = (1 << CB) - 1;
    // A stage holds what was loaded, untouched (any arithmetic on it would wait for the loads at
    // once), and loading is free of branches: indices past the end are clamped to valid addresses
    // and their products masked in compute(), a missing scale reads the gradient's address instead
    // and is replaced by one.  With a branch around the loads the compiler can no longer count how
    // many are in flight and waits for all of them before the matrix instructions.
    struct Stage {
        float gv[NT][4];
        float sv[4];
        uint32_t pw[4][CT][CB];
    };
    const bool has_scale = a.scale != nullptr;
    auto load = [&](int j0, Stage &st) {
        const int jb = j0 + 4 * half;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int jc = min(jb + u, jend - 1);
#pragma unroll
            for (int c = 0; c < CT; ++c)
#pragma unroll
                for (int q = 0; q < CB; ++q) st.pw[u][c][q] = a.planes[((int64_t)jc * CB + q) * a.Cw + cwc[c]];
        }
        if constexpr (VEC) {
            const int jbc = min(jb, jend - 4);           // jb, jend multiples of 4, jend >= 8
            const float *sp = has_scale ? a.scale + jbc : a.g + (int64_t)rowc[0] * a.ldg + jbc;
            const f32x4 sv = *reinterpret_cast<const f32x4 *>(sp);
#pragma unroll
            for (int u = 0; u < 4; ++u) st.sv[u] = sv[u];
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const f32x4 gv = *reinterpret_cast<const f32x4 *>(a.g + (int64_t)rowc[t] * a.ldg + jbc);
#pragma unroll
                for (int u = 0; u < 4; ++u) st.gv[t][u] = gv[u];
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int jc = min(jb + u, jend - 1);
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    st.gv[t][u] = GT ? a.g[(int64_t)jc * a.ldg + rowc[t]] : a.g[(int64_t)rowc[t] * a.ldg + jc];
                if constexpr (!GT) {
                    const float *sp = has_scale ? a.scale + jc : a.g + (int64_t)rowc[0] * a.ldg + jc;
                    st.sv[u] = *sp;
                } else {
                    st.sv[u] = 1.0f;
                }
            }
        }
    };
    auto compute = [&](int j0, const Stage &st) {
        const int jb = j0 + 4 * half;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const bool jok = jb + u < jend;
            const float sj = (GT || !has_scale) ? 1.0f : st.sv[u];
            float av[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const float val = GT ? st.gv[t][u] * srow[t] : st.gv[t][u] * sj;
                av[t] = jok ? val : 0.0f;
            }
#pragma unroll
            for (int c = 0; c < CT; ++c) {
                uint32_t bits = 0;
#pragma unroll
                for (int q = 0; q < CB; ++q) bits |= ((st.pw[u][c][q] >> l5) & 1u) << q;
                const float bv = (float)(2 * (int)bits - kOffset);
#pragma unroll
                for (int t = 0; t < NT; ++t) acc[t][c] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[t], bv, acc[t][c], 0, 0, 0);
            }
        }
    };
    if (jbeg < jend) {
        Stage s0, s1;
        load(jbeg, s0);
        for (int j0 = jbeg; j0 < jend; j0 += 16) {       // the second half of the last pass may be all masked
            load(j0 + 8, s1);
            compute(j0, s0);
            load(j0 + 16, s0);
            compute(j0 + 8, s1);
        }
    }
    auto store = [&](int t, int c, int v, float val) {
        const int row = r0 + t * 32 + 8 * (v / 4) + 4 * half + (v % 4);
        const int col = (cw0 + c) * 32 + l5;
        if (row < a.R && col < a.C) {
            for (int p = 0; p < a.P; ++p) {
                a.out[((int64_t)p * a.R + row) * a.C + col] = val;
                val *= 2.0f;                              // exact
            }
        }
    };
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int c = 0; c < CT; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) store(t, c, v, acc[t][c][v]);
}

// Outputs of many tiles: the same block tile (128 rows x 128 columns, wavefront v the columns of
// plane word 4*cb + v), with the real operand staged through LDS in tiles of 32 reduction indices.
// Read straight from memory, a lane's values of one row lie 16 bytes apart from one iteration to the
// next and the rows of a tile a whole row of g apart: every cache line is fetched again for each
// 32 bytes used (measured: matrix pipes busy in 62 % of the cycles).  Here the 256 threads load a
// tile [128 rows][32 indices] with whole lines, scale it and keep it as [index][row] (row stride
// 132 words) in one of two LDS buffers; the next tile is loaded into registers before the matrix
// instructions of the current one and written to the other buffer after them, one barrier per tile.
// The plane words of a tile's 32 indices are loaded by lanes 0..31 (one index each) and handed out
// per step with ds_bpermute (one instruction per plane; two v_readlane and a select measured
// slower).  A wavefront whose plane word lies past the last one still loads, stores and waits with
// the others and only skips the products.  (Tried against this tile: a 2 x 2 arrangement of the
// wavefronts with two row tiles and two plane words each, 5-20 % slower without the LDS stage.)
// VEC: 16-byte loads (ldg, and J or R, multiples of 4; g and scale 16-byte aligned), else scalar loads.
template <int CB, bool GT, bool VEC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2)))
void backward_gemm_lds_kernel(const BackArgs a) {
    constexpr int KT = 32, LD = 132;
    __shared__ __attribute__((aligned(16))) float tile[2][KT][LD];
    const int tid = (int)threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int half = lane >> 5, l5 = lane & 31;
    const int rb = (int)(blockIdx.x / (unsigned)a.col_blocks);
    const int cb = (int)(blockIdx.x - (unsigned)rb * (unsigned)a.col_blocks);
    const int r0 = rb * 128;
    const int cw = cb * 4 + wave;
    const bool active = cw < a.Cw;
    const int cwc = active ? cw : a.Cw - 1;
    const bool has_scale = a.scale != nullptr;
    constexpr int kOffset = (1 << CB) - 1;
    f32x16 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;
    // this thread's part of a tile: four pieces of four values
    //   !GT: piece i = row r0 + tid / 8 + 32 i, indices j0 + 4 (tid % 8) .. + 3   (a quarter line of g)
    //    GT: piece i = index j0 + tid / 32 + 8 i, rows r0 + 4 (tid % 32) .. + 3
    struct Regs {
        f32x4 v[4];
        f32x4 sc;                                       // !GT: the scale of the piece's four indices
        uint32_t pw[CB];                                // lanes 0..31: plane words of index j0 + lane
    };
    f32x4 srow = {1.0f, 1.0f, 1.0f, 1.0f};              // GT: the scale of the piece's four rows
    if constexpr (GT) {
        if (has_scale) {
#pragma unroll
            for (int e = 0; e < 4; ++e) srow[e] = a.scale[min(r0 + 4 * (tid & 31) + e, a.R - 1)];
        }
    }
    auto load = [&](int j0, Regs &rg) {
        {
            const int jc = min(j0 + l5, a.J - 1);
#pragma unroll
            for (int q = 0; q < CB; ++q) rg.pw[q] = a.planes[((int64_t)jc * CB + q) * a.Cw + cwc];
        }
        if constexpr (!GT) {
            const int jp = j0 + 4 * (tid & 7);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = min(r0 + (tid >> 3) + 32 * i, a.R - 1);
                if constexpr (VEC) {
                    rg.v[i] = *reinterpret_cast<const f32x4 *>(a.g + (int64_t)row * a.ldg + min(jp, a.J - 4));
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) rg.v[i][e] = a.g[(int64_t)row * a.ldg + min(jp + e, a.J - 1)];
                }
            }
            if constexpr (VEC) {
                const float *sp = has_scale ? a.scale + min(jp, a.J - 4) : a.g;
                rg.sc = *reinterpret_cast<const f32x4 *>(sp);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) rg.sc[e] = has_scale ? a.scale[min(jp + e, a.J - 1)] : 1.0f;
            }
        } else {
            const int rp = r0 + 4 * (tid & 31);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int j = min(j0 + (tid >> 5) + 8 * i, a.J - 1);
                if constexpr (VEC) {
                    rg.v[i] = *reinterpret_cast<const f32x4 *>(a.g + (int64_t)j * a.ldg + min(rp, a.R - 4));
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) rg.v[i][e] = a.g[(int64_t)j * a.ldg + min(rp + e, a.R - 1)];
                }
            }
        }
    };
    // registers -> LDS [index][row], scaled; indices past J become zero
    auto stage = [&](int j0, const Regs &rg, int buf) {
        if constexpr (!GT) {
            const int jl = 4 * (tid & 7);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int rl = (tid >> 3) + 32 * i;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float s = has_scale ? rg.sc[e] : 1.0f;
                    tile[buf][jl + e][rl] = (j0 + jl + e < a.J) ? rg.v[i][e] * s : 0.0f;
                }
            }
        } else {
            const int rl = 4 * (tid & 31);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int jl = (tid >> 5) + 8 * i;
                f32x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (j0 + jl < a.J) ? rg.v[i][e] * srow[e] : 0.0f;
                *reinterpret_cast<f32x4 *>(&tile[buf][jl][rl]) = o;
            }
        }
    };
    auto compute = [&](const uint32_t (&pw)[CB], int buf) {
        // both operands of a step are fetched a step ahead: the real one from LDS, the code through ds_bpermute
        auto code = [&](int s) {
            uint32_t bits = 0;
#pragma unroll
            for (int q = 0; q < CB; ++q) {
                // the word of index 2s (lanes 0..31) or 2s+1 (lanes 32..63), held by the lane of that number
                const uint32_t w = (uint32_t)__builtin_amdgcn_ds_bpermute((2 * s + half) << 2, (int)pw[q]);
                bits |= ((w >> l5) & 1u) << q;
            }
            return (float)(2 * (int)bits - kOffset);
        };
        float an[4], bn = code(0);
#pragma unroll
        for (int t = 0; t < 4; ++t) an[t] = tile[buf][half][t * 32 + l5];
#pragma unroll
        for (int s = 0; s < KT / 2; ++s) {
            float ac[4];
            const float bc = bn;
#pragma unroll
            for (int t = 0; t < 4; ++t) ac[t] = an[t];
            if (s + 1 < KT / 2) {
#pragma unroll
                for (int t = 0; t < 4; ++t) an[t] = tile[buf][2 * (s + 1) + half][t * 32 + l5];
                bn = code(s + 1);
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(ac[t], bc, acc[t], 0, 0, 0);
        }
    };
    if (a.J > 0) {
        Regs rg;
        uint32_t pw_cur[CB];
        load(0, rg);
        stage(0, rg, 0);
#pragma unroll
        for (int q = 0; q < CB; ++q) pw_cur[q] = rg.pw[q];
        __syncthreads();
        int buf = 0;
        for (int j0 = 0; j0 < a.J; j0 += KT) {
            const bool more = j0 + KT < a.J;             // uniform over the block
            if (more) load(j0 + KT, rg);
            if (active) compute(pw_cur, buf);
            if (more) {
                stage(j0 + KT, rg, buf ^ 1);
#pragma unroll
                for (int q = 0; q < CB; ++q) pw_cur[q] = rg.pw[q];
            }
            __syncthreads();
            buf ^= 1;
        }
    }
    if (!active) return;
    const int col = cw * 32 + l5;
    if (col >= a.C) return;
#pragma unroll
    for (int t = 0; t < 4; ++t)
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

// Outputs of few tiles with long sums, staged through LDS: the block takes 32*RT rows x 32 columns
// (one plane word) and its four wavefronts a quarter of the sum each (four times the wavefronts of a
// tile per block, deterministic: no atomics); every wavefront brings its part of the real operand
// in through LDS in tiles of 32 indices
// (whole cache lines per load, [index][row] with a row stride of 32*RT + 4 words, two buffers, one
// barrier per tile: all wavefronts make the same number of passes, those past the end of the sum
// stage zeros).  The four partial tiles are then added in LDS in a fixed order.
template <int CB, int RT, bool GT, bool VEC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2)))
void backward_gemm_split_lds_kernel(const BackArgs a) {
    constexpr int KT = 32, ROWS = 32 * RT, LD = ROWS + 4, PIECES = 4 * RT;
    constexpr int TILE_WORDS = 2 * 4 * KT * LD, PART_WORDS = 4 * RT * 16 * 64;
    __shared__ __attribute__((aligned(16))) float lds[TILE_WORDS > PART_WORDS ? TILE_WORDS : PART_WORDS];
    const int wave = (int)(threadIdx.x >> 6), lane = (int)(threadIdx.x & 63);
    const int half = lane >> 5, l5 = lane & 31;
    const int rb = (int)(blockIdx.x / (unsigned)a.col_blocks);
    const int cw = (int)(blockIdx.x - (unsigned)rb * (unsigned)a.col_blocks);      // < Cw always
    const int r0 = rb * ROWS;
    const bool has_scale = a.scale != nullptr;
    constexpr int kOffset = (1 << CB) - 1;
    const int quarter = ((a.J + 4 * KT - 1) / (4 * KT)) * KT;                       // a multiple of 32
    const int jbeg = min(a.J, wave * quarter), jend = min(a.J, jbeg + quarter);
    auto tile = [&](int buf, int j, int r) -> float & { return lds[((buf * 4 + wave) * KT + j) * LD + r]; };
    f32x16 acc[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;
    // this lane's part of a tile: PIECES pieces of four values
    //   !GT: piece i = row r0 + lane / 8 + 8 i, indices j0 + 4 (lane % 8) .. + 3
    //    GT: piece i = index j0 + lane / (8 RT) + (8 / RT) i, rows r0 + 4 (lane % (8 RT)) .. + 3
    struct Regs {
        f32x4 v[PIECES];
        f32x4 sc;
        uint32_t pw[CB];
    };
    f32x4 srow = {1.0f, 1.0f, 1.0f, 1.0f};
    if constexpr (GT) {
        if (has_scale) {
#pragma unroll
            for (int e = 0; e < 4; ++e) srow[e] = a.scale[min(r0 + 4 * (lane % (8 * RT)) + e, a.R - 1)];
        }
    }
    const int jlast = max(jend - 1, 0);                                              // a valid index for clamped loads
    auto load = [&](int j0, Regs &rg) {
        {
            const int jc = min(j0 + l5, jlast);
#pragma unroll
            for (int q = 0; q < CB; ++q) rg.pw[q] = a.planes[((int64_t)jc * CB + q) * a.Cw + cw];
        }
        if constexpr (!GT) {
            const int jp = j0 + 4 * (lane & 7);
#pragma unroll
            for (int i = 0; i < PIECES; ++i) {
                const int row = min(r0 + (lane >> 3) + 8 * i, a.R - 1);
                if constexpr (VEC) {
                    rg.v[i] = *reinterpret_cast<const f32x4 *>(a.g + (int64_t)row * a.ldg + min(jp, a.J - 4));
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) rg.v[i][e] = a.g[(int64_t)row * a.ldg + min(jp + e, a.J - 1)];
                }
            }
            if constexpr (VEC) {
                const float *sp = has_scale ? a.scale + min(jp, a.J - 4) : a.g;
                rg.sc = *reinterpret_cast<const f32x4 *>(sp);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) rg.sc[e] = has_scale ? a.scale[min(jp + e, a.J - 1)] : 1.0f;
            }
        } else {
            const int rp = r0 + 4 * (lane % (8 * RT));
#pragma unroll
            for (int i = 0; i < PIECES; ++i) {
                const int j = min(j0 + lane / (8 * RT) + (8 / RT) * i, a.J - 1);
                if constexpr (VEC) {
                    rg.v[i] = *reinterpret_cast<const f32x4 *>(a.g + (int64_t)j * a.ldg + min(rp, a.R - 4));
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) rg.v[i][e] = a.g[(int64_t)j * a.ldg + min(rp + e, a.R - 1)];
                }
            }
        }
    };
    // registers -> LDS [index][row], scaled; indices past the wavefront's part of the sum become zero
    auto stage = [&](int j0, const Regs &rg, int buf) {
        if constexpr (!GT) {
            const int jl = 4 * (lane & 7);
#pragma unroll
            for (int i = 0; i < PIECES; ++i) {
                const int rl = (lane >> 3) + 8 * i;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float s = has_scale ? rg.sc[e] : 1.0f;
                    tile(buf, jl + e, rl) = (j0 + jl + e < jend) ? rg.v[i][e] * s : 0.0f;
                }
            }
        } else {
            const int rl = 4 * (lane % (8 * RT));
#pragma unroll
            for (int i = 0; i < PIECES; ++i) {
                const int jl = lane / (8 * RT) + (8 / RT) * i;
                f32x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (j0 + jl < jend) ? rg.v[i][e] * srow[e] : 0.0f;
                *reinterpret_cast<f32x4 *>(&tile(buf, jl, rl)) = o;
            }
        }
    };
    auto compute = [&](const uint32_t (&pw)[CB], int buf) {
        auto code = [&](int s) {
            uint32_t bits = 0;
#pragma unroll
            for (int q = 0; q < CB; ++q) {
                const uint32_t w = (uint32_t)__builtin_amdgcn_ds_bpermute((2 * s + half) << 2, (int)pw[q]);
                bits |= ((w >> l5) & 1u) << q;
            }
            return (float)(2 * (int)bits - kOffset);
        };
        float an[RT], bn = code(0);
#pragma unroll
        for (int t = 0; t < RT; ++t) an[t] = tile(buf, half, t * 32 + l5);
#pragma unroll
        for (int s = 0; s < KT / 2; ++s) {
            float ac[RT];
            const float bc = bn;
#pragma unroll
            for (int t = 0; t < RT; ++t) ac[t] = an[t];
            if (s + 1 < KT / 2) {
#pragma unroll
                for (int t = 0; t < RT; ++t) an[t] = tile(buf, 2 * (s + 1) + half, t * 32 + l5);
                bn = code(s + 1);
            }
#pragma unroll
            for (int t = 0; t < RT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(ac[t], bc, acc[t], 0, 0, 0);
        }
    };
    if (quarter > 0) {
        Regs rg;
        uint32_t pw_cur[CB];
        load(jbeg, rg);
        stage(jbeg, rg, 0);
#pragma unroll
        for (int q = 0; q < CB; ++q) pw_cur[q] = rg.pw[q];
        __syncthreads();
        int buf = 0;
        for (int k = 0; k < quarter; k += KT) {                                      // the same count in every wavefront
            const bool more = k + KT < quarter;
            if (more) load(jbeg + k + KT, rg);
            compute(pw_cur, buf);
            if (more) {
                stage(jbeg + k + KT, rg, buf ^ 1);
#pragma unroll
                for (int q = 0; q < CB; ++q) pw_cur[q] = rg.pw[q];
            }
            __syncthreads();
            buf ^= 1;
        }
    }
    // the four partial tiles meet in LDS (the tile buffers are free after the last barrier)
    float *part = lds;
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) part[((wave * RT + t) * 16 + v) * 64 + lane] = acc[t][v];
    __syncthreads();
    const int col = cw * 32 + l5;
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int v = wave * 4 + k;                  // a quarter of the tile's registers per wavefront
            auto at = [&](int w) { return part[((w * RT + t) * 16 + v) * 64 + lane]; };
            float val = ((at(0) + at(1)) + at(2)) + at(3);
            const int row = r0 + t * 32 + 8 * (v / 4) + 4 * half + (v % 4);
            if (row < a.R && col < a.C) {
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
    // rows per block: 128 where that still gives two blocks per compute unit, else 64 or 32; if even
    // that leaves fewer and the sum is long, blocks of 32 columns whose wavefronts split the sum
    const int64_t want = 2 * (int64_t)device_simd_count() / 4;
    auto blocks = [&](int rt, int words) { return ((int64_t)a.R + 32 * rt - 1) / (32 * rt) * ((a.Cw + words - 1) / words); };
    const bool split = blocks(1, 4) < want && a.J >= 256;
    int rt;
    if (split) rt = blocks(2, 1) >= want ? 2 : 1;           // (32-row tiles throughout measured 13 % slower on 256 x 4096 x 4096)
    else rt = blocks(4, 4) >= want ? 4 : blocks(2, 4) >= want ? 2 : 1;
    a.col_blocks = split ? a.Cw : (a.Cw + 3) / 4;
    const int64_t nb = blocks(rt, split ? 1 : 4);
    if (nb > 0x7fffffff) return hipErrorInvalidValue;
    const dim3 grid((unsigned)nb);
    if (split) {
        if (rt == 2) {
            if (a.lds_vec) launch_kernel((backward_gemm_split_lds_kernel<CB, 2, GT, true>), grid, dim3(256), 0, s, a);
            else launch_kernel((backward_gemm_split_lds_kernel<CB, 2, GT, false>), grid, dim3(256), 0, s, a);
        } else {
            if (a.lds_vec) launch_kernel((backward_gemm_split_lds_kernel<CB, 1, GT, true>), grid, dim3(256), 0, s, a);
            else launch_kernel((backward_gemm_split_lds_kernel<CB, 1, GT, false>), grid, dim3(256), 0, s, a);
        }
    } else {
        if (rt == 4) {
            if (a.lds_vec) launch_kernel((backward_gemm_lds_kernel<CB, GT, true>), grid, dim3(256), 0, s, a);
            else launch_kernel((backward_gemm_lds_kernel<CB, GT, false>), grid, dim3(256), 0, s, a);
        } else if (rt == 2) launch_one<CB, 2, GT>(a, vec, grid, s);
        else launch_one<CB, 1, GT>(a, vec, grid, s);
    }
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

// ---------------------------------------------------------------------------------------
// The same backward lines through a 3x3 / stride 1 / zero padding 1 convolution (NHWC).
//   towards the activations:  g_x[p][pixel q][c] = 2^p sum_{o, tap} s[o] g[q - off(tap)][o] w[o][tap][c]
//     rows = pixels, sum index j = tap * O + o (tap-major, so that consecutive indices are consecutive
//     filters of one gradient pixel: 16-byte loads; the packed weights' row of j is 9 o + tap), the
//     real operand gathered from the gradient image: G(q, j) = s[o] g[q - off(tap)][o] where that
//     output position exists, else 0;
//   towards the weights:      g_w[p][o][tap][c] = 2^p s[o] sum_{pixel q} g[q][o] x[q + off(tap)][c]
//     rows = filters, columns = channels, one pass per tap, sum index = pixel; the codes are the
//     activation planes of the neighbouring pixel, G is zero where that neighbour does not exist.
//     The output is small and the sum long, so the pixels are cut into `splits` ranges, every
//     range writes its partial result to a workspace [splits][O][9][C], and a second kernel adds
//     the ranges in a fixed order and writes the 2^p copies (deterministic, no atomics).
// Both on the LDS-staged tile scheme of backward_gemm_lds_kernel (128 x 128 per block, tiles of
// 32 sum indices, two buffers, one barrier per tile, plane words through ds_bpermute).
// ---------------------------------------------------------------------------------------
struct ConvBackArgs {
    const float *g;          // [pixels][O]
    const float *scale;      // [O] or nullptr
    const uint32_t *planes;  // weights [O][9][CB][Cw] (towards the activations) / activations [pixels][CB][Cw]
    float *out;              // towards the activations: [P][pixels][C]; towards the weights: workspace [splits][O][9][C]
    int pixels, H, W, O, C, Cw, P;
    int row_blocks, col_blocks, splits, per_split;     // per_split: pixels per range, a multiple of 32
    FastDiv div_w, div_h, div_o;
    int vec_in;              // towards the activations: 16-byte loads of the gradient and the scale are possible
};

// WC: plane words (32 columns each) per block, 4, 2 or 1 for layers of at least 97, 33 or fewer channels: the
// four wavefronts then form 4 / WC row groups of WC row tiles each, so that none of them idles on a narrow layer.
// HALF (towards the weights, at most 64 filters): only the first 64 rows of the tile exist, so every
// wavefront takes half as many row tiles (WC / 2) and no matrix instruction works on empty rows.
template <int CB, bool TW, bool VEC, int WC, bool HALF = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2)))
void backward_conv_kernel(const ConvBackArgs a) {
    static_assert(!HALF || (TW && WC >= 2), "half tiles: weight gradient, at least two plane words per block");
    constexpr int KT = 32, LD = 132, NT = HALF ? WC / 2 : WC;
    __shared__ __attribute__((aligned(16))) float tile[2][KT][LD];
    const int tid = (int)threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int half = lane >> 5, l5 = lane & 31;
    // block -> (range of pixels, tap, row block, column block); the first two only towards the weights
    uint32_t bid = blockIdx.x;
    const int cb = (int)(bid % (uint32_t)a.col_blocks);
    bid /= (uint32_t)a.col_blocks;
    const int rb = (int)(bid % (uint32_t)a.row_blocks);
    bid /= (uint32_t)a.row_blocks;
    const int tap = TW ? (int)(bid % 9u) : 0, split = TW ? (int)(bid / 9u) : 0;
    const int R = TW ? a.O : a.pixels;
    const int jbeg = TW ? min(a.pixels, split * a.per_split) : 0;
    const int jend = TW ? min(a.pixels, jbeg + a.per_split) : 9 * a.O;
    const int r0 = rb * 128;
    const int cw = cb * WC + wave % WC;
    const int rw = (wave / WC) * (32 * NT);             // this wavefront's rows inside the block's 128
    const bool active = cw < a.Cw;
    const int cwc = active ? cw : a.Cw - 1;
    const bool has_scale = a.scale != nullptr;
    const int tdh = tap / 3 - 1, tdw = tap % 3 - 1;    // towards the weights: this pass's tap
    constexpr int kOffset = (1 << CB) - 1;
    f32x16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;
    struct Regs {
        f32x4 v[4];
        f32x4 sc;
        uint32_t ok;                                    // which of the values take part (their image position exists)
        uint32_t pw[CB];
    };
    // towards the activations: the four pixels of this thread's pieces (row r0 + tid / 8 + 32 i)
    int pq[4], ph[4], pwd[4];
    f32x4 srow = {1.0f, 1.0f, 1.0f, 1.0f};
    if constexpr (!TW) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            pq[i] = min(r0 + (tid >> 3) + 32 * i, a.pixels - 1);
            int line, n;
            fast_divmod((uint32_t)pq[i], a.div_w, line, pwd[i]);
            fast_divmod((uint32_t)line, a.div_h, n, ph[i]);
        }
    } else {
        if (has_scale) {
#pragma unroll
            for (int e = 0; e < 4; ++e) srow[e] = a.scale[min(r0 + 4 * (tid & 31) + e, a.O - 1)];
        }
    }
    const int jlast = max(jend - 1, 0);
    auto load = [&](int j0, Regs &rg) {
        rg.ok = 0u;
        if constexpr (!TW) {
            {
                const int jc = min(j0 + l5, jlast);
                int t, o;
                fast_divmod((uint32_t)jc, a.div_o, t, o);
                const int wrow = 9 * o + t;                      // the packed weights are [O][9]
#pragma unroll
                for (int q = 0; q < CB; ++q) rg.pw[q] = a.planes[((int64_t)wrow * CB + q) * a.Cw + cwc];
            }
            const int jp = j0 + 4 * (tid & 7);
            if constexpr (VEC) {
                // O is a multiple of 4: the four indices of a piece are four filters of one tap
                int t, o;
                fast_divmod((uint32_t)min(jp, jlast - 3), a.div_o, t, o);
                const int dh = t / 3 - 1, dw = t - 3 * (t / 3) - 1;
                const float *sp = has_scale ? a.scale + o : a.g;
                rg.sc = *reinterpret_cast<const f32x4 *>(sp);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const bool ok = (unsigned)(ph[i] - dh) < (unsigned)a.H && (unsigned)(pwd[i] - dw) < (unsigned)a.W;
                    const int src = ok ? pq[i] - dh * a.W - dw : pq[i];
                    rg.v[i] = *reinterpret_cast<const f32x4 *>(a.g + (int64_t)src * a.O + o);
                    rg.ok |= (ok ? 15u : 0u) << (4 * i);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    int t, o;
                    fast_divmod((uint32_t)min(jp + e, jlast), a.div_o, t, o);
                    const int dh = t / 3 - 1, dw = t - 3 * (t / 3) - 1;
                    rg.sc[e] = has_scale ? a.scale[o] : 1.0f;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const bool ok = (unsigned)(ph[i] - dh) < (unsigned)a.H && (unsigned)(pwd[i] - dw) < (unsigned)a.W;
                        const int src = ok ? pq[i] - dh * a.W - dw : pq[i];
                        rg.v[i][e] = a.g[(int64_t)src * a.O + o];
                        rg.ok |= (ok ? 1u : 0u) << (4 * i + e);
                    }
                }
            }
        } else {
            {
                // the neighbour of pixel j0 + lane under this tap (any valid pixel if it does not exist)
                const int pj = min(j0 + l5, jlast) + tdh * a.W + tdw;
                const int pc = min(max(pj, 0), a.pixels - 1);
#pragma unroll
                for (int q = 0; q < CB; ++q) rg.pw[q] = a.planes[((int64_t)pc * CB + q) * a.Cw + cwc];
            }
            const int rp = r0 + 4 * (tid & 31);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int j = min(j0 + (tid >> 5) + 8 * i, jlast);
                int line, n, h, w;
                fast_divmod((uint32_t)j, a.div_w, line, w);
                fast_divmod((uint32_t)line, a.div_h, n, h);
                const bool ok = (unsigned)(h + tdh) < (unsigned)a.H && (unsigned)(w + tdw) < (unsigned)a.W;
                rg.ok |= (ok ? 1u : 0u) << i;
                if constexpr (VEC) {
                    rg.v[i] = *reinterpret_cast<const f32x4 *>(a.g + (int64_t)j * a.O + min(rp, a.O - 4));
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) rg.v[i][e] = a.g[(int64_t)j * a.O + min(rp + e, a.O - 1)];
                }
            }
        }
    };
    auto stage = [&](int j0, const Regs &rg, int buf) {
        if constexpr (!TW) {
            const int jl = 4 * (tid & 7);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int rl = (tid >> 3) + 32 * i;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool use = (j0 + jl + e < jend) && ((rg.ok >> (4 * i + e)) & 1u);
                    tile[buf][jl + e][rl] = use ? rg.v[i][e] * (has_scale ? rg.sc[e] : 1.0f) : 0.0f;
                }
            }
        } else {
            const int rl = 4 * (tid & 31);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int jl = (tid >> 5) + 8 * i;
                const bool use = (j0 + jl < jend) && ((rg.ok >> i) & 1u);
                f32x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = use ? rg.v[i][e] * srow[e] : 0.0f;
                *reinterpret_cast<f32x4 *>(&tile[buf][jl][rl]) = o;
            }
        }
    };
    auto compute = [&](const uint32_t (&pw)[CB], int buf) {
        auto code = [&](int s) {
            uint32_t bits = 0;
#pragma unroll
            for (int q = 0; q < CB; ++q) {
                const uint32_t w = (uint32_t)__builtin_amdgcn_ds_bpermute((2 * s + half) << 2, (int)pw[q]);
                bits |= ((w >> l5) & 1u) << q;
            }
            return (float)(2 * (int)bits - kOffset);
        };
        float an[NT], bn = code(0);
#pragma unroll
        for (int t = 0; t < NT; ++t) an[t] = tile[buf][half][rw + t * 32 + l5];
#pragma unroll
        for (int s = 0; s < KT / 2; ++s) {
            float ac[NT];
            const float bc = bn;
#pragma unroll
            for (int t = 0; t < NT; ++t) ac[t] = an[t];
            if (s + 1 < KT / 2) {
#pragma unroll
                for (int t = 0; t < NT; ++t) an[t] = tile[buf][2 * (s + 1) + half][rw + t * 32 + l5];
                bn = code(s + 1);
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(ac[t], bc, acc[t], 0, 0, 0);
        }
    };
    if (jbeg < jend) {                                  // uniform over the block
        Regs rg;
        uint32_t pw_cur[CB];
        load(jbeg, rg);
        stage(jbeg, rg, 0);
#pragma unroll
        for (int q = 0; q < CB; ++q) pw_cur[q] = rg.pw[q];
        __syncthreads();
        int buf = 0;
        for (int j0 = jbeg; j0 < jend; j0 += KT) {
            const bool more = j0 + KT < jend;
            if (more) load(j0 + KT, rg);
            if (active) compute(pw_cur, buf);
            if (more) {
                stage(j0 + KT, rg, buf ^ 1);
#pragma unroll
                for (int q = 0; q < CB; ++q) pw_cur[q] = rg.pw[q];
            }
            __syncthreads();
            buf ^= 1;
        }
    }
    if (!active) return;
    const int col = cw * 32 + l5;
    if (col >= a.C) return;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = r0 + rw + t * 32 + 8 * (v / 4) + 4 * half + (v % 4);
            if (row < R) {
                float val = acc[t][v];
                if constexpr (TW) {
                    a.out[(((int64_t)split * a.O + row) * 9 + tap) * a.C + col] = val;
                } else {
                    for (int p = 0; p < a.P; ++p) {
                        a.out[((int64_t)p * a.pixels + row) * a.C + col] = val;
                        val *= 2.0f;                      // exact
                    }
                }
            }
        }
}

// out[p][i] = 2^p * (ws[0][i] + ws[1][i] + ...), the ranges added in their order
__global__ __launch_bounds__(256) void backward_conv_reduce_kernel(const float *__restrict__ ws, int splits, int64_t n, int P,
                                                                    float *__restrict__ out) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        float val = ws[i];
        for (int s = 1; s < splits; ++s) val += ws[(int64_t)s * n + i];
        for (int p = 0; p < P; ++p) {
            out[(int64_t)p * n + i] = val;
            val *= 2.0f;
        }
    }
}

template <bool TW, int WC>
hipError_t launch_conv_back_wc(int cb, const ConvBackArgs &a, bool vec, dim3 grid, hipStream_t s) {
#define QNN_CB(N)                                                                                          \
    case N:                                                                                                \
        if constexpr (TW) {                                                                                \
            if constexpr (WC >= 2) {                                                                       \
                if (a.O <= 64) {                                                                           \
                    if (vec) launch_kernel((backward_conv_kernel<N, true, true, WC, true>), grid, dim3(256), 0, s, a);   \
                    else launch_kernel((backward_conv_kernel<N, true, false, WC, true>), grid, dim3(256), 0, s, a);      \
                    break;                                                                                 \
                }                                                                                          \
            }                                                                                              \
            if (vec) launch_kernel((backward_conv_kernel<N, true, true, WC>), grid, dim3(256), 0, s, a);   \
            else launch_kernel((backward_conv_kernel<N, true, false, WC>), grid, dim3(256), 0, s, a);      \
        } else {                                                                                           \
            if (vec) launch_kernel((backward_conv_kernel<N, false, true, WC>), grid, dim3(256), 0, s, a);  \
            else launch_kernel((backward_conv_kernel<N, false, false, WC>), grid, dim3(256), 0, s, a);     \
        }                                                                                                  \
        break;
    switch (cb) {
        QNN_CB(1) QNN_CB(2) QNN_CB(3) QNN_CB(4) QNN_CB(5) QNN_CB(6) QNN_CB(7) QNN_CB(8)
        default: return hipErrorInvalidValue;
    }
#undef QNN_CB
    return launch_status();
}

// plane words per block: four from 97 channels on, two from 33, else one
inline int conv_back_words(int Cw) { return Cw >= 3 ? 4 : Cw; }

template <bool TW>
hipError_t launch_conv_back(int cb, const ConvBackArgs &a, bool vec, dim3 grid, hipStream_t s) {
    switch (conv_back_words(a.Cw)) {
        case 4: return launch_conv_back_wc<TW, 4>(cb, a, vec, grid, s);
        case 2: return launch_conv_back_wc<TW, 2>(cb, a, vec, grid, s);
        default: return launch_conv_back_wc<TW, 1>(cb, a, vec, grid, s);
    }
}

// Adam: every step one correctly rounded binary32 operation, in this order (the CPU reference does the same)
__global__ __launch_bounds__(256) void update_adam_kernel(float *__restrict__ w, const float *__restrict__ g, float *__restrict__ m,
                                                           float *__restrict__ v, int64_t n, float lr, float b1, float b2,
                                                           float omb1, float omb2, float bc1, float bc2, float eps) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const float gi = g[i];
        const float mn = __fadd_rn(__fmul_rn(b1, m[i]), __fmul_rn(omb1, gi));
        const float vn = __fadd_rn(__fmul_rn(b2, v[i]), __fmul_rn(omb2, __fmul_rn(gi, gi)));
        // plain division and sqrtf: correctly rounded in this compiler's default mode for device code (the
        // __fdiv_rn / __fsqrt_rn intrinsics map to the approximate hardware operations unless the math
        // library is built with rounded operations)
        const float mh = mn / bc1, vh = vn / bc2;
        const float step = __fmul_rn(lr, mh) / __fadd_rn(sqrtf(vh), eps);
        m[i] = mn;
        v[i] = vn;
        w[i] = __fsub_rn(w[i], step);
    }
}

}  // namespace

// out[p][r][c] = 2^p sum_j G(r, j) code[j][c]; towards_weights selects G(r, j) = g[j][r] scale[r],
// else g[r][j] scale[j].  R, C >= 1; J may be 0 (the output is then zero).
hipError_t launch_backward_gemm(const float *g, int64_t ldg, const float *scale, const uint32_t *planes, int code_bits,
                                int R, int J, int C, int P, bool towards_weights, float *out, hipStream_t s) {
    BackArgs a;
    a.g = g; a.scale = scale; a.planes = planes; a.out = out;
    a.R = R; a.J = J; a.C = C; a.Cw = (C + 31) / 32; a.P = P; a.col_blocks = 0; a.ldg = ldg;
    const bool aligned = ldg % 4 == 0 && ((((uintptr_t)g) & 15u) == 0) && (scale == nullptr || (((uintptr_t)scale) & 15u) == 0);
    a.lds_vec = (aligned && (towards_weights ? R % 4 == 0 && R >= 4 : J % 4 == 0 && J >= 4)) ? 1 : 0;
    const bool vec = !towards_weights && J % 8 == 0 && ldg % 4 == 0 && ((((uintptr_t)g) & 15u) == 0) &&
                     (scale == nullptr || (((uintptr_t)scale) & 15u) == 0);
    return towards_weights ? launch_form<true>(code_bits, a, vec, s) : launch_form<false>(code_bits, a, vec, s);
}

// pixel ranges of the weight gradient: enough blocks for two per compute unit of a 256-unit chip, at
// least 512 pixels per range, at most 64 ranges (a function of the sizes only: the workspace depends on it)
int conv_backward_splits(int64_t pixels, int64_t O, int64_t C) {
    const int64_t tiles = ((O + 127) / 128) * ((((C + 31) / 32) + 3) / 4) * 9;
    int64_t s = (512 + tiles - 1) / tiles;
    const int64_t most = pixels / 512 > 1 ? pixels / 512 : 1;
    if (s > most) s = most;
    if (s > 64) s = 64;
    return (int)(s < 1 ? 1 : s);
}

hipError_t launch_conv_backward_input(const float *g, const float *scale, const uint32_t *Wt, int wb, int64_t Nb, int H, int W,
                                      int C, int O, int P, float *out, hipStream_t s) {
    ConvBackArgs a;
    a.g = g; a.scale = scale; a.planes = Wt; a.out = out;
    a.pixels = (int)(Nb * H * W); a.H = H; a.W = W; a.O = O; a.C = C; a.Cw = (C + 31) / 32; a.P = P;
    a.row_blocks = (a.pixels + 127) / 128; a.col_blocks = (a.Cw + conv_back_words(a.Cw) - 1) / conv_back_words(a.Cw);
    a.splits = 1; a.per_split = 0;
    a.div_w = fast_div_for(W); a.div_h = fast_div_for(H); a.div_o = fast_div_for(O);
    const bool vec = O % 4 == 0 && O >= 4 && ((((uintptr_t)g) & 15u) == 0) && (scale == nullptr || (((uintptr_t)scale) & 15u) == 0);
    a.vec_in = vec ? 1 : 0;
    const int64_t nb = (int64_t)a.row_blocks * a.col_blocks;
    if (nb > 0x7fffffff) return hipErrorInvalidValue;
    return launch_conv_back<false>(wb, a, vec, dim3((unsigned)nb), s);
}

hipError_t launch_conv_backward_weight(const float *g, const float *scale, const uint32_t *x_planes, int ab, int64_t Nb, int H,
                                       int W, int C, int O, int P, float *out, float *workspace, hipStream_t s) {
    ConvBackArgs a;
    a.g = g; a.scale = scale; a.planes = x_planes; a.out = workspace;
    a.pixels = (int)(Nb * H * W); a.H = H; a.W = W; a.O = O; a.C = C; a.Cw = (C + 31) / 32; a.P = P;
    a.row_blocks = (O + 127) / 128; a.col_blocks = (a.Cw + conv_back_words(a.Cw) - 1) / conv_back_words(a.Cw);
    a.splits = conv_backward_splits(a.pixels, O, C);
    a.per_split = (int)(((((int64_t)a.pixels + a.splits - 1) / a.splits) + 31) / 32 * 32);
    a.div_w = fast_div_for(W); a.div_h = fast_div_for(H); a.div_o = fast_div_for(O); a.vec_in = 0;
    const int64_t nb = (int64_t)a.row_blocks * a.col_blocks * 9 * a.splits;
    if (nb > 0x7fffffff) return hipErrorInvalidValue;
    const bool vec = O % 4 == 0 && O >= 4 && ((((uintptr_t)g) & 15u) == 0);
    hipError_t e = launch_conv_back<true>(ab, a, vec, dim3((unsigned)nb), s);
    if (e != hipSuccess) return e;
    const int64_t n = (int64_t)O * 9 * C;
    const int64_t want = (n + 255) / 256, cap = (int64_t)device_simd_count() * 16;
    launch_kernel(backward_conv_reduce_kernel, dim3((unsigned)(want < cap ? want : cap)), dim3(256), 0, s,
                  (const float *)workspace, a.splits, n, P, out);
    return launch_status();
}

hipError_t launch_update_sgd(float *w, const float *g, int64_t n, float lr, hipStream_t s) {
    const int64_t want = (n + 255) / 256;
    const int64_t cap = (int64_t)device_simd_count() * 16;
    launch_kernel(update_sgd_kernel, dim3((unsigned)(want < cap ? want : cap)), dim3(256), 0, s, w, g, n, lr);
    return launch_status();
}

hipError_t launch_update_adam(float *w, const float *g, float *m, float *v, int64_t n, float lr, float b1, float b2,
                              float omb1, float omb2, float bc1, float bc2, float eps, hipStream_t s) {
    const int64_t want = (n + 255) / 256;
    const int64_t cap = (int64_t)device_simd_count() * 16;
    launch_kernel(update_adam_kernel, dim3((unsigned)(want < cap ? want : cap)), dim3(256), 0, s, w, g, m, v, n, lr, b1, b2,
                  omb1, omb2, bc1, bc2, eps);
    return launch_status();
}

}  // namespace qnn
