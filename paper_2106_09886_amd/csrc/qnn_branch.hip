// Multi-branch binary product kernels (paper Eq. (8)): GEMM and implicit-im2col 3x3
// convolution.  Compiled once per activation bit width, -DQNN_AB=<1..8>.
//
// Mapping (gfx950, 64-lane wavefronts).  A wavefront owns 64 output columns (lane = column
// / filter) and a contiguous run of rows (GEMM rows or output pixels):
//   * the weight words of the lane's column for the current K chunk stay in VGPRs;
//   * the activation words of the current row are the same for all 64 lanes, so they are
//     fetched with scalar loads and used as the SGPR operand of v_xor_b32;
//   * per 32 binary products and branch the loop issues exactly v_xor_b32 +
//     v_bcnt_u32_b32 (popcount with fused accumulate);
//   * branches with equal p+q share an accumulator; the 2^(p+q) weights are applied once
//     per row and chunk with AB+WB-2 shift-adds (Eq. (8) regrouped by p+q);
//   * stores are lane-contiguous: one 256-byte segment per row and wavefront, addressed
//     through a buffer descriptor (wave-uniform row offset in an SGPR, no vector address math).
// A product whose K extent does not fit the VGPR chunk is done in several chunk passes by
// the same wavefront; partial sums round-trip through the output buffer (same lane, same
// address, program order).
#include <type_traits>
#include "qnn_internal.h"
#include "qnn_device_util.h"

#ifndef QNN_AB
#error "compile with -DQNN_AB=<activation bits>"
#endif

namespace qnn {
namespace {

// S = sum_s 2^s part[s]  (Eq. (8) weights, grouped by s = p + q)
template <int NP>
__device__ __forceinline__ int weighted_sum(const int (&part)[NP]) {
    int s = part[NP - 1];
#pragma unroll
    for (int i = NP - 2; i >= 0; --i) s = (s << 1) + part[i];
    return s;
}

// Position of a wavefront.  Consecutive wavefronts (the four of a block first) take
// consecutive column tiles of the SAME row block: they request the same activation words, which
// then hit in the scalar cache, while each loads its own weight tile once.
struct WavePos {
    int ct;        // column tile
    int rb;        // row block
    int index;     // wavefront number in the grid
};
template <bool XCD_RANGES = false>                   // number the blocks by xcd_block()
__device__ __forceinline__ WavePos wave_pos(const FastDiv &col_tiles, int xcd_ranges = 0, uint32_t grid_blocks = 0) {
    WavePos p;
    const uint32_t block = XCD_RANGES ? xcd_block(xcd_ranges, grid_blocks) : blockIdx.x;
    p.index = __builtin_amdgcn_readfirstlane((int)(block * 4u + (threadIdx.x >> 6)));   // blocks of four wavefronts
    fast_divmod((uint32_t)p.index, col_tiles, p.rb, p.ct);
    return p;
}

// Optional per-wavefront trace (see qnn_set_wave_trace): four 64-bit words per wavefront,
// {start shader clock, end shader clock, HW_ID | XCC_ID << 32, start real-time clock}.
__device__ __forceinline__ void trace_begin(const BranchArgs &g, const WavePos &wp) {
    if (g.trace != nullptr && (uint32_t)wp.index < g.trace_waves && (threadIdx.x & 63) == 0) {
        uint64_t *t = g.trace + 4 * (int64_t)wp.index;
        t[0] = __builtin_amdgcn_s_memtime();                            // shader clock (local to the CU)
        t[2] = (uint64_t)__builtin_amdgcn_s_getreg((31 << 11) | 4)      // HW_ID: wave, SIMD, CU, SH, SE ids
             | ((uint64_t)__builtin_amdgcn_s_getreg((31 << 11) | 20) << 32);   // XCC_ID
        t[3] = __builtin_amdgcn_s_memrealtime();                        // constant 100 MHz clock (chip-wide)
    }
}
__device__ __forceinline__ void trace_end(const BranchArgs &g, const WavePos &wp) {
    if (g.trace != nullptr && (uint32_t)wp.index < g.trace_waves && (threadIdx.x & 63) == 0)
        g.trace[4 * (int64_t)wp.index + 1] = __builtin_amdgcn_s_memtime();
}

// Two-buffer software pipeline: stages ST .. NS-1 of one row.  Stage s is consumed from
// buffer (s + FLIP) & 1 while stage s+1 (or stage 0 of the next row) is in flight into the
// other buffer.  On entry stage ST has been requested; on exit stage 0 of the next row has.
template <int ST, bool FLIP, class Ctx>
__device__ __forceinline__ void run_stages(Ctx &c) {
    if constexpr (ST < Ctx::NS) {
        constexpr bool cur_is_a = (((ST & 1) == 0) != FLIP);
        auto &cur = cur_is_a ? c.bufA : c.bufB;
        auto &nxt = cur_is_a ? c.bufB : c.bufA;
        cur.template arrive<true>();
        if constexpr (ST + 1 < Ctx::NS) c.template request<ST + 1>(nxt, false);
        else c.template request<0>(nxt, true);
        c.template consume<ST>(cur);
        run_stages<ST + 1, FLIP>(c);
    }
}

// ---------------------------------------------------------------------------------------
// GEMM: acc[i][n] = sum_{p,q} 2^(p+q) (K - 2 popc(A[i][p] ^ Wt[n][q]))
// Chunk = SEGS segments (pipeline stages) of CWT words of every plane.
// ---------------------------------------------------------------------------------------
template <int AB, int WB, int SEGS, int CWT>
struct GemmCtx {
    static constexpr int NS = SEGS;
    typedef SStage<AB, CWT> Buf;     // run p = plane p, CWT consecutive K words
    uint64_t base;                   // byte address of A
    uint32_t plane_bytes;            // Kw * 4
    uint32_t off_cur, off_nxt;       // byte offset of (row, plane 0, word k0) for this / next row
    uint32_t w[SEGS][WB][CWT];
    int part[AB + WB - 1];
    Buf bufA, bufB;

    template <int ST>
    __device__ __forceinline__ void request(Buf &b, bool next_row) {
        const uint32_t off = (next_row ? off_nxt : off_cur);
#pragma unroll
        for (int p = 0; p < AB; ++p) b.run[p].template request<ST * CWT * 4>(base, off + (uint32_t)p * plane_bytes);
    }
    template <int ST>
    __device__ __forceinline__ void consume(const Buf &b) {
#pragma unroll
        for (int q = 0; q < WB; ++q)
#pragma unroll
            for (int p = 0; p < AB; ++p)
#pragma unroll
                for (int j = 0; j < CWT; ++j) popc_acc(part[p + q], b.run[p].get(j) ^ w[ST][q][j]);
    }
};

// full chunk (all KC words inside Kw): pipelined
// `fetch(rel_row)` returns what earlier chunks left for row r0 + rel_row; it is asked for before
// the row's products are formed, so that its latency hides behind them.
// `sink(rel_row, v, prev)` receives v = -2 * S of the chunk and that value.
//
// GATHER: row r of the product is output pixel r of a single-tap strided convolution, i.e. the
// activation row of input pixel (oh*sh, ow*sw) of its image.  `walk` is the state for row r0:
// byte offset of that pixel and its position; stepping to the next row is two additions and
// compares on the scalar unit, no division.
struct RowWalk {
    uint32_t off;      // byte offset of the row's activation words (plane 0, word 0)
    int ow, oh;        // output column and row inside the image
};
__device__ __forceinline__ RowWalk row_walk_at(const BranchArgs &g, int r, uint32_t row_bytes) {
    const ConvGeom &q = g.geo;
    RowWalk w;
    int line, img;                                  // output row counted over all images
    fast_divmod((uint32_t)r, g.div_w, line, w.ow);
    fast_divmod((uint32_t)line, g.div_h, img, w.oh);
    w.off = __builtin_amdgcn_readfirstlane((uint32_t)((img * g.H + w.oh * q.sh) * g.W + w.ow * q.sw) * row_bytes);
    return w;
}
__device__ __forceinline__ void row_walk_step(const BranchArgs &g, RowWalk &w, uint32_t row_bytes) {
    const ConvGeom &q = g.geo;
    w.off += (uint32_t)q.sw * row_bytes;
    if (++w.ow == q.Wo) {                       // next output row: back Wo*sw pixels, down sh input rows
        w.ow = 0;
        w.off += (uint32_t)(q.sh * g.W - q.Wo * q.sw) * row_bytes;          // modulo 2^32 on purpose
        if (++w.oh == q.Ho) {                   // next image
            w.oh = 0;
            w.off += (uint32_t)((g.H - q.Ho * q.sh) * g.W) * row_bytes;
        }
    }
}

template <int AB, int WB, int SEGS, int CWT, bool GATHER = false, class Fetch, class Sink>
__device__ __forceinline__ void gemm_chunk_full(const BranchArgs &g, int nload, int r0, int r1, int k0,
                                                Fetch fetch, Sink sink, RowWalk walk = RowWalk()) {
    GemmCtx<AB, WB, SEGS, CWT> c;
    const int Kw = g.Cw;
    c.base = (uint64_t)g.A;
    c.plane_bytes = (uint32_t)Kw * 4u;
    {
        constexpr int KC = SEGS * CWT, NW = WB * KC;
        uint32_t wl[NW];                              // word k = q * KC + (t * CWT + j)
        // (Fetching the block's tile once through LDS instead was measured and is not faster: these
        // loads happen once per chunk and wavefront and hit in L2.)
#pragma unroll
        for (int q = 0; q < WB; ++q) load_run<KC>(g.Wt + (nload * WB + q) * Kw + k0, wl + q * KC);
#pragma unroll
        for (int t = 0; t < SEGS; ++t)
#pragma unroll
            for (int q = 0; q < WB; ++q)
#pragma unroll
                for (int j = 0; j < CWT; ++j) c.w[t][q][j] = wl[q * KC + t * CWT + j];
    }
    const uint32_t row_bytes = (uint32_t)AB * c.plane_bytes;
    c.off_cur = (GATHER ? walk.off : (uint32_t)r0 * row_bytes) + (uint32_t)k0 * 4u;
    c.off_nxt = c.off_cur;
    c.template request<0>(c.bufA, false);
    int r = r0;
    auto one_row = [&](auto flip_tag) {
        constexpr bool FLIP = decltype(flip_tag)::value;
#pragma unroll
        for (int s = 0; s < AB + WB - 1; ++s) c.part[s] = 0;
        if constexpr (GATHER) {
            row_walk_step(g, walk, row_bytes);
            c.off_nxt = (r + 1 < r1) ? walk.off + (uint32_t)k0 * 4u : c.off_cur;
        } else {
            c.off_nxt = (r + 1 < r1) ? c.off_cur + row_bytes : c.off_cur;   // last row prefetches itself
        }
        const int prev = fetch(r - r0);
        run_stages<0, FLIP>(c);
        sink(r - r0, -2 * weighted_sum(c.part), prev);
        c.off_cur = c.off_nxt;
        ++r;
    };
    if constexpr ((SEGS & 1) == 0) {                   // stage 0 of every row uses the same buffer
        while (r < r1) one_row(std::integral_constant<bool, false>());
    } else {                                           // the starting buffer alternates from row to row
        while (r + 2 <= r1) {
            one_row(std::integral_constant<bool, false>());
            one_row(std::integral_constant<bool, true>());
        }
        if (r < r1) one_row(std::integral_constant<bool, false>());
    }
    // Drain the prefetch issued by the last row.  Both buffers are named so that their
    // registers stay reserved until the wait, whichever of them the prefetch went to.
    c.bufA.template arrive<true>();
    c.bufB.template arrive<false>();
}

// tail chunk (runs past Kw): plain loads with a guard per word
template <int AB, int WB, int SEGS, int CWT, bool GATHER = false, class Fetch, class Sink>
__device__ __forceinline__ void gemm_chunk_tail(const BranchArgs &g, uniform_words As, int nload, int r0,
                                                int r1, int k0, Fetch fetch, Sink sink, RowWalk walk = RowWalk()) {
    const int Kw = g.Cw;
    uint32_t w[SEGS][WB][CWT];
#pragma unroll
    for (int t = 0; t < SEGS; ++t)
#pragma unroll
        for (int q = 0; q < WB; ++q)
#pragma unroll
            for (int j = 0; j < CWT; ++j) {
                const int k = k0 + t * CWT + j;
                w[t][q][j] = (k < Kw) ? g.Wt[(nload * WB + q) * Kw + k] : 0u;
            }
    for (int r = r0; r < r1; ++r) {
        int part[AB + WB - 1];
#pragma unroll
        for (int s = 0; s < AB + WB - 1; ++s) part[s] = 0;
        const int prev = fetch(r - r0);
        const int row_word = GATHER ? (int)(walk.off >> 2) : r * AB * Kw;    // first word of the row
        if constexpr (GATHER) row_walk_step(g, walk, (uint32_t)(AB * Kw) * 4u);
#pragma unroll
        for (int t = 0; t < SEGS; ++t) {
            if (k0 + t * CWT < Kw) {             // uniform: skip segments that are all padding
                uint32_t a[AB][CWT];
#pragma unroll
                for (int p = 0; p < AB; ++p)
#pragma unroll
                    for (int j = 0; j < CWT; ++j) {
                        const int k = k0 + t * CWT + j;
                        a[p][j] = (k < Kw) ? As[row_word + p * Kw + k] : 0u;
                    }
#pragma unroll
                for (int q = 0; q < WB; ++q)
#pragma unroll
                    for (int p = 0; p < AB; ++p)
#pragma unroll
                        for (int j = 0; j < CWT; ++j) popc_acc(part[p + q], a[p][j] ^ w[t][q][j]);
            }
        }
        sink(r - r0, -2 * weighted_sum(part), prev);
    }
}

// Partial sums between the chunk passes of a wavefront, kept on chip: kLdsPartialRows rows x 64
// columns of int32 per wavefront (24 KB per block, six blocks per compute unit).  Every lane
// reads only what it wrote itself, so no barrier is involved.
template <bool ON> struct PartialSlab {
    __device__ static __forceinline__ int *mine() { return nullptr; }
};
template <> struct PartialSlab<true> {
    __device__ static __forceinline__ int *mine() {
        __shared__ int slab[4 * kLdsPartialRows * 64];
        return slab + (threadIdx.x >> 6) * (kLdsPartialRows * 64) + (threadIdx.x & 63);
    }
};

// LDSP: the partial sums of rows_per_wave <= kLdsPartialRows rows stay in LDS between chunk
// passes instead of passing through the output buffer.
template <int AB, int WB, int SEGS, int CWT, bool EMIT, bool GATHER = false, bool LDSP = false>
__global__ __launch_bounds__(256) void gemm_kernel(const BranchArgs g) {
    typedef typename std::conditional<EMIT, OutViewEmit, OutView>::type OV;
    static_assert(!(GATHER && LDSP), "not combined");
    int *const slab = PartialSlab<LDSP>::mine();
    const WavePos wp = wave_pos(g.div_tiles);
    // a wavefront past the last row block keeps an empty row range
    const bool active = (int64_t)wp.rb * g.rows_per_wave < g.rows;
    const int r0 = active ? wp.rb * g.rows_per_wave : 0;
    const int r1 = active ? min(g.rows, r0 + g.rows_per_wave) : 0;
    const int n = wp.ct * 64 + (int)(threadIdx.x & 63);
    const bool n_ok = n < g.N;
    const int nload = n_ok ? n : g.N - 1;
    const float sc = (g.scale != nullptr) ? g.scale[nload] : 1.0f;
    const OV ov = make_out_view<OV>(g, r0, r1, nload, sc, wp.ct);
    uniform_words As = as_uniform(g.A);
    constexpr int KC = SEGS * CWT;
    const int Kw = g.Cw;
    trace_begin(g, wp);
    if (Kw == 0) {  // K == 0: every product is the empty sum
        for (int r = r0; r < r1; ++r) finish_row<true>(ov, r - r0, 0, true, true);
        trace_end(g, wp);
        return;
    }
    RowWalk walk = RowWalk();
    if constexpr (GATHER) walk = row_walk_at(g, r0, (uint32_t)(AB * Kw) * 4u);
    for (int k0 = 0; k0 < Kw; k0 += KC) {
        const bool first = (k0 == 0);
        const bool last = (k0 + KC >= Kw);
        auto fetch = [&](int rel_row) -> int {
            if (first) return g.kconst;
            if constexpr (LDSP) return slab[rel_row * 64];
            else return __builtin_amdgcn_raw_buffer_load_b32(ov.d0, ov.col_bytes, (int)((uint32_t)rel_row * ov.row_bytes), 0);
        };
        auto sink = [&](int rel_row, int v, int prev) {
            if constexpr (LDSP) {
                if (!last) {
                    slab[rel_row * 64] = v + prev;
                    return;
                }
            }
            finish_row<false>(ov, rel_row, v + prev, /*first=*/true, last);   // the earlier part is already added
        };
        if (k0 + KC <= Kw) gemm_chunk_full<AB, WB, SEGS, CWT, GATHER>(g, nload, r0, r1, k0, fetch, sink, walk);
        else gemm_chunk_tail<AB, WB, SEGS, CWT, GATHER>(g, As, nload, r0, r1, k0, fetch, sink, walk);
    }
    trace_end(g, wp);
}

// ---------------------------------------------------------------------------------------
// GEMM with the K chunks split over the four wavefronts of a block (long K, few rows, e.g. a
// fully connected layer on a small batch).  All four wavefronts own the same 64 columns and
// the same block of rows; wavefront v takes chunks v, v+4, ...  A weight chunk is therefore
// loaded once per block and reused for every row of the block (four times the reuse of the
// kernel above at the same number of wavefronts), and partial sums never touch global memory:
// they are summed per wavefront in LDS and combined after one barrier.
// ---------------------------------------------------------------------------------------
constexpr int kSplitRowsMax = 32;

template <int AB, int WB, int SEGS, int CWT, bool EMIT>
__global__ __launch_bounds__(256) void gemm_splitk_kernel(const BranchArgs g) {
    typedef typename std::conditional<EMIT, OutViewEmit, OutView>::type OV;
    __shared__ int partial[4][kSplitRowsMax][64];
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    WavePos wp;
    wp.index = (int)blockIdx.x * 4 + wv;
    fast_divmod(blockIdx.x, g.div_tiles, wp.rb, wp.ct);
    const int r0 = wp.rb * g.rows_per_wave;                   // rows per BLOCK here (<= kSplitRowsMax)
    const int r1 = min(g.rows, r0 + g.rows_per_wave);
    const int n = wp.ct * 64 + lane;
    const int nload = (n < g.N) ? n : g.N - 1;
    const float sc = (g.scale != nullptr) ? g.scale[nload] : 1.0f;
    const OV ov = make_out_view<OV>(g, r0, r1, nload, sc, wp.ct);
    uniform_words As = as_uniform(g.A);
    constexpr int KC = SEGS * CWT;
    const int Kw = g.Cw;
    trace_begin(g, wp);
    bool mine = false;                                        // has this wavefront written its slab yet
    for (int k0 = wv * KC; k0 < Kw; k0 += 4 * KC) {
        const bool first = !mine;
        auto fetch = [&](int rel_row) -> int { return first ? 0 : partial[wv][rel_row][lane]; };
        auto sink = [&](int rel_row, int v, int prev) { partial[wv][rel_row][lane] = v + prev; };
        if (k0 + KC <= Kw) gemm_chunk_full<AB, WB, SEGS, CWT>(g, nload, r0, r1, k0, fetch, sink);
        else gemm_chunk_tail<AB, WB, SEGS, CWT>(g, As, nload, r0, r1, k0, fetch, sink);
        mine = true;
    }
    if (!mine)
        for (int r = 0; r < r1 - r0; ++r) partial[wv][r][lane] = 0;
    __syncthreads();
    for (int r = wv; r < r1 - r0; r += 4) {
        const int v = g.kconst + partial[0][r][lane] + partial[1][r][lane] + partial[2][r][lane] + partial[3][r][lane];
        finish_row<true>(ov, r, v, true, true);
    }
    trace_end(g, wp);
}

// ---------------------------------------------------------------------------------------
// 3x3 convolution, pad 1, stride S = 1 or 2 (both axes).  Rows are output pixels in NHWC order;
// the K axis of a pixel is the plane words of the nine input pixels around (S*oh, S*ow), never
// materialised.  Taps outside the
// image contribute nothing: they are skipped, and the constant term of a pixel uses its
// number of valid taps.
//
// Template shape:  CWS  words per (pixel, plane) if known at compile time, else 0;
//                  CWT  channel words per chunk;  TPC  taps per chunk (9, 3 or 1);
//                  GT   taps per pipeline stage (divides TPC, TPC/GT odd; GT == 3 only when
//                       CWT == CWS, so that the three taps of a kernel row are contiguous);
//                  P    output pixels per loop iteration (P > 1 only for single-chunk shapes
//                       with GT == 3: the P pixels share the P+2 input pixels of each kernel row,
//                       one scalar load and one wait per kernel row serve all of them).
// A chunk = TPC taps x CWT channel words; its weight words (TPC*WB*CWT) stay in VGPRs.
// ---------------------------------------------------------------------------------------
struct PixelPos {
    int n, oh, ow;        // image, output row, output column
};

__device__ __forceinline__ int tap_dh(int t) { return t / 3 - 1; }
__device__ __forceinline__ int tap_dw(int t) { return t % 3 - 1; }

// State of one chunk pass over a run of output pixels that lie in ONE image row.  For such a
// run the validity of a kernel row is constant, and only the run's first / last pixel can sit
// in the first / last image column, so the inner loop needs no position tracking:
//   stage_off[s]  byte offset of the first tap of stage s relative to the output pixel's own
//                 words; a tap whose image row does not exist points at the pixel's own row
//                 (in bounds) and is skipped when consumed;
//   stage_ok      bit s: the kernel row of stage s exists;
//   edge          bit 0: the first pixel of the current group is in column 0 (its taps with
//                 dw = -1 are skipped), bit 1: the last one is in column W-1 (dw = +1 skipped).
// Addresses are not tested: a +-1 column step from a pixel of an existing row stays inside
// [0, rows) except for the four pixels 0, W, rows-1-W and rows-1, which never come here.
template <int AB, int WB, int CWS, int CWT, int TPC, int GT, int P, int S = 1>
struct ConvCtx {
    static constexpr int NS = TPC / GT;
    static constexpr bool CONTIG = (CWS > 0 && CWT == CWS);   // a pixel's AB*CWT words are consecutive
    // CONTIG: one run of GT*AB*CWT words (consecutive pixels are consecutive too);
    // otherwise one run of CWT words per (tap, plane).
    static_assert(P == 1 || (GT == 3 && CONTIG), "pixel groups need contiguous kernel rows");
    // the P output pixels of a group are S input pixels apart: a kernel row spans GT + S*(P-1) input pixels
    typedef typename std::conditional<CONTIG, SStage<1, (GT + S * (P - 1)) * AB * CWT>, SStage<GT * AB, CWT>>::type Buf;
    uint64_t base;                   // byte address of the activation planes
    int Cw, c0, t0;                  // runtime words per plane, chunk's first channel word / tap
    uint32_t off_cur, off_nxt;       // byte offset of (pixel, plane 0, word c0) for this / the next pixel
    uint32_t stage_off[NS];
    uint32_t stage_ok;               // bit s: the kernel row of stage s exists
    uint32_t edge;                   // bit 0: column 0, bit 1: column W-1 (current group)
    uint32_t w[TPC][WB][CWT];
    int part[P][AB + WB - 1];
    Buf bufA, bufB;

    __device__ __forceinline__ int plane_stride() const { return CWS > 0 ? CWS : Cw; }
    __device__ __forceinline__ uint32_t pixel_bytes() const { return (uint32_t)(AB * plane_stride() * 4); }

    // Stages that are whole kernel rows are taken centre row first: the centre tap of the
    // centre row exists for every pixel, so it can initialise the accumulators (popc_set)
    // instead of a zeroing pass.
    static constexpr bool CENTER_FIRST = (TPC == 9 && GT == 3);
    static constexpr int first_tap(int st) {           // first tap (kh*3 + kw) of stage st, TPC == 9
        return CENTER_FIRST ? (st == 0 ? 3 : st == 1 ? 0 : 6) : st * GT;
    }

    // column offset of tap i of stage ST (compile-time unless a chunk is a single tap)
    template <int ST>
    __device__ __forceinline__ int dw_of(int i) const {
        return (TPC == 1) ? tap_dw(t0) : (ST * GT + i) % 3 - 1;
    }

    __device__ __forceinline__ void set_image_row(int oh, int H, int W) {
        stage_ok = 0u;
#pragma unroll
        for (int st = 0; st < NS; ++st) {
            const int dh = (TPC == 9) ? first_tap(st) / 3 - 1 : tap_dh(t0 + st * GT);
            const int dw = (TPC == 1) ? tap_dw(t0) : (st * GT) % 3 - 1;
            const bool ok = (unsigned)(S * oh + dh) < (unsigned)H;
            if (ok) stage_ok |= 1u << st;
            stage_off[st] = (uint32_t)((ok ? dh * W : 0) + dw) * pixel_bytes();
        }
        stage_ok = spin(stage_ok);
    }

    // Any odd KH x KW window with "same" padding and dilation D (shapes with one tap per stage): stage
    // st holds tap t0 + st of the KH*KW, decoded on the scalar unit.  A tap is used if it exists
    // (t < KH*KW), its image row exists, and its column exists for the run's first column ow (the caller
    // cuts the runs so that this holds for all of a run's pixels or for none).  A tap that is not used
    // points at the pixel itself, so every address of the run is inside the image.
    // Returns the number of taps used.
    __device__ __forceinline__ int set_window_taps(int oh, int ow, int H, int W, int KH, int KW, int D) {
        stage_ok = 0u;
        int used = 0;
        const int T = KH * KW;
        const int recip = (65536 + KW - 1) / KW;            // t / KW == (t * recip) >> 16 for the few taps there are
#pragma unroll
        for (int st = 0; st < NS; ++st) {
            const int t = t0 + st;
            const int kh = (t * recip) >> 16, kw = t - kh * KW;
            const int dh = (kh - (KH >> 1)) * D, dw = (kw - (KW >> 1)) * D;
            const bool ok = t < T && (unsigned)(oh + dh) < (unsigned)H && (unsigned)(ow + dw) < (unsigned)W;
            if (ok) { stage_ok |= 1u << st; ++used; }
            stage_off[st] = ok ? (uint32_t)(dh * W + dw) * pixel_bytes() : 0u;
        }
        stage_ok = spin(stage_ok);
        return used;
    }

    template <int ST>
    __device__ __forceinline__ void request(Buf &b, bool next_row) {
        const uint32_t off = (next_row ? off_nxt : off_cur) + stage_off[ST];
        if constexpr (CONTIG) {
            b.run[0].template request<0>(base, off);
        } else {
            const uint32_t psb = (uint32_t)plane_stride() * 4u;
#pragma unroll
            for (int i = 0; i < GT * AB; ++i) b.run[i].template request<0>(base, off + (uint32_t)i * psb);
        }
    }
    __device__ __forceinline__ uint32_t word(const Buf &b, int i, int p, int j) const {
        if constexpr (CONTIG) return b.run[0].get((i * AB + p) * CWT + j);
        else return b.run[i * AB + p].get(j);
    }
    // all branches of tap i of stage ST for output pixel x of the group; SET: first contribution
    template <int ST, bool SET>
    __device__ __forceinline__ void tap(const Buf &b, int x, int i) {
        const int t = (TPC == 9) ? first_tap(ST) + i : ST * GT + i;      // index into w[]
#pragma unroll
        for (int q = 0; q < WB; ++q)
#pragma unroll
            for (int p = 0; p < AB; ++p)
#pragma unroll
                for (int j = 0; j < CWT; ++j) {
                    const uint32_t v = word(b, x * S + i, p, j) ^ w[t][q][j];
                    // accumulator p+q is first reached at j == 0 with the smallest q that pairs with it
                    const bool first_hit = SET && j == 0 && q == ((p + q) < AB ? 0 : (p + q) - (AB - 1));
                    if (first_hit) popc_set(part[x][p + q], v);
                    else popc_acc(part[x][p + q], v);
                }
    }
    template <int ST>
    __device__ __forceinline__ void consume(const Buf &b) {
        if constexpr (CENTER_FIRST && ST == 0) {
            // centre kernel row: always exists; its centre tap goes first and sets the accumulators
#pragma unroll
            for (int x = 0; x < P; ++x) {
                tap<ST, true>(b, x, 1);
                if (!(x == 0 && sflag(edge, 1u))) tap<ST, false>(b, x, 0);
                if (!(x == P - 1 && sflag(edge, 2u))) tap<ST, false>(b, x, 2);
            }
        } else if (sflag(stage_ok, 1u << ST)) {
#pragma unroll
            for (int x = 0; x < P; ++x)               // output pixel of the group
#pragma unroll
                for (int i = 0; i < GT; ++i) {
                    const int dw = dw_of<ST>(i);
                    // skip the tap that hangs over the left / right image border
                    const bool skip = (x == 0 && dw < 0 && sflag(edge, 1u)) || (x == P - 1 && dw > 0 && sflag(edge, 2u));
                    if (!skip) tap<ST, false>(b, x, i);
                }
        }
    }
};

__device__ __forceinline__ PixelPos next_pixel(PixelPos p, int Ho, int Wo) {
    if (++p.ow == Wo) {
        p.ow = 0;
        if (++p.oh == Ho) { p.oh = 0; ++p.n; }
    }
    return p;
}

__device__ __forceinline__ PixelPos pixel_pos(int r, const BranchArgs &g) {     // divisors: the OUTPUT image size
    PixelPos p;
    int line;
    fast_divmod((uint32_t)r, g.div_w, line, p.ow);
    fast_divmod((uint32_t)line, g.div_h, p.n, p.oh);
    return p;
}

// number of taps of the 3x3 window of an output pixel that fall inside the image
template <int S>
__device__ __forceinline__ int valid_taps(PixelPos p, int H, int W) {
    const int nh = 3 - (S * p.oh == 0 ? 1 : 0) - (S * p.oh + 1 >= H ? 1 : 0);
    const int nw = 3 - (S * p.ow == 0 ? 1 : 0) - (S * p.ow + 1 >= W ? 1 : 0);
    return nh * nw;
}

// Pipelined pixels ra .. rb-1 of one chunk, all in image row oh, rb - ra >= P.  left_first = 1:
// pixel ra is in column 0; right_last = 2: pixel rb-1 is in column W-1 (else 0; flag words, made
// where the comparison is, see sflag()).  Pixels are taken in
// groups of P; if P does not divide the run, the last group is placed at rb-P and recomputes
// pixels of the group before it (P > 1 is used for single-chunk shapes only, where a
// recomputed pixel is simply stored again with the same value).
// in_a: number of the input pixel under output pixel ra, (n*H + S*oh)*W + S*ow.
// WIDE: another window than the plain 3x3 (see set_window_taps); wide_ow: the first column of the run,
// whose pixels all have the same taps.
template <bool WIDE = false, int AB, int WB, int CWS, int CWT, int TPC, int GT, int P, int S, class OV>
__device__ __forceinline__ void conv_run_pipelined(ConvCtx<AB, WB, CWS, CWT, TPC, GT, P, S> &c,
                                                   const BranchArgs &g, const OV &ov, int r0, int ra,
                                                   int rb, int oh, int in_a, uint32_t left_first, uint32_t right_last,
                                                   bool first, bool last, int wide_ow = -1) {
    constexpr bool SINGLE_SHAPE = (TPC == 9 && CWS > 0 && CWT == CWS);
    static_assert(P == 1 || SINGLE_SHAPE, "pixel groups only where a chunk pass is the whole product");
    // a window of more than TPC taps is taken in several tap chunks even where the chunk is the whole plane
    const bool single = SINGLE_SHAPE && !(WIDE && g.geo.KH * g.geo.KW > TPC);
    int krow = 0, wide_add = 0;                      // constant term: per valid column / for the whole pixel
    if constexpr (WIDE) {
        // the constant of a tap covers all its channels: counted with the first channel chunk, for the
        // taps of this tap chunk
        const int used = c.set_window_taps(oh, wide_ow, g.H, g.W, g.geo.KH, g.geo.KW, g.geo.dh);
        wide_add = (c.c0 == 0) ? used * g.kconst : 0;
    } else {
        c.set_image_row(oh, g.H, g.W);
        krow = (3 - (S * oh == 0 ? 1 : 0) - (S * oh + 1 >= g.H ? 1 : 0)) * g.kconst;   // per valid column
    }
    const uint32_t pb = c.pixel_bytes();
    const uint32_t edge_first = left_first, edge_last = right_last;
    const uint32_t off_a = (uint32_t)in_a * pb + (uint32_t)c.c0 * 4u;
    const int r_last = rb - P;                       // start of the last group
    c.off_cur = off_a;
    c.off_nxt = off_a;
    c.template request<0>(c.bufA, false);
    int r = ra;
    auto one_group = [&](auto flip_tag) {
        constexpr bool FLIP = decltype(flip_tag)::value;
        if constexpr (!ConvCtx<AB, WB, CWS, CWT, TPC, GT, P, S>::CENTER_FIRST) {
#pragma unroll
            for (int x = 0; x < P; ++x)
#pragma unroll
                for (int s = 0; s < AB + WB - 1; ++s) c.part[x][s] = 0;
        }
        // the group after this one (the last group prefetches itself, unused)
        const int rn = (r < r_last) ? min(r + P, r_last) : r;
        c.off_nxt = off_a + (uint32_t)((rn - ra) * S) * pb;
        // integer selects only: keeps the edge bookkeeping on the scalar unit
        uint32_t edge = 0u;
        if (r == ra) edge |= edge_first;
        if (r == r_last) edge |= edge_last;
        c.edge = edge = spin(edge);
        // what earlier chunk passes left for this pixel, asked for before its products are formed
        int prev = 0;
        if (!single) {
            if (!first) prev = partial_load(ov, r - r0);
        }
        run_stages<0, FLIP>(c);
#pragma unroll
        for (int x = 0; x < P; ++x) {
            int val = -2 * weighted_sum(c.part[x]) + prev;
            int ncols = 3;
            if (x == 0) ncols -= (int)(edge & 1u);
            if (x == P - 1) ncols -= (int)(edge >> 1);
            if constexpr (WIDE) {
                if (adds_const(ov)) val += wide_add;
                if (single) finish_row<true>(ov, r - r0 + x, val, true, true);
                else finish_row<false>(ov, r - r0 + x, val, /*first=*/true, last);
            } else {
                if (first && adds_const(ov)) val += ncols * krow;
                finish_row<SINGLE_SHAPE>(ov, r - r0 + x, val, /*first=*/true, last);   // earlier part already added
            }
        }
        c.off_cur = c.off_nxt;
        r = rn;
    };
    // groups in pairs (the two buffers swap roles from one group to the next), then a last one
    const int ngroups = (rb - ra + P - 1) / P;
    int done = 0;
    while (done + 1 < ngroups) {
        one_group(std::integral_constant<bool, false>());
        one_group(std::integral_constant<bool, true>());
        done += 2;
    }
    if (done < ngroups) one_group(std::integral_constant<bool, false>());
    // Drain the prefetch issued by the last group.  Both buffers are named so that their
    // registers stay reserved until the wait, whichever of them the prefetch went to.
    c.bufA.template arrive<true>();
    c.bufB.template arrive<false>();
}

// One pixel of one chunk with every tap and address tested (the four end pixels).
template <int AB, int WB, int CWS, int CWT, int TPC, int GT, int P, int S, class OV>
__device__ __forceinline__ void conv_row_checked(ConvCtx<AB, WB, CWS, CWT, TPC, GT, P, S> &c, uniform_words As,
                                                 const BranchArgs &g, const OV &ov, int r0, int r,
                                                 PixelPos pos, bool first, bool last) {
#pragma unroll
    for (int s = 0; s < AB + WB - 1; ++s) c.part[0][s] = 0;
#pragma unroll
    for (int t = 0; t < TPC; ++t) {
        const int dh = (TPC == 9) ? t / 3 - 1 : tap_dh(c.t0 + t);
        const int dw = (TPC == 1) ? tap_dw(c.t0) : t % 3 - 1;
        const int ih = S * pos.oh + dh, iw = S * pos.ow + dw;
        const bool ok = (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W;
        if (ok) {
            const int pix = (pos.n * g.H + ih) * g.W + iw;
            uint32_t a[AB][CWT];
#pragma unroll
            for (int p = 0; p < AB; ++p)
#pragma unroll
                for (int j = 0; j < CWT; ++j) a[p][j] = As[(pix * AB + p) * c.plane_stride() + c.c0 + j];
#pragma unroll
            for (int q = 0; q < WB; ++q)
#pragma unroll
                for (int p = 0; p < AB; ++p)
#pragma unroll
                    for (int j = 0; j < CWT; ++j) popc_acc(c.part[0][p + q], a[p][j] ^ c.w[t][q][j]);
        }
    }
    int val = -2 * weighted_sum(c.part[0]);
    if (first && adds_const(ov)) val += valid_taps<S>(pos, g.H, g.W) * g.kconst;
    finish_row<(TPC == 9 && CWS > 0 && CWT == CWS)>(ov, r - r0, val, first, last);
}

// full chunk: every word c0 .. c0+CWT-1 exists.  The wavefront's pixel range is cut into
// runs inside one image row; the four pixels whose untested neighbour addresses could leave
// the buffer (0, W, rows-1-W, rows-1) go through the tested path.
template <int AB, int WB, int CWS, int CWT, int TPC, int GT, int P, int S, bool WIDE = false, class OV>
__device__ __forceinline__ void conv_chunk_full(const BranchArgs &g, const OV &ov, uniform_words As,
                                                int nload, int r0, int r1, int c0, int t0, bool first,
                                                bool last) {
    static_assert(!WIDE || (GT == 1 && S == 1 && P == 1), "other windows: one tap per stage, stride 1");
    static_assert(TPC % GT == 0 && ((TPC / GT) & 1) == 1, "odd number of stages per pixel");
    ConvCtx<AB, WB, CWS, CWT, TPC, GT, P, S> c;
    c.base = (uint64_t)g.A; c.Cw = g.Cw; c.c0 = c0; c.t0 = t0;
    const int ps = c.plane_stride();
    {
        constexpr int NW = TPC * WB * CWT;            // word k = (t * WB + q) * CWT + j
        uint32_t wl[NW];
        if constexpr (WIDE) {
            // a window of T taps: the last tap chunk may run past them; such a slot repeats tap T-1 and is never used
            const int T = g.geo.KH * g.geo.KW;
#pragma unroll
            for (int k = 0; k < TPC * WB; ++k) {
                const int t = min(t0 + k / WB, T - 1);
                load_run<CWT>(g.Wt + ((nload * T + t) * WB + k % WB) * ps + c0, wl + k * CWT);
            }
        } else if constexpr (CWS > 0 && CWT == CWS) {        // the chunk takes every channel word: one contiguous run
            load_run<NW>(g.Wt + (nload * 9 + t0) * WB * CWS, wl);
        } else {
#pragma unroll
            for (int k = 0; k < TPC * WB; ++k) load_run<CWT>(g.Wt + ((nload * 9 + t0) * WB + k) * ps + c0, wl + k * CWT);
        }
#pragma unroll
        for (int t = 0; t < TPC; ++t)
#pragma unroll
            for (int q = 0; q < WB; ++q)
#pragma unroll
                for (int j = 0; j < CWT; ++j) c.w[t][q][j] = wl[(t * WB + q) * CWT + j];
    }
    // Output pixels whose untested window addresses could leave the plane buffer go through the
    // tested path.  Below 0: the window of the very first input pixel, read by output pixel 0 (and,
    // at stride 1, by pixel Wo from its upper kernel row).  Past the end: a window that sits on the
    // last input row of the last image and whose right column is W, which happens for the last
    // output column when (W - 1) is a multiple of the stride, in the output rows with
    // |S*oh - (H - 1)| <= 1 (the last one or two).
    const int Ho = g.geo.Ho, Wo = g.geo.Wo;
    if constexpr (WIDE) {
        // The first and last (KW/2)*D pixels of an image row miss taps.  Which ones depends on the column
        // only through floor(ow / D) on the left and floor((W-1-ow) / D) on the right (both saturating at
        // KW/2), so a row is cut where one of the two changes -- at the multiples of D up to (KW/2)*D and at
        // W - k*D, k = KW/2 .. 1 -- and every piece is a run with one set of taps, given by its first column.
        // No address of such a run leaves the image, so there are no end pixels to test.
        const int D = g.geo.dh, half_taps = g.geo.KW >> 1;
        PixelPos pos = pixel_pos(r0, g);
        int r = r0;
        while (r < r1) {
            const int row_end = r - pos.ow + Wo;
            int cut = Wo;
            for (int k = 1; k <= half_taps; ++k)
                if (pos.ow < k * D) { cut = k * D; break; }
            for (int k = half_taps; k >= 1; --k)
                if (g.W - k * D > pos.ow) { cut = min(cut, g.W - k * D); break; }
            const int stop = min(min(r1, row_end), r - pos.ow + cut);
            const int wide_ow = pos.ow;
            conv_run_pipelined<true>(c, g, ov, r0, r, stop, pos.oh, (pos.n * g.H + pos.oh) * g.W + pos.ow, spin(0u), spin(0u),
                                     first, last, wide_ow);
            pos.ow += stop - r;
            r = stop;
            if (pos.ow == Wo) {
                pos.ow = 0;
                if (++pos.oh == Ho) { pos.oh = 0; ++pos.n; }
            }
        }
        return;
    }
    int special[4] = {0, (S == 1) ? Wo : -1, -1, -1};
    if ((g.W - 1) % S == 0) {
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int oh = Ho - 1 - k;
            if (oh >= 0 && S * oh + 1 >= g.H - 1) special[2 + k] = g.rows - 1 - k * Wo;    // S*oh <= H-1 always
        }
    }
    // the right-hand tap of the last output column is outside the image exactly in that case
    const bool right_edge = ((g.W - 1) % S == 0);
    PixelPos pos = pixel_pos(r0, g);
    int r = r0;
    while (r < r1) {
        const int row_end = r - pos.ow + Wo;             // first pixel of the next output row
        int stop = min(r1, row_end);
        bool is_special = false;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (special[i] == r) is_special = true;
            if (special[i] > r && special[i] < stop) stop = special[i];
        }
        if (is_special || stop - r < P) {              // end pixels, and runs shorter than a group
            conv_row_checked(c, As, g, ov, r0, r, pos, first, last);
            stop = r + 1;
        } else {
            conv_run_pipelined(c, g, ov, r0, r, stop, pos.oh, (pos.n * g.H + S * pos.oh) * g.W + S * pos.ow,
                               spin(pos.ow == 0 ? 1u : 0u), spin((stop == row_end && right_edge) ? 2u : 0u), first,
                               last);
        }
        pos.ow += stop - r;
        r = stop;
        if (pos.ow == Wo) {
            pos.ow = 0;
            if (++pos.oh == Ho) { pos.oh = 0; ++pos.n; }
        }
    }
}

// tail chunk (channel words past Cw are padding): plain loads with a guard per word
template <int AB, int WB, int CWT, class OV>
__device__ __forceinline__ void conv_chunk_tail(const BranchArgs &g, const OV &ov, uniform_words As,
                                                int nload, int r0, int r1, int c0, bool first, bool last) {
    const int Cw = g.Cw;
    uint32_t w[9][WB][CWT];
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int q = 0; q < WB; ++q)
#pragma unroll
            for (int j = 0; j < CWT; ++j)
                w[t][q][j] = (c0 + j < Cw) ? g.Wt[((nload * 9 + t) * WB + q) * Cw + c0 + j] : 0u;
    PixelPos pos = pixel_pos(r0, g);
    for (int r = r0; r < r1; ++r) {
        int part[AB + WB - 1];
#pragma unroll
        for (int s = 0; s < AB + WB - 1; ++s) part[s] = 0;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const int dh = t / 3 - 1, dw = t % 3 - 1;
            const bool ok = (unsigned)(pos.oh + dh) < (unsigned)g.H && (unsigned)(pos.ow + dw) < (unsigned)g.W;
            if (ok) {
                const int pix = r + dh * g.W + dw;                         // stride 1: output pixel r sits on input pixel r
                uint32_t a[AB][CWT];
#pragma unroll
                for (int p = 0; p < AB; ++p)
#pragma unroll
                    for (int j = 0; j < CWT; ++j)
                        a[p][j] = (c0 + j < Cw) ? As[(pix * AB + p) * Cw + c0 + j] : 0u;
#pragma unroll
                for (int q = 0; q < WB; ++q)
#pragma unroll
                    for (int p = 0; p < AB; ++p)
#pragma unroll
                        for (int j = 0; j < CWT; ++j) popc_acc(part[p + q], a[p][j] ^ w[t][q][j]);
            }
        }
        int val = -2 * weighted_sum(part);
        if (first) val += valid_taps<1>(pos, g.H, g.W) * g.kconst;
        finish_row<false>(ov, r - r0, val, first, last);
        pos = next_pixel(pos, g.H, g.W);
    }
}

// XR: the blocks are numbered so that each XCD takes one contiguous range of them (xcd_block();
// a compile-time choice: even a wave-uniform test of it at the start of every wavefront showed
// in the time of the ResNet-18-shaped layer).
// S: stride (1, or 2 for the fixed-shape instantiations; the tail paths are stride 1 only).
//
// SPLIT (layers with few output pixels and many input channels, e.g. 7x7 or 14x14 images with 512
// channels): a launch with one wavefront per (pixel run, 64 filters) would leave one or two
// wavefronts per SIMD, each making several chunk passes with nothing to hide its loads behind, and
// a quarter of the SIMDs one wavefront short of the others.  Instead the four wavefronts of a block
// share pixel run and filters and split the channel chunks (wavefront v takes chunks v, v+4, ...);
// their partial sums meet in LDS (no trip through the output buffer), and after one barrier each
// wavefront finishes every fourth row.  Four times the wavefronts, each with a single weight load.
constexpr int kSplitRows = kConvSplitRows;       // most rows per block in the SPLIT variant

// WIDE: another window than the plain 3x3 (any odd KH x KW with "same" padding at equal dilation,
// stride 1), a kernel of its own so that the 3x3 kernels carry none of its code; only for shapes
// with one tap per pipeline stage and a stage of at most 16 scalar registers.
template <int AB, int WB, int CWS, int CWT, int TPC, int GT, int P, bool EMIT, bool XR = false, int S = 1,
          bool SPLIT = false, bool WIDE = false>
__global__ __launch_bounds__(256) void conv_kernel(const BranchArgs g) {
    static_assert(S == 1 || CWS > 0, "strided: compile-time plane strides only");
    static_assert(!WIDE || (CWS > 0 && GT == 1 && S == 1 && P == 1 && !XR && conv_wide_stage_ok(AB, CWT)),
                  "other windows: one tap per stage, at most 16 scalar registers per stage");
    if constexpr (SPLIT) {
        static_assert(TPC == 9 && CWS > 0 && CWS / CWT >= 2 && !XR, "all taps per chunk, several channel chunks");
        typedef typename std::conditional<EMIT, OutViewEmit, OutView>::type OV;
        __shared__ int slab[4 * kSplitRows * 64];
        const int v = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
        const int lane = (int)(threadIdx.x & 63);
        int rb, ct;
        fast_divmod(blockIdx.x, g.div_tiles, rb, ct);
        const int r0 = rb * g.rows_per_wave;                      // rows per BLOCK here (<= kSplitRows)
        const int r1 = min(g.rows, r0 + g.rows_per_wave);
        const int n = ct * 64 + lane;
        const int nload = (n < g.N) ? n : g.N - 1;
        uniform_words As = as_uniform(g.A);
        const OutViewSlab sv = {slab + v * (kSplitRows * 64) + lane, v == 0};
        bool mine = false;
        if constexpr (WIDE) {      // another window: its taps nine at a time
            const int tap_chunks = (g.geo.KH * g.geo.KW + 8) / 9;
            for (int c0 = v * CWT; c0 < CWS; c0 += 4 * CWT)
                for (int tc = 0; tc < tap_chunks; ++tc) {
                    conv_chunk_full<AB, WB, CWS, CWT, TPC, GT, P, S, true>(g, sv, As, nload, r0, r1, c0, tc * 9, /*first=*/!mine, /*last=*/false);
                    mine = true;
                }
        } else {
            for (int c0 = v * CWT; c0 < CWS; c0 += 4 * CWT) {
                conv_chunk_full<AB, WB, CWS, CWT, TPC, GT, P, S>(g, sv, As, nload, r0, r1, c0, 0, /*first=*/!mine, /*last=*/false);
                mine = true;
            }
        }
        if (!mine)
            for (int r = 0; r < r1 - r0; ++r) sv.slab[r * 64] = 0;
        __syncthreads();
        // The output view is built only now: made opaque here, its inputs cannot be computed (and kept
        // in registers the chunk passes need) before the barrier.
        int r0_late = r0, ct_late = ct, nload_late = nload;
        asm volatile("" : "+s"(r0_late), "+s"(ct_late), "+v"(nload_late));
        const float sc = (g.scale != nullptr) ? g.scale[nload_late] : 1.0f;
        const OV ov = make_out_view<OV>(g, r0_late, r1, nload_late, sc, ct_late);
        for (int r = v; r < r1 - r0; r += 4) {
            const int *row = slab + r * 64 + lane;
            const int val = row[0] + row[kSplitRows * 64] + row[2 * kSplitRows * 64] + row[3 * kSplitRows * 64];
            finish_row<true>(ov, r, val, true, true);
        }
        return;
    }
    typedef typename std::conditional<EMIT, OutViewEmit, OutView>::type OV;
    const WavePos wp = wave_pos<XR>(g.div_tiles, 1, g.grid_blocks);
    // a wavefront past the last row block keeps an empty row range
    const bool active = (int64_t)wp.rb * g.rows_per_wave < g.rows;
    const int r0 = active ? wp.rb * g.rows_per_wave : 0;
    const int r1 = active ? min(g.rows, r0 + g.rows_per_wave) : 0;
    const int n = wp.ct * 64 + (int)(threadIdx.x & 63);
    const bool n_ok = n < g.N;
    const int nload = n_ok ? n : g.N - 1;
    const float sc = (g.scale != nullptr) ? g.scale[nload] : 1.0f;
    const OV ov = make_out_view<OV>(g, r0, r1, nload, sc, wp.ct);
    uniform_words As = as_uniform(g.A);
    const int Cw = (CWS > 0) ? CWS : g.Cw;
    trace_begin(g, wp);
    if (Cw == 0) {  // no input channels: every product is the empty sum
        for (int r = r0; r < r1; ++r) finish_row<true>(ov, r - r0, 0, true, true);
        trace_end(g, wp);
        return;
    }
    constexpr int TAP_CHUNKS = 9 / TPC;
    // Very wide activations leave too few SGPRs for the two hand-managed stage buffers next to
    // the runtime-stride address arithmetic; those (rare) shapes use compiler-managed loads.
    constexpr bool PIPELINED = (CWS > 0) || (AB <= 4);
    if constexpr (WIDE) {          // another window than the plain 3x3: its taps TPC at a time
        const int tap_chunks = (g.geo.KH * g.geo.KW + TPC - 1) / TPC;
        for (int c0 = 0; c0 < Cw; c0 += CWT)
            for (int tc = 0; tc < tap_chunks; ++tc)
                conv_chunk_full<AB, WB, CWS, CWT, TPC, GT, P, S, true>(g, ov, As, nload, r0, r1, c0, tc * TPC,
                                                                        c0 == 0 && tc == 0,
                                                                        c0 + CWT >= Cw && tc == tap_chunks - 1);
        trace_end(g, wp);
        return;
    }
    for (int c0 = 0; c0 < Cw; c0 += CWT) {
        const bool full = (c0 + CWT <= Cw);
        if constexpr (!PIPELINED) {
            conv_chunk_tail<AB, WB, CWT>(g, ov, As, nload, r0, r1, c0, c0 == 0, c0 + CWT >= Cw);
        } else if (full) {
            for (int tc = 0; tc < TAP_CHUNKS; ++tc) {
                const bool first = (c0 == 0) && (tc == 0);
                const bool last = (c0 + CWT >= Cw) && (tc == TAP_CHUNKS - 1);
                conv_chunk_full<AB, WB, CWS, CWT, TPC, GT, P, S>(g, ov, As, nload, r0, r1, c0, tc * TPC, first, last);
            }
        } else if constexpr (CWS == 0 && CWT > 1) {
            conv_chunk_tail<AB, WB, CWT>(g, ov, As, nload, r0, r1, c0, c0 == 0, true);
        }
    }
    trace_end(g, wp);
}

// ---------------------------------------------------------------------------------------
// Chunk shapes.
// ---------------------------------------------------------------------------------------
constexpr int pow2_floor(int x) { return x >= 16 ? 16 : x >= 8 ? 8 : x >= 4 ? 4 : x >= 2 ? 2 : 1; }
constexpr int imin(int a, int b) { return a < b ? a : b; }

// GEMM: one stage holds AB*CWT activation words in SGPRs (<= 16, twice for the two buffers);
// one chunk holds WB*KC weight words in VGPRs.
template <int AB, int WB> struct GemmShape {
    static constexpr int KC = (WB == 1) ? 64 : (WB == 2) ? 32 : (WB <= 4) ? 16 : 8;
    static constexpr int CWT = imin(pow2_floor(16 / AB), KC / 2);   // at least two stages per row
    static constexpr int SEGS = KC / CWT;
};

// Convolution with a compile-time plane stride CWS: the chunk shape is conv_shape() of
// qnn_internal.h (shared with the host, which sizes the launch from the number of passes).
template <int AB, int WB, int CWS> struct ConvShape {
    static constexpr ConvShapeV v = conv_shape(AB, WB, CWS);
    static constexpr int CWT = v.cwt, TPC = v.tpc, GT = v.gt, P = v.p;
};

inline dim3 grid_for(const BranchArgs &g) {
    const int64_t row_blocks = ((int64_t)g.rows + g.rows_per_wave - 1) / g.rows_per_wave;
    const int64_t waves = row_blocks * g.col_tiles;
    return dim3((unsigned)((waves + 3) / 4));
}

// GEMM kernel with a chunk of KC words (two or more pipeline stages of CWT words)
template <int AB, int WB, int SEGS, int CWT>
void launch_gemm_plain(const BranchArgs &g, bool emit, hipStream_t s) {
    if constexpr (AB <= 4 && WB <= 4) {       // strided rows: bit widths up to 4 only, to bound build time
        if (g.gather_rows) {
            if (emit) launch_kernel((gemm_kernel<AB, WB, SEGS, CWT, true, true>), grid_for(g), dim3(256), 0, s, g);
            else launch_kernel((gemm_kernel<AB, WB, SEGS, CWT, false, true>), grid_for(g), dim3(256), 0, s, g);
            return;
        }
    }
    if constexpr (AB <= 4 && WB <= 4) {
        if (g.lds_partials) {
            if (emit) launch_kernel((gemm_kernel<AB, WB, SEGS, CWT, true, false, true>), grid_for(g), dim3(256), 0, s, g);
            else launch_kernel((gemm_kernel<AB, WB, SEGS, CWT, false, false, true>), grid_for(g), dim3(256), 0, s, g);
            return;
        }
    }
    if (emit) launch_kernel((gemm_kernel<AB, WB, SEGS, CWT, true>), grid_for(g), dim3(256), 0, s, g);
    else launch_kernel((gemm_kernel<AB, WB, SEGS, CWT, false>), grid_for(g), dim3(256), 0, s, g);
}

template <int AB, int WB, int KC>
void launch_gemm_short(const BranchArgs &g, bool emit, hipStream_t s) {
    // one stage per row where the row's words fit a stage (16 SGPRs): a stage of 2*AB*WB*KC vector
    // instructions covers a scalar load better than two of half the length
    constexpr int CWT = imin(pow2_floor(16 / AB), KC);
    constexpr int SEGS = KC / CWT;
    launch_gemm_plain<AB, WB, SEGS, CWT>(g, emit, s);
}

template <int AB, int WB>
hipError_t launch_gemm_t(const BranchArgs &g, hipStream_t s) {
    using S = GemmShape<AB, WB>;
    const bool emit = g.planes_out != nullptr;
    if (g.gather_rows && (AB > 4 || WB > 4 || g.split_k)) return hipErrorInvalidValue;   // host bug
    if (g.lds_partials && (AB > 4 || WB > 4 || g.split_k || g.gather_rows || g.rows_per_wave > kLdsPartialRows))
        return hipErrorInvalidValue;                                                       // host bug
    if (g.split_k) {
        const int64_t row_blocks = ((int64_t)g.rows + g.rows_per_wave - 1) / g.rows_per_wave;
        const dim3 grid((unsigned)(row_blocks * g.col_tiles));
        if (emit) launch_kernel((gemm_splitk_kernel<AB, WB, S::SEGS, S::CWT, true>), grid, dim3(256), 0, s, g);
        else launch_kernel((gemm_splitk_kernel<AB, WB, S::SEGS, S::CWT, false>), grid, dim3(256), 0, s, g);
    } else {
        // A product shorter than the regular chunk (1x1 convolutions, narrow layers) would run
        // entirely through the guarded tail path: take the largest shorter chunk that fits instead
        // (bit widths up to 4 only, to bound build time).
        if constexpr (AB <= 4 && WB <= 4) {
            if (g.Cw < S::KC && g.Cw >= 2) {
                if (S::KC > 16 && g.Cw >= 16) launch_gemm_short<AB, WB, 16>(g, emit, s);
                else if (S::KC > 8 && g.Cw >= 8) launch_gemm_short<AB, WB, 8>(g, emit, s);
                else if (g.Cw >= 4) launch_gemm_short<AB, WB, 4>(g, emit, s);
                else launch_gemm_short<AB, WB, 2>(g, emit, s);
                return launch_status();
            }
        }
        launch_gemm_plain<AB, WB, S::SEGS, S::CWT>(g, emit, s);
    }
    return launch_status();
}



template <int AB, int WB, int CWS>
hipError_t launch_conv_fixed(const BranchArgs &g, hipStream_t s) {
    using S = ConvShape<AB, WB, CWS>;
    const bool other_window = g.geo.KH != 3 || g.geo.KW != 3 || g.geo.dh != 1;
    if constexpr (conv_can_split(AB, WB, CWS)) {
        if (g.split_k) {           // the block's wavefronts split the channel chunks
            constexpr int SC = conv_split_shape(AB, WB, CWS).cwt;
            const int64_t row_blocks = ((int64_t)g.rows + g.rows_per_wave - 1) / g.rows_per_wave;
            const dim3 grid((unsigned)(row_blocks * g.col_tiles));
            if (g.rows_per_wave > kSplitRows) return hipErrorInvalidValue;                 // host bug
            const bool emit = g.planes_out != nullptr;
            if (other_window) {
                if constexpr (conv_wide_split_ok(AB, WB, CWS)) {
                    if (g.geo.sh != 1) return hipErrorInvalidValue;                        // host bug
                    if (emit) launch_kernel((conv_kernel<AB, WB, CWS, SC, 9, 1, 1, true, false, 1, true, true>), grid, dim3(256), 0, s, g);
                    else launch_kernel((conv_kernel<AB, WB, CWS, SC, 9, 1, 1, false, false, 1, true, true>), grid, dim3(256), 0, s, g);
                    return launch_status();
                }
                return hipErrorInvalidValue;                                               // host bug
            }
            if (g.geo.sh == 2) {
                if (emit) launch_kernel((conv_kernel<AB, WB, CWS, SC, 9, 1, 1, true, false, 2, true>), grid, dim3(256), 0, s, g);
                else launch_kernel((conv_kernel<AB, WB, CWS, SC, 9, 1, 1, false, false, 2, true>), grid, dim3(256), 0, s, g);
            } else {
                if (emit) launch_kernel((conv_kernel<AB, WB, CWS, SC, 9, 1, 1, true, false, 1, true>), grid, dim3(256), 0, s, g);
                else launch_kernel((conv_kernel<AB, WB, CWS, SC, 9, 1, 1, false, false, 1, true>), grid, dim3(256), 0, s, g);
            }
            return launch_status();
        }
    }
    if (g.split_k) return hipErrorInvalidValue;                                            // host bug
    if (other_window) {            // the kernels of their own for other windows
        if (g.geo.sh != 1 || g.xcd_ranges) return hipErrorInvalidValue;                    // host bug
        if constexpr (conv_wide_plain_ok(AB, WB, CWS)) {
            if (g.planes_out != nullptr)
                launch_kernel((conv_kernel<AB, WB, CWS, S::CWT, S::TPC, 1, 1, true, false, 1, false, true>), grid_for(g), dim3(256), 0, s, g);
            else
                launch_kernel((conv_kernel<AB, WB, CWS, S::CWT, S::TPC, 1, 1, false, false, 1, false, true>), grid_for(g), dim3(256), 0, s, g);
            return launch_status();
        } else if constexpr (conv_wide_extra_ok(AB, WB, CWS)) {   // an instantiation with one tap per stage
            constexpr int EC = conv_wide_extra_shape(AB, WB, CWS).cwt;
            if (g.planes_out != nullptr)
                launch_kernel((conv_kernel<AB, WB, CWS, EC, 9, 1, 1, true, false, 1, false, true>), grid_for(g), dim3(256), 0, s, g);
            else
                launch_kernel((conv_kernel<AB, WB, CWS, EC, 9, 1, 1, false, false, 1, false, true>), grid_for(g), dim3(256), 0, s, g);
            return launch_status();
        }
        return hipErrorInvalidValue;                                                       // host bug
    }
    if (g.geo.sh == 2) {           // stride 2: pixel groups of two only where five input pixels fit a stage
        constexpr int P2 = conv_group_strided(AB, WB, CWS);
        if (g.planes_out != nullptr)
            launch_kernel((conv_kernel<AB, WB, CWS, S::CWT, S::TPC, S::GT, P2, true, false, 2>), grid_for(g), dim3(256), 0, s, g);
        else
            launch_kernel((conv_kernel<AB, WB, CWS, S::CWT, S::TPC, S::GT, P2, false, false, 2>), grid_for(g), dim3(256), 0, s, g);
        return launch_status();
    }
    if constexpr (CWS >= 2) {      // 64 channels and more: the automatic choice asks for it from 256 filters on
        if (g.xcd_ranges) {
            if (g.planes_out != nullptr)
                launch_kernel((conv_kernel<AB, WB, CWS, S::CWT, S::TPC, S::GT, S::P, true, true>), grid_for(g), dim3(256), 0, s, g);
            else
                launch_kernel((conv_kernel<AB, WB, CWS, S::CWT, S::TPC, S::GT, S::P, false, true>), grid_for(g), dim3(256), 0, s, g);
            return launch_status();
        }
    }
    if (g.planes_out != nullptr)
        launch_kernel((conv_kernel<AB, WB, CWS, S::CWT, S::TPC, S::GT, S::P, true>), grid_for(g), dim3(256), 0, s, g);
    else
        launch_kernel((conv_kernel<AB, WB, CWS, S::CWT, S::TPC, S::GT, S::P, false>), grid_for(g), dim3(256), 0, s, g);
    return launch_status();
}

template <int AB, int WB>
hipError_t launch_conv_t(const BranchArgs &g, hipStream_t s) {
    // plane strides with a dedicated instantiation (a bounded list of bit widths, see conv_has_fixed_widths)
    if constexpr (conv_has_fixed_widths(AB, WB)) {
        switch (g.Cw) {
            case 1: return launch_conv_fixed<AB, WB, 1>(g, s);
            case 2: return launch_conv_fixed<AB, WB, 2>(g, s);
            case 4: return launch_conv_fixed<AB, WB, 4>(g, s);
            case 8: return launch_conv_fixed<AB, WB, 8>(g, s);
            case 16: return launch_conv_fixed<AB, WB, 16>(g, s);
            default: break;
        }
    }
    if (g.geo.sh != 1) return hipErrorInvalidValue;                  // host bug: strided needs a fixed shape
    // any other channel count: runtime stride, chunks of two channel words while the two stage
    // buffers (2 * AB * CWT SGPRs) leave the allocator room, else one word
    const bool emit = g.planes_out != nullptr;
    if constexpr (AB <= 4 && WB <= 2) {
        // plane strides that are multiples of four words (384, 640 ... channels): chunks of four words
        if (g.Cw % 4 == 0) {
            if (emit) launch_kernel((conv_kernel<AB, WB, 0, 4, 9, 1, 1, true>), grid_for(g), dim3(256), 0, s, g);
            else launch_kernel((conv_kernel<AB, WB, 0, 4, 9, 1, 1, false>), grid_for(g), dim3(256), 0, s, g);
            return launch_status();
        }
    }
    if (g.Cw == 1 || AB > 4) {
        if (emit) launch_kernel((conv_kernel<AB, WB, 0, 1, 9, 1, 1, true>), grid_for(g), dim3(256), 0, s, g);
        else launch_kernel((conv_kernel<AB, WB, 0, 1, 9, 1, 1, false>), grid_for(g), dim3(256), 0, s, g);
    } else if constexpr (AB <= 4) {
        if (emit) launch_kernel((conv_kernel<AB, WB, 0, 2, 9, 1, 1, true>), grid_for(g), dim3(256), 0, s, g);
        else launch_kernel((conv_kernel<AB, WB, 0, 2, 9, 1, 1, false>), grid_for(g), dim3(256), 0, s, g);
    }
    return launch_status();
}

}  // namespace

#define QNN_CAT2(a, b) a##b
#define QNN_CAT(a, b) QNN_CAT2(a, b)

hipError_t QNN_CAT(launch_gemm_ab, QNN_AB)(const BranchArgs &g, int wb, hipStream_t s) {
    switch (wb) {
        case 1: return launch_gemm_t<QNN_AB, 1>(g, s);
        case 2: return launch_gemm_t<QNN_AB, 2>(g, s);
        case 3: return launch_gemm_t<QNN_AB, 3>(g, s);
        case 4: return launch_gemm_t<QNN_AB, 4>(g, s);
        case 5: return launch_gemm_t<QNN_AB, 5>(g, s);
        case 6: return launch_gemm_t<QNN_AB, 6>(g, s);
        case 7: return launch_gemm_t<QNN_AB, 7>(g, s);
        case 8: return launch_gemm_t<QNN_AB, 8>(g, s);
    }
    return hipErrorInvalidValue;
}

hipError_t QNN_CAT(launch_conv_ab, QNN_AB)(const BranchArgs &g, int wb, hipStream_t s) {
    if (g.xcd_ranges && g.grid_blocks != grid_for(g).x) return hipErrorInvalidValue;   // host bug
    if (g.split_k && g.xcd_ranges) return hipErrorInvalidValue;
    if (g.geo.sh != g.geo.sw || (g.geo.sh != 1 && g.geo.sh != 2)) return hipErrorInvalidValue;
    switch (wb) {
        case 1: return launch_conv_t<QNN_AB, 1>(g, s);
        case 2: return launch_conv_t<QNN_AB, 2>(g, s);
        case 3: return launch_conv_t<QNN_AB, 3>(g, s);
        case 4: return launch_conv_t<QNN_AB, 4>(g, s);
        case 5: return launch_conv_t<QNN_AB, 5>(g, s);
        case 6: return launch_conv_t<QNN_AB, 6>(g, s);
        case 7: return launch_conv_t<QNN_AB, 7>(g, s);
        case 8: return launch_conv_t<QNN_AB, 8>(g, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace qnn
