/*
 * CPU oracle for the {-1,+1} encoding decomposition of quantized layers.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It is never part of the product path: only
 * the tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 * It shares no code, header, table or helper with the HIP sources.
 *
 * The decomposition is an exact identity on odd-integer codes (Sec. 3.1,
 * Eq. (8) equals Eq. (1)), so the reference result of a layer is the ordinary
 * integer product of the decoded codes, accumulated in int64.  The encoding
 * itself (Eq. (7)), the literal multi-branch sum (Eq. (8)) and the bit-plane
 * store are written out as well, so that each can be pinned against the values
 * and identities the paper fixes.
 *
 * Conventions (readings of the paper where it is silent are listed in the
 * design notes of the repository):
 *   - codes are odd integers v with |v| <= 2^bits - 1, held as int16;
 *   - element c_m (m = 1..bits) has weight 2^(m-1); c_1 is the low element
 *     (Sec. 3.2: x = x_1 + 2 x_2 with x_2 the high bit);
 *   - in a stored bit-plane a set bit means +1, a clear bit means -1.
 *
 * Parallelism: an OpenMP "parallel for" over the outermost loop only.
 */
#include <stdint.h>
#include <stddef.h>
#include <math.h>

/* ---- Eq. (7): x = sum_{m=1..M} 2^(m-1) c_m, c_m in {-1,+1} ------------- */

/* Writes c[0..bits-1] = c_1..c_M.  Returns 0, or -1 if v is not a code.
 * Greedy from the high element down: the remaining elements can represent
 * magnitudes up to 2^(m-1)-1 only, so the sign of the residual fixes c_m. */
int qnn_oracle_encode(int64_t v, int bits, int8_t *c)
{
    if (bits < 1 || bits > 8) return -1;
    int64_t vmax = ((int64_t)1 << bits) - 1;
    if (v < -vmax || v > vmax || ((v & 1) == 0)) return -1;
    int64_t r = v;
    for (int m = bits; m >= 1; --m) {
        int8_t s = (r > 0) ? 1 : -1;
        c[m - 1] = s;
        r -= (int64_t)s * ((int64_t)1 << (m - 1));
    }
    return (r == 0) ? 0 : -1;
}

int64_t qnn_oracle_decode(const int8_t *c, int bits)
{
    int64_t v = 0;
    for (int m = 1; m <= bits; ++m) v += ((int64_t)1 << (m - 1)) * (int64_t)c[m - 1];
    return v;
}

/* ---- bit-plane store (Sec. 3.1 bit-plane rows; Sec. 5.4 bit-wise storage) - */

/* codes[rows][K] -> planes[rows][bits][Kw], Kw = ceil(K/32).
 * Plane p (0-based) holds element c_{p+1}; element k of a row is bit (k mod 32)
 * of word k/32; bit set <=> +1.  Bits past K are zero.
 * Returns the number of entries that are not valid codes (they pack as zeros). */
int64_t qnn_oracle_pack_planes(const int16_t *codes, int64_t rows, int64_t K, int bits,
                               uint32_t *planes)
{
    int64_t Kw = (K + 31) / 32;
    int64_t bad = 0;
    for (int64_t r = 0; r < rows; ++r) {
        for (int p = 0; p < bits; ++p)
            for (int64_t w = 0; w < Kw; ++w) planes[(r * bits + p) * Kw + w] = 0u;
        for (int64_t k = 0; k < K; ++k) {
            int8_t c[8];
            if (qnn_oracle_encode(codes[r * K + k], bits, c) != 0) { ++bad; continue; }
            for (int p = 0; p < bits; ++p)
                if (c[p] == 1) planes[(r * bits + p) * Kw + k / 32] |= (uint32_t)1 << (k % 32);
        }
    }
    return bad;
}

/* ---- Eq. (1): plain integer product ------------------------------------ */

/* C[M][N] = A[M][K] * W[K][N], int64 accumulate. */
void qnn_oracle_gemm(const int16_t *A, const int16_t *W, int64_t M, int64_t N, int64_t K,
                     int64_t *C)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k) s += (int64_t)A[i * K + k] * (int64_t)W[k * N + j];
            C[i * N + j] = s;
        }
}

/* Same product with the second operand given transposed: Wt[N][K]. */
void qnn_oracle_gemm_wt(const int16_t *A, const int16_t *Wt, int64_t M, int64_t N, int64_t K,
                        int64_t *C)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k) s += (int64_t)A[i * K + k] * (int64_t)Wt[j * K + k];
            C[i * N + j] = s;
        }
}

/* ---- direct 3x3 convolution (Sec. 3.2: Op may be a convolution) --------- */

/* O[n][oh][ow][f] = sum_{kh,kw,c} X[n][oh+kh-1][ow+kw-1][c] * Wt[f][kh][kw][c]
 * NHWC, stride 1, pad 1, cross-correlation, X taken as 0 outside the image. */
void qnn_oracle_conv3x3(const int16_t *X, const int16_t *Wt, int64_t Nb, int64_t H, int64_t W,
                        int64_t C, int64_t Cout, int64_t *O)
{
#pragma omp parallel for schedule(static)
    for (int64_t nh = 0; nh < Nb * H; ++nh) {
        int64_t n = nh / H, oh = nh % H;
        for (int64_t ow = 0; ow < W; ++ow)
            for (int64_t f = 0; f < Cout; ++f) {
                int64_t s = 0;
                for (int kh = 0; kh < 3; ++kh) {
                    int64_t ih = oh + kh - 1;
                    if (ih < 0 || ih >= H) continue;
                    for (int kw = 0; kw < 3; ++kw) {
                        int64_t iw = ow + kw - 1;
                        if (iw < 0 || iw >= W) continue;
                        const int16_t *x = X + ((n * H + ih) * W + iw) * C;
                        const int16_t *w = Wt + ((f * 3 + kh) * 3 + kw) * C;
                        for (int64_t c = 0; c < C; ++c) s += (int64_t)x[c] * (int64_t)w[c];
                    }
                }
                O[((n * H + oh) * W + ow) * Cout + f] = s;
            }
    }
}

/* ---- general 2-D convolution and transposed convolution ------------------
 * (Sec. 3.2: "Op" stands for the layer's linear operation; the networks of Sec. 5 use strided,
 *  7x7, 1x1, dilated and transposed forms of it.)  NHWC, cross-correlation, X taken as 0 outside
 *  the image.  Output size  Ho = (H + 2*ph - dh*(KH-1) - 1)/sh + 1  (likewise Wo):
 *    O[n][oh][ow][f] = sum_{kh,kw,c} X[n][oh*sh - ph + kh*dh][ow*sw - pw + kw*dw][c] * Wt[f][kh][kw][c] */
void qnn_oracle_conv2d(const int16_t *X, const int16_t *Wt, int64_t Nb, int64_t H, int64_t W, int64_t C,
                       int64_t Cout, int KH, int KW, int sh, int sw, int ph, int pw, int dh, int dw,
                       int64_t Ho, int64_t Wo, int64_t *O)
{
#pragma omp parallel for schedule(static)
    for (int64_t nh = 0; nh < Nb * Ho; ++nh) {
        int64_t n = nh / Ho, oh = nh % Ho;
        for (int64_t ow = 0; ow < Wo; ++ow)
            for (int64_t f = 0; f < Cout; ++f) {
                int64_t s = 0;
                for (int kh = 0; kh < KH; ++kh) {
                    int64_t ih = oh * sh - ph + (int64_t)kh * dh;
                    if (ih < 0 || ih >= H) continue;
                    for (int kw = 0; kw < KW; ++kw) {
                        int64_t iw = ow * sw - pw + (int64_t)kw * dw;
                        if (iw < 0 || iw >= W) continue;
                        const int16_t *x = X + ((n * H + ih) * W + iw) * C;
                        const int16_t *w = Wt + ((f * KH + kh) * KW + kw) * C;
                        for (int64_t c = 0; c < C; ++c) s += (int64_t)x[c] * (int64_t)w[c];
                    }
                }
                O[((n * Ho + oh) * Wo + ow) * Cout + f] = s;
            }
    }
}

/* Transposed convolution ("deconvolution"), written as the scatter it is defined by: every input
 * pixel (ih, iw) adds X[n][ih][iw][c] * Wt[f][kh][kw][c] to the output pixel
 *   oh = ih*sh - ph + kh*dh,  ow = iw*sw - pw + kw*dw   (if inside the Ho x Wo output).
 * O must hold Nb*Ho*Wo*Cout values; it is cleared here. */
void qnn_oracle_conv2d_transposed(const int16_t *X, const int16_t *Wt, int64_t Nb, int64_t H, int64_t W,
                                  int64_t C, int64_t Cout, int KH, int KW, int sh, int sw, int ph, int pw,
                                  int dh, int dw, int64_t Ho, int64_t Wo, int64_t *O)
{
    for (int64_t i = 0; i < Nb * Ho * Wo * Cout; ++i) O[i] = 0;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < Nb; ++n)
        for (int64_t ih = 0; ih < H; ++ih)
            for (int64_t iw = 0; iw < W; ++iw) {
                const int16_t *x = X + ((n * H + ih) * W + iw) * C;
                for (int kh = 0; kh < KH; ++kh) {
                    int64_t oh = ih * sh - ph + (int64_t)kh * dh;
                    if (oh < 0 || oh >= Ho) continue;
                    for (int kw = 0; kw < KW; ++kw) {
                        int64_t ow = iw * sw - pw + (int64_t)kw * dw;
                        if (ow < 0 || ow >= Wo) continue;
                        for (int64_t f = 0; f < Cout; ++f) {
                            const int16_t *w = Wt + ((f * KH + kh) * KW + kw) * C;
                            int64_t s = 0;
                            for (int64_t c = 0; c < C; ++c) s += (int64_t)x[c] * (int64_t)w[c];
                            O[((n * Ho + oh) * Wo + ow) * Cout + f] += s;
                        }
                    }
                }
            }
}

/* ---- Eq. (8): the multi-branch sum, written out literally --------------- */

/* XnorPopcount of two {-1,+1} vectors: the number of positions where they
 * agree minus the number where they differ (= their dot product). */
static int64_t xnor_popcount_pm1(const int8_t *c, const int8_t *d, int64_t n)
{
    int64_t agree = 0;
    for (int64_t i = 0; i < n; ++i) agree += (c[i] == d[i]) ? 1 : 0;
    return 2 * agree - n;
}

/* x^T w via Eq. (8): encode both vectors element by element with Eq. (7),
 * form the xb*wb branch results and add them with weights 2^(m-1) 2^(k-1).
 * cm / dk are caller scratch of n int8 each.  Returns INT64_MIN on a bad code. */
int64_t qnn_oracle_branch_dot(const int16_t *x, const int16_t *w, int64_t n, int xb, int wb,
                              int8_t *cm, int8_t *dk)
{
    int64_t total = 0;
    int8_t e[8];
    for (int m = 1; m <= xb; ++m)
        for (int k = 1; k <= wb; ++k) {
            for (int64_t i = 0; i < n; ++i) {
                if (qnn_oracle_encode(x[i], xb, e) != 0) return INT64_MIN;
                cm[i] = e[m - 1];
                if (qnn_oracle_encode(w[i], wb, e) != 0) return INT64_MIN;
                dk[i] = e[k - 1];
            }
            total += ((int64_t)1 << (m - 1)) * ((int64_t)1 << (k - 1)) * xnor_popcount_pm1(cm, dk, n);
        }
    return total;
}

/* ---- Eq. (9): scale --------------------------------------------------- */

/* y[i][j] = acc[i][j] * s[j] in double precision (the reference value). */
void qnn_oracle_scale_f64(const int64_t *acc, int64_t rows, int64_t cols, const float *s, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j) y[i * cols + j] = (double)acc[i * cols + j] * (double)s[j];
}

/* The same scale as one IEEE binary32 multiply of (float)acc by s[j].  Used
 * where a later integer decision (requantisation) depends on the rounded
 * value, so that both sides decide in binary32.  Build with -ffp-contract=off. */
void qnn_oracle_scale_f32(const int64_t *acc, int64_t rows, int64_t cols, const float *s, float *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j) {
            volatile float a = (float)acc[i * cols + j];
            y[i * cols + j] = a * s[j];
        }
}

/* ---- layer chain: pooling and re-encoding (Alg. 1 forward, Table 2) ------ */

/* 2x2 max pool, stride 2, NHWC float; H and W even. */
void qnn_oracle_maxpool2x2(const float *y, int64_t Nb, int64_t H, int64_t W, int64_t C, float *o)
{
    int64_t Ho = H / 2, Wo = W / 2;
#pragma omp parallel for schedule(static)
    for (int64_t nh = 0; nh < Nb * Ho; ++nh) {
        int64_t n = nh / Ho, oh = nh % Ho;
        for (int64_t ow = 0; ow < Wo; ++ow)
            for (int64_t c = 0; c < C; ++c) {
                float m = y[((n * H + 2 * oh) * W + 2 * ow) * C + c];
                for (int dh = 0; dh < 2; ++dh)
                    for (int dw = 0; dw < 2; ++dw) {
                        float v = y[((n * H + 2 * oh + dh) * W + 2 * ow + dw) * C + c];
                        if (v > m) m = v;
                    }
                o[((n * Ho + oh) * Wo + ow) * C + c] = m;
            }
    }
}

/* Real value (in code units) -> nearest-below-in-magnitude odd code, following
 * the interval closures of Table 2 scaled by 2^bits-1:
 *   magnitude a = |y| falls in [2j, 2j+2) -> 2j+1, clamped to 2^bits-1;
 *   y > 0 -> +, otherwise (including 0) -> -.                                  */
int16_t qnn_oracle_round_odd(float y, int bits)
{
    double a = fabs((double)y);
    double cmax = (double)(((int64_t)1 << bits) - 1);
    double c = 2.0 * floor(a / 2.0) + 1.0;
    if (!(c <= cmax)) c = cmax;            /* also catches inf/nan -> clamp */
    return (int16_t)((y > 0.0f) ? c : -c);
}

void qnn_oracle_requant(const float *y, int64_t n, int bits, int16_t *codes)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) codes[i] = qnn_oracle_round_odd(y[i], bits);
}

/* ---- real-valued front end (Sec. 3.2: clip, then encode) -------------------
 * Table 1 limits the data to [-1,1] (HTanh) or [0,1] (HReLU); Table 2 then maps the number
 * space to the encoded states (for 2 bits: [-1,-2/3] -> -1, (-2/3,0] -> -1/3, (0,2/3) -> 1/3,
 * [2/3,1] -> 1, i.e. odd codes over alpha = 2^bits - 1).  The product x * alpha is formed in
 * binary32 (one rounding, volatile so that it is not contracted or widened): that is the
 * precision in which the interval decision is taken; everything after it is exact.
 * hrelu != 0 clips to [0,1] first (x <= 0 and NaN -> 0); values beyond +-1 clamp in round_odd. */
void qnn_oracle_encode_real(const float *x, int64_t n, int bits, int hrelu, int16_t *codes)
{
    const float alpha = (float)(((int64_t)1 << bits) - 1);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        float v = x[i];
        if (hrelu) v = (v > 0.0f) ? v : 0.0f;
        volatile float y = v * alpha;
        codes[i] = qnn_oracle_round_odd(y, bits);
    }
}

/* The smooth range limiters of Table 1 in front of the same encoder: Tanh(x) (range (-1,1), then
 * the number space of Table 2 as after HTanh) and Sigmoid(x) (range (0,1), as after HReLU).
 * The limiter is evaluated in double precision with the C library and rounded once to binary32;
 * that value times alpha (one binary32 multiply) is what the interval rule sees.
 * clip: 2 = Tanh, 3 = Sigmoid.  Also returns the limited value in binary32 (`limited`, may be
 * NULL) so that a test can tell how far an element is from an interval boundary.             */
void qnn_oracle_encode_smooth(const float *x, int64_t n, int bits, int clip, int16_t *codes, float *limited)
{
    const float alpha = (float)(((int64_t)1 << bits) - 1);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const double xd = (double)x[i];
        const double l = (clip == 2) ? tanh(xd) : 1.0 / (1.0 + exp(-xd));
        const float v = (float)l;
        if (limited) limited[i] = v;
        volatile float y = v * alpha;
        codes[i] = qnn_oracle_round_odd(y, bits);
    }
}

/* ---- training-side element-wise pieces (Sec. 4) ----------------------------------------------
 * Derivative of the M-bit encoder used in back-propagation (Eq. (12); Eq. (13) prints the 2-bit
 * case): for bit m = 1..M (m = 1 the low bit), with c_m = (2^M - 1) / 2^m,
 *     d phi_M^m / dx = +c_m pi cos(c_m pi x)  for m = M,   -c_m pi cos(c_m pi x)  for m < M,
 * inside -1 <= x <= 1 and 0 outside.  Alg. 1's BackMBitEncoder sums the M incoming gradients:
 *     g_x[i] = sum_m g[m-1][i] * d phi_M^m / dx (x[i]).
 * g is [M][n] (bit-major, low bit first), all in double precision.                            */
void qnn_oracle_encoder_backward(const float *x, const float *g, int64_t n, int M, double *gx)
{
    const double pi = 3.14159265358979323846;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const double xv = (double)x[i];
        double acc = 0.0;
        if (xv >= -1.0 && xv <= 1.0) {
            for (int m = 1; m <= M; ++m) {
                const double c = (double)(((int64_t)1 << M) - 1) / (double)((int64_t)1 << m);
                const double d = c * pi * cos(c * pi * xv);
                acc += (double)g[(int64_t)(m - 1) * n + i] * ((m == M) ? d : -d);
            }
        }
        gx[i] = acc;
    }
}

/* Binarize(w) = sign(HTanh(w)) (Eq. (14)), the weight binarisation of Alg. 1.  HTanh keeps the
 * sign, so this is the sign of w; sign(0) = +1 as in the binarised networks the section follows
 * (a NaN compares false and gives -1).  Its gradient passes where HTanh is the identity:
 *     g_w = g_wb  for |w| <= 1,   0 otherwise.                                                */
void qnn_oracle_binarize(const float *w, int64_t n, int8_t *wb)
{
    for (int64_t i = 0; i < n; ++i) wb[i] = (w[i] >= 0.0f) ? 1 : -1;
}

void qnn_oracle_binarize_backward(const float *w, const float *g_wb, int64_t n, float *g_w)
{
    for (int64_t i = 0; i < n; ++i) g_w[i] = (w[i] >= -1.0f && w[i] <= 1.0f) ? g_wb[i] : 0.0f;
}

/* Quantize_K(x) = round(clamp(x / t, 1) * (2^(K-1) - 1)) * d,  d = t / (2^(K-1) - 1)  (Eq. (15)),
 * K >= 2, t > 0.  Every step is one binary32 operation (division, clamp to [-1,1], multiply,
 * round to nearest with ties to even, multiply); the volatile temporaries keep the compiler from
 * contracting or widening them.  levels (may be NULL) receives the integer state.  The
 * straight-through gradient passes inside the clamp: g_x = g_q for |x / t| <= 1, else 0.        */
void qnn_oracle_quantize_k(const float *x, int64_t n, int K, float t, float *q, int32_t *levels)
{
    const float nlev = (float)(((int64_t)1 << (K - 1)) - 1);
    volatile float d = t / nlev;
    for (int64_t i = 0; i < n; ++i) {
        volatile float r = x[i] / t;
        float c = r;
        if (!(c <= 1.0f)) c = 1.0f;          /* also a NaN clamps to +1 */
        if (c < -1.0f) c = -1.0f;
        volatile float sc = c * nlev;
        const float k = rintf(sc);           /* default rounding mode: ties to even */
        volatile float out = k * d;
        q[i] = out;
        if (levels) levels[i] = (int32_t)k;
    }
}

void qnn_oracle_quantize_k_backward(const float *x, const float *g_q, int64_t n, float t, float *g_x)
{
    for (int64_t i = 0; i < n; ++i) {
        volatile float r = x[i] / t;
        g_x[i] = (r >= -1.0f && r <= 1.0f) ? g_q[i] : 0.0f;
    }
}

/* ---- Alg. 1, lines of the backward propagation through the multi-branch product ----------------
 * Fully connected layer, forward lines of Alg. 1 with a per-channel scale s[n] in the place of
 * r / ((2^M - 1)(2^K - 1)):
 *     a_hat[i][n] = sum_{m=1..M} sum_{k=1..K} 2^(m+k-2) sum_c a^{mb}[i][c] W^{kb}[n][c],   a[i][n] = s[n] a_hat[i][n].
 * Backward lines, given g_a = dC/da:
 *     g_ahat[i][n]     = s[n] g_a[i][n]
 *     g_{a^{mb}}[i][c] = sum_{k=1..K} 2^(m+k-2) backward(...),   backward(...)[i][c] = sum_n g_ahat[i][n] W^{kb}[n][c]
 *     g_{W^{kb}}[n][c] = sum_{m=1..M} 2^(m+k-2) backward(...),   backward(...)[n][c] = sum_i g_ahat[i][n] a^{mb}[i][c]
 * where backward() of a matrix product is the incoming gradient times the other operand (the
 * listing prints g_{a^{mb}} as the last argument of the second backward(); the gradient that
 * reaches the product is g_ahat, which is what is used here).  Everything in double precision;
 * the elements a^{mb}, W^{kb} in {-1,+1} come from the encoding of the codes (Eq. (7)).
 * A[M_rows][Kc] and W[N][Kc] hold odd-integer codes of xb and wb bits.
 * g_bits is [xb][M_rows][Kc] (low element first), g_wb is [wb][N][Kc].  s may be NULL (all ones). */
void qnn_oracle_branch_backward_input(const float *g_a, const float *s, const int16_t *W, int64_t M_rows,
                                      int64_t N, int64_t Kc, int xb, int wb, double *g_bits)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M_rows; ++i) {
        for (int64_t c = 0; c < Kc; ++c) {
            for (int m = 1; m <= xb; ++m) {
                double acc = 0.0;
                for (int k = 1; k <= wb; ++k) {
                    double back = 0.0;                     /* backward(a^{mb}, W^{kb}, g_ahat)[i][c] */
                    for (int64_t n = 0; n < N; ++n) {
                        int8_t e[8];
                        qnn_oracle_encode(W[n * Kc + c], wb, e);
                        const double g_ahat = (double)g_a[i * N + n] * (s ? (double)s[n] : 1.0);
                        back += g_ahat * (double)e[k - 1];
                    }
                    acc += (double)((int64_t)1 << (m + k - 2)) * back;
                }
                g_bits[((int64_t)(m - 1) * M_rows + i) * Kc + c] = acc;
            }
        }
    }
}

void qnn_oracle_branch_backward_weight(const float *g_a, const float *s, const int16_t *A, int64_t M_rows,
                                       int64_t N, int64_t Kc, int xb, int wb, double *g_wb)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t c = 0; c < Kc; ++c) {
            for (int k = 1; k <= wb; ++k) {
                double acc = 0.0;
                for (int m = 1; m <= xb; ++m) {
                    double back = 0.0;                     /* backward(a^{mb}, W^{kb}, g_ahat)[n][c] */
                    for (int64_t i = 0; i < M_rows; ++i) {
                        int8_t e[8];
                        qnn_oracle_encode(A[i * Kc + c], xb, e);
                        const double g_ahat = (double)g_a[i * N + n] * (s ? (double)s[n] : 1.0);
                        back += g_ahat * (double)e[m - 1];
                    }
                    acc += (double)((int64_t)1 << (m + k - 2)) * back;
                }
                g_wb[((int64_t)(k - 1) * N + n) * Kc + c] = acc;
            }
        }
    }
}

/* Update(W, g, eta) of Alg. 1 / Alg. 2 with plain stochastic gradient descent (the text names SGD
 * and Adam as the usual choices): w <- w - eta * g, one binary32 multiply and one subtraction.   */
void qnn_oracle_update_sgd(float *w, const float *g, int64_t n, float eta)
{
    for (int64_t i = 0; i < n; ++i) {
        volatile float step = eta * g[i];
        w[i] = w[i] - step;
    }
}

/* Update(W, g, eta) with Adam, the other optimiser the text names (Kingma & Ba's update rule):
 *     m <- b1 m + (1 - b1) g,   v <- b2 v + (1 - b2) g^2,
 *     w <- w - eta * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps).
 * Every operation is one binary32 operation in the order written (IEEE multiply, add, divide and
 * square root are correctly rounded, so a device that does the same steps gives the same bits);
 * 1 - b1, 1 - b2 and the two bias corrections 1 - b^t are formed in double precision and rounded
 * to binary32 once.  m, v, w are updated in place; t >= 1 is the step number.                   */
void qnn_oracle_update_adam(float *w, const float *g, float *m, float *v, int64_t n, float eta,
                            float b1, float b2, float eps, int t)
{
    const float omb1 = (float)(1.0 - (double)b1), omb2 = (float)(1.0 - (double)b2);
    const float bc1 = (float)(1.0 - pow((double)b1, (double)t)), bc2 = (float)(1.0 - pow((double)b2, (double)t));
    for (int64_t i = 0; i < n; ++i) {
        volatile float a = b1 * m[i];
        volatile float b = omb1 * g[i];
        volatile float mn = a + b;
        volatile float g2 = g[i] * g[i];
        volatile float c = b2 * v[i];
        volatile float d = omb2 * g2;
        volatile float vn = c + d;
        volatile float mh = mn / bc1;
        volatile float vh = vn / bc2;
        volatile float rt = sqrtf(vh);
        volatile float den = rt + eps;
        volatile float num = eta * mh;
        volatile float step = num / den;
        m[i] = mn;
        v[i] = vn;
        w[i] = w[i] - step;
    }
}

/* ---- Alg. 1, backward lines through the multi-branch product of a 3x3 convolution -------------
 * Forward (stride 1, zero padding 1, NHWC): a[n,h,w,o] = s[o] * sum_{m,k} 2^(m+k-2) sum_{kh,kw,c}
 * x^{mb}[n,h+kh-1,w+kw-1,c] W^{kb}[o,kh,kw,c], positions outside the image contributing nothing.
 * Backward, with g_ahat = s * g_a and backward() of a product = incoming gradient times the other
 * operand, summed over every output position the element took part in:
 *   g_{x^{mb}}[n,h,w,c]   = sum_k 2^(m+k-2) sum_{kh,kw,o} g_ahat[n,h-(kh-1),w-(kw-1),o] W^{kb}[o,kh,kw,c]
 *   g_{W^{kb}}[o,kh,kw,c] = sum_m 2^(m+k-2) sum_{n,h,w}   g_ahat[n,h,w,o] x^{mb}[n,h+kh-1,w+kw-1,c]
 * (terms whose image position does not exist are absent).  X codes [Nb][H][W][C] of xb bits, Wt
 * codes [O][3][3][C] of wb bits, g_a fp32 [Nb][H][W][O]; outputs double [xb][Nb][H][W][C] and
 * [wb][O][3][3][C].                                                                             */
void qnn_oracle_conv3x3_backward_input(const float *g_a, const float *s, const int16_t *Wt, int64_t Nb, int64_t H,
                                       int64_t W, int64_t C, int64_t O, int xb, int wb, double *g_bits)
{
#pragma omp parallel for schedule(static)
    for (int64_t pix = 0; pix < Nb * H * W; ++pix) {
        const int64_t n = pix / (H * W), h = (pix / W) % H, w = pix % W;
        for (int64_t c = 0; c < C; ++c)
            for (int m = 1; m <= xb; ++m) {
                double acc = 0.0;
                for (int k = 1; k <= wb; ++k) {
                    double back = 0.0;
                    for (int kh = 0; kh < 3; ++kh)
                        for (int kw = 0; kw < 3; ++kw) {
                            const int64_t oh = h - (kh - 1), ow = w - (kw - 1);     /* the output that read this pixel through (kh,kw) */
                            if (oh < 0 || oh >= H || ow < 0 || ow >= W) continue;
                            for (int64_t o = 0; o < O; ++o) {
                                int8_t e[8];
                                qnn_oracle_encode(Wt[((o * 3 + kh) * 3 + kw) * C + c], wb, e);
                                const double g_ahat = (double)g_a[((n * H + oh) * W + ow) * O + o] * (s ? (double)s[o] : 1.0);
                                back += g_ahat * (double)e[k - 1];
                            }
                        }
                    acc += (double)((int64_t)1 << (m + k - 2)) * back;
                }
                g_bits[((int64_t)(m - 1) * Nb * H * W + pix) * C + c] = acc;
            }
    }
}

void qnn_oracle_conv3x3_backward_weight(const float *g_a, const float *s, const int16_t *X, int64_t Nb, int64_t H,
                                        int64_t W, int64_t C, int64_t O, int xb, int wb, double *g_wb)
{
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < O; ++o)
        for (int kh = 0; kh < 3; ++kh)
            for (int kw = 0; kw < 3; ++kw)
                for (int64_t c = 0; c < C; ++c)
                    for (int k = 1; k <= wb; ++k) {
                        double acc = 0.0;
                        for (int m = 1; m <= xb; ++m) {
                            double back = 0.0;
                            for (int64_t n = 0; n < Nb; ++n)
                                for (int64_t h = 0; h < H; ++h)
                                    for (int64_t w = 0; w < W; ++w) {
                                        const int64_t ih = h + kh - 1, iw = w + kw - 1;
                                        if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                                        int8_t e[8];
                                        qnn_oracle_encode(X[((n * H + ih) * W + iw) * C + c], xb, e);
                                        const double g_ahat = (double)g_a[((n * H + h) * W + w) * O + o] * (s ? (double)s[o] : 1.0);
                                        back += g_ahat * (double)e[m - 1];
                                    }
                            acc += (double)((int64_t)1 << (m + k - 2)) * back;
                        }
                        g_wb[((int64_t)(k - 1) * O + o) * 9 * C + (kh * 3 + kw) * C + c] = acc;
                    }
}
