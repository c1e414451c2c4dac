/*
 * libqnn — C ABI of the {-1,+1} multi-branch binary matrix product on MI355X (gfx950).
 *
 * The method (paper Sec. 3.1, Eq. (7)-(8)): an odd integer code v, |v| <= 2^b - 1, is
 * written v = sum_{m=1..b} 2^(m-1) c_m with c_m in {-1,+1}.  A product of a b_a-bit
 * activation matrix with a b_w-bit weight matrix then splits into b_a*b_w binary
 * branch products; each is evaluated on bit-packed words as  L - 2*popcount(a xor w)
 * (= 2*popcount(xnor) - L) and the branches are summed with weights 2^(p+q).
 *
 * Conventions shared by every entry point
 *   - All pointers are DEVICE pointers (HBM) unless the parameter name starts with h_.
 *   - The caller owns every buffer.  Except where a function says otherwise the library
 *     allocates nothing, frees nothing and never synchronises: work is enqueued on
 *     `stream` (a hipStream_t passed as void*; NULL = the default stream) and the
 *     function returns at once.
 *   - Outputs are fully overwritten; inputs and outputs must not overlap.
 *   - Argument errors are detected on the host before anything is launched and are
 *     reported by the return code only (no exceptions, no aborts, no global state).
 *     Asynchronous device faults surface at the caller's next synchronisation.
 *   - Bit-plane layout ("planes"): uint32 [rows][bits][Kw], Kw = ceil(K/32).  Plane p
 *     (p = 0 low ... bits-1 high) holds element c_{p+1} of every code of the row;
 *     element k of the row is bit (k mod 32) of word k/32; bit 1 <=> +1, bit 0 <=> -1;
 *     bits at positions >= K are 0.  Plane buffers must be 16-byte aligned.
 */
#ifndef QNN_H
#define QNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    QNN_OK = 0,
    QNN_EINVAL = 1,        /* null pointer, bits outside 1..8, negative size, bad flag/enum   */
    QNN_EALIGN = 2,        /* a buffer is not aligned as documented                          */
    QNN_EUNSUPPORTED = 3,  /* a size beyond the documented limits                            */
    QNN_EWORKSPACE = 4,    /* workspace smaller than the matching *_workspace_bytes()         */
    QNN_EHIP = 5           /* the HIP runtime refused a launch (see qnn_last_hip_error)       */
} qnn_status;

/* Static, NUL-terminated description of a status code (never NULL). */
const char *qnn_status_string(int status);

/* hipError_t (as int) of the most recent failed launch on the calling thread, 0 if none. */
int qnn_last_hip_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int qnn_version(void);

/*
 * Compute units and peak shader clock (kHz) of the current GPU as the HIP runtime reports them,
 * written to HOST integers: the two factors of the integer vector-ALU peak (units x 64 lanes x
 * clock) that a benchmark prices the branch kernels against.  QNN_EINVAL for a NULL pointer,
 * QNN_EHIP if the runtime cannot be asked (no GPU).
 */
qnn_status qnn_device_info(int *h_compute_units, int *h_clock_khz);

/*
 * Performance knobs (process-wide; results never depend on them).  value 0 restores the
 * automatic choice.  Returns QNN_OK or QNN_EINVAL.
 * Who reads them: qnn_gemm_packed, qnn_conv2d_packed, qnn_conv2d_general, qnn_conv2d_im2col and
 * qnn_conv2d_im2col_static, on the host while they size their launch; no kernel and no other
 * entry point does.  Each knob is an atomic word read once per call, so qnn_tune may be called
 * from any thread at any time: a call that is already sizing its launch may use the old or the
 * new value of a knob (and the old value of one with the new value of another), a call that
 * starts after qnn_tune returns uses the new one.
 */
#define QNN_TUNE_WAVES_PER_SIMD 1 /* resident wavefronts per SIMD the launch sizing aims for */
#define QNN_TUNE_ROWS_PER_WAVE 2  /* rows (GEMM rows / output pixels) per wavefront        */
#define QNN_TUNE_GENERAL_ONLY 3   /* nonzero: qnn_conv2d_general keeps the windows it would  */
                                  /* hand to the kernel behind qnn_conv2d_packed (3x3, odd   */
                                  /* windows with "same" padding) in its own kernel (for     */
                                  /* comparisons)                                            */
#define QNN_TUNE_BLOCK_ORDER 4    /* convolution kernels: 1 plain block numbers, 2 one         */
                                  /* contiguous range of blocks (of pixels) per XCD            */
#define QNN_TUNE_LDS_PARTIALS 5   /* GEMM with several K chunks per wavefront: 1 partial sums   */
                                  /* through the output buffer, 2 in LDS where possible        */
#define QNN_TUNE_SPLIT_CHANNELS 6 /* 3x3 convolution: 1 one wavefront per (pixel run, 64 filters), 2 the   */
                                  /* four wavefronts of a block split the channel chunks where a      */
                                  /* kernel for that exists (automatic: layers with few pixels, and    */
                                  /* wherever the chunks divide evenly among the four wavefronts)     */
int qnn_tune(int key, int value);

/*
 * Profiling aid.  With a non-NULL device buffer, every wavefront w < bytes/32 of the branch
 * kernels launched afterwards (process-wide) writes four uint64 words at buffer + 32*w:
 * {start clock, end clock, HW_ID | XCC_ID << 32, start real-time clock}: the first two are the
 * shader clock of s_memtime (local to a compute unit), the last the chip-wide 100 MHz clock.
 * NULL switches tracing off.  The buffer must be 8-byte aligned and stay valid while traced
 * kernels run; results of the kernels do not change.  The address and the size are two words:
 * do not call this while another thread is inside one of the entry points that qnn_tune lists.
 */
int qnn_set_wave_trace(void *buffer, size_t bytes);

/* flags of qnn_encode_pack */
#define QNN_PACK_VALIDATE 1u /* count entries that are not codes into *bad_count */

/*
 * Encode + pack (Eq. (7); the bit-wise storage of the encoded matrices that Sec. 5.4 starts from).
 *   codes      [rows][K] row-major integer codes; element size code_bytes = 1 (int8,
 *              bits <= 7) or 2 (int16, any bits).  A valid code is odd with
 *              |v| <= 2^bits - 1.
 *   planes     out, uint32 [rows][bits][Kw] in the bit-plane layout above.
 *   bad_count  optional device int32.  With QNN_PACK_VALIDATE the number of entries that
 *              are not valid codes is ADDED to it (caller zeroes it); such entries pack
 *              as the lowest code (all plane bits 0).  Without the flag, or if NULL, no
 *              check is made and an invalid entry packs as the low `bits` binary digits
 *              of (v + 2^bits - 1) >> 1.
 *   rows == 0 or K == 0 is valid and launches nothing.
 * Limits: rows * bits * Kw < 2^40, K < 2^31.
 */
qnn_status qnn_encode_pack(const void *codes, int code_bytes, int64_t rows, int64_t K, int bits,
                           uint32_t *planes, int32_t *bad_count, unsigned flags, void *stream);

/*
 * Multi-branch binary GEMM with fused weighted accumulation (Eq. (8); Alg. 1 forward).
 *   A    activation planes [M][ab][Kw];  Wt  weight planes [N][wb][Kw] (the weight matrix
 *        transposed: row n holds output column n);  K = true inner length.
 *   acc  out int32 [M][N] row-major:
 *          acc[i][j] = sum_{p<ab} sum_{q<wb} 2^(p+q) * (K - 2*popcount(A[i][p] xor Wt[j][q]))
 *        which equals the integer product of the decoded codes.  May be NULL if out_f32
 *        is given.
 *   scale, out_f32   optional fused scale (Eq. (9)): if both non-NULL,
 *        out_f32[i][j] = (float)acc[i][j] * scale[j]  (one IEEE binary32 multiply).
 *        scale is fp32 [N]; out_f32 is fp32 [M][N].  Both NULL = no epilogue.
 *   M == 0 or N == 0 launches nothing.  K == 0 gives all zeros.
 * Limits (else QNN_EUNSUPPORTED): K*(2^ab-1)*(2^wb-1) < 2^31; M < 2^31; N <= 2^24; each
 *        plane buffer below 4 GiB (M*ab*Kw < 2^30 and N*wb*Kw < 2^30 words).
 */
qnn_status qnn_branch_gemm(const uint32_t *A, int ab, const uint32_t *Wt, int wb, int64_t M,
                           int64_t N, int64_t K, int32_t *acc, const float *scale,
                           float *out_f32, void *stream);

/*
 * 3x3 convolution, stride 1, zero padding 1, NHWC, as an implicit-im2col multi-branch
 * GEMM (Sec. 3.2: Op may be a convolution).  K order is (kh, kw, c), cross-correlation.
 *   x_codes   [Nb][H][W][C] codes (code_bytes as in qnn_encode_pack), ab bits.
 *   Wt        weight planes of the codes viewed as [Cout*9][C] rows, i.e. the output of
 *             qnn_encode_pack(codes = Wt[Cout][3][3][C], rows = Cout*9, K = C, bits = wb):
 *             uint32 [Cout][9][wb][Cw], Cw = ceil(C/32).
 *   acc       out int32 NHWC [Nb][H][W][Cout] (may be NULL if out_f32 is given);
 *             taps that fall outside the image contribute exactly 0.
 *   scale, out_f32  optional fused per-output-channel scale as in qnn_branch_gemm.
 *   workspace device scratch of at least qnn_conv2d_im2col_workspace_bytes() bytes,
 *             16-byte aligned; holds the per-pixel activation planes
 *             uint32 [Nb*H*W][ab][Cw] between the two kernels of this call.
 * Limits: 9*C*(2^ab-1)*(2^wb-1) < 2^31, Nb*H*W < 2^31, Cout <= 2^24, each plane buffer
 *         below 4 GiB (Nb*H*W*ab*Cw < 2^30 and Cout*9*wb*Cw < 2^30 words).
 */
size_t qnn_conv2d_im2col_workspace_bytes(int64_t Nb, int64_t H, int64_t W, int64_t C, int ab);

qnn_status qnn_conv2d_im2col(const void *x_codes, int code_bytes, int ab, const uint32_t *Wt,
                             int wb, int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Cout,
                             int32_t *acc, const float *scale, float *out_f32, void *workspace,
                             size_t workspace_bytes, void *stream);

/*
 * qnn_conv2d_im2col for callers that cannot allocate device memory or hand over a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same two
 * kernels, with the per-pixel activation planes in a scratch array that is part of the library
 * image (QNN_STATIC_SCRATCH_BYTES of device memory on every GPU the library runs on, held until the
 * process ends).  Arguments, results, limits and errors as for qnn_conv2d_im2col without the two
 * workspace arguments; additionally QNN_EUNSUPPORTED if the planes do not fit:
 *     Nb*H*W * ab * ceil(C/32) * 4  >  QNN_STATIC_SCRATCH_BYTES.
 * The call allocates and frees nothing.  The first call on a GPU looks up the array's address on
 * that GPU (the current device); make that call outside a stream capture.  All calls on one GPU
 * share the array: two calls that can overlap there (different streams, different threads) race on
 * it; calls on one stream are ordered and safe.  Nothing needs to start at zero: every word a call
 * reads was written by its own first kernel.
 */
#define QNN_STATIC_SCRATCH_BYTES (8u << 20)
qnn_status qnn_conv2d_im2col_static(const void *x_codes, int code_bytes, int ab, const uint32_t *Wt,
                                    int wb, int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Cout,
                                    int32_t *acc, const float *scale, float *out_f32, void *stream);

/*
 * The same convolution from activations that are already packed per pixel
 * (x_planes = qnn_encode_pack(codes viewed as [Nb*H*W][C], bits = ab), uint32
 * [Nb*H*W][ab][Cw]).  This is the second kernel of qnn_conv2d_im2col on its own; it is
 * what a layer chain calls when the previous layer already emitted packed planes.
 */
qnn_status qnn_conv2d_packed(const uint32_t *x_planes, int ab, const uint32_t *Wt, int wb,
                             int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Cout,
                             int32_t *acc, const float *scale, float *out_f32, void *stream);

/*
 * Re-encoding between layers (Alg. 1 forward: the scaled output of layer l is encoded for layer
 * l+1; Table 2 gives the rule for 2 bits): optional 2x2 max-pool (stride 2) of y, then each
 * value is mapped to the odd code grid of `bits` bits,
 *     a = |v|;  c = min(2*floor(a/2) + 1, 2^bits - 1);  code = (v > 0) ? +c : -c
 * (so [2j, 2j+2) -> 2j+1 in magnitude, 0 -> -1, NaN -> -(2^bits-1)), and written as
 *   codes   optional, [Nb][Ho][Wo][C] int8 (bits <= 7) or int16 (bits == 8);
 *   planes  optional, per-pixel bit planes uint32 [Nb*Ho*Wo][bits][ceil(C/32)] as consumed by
 *           qnn_conv2d_packed (16-byte aligned).
 * y is fp32 NHWC [Nb][H][W][C]; Ho = H/2, Wo = W/2 with pooling (H, W even), else H, W.
 * At least one of codes / planes must be given.  Outside the four entry points named by the
 * task; it exists for layer chains.
 */
qnn_status qnn_requant_pack(const float *y, int64_t Nb, int64_t H, int64_t W, int64_t C, int pool2x2,
                            int bits, void *codes, uint32_t *planes, void *stream);

/*
 * Real-valued front end (Sec. 3.2: the data is limited to a fixed range, Table 1, and then mapped
 * to its encoded state, Table 2 / the look-up form of the MBitEncoder of Eq. (10)).
 *   x      fp32 [rows][K];  clip selects the range limiter of Table 1:
 *            QNN_CLIP_HTANH    values beyond +-1 take the extreme states (the clamp of the rule below),
 *            QNN_CLIP_HRELU    first clips to [0,1] (x <= 0 and NaN -> 0),
 *            QNN_CLIP_TANH     x -> tanh(x),
 *            QNN_CLIP_SIGMOID  x -> 1 / (1 + exp(-x))
 *          (the two smooth ones in binary32 with the device math library, accurate to a few units of
 *          the last place: an input whose limited value lies within about 1e-6 of an interval
 *          boundary may land in the neighbouring state).
 *   y = limited x * (2^bits - 1) in binary32 (one multiply), then the rule of qnn_requant_pack:
 *   [2j, 2j+2)/(2^bits-1) -> code 2j+1, zero -> -1.  Outputs as in qnn_requant_pack: codes
 *   int8/int16 [rows][K] and/or planes uint32 [rows][bits][ceil(K/32)]; at least one must be given.
 */
#define QNN_CLIP_HTANH 0
#define QNN_CLIP_HRELU 1
#define QNN_CLIP_TANH 2
#define QNN_CLIP_SIGMOID 3
qnn_status qnn_encode_real(const float *x, int64_t rows, int64_t K, int bits, int clip, void *codes,
                           uint32_t *planes, void *stream);

/*
 * Element-wise pieces of the training procedures of Sec. 4 (none of them is on the inference path).
 *
 * qnn_encoder_backward   Eq. (12) / Alg. 1 "BackMBitEncoder": the gradient with respect to the real
 *   activation x from the gradients of its `bits` encoded elements,
 *       g_x[i] = sum_{m=1..bits} g_bits[m-1][i] * d phi^m / dx (x[i]),
 *       d phi^m / dx = s_m c_m pi cos(c_m pi x) for -1 <= x <= 1, else 0,
 *       c_m = (2^bits - 1) / 2^m,  s_m = +1 for m = bits (the high element), -1 otherwise.
 *   x fp32 [n], g_bits fp32 [bits][n] (low element first), g_x fp32 [n].
 *
 * qnn_binarize           Eq. (14): w_b = sign(HTanh(w)) with sign(0) = +1 (NaN -> -1), w fp32 [rows][K].
 *   codes   optional int8 [rows][K], values -1 / +1;
 *   planes  optional 1-bit planes uint32 [rows][1][ceil(K/32)] (16-byte aligned) in the layout of
 *           qnn_encode_pack, i.e. directly usable as the weight operand of the product entry points.
 * qnn_binarize_backward  g_w = g_wb where |w| <= 1 (HTanh is the identity there), else 0; fp32 [n].
 *
 * qnn_quantize_k         Eq. (15): q = round(clamp(x / t, 1) * (2^(bits-1) - 1)) * d with
 *   d = t / (2^(bits-1) - 1), every step one binary32 operation, round = to nearest, ties to even;
 *   2 <= bits <= 24, t > 0 finite (else QNN_EINVAL).  q fp32 [n] and/or levels int32 [n] (the integer
 *   state in -(2^(bits-1)-1) .. 2^(bits-1)-1); at least one must be given.
 * qnn_quantize_k_backward  straight-through gradient: g_x = g_q where |x / t| <= 1, else 0.
 *
 * n == 0 (rows == 0 or K == 0) launches nothing.  Limits: n * bits < 2^40.
 */
qnn_status qnn_encoder_backward(const float *x, const float *g_bits, int64_t n, int bits, float *g_x, void *stream);
qnn_status qnn_binarize(const float *w, int64_t rows, int64_t K, int8_t *codes, uint32_t *planes, void *stream);
qnn_status qnn_binarize_backward(const float *w, const float *g_wb, int64_t n, float *g_w, void *stream);
qnn_status qnn_quantize_k(const float *x, int64_t n, int bits, float t, float *q, int32_t *levels, void *stream);
qnn_status qnn_quantize_k_backward(const float *x, const float *g_q, int64_t n, float t, float *g_x, void *stream);

/*
 * Backward propagation through the multi-branch product of a fully connected layer (Alg. 1, the
 * backward lines; not on the inference path).  The forward call is qnn_branch_gemm: a[i][n] =
 * scale[n] * sum_{m,k} 2^(m+k-2) sum_c a^{mb}[i][c] W^{kb}[n][c].  Given g_out = dC/da, fp32 [M][N]
 * row-major, Alg. 1 first forms g_ahat[i][n] = scale[n] * g_out[i][n] (one binary32 multiply; scale
 * NULL = all ones) and then
 *   qnn_branch_gemm_backward_input    g_bits[m-1][i][c] = sum_k 2^(m+k-2) sum_n g_ahat[i][n] W^{kb}[n][c]
 *       the gradient of every encoded activation element, fp32 [ab][M][K] (low element first): what
 *       qnn_encoder_backward takes.  Wt = the packed weights of the forward call, uint32 [N][wb][ceil(K/32)].
 *   qnn_branch_gemm_backward_weight   g_wb[k-1][n][c] = sum_m 2^(m+k-2) sum_i g_ahat[i][n] a^{mb}[i][c]
 *       the gradient of every binary weight element, fp32 [wb][N][K]: what qnn_binarize_backward takes,
 *       element by element.  A = the packed activations of the forward call, uint32 [M][ab][ceil(K/32)].
 * (The listing prints g_{a^{mb}} as the last argument of the second backward(); the gradient that
 * reaches the product is g_ahat, which is used.)  Summed over the other operand's elements these
 * are 2^(m-1) * g_ahat . w and 2^(k-1) * g_ahat^T . a with the odd-integer codes w, a (Eq. (7)):
 * real-valued contractions, evaluated in binary32 on the matrix cores with the codes decoded from
 * the planes; the result differs from the exact sum by at most (J + 2) * 2^-24 * sum_j |term_j| per
 * output, J = N or M the length of the sum.
 * All buffers device memory, outputs written in full; g_out, scale, outputs 4-byte aligned, planes
 * 16-byte aligned.  M, N, K >= 0: an empty output launches nothing, an empty sum writes zeros.
 * Limits: M, N, K < 2^31; ab, wb in 1..8.  QNN_EINVAL / QNN_EALIGN / QNN_EUNSUPPORTED / QNN_EHIP as elsewhere.
 *
 * qnn_update_sgd   Update(W, g, eta) of Alg. 1 / Alg. 2 as plain gradient descent (the text names SGD
 *   and Adam as the usual choices): w[i] <- w[i] - lr * g[i], one binary32 multiply and one
 *   subtraction, in place; w, g fp32 [n].
 */
qnn_status qnn_branch_gemm_backward_input(const float *g_out, const float *scale, const uint32_t *Wt, int wb,
                                          int64_t M, int64_t N, int64_t K, int ab, float *g_bits, void *stream);
qnn_status qnn_branch_gemm_backward_weight(const float *g_out, const float *scale, const uint32_t *A, int ab,
                                           int64_t M, int64_t N, int64_t K, int wb, float *g_wb, void *stream);
/*
 * The same backward lines through the 3x3 / stride 1 / zero padding 1 convolution of qnn_conv2d_packed
 * (NHWC).  g_out = dC/da fp32 [Nb][H][W][Cout], g_ahat = scale[o] * g_out (scale NULL = ones);
 *   qnn_conv2d_backward_input    g_bits[m-1][n][h][w][c] = sum_k 2^(m+k-2) sum_{kh,kw,o}
 *       g_ahat[n][h-(kh-1)][w-(kw-1)][o] W^{kb}[o][kh][kw][c]      fp32 [ab][Nb][H][W][C]
 *       Wt = the packed weights of the forward call, uint32 [Cout][9][wb][ceil(C/32)].
 *   qnn_conv2d_backward_weight   g_wb[k-1][o][kh][kw][c] = sum_m 2^(m+k-2) sum_{n,h,w}
 *       g_ahat[n][h][w][o] x^{mb}[n][h+kh-1][w+kw-1][c]            fp32 [wb][Cout][3][3][C]
 *       x_planes = the packed activations of the forward call, uint32 [Nb*H*W][ab][ceil(C/32)];
 *       the pixels are summed in several ranges whose partial results pass through `workspace`
 *       (device memory, 16-byte aligned, at least qnn_conv2d_backward_weight_workspace_bytes(...) bytes)
 *       and are added in a fixed order: the result does not depend on the launch.
 * Positions outside the image contribute nothing.  Accuracy, alignment, empty sizes and status
 * codes as for the fully connected pair; QNN_EWORKSPACE for a workspace that is too small.
 * Limits: Nb*H*W < 2^30, C, Cout < 2^20.
 */
qnn_status qnn_conv2d_backward_input(const float *g_out, const float *scale, const uint32_t *Wt, int wb, int64_t Nb,
                                     int64_t H, int64_t W, int64_t C, int64_t Cout, int ab, float *g_bits, void *stream);
size_t qnn_conv2d_backward_weight_workspace_bytes(int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Cout);
qnn_status qnn_conv2d_backward_weight(const float *g_out, const float *scale, const uint32_t *x_planes, int ab, int64_t Nb,
                                      int64_t H, int64_t W, int64_t C, int64_t Cout, int wb, float *g_wb, void *workspace,
                                      size_t workspace_bytes, void *stream);
qnn_status qnn_update_sgd(float *w, const float *g, int64_t n, float lr, void *stream);
/*
 * qnn_update_adam   the same Update() with Adam (the text's other choice; Kingma & Ba's rule), in place:
 *   m <- beta1 m + (1 - beta1) g,  v <- beta2 v + (1 - beta2) g^2,
 *   w <- w - lr * (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps),
 *   every operation one correctly rounded binary32 operation in the order written; 1 - beta and the two
 *   bias corrections are formed in double precision on the host and rounded once.  w, g, m, v fp32 [n];
 *   step >= 1, 0 <= beta1, beta2 < 1, eps >= 0 (else QNN_EINVAL).
 */
qnn_status qnn_update_adam(float *w, const float *g, float *m, float *v, int64_t n, float lr, float beta1, float beta2,
                           float eps, int step, void *stream);

/*
 * Chained layers (Alg. 1 forward as one kernel: branch sum, scale, re-encode).  The *_requant
 * variants of the three product entry points compute the same int32 product, multiply by
 * scale[n] (scale == NULL: y = (float)acc), map y to the odd code grid of out_bits bits with the
 * rule of qnn_requant_pack, and write the result as the next layer's activation planes
 *   out_planes  uint32 [rows][out_bits][ceil(N/32)]   (rows = M, or Nb*H*W; N = Cout), 16-byte
 *               aligned, in the bit-plane layout above — exactly what qnn_requant_pack would
 *               produce from out_f32 without pooling.
 * acc and out_f32 are optional extra outputs (out_f32 needs scale).  If neither is given the
 * caller passes a workspace of qnn_requant_workspace_bytes(rows, N) bytes (16-byte aligned) that
 * holds partial sums of products done in several passes; qnn_conv2d_im2col_requant takes ONE
 * workspace of qnn_conv2d_im2col_requant_workspace_bytes() bytes for both purposes.
 * Other arguments, limits and errors as for the plain entry points; additionally
 * rows * out_bits * ceil(N/32) < 2^30.
 */
size_t qnn_requant_workspace_bytes(int64_t rows, int64_t N);

qnn_status qnn_branch_gemm_requant(const uint32_t *A, int ab, const uint32_t *Wt, int wb, int64_t M,
                                   int64_t N, int64_t K, const float *scale, int out_bits,
                                   uint32_t *out_planes, int32_t *acc, float *out_f32, void *workspace,
                                   size_t workspace_bytes, void *stream);

qnn_status qnn_conv2d_packed_requant(const uint32_t *x_planes, int ab, const uint32_t *Wt, int wb,
                                     int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Cout,
                                     const float *scale, int out_bits, uint32_t *out_planes,
                                     int32_t *acc, float *out_f32, void *workspace,
                                     size_t workspace_bytes, void *stream);

size_t qnn_conv2d_im2col_requant_workspace_bytes(int64_t Nb, int64_t H, int64_t W, int64_t C, int ab,
                                                 int64_t Cout);

qnn_status qnn_conv2d_im2col_requant(const void *x_codes, int code_bytes, int ab, const uint32_t *Wt,
                                     int wb, int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Cout,
                                     const float *scale, int out_bits, uint32_t *out_planes,
                                     int32_t *acc, float *out_f32, void *workspace,
                                     size_t workspace_bytes, void *stream);

/*
 * Convolution of any geometry (Sec. 3.2: "Op" is the layer's linear operation; the networks of
 * Sec. 5 use 7x7 stride-2, strided 3x3 and 1x1, dilated and transposed convolutions), NHWC,
 * cross-correlation, zero padding (taps outside the image contribute exactly 0).
 *   h_geo  HOST pointer to the window geometry (read during the call only).
 *          Convolution:  Ho = (H + 2*pad_h - dil_h*(kh-1) - 1) / stride_h + 1  (likewise Wo),
 *            out[n][oh][ow][f] = sum_{i,j,c} x[n][oh*stride_h - pad_h + i*dil_h][ow*stride_w - pad_w + j*dil_w][c]
 *                                            * w[f][i][j][c]
 *          Transposed (transposed = 1):  Ho = (H-1)*stride_h - 2*pad_h + dil_h*(kh-1) + out_pad_h + 1,
 *            input pixel (ih, iw) contributes x[n][ih][iw][c] * w[f][i][j][c] to the output pixel
 *            (ih*stride_h - pad_h + i*dil_h, iw*stride_w - pad_w + j*dil_w).
 *   x_planes  per-pixel activation planes uint32 [Nb*H*W][ab][ceil(C/32)] (qnn_encode_pack of the
 *          codes viewed as [Nb*H*W][C]).
 *   Wt     weight planes uint32 [Cout][kh*kw][wb][ceil(C/32)] = qnn_encode_pack of the weight
 *          codes w[Cout][kh][kw][C] viewed as [Cout*kh*kw][C].
 *   acc, scale, out_f32  as in qnn_conv2d_packed, NHWC [Nb][Ho][Wo][Cout].
 *   out_bits, out_planes  optional re-encoded result as in the *_requant entry points (out_bits = 0:
 *          none; then out_planes is ignored).
 *   workspace  optional device scratch (16-byte aligned).  It is REQUIRED (at least
 *          Nb*Ho*Wo*Cout*4 bytes) only when out_bits != 0 and neither acc nor out_f32 is given.
 *          With qnn_conv2d_general_workspace_bytes() bytes it also enables the packed-window path
 *          for few input channels (C <= 32, kh*kw*C <= 256, not transposed: e.g. a 7x7x3
 *          stem), which is several times faster; without it the result is the same.
 * qnn_conv2d_general_output_size writes Ho and Wo to HOST integers; both functions return
 * QNN_EINVAL for a geometry that is not positive (kernel, stride, dilation >= 1, padding >= 0,
 * out_pad only with transposed = 1 and smaller than max(stride, dilation), Ho, Wo >= 1).
 * Limits as for qnn_conv2d_packed with 9 replaced by kh*kw, for input and output pixel counts.
 * dense_rows = 1 (images with few channels, e.g. the 3-channel input of a network's stem): the
 * activations are packed per image ROW instead of per pixel, x_planes = qnn_encode_pack(codes
 * viewed as [Nb*H][W*C], bits = ab) = uint32 [Nb*H][ab][ceil(W*C/32)], an eighth of the per-pixel
 * size for C = 3, and a kernel row of the window is a run of KW*C consecutive bits.  Accepted
 * only where the packed-window path applies (forward convolution, C <= 32, kh*kw*C <= 256)
 * and with its workspace; QNN_EUNSUPPORTED otherwise.
 * The 3x3 / stride 1 / pad 1 / dilation 1 convolution with more than 32 channels, or without
 * the window workspace, runs on the kernel of qnn_conv2d_packed (same operands, same outputs;
 * QNN_TUNE_GENERAL_ONLY keeps it here); so do the 3x3 / stride 2 / pad 1 convolution and, at
 * stride 1, any odd window of at most 49 taps with "same" padding ((k/2) * dilation; equal
 * dilation in both directions) -- atrous 3x3, 5x5, 7x7, 1x3 ... -- for 64, 128, 256 or 512 input
 * channels at the bit widths that kernel has fixed shapes for (up to 4 x 4 bits all of these;
 * wider pairs where the shape takes one tap per pipeline stage).  A 1x1 convolution
 * without padding runs on the kernels of qnn_branch_gemm (rows = output pixels; with a stride and
 * bit widths up to 4 the rows are the strided selection of the input pixels).
 */
typedef struct {
    int kh, kw;
    int stride_h, stride_w;
    int pad_h, pad_w;
    int dil_h, dil_w;
    int transposed;
    int out_pad_h, out_pad_w;
    int dense_rows;   /* 1: x_planes is ROW-DENSE, see below (few input channels only); else 0 */
} qnn_conv_geometry;

qnn_status qnn_conv2d_general_output_size(int64_t H, int64_t W, const qnn_conv_geometry *h_geo,
                                          int64_t *h_Ho, int64_t *h_Wo);

size_t qnn_conv2d_general_workspace_bytes(int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Cout, int ab,
                                          int wb, const qnn_conv_geometry *h_geo);

qnn_status qnn_conv2d_general(const uint32_t *x_planes, int ab, const uint32_t *Wt, int wb, int64_t Nb,
                              int64_t H, int64_t W, int64_t C, int64_t Cout,
                              const qnn_conv_geometry *h_geo, int32_t *acc, const float *scale,
                              float *out_f32, int out_bits, uint32_t *out_planes, void *workspace,
                              size_t workspace_bytes, void *stream);

/*
 * 2x2 max-pool (stride 2) of activations that are already bit planes: planes uint32
 * [Nb*H*W][bits][ceil(C/32)] -> out_planes [Nb*(H/2)*(W/2)][bits][ceil(C/32)], H and W even.
 * The re-encoding rule is monotone, so pooling the codes equals re-encoding the pooled values
 * (Alg. 1 places the encoder after the layer's output; a pooling layer commutes with it).
 */
qnn_status qnn_maxpool2x2_planes(const uint32_t *planes, int64_t Nb, int64_t H, int64_t W, int64_t C,
                                 int bits, uint32_t *out_planes, void *stream);

/*
 * COMPARISON LINE, not part of the method: the same integer product of decoded int8 codes on the
 * int8 matrix cores, so that a benchmark can report what the decomposition costs on this chip.
 *   qnn_compare_mfma_arrange  codes int8 [rows][K] (any int8 values) -> `arranged`, an opaque
 *       buffer of qnn_compare_mfma_arranged_bytes(rows, K) bytes, 16-byte aligned (rows and K are
 *       padded to multiples of 32 with zeros).  Use it for A (rows = M) and for the transposed
 *       weights (rows = N).
 *   qnn_compare_mfma_gemm     acc int32 [M][N] = A . Wt^T from two arranged buffers.
 * Limits: K * 127 * 127 < 2^31, M, N < 2^31.
 */
size_t qnn_compare_mfma_arranged_bytes(int64_t rows, int64_t K);
qnn_status qnn_compare_mfma_arrange(const int8_t *codes, int64_t rows, int64_t K, void *arranged, void *stream);
qnn_status qnn_compare_mfma_gemm(const void *A_arranged, const void *Wt_arranged, int64_t M, int64_t N,
                                 int64_t K, int32_t *acc, void *stream);

/*
 * COMPARISON LINE, not part of the method: the same integer product of decoded int8 codes with
 * the vector ALU's packed int8 dot product (four multiply-adds per lane and instruction).
 *   A_codes int8 [M][K], Wt_codes int8 [N][K] (the weight matrix transposed), both row-major and
 *   4-byte aligned; acc int32 [M][N] = A . Wt^T.
 * Limits: K a multiple of 4 (else QNN_EUNSUPPORTED), K * 127 * 127 < 2^31, M, N < 2^31.
 */
qnn_status qnn_compare_dot4_gemm(const int8_t *A_codes, const int8_t *Wt_codes, int64_t M, int64_t N,
                                 int64_t K, int32_t *acc, void *stream);

/*
 * Stand-alone scale epilogue (Eq. (9); Eq. (19)): out_f32[i][j] = (float)acc[i][j] * scale[j],
 * acc int32 [M][N], scale fp32 [N], out fp32 [M][N].  One IEEE binary32 multiply per
 * element, no fused multiply-add.  M == 0 or N == 0 launches nothing.
 */
qnn_status qnn_scale_epilogue(const int32_t *acc, int64_t M, int64_t N, const float *scale,
                              float *out_f32, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QNN_H */
