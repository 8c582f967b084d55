/*
 * quartet.h -- C ABI of the MI355X (gfx950) Quartet MXFP4 linear-layer library.
 *
 * The library implements the linear-layer hot path of "Quartet: Native FP4 Training Can Be
 * Optimal for Large Language Models" (arXiv 2505.14669), Algorithm 1:
 *   Forward : X_q,M_x = QuEST(H_g X);  W_q,M_w = QuEST(H_g W);  y = GEMM_LP(X_q, W_q)
 *   Backward: G_q = Q(3/4 H^_g(dy, xi)), W'_q = Q(3/4 H^_g(W_q^T, xi)), dx = 16/9 H_g^-1((G_q W'_q^T) . M_x)
 *             and the same with dy^T, X_q^T for dW.
 * with g = 32 = the MXFP4 group size (Section 4.4).
 *
 * Conventions for every entry point
 *  - All data pointers are DEVICE pointers owned by the caller (hipMalloc'ed or a torch CUDA/HIP
 *    tensor's data_ptr).  The library never frees or keeps them.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is enqueued on it
 *    and the call returns without synchronizing; results are valid after the stream reaches that point.
 *  - Matrices are row-major.  bf16 = upper 16 bits of an IEEE binary32.
 *  - MXFP4 tensor [rows x k] (k % 32 == 0):
 *      codes  uint8 [rows x k/2] : E2M1 element 2j in bits 3:0 of byte j, element 2j+1 in bits 7:4;
 *                                  code = s e1 e0 m, magnitudes {0,.5,1,1.5,2,3,4,6}, bit 3 = sign;
 *      scales uint8, E8M0, value 2^(b-127), one per group of 32 consecutive elements of a row,
 *             stored TILED so that they are already in matrix-core lane order (on CDNA4 a scale is
 *             a per-lane register byte, so the scale-rearrangement pass of the paper's Section 4.4
 *             is folded into this layout): tiles of 32 rows x 8 groups, 256 bytes each, ordered
 *             [row/32][group/8]; the scale of (row, group g) is byte
 *               ((row/32) * ceil(k/256) + g/8) * 256 + ((g%2)*32 + row%32) * 4 + (g%8)/2.
 *             The buffer holds quartet_scale_bytes(rows, k) = ceil(rows/32) * ceil(k/256) * 256
 *             bytes, 4-byte aligned; bytes of rows >= rows or groups >= k/32 are never written
 *             and never used.
 *      mask   uint32 [rows x k/32] row-major: bit i of word j is 1 iff element 32j+i was NOT clipped.
 *  - Return value: QUARTET_OK, or a negative error.  Arguments are validated on the host before
 *    anything is launched; on QUARTET_EINVAL / QUARTET_ENOTSUP nothing has been enqueued.
 *    QUARTET_EHIP: a HIP call failed; quartet_last_hip_error() returns its hipError_t.
 *  - Pointers must be 16-byte aligned; leading dimensions are in elements and multiples of 8.
 *  - Inputs are finite with magnitude below 2^60; group sums of squares / maxima that are zero or
 *    subnormal are treated as zero (scale byte 127).
 *  - Thread safety: calls are independent except for the last-error slot, which is per thread.
 */
#ifndef QUARTET_H
#define QUARTET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QUARTET_OK 0
#define QUARTET_EINVAL (-1)  /* null pointer, bad shape, misaligned pointer or leading dimension */
#define QUARTET_ENOTSUP (-2) /* valid request this build does not support (size limit, dtype) */
#define QUARTET_EHIP (-3)    /* a HIP runtime call failed */

#define QUARTET_DTYPE_F32 0
#define QUARTET_DTYPE_BF16 1

#define QUARTET_ROUND_STOCHASTIC 0
#define QUARTET_ROUND_NEAREST 1

/* hipError_t of the last failed HIP call made by this thread through the library (0 if none). */
int quartet_last_hip_error(void);

/* Number of random bits one element's stochastic-rounding decision looks at (22). */
int quartet_sr_bits(void);

/* Size in bytes of the tiled scale buffer of an MXFP4 tensor [rows x k] (0 if an argument is negative). */
size_t quartet_scale_bytes(int64_t rows, int64_t k);

/*
 * Launch profiling (measurement support; the paper reports a per-stage runtime breakdown in its
 * appendix "Performance breakdown").  quartet_profile_enable(n > 0) makes the library bracket each
 * of its next kernel launches, up to n, with a pair of hipEvents recorded on the caller's stream;
 * n = 0 disables it and frees the events.  quartet_profile_read() waits for the recorded launches,
 * writes kind (QUARTET_KIND_*) and duration in milliseconds of each, in launch order, returns how
 * many it wrote (or a negative error) and restarts the record.  quartet_profile_kinds(mask) limits
 * the record to the kinds whose bit (1 << QUARTET_KIND_*) is set (default: all); an event pair costs
 * a few microseconds of stream time, so a timed region records only the kernel it is about.  The
 * record is process-global: use it from one thread, with profiling calls and launches on the same
 * device.
 */
#define QUARTET_KIND_QUANT_FWD 0
#define QUARTET_KIND_QUANT_BWD 1
#define QUARTET_KIND_REQUANT 2
#define QUARTET_KIND_GEMM 3
#define QUARTET_KIND_EPILOGUE 4
#define QUARTET_KIND_DEQUANT 5
#define QUARTET_KIND_FP8_QUANT 6
#define QUARTET_KIND_FP8_GEMM 7
int quartet_profile_enable(int max_records);
int quartet_profile_kinds(unsigned kind_mask);
int quartet_profile_read(int *kinds, float *ms, int capacity);

/*
 * Clock and ceiling measurements (measurement support, as above; no step of the method).
 *
 * quartet_profile_clock(c): c is a DEVICE pointer to two uint64 the caller has zeroed, or NULL to switch the
 * measurement off (the default).  While set, every block of the large-tile GEMM kernel launched through
 * quartet_mxfp4_gemm / quartet_mxfp4_gemm_grad (and through the linear-layer calls) adds the shader-clock ticks
 * it ran for to c[0] and the constant-clock ticks of the same interval to c[1] (two atomic additions per block);
 * c[0] / c[1] * quartet_wall_clock_khz() is the shader clock in kHz the chip held under that kernel.  8-byte
 * aligned; process-global, not thread-safe.
 * quartet_wall_clock_khz(): rate of the device's constant clock in kHz (negative: error).
 * quartet_probe_mfma_ceiling: launches `blocks` blocks of 4 waves that each run `iterations` rounds of the 16
 * v_mfma_scale_f32_32x32x64_f8f6f4 instructions of one K-step of the GEMM's 128 x 128 wave tile on operands held in
 * registers (no LDS or memory traffic inside the loop):
 * blocks * 4 * iterations * 16 * 2 * 32 * 32 * 64 flop.  codes: 32768 device bytes (8 fragments x 256 lanes x 16 B,
 * any E2M1 codes: the rate depends on the data, so pass quantized tensors of the workload), scales: 8192 device
 * bytes (8 x 256 dwords of E8M0 bytes), sink: blocks * 256 floats the kernel writes once at its end,
 * device_counters as for quartet_profile_clock or NULL.  The caller times the launch with events on `stream`.
 */
int quartet_profile_clock(uint64_t *device_counters);
int quartet_wall_clock_khz(void);
int quartet_probe_mfma_ceiling(const uint8_t *codes, const uint8_t *scales, int64_t iterations, int blocks,
                               float *sink, uint64_t *device_counters, void *stream);

/*
 * Forward quantizer (Algorithm 1 Forward, lines H_g then QuEST; Section 4.4 "Stage 1").
 * Logical input A[rows x k]:  transpose = 0: A = x, stored [rows x ldx];
 *                             transpose = 1: A = x^T, x stored [k x ldx] (ldx >= rows).
 * Per group of 32 along k: h = H_32 a (normalized Sylvester-Hadamard, butterflies of stride
 * 1,2,4,8,16 in fp32, then one multiply by fl(1/sqrt 32)); ss = sum h_i^2 (pairwise tree);
 * scale 2^e with e = floor((floor(log2 ss) - 6) / 2)  (= 2^floor(log2(RMS/sqrt 2)), the RMS-based
 * clipping of QuEST snapped to a power of two); code_i = round-to-nearest-even E2M1 of h_i 2^-e,
 * saturating at +-6; mask bit i = (|h_i 2^-e| <= 6).
 * Outputs: codes [rows x k/2], scales (tiled, quartet_scale_bytes(rows, k)), mask [rows x k/32]
 * (mask may be NULL).
 * Requires k % 32 == 0; transpose = 1 also rows % 8 == 0.  rows*k/32 must be below 2^31.
 */
int quartet_quant_fwd(const void *x_bf16, int64_t rows, int64_t k, int64_t ldx, int transpose,
                      uint8_t *codes, uint8_t *scales, uint32_t *mask, void *stream);

/*
 * Backward quantizer (Algorithm 1 Backward: H^_g(., xi) then Q(3/4 .); Section 3 "Rounding").
 * Same logical input as quartet_quant_fwd.  Per group: h = H_32 (d . a), d_i = -1 iff bit i of
 * sign_word (the same word for every group and for both operands of a GEMM, so the rotation
 * cancels in the product); m = max |h_i|; scale 2^e with e = floor(log2 m) - 2 (AbsMax, power of
 * two); v_i = fl((h_i 2^-e) * 3/4), so |v_i| < 6 and nothing clips; code_i = E2M1 of v_i by
 *   rounding = QUARTET_ROUND_NEAREST   : round-to-nearest-even (Algorithm 1 as printed), or
 *   rounding = QUARTET_ROUND_STOCHASTIC: with lo <= |v| < hi the neighbouring grid points and
 *     f = (|v|-lo)/(hi-lo), round up iff floor(f 2^22) + r >= 2^22, r = the element's 22-bit
 *     draw (probability floor(f 2^22) / 2^22 of rounding up).
 * Draws: Philox4x32-10 with key (seed & 0xFFFFFFFF, seed >> 32); the element at output position
 * L = row*k + kk uses call q = L / 16 with counter (q_lo, q_hi, stream_id, 0); with j = L mod 16,
 * output word j / 4 serves four elements, element t = j mod 4 rotates it so that byte t leads,
 * R = rotr32(word, 8 t + 8), and draws r = R >> 10.  The leading 8 bits of a word's four draws
 * are disjoint; the bits below are shared with the neighbours' leading bytes.  Row and transposed
 * mode give identical bytes for the same logical matrix.
 * The stored scale is 2^e: the 3/4 is NOT folded in; consumers multiply the product of two such
 * tensors by 16/9.
 */
int quartet_quant_bwd_sr(const void *x_bf16, int64_t rows, int64_t k, int64_t ldx, int transpose,
                         uint32_t sign_word, uint64_t seed, uint32_t stream_id, int rounding,
                         uint8_t *codes, uint8_t *scales, void *stream);

/*
 * Re-quantization of a saved MXFP4 tensor along its other dimension (Algorithm 1 Backward:
 * H^_g(W_q^T, xi), H^_g(X_q^T, xi) and their rounding).  src is an MXFP4 tensor stored [k x rows]
 * (codes [k x rows/2], tiled scales of a [k x rows] tensor, groups along `rows`).  The output is
 * quartet_quant_bwd_sr applied to decode(src)^T, a [rows x k] matrix with groups along k
 * (decoding is exact, so this step adds no rounding of its own).  rows % 32 == 0 and k % 32 == 0.
 */
int quartet_requant_transpose_sr(const uint8_t *src_codes, const uint8_t *src_scales,
                                 int64_t rows, int64_t k, uint32_t sign_word, uint64_t seed,
                                 uint32_t stream_id, int rounding,
                                 uint8_t *codes, uint8_t *scales, void *stream);

/*
 * The two operand quantizations of Algorithm 1 Forward in one launch: X [tokens x in] and W [out x in]
 * (bf16 row-major, leading dimension in), in % 32 == 0.  The outputs are bit-identical to
 *   quartet_quant_fwd(x, tokens, in, in, 0, xq_codes, xq_scales, x_mask) and
 *   quartet_quant_fwd(w, out,    in, in, 0, wq_codes, wq_scales, w_mask);
 * both masks are required.  quartet_linear_fwd runs this and the product.  Errors as for the two calls.
 */
int quartet_fwd_operands(const void *x_bf16, const void *w_bf16, int64_t tokens, int64_t in, int64_t out,
                         uint8_t *xq_codes, uint8_t *xq_scales, uint32_t *x_mask,
                         uint8_t *wq_codes, uint8_t *wq_scales, uint32_t *w_mask, void *stream);

/*
 * The three operand conversions of Algorithm 1 Backward that do not depend on each other, in one
 * launch (dy [tokens x out] bf16 row-major; X_q [tokens x in] and W_q [out x in] as
 * quartet_quant_fwd wrote them; tokens, in, out all % 32 == 0):
 *   dyt = quartet_quant_bwd_sr(dy, rows = out, k = tokens, ldx = out, transpose = 1, stream id 2)
 *   xt  = quartet_requant_transpose_sr(X_q, rows = in, k = tokens, stream id 3)
 *   wt  = quartet_requant_transpose_sr(W_q, rows = in, k = out,    stream id 1)
 * with the same sign_word, seed and rounding; the six outputs are bit-identical to those of the
 * three calls (dyt [out x tokens], xt [in x tokens], wt [in x out], codes and tiled scales).
 * quartet_linear_bwd runs the same kernel with quartet_quant_bwd_sr on dy (stream id 0) as a fourth
 * part of the grid, then the dW and the dx product.  Errors as for the three calls.
 */
int quartet_bwd_operands(const void *dy_bf16, int64_t tokens, int64_t in, int64_t out,
                         const uint8_t *xq_codes, const uint8_t *xq_scales,
                         const uint8_t *wq_codes, const uint8_t *wq_scales,
                         uint32_t sign_word, uint64_t seed, int rounding,
                         uint8_t *dyt_codes, uint8_t *dyt_scales, uint8_t *xt_codes, uint8_t *xt_scales,
                         uint8_t *wt_codes, uint8_t *wt_scales, void *stream);

/*
 * GEMM_LP (Section 4.4 "Stage 2": D = (A x SFA)(B x SFB), scales along K, one per 32):
 *   D[m x n] = alpha * sum_k dec(A)[m,k] * dec(B)[n,k]
 * A = (a_codes [m x k/2], a_scales tiled for [m x k]), B = (b_codes [n x k/2], b_scales tiled for
 * [n x k]), both K-contiguous.  Products are exact, accumulation is fp32 on the matrix cores.  d is fp32 or bf16
 * (d_dtype), row-major with leading dimension n <= ldd <= 2^21.  k % 32 == 0, k <= 2^23; m, n arbitrary.
 */
int quartet_mxfp4_gemm(const uint8_t *a_codes, const uint8_t *a_scales,
                       const uint8_t *b_codes, const uint8_t *b_scales,
                       int64_t m, int64_t n, int64_t k, float alpha,
                       void *d, int d_dtype, int64_t ldd, void *stream);

/*
 * Test and tuning aid (no part of the method): which of the library's GEMM kernels quartet_mxfp4_gemm and
 * quartet_mxfp4_gemm_grad launch from now on.  variant -1 = choose by problem size (the default); 0, 1, 2 = tiles
 * of 256 x 256, 128 x 256 or 128 x 128 (all three: one block per compute unit streams its tiles through a ring of
 * four LDS stages).  band_height 0 = choose by shape (the default), 1..64 = tile rows each XCD walks at a time.
 * Every combination gives the same results up to fp32 summation order; the parity tests use this to
 * reach each kernel.  Process-global, not thread-safe.  QUARTET_EINVAL outside those ranges.
 */
int quartet_debug_set_gemm_plan(int variant, int band_height);

/*
 * GEMM_LP with the gradient epilogue applied in the same kernel (Algorithm 1 Backward:
 * dx = 16/9 H_g^-1(dx_q . M_x), dW likewise):
 *   D[m x n] = scale * H_32_along_n( (sum_k dec(A)[m,k] dec(B)[n,k]) . mask )
 * Operands and limits as quartet_mxfp4_gemm, plus n % 32 == 0; mask is [m x n/32] words (bit i of
 * word [r, g] = column 32 g + i) or NULL (all ones).  The result equals quartet_mxfp4_gemm with
 * alpha = 1 into fp32 followed by quartet_grad_epilogue, bit for bit, without the fp32
 * intermediate ever reaching memory.
 */
int quartet_mxfp4_gemm_grad(const uint8_t *a_codes, const uint8_t *a_scales,
                            const uint8_t *b_codes, const uint8_t *b_scales,
                            int64_t m, int64_t n, int64_t k, const uint32_t *mask, float scale,
                            void *d, int d_dtype, int64_t ldd, void *stream);

/*
 * Two products with the gradient epilogue in one launch (Algorithm 1 Backward computes dW and dx from four operands
 * that are all known before either product starts, so neither waits for the other).  Each argument block describes one
 * product exactly as the arguments of quartet_mxfp4_gemm_grad do; both results have the type d_dtype.  The structures
 * are read on the host during the call; every pointer inside them is a device pointer.  The results are those of two
 * calls of quartet_mxfp4_gemm_grad (first, then second): bit for bit when the pair runs on the tile shape each product
 * would get alone (always, under quartet_debug_set_gemm_plan with a forced shape), else up to the order of the fp32 sums
 * along k.  The compute units go through the first product's tiles,
 * then the second's, without draining in between: one ramp-up and one drain, and the second product fills the compute
 * units the first leaves idle in its last round.  One tile shape serves both products (chosen for the pair, or the one
 * quartet_debug_set_gemm_plan forces).  The two results must not overlap.  Errors as
 * quartet_mxfp4_gemm_grad, checked for both products before anything is launched.
 */
typedef struct quartet_gemm_grad_args {
    const uint8_t *a_codes, *a_scales;   /* A: [m x k/2] codes, scales tiled for [m x k] */
    const uint8_t *b_codes, *b_scales;   /* B: [n x k/2] codes, scales tiled for [n x k] */
    int64_t m, n, k;
    const uint32_t *mask;                /* [m x n/32] words or NULL */
    float scale;
    void *d;                             /* [m x ldd] fp32 or bf16 */
    int64_t ldd;
} quartet_gemm_grad_args;
int quartet_mxfp4_gemm_grad_pair(const quartet_gemm_grad_args *first, const quartet_gemm_grad_args *second,
                                 int d_dtype, void *stream);

/*
 * MXFP8 twin of the quantizer and the GEMM, for the comparison the paper draws (Section 5, "Speedup
 * results": MXFP4 linear layers against MXFP8 ones; Section 3 names the format).  Elements are E4M3
 * (OCP 8-bit floating point: bias 7, largest magnitude 448, S.1111.111 = NaN, no infinities), one
 * byte each, with one E8M0 scale per 32 along k in the same tiled layout as MXFP4.
 *
 * quartet_mxfp8_quant: x bf16 [rows x ldx] -> codes [rows x k] bytes, scales tiled for [rows x k].
 *   Per group: scale byte b = max(E - 8, 0), E the biased fp32 exponent of the largest magnitude
 *   (which lands in the format's top binade); element = round-to-nearest-even of v 2^(127-b),
 *   saturating at 448.  No rotation, no clipping mask.  k % 32 == 0, ldx % 8 == 0, ldx >= k.
 * quartet_mxfp8_gemm: D[m x n] = alpha * sum_k dec(A)[m,k] dec(B)[n,k], operands as above
 *   (a_codes [m x k], b_codes [n x k]), fp32 accumulation on the matrix cores, which align the 64
 *   products of one instruction to a common exponent: results agree with exact accumulation to
 *   about 2^-12 of the sum of the products' magnitudes in the worst case (relative Frobenius error
 *   below 1e-4), not to the last bit.  Arguments and limits
 *   otherwise as quartet_mxfp4_gemm.
 */
int quartet_mxfp8_quant(const void *x_bf16, int64_t rows, int64_t k, int64_t ldx,
                        uint8_t *codes, uint8_t *scales, void *stream);
int quartet_mxfp8_gemm(const uint8_t *a_codes, const uint8_t *a_scales,
                       const uint8_t *b_codes, const uint8_t *b_scales,
                       int64_t m, int64_t n, int64_t k, float alpha,
                       void *d, int d_dtype, int64_t ldd, void *stream);

/*
 * Gradient epilogue (Algorithm 1 Backward: 16/9 H_g^-1(G . M)):
 *   out[m x n] = scale * H_32_along_n( g . mask ),  g fp32 [m x n], mask [m x n/32] or NULL (all ones).
 * g . mask keeps g where the bit is set and is +0 elsewhere; H_32 is its own inverse; fp32 steps
 * in the butterfly order of quartet_quant_fwd, the multiply by `scale` last.  out is fp32 or bf16
 * (round-to-nearest-even) and may alias g only if out_dtype is fp32.  n % 32 == 0.
 */
int quartet_grad_epilogue(const float *g, const uint32_t *mask, int64_t m, int64_t n, float scale,
                          void *out, int out_dtype, void *stream);

/* fp32 values of an MXFP4 tensor: out[rows x k] = E2M1 value * 2^(scale-127).  Test/debug helper. */
int quartet_mxfp4_dequant(const uint8_t *codes, const uint8_t *scales, int64_t rows, int64_t k,
                          float *out, void *stream);

/*
 * Algorithm 1 Forward.  x [tokens x in], w [out x in] bf16 -> y [tokens x out] (y_dtype) and the
 * context {X_q, W_q, M_x, M_w} written to caller buffers (shapes as for quartet_quant_fwd with
 * k = in).  in % 32 == 0.
 */
int quartet_linear_fwd(const void *x_bf16, const void *w_bf16, int64_t tokens, int64_t in, int64_t out,
                       void *y, int y_dtype,
                       uint8_t *xq_codes, uint8_t *xq_scales, uint32_t *x_mask,
                       uint8_t *wq_codes, uint8_t *wq_scales, uint32_t *w_mask,
                       void *stream);

/* Bytes of device workspace quartet_linear_bwd needs for these shapes (0 on invalid shapes). */
size_t quartet_linear_workspace_bytes(int64_t tokens, int64_t in, int64_t out);

/*
 * Algorithm 1 Backward with seed xi.  dy [tokens x out] bf16 and the forward context ->
 * dx [tokens x in], dw [out x in] (grad_dtype).  sign_word = first output word of Philox4x32-10 at
 * counter (0,0,0,0xFFFFFFFF) under the seed's key; Philox stream ids 0,1,2,3 serve dy, W_q^T, dy^T,
 * X_q^T.  tokens, in, out all % 32 == 0.  workspace: device memory of at least
 * quartet_linear_workspace_bytes() bytes, 256-byte aligned, used only during the call's work (it holds
 * the four quantized operands of the two gradient products, each in a region of its own).
 * Launches: Q(dy), Q(dy^T), Q(X_q^T) and Q(W_q^T) in one kernel, then the dW and the dx product in one kernel
 * (quartet_mxfp4_gemm_grad_pair); the results do not depend on the order (every operand has its own Philox stream).
 */
int quartet_linear_bwd(const void *dy_bf16, int64_t tokens, int64_t in, int64_t out,
                       const uint8_t *xq_codes, const uint8_t *xq_scales, const uint32_t *x_mask,
                       const uint8_t *wq_codes, const uint8_t *wq_scales, const uint32_t *w_mask,
                       uint64_t seed, int rounding,
                       void *dx, void *dw, int grad_dtype,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * quartet_linear_bwd for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving or training loops, harnesses that forbid hipMalloc.  Same arguments, results and launch
 * order as quartet_linear_bwd (bit for bit), but the four quantized operands live in a device array that is part
 * of the library's code object: QUARTET_STATIC_SCRATCH_BYTES (64 MiB) on every GPU the library is loaded on, held
 * until the process ends.  The call allocates and frees nothing and clears nothing (every byte it reads from the
 * array it has written before in the same call).  Shapes whose workspace (quartet_linear_workspace_bytes) exceeds
 * the array return QUARTET_ENOTSUP with nothing enqueued; other errors as quartet_linear_bwd.  The first call on a
 * device looks the array's address up (hipGetSymbolAddress), so make that call outside a graph capture.  All calls
 * on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two threads) race; calls
 * on one stream are ordered and safe.  quartet_static_scratch_bytes() returns the array's size.
 */
#define QUARTET_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
size_t quartet_static_scratch_bytes(void);
int quartet_linear_bwd_static(const void *dy_bf16, int64_t tokens, int64_t in, int64_t out,
                              const uint8_t *xq_codes, const uint8_t *xq_scales, const uint32_t *x_mask,
                              const uint8_t *wq_codes, const uint8_t *wq_scales, const uint32_t *w_mask,
                              uint64_t seed, int rounding,
                              void *dx, void *dw, int grad_dtype, void *stream);

/* sign word quartet_linear_bwd derives from a seed (host computation, no GPU work). */
uint32_t quartet_sign_word(uint64_t seed);

/*
 * Larger Hadamard blocks (Section 4.4, "Costs and format specialization": the rotation costs
 * O(g log g) and stays negligible up to g = 256).  hadamard_block = 32, 64, 128 or 256 elements; the
 * MXFP4 group stays 32, so scales, masks, draw positions and every layout are those of the functions
 * above, and hadamard_block = 32 gives exactly those functions.  H_g = H_{g/32} (x) H_32 is the
 * normalized Sylvester matrix of order g, evaluated as butterflies in this order: the stages that
 * combine whole 32-element groups first (stride 32, 64, ..., g/2), then stride 1, 2, 4, 8, 16 inside
 * each group, then one multiply by fl(1/sqrt g).  The dimension the blocks run along must be a
 * multiple of hadamard_block.
 *
 * Sign vector of the randomized rotation: g/32 words, element i of a block negated iff bit i%32 of
 * word i/32.  quartet_sign_words (host computation, no GPU work) writes the eight words a seed
 * stands for: words 0..3 are the outputs of Philox4x32-10 at counter (0,0,0,0xFFFFFFFF) under the
 * seed's key, words 4..7 those at counter (1,0,0,0xFFFFFFFF); word 0 = quartet_sign_word(seed).
 * sign_words arguments are HOST pointers to at least hadamard_block/32 words.
 *
 * quartet_mxfp4_gemm_grad_block is quartet_mxfp4_gemm_grad for blocks of 32, 64 or 128 columns (n a
 * multiple of the block); a block of 256 spans the tiles of two waves and returns QUARTET_ENOTSUP:
 * quartet_linear_bwd_block then runs the plain GEMM into its workspace and quartet_grad_epilogue_block
 * after it (quartet_linear_workspace_bytes_block accounts for that).
 */
int quartet_sign_words(uint64_t seed, uint32_t *out8);
int quartet_quant_fwd_block(const void *x_bf16, int64_t rows, int64_t k, int64_t ldx, int transpose,
                            int hadamard_block, uint8_t *codes, uint8_t *scales, uint32_t *mask, void *stream);
int quartet_quant_bwd_sr_block(const void *x_bf16, int64_t rows, int64_t k, int64_t ldx, int transpose,
                               int hadamard_block, const uint32_t *sign_words, uint64_t seed,
                               uint32_t stream_id, int rounding, uint8_t *codes, uint8_t *scales, void *stream);
int quartet_requant_transpose_sr_block(const uint8_t *src_codes, const uint8_t *src_scales,
                                       int64_t rows, int64_t k, int hadamard_block,
                                       const uint32_t *sign_words, uint64_t seed, uint32_t stream_id,
                                       int rounding, uint8_t *codes, uint8_t *scales, void *stream);
int quartet_mxfp4_gemm_grad_block(const uint8_t *a_codes, const uint8_t *a_scales,
                                  const uint8_t *b_codes, const uint8_t *b_scales,
                                  int64_t m, int64_t n, int64_t k, int hadamard_block, const uint32_t *mask,
                                  float scale, void *d, int d_dtype, int64_t ldd, void *stream);
int quartet_grad_epilogue_block(const float *g, const uint32_t *mask, int64_t m, int64_t n, int hadamard_block,
                                float scale, void *out, int out_dtype, void *stream);
int quartet_linear_fwd_block(const void *x_bf16, const void *w_bf16, int64_t tokens, int64_t in, int64_t out,
                             int hadamard_block, void *y, int y_dtype,
                             uint8_t *xq_codes, uint8_t *xq_scales, uint32_t *x_mask,
                             uint8_t *wq_codes, uint8_t *wq_scales, uint32_t *w_mask, void *stream);
size_t quartet_linear_workspace_bytes_block(int64_t tokens, int64_t in, int64_t out, int hadamard_block);
int quartet_linear_bwd_block(const void *dy_bf16, int64_t tokens, int64_t in, int64_t out, int hadamard_block,
                             const uint8_t *xq_codes, const uint8_t *xq_scales, const uint32_t *x_mask,
                             const uint8_t *wq_codes, const uint8_t *wq_scales, const uint32_t *w_mask,
                             uint64_t seed, int rounding, void *dx, void *dw, int grad_dtype,
                             void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QUARTET_H */
