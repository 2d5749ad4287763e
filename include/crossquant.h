/*
 * crossquant.h -- C ABI of the MI355X (gfx950) CrossQuant activation-quantization library.
 *
 * Implements the hot path of "CrossQuant" (arxiv 2410.07505): for an activation matrix
 * X in R^{T x I} (tokens x input channels; Background section) it computes the row-wise and
 * column-wise absolute maxima t and c, forms each element's step
 *     Delta~_ij = t_i^alpha * c_j^(1-alpha) / (2^(N-1) - 1)         (the CrossQuant equation)
 * quantizes, dequantizes, counts the quantization kernel (Definition 1) and runs the
 * integer linear layer Y = X . W (Background section) on the codes.
 *
 * Conventions common to every call
 *   - Every pointer is a DEVICE pointer owned by the caller; the library allocates nothing,
 *     frees nothing and never synchronises with the host.  `stream` is a hipStream_t passed as
 *     void* (NULL = the default stream).  All work is enqueued on that stream, in order.
 *   - X and W are IEEE binary16, row-major.  Outputs are fully overwritten; vectors that the
 *     kernels accumulate into (t, c, zero_count) are cleared on the stream inside the call.
 *   - Return value: CQ_OK (0) or a negative cq_status.  Argument errors, sizes over a limit and
 *     unsupported requests are found on the host before anything is enqueued: such a return means
 *     nothing was launched.  Only CQ_ERR_HIP (the runtime refused a launch) can follow earlier
 *     launches of the same call.
 *   - Preconditions not checked: X and W finite; buffers at least as large as stated.
 *   - Arithmetic is fixed so results are reproducible bit for bit: scale factors use binary64
 *     pow rounded once to binary32; every per-element result equals a single correctly rounded
 *     binary32 multiply/divide; round() is round-half-to-even; counters and accumulators are
 *     integers.  Order of accumulation never affects a result.
 */
#ifndef CROSSQUANT_H
#define CROSSQUANT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CQ_OK = 0,
    CQ_ERR_NULL = -1,        /* a required pointer is NULL */
    CQ_ERR_SHAPE = -2,       /* T, I or O < 1, a leading dimension too small, or a size over the limit */
    CQ_ERR_BITS = -3,        /* bits is neither 4 nor 8 (or INT4 packing with odd I) */
    CQ_ERR_ALPHA = -4,       /* alpha outside [0, 1] or not a number */
    CQ_ERR_ALIGN = -5,       /* a pointer violates the stated alignment */
    CQ_ERR_UNSUPPORTED = -6, /* valid request this build does not implement */
    CQ_ERR_HIP = -7,         /* a kernel launch failed (hipGetLastError) */
    CQ_ERR_ALIAS = -8        /* an output vector overlaps an input vector it must not overlap */
} cq_status;

/* Upper limits on sizes (keeps every index in 32 bits inside the kernels). */
#define CQ_MAX_DIM ((int64_t)1 << 24)        /* T, I, O, leading dimensions */
#define CQ_MAX_ELEMS ((int64_t)1 << 40)      /* T*I, I*O, T*O */
/* A launch is also limited to fewer than 2^32 threads, which only inputs made of millions of tiny
 * pieces reach (e.g. a batch of 2^23 or more one-token sequences: a sequence takes at least one
 * block of 512 threads); such a call returns CQ_ERR_SHAPE with nothing enqueued. */

/*
 * Row and column absolute maxima in one pass over X.
 *   t_i = max_j |X_ij|   (Eq. 1, per-token quantization)
 *   c_j = max_i |X_ij|   (the CrossQuant equation)
 * X: binary16 [T][ldx], ldx >= I (elements), 2-byte aligned (16-byte alignment of X together
 *    with ldx % 8 == 0 selects the vectorised path; any other layout takes a slower one).
 * t: out, float[T].  c: out, float[I].  Both are exact (a maximum of binary16 values).
 * The maxima are accumulated with atomics, so t and c are cleared first, inside the call.  In the
 * vectorised layout with I % 8 == 0 that is done by the one launch itself: its first blocks store the
 * zeros and the others wait for them (a bounded wait on a counter in library-owned device memory, one
 * per stream handle as for crossquant_quantize's zero count) before their atomics.  Calls captured
 * into a graph, calls on a stream without a counter of its own, and other layouts clear with a small
 * kernel of their own before the pass.
 */
int crossquant_absmax(const void *X, int64_t T, int64_t I, int64_t ldx, float *t, float *c,
                      void *stream);

/*
 * CrossQuant quantize + dequantize + kernel count (the CrossQuant equation, Definition 1, and
 * the dequantization of the appendix fake-quant listing).
 *   a_i = t_i^alpha / q_max,  b_j = c_j^(1-alpha),  q_max = 2^(bits-1) - 1
 *   D_ij = fl32(a_i * b_j);  q_ij = D_ij == 0 ? 0 : clamp(rne(fl32(X_ij / D_ij)), +-q_max)
 *   xhat_ij = fl16(fl32(q_ij * D_ij));   zero_count = #{(i,j): q_ij == 0}
 * t, c: in, float[T], float[I] (normally from crossquant_absmax; any non-negative finite values
 *       are accepted, e.g. calibrated ones -- codes are clamped to +-q_max).
 * alpha in [0,1]; bits in {8, 4}.
 * codes: out.  bits == 8: int8 [T][I].  bits == 4: I must be even; packed two's-complement
 *        nibbles [T][I/2], even column in the low nibble.
 * xhat: out, nullable, binary16 [T][I].
 * row_scale: out, float[T] (a).  col_scale: out, float[I] (b).  Required: the linear layer and
 *        the weight folding consume them.  They must not overlap t or c (CQ_ERR_ALIAS): the one
 *        kernel of this call reads t and c in every block while some blocks write a and b.
 * zero_count: out, nullable, one unsigned 64-bit counter.  It is accumulated in a word of
 *        library-owned device memory and stored by the last block to finish.  Every stream handle
 *        gets a word of its own (16 per process; calls on further streams, and on the per-thread
 *        default stream, clear the caller's counter with a small kernel first and add to it
 *        directly), so calls on different streams may overlap.  A call captured into a graph keeps
 *        the word of the stream it was captured on: replays of that graph must not overlap each
 *        other or calls on that stream.  The same holds for the batched, FP6 and count-only forms.
 */
int crossquant_quantize(const void *X, int64_t T, int64_t I, int64_t ldx, const float *t,
                        const float *c, float alpha, int bits, void *codes, void *xhat,
                        float *row_scale, float *col_scale, unsigned long long *zero_count,
                        void *stream);

/*
 * crossquant_absmax followed by crossquant_quantize as one call: same arguments, outputs and arithmetic
 * as the two (t and c included; row_scale / col_scale must not overlap them), any layout and size.
 * It enqueues the same two kernels the two calls do, so it costs what they cost: one-launch forms (a grid
 * barrier between the maxima and the quantize phase, with X kept on chip or re-read from the caches) were
 * measured slower on this device than the boundary between two kernels (see the next call).
 */
int crossquant_absmax_quantize(const void *X, int64_t T, int64_t I, int64_t ldx, float alpha, int bits,
                               float *t, float *c, void *codes, void *xhat, float *row_scale,
                               float *col_scale, unsigned long long *zero_count, void *stream);

/*
 * The same call as ONE kernel that reads X from HBM once and holds it in the chip's registers and LDS
 * across a grid-wide barrier (3 bytes of traffic per element instead of 5; 5 instead of 7 with xhat):
 * possible when the matrix fits, ceil(T/256) * ceil(I/512) <= number of CUs (256 on MI355X, i.e. up to
 * 4096 x 8192).  Arguments, outputs and arithmetic are exactly those of crossquant_absmax_quantize.
 * On this device it is SLOWER than crossquant_absmax_quantize although it moves fewer bytes (the barrier
 * keeps reads and writes apart in time and costs more than a kernel boundary): it is for input that is
 * expensive to read twice, and for measuring that trade.
 * Returns CQ_ERR_UNSUPPORTED, with nothing enqueued, if the matrix is too large or if the layout
 * is not the vector one (X and xhat 16-byte aligned, codes 8-byte aligned, ldx % 8 == 0, I % 8 == 0).
 * The barrier needs all blocks resident at once (one block per CU).  Other kernels running on the
 * device only delay it; if part of the device stays unavailable for seconds the kernel gives up
 * (it always terminates) and writes NaN into row_scale and col_scale.  The barrier's counters are
 * library-owned device memory, one pair per stream handle (16 per process, shared with the zero
 * counters of crossquant_quantize): calls on different streams may overlap; a stream without a
 * pair of its own (the 17th, or the per-thread default stream) gets CQ_ERR_UNSUPPORTED; calls captured
 * into a graph keep the pair of the stream they were captured on, so replays must not overlap.
 */
int crossquant_absmax_quantize_single_read(const void *X, int64_t T, int64_t I, int64_t ldx, float alpha,
                                           int bits, float *t, float *c, void *codes, void *xhat,
                                           float *row_scale, float *col_scale,
                                           unsigned long long *zero_count, void *stream);

/*
 * Batched forms for a [B][S][I] activation tensor (the shape the appendix fake-quant listing is
 * written for: the row maximum runs over the last axis, the column maximum over the second to
 * last, i.e. over the S tokens of ONE sequence).  Every sequence b is an independent S x I
 * problem with its own column maxima: results equal B separate calls of the plain forms, in one
 * launch.  Sequence b starts at X + b * batch_stride (elements; >= (S-1)*ldx + I); rows inside a
 * sequence are ldx apart.
 * t, row_scale: float[B*S] (token b*S + s).  c, col_scale: float[B][I].
 * codes: [B*S][I] (or [B*S][I/2] packed); NULL = count only (then xhat must be NULL and
 *        zero_count non-NULL).  xhat: nullable, binary16 [B*S][I].
 * zero_count: one counter for the whole batch.
 * Limits: B*S and B*I <= CQ_MAX_DIM.
 */
int crossquant_absmax_batched(const void *X, int64_t B, int64_t S, int64_t I, int64_t ldx,
                              int64_t batch_stride, float *t, float *c, void *stream);
int crossquant_quantize_batched(const void *X, int64_t B, int64_t S, int64_t I, int64_t ldx,
                                int64_t batch_stride, const float *t, const float *c, float alpha,
                                int bits, void *codes, void *xhat, float *row_scale, float *col_scale,
                                unsigned long long *zero_count, void *stream);

/*
 * Size of the quantization kernel K(CQ) = {X_ij : CQ(X_ij) = 0} (Definition 1) without writing
 * codes; the kernel proportion of the paper is zero_count / (T*I).  alpha = 1 gives the
 * per-token baseline K(Q) of Eq. 1.
 * row_scale / col_scale: nullable (both or neither): float[T] / float[I], receive a and b when given.
 *        The kernel keeps the factors it needs on chip, so NULL, NULL costs nothing and is the usual form.
 */
int crossquant_kernel_count(const void *X, int64_t T, int64_t I, int64_t ldx, const float *t,
                            const float *c, float alpha, int bits, float *row_scale,
                            float *col_scale, unsigned long long *zero_count, void *stream);

/*
 * Quantization-kernel analysis: the "Remove Kernel" matrix (captions of the zero-shot accuracy
 * figures: the elements of the kernel are set to zero, all others stay in FP16) and the two
 * indicators of Table 1 / the kernel-size analysis (cases I and II).
 *   xrk_ij = q_ij == 0 ? 0 : X_ij          (q as in crossquant_quantize for this alpha, bits)
 *   counters[0] = #{q_ij == 0}             the kernel size Z
 *   counters[1] = #{(i,j): c_j >= t_i}     case II
 *   counters[2] = #{(i,j): B~_ij < B_ij}   B~ = 0.5 fl32(a_i b_j), B = 0.5 fl32(t_i / q_max) (Eq. 1's step)
 * xrk: out, nullable, binary16 [T][I].  counters: out, three unsigned 64-bit values, 8-byte aligned.
 * row_scale / col_scale: nullable (both or neither): float[T] / float[I] work vectors, overwritten with a and
 *        b (must not overlap t or c: CQ_ERR_ALIAS).  With them the factors are formed once, by a small kernel
 *        of their own; with NULL, NULL every block forms the factors of its own rows and columns, which makes
 *        the call about a tenth slower on a 4096 x 8192 matrix.
 */
int crossquant_kernel_analysis(const void *X, int64_t T, int64_t I, int64_t ldx, const float *t,
                               const float *c, float alpha, int bits, void *xrk, float *row_scale,
                               float *col_scale, unsigned long long *counters, void *stream);

/*
 * crossquant_kernel_analysis for callers that cannot allocate device memory and therefore cannot
 * supply the two work vectors: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, outputs and arithmetic, but the scale factors are kept in a
 * static device array of the library (2 x CQ_ANALYSIS_STATIC_MAX floats = 4 MiB, one copy on every
 * device the library runs on, there until the process ends).  The call allocates nothing.
 * Limits: T <= CQ_ANALYSIS_STATIC_MAX and I <= CQ_ANALYSIS_STATIC_MAX, else CQ_ERR_SHAPE with
 * nothing enqueued.  All calls on one device share that device's array: calls that overlap on one
 * device (different streams, or replays of graphs that contain it) race and must be ordered by the
 * caller; calls on one stream are ordered anyway.
 */
#define CQ_ANALYSIS_STATIC_MAX (1 << 19)
int crossquant_kernel_analysis_static(const void *X, int64_t T, int64_t I, int64_t ldx, const float *t,
                                      const float *c, float alpha, int bits, void *xrk,
                                      unsigned long long *counters, void *stream);

/*
 * Expand packed INT4 codes (crossquant_quantize with bits == 4) to int8 codes in [-7, 7], so that
 * A4 activations can feed crossquant_w8a8_linear (gfx950 has no INT4 matrix instruction; weight
 * codes from crossquant_weight_quantize with bits == 4 are already stored one per byte).
 * packed: [T][I/2], even column in the low nibble; I even.  codes: out, int8 [T][I].
 */
int crossquant_unpack_int4(const void *packed, int64_t T, int64_t I, int8_t *codes, void *stream);

/*
 * Per-channel weight quantization (Eq. 2), one step per OUTPUT channel k, stored transposed.
 *   W'_jk = fl32(fold_j * W_jk)  (fold NULL = 1);  s_k = fl32(max_j |W'_jk| / q_max)
 *   qw_kj = s_k == 0 ? 0 : clamp(rne(fl32(W'_jk / s_k)), +-q_max)
 * Passing fold = col_scale (b_j) carries the column factor of the element-wise CrossQuant step
 * into the weights, so that sum_j q_ij qw_kj * a_i * s_k approximates (X W)_ik.
 * W: binary16 [I][O] row-major (the paper's layout).  qw: out, int8 [O][I].  w_scale: out, float[O].
 */
int crossquant_weight_quantize(const void *W, int64_t I, int64_t O, const float *fold, int bits,
                               int8_t *qw, float *w_scale, void *stream);

/*
 * Group-wise weight quantization (Background section: W reshaped to (I*O/g) x g, one step per
 * group).  Every output channel k is cut into groups of `group` consecutive input channels (the
 * contraction axis, as in the weight-only code bases the paper builds on; group = 128 is the
 * paper's W4A8-g128 setting, group = I is crossquant_weight_quantize):
 *   s_{k,G} = fl32(max_{j in G} |W'_jk| / q_max);  qw_kj = clamp(rne(fl32(W'_jk / s_{k, j/group})), +-q_max)
 * W: binary16 [I][O].  I % group == 0.  qw: out, int8 [O][I].  w_scale: out, float [O][I/group].
 * w_dq: out, nullable, binary16 [I][O]: the dequantized (fake-quantized) weights fl16(fl32(q * s)).
 */
int crossquant_weight_quantize_grouped(const void *W, int64_t I, int64_t O, const float *fold,
                                       int64_t group, int bits, int8_t *qw, float *w_scale, void *w_dq,
                                       void *stream);

/*
 * W8A8 linear layer Y = X . W on integer codes (Background section), INT8 MFMA, int32 accumulate.
 *   acc_ik = sum_j qx_ij * qw_kj  (exact);  Y_ik = fl16(fl32(fl32(float(acc_ik) * row_scale_i) * w_scale_k))
 * qx: int8 [T][I].  qw: int8 [O][I] (contraction axis contiguous).  Fast path: qx, qw, Y and
 *     w_scale 16-byte aligned, I % 128 == 0, O % 8 == 0, ldy % 8 == 0 (any T); other layouts take a
 *     slower, fully bounds-checked kernel with identical results.
 * Y: out, binary16 [T][ldy], ldy >= O.  acc_debug: out, nullable, int32 [T][O] raw accumulators.
 * I * 127 * 127 must fit in int32 (I <= 133,000).
 */
int crossquant_w8a8_linear(const int8_t *qx, const float *row_scale, const int8_t *qw,
                           const float *w_scale, int64_t T, int64_t I, int64_t O, void *Y,
                           int64_t ldy, int32_t *acc_debug, void *stream);

/*
 * crossquant_quantize followed by crossquant_w8a8_linear with the quantize step inside the GEMM's
 * activation load (the W8A8 / W4A4 layers of the paper's tables computed from X directly): X goes in,
 * Y comes out, the codes never exist in memory.  Results equal the two calls bit for bit (bits = 4:
 * codes in [-7, 7] on the INT8 matrix instruction, qw as crossquant_weight_quantize(bits = 4) stores
 * them).  t, c, alpha, bits, row_scale, col_scale as in crossquant_quantize (the factors are written
 * first, by a small kernel); qw, w_scale, Y, ldy, acc_debug as in crossquant_w8a8_linear.
 * Every activation element is quantized once per 256 output channels, so this call is SLOWER than the
 * two calls on any layer with more than a few hundred output channels (measured: bench.py's
 * `quantize_inside_gemm`); it exists to put a number on that trade, and for callers that cannot afford
 * the T x I bytes of codes.  Requires I % 128 == 0, ldx % 8 == 0 and 16-byte aligned X, qw, col_scale,
 * else CQ_ERR_UNSUPPORTED.
 */
int crossquant_quantize_linear_fused(const void *X, int64_t T, int64_t I, int64_t ldx, const float *t,
                                     const float *c, float alpha, int bits, const int8_t *qw,
                                     const float *w_scale, int64_t O, void *Y, int64_t ldy, float *row_scale,
                                     float *col_scale, int32_t *acc_debug, void *stream);

/*
 * A4W4 linear layer on the FP6 matrix instruction (the W4A4 setting of the paper's accuracy
 * tables).  gfx950 multiplies 6-bit floats at twice the INT8 rate and every INT4 code in [-7, 7] is
 * exact in FP6 E2M3; with binary32 accumulation the dot product is exact for I <= 2^18, so
 *   acc_ik = sum_j qx_ij * qw_kj ;  Y_ik = fl16(fl32(fl32(float(acc_ik) * row_scale_i) * w_scale_k))
 * equals the integer path (crossquant_unpack_int4 + crossquant_w8a8_linear) bit for bit.
 *
 * crossquant_pack_fp6 rewrites codes into the operand format: fragments of 32 rows x 64 columns,
 *   1536 bytes each, ordered [ceil(R/32)][K/64].  Lane l = row (l & 31), columns [32 (l >> 5), +32),
 *   element j of the lane in bits [6j, 6j+6) of its 192-bit little-endian stream; a fragment is 64
 *   lanes x 16 bytes (bits [0, 128) of each stream) followed by 64 lanes x 8 bytes (bits [128, 192)).
 *   Rows past R are zero.
 *   codes: src_format 8 = int8 [R][K] (e.g. qw of crossquant_weight_quantize with bits = 4),
 *          src_format 4 = packed nibbles [R][K/2] (crossquant_quantize with bits = 4);
 *          values outside [-7, 7] are clamped.  K % 128 == 0 (else CQ_ERR_UNSUPPORTED).
 *   packed: out, crossquant_fp6_packed_bytes(R, K) bytes (-1 for invalid sizes), 16-byte aligned.
 * crossquant_pack_fp6_weights does the same for the weight operand, codes [O][K], whose rows the kernel wants
 *   interleaved four ways: inside every group of 64 output channels, row 16 n + f of the packed matrix holds
 *   channel 4 f + n (n = 0..3, f = 0..15), so that a lane of the matrix kernel ends up with four adjacent
 *   channels of a token and stores them straight from its registers.  The packed matrix has whole groups:
 *   crossquant_fp6_packed_weight_bytes(O, K) = crossquant_fp6_packed_bytes(64 ceil(O / 64), K) bytes; channels
 *   past O are zero rows.  Arguments and errors as for crossquant_pack_fp6.
 * crossquant_quantize_fp6: crossquant_quantize with bits = 4 whose codes leave the kernel already in
 *   this format (no nibble buffer, no packing pass): packed receives crossquant_fp6_packed_bytes(T, I)
 *   bytes; the rows past T of the last row block are left untouched (they only feed outputs that
 *   crossquant_w4a4_linear never stores).  I % 128 == 0 and packed 16-byte aligned, else
 *   CQ_ERR_UNSUPPORTED.  Other arguments as in crossquant_quantize.
 * crossquant_w4a4_linear: qx_fp6 are the packed activations (crossquant_pack_fp6 or crossquant_quantize_fp6,
 *   R = T, K = I), qw_fp6 the packed weights (crossquant_pack_fp6_weights, O channels, K = I).  Y, acc_debug, row_scale, w_scale as in crossquant_w8a8_linear.  Requires
 *   I % 128 == 0, O % 8 == 0, ldy % 8 == 0, ldy < 2^22 and 16-byte aligned pointers, else CQ_ERR_UNSUPPORTED
 *   (the caller then takes the integer path); I <= 2^18.
 */
int64_t crossquant_fp6_packed_bytes(int64_t R, int64_t K);
int64_t crossquant_fp6_packed_weight_bytes(int64_t O, int64_t K);
int crossquant_pack_fp6(const void *codes, int src_format, int64_t R, int64_t K, void *packed, void *stream);
int crossquant_pack_fp6_weights(const void *codes, int src_format, int64_t O, int64_t K, void *packed, void *stream);
int crossquant_quantize_fp6(const void *X, int64_t T, int64_t I, int64_t ldx, const float *t,
                            const float *c, float alpha, void *packed, void *xhat, float *row_scale,
                            float *col_scale, unsigned long long *zero_count, void *stream);
int crossquant_w4a4_linear(const void *qx_fp6, const float *row_scale, const void *qw_fp6,
                           const float *w_scale, int64_t T, int64_t I, int64_t O, void *Y, int64_t ldy,
                           int32_t *acc_debug, void *stream);

/* Human-readable name of a status code (static storage, never NULL). */
const char *crossquant_status_string(int status);

/* Library version, major * 10000 + minor * 100 + patch. */
int crossquant_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CROSSQUANT_H */
