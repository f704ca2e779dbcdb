/*
 * fog.h -- C ABI of the MI355X (gfx950) FP8 hot path of FOG-style training.
 *
 * The library computes what the paper states as the end-to-end FP8 product
 * (Appendix E):
 *
 *     GEMM(X, Y) = 1 / (rho(X) rho(Y)) * FP8GEMM(FP8cast(rho(X) X), FP8cast(rho(Y) Y)),
 *     rho(X)     = FP8MaxValue / (2^m * max H),        H = history of abs-max values,
 *
 * for every GEMM of a transformer block in forward and backward, and for the two
 * products inside attention, P = Softmax(s Q K^T + M) and P V (Appendix B, eq. P;
 * Appendix E, table of FP8 methods: under FP8DPA both run in FP8).  Forward tensors
 * use E4M3, backward tensors E5M2 (Section 2).
 *
 * Conventions (all entry points)
 *   - Every data pointer is a DEVICE pointer.  Scalars that depend on data
 *     (abs-max, scales) also live in device memory, so that just-in-time scaling
 *     needs no host round trip.  Matrices are row-major; ld* are in ELEMENTS.
 *   - The caller owns every buffer.  The library never allocates, frees or keeps a
 *     pointer after the call; scratch memory is passed in as `workspace`, sized by
 *     the fog_*_workspace queries (which are pure host functions).
 *   - Every call only enqueues work on `stream` (a hipStream_t cast to void*; NULL is
 *     the default stream) and returns without synchronising.
 *   - Errors are returned as fog_status; nothing is thrown and nothing aborts.
 *     Argument errors are detected on the host before anything is launched, so a
 *     failing call has no effect on device memory.
 *   - FP8 codes are OCP E4M3 / E5M2 bytes.  The casts (fog_quantize and its variants, the fused
 *     producers) give a NaN input the NaN code 0x7F with the input's sign and saturate infinities; the
 *     abs-max of a tensor that holds a NaN is NaN (and its scale therefore 1).  The GEMM and attention
 *     entry points expect finite operands.
 */
#ifndef FOG_H_
#define FOG_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FOG_OK = 0,
  FOG_ERR_NULL = 1,        /* a required pointer is NULL */
  FOG_ERR_SHAPE = 2,       /* negative size, or a leading dimension smaller than the row */
  FOG_ERR_ALIGN = 3,       /* a pointer or leading dimension breaks the stated alignment */
  FOG_ERR_UNSUPPORTED = 4, /* valid problem the kernels do not cover (stated per call) */
  FOG_ERR_WORKSPACE = 5,   /* workspace missing or smaller than the query says */
  FOG_ERR_HIP = 6          /* the HIP runtime refused a launch */
} fog_status;

typedef enum { FOG_E4M3 = 0, FOG_E5M2 = 1 } fog_fp8;

typedef enum {
  FOG_NT = 0, /* C[M,N] = A[M,K] . B[N,K]^T   forward:      Y  = X~ . W~^T   */
  FOG_NN = 1, /* C[M,N] = A[M,K] . B[K,N]     data grad:    dX = dY~ . W~    */
  FOG_TN = 2  /* C[M,N] = A[K,M]^T . B[K,N]   weight grad:  dW = dY~^T . X~  */
} fog_layout;

const char* fog_status_string(fog_status s);
int fog_version(void);

/*
 * Abs-max of a tensor, max_i |x_i| -- the only statistic per-tensor scaling needs
 * (Appendix E, history update; Appendix C, absmax).
 *   x_bf16 : n bfloat16 values, contiguous, 16-byte aligned.
 *   amax   : one float, overwritten (0 for n == 0).
 * Errors: NULL, n < 0 (SHAPE), misaligned x (ALIGN).
 */
fog_status fog_amax(const void* x_bf16, int64_t n, float* amax, void* stream);

/*
 * Scale from an abs-max (Appendix E): scale = fl32(FP8MaxValue / (2^margin * amax)),
 * FP8MaxValue = 448 (E4M3) or 57344 (E5M2); scale_inv = fl32(1 / scale).
 * scale = 1 when amax is zero or not finite; scale is capped at FLT_MAX.
 *   amax      : one float (for delayed scaling: the maximum of the history).
 *   scale, scale_inv : one float each, overwritten.  scale_inv may be NULL.
 */
fog_status fog_scale(const float* amax, fog_fp8 fmt, int margin, float* scale, float* scale_inv, void* stream);

/*
 * Delayed scaling (Appendix E, history length l = 1024 in the paper's runs): folds the abs-max
 * of the tensor just cast into the history, H <- {new_amax} U {h_t}_{t>=2} (the history is kept
 * newest first; the oldest entry, the last, falls out), then writes
 * scale = fl32(FP8MaxValue / (2^margin * max H)) and scale_inv for the NEXT iteration's cast.
 * One small kernel, no host round trip.
 *   history : len >= 1 floats, updated in place;  new_amax : one float;  scale_inv may be NULL.
 */
fog_status fog_scale_delayed(float* history, int len, const float* new_amax, fog_fp8 fmt, int margin,
                             float* scale, float* scale_inv, void* stream);

/*
 * FP8cast(scale * X) (Appendix E), optionally also laid out transposed so that the
 * weight-gradient and data-gradient products find their contraction index contiguous:
 *     q[r, c] = sat_rne_fmt( fl32( float(x[r, c]) * scale ) ),      qT[c, r] = q[r, c].
 * The product is rounded to binary32 once, then to FP8 with round-to-nearest-even,
 * saturating at +-FP8MaxValue.
 *   x_bf16 : [rows, cols], leading dimension ldx.
 *   scale  : one float (from fog_scale, or from a history under delayed scaling).
 *   q      : [rows, cols] bytes, leading dimension ldq.   May be NULL if qT is given.
 *   qT     : [cols, rows] bytes, leading dimension ldqT, or NULL.
 *   amax_out : NULL, or one float that receives max |x| in the same pass (the single-pass
 *              flow of delayed scaling, Section 2).  Overwritten.
 * The fast path needs cols % 16 == 0 (rows % 16 == 0 too when qT is given), 16-byte aligned
 * pointers and leading dimensions that are multiples of 16; other shapes take a slower
 * general kernel with identical results.
 * Errors: NULL scale, NULL x or both outputs NULL for a non-empty input, negative sizes or
 * ld < row length (SHAPE).
 */
fog_status fog_quantize(const void* x_bf16, int64_t rows, int64_t cols, int64_t ldx, fog_fp8 fmt,
                        const float* scale, uint8_t* q, int64_t ldq, uint8_t* qT, int64_t ldqT,
                        float* amax_out, void* stream);

/*
 * Just-in-time scaling in one call (Section 2: abs-max of the tensor being cast, then the cast;
 * Appendix E for the scale): the same results, bit for bit, as fog_amax -> fog_scale -> fog_quantize,
 * in two launches instead of four and without atomics: every workgroup of the abs-max pass leaves
 * its maximum in its own word of the workspace; every workgroup of the cast pass, which follows on
 * the same stream, reduces those words (4 KB at most) and derives the scale itself, and the first
 * one publishes abs-max, scale and 1/scale.
 *   amax, scale : one float each, overwritten.   scale_inv : one float or NULL.
 *   q, qT, x_bf16, leading dimensions, fmt : as in fog_quantize.   margin : as in fog_scale.
 *   workspace : fog_quantize_jit_workspace() bytes (4 KB), 4-byte aligned, owned by the caller; its
 *               contents on entry do not matter.  Calls that may overlap in time (different
 *               streams) need a workspace each.
 * Errors: as fog_quantize and fog_scale; WORKSPACE when the workspace is too small.
 */
fog_status fog_quantize_jit(const void* x_bf16, int64_t rows, int64_t cols, int64_t ldx, fog_fp8 fmt, int margin,
                            uint8_t* q, int64_t ldq, uint8_t* qT, int64_t ldqT,
                            float* amax, float* scale, float* scale_inv,
                            void* workspace, size_t workspace_bytes, void* stream);
size_t fog_quantize_jit_workspace(void);

/*
 * fog_quantize_jit for up to FOG_CAST_BATCH_MAX tensors in two launches (one abs-max pass over all of them,
 * one cast pass over all of them) instead of two per tensor: a launch costs a few microseconds of ramp and
 * tail whatever it does, which is a fifth of either pass over a 100 MB tensor.  Results are those of
 * fog_quantize_jit on each job, bit for bit.
 *   jobs   : HOST array of `count` (0..FOG_CAST_BATCH_MAX) descriptions; the device buffers they name follow the rules
 *            of fog_quantize_jit, restricted to what the fast kernels cover: x_bf16 [rows, cols]
 *            contiguous (leading dimension cols) and 16-byte aligned, rows * cols a positive multiple of
 *            16, q contiguous and 16-byte aligned, no transposed copy.
 *   workspace : fog_quantize_jit_batch_workspace(count) bytes (4 KB per job), 4-byte aligned; contents on
 *            entry do not matter.
 * Errors: NULL, SHAPE (count outside 0..FOG_CAST_BATCH_MAX, non-positive sizes, margin), ALIGN, WORKSPACE, UNSUPPORTED
 * (format; rows * cols not a multiple of 16: use fog_quantize_jit for that tensor).
 */
#define FOG_CAST_BATCH_MAX 32
typedef struct {
  const void* x_bf16;
  int64_t rows, cols;
  fog_fp8 fmt;
  int margin;
  uint8_t* q;
  float* amax;
  float* scale;
  float* scale_inv;   /* may be NULL */
} fog_cast_job;
fog_status fog_quantize_jit_batch(const fog_cast_job* jobs, int count, void* workspace, size_t workspace_bytes, void* stream);
size_t fog_quantize_jit_batch_workspace(int count);

/*
 * Delayed scaling in ONE launch per cast (Appendix E: the scale of a cast comes from the maximum of
 * the last history_len abs-maxes of the same tensor; Section 2: one pass over the data, against two
 * for just-in-time scaling).  Call number `step` (0, 1, 2, ... for one tensor, no gaps):
 *     a_prev  = abs-max of the tensor cast by call step - 1   (0 for step 0)
 *     history[step mod history_len] = a_prev                   (the oldest entry is replaced)
 *     scale   = FP8MAX / (2^margin * max(history)),  scale_inv = 1 / scale     (rules of fog_scale)
 *     q, qT   = casts of x with that scale                     (as fog_quantize)
 * and the abs-max of x is left in `state` for call step + 1.  Same results, bit for bit, as
 * fog_scale_delayed followed by fog_quantize(..., amax_out), without their two small launches; the
 * history is a ring here (entry step mod history_len is the one replaced) where fog_scale_delayed
 * shifts it, which leaves its maximum, the only thing used, the same.
 *   history : history_len floats, caller-initialised (zeros: scale 1 until an abs-max exists).
 *   state   : fog_quantize_delayed_state() bytes (12 KB), 4-byte aligned, owned by the caller, ALL ZERO
 *             before step 0 and untouched by the caller afterwards; one per tensor.
 *   amax_prev : NULL or one float, receives a_prev.   scale : one float.   scale_inv : one float or NULL.
 *   x_bf16, q, qT, leading dimensions, fmt : as in fog_quantize.   margin : as in fog_scale.
 * An empty tensor advances the history with abs-max 0.  fog_delayed_amax reads the abs-max that call
 * `step` left in the state (for a checkpoint of the scaling state, or after the last step).
 * Errors: as fog_quantize and fog_scale; WORKSPACE when the state is too small; SHAPE for step < 0 or
 * history_len < 1.
 */
fog_status fog_quantize_delayed(const void* x_bf16, int64_t rows, int64_t cols, int64_t ldx, fog_fp8 fmt, int margin,
                                float* history, int history_len, int64_t step, void* state, size_t state_bytes,
                                uint8_t* q, int64_t ldq, uint8_t* qT, int64_t ldqT,
                                float* amax_prev, float* scale, float* scale_inv, void* stream);
size_t fog_quantize_delayed_state(void);
fog_status fog_delayed_amax(const void* state, int64_t step, float* amax, void* stream);

/*
 * fog_quantize_delayed for up to FOG_CAST_BATCH_MAX tensors in ONE launch (a launch costs about 4 us of ramp and tail
 * whatever it does; the casts of a layer's tensors are independent of each other).  Same results, bit for bit, as the
 * calls one by one with the same `step`.  A job describes a dense row-major tensor (ldx = ldq = cols, no transposed
 * copy) of rows * cols elements, a multiple of 16, at 16-byte aligned x_bf16 and q; history, state, amax_prev, scale and
 * scale_inv are as in fog_quantize_delayed and belong to that tensor alone (no two jobs may share any of them).
 *   jobs : HOST array of `count` (0..FOG_CAST_BATCH_MAX) descriptions, read before the call returns.
 *   step : the call number, the same for every job of the batch (tensors cast once per training step).
 * Errors: NULL, SHAPE (count, non-positive sizes, history_len < 1, step < 0, margin), ALIGN, WORKSPACE (a state too
 * small), UNSUPPORTED (a format, or a size that is not a multiple of 16: cast that tensor with fog_quantize_delayed).
 */
typedef struct {
  const void* x_bf16;
  int64_t rows, cols;
  fog_fp8 fmt;
  int margin;
  float* history;
  int history_len;
  void* state;
  size_t state_bytes;
  uint8_t* q;
  float* amax_prev;   /* may be NULL */
  float* scale;
  float* scale_inv;   /* may be NULL */
} fog_delayed_job;
fog_status fog_quantize_delayed_batch(const fog_delayed_job* jobs, int count, int64_t step, void* stream);

/*
 * QK RMS normalisation with a frozen gain, fused with the FP8 cast (Section 3: N_gamma(x) =
 * gamma x / rms(x), rms(x) = ||x||_2 / sqrt(D), applied to every query / key vector; the FOG
 * variants freeze the gains and Appendix A folds their value into the softmax scale, which
 * leaves one scalar).  Per row x of the matrix (one head of one token):
 *     y = gain * x / rms(x)   (binary32; a row of zeros gives zeros: the formula has no epsilon)
 *     q = sat_rne_fmt( fl32( y * scale ) ),      amax_out = max |y| over the matrix.
 * The scale is the caller's (delayed scaling: from the history that amax_out feeds; |y| never
 * exceeds gain * sqrt(cols), so FP8MaxValue / (gain * sqrt(cols)) is a scale that cannot saturate).
 * y is never stored, so a code is a rounding decision on a binary32 value whose last bits depend
 * on the summation order: codes agree with a float64 evaluation except where rho * y lies within
 * about 2^-21 (relative) of a rounding boundary.
 *   x_bf16 : [rows, cols] bfloat16, leading dimension ldx.   q : [rows, cols] bytes, leading dimension ldq.
 *   gain   : > 0 and finite.   amax_out : NULL or one float, overwritten.
 * Fast paths: cols in {64, 128, 256, 512} with x 16-byte and q 8-byte aligned, ldx and ldq multiples
 * of 8; every other shape takes a one-wave-per-row kernel.
 * Errors: NULL, SHAPE, ALIGN (odd x), UNSUPPORTED (format, gain).
 */
fog_status fog_rmsnorm_quantize(const void* x_bf16, int64_t rows, int64_t cols, int64_t ldx, float gain, fog_fp8 fmt,
                                const float* scale, uint8_t* q, int64_t ldq, float* amax_out, void* stream);

/*
 * xIELU activation fused with the FP8 cast (Appendix B, equation xIELU: the activation of the
 * FOG-max variant, between the two GEMMs of the feed-forward block):
 *     y = alpha_p x^2 + 0.5 x                       for x > 0
 *     y = alpha_n (e^x - 1) - alpha_n x + 0.5 x     for x <= 0        (binary32; e^x - 1 by expm1)
 *     q = sat_rne_fmt( fl32( y * scale ) ),         amax_out = max |y| over the matrix.
 * The scale is the caller's (delayed scaling, fed by amax_out).  y is never stored, so a code is a
 * rounding decision on a binary32 value: codes agree with a float64 evaluation except where
 * scale * y lies within about 2^-20 (relative) of a rounding boundary.
 *   x_bf16 : [rows, cols] bfloat16, leading dimension ldx.   q : [rows, cols] bytes, leading dimension ldq.
 *   alpha_p, alpha_n : >= 0 and finite (the layer's two scalars as plain numbers).
 *   amax_out : NULL or one float, overwritten.
 * Fast path: cols, ldx, ldq multiples of 16 and 16-byte aligned pointers; other shapes take an
 * element-wise kernel with the same arithmetic.
 * Errors: NULL, SHAPE, ALIGN (odd x), UNSUPPORTED (format, negative or non-finite alpha).
 */
fog_status fog_xielu_quantize(const void* x_bf16, int64_t rows, int64_t cols, int64_t ldx, float alpha_p, float alpha_n,
                              fog_fp8 fmt, const float* scale, uint8_t* q, int64_t ldq, float* amax_out, void* stream);

/*
 * GeLU fused with the FP8 cast (Section 3, architecture table: the activation of two of the FOG
 * variants, between the two GEMMs of the feed-forward block).  The paper names GeLU without a
 * formula; it is taken as the exact form
 *     y = x Phi(x) = 0.5 x erfc(-x / sqrt 2)        (binary32)
 *     q = sat_rne_fmt( fl32( y * scale ) ),         amax_out = max |y| over the matrix.
 * Arguments, fast path and errors as for fog_xielu_quantize (no activation parameters).  Codes agree
 * with a float64 evaluation except where scale * y lies within about 2^-19 + x^2 2^-23 (relative,
 * the second term for x < 0 only) of a rounding boundary.
 */
fog_status fog_gelu_quantize(const void* x_bf16, int64_t rows, int64_t cols, int64_t ldx, fog_fp8 fmt, const float* scale,
                             uint8_t* q, int64_t ldq, float* amax_out, void* stream);

/*
 * tanh_alpha fused with the FP8 cast (Section 3: tanh(alpha x) applied element-wise to queries and
 * keys, the entropy regulariser of the FOG-flash variant, in place of the QK RMSNorm):
 *     y = tanh(alpha * x)                           (binary32)
 *     q = sat_rne_fmt( fl32( y * scale ) ),         amax_out = max |y| over the matrix.
 * |y| <= 1, so a caller may use the constant scale FP8MAX and skip the abs-max altogether.
 *   alpha : finite (the layer's trainable scalar as a plain number).
 * Other arguments, fast path and errors as for fog_xielu_quantize; codes agree with a float64
 * evaluation except where scale * y lies within about 2^-19 (relative) of a rounding boundary.
 */
fog_status fog_tanh_quantize(const void* x_bf16, int64_t rows, int64_t cols, int64_t ldx, float alpha, fog_fp8 fmt,
                             const float* scale, uint8_t* q, int64_t ldq, float* amax_out, void* stream);

/*
 * Post-RMSNorm with its residual connection, fused with the FP8 cast of the result (Section 3: every
 * sub-layer output y passes N_gamma(y) = gamma (.) y / rms(y), rms(y) = ||y||_2 / sqrt(cols), with a
 * trainable gains vector, before it is added to the residual stream x; the block has no
 * pre-normalisation, so the sum is the next GEMM's input and is cast as in Appendix E):
 *     xnew = bf16( x + gamma (.) y / rms(y) )       (binary32 evaluation, one rounding to bfloat16;
 *                                                    a zero vector y adds nothing: no epsilon)
 *     q    = sat_rne_fmt( fl32( xnew * scale ) )    (the cast of the STORED bfloat16 value: bit-exact
 *                                                    given xnew)
 *     amax_out = max |xnew| over the matrix         (bit-exact given xnew)
 *   x_bf16, y_bf16 : [rows, cols] bfloat16, leading dimensions ldx, ldy.
 *   gamma  : [cols] floats.        scale : one float (delayed scaling, fed by amax_out).
 *   xnew_bf16 : [rows, cols] bfloat16, leading dimension ldo; may be the same buffer as x_bf16 with the
 *            same leading dimension (residual stream updated in place), must not overlap anything else.
 *   q      : NULL (only the residual update and the abs-max) or [rows, cols] bytes, leading dimension ldq.
 *   amax_out : NULL or one float, overwritten.
 * xnew agrees with a float64 evaluation except where the exact sum lies within about
 * 2^-20 |N(y)| + 2^-23 |xnew| of a bfloat16 rounding boundary.
 * Fast path (one wave per row, every element read once): cols a multiple of 512 up to 8192, x, y, xnew
 * and gamma 16-byte aligned, q 8-byte aligned, leading dimensions multiples of 8; other shapes take a
 * one-wave-per-row kernel that reads y twice.
 * Errors: NULL, SHAPE, ALIGN (odd bf16 addresses, gamma not 4-byte aligned), UNSUPPORTED (format).
 */
fog_status fog_postnorm_residual_quantize(const void* x_bf16, int64_t ldx, const void* y_bf16, int64_t ldy, int64_t rows,
                                          int64_t cols, const float* gamma, fog_fp8 fmt, const float* scale, void* xnew_bf16,
                                          int64_t ldo, uint8_t* q, int64_t ldq, float* amax_out, void* stream);

/*
 * Activation kurtosis, the paper's outlier diagnostic (Section 4): for each token vector x (a row),
 * kurt(x) = mu[x^4] / (mu[x^2])^2 (element-wise powers, x not centred); the result is the mean over
 * the rows.  The denominator is read as the squared un-centred second moment (1 for a constant
 * vector, cols for a one-hot vector, 3 for Gaussian data).  Rows of zeros contribute 0.
 *   x_bf16 : [rows, cols] bfloat16, leading dimension ldx; one pass, binary32 sums.
 *   kurt   : one float, overwritten.  Rows are summed with float atomics: the last bits may vary
 *            from run to run.
 *   amax_out : NULL or one float, overwritten with max |x| over the matrix, bit-exact (Appendix E:
 *            the entry this tensor adds to the scaling history), so that the monitor and the
 *            delayed-scaling abs-max share one read of the activations.
 * The fast path needs a 16-byte aligned x and cols, ldx multiples of 8; other shapes take a scalar path.
 * Errors: NULL, negative sizes or ldx < cols (SHAPE), odd address (ALIGN).
 */
fog_status fog_kurtosis(const void* x_bf16, int64_t rows, int64_t cols, int64_t ldx, float* kurt, float* amax_out, void* stream);

/*
 * Scaled FP8 product (Appendix E): C = scale_inv_A * scale_inv_B * (decode(A) x decode(B)) in
 * the given layout, FP8 products accumulated in binary32, result rounded once to bfloat16.
 *   A, B   : FP8 codes (fmtA / fmtB may differ: E5M2 gradients times E4M3 weights), lda / ldb.
 *   scale_inv_A / _B : one float each (the reciprocal scales of the casts).
 *   C_bf16 : [M, N] bfloat16, leading dimension ldc.
 *   workspace : NULL, or fog_fp8_gemm_workspace(layout, M, N, K) bytes, 16-byte aligned.  The query returns 0
 *            for most shapes.  For products with fewer output tiles (256 x 256) than the GPU has compute
 *            units and a long contraction (the weight gradient of a small projection over many tokens) it
 *            returns room for binary32 partial tiles: the call then cuts the contraction into chunks that
 *            run side by side and adds them in a fixed order in a second kernel (deterministic; against the
 *            unsplit kernel only the order of binary32 additions differs).  Without a workspace, or with a
 *            smaller one, the unsplit kernel runs: never an error.
 * Requirements: A, B 16-byte aligned, lda, ldb multiples of 16; C 2-byte aligned, any ldc >= N (a
 * 16-byte aligned C with ldc a multiple of 8 takes 16-byte stores, anything else element-wise ones);
 * the contiguous dimension of each operand a multiple of 16 (K for row-major-in-K operands,
 * M or N for the K-major operands of NN / TN).  M, N, K otherwise arbitrary; M == 0 or N == 0
 * is a no-op and K == 0 writes zeros.
 * Errors: NULL, SHAPE, ALIGN, UNSUPPORTED (a multiple-of-16 rule above broken).
 */
fog_status fog_fp8_gemm(fog_layout layout, int64_t M, int64_t N, int64_t K,
                        const uint8_t* A, fog_fp8 fmtA, int64_t lda, const float* scale_inv_A,
                        const uint8_t* B, fog_fp8 fmtB, int64_t ldb, const float* scale_inv_B,
                        void* C_bf16, int64_t ldc, void* workspace, size_t workspace_bytes, void* stream);
size_t fog_fp8_gemm_workspace(fog_layout layout, int64_t M, int64_t N, int64_t K);

/*
 * FP8 dot-product attention forward (Appendix B, eq. P; Appendix E, FP8DPA row):
 *     O = Softmax(s Q K^T + M) V   per (batch, head), M the causal mask when causal != 0,
 * with Q~, K~, V~ in E4M3 and the probabilities cast to E4M3 for the P V product.
 * Steps, in the log2 domain: x = s log2(e) sinv_q sinv_k (Q~ K~^T); row reference
 * m_i = ceil(max_j x_ij) (an integer, so that the cast of p is independent of the order in
 * which keys are visited); p = 2^(x - m_i); l_i = sum_j p_ij (binary32, p not cast);
 * P~ = sat_rne_E4M3(scale_p * p);  O = sinv_v (P~ V~) / (scale_p l_i);  lse_i = m_i + log2 l_i.
 * Grouped-query attention (Appendix B; the paper's models use 4 to 8 query groups): H_kv key/value
 * heads serve H query heads, query head h reading key/value head h / (H / H_kv); H_kv == H is
 * ordinary multi-head attention.
 *   Q       : [B, H, S, D] contiguous E4M3 bytes;  D must be 128, S a multiple of 64 (any length
 *             whose head, S * D bytes, stays below 2^31).
 *   K, V    : [B, H_kv, S, D] contiguous E4M3 bytes;  H must be a multiple of H_kv.
 *   sinv_* : reciprocal scales of the casts, one float each.  scale_p: one float; p <= 1, so the
 *            paper's formula gives 448, and a larger value is used as 448 (it could only saturate,
 *            and against the running row reference of an online softmax which entries saturate
 *            would depend on the order in which key blocks are visited).
 *   O_bf16 : [B, H, S, D] bfloat16;  lse : [B, H, S] floats (log2 domain).
 *   amax_p : NULL or one float receiving max p (for a delayed scale_p).  Overwritten.
 * Errors: NULL, SHAPE (negative sizes, H not a multiple of H_kv), ALIGN (16 bytes), UNSUPPORTED
 * (D != 128, S % 64 != 0).
 */
fog_status fog_fp8_attn_fwd(int B, int H, int H_kv, int S, int D, float softmax_scale, int causal,
                            const uint8_t* Q, const uint8_t* K, const uint8_t* V,
                            const float* sinv_q, const float* sinv_k, const float* sinv_v, const float* scale_p,
                            void* O_bf16, float* lse, float* amax_p,
                            void* workspace, size_t workspace_bytes, void* stream);

/*
 * FP8 attention backward: the gradient of the forward above with all five products in FP8
 * (Section 2: E5M2 for backward tensors).  Per (batch, head):
 *     D_i  = sum_d dO_id O_id                      (from the bf16 tensors, binary32)
 *     P    = 2^(x - lse_i);  P~ = sat_rne_E4M3(scale_p P)
 *     dV   = sinv_do / scale_p  * (P~^T dO~)
 *     dP   = sinv_do sinv_v     * (dO~ V~^T)
 *     dS   = P o (dP - D_i);    dS~ = sat_rne_E5M2(scale_ds dS)
 *     dQ   = s sinv_k / scale_ds * (dS~ K~),   dK = s sinv_q / scale_ds * (dS~^T Q~)
 *   dO_e5m2 : dO cast to E5M2 with reciprocal scale sinv_do;  dO_bf16, O_bf16: the bf16 tensors.
 *   lse : from the forward.  scale_ds : one float (delayed-style: amax_ds of a previous call).
 *   dQ : [B, H, S, D], dK, dV : [B, H_kv, S, D] bfloat16, overwritten; under grouped-query attention
 *        dK and dV of a key/value head are the sums over its H / H_kv query heads, accumulated
 *        in binary32 and rounded once.   amax_ds : NULL or one float, max |dS|.
 *   workspace : fog_fp8_attn_workspace(B, H, H_kv, S, D, 1) bytes (three floats per row: D_i and two
 *               per-row constants with the scales folded in), 4-byte aligned.
 * Same shape rules and errors as the forward; WORKSPACE when the workspace is too small.
 */
fog_status fog_fp8_attn_bwd(int B, int H, int H_kv, int S, int D, float softmax_scale, int causal,
                            const uint8_t* Q, const uint8_t* K, const uint8_t* V,
                            const float* sinv_q, const float* sinv_k, const float* sinv_v,
                            const void* O_bf16, const void* dO_bf16, const uint8_t* dO_e5m2, const float* sinv_do,
                            const float* lse, const float* scale_p, const float* scale_ds,
                            void* dQ_bf16, void* dK_bf16, void* dV_bf16, float* amax_ds,
                            void* workspace, size_t workspace_bytes, void* stream);
size_t fog_fp8_attn_workspace(int B, int H, int H_kv, int S, int D, int is_bwd);

/*
 * fog_fp8_attn_bwd for callers that cannot allocate device memory or pass a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation): the same kernels and the same
 * results, bit for bit, with the per-row constants (three floats per query row) kept in a device array
 * that is part of the library instead of a caller workspace.  The call allocates nothing.
 *   Limit: B * H * S <= FOG_ATTN_BWD_STATIC_MAX_ROWS (the array is 6 MB per GPU the library is used on and
 *   stays until the process ends); a larger problem returns FOG_ERR_WORKSPACE and takes fog_fp8_attn_bwd.
 *   All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (different
 *   streams) race; serialise them or use fog_fp8_attn_bwd with a workspace each.  Nothing in the array has
 *   to survive between calls and nothing has to be cleared (every call first overwrites what it reads).
 * Arguments, shape rules and other errors as fog_fp8_attn_bwd.
 */
#define FOG_ATTN_BWD_STATIC_MAX_ROWS 524288
fog_status fog_fp8_attn_bwd_static(int B, int H, int H_kv, int S, int D, float softmax_scale, int causal,
                                   const uint8_t* Q, const uint8_t* K, const uint8_t* V,
                                   const float* sinv_q, const float* sinv_k, const float* sinv_v,
                                   const void* O_bf16, const void* dO_bf16, const uint8_t* dO_e5m2, const float* sinv_do,
                                   const float* lse, const float* scale_p, const float* scale_ds,
                                   void* dQ_bf16, void* dK_bf16, void* dV_bf16, float* amax_ds, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FOG_H_ */
