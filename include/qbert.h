/*
 * qbert.h -- C ABI of the MI355X (gfx950) library for the group-wise k-bit quantized linear
 * layer of Q-BERT (arXiv 1909.05840).
 *
 * Notation: T tokens (rows of X), K input features, N output neurons, W[N,K] row-major
 * (one row per output neuron), G groups, k = bits, L = 2^k - 1.
 *
 * Conventions that hold for every entry point unless its comment says otherwise
 *   - Pointers are DEVICE pointers into memory the caller owns; the library allocates nothing,
 *     keeps no state between calls and is re-entrant.  Base pointers must be 16-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls only enqueue
 *     kernels on it: they never synchronise, never use another stream, and may be captured
 *     into a HIP graph.
 *   - Arguments are validated on the host before anything is launched: on QB_ERR_NULL, _BITS, _SHAPE,
 *     _CLIP and _WORKSPACE nothing has been enqueued and no output has been written.  QB_ERR_HIP is the
 *     one status that can come after work was enqueued: it reports that the runtime refused a launch of
 *     the call (earlier launches of the same call may already be in the stream; the outputs are then
 *     undefined), or, for qb_power_iteration, that the caller's callback failed (see there).
 *   - Inputs must be finite (activations may be +-inf, which the clamp removes; NaN is not
 *     allowed).  Faults on the device are not detected.
 *   - Matrices are dense row-major.  K must be a multiple of QB_K_ALIGN.
 */
#ifndef QBERT_H
#define QBERT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QB_K_ALIGN 64          /* K (and the embedding dimension d) must be a multiple of this */
#define QB_N_BLOCK 32          /* packed weights are stored in blocks of this many rows      */
#define QB_MAX_K 32768         /* keeps |A4| <= 255^2 * K inside int32                       */

typedef enum {
    QB_OK = 0,
    QB_ERR_NULL = 1,       /* a required pointer is NULL                                     */
    QB_ERR_BITS = 2,       /* bits not in {2,3,4,8}                                           */
    QB_ERR_SHAPE = 3,      /* non-positive dim, K % QB_K_ALIGN != 0, K > QB_MAX_K, N % G != 0  */
    QB_ERR_CLIP = 4,       /* activation range not a positive finite number                  */
    QB_ERR_WORKSPACE = 5,  /* workspace NULL or misaligned although the call needs one       */
    QB_ERR_HIP = 6         /* the HIP runtime refused a launch (its error state is cleared) */
} qb_status;

/* Host, pure.  Static string for a status. */
const char *qb_status_string(qb_status s);

/* Host, pure.  Bytes of the packed weight buffer of an N x K matrix at `bits` bits:
 * ceil(N / QB_N_BLOCK) * QB_N_BLOCK * K * bits / 8, i.e. exactly N*K*bits/8 (the size
 * arithmetic behind the paper's Table 1) whenever N is a multiple of QB_N_BLOCK.  Returns 0
 * for invalid arguments.  The layout inside the buffer is private to the library
 * (qb_unpack_codes gives the codes back in row-major order). */
size_t qb_packed_nbytes(int64_t N, int64_t K, int bits);

/* Host, pure.  Bytes of scratch that qb_qlinear_bwd_ste and its _masked and _asym variants need for
 * the given shape (of the other calls only qb_power_iteration takes scratch, sized by
 * qb_power_iteration_scratch_floats).  Returns 0 for invalid arguments. */
size_t qb_bwd_workspace_nbytes(int64_t T, int64_t N, int64_t K);

/* Host, pure.  The same question for any entry point: bytes of caller-provided scratch that operation `op`
 * needs for the given shape and bit-width (arguments an operation does not depend on are ignored).  Only the
 * backward calls (qb_qlinear_bwd_ste and its _masked / _asym variants: qb_bwd_workspace_nbytes) and
 * qb_power_iteration (qb_power_iteration_scratch_floats() floats) take scratch; every other operation
 * returns 0, as do invalid arguments. */
enum {
    QB_OP_QUANTIZE_GROUPWISE = 0,
    QB_OP_QUANTIZE_ACT = 1,
    QB_OP_QLINEAR_FWD = 2,
    QB_OP_QLINEAR_BWD_STE = 3,
    QB_OP_EMBEDDING = 4,
    QB_OP_POWER_ITERATION = 5
};
size_t qb_workspace_nbytes(int op, int64_t T, int64_t N, int64_t K, int bits);

/*
 * Group-wise symmetric uniform weight quantization and packing.
 * Paper: Sec. 3.3 (consecutive output neurons share one quantization range; 12 heads x
 * sub-groups of 6 neurons = 128 groups per matrix, Fig. 3) and App. "Detailed quantization
 * process" (X' = Clamp(X, q0, q_{2^k-1}); X^I = round((X' - q0)/Delta);
 * Delta = (q_{2^k-1} - q0)/(2^k - 1)), with the range of group g taken as [-m_g, +m_g],
 * m_g = max |w| over rows [g*N/G, (g+1)*N/G), and round = round-half-to-even.
 *   W       in   [N,K] fp32
 *   packed  out  qb_packed_nbytes(N,K,bits) bytes: the codes u in 0..L
 *   h       out  [G] fp32, h_g = m_g / L (half of Delta); Q(w) = h_g * (2u - L)
 *   m       out  [G] fp32, m_g
 *   rs_w    out  [N] int32, sum over the row of (u - 2^(k-1))
 * An all-zero group gets m = h = 0 and codes 0.  Requires N % groups == 0.
 */
qb_status qb_quantize_groupwise(const float *W, int64_t N, int64_t K, int bits, int groups,
                                void *packed, float *h, float *m, int32_t *rs_w, void *stream);

/*
 * The same operation for several matrices in as few launches as possible (quantization-aware
 * fine-tuning re-quantizes every matrix of the model from its fp32 master copy each step, each
 * layer at its own bit-width: Sec. 3.2 mixed precision, Tables 6 and 7).  `jobs` is a HOST array of
 * n_jobs descriptors whose pointer fields are DEVICE pointers with the meaning of the arguments
 * of qb_quantize_groupwise; the array is read during the call only.  Jobs must not overlap in
 * their outputs.  All jobs are validated before anything is launched.
 */
#define QB_MAX_BATCH 16        /* jobs per launch of the activation and forward batches (the weight quantizer
                                  takes 48); longer lists are split into several launches */
typedef struct {
    const float *W;
    int64_t N, K;
    int bits, groups;
    void *packed;
    float *h, *m;
    int32_t *rs_w;
} qb_quant_job;
qb_status qb_quantize_groupwise_batched(const qb_quant_job *jobs, int n_jobs, void *stream);

/*
 * qb_quantize_groupwise with the range of every group given by the caller instead of taken as
 * the max-abs (App.: the range [q0, q_{2^k-1}] may be a sub-interval of the tensor's range,
 * X' = Clamp(X, q0, q_{2^k-1})): [-m_in[g], +m_in[g]], e.g. a percentile; weights outside are
 * clamped and get the end codes.  m_in = the max-abs gives the codes of qb_quantize_groupwise.
 *   m_in  in  [G] fp32, >= 0 and finite (not checked on the device)
 * The packed result feeds qb_qlinear_fwd and qb_qlinear_bwd_ste unchanged (the backward passes the
 * gradient through the clamp as well: plain straight-through; qb_qlinear_bwd_ste_masked does not).
 */
qb_status qb_quantize_groupwise_clip(const float *W, int64_t N, int64_t K, int bits, int groups,
                                     const float *m_in, void *packed, float *h, int32_t *rs_w,
                                     void *stream);

/*
 * 8-bit activation quantization (Table 1 caption: all models use 8-bit activations; same
 * appendix formulas with k = 8 and the caller-given range [-clip, +clip]).
 *   X     in   [T,K] fp32
 *   Xq    out  [T,K] int8, the code minus 128 (u in 0..255); Q(x) = h_x * (2*Xq + 1),
 *              h_x = clip / 255 evaluated in fp32
 *   rs_x  out  [T] int32, sum over the row of Xq
 */
qb_status qb_quantize_act(const float *X, int64_t T, int64_t K, float clip,
                          int8_t *Xq, int32_t *rs_x, void *stream);

/*
 * qb_quantize_act for several tensors in one launch (the inputs of a layer's linears; Table 1 caption: every
 * matrix product takes 8-bit activations).  `jobs` is a HOST array of n_jobs descriptors whose pointer fields are
 * DEVICE pointers with the meaning of the arguments of qb_quantize_act; it is read during the call only.  Jobs
 * must not overlap in their outputs.  All jobs are validated before anything is launched; the sum of the T must
 * not exceed 2^30.
 */
typedef struct {
    const float *X;
    int64_t T, K;
    float clip;
    int8_t *Xq;
    int32_t *rs_x;
} qb_act_job;
qb_status qb_quantize_act_batched(const qb_act_job *jobs, int n_jobs, void *stream);

/*
 * Forward of the quantized linear layer (App., last paragraph: integer matrix product on the
 * codes followed by one de-quantization).  With x' = Xq and c' = u - 2^(k-1),
 *   acc[t,n] = sum_j x'[t,j] * c'[n,j]                       (int8 x int8 -> int32)
 *   A4[t,n]  = 4*acc + 2*rs_x[t] + 2*rs_w[n] + K  = sum_j (2x'+1)(2c'+1)
 *   Y[t,n]   = (h_x * h_{g(n)}) * float(A4[t,n])  (+ bias[n])
 * which is sum_j Q(x)[t,j] * Q(w)[n,j] with the sum taken exactly.
 *   Xq, rs_x            from qb_quantize_act with the same clip
 *   packed, h, rs_w     from qb_quantize_groupwise with the same N, K, bits, groups
 *   bias      in   [N] fp32 or NULL
 *   Y         out  [T,N] fp32
 *   A4_debug  out  [T,N] int32 or NULL: the exact integer, for bit-exact checks
 */
qb_status qb_qlinear_fwd(const int8_t *Xq, const int32_t *rs_x, float clip,
                         const void *packed, const float *h, const int32_t *rs_w,
                         int bits, int groups, int64_t T, int64_t N, int64_t K,
                         const float *bias, float *Y, int32_t *A4_debug, void *stream);

/*
 * qb_qlinear_fwd for several independent linear layers in as few launches as possible (the linears of
 * different layers or micro-batches of a model: Sec. 3.2, every layer at its own bit-width).  `jobs` is a
 * HOST array of n_jobs descriptors whose pointer fields are DEVICE pointers with the meaning of the
 * arguments of qb_qlinear_fwd (no A4_debug output); it is read during the call only.  The jobs must
 * not depend on each other: no job's Y may be another job's input or output.  Jobs of one bit-width
 * whose size makes a launch's fixed cost matter share launches (their tiles are walked as one
 * sequence by one persistent grid); the results are those of separate qb_qlinear_fwd calls, bit for
 * bit.  All jobs are validated before anything is launched.
 */
typedef struct {
    const int8_t *Xq;
    const int32_t *rs_x;
    float clip;
    const void *packed;
    const float *h;
    const int32_t *rs_w;
    int bits, groups;
    int64_t T, N, K;
    const float *bias;   /* [N] or NULL */
    float *Y;            /* [T,N] */
} qb_fwd_job;
qb_status qb_qlinear_fwd_batched(const qb_fwd_job *jobs, int n_jobs, void *stream);

/*
 * Forward with an 8-bit output: the layer's result goes through the activation quantizer at once
 * (Table 1 caption: every matrix product takes 8-bit activations; App. quantizer with k = 8), so
 * the next layer's input is written instead of the fp32 result, a quarter of its bytes.
 *   A4 as in qb_qlinear_fwd;  y = (h_x * h_{g(n)}) * float(A4) (+ bias[n]), each step one binary32
 *   rounding;  act = 1 applies GELU(y) = y/2 * (1 + erf(y / sqrt 2)) in binary32 (act = 0: nothing);
 *   Yq[t,n] = code(clamp(y, -clip_out, clip_out)) - 128 with the quantizer of qb_quantize_act
 *   for the range [-clip_out, +clip_out];  rs_y[t] = sum_n Yq[t,n].
 * With act = 0 the codes are a function of the inputs alone (bit-exact); with act = 1 they depend
 * on the erf implementation by at most one code next to a rounding boundary.
 *   Yq    out  [T,N] int8        rs_y  out  [T] int32 (cleared and accumulated by this call)
 *   K must be a multiple of 128 (QB_ERR_SHAPE otherwise); other arguments as qb_qlinear_fwd.
 */
qb_status qb_qlinear_fwd_q8(const int8_t *Xq, const int32_t *rs_x, float clip,
                            const void *packed, const float *h, const int32_t *rs_w,
                            int bits, int groups, int64_t T, int64_t N, int64_t K,
                            const float *bias, int act, float clip_out,
                            int8_t *Yq, int32_t *rs_y, void *stream);

/*
 * Activation quantization with a range per token (the appendix's quantizer takes any range
 * [q0, q_255]; the paper fixes none for activations): c_t = max_j |X[t,j]|, otherwise as
 * qb_quantize_act.  Needs no calibrated clip and never clips.
 *   hx_rows  out  [T] fp32, c_t / 255 (0 for an all-zero row, whose codes are 0)
 * and the forward that takes those scales: Y[t,n] = (hx_rows[t] * h_{g(n)}) * float(A4[t,n]) (+ bias[n]);
 * other arguments as qb_qlinear_fwd.
 */
qb_status qb_quantize_act_dyn(const float *X, int64_t T, int64_t K,
                              int8_t *Xq, int32_t *rs_x, float *hx_rows, void *stream);
qb_status qb_qlinear_fwd_dyn(const int8_t *Xq, const int32_t *rs_x, const float *hx_rows,
                             const void *packed, const float *h, const int32_t *rs_w,
                             int bits, int groups, int64_t T, int64_t N, int64_t K,
                             const float *bias, float *Y, int32_t *A4_debug, void *stream);

/*
 * Activation quantization with one range for the whole tensor, taken from the data (the appendix's
 * quantizer takes any range [q0, q_255]): c = max |X|, otherwise as qb_quantize_act with clip = c.  One scale
 * per matmul like a calibrated clip, but nothing is clipped and no calibration is needed.
 *   c_out    out  [1] fp32 device, c (also the reduction's scratch: the call zero-fills it first)
 *   hx_rows  out  [T] fp32, c / 255 in every entry (0 for an all-zero tensor, whose codes are 0), the form
 *                 qb_qlinear_fwd_dyn takes; its Y equals qb_qlinear_fwd's with clip = c
 * Three launches on `stream` (fill, reduce, quantize); no host synchronisation.  Errors as qb_quantize_act.
 */
qb_status qb_quantize_act_dyn_tensor(const float *X, int64_t T, int64_t K,
                                     int8_t *Xq, int32_t *rs_x, float *hx_rows, float *c_out,
                                     void *stream);

/*
 * Straight-through-estimator backward (Sec. 3.1, last paragraph; App., last sentence): both
 * quantizers pass the gradient through unchanged, so
 *   dX[t,j] = sum_n dY[t,n] * Q(w)[n,j]        dW[n,j] = sum_t dY[t,n] * Q(x)[t,j]
 * computed on bf16 matrix cores with fp32 accumulation.
 *   dY   in   [T,N] bfloat16 (bit patterns)
 *   dX   out  [T,K] bfloat16 or NULL
 *   dW   out  [N,K] fp32 or NULL; overwritten, not accumulated into
 *   workspace  qb_bwd_workspace_nbytes(T,N,K) bytes, 256-byte aligned; contents undefined
 *              before and after the call
 * Two launches on `stream` (operand staging, then one launch that computes both products, its workgroups sharing
 * the contraction steps evenly and adding the partial sums of a shared tile in a fixed order): the same call gives
 * the same bits every time.  Which of dX and dW a call computes decides how the steps are shared, so dX of a
 * dX-only call may differ from dX of a call that also computes dW in the last bf16 bit (order of the fp32
 * additions).  Inside the launch a workgroup may wait for partial sums of workgroups dispatched before it; the
 * wait is bounded (about two seconds), after which the tile concerned is written as NaN.  Calls that share a
 * workspace must not overlap in time.
 */
qb_status qb_qlinear_bwd_ste(const uint16_t *dY, const int8_t *Xq, float clip,
                             const void *packed, const float *h, int bits, int groups,
                             int64_t T, int64_t N, int64_t K,
                             uint16_t *dX, float *dW, void *workspace, void *stream);

/*
 * qb_qlinear_bwd_ste for callers that cannot allocate device memory or carry a workspace around (code under
 * HIP graph capture, tight serving or training loops, harnesses that forbid hipMalloc): the same kernels and
 * results, with the staging area taken from a fixed array inside the library instead of a `workspace`
 * argument.  The call allocates and frees nothing.  The array has QB_BWD_STATIC_BYTES bytes on every GPU the
 * library runs on, for as long as the process lives; shapes that need more (qb_bwd_workspace_nbytes(T,N,K) >
 * QB_BWD_STATIC_BYTES; the limit covers every linear of a BERT-base layer at up to 4096 tokens: 58.5 MiB) are refused with
 * QB_ERR_WORKSPACE before anything is enqueued.  All calls on one GPU share that GPU's array: calls that overlap
 * in time on one GPU (different streams, different threads) race on it and must be serialised by the caller;
 * successive calls on one stream are safe, whatever their shapes.  Other arguments and errors as
 * qb_qlinear_bwd_ste.
 */
#define QB_BWD_STATIC_BYTES (60u << 20)
qb_status qb_qlinear_bwd_ste_static(const uint16_t *dY, const int8_t *Xq, float clip,
                                    const void *packed, const float *h, int bits, int groups,
                                    int64_t T, int64_t N, int64_t K,
                                    uint16_t *dX, float *dW, void *stream);

/*
 * The same backward with the clamp's own derivative kept (App.: X' = Clamp(X, q0, q_{2^k-1}) precedes the
 * rounding; only the rounding is passed straight through): the gradient of a value that lay outside its
 * range is zero, that of a value inside (ends included) is unchanged.
 *   X  in  [T,K] fp32, the activations that qb_quantize_act saw, range [-clip, +clip]; NULL: dX unmasked
 *   W  in  [N,K] fp32, the weights that qb_quantize_groupwise[_clip] saw, and
 *   m  in  [G] fp32, the group ranges it used (its m output, or the m_in given); both NULL: dW unmasked
 *          (one of the two NULL: QB_ERR_NULL)
 * The masks are applied where the two products are written (no extra pass); other arguments, workspace
 * and errors as qb_qlinear_bwd_ste.
 */
qb_status qb_qlinear_bwd_ste_masked(const uint16_t *dY, const int8_t *Xq, float clip,
                                    const void *packed, const float *h, int bits, int groups,
                                    int64_t T, int64_t N, int64_t K,
                                    const float *X, const float *W, const float *m,
                                    uint16_t *dX, float *dW, void *workspace, void *stream);

/*
 * Asymmetric group ranges (App., the quantizer in its general form: range [q0, q_{2^k-1}],
 * Delta = (q_{2^k-1} - q0)/(2^k - 1), X^I = round((X - q0)/Delta), Q(X) = Delta*X^I + q0): the range of a group
 * is its own [min, max] instead of the symmetric [-max|w|, +max|w|] of qb_quantize_groupwise, so that no level
 * is spent outside the data (one-sided or shifted weight groups).
 *   delta  out  [G] fp32, Delta_g (0 for a constant group, whose codes are 0)
 *   q0     out  [G] fp32, the group's minimum
 *   packed, rs_w  as qb_quantize_groupwise (same layout, same row sums: qb_unpack_codes applies)
 * One launch when a group (N/G rows of K) has at most 32768 weights, else four (delta and q0 then serve as
 * scratch of the min/max reduction during the call).
 *
 * qb_qlinear_fwd_asym: Y[t,n] = h_x * (Delta_g * S[t,n] + q0_g * R[t]) (+ bias[n]) with the integer sums
 * S = sum_j (2x'+1) u[n,j] and R = sum_j (2x'+1) = 2 rs_x[t] + K, both taken from the same int8 matrix-core
 * product as qb_qlinear_fwd (S = (A4 + (2^k-1) R)/2, exact).  A4_debug as there.  Fixed activation clip.
 *
 * qb_qlinear_fwd_asym_dyn: the same with one activation scale per token, Y[t,n] = hx_rows[t] * (Delta_g * S[t,n] +
 * q0_g * R[t]) (+ bias[n]); hx_rows [T] fp32 as written by qb_quantize_act_dyn or qb_quantize_act_dyn_tensor.
 *
 * qb_qlinear_bwd_ste_asym: qb_qlinear_bwd_ste with Q(w) = Delta*u + q0 in dX; dW does not involve the weights.
 * Errors as the symmetric calls.
 */
qb_status qb_quantize_groupwise_asym(const float *W, int64_t N, int64_t K, int bits, int groups,
                                     void *packed, float *delta, float *q0, int32_t *rs_w, void *stream);
/*
 * qb_quantize_groupwise_asym with the range of every group given by the caller (App.: the range [q0, q_{2^k-1}] may be
 * a sub-interval of the data's [min, max], X' = Clamp(X, q0, q_{2^k-1})): group g uses [lo[g], hi[g]]; weights outside
 * are clamped first and get the end codes; Delta_g = fl(fl(hi - lo)/L), q0_g = lo.  lo = min and hi = max of the group
 * give the codes of qb_quantize_groupwise_asym.
 *   lo, hi  in  [G] fp32, finite, lo <= hi (not checked on the device; lo == hi gives Delta = 0 and codes 0)
 * The result feeds qb_qlinear_fwd_asym and qb_qlinear_bwd_ste_asym unchanged.
 */
qb_status qb_quantize_groupwise_asym_range(const float *W, int64_t N, int64_t K, int bits, int groups,
                                           const float *lo, const float *hi,
                                           void *packed, float *delta, float *q0, int32_t *rs_w, void *stream);
qb_status qb_qlinear_fwd_asym(const int8_t *Xq, const int32_t *rs_x, float clip,
                              const void *packed, const float *delta, const float *q0, const int32_t *rs_w,
                              int bits, int groups, int64_t T, int64_t N, int64_t K,
                              const float *bias, float *Y, int32_t *A4_debug, void *stream);
qb_status qb_qlinear_fwd_asym_dyn(const int8_t *Xq, const int32_t *rs_x, const float *hx_rows,
                                  const void *packed, const float *delta, const float *q0, const int32_t *rs_w,
                                  int bits, int groups, int64_t T, int64_t N, int64_t K,
                                  const float *bias, float *Y, int32_t *A4_debug, void *stream);
qb_status qb_qlinear_bwd_ste_asym(const uint16_t *dY, const int8_t *Xq, float clip,
                                  const void *packed, const float *delta, const float *q0, int bits, int groups,
                                  int64_t T, int64_t N, int64_t K,
                                  uint16_t *dX, float *dW, void *workspace, void *stream);

/*
 * Hessian-based sensitivity (Sec. 3.2).  The Hessian-vector product itself (Eq. 1: a second back-propagation
 * through the model) is the caller's: it is handed in as a function.
 *
 * qb_power_iteration -- Alg. 1: v = v/|v|; `iters` times: Hv = hv(v); estimate = v.Hv; v = Hv/|Hv|.
 *   hv         host function; must enqueue on `stream` work that reads v[n] and writes out[n] (device fp32),
 *              and return 0 (anything else ends the call with QB_ERR_HIP).  Called `iters` times, in order.
 *   v          in/out [n] fp32 device: the random start vector drawn by the caller (Alg. 1, line 2), on
 *              return the last normalised vector (all zeros if some Hv was the zero vector)
 *   hv_buf     [n] fp32 device, the product's destination; contents undefined afterwards
 *   scratch    [qb_power_iteration_scratch_floats()] fp32 device
 *   estimates  out [iters] fp32 device: v.Hv of every step, the last one being the top eigenvalue's estimate
 * Nothing is copied to the host and nothing waits: 3 + 3*iters small launches around the caller's own.  The
 * reductions run in a fixed order (the result does not depend on scheduling).
 * If the callback returns non-zero in step i, the call returns QB_ERR_HIP at once: the normalisation of v and the
 * steps 0 .. i-1 are already in the stream (they stay valid work: v holds the normalised vector of step i,
 * estimates[0 .. i-1] are defined, estimates[i ..] are not written), and nothing further is enqueued.
 *
 * qb_sensitivity_omega -- Eq. 2, host only: omega[i] = |mean_r lambdas[i][r]| + std_r lambdas[i][r] (population
 * standard deviation over the `runs` estimates of layer i; arithmetic in binary64).
 * qb_rank_by_sensitivity -- host only: order[] = the layers by descending omega (ties keep layer order); the
 * paper gives more bits to the layers that come first and sets the cut by hand.
 */
typedef int (*qb_hv_fn)(void *ctx, const float *v, float *out, void *stream);
size_t qb_power_iteration_scratch_floats(void);
qb_status qb_power_iteration(qb_hv_fn hv, void *ctx, int64_t n, int iters,
                             float *v, float *hv_buf, float *scratch, float *estimates, void *stream);
qb_status qb_sensitivity_omega(const float *lambdas, int layers, int runs, float *omega);
qb_status qb_rank_by_sensitivity(const float *omega, int layers, int32_t *order);

/*
 * Measurement aid (no part of the method): `workgroups` x 4 wavefronts each issue `iters` rounds of four
 * independent 32x32x32 int8 matrix-core instructions on registers, i.e. workgroups * 4 * iters * 4 * 65536
 * integer operations and nothing else; timed by the caller, it gives the issue-rate peak that the GEMM's
 * percentage can be read against beside the published one.  sink: [1] int32 device (practically never written).
 */
qb_status qb_probe_mfma_i8(int workgroups, int iters, int32_t *sink, void *stream);

/* Test hook: packed buffer -> codes[N,K] uint8 in row-major order (inverse of the packing,
 * Sec. 4: low-bit codes are loaded as stored and widened before the arithmetic). */
qb_status qb_unpack_codes(const void *packed, int64_t N, int64_t K, int bits,
                          uint8_t *codes, void *stream);

/*
 * 8-bit group-wise embedding table (Sec. 3: the embedding layer is kept at 8 bits; App. "Mixed Precision
 * Quantization for Embedding": the d output neurons of the embedding are bucketed into
 * groups).  Group g = columns [g*d/G, (g+1)*d/G) over all V rows; same quantizer, k = 8.
 *   E      in   [V,d] fp32       codes  out  [V,d] uint8 (u in 0..255)
 *   h, m   out  [G] fp32
 * Requires d % groups == 0 and d % QB_K_ALIGN == 0.
 */
qb_status qb_embedding_quantize(const float *E, int64_t V, int64_t d, int groups,
                                uint8_t *codes, float *h, float *m, void *stream);

/* Lookup with de-quantization: out[i,j] = h[g(j)] * (2*codes[ids[i],j] - 255).
 *   ids  in  [n_ids] int64; an id outside [0,V) yields a row of zeros
 *   out  out [n_ids,d] fp32.   n_ids == 0 is allowed and does nothing. */
qb_status qb_embedding_gather(const uint8_t *codes, const float *h, int64_t V, int64_t d, int groups,
                              const int64_t *ids, int64_t n_ids, float *out, void *stream);

/*
 * The same two calls for k = 4 or 8 bits (App. "Mixed Precision Quantization for Embedding":
 * 4-bit word embeddings next to 8-bit position embeddings, 128 groups).  bits = 8 is exactly
 * the pair above.  bits = 4: codes is [V, d/2] bytes, column 2i in the low and column 2i+1 in
 * the high nibble of byte i of the row; out[i,j] = h[g(j)] * (2u - 15).  Other bit-widths:
 * QB_ERR_BITS.
 */
qb_status qb_embedding_quantize_bits(const float *E, int64_t V, int64_t d, int bits, int groups,
                                     uint8_t *codes, float *h, float *m, void *stream);
qb_status qb_embedding_gather_bits(const uint8_t *codes, const float *h, int64_t V, int64_t d, int bits,
                                   int groups, const int64_t *ids, int64_t n_ids, float *out,
                                   void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QBERT_H */
