/*
 * qbert_oracle.c -- plain CPU oracle for the Q-BERT group-wise quantized linear layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the parity authority for the HIP library and the
 * timed CPU baseline of the benchmark.  It shares no code, header, table or helper with the
 * GPU path and nothing in the product package may include, link or call it.
 *
 * It is deliberately slow and literal: every function walks the steps of the paper's
 * quantizer in the paper's order (Appendix "Detailed quantization process": clamp, subtract
 * q0, divide by Delta, round, Q(X) = Delta*X^I + q0), the grouping rule of Sec. 3.3
 * (consecutive output neurons share one range), and a triple-loop integer matrix product
 * followed by de-quantization (same appendix, last paragraph).  There is no blocking, fusion
 * or vectorisation.  Build with  gcc -O2 -ffp-contract=off  (add -fopenmp for the timed
 * baseline: the pragmas only spread independent outer iterations over threads).
 *
 * Precision.  The paper fixes none.  Steps that decide an integer code are single IEEE-754
 * binary32 operations, round-to-nearest-even, one rounding per operation, in the order
 * written below, because codes must agree bit for bit with any other implementation.
 * Everything downstream of the integer accumulator is evaluated in binary64.
 *
 * Readings of the paper taken here (each is a choice where the text is silent):
 *   - range of a group is the symmetric interval [-m, +m], m = max |w| over the group
 *     (the appendix allows any [q0, q_{2^k-1}]);
 *   - codes are the paper's unsigned integers 0..2^k-1, all 2^k levels are used, so
 *     Q(w) = Delta*u + q0 = h*(2u - L) with h = m/L, L = 2^k-1 (zero is not a level);
 *   - the round operator is round-half-to-even;
 *   - Delta is formed as 2*(m/L);
 *   - groups are G equal blocks of N/G consecutive rows (output neurons) of W[N,K];
 *   - activations use the same quantizer with k = 8 and a caller-given range [-c, +c];
 *     the stored byte is u - 128; the dynamic variant takes c per token as the row's max-abs;
 *   - the straight-through estimator is the identity through both quantizers, and the
 *     weight gradient uses the de-quantized activation;
 *   - the embedding table is grouped over its columns (embedding dimension);
 *   - where a layer's output is quantized again at once (8-bit output), the value that decides
 *     the code is the binary32 product (h_x*h_g)*float(A4) (+ bias), not the binary64 one.
 *
 * Parity pins live in tests/test_oracle_pins.py.  Unpinned: nothing in this file depends on
 * the paper's accuracy tables (those need its datasets and checkpoints).
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>

#define QBO_OK 0
#define QBO_ERR_ARG 1
#define QBO_ERR_NONFINITE 2
#define QBO_ERR_OVERFLOW 3

static int bits_ok(int bits) { return bits == 2 || bits == 3 || bits == 4 || bits == 8; }

/* exact widening of a bfloat16 bit pattern */
static double bf16_to_double(uint16_t b)
{
    uint32_t w = (uint32_t)b << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* ---- the uniform quantizer on one value (App. "Detailed quantization process") ----------
 * range [q0, q_{2^k-1}] = [-m, +m];  h = m/L is half of Delta.
 *   X'  = Clamp(X, -m, +m)
 *   X^I = round((X' - q0) / Delta)
 * each arithmetic step is one binary32 operation. */
static int quantize_one(float x, float m, float delta, int L)
{
    float xc, s, t, r;
    int u;
    if (m == 0.0f) return 0;
    xc = x;
    if (xc < -m) xc = -m;
    if (xc > m) xc = m;
    s = xc + m;              /* X' - q0, q0 = -m */
    t = s / delta;
    r = rintf(t);            /* default rounding mode: half to even */
    u = (int)r;
    if (u < 0) u = 0;
    if (u > L) u = L;
    return u;
}

/* Sec. 3.3 grouping + App. quantizer, weights.
 * W[N,K] row-major fp32.  Group g = rows [g*N/G, (g+1)*N/G).
 * out: codes[N,K] (u in 0..L), h[G] = m/L, m[G] = max|w|, rs_w[N] = sum_j (u - 2^(k-1)). */
int qbo_quantize_groupwise(const float *W, int64_t N, int64_t K, int bits, int64_t G,
                           uint8_t *codes, float *h, float *m, int32_t *rs_w)
{
    int64_t g, rows;
    int L, half;
    if (!W || !codes || !h || !m || !rs_w) return QBO_ERR_ARG;
    if (!bits_ok(bits) || N <= 0 || K <= 0 || G <= 0 || N % G != 0) return QBO_ERR_ARG;
    L = (1 << bits) - 1;
    half = 1 << (bits - 1);
    rows = N / G;
    for (g = 0; g < G; ++g) {
        const float *Wg = W + g * rows * K;
        uint8_t *cg = codes + g * rows * K;
        float mg = 0.0f, hg, delta;
        int64_t i, r, j;
        for (i = 0; i < rows * K; ++i) {
            float a = fabsf(Wg[i]);
            if (!isfinite(a)) return QBO_ERR_NONFINITE;
            if (a > mg) mg = a;
        }
        hg = (mg == 0.0f) ? 0.0f : mg / (float)L;
        delta = 2.0f * hg;
        m[g] = mg;
        h[g] = hg;
        for (r = 0; r < rows; ++r) {
            int32_t acc = 0;
            for (j = 0; j < K; ++j) {
                int u = quantize_one(Wg[r * K + j], mg, delta, L);
                cg[r * K + j] = (uint8_t)u;
                acc += u - half;
            }
            rs_w[g * rows + r] = acc;
        }
    }
    return QBO_OK;
}

/* The same with the range of every group given by the caller instead of taken as the max-abs:
 * [-m_g, +m_g] may be a clipped sub-interval of the weights' range (App.: the range is
 * [q0, q_{2^k-1}], "X' = Clamp(X, q0, q_{2^k-1})"), e.g. a percentile; weights outside are clamped and
 * get the end codes 0 or L.  m_in[G] >= 0 finite. */
int qbo_quantize_groupwise_clip(const float *W, int64_t N, int64_t K, int bits, int64_t G, const float *m_in,
                                uint8_t *codes, float *h, int32_t *rs_w)
{
    int64_t g, rows;
    int L, half;
    if (!W || !m_in || !codes || !h || !rs_w || !bits_ok(bits)) return QBO_ERR_ARG;
    if (N <= 0 || K <= 0 || G <= 0 || N % G) return QBO_ERR_ARG;
    L = (1 << bits) - 1;
    half = 1 << (bits - 1);
    rows = N / G;
    for (g = 0; g < G; ++g) {
        float mg = m_in[g], hg, delta;
        int64_t r, j;
        if (!(mg >= 0.0f) || !isfinite(mg)) return QBO_ERR_ARG;
        hg = (mg == 0.0f) ? 0.0f : mg / (float)L;
        delta = 2.0f * hg;
        h[g] = hg;
        for (r = g * rows; r < (g + 1) * rows; ++r) {
            int32_t acc = 0;
            for (j = 0; j < K; ++j) {
                float w = W[r * K + j];
                int u;
                if (isnan(w)) return QBO_ERR_NONFINITE;
                u = quantize_one(w, mg, delta, L);
                codes[r * K + j] = (uint8_t)u;
                acc += u - half;
            }
            rs_w[r] = acc;
        }
    }
    return QBO_OK;
}

/* Q(w) = Delta*u + q0, written as h*(2u - L): the same real number, one rounding. */
int qbo_dequantize_groupwise(const uint8_t *codes, const float *h, int64_t N, int64_t K,
                             int bits, int64_t G, double *Wq)
{
    int64_t n, j, rows;
    int L;
    if (!codes || !h || !Wq || !bits_ok(bits) || N <= 0 || K <= 0 || G <= 0 || N % G) return QBO_ERR_ARG;
    L = (1 << bits) - 1;
    rows = N / G;
    for (n = 0; n < N; ++n)
        for (j = 0; j < K; ++j)
            Wq[n * K + j] = (double)h[n / rows] * (double)(2 * (int)codes[n * K + j] - L);
    return QBO_OK;
}

/* Canonical packed form used only on the oracle side (the paper stores k-bit codes; the size
 * rows of its Table 1 are params*k/8): each row is a little-endian bit stream, code j of a
 * row occupies bits [j*k, (j+1)*k).  Row stride = ceil(K*k/8) bytes. */
int64_t qbo_packed_row_bytes(int64_t K, int bits) { return (K * bits + 7) / 8; }

int qbo_pack(const uint8_t *codes, int64_t N, int64_t K, int bits, uint8_t *packed)
{
    int64_t n, j, rb;
    if (!codes || !packed || !bits_ok(bits) || N <= 0 || K <= 0) return QBO_ERR_ARG;
    rb = qbo_packed_row_bytes(K, bits);
    memset(packed, 0, (size_t)(N * rb));
    for (n = 0; n < N; ++n)
        for (j = 0; j < K; ++j) {
            int b;
            unsigned u = codes[n * K + j];
            for (b = 0; b < bits; ++b) {
                int64_t pos = j * bits + b;
                if ((u >> b) & 1u) packed[n * rb + pos / 8] |= (uint8_t)(1u << (pos % 8));
            }
        }
    return QBO_OK;
}

int qbo_unpack(const uint8_t *packed, int64_t N, int64_t K, int bits, uint8_t *codes)
{
    int64_t n, j, rb;
    if (!codes || !packed || !bits_ok(bits) || N <= 0 || K <= 0) return QBO_ERR_ARG;
    rb = qbo_packed_row_bytes(K, bits);
    for (n = 0; n < N; ++n)
        for (j = 0; j < K; ++j) {
            int b;
            unsigned u = 0;
            for (b = 0; b < bits; ++b) {
                int64_t pos = j * bits + b;
                u |= (unsigned)((packed[n * rb + pos / 8] >> (pos % 8)) & 1u) << b;
            }
            codes[n * K + j] = (uint8_t)u;
        }
    return QBO_OK;
}

/* 8-bit activation quantizer (Table 1 caption: 8-bit activations; same appendix formulas),
 * range [-c, +c] given by the caller.  X[T,K] fp32 -> xq[T,K] = u - 128, rs_x[t] = sum_j xq. */
int qbo_quantize_act(const float *X, int64_t T, int64_t K, float clip, int8_t *xq, int32_t *rs_x)
{
    int64_t t, j;
    float hx, delta;
    if (!X || !xq || !rs_x || T <= 0 || K <= 0) return QBO_ERR_ARG;
    if (!(clip > 0.0f) || !isfinite(clip)) return QBO_ERR_ARG;
    hx = clip / 255.0f;
    delta = 2.0f * hx;
    for (t = 0; t < T; ++t) {
        int32_t acc = 0;
        for (j = 0; j < K; ++j) {
            float x = X[t * K + j];
            int u;
            if (isnan(x)) return QBO_ERR_NONFINITE;
            u = quantize_one(x, clip, delta, 255);
            xq[t * K + j] = (int8_t)(u - 128);
            acc += u - 128;
        }
        rs_x[t] = acc;
    }
    return QBO_OK;
}

/* The same quantizer with a range per token (row): [-c_t, +c_t], c_t = max_j |X[t,j]| (the appendix
 * allows any range [q0, q_255]; the paper fixes none for activations).  A dynamic range needs no
 * calibration and never clips.  out: xq[T,K] = u - 128, rs_x[t], hx[t] = c_t/255 (0 for a zero row,
 * whose codes are 0 like those of an all-zero weight group). */
int qbo_quantize_act_dyn(const float *X, int64_t T, int64_t K, int8_t *xq, int32_t *rs_x, float *hx)
{
    int64_t t, j;
    if (!X || !xq || !rs_x || !hx || T <= 0 || K <= 0) return QBO_ERR_ARG;
    for (t = 0; t < T; ++t) {
        float c = 0.0f, h, delta;
        int32_t acc = 0;
        for (j = 0; j < K; ++j) {
            float a = fabsf(X[t * K + j]);
            if (!isfinite(a)) return QBO_ERR_NONFINITE;
            if (a > c) c = a;
        }
        h = (c == 0.0f) ? 0.0f : c / 255.0f;
        delta = 2.0f * h;
        hx[t] = h;
        for (j = 0; j < K; ++j) {
            int u = quantize_one(X[t * K + j], c, delta, 255);
            xq[t * K + j] = (int8_t)(u - 128);
            acc += u - 128;
        }
        rs_x[t] = acc;
    }
    return QBO_OK;
}

/* The same quantizer with one range for the whole tensor taken from the data: [-c, +c], c = max |X|
 * (the appendix allows any range [q0, q_255]).  Like a calibrated clip it is one scale per matmul, but
 * it needs no calibration and never clips.  out: xq[T,K] = u - 128, rs_x[t], hx[0] = c/255 (0 for an
 * all-zero tensor, whose codes are 0). */
int qbo_quantize_act_dyn_tensor(const float *X, int64_t T, int64_t K, int8_t *xq, int32_t *rs_x, float *hx)
{
    int64_t t, j;
    float c = 0.0f, h, delta;
    if (!X || !xq || !rs_x || !hx || T <= 0 || K <= 0) return QBO_ERR_ARG;
    for (t = 0; t < T * K; ++t) {
        float a = fabsf(X[t]);
        if (!isfinite(a)) return QBO_ERR_NONFINITE;
        if (a > c) c = a;
    }
    h = (c == 0.0f) ? 0.0f : c / 255.0f;
    delta = 2.0f * h;
    hx[0] = h;
    for (t = 0; t < T; ++t) {
        int32_t acc = 0;
        for (j = 0; j < K; ++j) {
            int u = quantize_one(X[t * K + j], c, delta, 255);
            xq[t * K + j] = (int8_t)(u - 128);
            acc += u - 128;
        }
        rs_x[t] = acc;
    }
    return QBO_OK;
}

/* De-quantized activation: h_x*(2u - 255) = h_x*(2*xq + 1). */
int qbo_dequantize_act(const int8_t *xq, int64_t T, int64_t K, float clip, double *Xhat)
{
    int64_t i;
    float hx;
    if (!xq || !Xhat || T <= 0 || K <= 0 || !(clip > 0.0f)) return QBO_ERR_ARG;
    hx = clip / 255.0f;
    for (i = 0; i < T * K; ++i) Xhat[i] = (double)hx * (double)(2 * (int)xq[i] + 1);
    return QBO_OK;
}

/* One output of the integer product (App., last paragraph: integer matmul on X^I, then a
 * de-quantization).  acc = sum_j x'[t,j]*c'[n,j] with c' = u - 2^(k-1);
 * A4 = sum_j (2x'+1)(2c'+1) = 4*acc + 2*rs_x + 2*rs_w + K is the integer whose product with
 * h_x*h_g is exactly sum_j Xhat*What.  Both forms are evaluated and must agree. */
static int fwd_one(const int8_t *xrow, const uint8_t *crow, int64_t K, int bits,
                   int64_t *acc_out, int64_t *a4_out)
{
    int64_t j, acc = 0, rsx = 0, rsw = 0, a4 = 0, a4_direct = 0;
    int half = 1 << (bits - 1);
    for (j = 0; j < K; ++j) {
        int xp = xrow[j];
        int cp = (int)crow[j] - half;
        acc += (int64_t)xp * cp;
        rsx += xp;
        rsw += cp;
        a4_direct += (int64_t)(2 * xp + 1) * (2 * cp + 1);
    }
    a4 = 4 * acc + 2 * rsx + 2 * rsw + K;
    if (a4 != a4_direct) return QBO_ERR_OVERFLOW;
    if (a4 > INT32_MAX || a4 < INT32_MIN || acc > INT32_MAX || acc < INT32_MIN) return QBO_ERR_OVERFLOW;
    *acc_out = acc;
    *a4_out = a4;
    return QBO_OK;
}

/* Forward of the quantized linear layer.  xq[T,K] int8, codes[N,K] u8, h[G].
 * out: Y[T,N] fp32 = float(h_x*h_g*A4 (+bias)), A4[T,N] int32 (nullable), acc[T,N] (nullable). */
int qbo_qlinear_fwd(const int8_t *xq, float clip, const uint8_t *codes, const float *h,
                    int bits, int64_t G, int64_t T, int64_t N, int64_t K, const float *bias,
                    float *Y, int32_t *A4, int32_t *acc)
{
    int64_t t, rows;
    float hx;
    int bad = 0;
    if (!xq || !codes || !h || !Y || !bits_ok(bits)) return QBO_ERR_ARG;
    if (T <= 0 || N <= 0 || K <= 0 || G <= 0 || N % G || !(clip > 0.0f)) return QBO_ERR_ARG;
    hx = clip / 255.0f;
    rows = N / G;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (t = 0; t < T; ++t) {
        int64_t n;
        for (n = 0; n < N; ++n) {
            int64_t a = 0, a4 = 0;
            double y;
            if (fwd_one(xq + t * K, codes + n * K, K, bits, &a, &a4) != QBO_OK) { bad = 1; continue; }
            y = (double)hx * (double)h[n / rows] * (double)a4;
            if (bias) y += (double)bias[n];
            Y[t * N + n] = (float)y;
            if (A4) A4[t * N + n] = (int32_t)a4;
            if (acc) acc[t * N + n] = (int32_t)a;
        }
    }
    return bad ? QBO_ERR_OVERFLOW : QBO_OK;
}

/* Forward with one activation scale per token: Y[t,n] = float(hx[t]*h_g*A4 (+bias)). */
int qbo_qlinear_fwd_dyn(const int8_t *xq, const float *hx, const uint8_t *codes, const float *h,
                        int bits, int64_t G, int64_t T, int64_t N, int64_t K, const float *bias,
                        float *Y, int32_t *A4)
{
    int64_t t, rows;
    int bad = 0;
    if (!xq || !hx || !codes || !h || !Y || !bits_ok(bits)) return QBO_ERR_ARG;
    if (T <= 0 || N <= 0 || K <= 0 || G <= 0 || N % G) return QBO_ERR_ARG;
    rows = N / G;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (t = 0; t < T; ++t) {
        int64_t n;
        for (n = 0; n < N; ++n) {
            int64_t a = 0, a4 = 0;
            double y;
            if (fwd_one(xq + t * K, codes + n * K, K, bits, &a, &a4) != QBO_OK) { bad = 1; continue; }
            y = (double)hx[t] * (double)h[n / rows] * (double)a4;
            if (bias) y += (double)bias[n];
            Y[t * N + n] = (float)y;
            if (A4) A4[t * N + n] = (int32_t)a4;
        }
    }
    return bad ? QBO_ERR_OVERFLOW : QBO_OK;
}

/* The same, for a list of (t, n) positions only: used to check full-size GPU runs. */
int qbo_qlinear_fwd_sampled(const int8_t *xq, float clip, const uint8_t *codes, const float *h,
                            int bits, int64_t G, int64_t T, int64_t N, int64_t K, const float *bias,
                            const int64_t *ts, const int64_t *ns, int64_t count,
                            float *Y, int32_t *A4)
{
    int64_t i, rows;
    float hx;
    if (!xq || !codes || !h || !Y || !A4 || !ts || !ns || !bits_ok(bits)) return QBO_ERR_ARG;
    if (T <= 0 || N <= 0 || K <= 0 || G <= 0 || N % G || !(clip > 0.0f)) return QBO_ERR_ARG;
    hx = clip / 255.0f;
    rows = N / G;
    for (i = 0; i < count; ++i) {
        int64_t a = 0, a4 = 0, t = ts[i], n = ns[i];
        double y;
        if (t < 0 || t >= T || n < 0 || n >= N) return QBO_ERR_ARG;
        if (fwd_one(xq + t * K, codes + n * K, K, bits, &a, &a4) != QBO_OK) return QBO_ERR_OVERFLOW;
        y = (double)hx * (double)h[n / rows] * (double)a4;
        if (bias) y += (double)bias[n];
        Y[i] = (float)y;
        A4[i] = (int32_t)a4;
    }
    return QBO_OK;
}

/* Forward with an 8-bit output: the layer's result goes through the activation quantizer right
 * away (Table 1 caption: every matmul input is an 8-bit activation; App. quantizer with k = 8 and
 * the caller's range [-c_out, +c_out]), optionally after BERT's feed-forward non-linearity
 * GELU(y) = y/2 * (1 + erf(y/sqrt 2)).  What the next layer needs is returned: yq[T,N] = u - 128 and
 * rs_y[t] = sum_n yq[t,n].
 * Precision: the value that decides the code is formed in binary32, one rounding per operation,
 *   scale = h_x * h_g;   y = scale * float(A4);   y = y + bias[n]   (if a bias is given)
 * (int -> float conversion rounds to nearest even).  GELU is evaluated in binary64 on that y and
 * rounded once to binary32; an implementation with a binary32 erf may differ from it by a code
 * on inputs next to a rounding boundary.  act: 0 = none, 1 = GELU. */
int qbo_qlinear_fwd_q8(const int8_t *xq, float clip, const uint8_t *codes, const float *h,
                       int bits, int64_t G, int64_t T, int64_t N, int64_t K, const float *bias,
                       int act, float clip_out, int8_t *yq, int32_t *rs_y)
{
    int64_t t, rows;
    float hx, delta_out;
    int bad = 0;
    if (!xq || !codes || !h || !yq || !rs_y || !bits_ok(bits)) return QBO_ERR_ARG;
    if (T <= 0 || N <= 0 || K <= 0 || G <= 0 || N % G || !(clip > 0.0f)) return QBO_ERR_ARG;
    if (!(clip_out > 0.0f) || !isfinite(clip_out) || (act != 0 && act != 1)) return QBO_ERR_ARG;
    hx = clip / 255.0f;
    delta_out = 2.0f * (clip_out / 255.0f);
    rows = N / G;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (t = 0; t < T; ++t) {
        int64_t n;
        int32_t rs = 0;
        for (n = 0; n < N; ++n) {
            int64_t a = 0, a4 = 0;
            float scale, y;
            int u;
            if (fwd_one(xq + t * K, codes + n * K, K, bits, &a, &a4) != QBO_OK) { bad = 1; continue; }
            scale = hx * h[n / rows];
            y = scale * (float)(int32_t)a4;
            if (bias) y = y + bias[n];
            if (act == 1) y = (float)(0.5 * (double)y * (1.0 + erf((double)y / sqrt(2.0))));
            u = quantize_one(y, clip_out, delta_out, 255);
            yq[t * N + n] = (int8_t)(u - 128);
            rs += u - 128;
        }
        rs_y[t] = rs;
    }
    return bad ? QBO_ERR_OVERFLOW : QBO_OK;
}

/* Straight-through backward (Sec. 3.1 last paragraph; App. last sentence): the quantizers
 * pass the gradient unchanged, so the layer's gradients are those of Y = Xhat * What^T:
 *   dX[t,j] = sum_n dY[t,n] * What[n,j]      dW[n,j] = sum_t dY[t,n] * Xhat[t,j]
 * dY is bfloat16 (bit patterns), results in binary64.  Either output may be NULL. */
int qbo_qlinear_bwd_ste(const uint16_t *dY, const int8_t *xq, float clip, const uint8_t *codes,
                        const float *h, int bits, int64_t G, int64_t T, int64_t N, int64_t K,
                        double *dX, double *dW)
{
    int64_t rows;
    int L;
    float hx;
    if (!dY || !xq || !codes || !h || !bits_ok(bits)) return QBO_ERR_ARG;
    if (T <= 0 || N <= 0 || K <= 0 || G <= 0 || N % G || !(clip > 0.0f)) return QBO_ERR_ARG;
    L = (1 << bits) - 1;
    hx = clip / 255.0f;
    rows = N / G;
    if (dX) {
        int64_t t;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
        for (t = 0; t < T; ++t) {
            int64_t n, j;
            for (j = 0; j < K; ++j) dX[t * K + j] = 0.0;
            for (n = 0; n < N; ++n) {
                double g = bf16_to_double(dY[t * N + n]);
                double hg = (double)h[n / rows];
                for (j = 0; j < K; ++j)
                    dX[t * K + j] += g * (hg * (double)(2 * (int)codes[n * K + j] - L));
            }
        }
    }
    if (dW) {
        int64_t n;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
        for (n = 0; n < N; ++n) {
            int64_t t, j;
            for (j = 0; j < K; ++j) dW[n * K + j] = 0.0;
            for (t = 0; t < T; ++t) {
                double g = bf16_to_double(dY[t * N + n]);
                for (j = 0; j < K; ++j)
                    dW[n * K + j] += g * ((double)hx * (double)(2 * (int)xq[t * K + j] + 1));
            }
        }
    }
    return QBO_OK;
}

/* The same backward with the clamp's own derivative kept (App.: X' = Clamp(X, q0, q_{2^k-1}) comes before the
 * rounding; only the rounding is passed straight through): a value outside its range was moved to the range's
 * end and has derivative 0, one inside (ends included) has derivative 1.
 *   X [T,K] raw activations, range [-clip, +clip]  -> dX[t,j] = 0 where |X[t,j]| > clip     (NULL: no mask)
 *   W [N,K] raw weights, m[G] the group ranges     -> dW[n,j] = 0 where |W[n,j]| > m[g(n)]  (NULL: no mask) */
int qbo_qlinear_bwd_ste_masked(const uint16_t *dY, const int8_t *xq, float clip, const uint8_t *codes,
                               const float *h, int bits, int64_t G, int64_t T, int64_t N, int64_t K,
                               const float *X, const float *W, const float *m, double *dX, double *dW)
{
    int64_t i, rows;
    int rc = qbo_qlinear_bwd_ste(dY, xq, clip, codes, h, bits, G, T, N, K, dX, dW);
    if (rc != QBO_OK) return rc;
    if ((W == NULL) != (m == NULL)) return QBO_ERR_ARG;
    rows = N / G;
    if (dX && X)
        for (i = 0; i < T * K; ++i)
            if (fabsf(X[i]) > clip) dX[i] = 0.0;
    if (dW && W)
        for (i = 0; i < N * K; ++i)
            if (fabsf(W[i]) > m[(i / K) / rows]) dW[i] = 0.0;
    return QBO_OK;
}

/* Single entries of the two gradients, for full-size checks. */
int qbo_bwd_dx_sampled(const uint16_t *dY, const uint8_t *codes, const float *h, int bits,
                       int64_t G, int64_t T, int64_t N, int64_t K,
                       const int64_t *ts, const int64_t *js, int64_t count, double *out)
{
    int64_t i, rows;
    int L;
    if (!dY || !codes || !h || !ts || !js || !out || !bits_ok(bits) || G <= 0 || N % G) return QBO_ERR_ARG;
    L = (1 << bits) - 1;
    rows = N / G;
    for (i = 0; i < count; ++i) {
        int64_t n, t = ts[i], j = js[i];
        double s = 0.0;
        if (t < 0 || t >= T || j < 0 || j >= K) return QBO_ERR_ARG;
        for (n = 0; n < N; ++n)
            s += bf16_to_double(dY[t * N + n]) * ((double)h[n / rows] * (double)(2 * (int)codes[n * K + j] - L));
        out[i] = s;
    }
    return QBO_OK;
}

int qbo_bwd_dw_sampled(const uint16_t *dY, const int8_t *xq, float clip,
                       int64_t T, int64_t N, int64_t K,
                       const int64_t *ns, const int64_t *js, int64_t count, double *out)
{
    int64_t i;
    float hx;
    if (!dY || !xq || !ns || !js || !out || !(clip > 0.0f)) return QBO_ERR_ARG;
    hx = clip / 255.0f;
    for (i = 0; i < count; ++i) {
        int64_t t, n = ns[i], j = js[i];
        double s = 0.0;
        if (n < 0 || n >= N || j < 0 || j >= K) return QBO_ERR_ARG;
        for (t = 0; t < T; ++t)
            s += bf16_to_double(dY[t * N + n]) * ((double)hx * (double)(2 * (int)xq[t * K + j] + 1));
        out[i] = s;
    }
    return QBO_OK;
}

/* Embedding table (App. "Mixed Precision Quantization for Embedding": the output neurons,
 * i.e. the embedding dimension, are bucketed into groups; 4-bit word embeddings next to 8-bit
 * position embeddings).  E[V,d] fp32, k-bit codes (k = 4 or 8) with the same quantizer as the
 * weights, group g = columns [g*d/G, (g+1)*d/G) over all V rows. */
int qbo_embedding_quantize_bits(const float *E, int64_t V, int64_t d, int bits, int64_t G,
                                uint8_t *codes, float *h, float *m)
{
    int64_t g, cols;
    int L;
    if (!E || !codes || !h || !m || V <= 0 || d <= 0 || G <= 0 || d % G) return QBO_ERR_ARG;
    if (bits != 4 && bits != 8) return QBO_ERR_ARG;
    L = (1 << bits) - 1;
    cols = d / G;
    for (g = 0; g < G; ++g) {
        float mg = 0.0f, hg, delta;
        int64_t v, c;
        for (v = 0; v < V; ++v)
            for (c = 0; c < cols; ++c) {
                float a = fabsf(E[v * d + g * cols + c]);
                if (!isfinite(a)) return QBO_ERR_NONFINITE;
                if (a > mg) mg = a;
            }
        hg = (mg == 0.0f) ? 0.0f : mg / (float)L;
        delta = 2.0f * hg;
        m[g] = mg;
        h[g] = hg;
        for (v = 0; v < V; ++v)
            for (c = 0; c < cols; ++c) {
                int64_t at = v * d + g * cols + c;
                codes[at] = (uint8_t)quantize_one(E[at], mg, delta, L);
            }
    }
    return QBO_OK;
}

int qbo_embedding_quantize(const float *E, int64_t V, int64_t d, int64_t G,
                           uint8_t *codes, float *h, float *m)
{
    return qbo_embedding_quantize_bits(E, V, d, 8, G, codes, h, m);
}

/* Lookup with de-quantization: out[i,j] = h[g(j)] * (2*u[ids[i], j] - L), L = 2^k - 1, binary64. */
int qbo_embedding_gather_bits(const uint8_t *codes, const float *h, int64_t V, int64_t d, int bits, int64_t G,
                              const int64_t *ids, int64_t n_ids, double *out)
{
    int64_t i, j, cols;
    int L;
    if (!codes || !h || !ids || !out || V <= 0 || d <= 0 || G <= 0 || d % G || n_ids < 0) return QBO_ERR_ARG;
    if (bits != 4 && bits != 8) return QBO_ERR_ARG;
    L = (1 << bits) - 1;
    cols = d / G;
    for (i = 0; i < n_ids; ++i) {
        if (ids[i] < 0 || ids[i] >= V) return QBO_ERR_ARG;
        for (j = 0; j < d; ++j)
            out[i * d + j] = (double)h[j / cols] * (double)(2 * (int)codes[ids[i] * d + j] - L);
    }
    return QBO_OK;
}

int qbo_embedding_gather(const uint8_t *codes, const float *h, int64_t V, int64_t d, int64_t G,
                         const int64_t *ids, int64_t n_ids, double *out)
{
    return qbo_embedding_gather_bits(codes, h, V, d, 8, G, ids, n_ids, out);
}

int qbo_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- asymmetric group ranges -------------------------------------------------------------------------
 * The appendix states the quantizer for a general range [q0, q_{2^k-1}] (Delta = (q_{2^k-1} - q0)/(2^k - 1),
 * X^I = round((X' - q0)/Delta), Q(X) = Delta*X^I + q0); the hot path takes the symmetric [-m, +m].  Here the
 * range of a group is its own [min, max].  Each arithmetic step that decides a code is one binary32
 * operation, as in quantize_one.  A constant group (max == min) has Delta = 0, codes 0 and Q = q0.
 * out: codes[N,K], delta[G], q0[G], rs_w[N] = sum_j (u - 2^(k-1)) (the row sums the integer product uses). */
int qbo_quantize_groupwise_asym(const float *W, int64_t N, int64_t K, int bits, int64_t G, uint8_t *codes,
                                float *delta, float *q0, int32_t *rs_w)
{
    int64_t g, rows;
    int L, half;
    if (!W || !codes || !delta || !q0 || !rs_w || !bits_ok(bits)) return QBO_ERR_ARG;
    if (N <= 0 || K <= 0 || G <= 0 || N % G) return QBO_ERR_ARG;
    L = (1 << bits) - 1;
    half = 1 << (bits - 1);
    rows = N / G;
    for (g = 0; g < G; ++g) {
        const float *Wg = W + g * rows * K;
        uint8_t *cg = codes + g * rows * K;
        float lo = Wg[0], hi = Wg[0], d;
        int64_t i, r, j;
        for (i = 0; i < rows * K; ++i) {
            if (!isfinite(Wg[i])) return QBO_ERR_NONFINITE;
            if (Wg[i] < lo) lo = Wg[i];
            if (Wg[i] > hi) hi = Wg[i];
        }
        d = hi - lo;
        d = d / (float)L;
        delta[g] = d;
        q0[g] = lo;
        for (r = 0; r < rows; ++r) {
            int32_t acc = 0;
            for (j = 0; j < K; ++j) {
                int u = 0;
                if (d != 0.0f) {
                    float sft = Wg[r * K + j] - lo;   /* X' - q0; nothing to clamp: the range is the data's */
                    float t = sft / d;
                    u = (int)rintf(t);
                    if (u < 0) u = 0;
                    if (u > L) u = L;
                }
                cg[r * K + j] = (uint8_t)u;
                acc += u - half;
            }
            rs_w[g * rows + r] = acc;
        }
    }
    return QBO_OK;
}

/* The same quantizer with the range of every group given by the caller (App.: the range [q0, q_{2^k-1}] may be a
 * sub-interval of the data's [min, max]; X' = Clamp(X, q0, q_{2^k-1})): group g uses [lo[g], hi[g]], lo <= hi.
 * Weights outside are clamped first and so get the end codes.  Delta = fl(fl(hi - lo)/L), q0 = lo.
 * With lo = min and hi = max of the group this is qbo_quantize_groupwise_asym. */
int qbo_quantize_groupwise_asym_range(const float *W, int64_t N, int64_t K, int bits, int64_t G, const float *lo_in,
                                      const float *hi_in, uint8_t *codes, float *delta, float *q0, int32_t *rs_w)
{
    int64_t g, rows;
    int L, half;
    if (!W || !lo_in || !hi_in || !codes || !delta || !q0 || !rs_w || !bits_ok(bits)) return QBO_ERR_ARG;
    if (N <= 0 || K <= 0 || G <= 0 || N % G) return QBO_ERR_ARG;
    L = (1 << bits) - 1;
    half = 1 << (bits - 1);
    rows = N / G;
    for (g = 0; g < G; ++g) {
        const float *Wg = W + g * rows * K;
        uint8_t *cg = codes + g * rows * K;
        const float lo = lo_in[g], hi = hi_in[g];
        float d;
        int64_t r, j;
        if (!isfinite(lo) || !isfinite(hi) || lo > hi) return QBO_ERR_ARG;
        d = hi - lo;
        d = d / (float)L;
        delta[g] = d;
        q0[g] = lo;
        for (r = 0; r < rows; ++r) {
            int32_t acc = 0;
            for (j = 0; j < K; ++j) {
                int u = 0;
                float w = Wg[r * K + j];
                if (!isfinite(w)) return QBO_ERR_NONFINITE;
                if (d != 0.0f) {
                    float sft, t;
                    if (w < lo) w = lo;               /* X' = Clamp(X, q0, q_{2^k-1}) */
                    if (w > hi) w = hi;
                    sft = w - lo;                     /* X' - q0 */
                    t = sft / d;
                    u = (int)rintf(t);
                    if (u < 0) u = 0;
                    if (u > L) u = L;
                }
                cg[r * K + j] = (uint8_t)u;
                acc += u - half;
            }
            rs_w[g * rows + r] = acc;
        }
    }
    return QBO_OK;
}

/* Q(w) = Delta*u + q0 in binary64 from the binary32 Delta and q0. */
int qbo_dequantize_groupwise_asym(const uint8_t *codes, const float *delta, const float *q0, int64_t N, int64_t K,
                                  int64_t G, double *Wq)
{
    int64_t n, j, rows;
    if (!codes || !delta || !q0 || !Wq || N <= 0 || K <= 0 || G <= 0 || N % G) return QBO_ERR_ARG;
    rows = N / G;
    for (n = 0; n < N; ++n)
        for (j = 0; j < K; ++j)
            Wq[n * K + j] = (double)delta[n / rows] * (double)codes[n * K + j] + (double)q0[n / rows];
    return QBO_OK;
}

/* Forward with asymmetric weights: integer sums first, one de-quantization after (App., last paragraph).
 * With x' = xq (the activation level is h_x*(2x'+1)):
 *   S[t,n] = sum_j (2x'+1)*u[n,j]      R[t] = sum_j (2x'+1)
 *   Y[t,n] = h_x*(Delta_g*S + q0_g*R) (+ bias[n]),  evaluated in binary64 from the binary32 scales.
 * out: Y[T,N] fp32, S[T,N] int64 or NULL. */
int qbo_qlinear_fwd_asym(const int8_t *xq, float clip, const uint8_t *codes, const float *delta, const float *q0,
                         int64_t G, int64_t T, int64_t N, int64_t K, const float *bias, float *Y, int64_t *S_out)
{
    int64_t t, rows;
    float hx;
    if (!xq || !codes || !delta || !q0 || !Y || !(clip > 0.0f)) return QBO_ERR_ARG;
    if (T <= 0 || N <= 0 || K <= 0 || G <= 0 || N % G) return QBO_ERR_ARG;
    hx = clip / 255.0f;
    rows = N / G;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (t = 0; t < T; ++t) {
        int64_t n, j, R = 0;
        for (j = 0; j < K; ++j) R += 2 * (int)xq[t * K + j] + 1;
        for (n = 0; n < N; ++n) {
            int64_t S = 0;
            double y;
            for (j = 0; j < K; ++j) S += (int64_t)(2 * (int)xq[t * K + j] + 1) * (int64_t)codes[n * K + j];
            y = (double)hx * ((double)delta[n / rows] * (double)S + (double)q0[n / rows] * (double)R);
            if (bias) y += (double)bias[n];
            Y[t * N + n] = (float)y;
            if (S_out) S_out[t * N + n] = S;
        }
    }
    return QBO_OK;
}

/* The same with one activation scale per token (the dynamic range of qbo_quantize_act_dyn applied to the general
 * quantizer of the appendix): Y[t,n] = hx[t]*(Delta_g*S + q0_g*R) (+ bias[n]). */
int qbo_qlinear_fwd_asym_dyn(const int8_t *xq, const float *hx, const uint8_t *codes, const float *delta, const float *q0,
                             int64_t G, int64_t T, int64_t N, int64_t K, const float *bias, float *Y)
{
    int64_t t, rows;
    if (!xq || !hx || !codes || !delta || !q0 || !Y) return QBO_ERR_ARG;
    if (T <= 0 || N <= 0 || K <= 0 || G <= 0 || N % G) return QBO_ERR_ARG;
    rows = N / G;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (t = 0; t < T; ++t) {
        int64_t n, j, R = 0;
        for (j = 0; j < K; ++j) R += 2 * (int)xq[t * K + j] + 1;
        for (n = 0; n < N; ++n) {
            int64_t S = 0;
            double y;
            for (j = 0; j < K; ++j) S += (int64_t)(2 * (int)xq[t * K + j] + 1) * (int64_t)codes[n * K + j];
            y = (double)hx[t] * ((double)delta[n / rows] * (double)S + (double)q0[n / rows] * (double)R);
            if (bias) y += (double)bias[n];
            Y[t * N + n] = (float)y;
        }
    }
    return QBO_OK;
}

/* Straight-through backward with asymmetric weights: dX = dY * Q(W), dW as in qbo_qlinear_bwd_ste (it does
 * not involve the weights). */
int qbo_qlinear_bwd_dx_asym(const uint16_t *dY, const uint8_t *codes, const float *delta, const float *q0,
                            int64_t G, int64_t T, int64_t N, int64_t K, double *dX)
{
    int64_t t, rows;
    if (!dY || !codes || !delta || !q0 || !dX || T <= 0 || N <= 0 || K <= 0 || G <= 0 || N % G) return QBO_ERR_ARG;
    rows = N / G;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (t = 0; t < T; ++t) {
        int64_t n, j;
        for (j = 0; j < K; ++j) dX[t * K + j] = 0.0;
        for (n = 0; n < N; ++n) {
            double g = bf16_to_double(dY[t * N + n]);
            double d = (double)delta[n / rows], z = (double)q0[n / rows];
            for (j = 0; j < K; ++j) dX[t * K + j] += g * (d * (double)codes[n * K + j] + z);
        }
    }
    return QBO_OK;
}
