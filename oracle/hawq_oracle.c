/*
 * CPU oracle for the integer-only inference path of HAWQ-V3 ("Dyadic Neural
 * Network Quantization").
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, obviously-correct
 * definition that the HIP library is compared against.  It is used by the
 * tests, by the smoke check and by the benchmark's CPU-baseline leg, and by
 * nothing else; it shares no code with the HIP library.
 *
 * Every routine is the textbook definition written as nested loops.  Integer
 * arithmetic is exact and independent of summation order, so the definition
 * *is* the result: there is no blocking, fusion or reordering here.
 *
 * Pinned by tests/test_oracle_*.py against: exact rationals (dyadic rounding),
 * a pure-Python 7-loop convolution, float64 library convolution / matmul /
 * max-pool (exact at these magnitudes), the paper's printed residual rounding
 * example (Appendix G), the batch-norm folding identity (Appendix D), the
 * packed/unpacked encoding invariant, and the paper's Table 1 BOPS totals for
 * the network topology; the two-convolution block output additionally against
 * its composition from the single-convolution and residual-addition routines;
 * the INT32 window-sum pool against the float64 library average pool and exact
 * rationals, the per-branch concatenation against exact rationals and the
 * real-valued module output (Appendix E).  Parity unpinned (paper silent; fixed by the readings
 * stated in the design notes): tie-breaking direction of the rounding shift,
 * nibble order of packed 4-bit data, storage precision of the shortcut
 * tensor, the max-pool after the first convolution, the form of the global
 * average pool, the clamp ranges.
 *
 * Tensor layouts: activations NHWC, weights KRSC (K output channels, R x S
 * taps, C input channels), innermost axis contiguous.  4-bit tensors hold two
 * elements per byte along the innermost axis, even element in the low nibble.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { OR_U8 = 0, OR_S8 = 1, OR_U4 = 2, OR_S4 = 3, OR_S32 = 4 };
enum { OR_OK = 0, OR_ERR_ARG = 1, OR_ERR_OVERFLOW = 2, OR_ERR_ALLOC = 3 };

/* ---- dyadic requantisation (Section 3.1, the requantisation equation and DN) ----
 * The real scale S_w*S_h/S_a is replaced by the dyadic number b / 2^c, applied
 * as one integer multiply and one right shift.  The shift rounds to nearest,
 * ties toward +infinity:  rq(t) = floor(t*b / 2^c + 1/2).                        */
int64_t oracle_rq(int64_t t, int32_t b, int32_t c)
{
    int64_t prod = t * (int64_t)b;
    int64_t half = (int64_t)1 << (c - 1);
    return (prod + half) >> c; /* arithmetic shift == floor division by 2^c */
}

void oracle_rq_array(const int64_t *t, const int32_t *b, const int32_t *c, int64_t n, int64_t *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = oracle_rq(t[i], b[i], c[i]);
}

/* ---- element access: step 1 of the path, unpacking ---- */
static int is4(int dt) { return dt == OR_U4 || dt == OR_S4; }

/* Read logical element `i` of a dense tensor of type dt. */
static int32_t load_elem(const void *p, int dt, int64_t i)
{
    switch (dt) {
    case OR_U8: return ((const uint8_t *)p)[i];
    case OR_S8: return ((const int8_t *)p)[i];
    case OR_S32: return ((const int32_t *)p)[i];
    case OR_U4: {
        uint8_t byte = ((const uint8_t *)p)[i >> 1];
        return (i & 1) ? (byte >> 4) : (byte & 0xF);
    }
    default: { /* OR_S4: two's complement nibble */
        uint8_t byte = ((const uint8_t *)p)[i >> 1];
        int32_t n = (i & 1) ? (byte >> 4) : (byte & 0xF);
        return n >= 8 ? n - 16 : n;
    }
    }
}

/* Write logical element `i`.  The value must already be clamped to the type's
 * range by the caller's y_lo / y_hi.  4-bit stores are read-modify-write on a
 * byte, so callers zero the buffer first and never store 4-bit data in parallel
 * on the same byte. */
static void store_elem(void *p, int dt, int64_t i, int64_t v)
{
    switch (dt) {
    case OR_U8: ((uint8_t *)p)[i] = (uint8_t)v; break;
    case OR_S8: ((int8_t *)p)[i] = (int8_t)v; break;
    case OR_S32: ((int32_t *)p)[i] = (int32_t)v; break;
    default: {
        uint8_t *q = (uint8_t *)p + (i >> 1);
        uint8_t nib = (uint8_t)(v & 0xF);
        if (i & 1) *q = (uint8_t)((*q & 0x0F) | (nib << 4));
        else *q = (uint8_t)((*q & 0xF0) | nib);
    }
    }
}

static int type_range_ok(int dt, int64_t lo, int64_t hi)
{
    int64_t tlo, thi;
    switch (dt) {
    case OR_U8: tlo = 0; thi = 255; break;
    case OR_S8: tlo = -128; thi = 127; break;
    case OR_U4: tlo = 0; thi = 15; break;
    case OR_S4: tlo = -8; thi = 7; break;
    case OR_S32: tlo = INT32_MIN; thi = INT32_MAX; break;
    default: return 0;
    }
    return lo <= hi && lo >= tlo && hi <= thi;
}

/* Widen a whole tensor to int32 (the "unpack" step made explicit). */
static int32_t *widen(const void *p, int dt, int64_t n)
{
    int32_t *out = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
    if (!out) return NULL;
    for (int64_t i = 0; i < n; ++i) out[i] = load_elem(p, dt, i);
    return out;
}

void oracle_unpack(const void *p, int dt, int64_t n, int32_t *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = load_elem(p, dt, i);
}

/* ---- quantised convolution layer --------------------------------------------
 * Section 3.1 (quantised convolution with INT32 accumulation, then dyadic
 * requantisation), Appendix D (folded batch-norm gives an INT32 bias at scale
 * S_h*S_w that is added to the accumulator), Section 3.3 (residual: each
 * branch is rescaled by its own dyadic number, rounded separately, then the
 * integers are added -- Appendix G's worked example), Figure 1 (ReLU / clamp
 * to the next layer's range).
 *
 *   acc  = sum_{r,s,c} x[n, p*stride_h - pad_h + r, q*stride_w - pad_w + s, c] * w[k,r,s,c]
 *          (cross-correlation; taps outside the image contribute 0)
 *   t    = acc + bias[k]                                  (must fit int32)
 *   y    = rq(t, b[k], c[k])  [+ rq(res[n,p,q,k], res_b[k], res_c[k])]
 *   y    = max(y, 0) if relu;  y = min(max(y, y_lo), y_hi);  store as y_dt
 *
 * With y_dt == OR_S32 and b == NULL the layer stops after t (raw logits).
 * Returns OR_ERR_OVERFLOW if any accumulator or t leaves the int32 range.      */
int oracle_conv2d_int(int32_t N, int32_t H, int32_t W, int32_t C, int32_t K, int32_t R, int32_t S,
                      int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                      int x_dt, int w_dt, int y_dt, int res_dt,
                      const void *x, const void *w, const int32_t *bias,
                      const int32_t *b, const uint8_t *c,
                      const void *residual, const int32_t *res_b, const uint8_t *res_c,
                      int32_t relu, int64_t y_lo, int64_t y_hi, void *y)
{
    if (!x || !w || !bias || !y) return OR_ERR_ARG;
    if (N < 0 || H <= 0 || W <= 0 || C <= 0 || K <= 0 || R <= 0 || S <= 0 || stride_h <= 0 || stride_w <= 0 ||
        pad_h < 0 || pad_w < 0)
        return OR_ERR_ARG;
    if ((b == NULL) != (c == NULL)) return OR_ERR_ARG;
    if (b == NULL && (y_dt != OR_S32 || residual)) return OR_ERR_ARG;
    if (residual && (!res_b || !res_c)) return OR_ERR_ARG;
    if (!type_range_ok(y_dt, y_lo, y_hi)) return OR_ERR_ARG;
    if ((is4(x_dt) || is4(w_dt)) && (C % 2)) return OR_ERR_ARG;
    if (is4(y_dt) && (K % 2)) return OR_ERR_ARG;
    if (residual && is4(res_dt) && (K % 2)) return OR_ERR_ARG;
    if (H + 2 * pad_h < R || W + 2 * pad_w < S) return OR_ERR_ARG;
    const int32_t P = (H + 2 * pad_h - R) / stride_h + 1;
    const int32_t Q = (W + 2 * pad_w - S) / stride_w + 1;

    int32_t *xw = widen(x, x_dt, (int64_t)N * H * W * C);
    int32_t *ww = widen(w, w_dt, (int64_t)K * R * S * C);
    if (!xw || !ww) { free(xw); free(ww); return OR_ERR_ALLOC; }
    if (is4(y_dt)) memset(y, 0, (size_t)(((int64_t)N * P * Q * K) / 2));

    int overflow = 0;
    /* one thread per output pixel: all K channels of a pixel are written by the
     * same thread (and K is even for 4-bit outputs), so packed stores never race */
#pragma omp parallel for collapse(3) schedule(static) reduction(| : overflow)
    for (int32_t n = 0; n < N; ++n)
        for (int32_t p = 0; p < P; ++p)
            for (int32_t q = 0; q < Q; ++q)
                for (int32_t k = 0; k < K; ++k) {
                    int64_t acc = 0;
                    for (int32_t r = 0; r < R; ++r) {
                        const int32_t ih = p * stride_h - pad_h + r;
                        if (ih < 0 || ih >= H) continue;
                        for (int32_t s = 0; s < S; ++s) {
                            const int32_t iw = q * stride_w - pad_w + s;
                            if (iw < 0 || iw >= W) continue;
                            const int32_t *xp = xw + (((int64_t)n * H + ih) * W + iw) * C;
                            const int32_t *wp = ww + (((int64_t)k * R + r) * S + s) * C;
                            for (int32_t ci = 0; ci < C; ++ci) acc += (int64_t)xp[ci] * (int64_t)wp[ci];
                        }
                    }
                    if (acc > INT32_MAX || acc < INT32_MIN) overflow |= 1;
                    int64_t t = acc + (int64_t)bias[k];
                    if (t > INT32_MAX || t < INT32_MIN) overflow |= 1;
                    const int64_t o = (((int64_t)n * P + p) * Q + q) * K + k;
                    int64_t yv;
                    if (b == NULL) {
                        yv = t;
                    } else {
                        yv = oracle_rq(t, b[k], c[k]);
                        if (residual) yv += oracle_rq(load_elem(residual, res_dt, o), res_b[k], res_c[k]);
                        if (relu && yv < 0) yv = 0;
                        if (yv < y_lo) yv = y_lo;
                        if (yv > y_hi) yv = y_hi;
                    }
                    store_elem(y, y_dt, o, yv);
                }
    free(xw);
    free(ww);
    return overflow ? OR_ERR_OVERFLOW : OR_OK;
}

/* ---- block output with a convolution on both branches ------------------------
 * Section 3.3, the residual equation as Figure 2 (right) draws it for a block that
 * changes shape: the main branch ends in a convolution and the shortcut is a
 * convolution too, both accumulators stay INT32, each is rescaled by its own dyadic
 * number (rounded separately -- Appendix G's worked example) and the integers are added:
 *
 *   t_m = sum x[n, p*s_h - pad_h + r, q*s_w - pad_w + s, c] * w[k,r,s,c] + bias[k]
 *   t_s = sum xs[n, p*ss_h - pads_h + r, q*ss_w - pads_w + s, c] * ws[k,r,s,c] + bias_s[k]
 *   y   = clamp( relu?( rq(t_m, b[k], c[k]) + rq(t_s, b_s[k], c_s[k]) ) )
 *
 * dims  = { N, H, W, C, R, S, stride_h, stride_w, pad_h, pad_w }   (main branch)
 * dimss = {    Hs, Ws, Cs, Rs, Ss, stride_h, stride_w, pad_h, pad_w } (shortcut, same N)
 * Both convolutions must produce the same P x Q x K output.                      */
static int64_t conv_acc_one(const int32_t *xw, const int32_t *ww, int32_t n, int32_t p, int32_t q, int32_t k,
                            int32_t H, int32_t W, int32_t C, int32_t R, int32_t S, int32_t stride_h, int32_t stride_w,
                            int32_t pad_h, int32_t pad_w)
{
    int64_t acc = 0;
    for (int32_t r = 0; r < R; ++r) {
        const int32_t ih = p * stride_h - pad_h + r;
        if (ih < 0 || ih >= H) continue;
        for (int32_t s = 0; s < S; ++s) {
            const int32_t iw = q * stride_w - pad_w + s;
            if (iw < 0 || iw >= W) continue;
            const int32_t *xp = xw + (((int64_t)n * H + ih) * W + iw) * C;
            const int32_t *wp = ww + (((int64_t)k * R + r) * S + s) * C;
            for (int32_t ci = 0; ci < C; ++ci) acc += (int64_t)xp[ci] * (int64_t)wp[ci];
        }
    }
    return acc;
}

int oracle_conv2d_dual_int(const int32_t *dims, const int32_t *dimss, int32_t K,
                           int x_dt, int w_dt, int xs_dt, int ws_dt, int y_dt,
                           const void *x, const void *w, const int32_t *bias, const int32_t *b, const uint8_t *c,
                           const void *xs, const void *ws, const int32_t *bias_s, const int32_t *b_s, const uint8_t *c_s,
                           int32_t relu, int64_t y_lo, int64_t y_hi, void *y)
{
    if (!dims || !dimss || !x || !w || !bias || !b || !c || !xs || !ws || !bias_s || !b_s || !c_s || !y) return OR_ERR_ARG;
    const int32_t N = dims[0], H = dims[1], W = dims[2], C = dims[3], R = dims[4], S = dims[5];
    const int32_t sh = dims[6], sw = dims[7], ph = dims[8], pw = dims[9];
    const int32_t Hs = dimss[0], Ws = dimss[1], Cs = dimss[2], Rs = dimss[3], Ss = dimss[4];
    const int32_t ssh = dimss[5], ssw = dimss[6], psh = dimss[7], psw = dimss[8];
    if (N < 0 || K <= 0 || H <= 0 || W <= 0 || C <= 0 || R <= 0 || S <= 0 || sh <= 0 || sw <= 0 || ph < 0 || pw < 0) return OR_ERR_ARG;
    if (Hs <= 0 || Ws <= 0 || Cs <= 0 || Rs <= 0 || Ss <= 0 || ssh <= 0 || ssw <= 0 || psh < 0 || psw < 0) return OR_ERR_ARG;
    if (H + 2 * ph < R || W + 2 * pw < S || Hs + 2 * psh < Rs || Ws + 2 * psw < Ss) return OR_ERR_ARG;
    const int32_t P = (H + 2 * ph - R) / sh + 1, Q = (W + 2 * pw - S) / sw + 1;
    if (P != (Hs + 2 * psh - Rs) / ssh + 1 || Q != (Ws + 2 * psw - Ss) / ssw + 1) return OR_ERR_ARG;
    if (!type_range_ok(y_dt, y_lo, y_hi)) return OR_ERR_ARG;
    if ((is4(x_dt) || is4(w_dt)) && (C % 2)) return OR_ERR_ARG;
    if ((is4(xs_dt) || is4(ws_dt)) && (Cs % 2)) return OR_ERR_ARG;
    if (is4(y_dt) && (K % 2)) return OR_ERR_ARG;

    int32_t *xw = widen(x, x_dt, (int64_t)N * H * W * C);
    int32_t *ww = widen(w, w_dt, (int64_t)K * R * S * C);
    int32_t *xsw = widen(xs, xs_dt, (int64_t)N * Hs * Ws * Cs);
    int32_t *wsw = widen(ws, ws_dt, (int64_t)K * Rs * Ss * Cs);
    if (!xw || !ww || !xsw || !wsw) { free(xw); free(ww); free(xsw); free(wsw); return OR_ERR_ALLOC; }
    if (is4(y_dt)) memset(y, 0, (size_t)(((int64_t)N * P * Q * K) / 2));
    int overflow = 0;
#pragma omp parallel for collapse(3) schedule(static) reduction(| : overflow)
    for (int32_t n = 0; n < N; ++n)
        for (int32_t p = 0; p < P; ++p)
            for (int32_t q = 0; q < Q; ++q)
                for (int32_t k = 0; k < K; ++k) {
                    const int64_t t_m = conv_acc_one(xw, ww, n, p, q, k, H, W, C, R, S, sh, sw, ph, pw) + (int64_t)bias[k];
                    const int64_t t_s = conv_acc_one(xsw, wsw, n, p, q, k, Hs, Ws, Cs, Rs, Ss, ssh, ssw, psh, psw) + (int64_t)bias_s[k];
                    if (t_m > INT32_MAX || t_m < INT32_MIN || t_s > INT32_MAX || t_s < INT32_MIN) overflow |= 1;
                    int64_t yv = oracle_rq(t_m, b[k], c[k]) + oracle_rq(t_s, b_s[k], c_s[k]);
                    if (relu && yv < 0) yv = 0;
                    if (yv < y_lo) yv = y_lo;
                    if (yv > y_hi) yv = y_hi;
                    store_elem(y, y_dt, (((int64_t)n * P + p) * Q + q) * K + k, yv);
                }
    free(xw); free(ww); free(xsw); free(wsw);
    return overflow ? OR_ERR_OVERFLOW : OR_OK;
}

/* ---- fully connected layer / GEMM: the same layer with a 1x1 window ----------
 *   y[m, n] = epilogue( sum_k x[m,k] * w[n,k] + bias[n] )                        */
int oracle_gemm_int(int32_t M, int32_t Nout, int32_t Kdim, int x_dt, int w_dt, int y_dt,
                    const void *x, const void *w, const int32_t *bias, const int32_t *b, const uint8_t *c,
                    int32_t relu, int64_t y_lo, int64_t y_hi, void *y)
{
    return oracle_conv2d_int(1, 1, M, Kdim, Nout, 1, 1, 1, 1, 0, 0, x_dt, w_dt, y_dt, OR_U8, x, w, bias, b, c,
                             NULL, NULL, NULL, relu, y_lo, y_hi, y);
}

/* ---- stand-alone residual addition (Section 3.3, the residual equation) ------
 *   y = clamp( relu?( rq(m, m_b[k], m_c[k]) + rq(r, r_b[k], r_c[k]) ) )
 * m may be the INT32 main-branch accumulator or a stored low-bit tensor.       */
int oracle_residual_add_dyadic(int64_t n_pixels, int32_t K, int m_dt, int r_dt, int y_dt,
                               const void *m, const int32_t *m_b, const uint8_t *m_c,
                               const void *r, const int32_t *r_b, const uint8_t *r_c,
                               int32_t relu, int64_t y_lo, int64_t y_hi, void *y)
{
    if (!m || !m_b || !m_c || !r || !r_b || !r_c || !y) return OR_ERR_ARG;
    if (n_pixels < 0 || K <= 0) return OR_ERR_ARG;
    if (!type_range_ok(y_dt, y_lo, y_hi)) return OR_ERR_ARG;
    if ((is4(m_dt) || is4(r_dt) || is4(y_dt)) && (K % 2)) return OR_ERR_ARG;
    if (is4(y_dt)) memset(y, 0, (size_t)((n_pixels * K) / 2));
#pragma omp parallel for schedule(static)
    for (int64_t px = 0; px < n_pixels; ++px)
        for (int32_t k = 0; k < K; ++k) {
            const int64_t o = px * K + k;
            int64_t yv = oracle_rq(load_elem(m, m_dt, o), m_b[k], m_c[k]) +
                         oracle_rq(load_elem(r, r_dt, o), r_b[k], r_c[k]);
            if (relu && yv < 0) yv = 0;
            if (yv < y_lo) yv = y_lo;
            if (yv > y_hi) yv = y_hi;
            store_elem(y, y_dt, o, yv);
        }
    return OR_OK;
}

/* ---- integer global average pool (Appendix E: pooling is done in INT32; no
 * integer division anywhere, so 1/(H*W) is folded into the dyadic multiplier) --
 *   s[n,k] = sum_{h,w} x[n,h,w,k]   (INT32);   y[n,k] = clamp(rq(s, b[k], c[k]))  */
int oracle_avgpool_int(int32_t N, int32_t H, int32_t W, int32_t C, int x_dt, int y_dt, const void *x,
                       const int32_t *b, const uint8_t *c, int64_t y_lo, int64_t y_hi, void *y)
{
    if (!x || !b || !c || !y) return OR_ERR_ARG;
    if (N < 0 || H <= 0 || W <= 0 || C <= 0) return OR_ERR_ARG;
    if (!type_range_ok(y_dt, y_lo, y_hi)) return OR_ERR_ARG;
    if ((is4(x_dt) || is4(y_dt)) && (C % 2)) return OR_ERR_ARG;
    if (is4(y_dt)) memset(y, 0, (size_t)(((int64_t)N * C) / 2));
    for (int32_t n = 0; n < N; ++n)
        for (int32_t k = 0; k < C; ++k) {
            int64_t s = 0;
            for (int32_t h = 0; h < H; ++h)
                for (int32_t wv = 0; wv < W; ++wv) s += load_elem(x, x_dt, (((int64_t)n * H + h) * W + wv) * C + k);
            if (s > INT32_MAX || s < INT32_MIN) return OR_ERR_OVERFLOW;
            int64_t yv = oracle_rq(s, b[k], c[k]);
            if (yv < y_lo) yv = y_lo;
            if (yv > y_hi) yv = y_hi;
            store_elem(y, y_dt, (int64_t)n * C + k, yv);
        }
    return OR_OK;
}

/* ---- max pool 3x3, stride 2, padding 1 (the pool after the first convolution
 * of every ResNet; the paper never discusses it -- it is an integer maximum over
 * the in-image taps, which commutes with the monotone requantiser).  The output
 * is clamped to [y_lo, y_hi] so an 8-bit tensor can be stored as 4-bit.         */
int oracle_maxpool_int(int32_t N, int32_t H, int32_t W, int32_t C, int x_dt, int y_dt, const void *x,
                       int64_t y_lo, int64_t y_hi, void *y)
{
    if (!x || !y) return OR_ERR_ARG;
    if (N < 0 || H <= 0 || W <= 0 || C <= 0) return OR_ERR_ARG;
    if (!type_range_ok(y_dt, y_lo, y_hi)) return OR_ERR_ARG;
    if ((is4(x_dt) || is4(y_dt)) && (C % 2)) return OR_ERR_ARG;
    const int32_t P = (H + 2 - 3) / 2 + 1, Q = (W + 2 - 3) / 2 + 1;
    if (is4(y_dt)) memset(y, 0, (size_t)(((int64_t)N * P * Q * C) / 2));
#pragma omp parallel for collapse(3) schedule(static)
    for (int32_t n = 0; n < N; ++n)
        for (int32_t p = 0; p < P; ++p)
            for (int32_t q = 0; q < Q; ++q)
                for (int32_t k = 0; k < C; ++k) {
                    int64_t best = INT64_MIN;
                    for (int32_t r = 0; r < 3; ++r) {
                        const int32_t ih = 2 * p - 1 + r;
                        if (ih < 0 || ih >= H) continue;
                        for (int32_t s = 0; s < 3; ++s) {
                            const int32_t iw = 2 * q - 1 + s;
                            if (iw < 0 || iw >= W) continue;
                            int64_t v = load_elem(x, x_dt, (((int64_t)n * H + ih) * W + iw) * C + k);
                            if (v > best) best = v;
                        }
                    }
                    if (best < y_lo) best = y_lo;
                    if (best > y_hi) best = y_hi;
                    store_elem(y, y_dt, (((int64_t)n * P + p) * Q + q) * C + k, best);
                }
    return OR_OK;
}

/* ---- pooling carried in INT32 (Appendix E: the pooling branch of an Inception module works on the INT32
 * feature map, because pooling 4-bit data loses information).  A window SUM; the divisor of an average
 * pool (R*S, padding counted, as in the Inception modules) is folded into the dyadic number that follows
 * -- the one given here, or the concatenation's (no integer division anywhere).
 *   s[n,p,q,k] = sum over the in-image taps of x[n, p*stride_h - pad_h + r, q*stride_w - pad_w + t, k]   (INT32)
 *   y = s                              if b == NULL (y_dt must be OR_S32)
 *   y = clamp(rq(s, b[k], c[k]))       otherwise                                                        */
int oracle_pool2d_sum_int(int32_t N, int32_t H, int32_t W, int32_t C, int32_t R, int32_t S, int32_t stride_h, int32_t stride_w,
                          int32_t pad_h, int32_t pad_w, int x_dt, int y_dt, const void *x, const int32_t *b, const uint8_t *c,
                          int64_t y_lo, int64_t y_hi, void *y)
{
    if (!x || !y) return OR_ERR_ARG;
    if (N < 0 || H <= 0 || W <= 0 || C <= 0 || R <= 0 || S <= 0 || stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0)
        return OR_ERR_ARG;
    if ((b == NULL) != (c == NULL)) return OR_ERR_ARG;
    if (b == NULL && y_dt != OR_S32) return OR_ERR_ARG;
    if (b != NULL && !type_range_ok(y_dt, y_lo, y_hi)) return OR_ERR_ARG;
    if ((is4(x_dt) || is4(y_dt)) && (C % 2)) return OR_ERR_ARG;
    if (H + 2 * pad_h < R || W + 2 * pad_w < S) return OR_ERR_ARG;
    const int32_t P = (H + 2 * pad_h - R) / stride_h + 1, Q = (W + 2 * pad_w - S) / stride_w + 1;
    if (is4(y_dt)) memset(y, 0, (size_t)(((int64_t)N * P * Q * C) / 2));
    int overflow = 0;
    for (int32_t n = 0; n < N; ++n)
        for (int32_t p = 0; p < P; ++p)
            for (int32_t q = 0; q < Q; ++q)
                for (int32_t k = 0; k < C; ++k) {
                    int64_t sum = 0;
                    for (int32_t r = 0; r < R; ++r) {
                        const int32_t ih = p * stride_h - pad_h + r;
                        if (ih < 0 || ih >= H) continue;
                        for (int32_t t = 0; t < S; ++t) {
                            const int32_t iw = q * stride_w - pad_w + t;
                            if (iw < 0 || iw >= W) continue;
                            sum += load_elem(x, x_dt, (((int64_t)n * H + ih) * W + iw) * C + k);
                        }
                    }
                    if (sum > INT32_MAX || sum < INT32_MIN) overflow = 1;
                    int64_t yv = sum;
                    if (b != NULL) {
                        yv = oracle_rq(sum, b[k], c[k]);
                        if (yv < y_lo) yv = y_lo;
                        if (yv > y_hi) yv = y_hi;
                    }
                    store_elem(y, y_dt, (((int64_t)n * P + p) * Q + q) * C + k, yv);
                }
    return overflow ? OR_ERR_OVERFLOW : OR_OK;
}

/* ---- concatenation with one dyadic number per branch (Appendix E: the branches of an Inception module end
 * at different scales; each is brought to the output scale S_a by its own DN(S_i / S_a), then the channels are
 * laid side by side):
 *   y[p, off_i + k] = clamp(rq(q_i[p,k], b_i[k], c_i[k])),   off_i = K_0 + ... + K_(i-1)
 * q_i: [n_pixels, K_i] of type dt[i] (an INT32 accumulator / pooled sum, or a stored low-bit tensor).      */
int oracle_concat_dyadic(int64_t n_pixels, int32_t n_branches, const int32_t *K, const int *dt, const void *const *q,
                         const int32_t *const *b, const uint8_t *const *c, int y_dt, int64_t y_lo, int64_t y_hi, void *y)
{
    if (!K || !dt || !q || !b || !c || !y || n_branches <= 0 || n_pixels < 0) return OR_ERR_ARG;
    if (!type_range_ok(y_dt, y_lo, y_hi)) return OR_ERR_ARG;
    int64_t Kt = 0;
    for (int32_t i = 0; i < n_branches; ++i) {
        if (K[i] <= 0 || !q[i] || !b[i] || !c[i]) return OR_ERR_ARG;
        if ((is4(dt[i]) || is4(y_dt)) && (K[i] % 2)) return OR_ERR_ARG;
        Kt += K[i];
    }
    if (is4(y_dt)) memset(y, 0, (size_t)((n_pixels * Kt) / 2));
    int64_t off = 0;
    for (int32_t i = 0; i < n_branches; ++i) {
        for (int64_t p = 0; p < n_pixels; ++p)
            for (int32_t k = 0; k < K[i]; ++k) {
                int64_t yv = oracle_rq(load_elem(q[i], dt[i], p * K[i] + k), b[i][k], c[i][k]);
                if (yv < y_lo) yv = y_lo;
                if (yv > y_hi) yv = y_hi;
                store_elem(y, y_dt, p * Kt + off + k, yv);
            }
        off += K[i];
    }
    return OR_OK;
}
