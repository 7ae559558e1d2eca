// C interface: host-side argument validation and dispatch.  Nothing here touches device memory.
#include "common.h"

using namespace hawq;

namespace {

bool dtype_range(int dt, int64_t &lo, int64_t &hi) {
    switch (dt) {
    case HAWQ_U8: lo = 0; hi = 255; return true;
    case HAWQ_S8: lo = -128; hi = 127; return true;
    case HAWQ_U4: lo = 0; hi = 15; return true;
    case HAWQ_S4: lo = -8; hi = 7; return true;
    case HAWQ_S32: lo = INT32_MIN; hi = INT32_MAX; return true;
    default: return false;
    }
}

bool low_bit(int dt) { return dt == HAWQ_U8 || dt == HAWQ_S8 || dt == HAWQ_U4 || dt == HAWQ_S4; }

hawq_status check_clamp(int y_dt, int32_t y_lo, int32_t y_hi) {
    int64_t lo, hi;
    if (!dtype_range(y_dt, lo, hi)) return HAWQ_ERR_DTYPE;
    if (y_lo > y_hi || y_lo < lo || y_hi > hi) return HAWQ_ERR_RANGE;
    return HAWQ_OK;
}

const int64_t kMaxBytes = (int64_t)1 << 31;

}  // namespace

namespace hawq {

// Validate a convolution request and fill the kernel argument block.  x_hi_out receives the
// effective activation bound.  Shared by hawq_conv2d_int, hawq_gemm_int and the network plan.
hawq_status make_conv_args(const hawq_conv_desc *d, const void *x, const void *w, const int32_t *bias, const int32_t *b,
                           const uint8_t *c, const void *residual, const int32_t *res_b, const uint8_t *res_c, void *y,
                           bool check_pointers, ConvArgs &a, int &x_hi_out) {
    if (!d) return HAWQ_ERR_NULL;
    if (check_pointers) {
        if (!x || !w || !bias || !y) return HAWQ_ERR_NULL;
        if ((b == nullptr) != (c == nullptr)) return HAWQ_ERR_NULL;
        if (residual && (!res_b || !res_c)) return HAWQ_ERR_NULL;
    }
    if (d->N < 0 || d->H <= 0 || d->W <= 0 || d->C <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0 || d->stride_h <= 0 ||
        d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0)
        return HAWQ_ERR_SHAPE;
    if ((int64_t)d->H + 2 * (int64_t)d->pad_h < d->R || (int64_t)d->W + 2 * (int64_t)d->pad_w < d->S) return HAWQ_ERR_SHAPE;
    // operand types: weights and activations of a layer share one bit width (Section 3.4)
    if (d->x_dtype == HAWQ_U8 || d->x_dtype == HAWQ_S8) {
        if (d->w_dtype != HAWQ_S8) return HAWQ_ERR_DTYPE;
    } else if (d->x_dtype == HAWQ_U4) {
        if (d->w_dtype != HAWQ_S4) return HAWQ_ERR_DTYPE;
    } else {
        return HAWQ_ERR_DTYPE;
    }
    int64_t tlo, thi;
    if (!dtype_range(d->y_dtype, tlo, thi)) return HAWQ_ERR_DTYPE;
    if (residual && !low_bit(d->res_dtype)) return HAWQ_ERR_DTYPE;
    const bool raw = (b == nullptr) && check_pointers;
    if (raw && (d->y_dtype != HAWQ_S32 || residual)) return HAWQ_ERR_DTYPE;
    if (is4(d->x_dtype) && (d->C & 1)) return HAWQ_ERR_SHAPE;
    if (is4(d->y_dtype) && (d->K & 1)) return HAWQ_ERR_SHAPE;
    if (residual && is4(d->res_dtype) && (d->K & 1)) return HAWQ_ERR_SHAPE;
    if (!raw) {
        hawq_status st = check_clamp(d->y_dtype, d->y_lo, d->y_hi);
        if (st != HAWQ_OK) return st;
    }
    // activation bound and the static INT32 overflow check
    const int x_type_hi = d->x_dtype == HAWQ_U8 ? 255 : (d->x_dtype == HAWQ_S8 ? 128 : 15);
    if (d->x_hi < 0 || d->x_hi > x_type_hi) return HAWQ_ERR_RANGE;
    const int x_hi = d->x_hi == 0 ? x_type_hi : d->x_hi;
    const int64_t w_hi = d->w_dtype == HAWQ_S8 ? 128 : 8;
    const int64_t kdim = (int64_t)d->R * d->S * d->C;
    if (kdim * x_hi * w_hi >= ((int64_t)1 << 31) - ((int64_t)1 << 24)) return HAWQ_ERR_OVERFLOW;

    const int64_t P = ((int64_t)d->H + 2 * d->pad_h - d->R) / d->stride_h + 1;
    const int64_t Q = ((int64_t)d->W + 2 * d->pad_w - d->S) / d->stride_w + 1;
    const int64_t M = (int64_t)d->N * P * Q;
    if (M >= kMaxBytes) return HAWQ_ERR_UNSUPPORTED;
    if (tensor_bytes((int64_t)d->N * d->H * d->W * d->C, d->x_dtype) >= kMaxBytes) return HAWQ_ERR_UNSUPPORTED;
    if (tensor_bytes(M * d->K, d->y_dtype) >= kMaxBytes) return HAWQ_ERR_UNSUPPORTED;
    if (tensor_bytes(kdim * d->K, d->w_dtype) >= kMaxBytes) return HAWQ_ERR_UNSUPPORTED;

    a.x = (const uint8_t *)x; a.w = (const uint8_t *)w; a.bias = bias; a.b = b; a.c = c;
    a.res = (const uint8_t *)residual; a.res_b = residual ? res_b : nullptr; a.res_c = residual ? res_c : nullptr;
    a.y = (uint8_t *)y;
    a.xs = nullptr; a.ws = nullptr; a.bias_s = nullptr; a.b_s = nullptr; a.c_s = nullptr;
    a.Hs = a.Ws = a.Cs = 0; a.stride_sh = a.stride_sw = 1; a.xs_dt = HAWQ_U8; a.ws_dt = HAWQ_S8; a.mid_s8 = 0; a.corun = 0; a.ws_t = nullptr; a.ws_f = nullptr; a.dual16 = 0;
    a.w_t = (d->w_blocked != nullptr && ((uintptr_t)d->w_blocked & 15) == 0) ? d->w_blocked : nullptr;
    a.w_f = (d->w_fragments != nullptr && ((uintptr_t)d->w_fragments & 15) == 0) ? d->w_fragments : nullptr;
    a.N = d->N; a.H = d->H; a.W = d->W; a.C = d->C; a.K = d->K; a.R = d->R; a.S = d->S;
    a.stride_h = d->stride_h; a.stride_w = d->stride_w; a.pad_h = d->pad_h; a.pad_w = d->pad_w;
    a.P = (int32_t)P; a.Q = (int32_t)Q; a.M = (int32_t)M;
    a.x_dt = d->x_dtype; a.w_dt = d->w_dtype; a.y_dt = d->y_dtype; a.res_dt = d->res_dtype;
    a.lo = (d->relu && d->y_lo < 0) ? 0 : d->y_lo;
    a.hi = d->y_hi;
    if (raw) { a.lo = INT32_MIN; a.hi = INT32_MAX; }
    // ReLU with a clamp interval entirely below zero: max(y,0) then min(.,hi) gives hi
    if (d->relu && d->y_hi < 0) { a.lo = d->y_hi; a.hi = d->y_hi; }
    x_hi_out = x_hi;
    return HAWQ_OK;
}

// The resident-pixel kernel's view of a validated 3x3 layer a1 (weights a1.w_f) and, when a2 is given, of the 1x1 layer
// that consumes its output in the same launch (weights w2f; a2's x / y-of-a1 pointers are not used).
bool make_rp_args(const ConvArgs &a1, int x_hi, const ConvArgs *a2, const void *w2f, RpArgs &r) {
    if (a1.R != 3 || a1.S != 3 || a1.stride_h != 1 || a1.stride_w != 1 || a1.pad_h != 1 || a1.pad_w != 1) return false;
    if (a1.w_f == nullptr || a1.b == nullptr || a1.xs != nullptr) return false;
    if ((uintptr_t)a1.x & 15) return false;
    r = RpArgs{};
    r.corun = a1.corun;
    r.x = a1.x; r.N = a1.N; r.H = a1.H; r.W = a1.W; r.C = a1.C; r.M = a1.M;
    r.w1f = (const uint8_t *)a1.w_f; r.bias1 = a1.bias; r.b1 = a1.b; r.c1 = a1.c; r.K1 = a1.K; r.lo1 = a1.lo; r.hi1 = a1.hi;
    if (a1.x_dt == HAWQ_U4) {   // packed 4-bit operands: plain form, no shortcut, 8-bit or packed unsigned 4-bit output
        if (a1.w_dt != HAWQ_S4 || a2 != nullptr || a1.res != nullptr) return false;
        if (a1.y_dt != HAWQ_U8 && a1.y_dt != HAWQ_S8 && a1.y_dt != HAWQ_U4) return false;
        if ((uintptr_t)a1.y & 15) return false;
        r.pk = 1; r.y4 = a1.y_dt == HAWQ_U4; r.y = a1.y; r.res_dt = HAWQ_U8;
        return conv_rp_shape_ok(r, false);
    }
    if (a1.w_dt != HAWQ_S8) return false;
    if (a1.x_dt == HAWQ_U8 ? x_hi > 127 : a1.x_dt != HAWQ_S8) return false;
    if (a1.y_dt != HAWQ_U8 && a1.y_dt != HAWQ_S8) return false;
    if (a2 == nullptr) {
        if (a1.res != nullptr && a1.res_dt != HAWQ_U8 && a1.res_dt != HAWQ_S8) return false;
        if (((uintptr_t)a1.y | (uintptr_t)a1.res) & 15) return false;
        r.res = a1.res; r.res_b = a1.res_b; r.res_c = a1.res_c; r.res_dt = a1.res_dt; r.y = a1.y;
        return conv_rp_shape_ok(r, false);
    }
    // the intermediate tensor becomes the signed matrix operand of the second convolution
    if (a1.res != nullptr || a1.lo < -128 || a1.hi > 127) return false;
    if (a2->R != 1 || a2->S != 1 || a2->stride_h != 1 || a2->stride_w != 1 || a2->pad_h != 0 || a2->pad_w != 0) return false;
    if (a2->N != a1.N || a2->H != a1.H || a2->W != a1.W || a2->C != a1.K || a2->x_dt != a1.y_dt || a2->w_dt != HAWQ_S8) return false;
    if (a2->b == nullptr || a2->res == nullptr || a2->xs != nullptr || w2f == nullptr) return false;
    if ((a2->y_dt != HAWQ_U8 && a2->y_dt != HAWQ_S8) || (a2->res_dt != HAWQ_U8 && a2->res_dt != HAWQ_S8)) return false;
    if (((uintptr_t)a2->y | (uintptr_t)a2->res | (uintptr_t)w2f) & 15) return false;
    r.res = a2->res; r.res_b = a2->res_b; r.res_c = a2->res_c; r.res_dt = a2->res_dt; r.y = a2->y;
    r.w2f = (const uint8_t *)w2f; r.bias2 = a2->bias; r.b2 = a2->b; r.c2 = a2->c; r.K2 = a2->K; r.lo2 = a2->lo; r.hi2 = a2->hi;
    return conv_rp_shape_ok(r, true);
}

// The resident-pixel 1x1 kernel's view of a validated request: one convolution (weights a.w_f) with an optional 8-bit
// shortcut tensor, or -- a.xs set -- the two-convolution block output (weights a.w_f and a.ws_f) when the caller vouches
// for the 16-bit form (a.dual16).
bool make_rp1_args(const ConvArgs &a, int x_hi, int xs_hi, Rp1Args &r) {
    if (a.R != 1 || a.S != 1 || a.stride_h != 1 || a.stride_w != 1 || a.pad_h != 0 || a.pad_w != 0) return false;
    if (a.w_f == nullptr || a.b == nullptr || a.w_dt != HAWQ_S8) return false;
    if (a.x_dt == HAWQ_U8 ? x_hi > 127 : a.x_dt != HAWQ_S8) return false;
    if (a.y_dt != HAWQ_U8 && a.y_dt != HAWQ_S8) return false;
    if (((uintptr_t)a.x | (uintptr_t)a.y | (uintptr_t)a.w_f) & 15) return false;
    if ((int64_t)a.M * a.C >= kMaxBytes || (int64_t)a.M * a.K >= kMaxBytes) return false;
    r = Rp1Args{};
    r.corun = a.corun;
    r.x = a.x; r.M = a.M; r.C = a.C;
    r.wf = (const uint8_t *)a.w_f; r.bias = a.bias; r.b = a.b; r.c = a.c; r.K = a.K; r.lo = a.lo; r.hi = a.hi;
    r.y = a.y; r.res_dt = HAWQ_U8;
    if (a.xs == nullptr) {
        if (a.res != nullptr) {
            if (a.res_dt != HAWQ_U8 && a.res_dt != HAWQ_S8) return false;
            if ((uintptr_t)a.res & 15) return false;
            r.res = a.res; r.res_b = a.res_b; r.res_c = a.res_c; r.res_dt = a.res_dt;
        }
        return conv_rp1_shape_ok(r);
    }
    if (!a.dual16 || a.ws_f == nullptr || a.res != nullptr || a.b_s == nullptr || a.ws_dt != HAWQ_S8) return false;
    if (a.xs_dt == HAWQ_U8 ? xs_hi > 127 : a.xs_dt != HAWQ_S8) return false;
    if (((uintptr_t)a.xs | (uintptr_t)a.ws_f) & 15) return false;
    if (a.mid_s8 && (a.res_b == nullptr || a.res_c == nullptr)) return false;
    r.xs = a.xs; r.wsf = (const uint8_t *)a.ws_f; r.bias_s = a.bias_s; r.b_s = a.b_s; r.c_s = a.c_s;
    r.Cs = a.Cs; r.PQ = a.P * a.Q; r.Q = a.Q; r.Hs = a.Hs; r.Ws = a.Ws; r.sh = a.stride_sh; r.sw = a.stride_sw;
    r.mid_s8 = a.mid_s8; r.res_b = a.res_b; r.res_c = a.res_c;
    r.xs_bytes = (int64_t)a.N * a.Hs * a.Ws * a.Cs;
    if (r.xs_bytes >= kMaxBytes) return false;
    return conv_rp1_shape_ok(r);
}

hawq_status dispatch_conv(const ConvArgs &a, int x_hi, hipStream_t s) {
    if (a.M == 0) return HAWQ_OK;
    if (a.x_dt == HAWQ_U8 && x_hi > 127 && gemm_splitk_eligible(a)) return launch_gemm_splitk(a, x_hi, s);
    if (conv_pw_eligible(a, x_hi)) return launch_conv_pw(a, s);
    if (tile_override() == 0 && conv_pws_eligible(a, x_hi)) return launch_conv_pws(a, s);
    if (tile_override() == 0 && conv3x3_c64_eligible(a, x_hi)) return launch_conv3x3_c64(a, s);
    if (tile_override() == 0 && a.w_f != nullptr) {
        RpArgs r;
        if (make_rp_args(a, x_hi, nullptr, nullptr, r)) return launch_conv_rp(r, false, s);
        Rp1Args r1;
        if (make_rp1_args(a, x_hi, 0, r1)) return launch_conv_rp1(r1, s);
    }
    if (conv_mfma_eligible(a, x_hi)) return launch_conv_mfma(a, s);
    return launch_conv_direct(a, s);
}

// Validate a two-convolution block output and fill the kernel argument block (main branch as make_conv_args; the
// shortcut convolution's fields from its own descriptor).
hawq_status make_dual_args(const hawq_conv_desc *d, const void *x, const void *w, const int32_t *bias, const int32_t *b,
                           const uint8_t *c, const hawq_conv_desc *ds, const void *xs, const void *ws, const int32_t *bias_s,
                           const int32_t *b_s, const uint8_t *c_s, void *y, bool check_pointers, ConvArgs &a, int &x_hi, int &xs_hi) {
    if (!d || !ds) return HAWQ_ERR_NULL;
    hawq_conv_desc dm = *d;
    dm.res_dtype = HAWQ_U8;
    hawq_status st = make_conv_args(&dm, x, w, bias, b, c, nullptr, nullptr, nullptr, y, check_pointers, a, x_hi);
    if (st != HAWQ_OK) return st;
    if (d->y_dtype == HAWQ_S32) return HAWQ_ERR_DTYPE;   // the block output is a requantised tensor
    // the shortcut convolution on its own terms: operand types, overflow bound, sizes (its output fields are the block's)
    hawq_conv_desc dsc = *ds;
    dsc.y_dtype = d->y_dtype; dsc.relu = d->relu; dsc.y_lo = d->y_lo; dsc.y_hi = d->y_hi; dsc.res_dtype = HAWQ_U8;
    ConvArgs t;
    st = make_conv_args(&dsc, xs, ws, bias_s, b_s, c_s, nullptr, nullptr, nullptr, y, check_pointers, t, xs_hi);
    if (st != HAWQ_OK) return st;
    if (t.R != 1 || t.S != 1 || t.pad_h != 0 || t.pad_w != 0) return HAWQ_ERR_SHAPE;
    if (t.N != a.N || t.P != a.P || t.Q != a.Q || t.K != a.K) return HAWQ_ERR_SHAPE;
    a.xs = t.x; a.ws = t.w; a.bias_s = t.bias; a.b_s = t.b; a.c_s = t.c;
    a.ws_t = t.w_t;      // (the shortcut's blocked / fragment-ordered weights, if its descriptor names them)
    a.ws_f = t.w_f;
    a.Hs = t.H; a.Ws = t.W; a.Cs = t.C; a.stride_sh = t.stride_h; a.stride_sw = t.stride_w; a.xs_dt = t.x_dt; a.ws_dt = t.w_dt;
    return HAWQ_OK;
}

hawq_status dispatch_conv_dual(const ConvArgs &a, int x_hi, int xs_hi, hipStream_t s) {
    if (a.M == 0) return HAWQ_OK;
    if (conv_pws_dual_eligible(a, x_hi, xs_hi)) return launch_conv_pws_dual(a, s);
    if (tile_override() == 0 && a.w_f != nullptr && a.ws_f != nullptr) {
        Rp1Args r1;
        if (make_rp1_args(a, x_hi, xs_hi, r1)) return launch_conv_rp1(r1, s);
    }
    if (conv_mfma_dual_eligible(a, x_hi, xs_hi)) return launch_conv_mfma_dual(a, s);
    return launch_conv_direct(a, s);
}

}  // namespace hawq

#ifdef HAWQ_RP_TIMING
static long long *g_rp_timing = nullptr;
extern "C" void hawq_debug_set_rp_timing(void *p) { g_rp_timing = (long long *)p; }
#endif

extern "C" {

size_t hawq_conv_blocked_weights_bytes(const hawq_conv_desc *desc) {
    if (!desc || desc->K <= 0 || desc->R <= 0 || desc->S <= 0 || desc->C <= 0) return 0;
    const bool four = hawq::is4(desc->w_dtype);
    if (desc->C % (four ? 128 : 64) != 0) return 0;
    const int64_t row = hawq::tensor_bytes((int64_t)desc->R * desc->S * desc->C, desc->w_dtype);
    return (size_t)((desc->K + 63) / 64) * (size_t)row * 64;
}

hawq_status hawq_conv_block_weights(const hawq_conv_desc *desc, const void *w, void *w_blocked, void *stream) {
    if (!desc || !w || !w_blocked) return HAWQ_ERR_NULL;
    if (hawq_conv_blocked_weights_bytes(desc) == 0) return HAWQ_ERR_UNSUPPORTED;
    if (((uintptr_t)w | (uintptr_t)w_blocked) & 15) return HAWQ_ERR_UNSUPPORTED;
    const int64_t row = hawq::tensor_bytes((int64_t)desc->R * desc->S * desc->C, desc->w_dtype);
    return hawq::launch_block_weights(w, w_blocked, desc->K, row, (hipStream_t)stream);
}

size_t hawq_conv_fragment_weights_bytes(const hawq_conv_desc *desc) {
    if (!desc || desc->K <= 0 || desc->R <= 0 || desc->S <= 0 || desc->C <= 0) return 0;
    if ((desc->w_dtype != HAWQ_S4 && desc->w_dtype != HAWQ_S8) || desc->C % 64 != 0) return 0;
    return (size_t)((desc->K + 31) / 32) * 32 * (size_t)desc->R * desc->S * desc->C;   // (4-bit weights are expanded to bytes)
}

hawq_status hawq_conv_fragment_weights(const hawq_conv_desc *desc, const void *w, void *w_fragments, void *stream) {
    if (!desc || !w || !w_fragments) return HAWQ_ERR_NULL;
    const size_t bytes = hawq_conv_fragment_weights_bytes(desc);
    if (bytes == 0 || bytes >= (size_t)kMaxBytes) return HAWQ_ERR_UNSUPPORTED;
    if (((uintptr_t)w | (uintptr_t)w_fragments) & 15) return HAWQ_ERR_UNSUPPORTED;
    return hawq::launch_fragment_weights(w, w_fragments, desc->K, hawq::tensor_bytes((int64_t)desc->R * desc->S * desc->C, desc->w_dtype),
                                         desc->w_dtype == HAWQ_S4, (hipStream_t)stream);
}

hawq_status hawq_bottleneck_tail_int(const hawq_conv_desc *desc2, const void *x, const void *w2_fragments, const int32_t *bias2,
                                     const int32_t *b2, const uint8_t *c2, const hawq_conv_desc *desc3, const void *w3_fragments,
                                     const int32_t *bias3, const int32_t *b3, const uint8_t *c3, const void *residual,
                                     const int32_t *res_b, const uint8_t *res_c, void *y, void *stream) {
    if (!desc2 || !desc3 || !b2 || !c2 || !b3 || !c3 || !residual || !w2_fragments || !w3_fragments) return HAWQ_ERR_NULL;
    // each layer on its own terms (types, clamp, overflow bound, sizes); the weights are given in fragment order only, and
    // the intermediate tensor has no address: stand-ins that pass the pointer checks and are never dereferenced
    ConvArgs a1, a2;
    int x_hi, h_hi;
    hawq_conv_desc d2 = *desc2, d3 = *desc3;
    d2.w_blocked = nullptr; d2.w_fragments = w2_fragments; d3.w_blocked = nullptr; d3.w_fragments = nullptr;
    hawq_status st = make_conv_args(&d2, x, w2_fragments, bias2, b2, c2, nullptr, nullptr, nullptr, y, true, a1, x_hi);
    if (st != HAWQ_OK) return st;
    // the second layer reads the first one's clamped output: that bounds its activations
    const int lo1 = a1.lo, hi1 = a1.hi;
    if (d3.x_dtype == HAWQ_U8 || d3.x_dtype == HAWQ_S8) {
        const int m = (-lo1 > hi1 ? -lo1 : hi1);
        d3.x_hi = m < 1 ? 1 : (m > (d3.x_dtype == HAWQ_U8 ? 255 : 128) ? 0 : m);
    }
    st = make_conv_args(&d3, x, w3_fragments, bias3, b3, c3, residual, res_b, res_c, y, true, a2, h_hi);
    if (st != HAWQ_OK) return st;
    if (((uintptr_t)w2_fragments) & 15) return HAWQ_ERR_UNSUPPORTED;
    RpArgs r;
    if (!make_rp_args(a1, x_hi, &a2, w3_fragments, r)) return HAWQ_ERR_UNSUPPORTED;
    if (a1.M == 0) return HAWQ_OK;
#ifdef HAWQ_RP_TIMING
    r.timing = g_rp_timing;
#endif
    return launch_conv_rp(r, true, (hipStream_t)stream);
}

hawq_status hawq_conv2d_int(const hawq_conv_desc *desc, const void *x, const void *w, const int32_t *bias, const int32_t *b,
                            const uint8_t *c, const void *residual, const int32_t *res_b, const uint8_t *res_c, void *y,
                            void *stream) {
    ConvArgs a;
    int x_hi;
    hawq_status st = make_conv_args(desc, x, w, bias, b, c, residual, res_b, res_c, y, true, a, x_hi);
    if (st != HAWQ_OK) return st;
    return dispatch_conv(a, x_hi, (hipStream_t)stream);
}

hawq_status hawq_conv2d_dual_int(const hawq_conv_desc *desc, const void *x, const void *w, const int32_t *bias, const int32_t *b,
                                 const uint8_t *c, const hawq_conv_desc *desc_s, const void *xs, const void *ws,
                                 const int32_t *bias_s, const int32_t *b_s, const uint8_t *c_s, void *y, void *stream) {
    if (!desc || !desc_s || !b || !c || !b_s || !c_s) return HAWQ_ERR_NULL;
    ConvArgs a;
    int x_hi, xs_hi;
    hawq_status st = make_dual_args(desc, x, w, bias, b, c, desc_s, xs, ws, bias_s, b_s, c_s, y, true, a, x_hi, xs_hi);
    if (st != HAWQ_OK) return st;
    return dispatch_conv_dual(a, x_hi, xs_hi, (hipStream_t)stream);
}

hawq_status hawq_gemm_int(int32_t M, int32_t N, int32_t Kdim, int32_t x_dt, int32_t w_dt, int32_t y_dt, const void *x,
                          const void *w, const int32_t *bias, const int32_t *b, const uint8_t *c, int32_t relu, int32_t y_lo,
                          int32_t y_hi, void *y, void *stream) {
    if (M < 0 || N <= 0 || Kdim <= 0) return HAWQ_ERR_SHAPE;
    hawq_conv_desc d = {};
    d.N = 1; d.H = 1; d.W = M > 0 ? M : 1; d.C = Kdim; d.K = N; d.R = 1; d.S = 1;
    d.stride_h = d.stride_w = 1; d.pad_h = d.pad_w = 0;
    d.x_dtype = x_dt; d.w_dtype = w_dt; d.y_dtype = y_dt; d.res_dtype = HAWQ_U8;
    d.relu = relu; d.y_lo = y_lo; d.y_hi = y_hi;
    d.x_hi = 0;   // the type's whole range: HAWQ_U8 rows may hold 0..255 (they then take an exact kernel off the signed matrix cores)
    ConvArgs a;
    int x_hi;
    hawq_status st = make_conv_args(&d, x, w, bias, b, c, nullptr, nullptr, nullptr, y, true, a, x_hi);
    if (st != HAWQ_OK) return st;
    if (M == 0) return HAWQ_OK;
    return dispatch_conv(a, x_hi, (hipStream_t)stream);
}

hawq_status hawq_residual_add_dyadic(int64_t n_pixels, int32_t K, int32_t m_dt, int32_t r_dt, int32_t y_dt, const void *m,
                                     const int32_t *m_b, const uint8_t *m_c, const void *r, const int32_t *r_b,
                                     const uint8_t *r_c, int32_t relu, int32_t y_lo, int32_t y_hi, void *y, void *stream) {
    if (!m || !m_b || !m_c || !r || !r_b || !r_c || !y) return HAWQ_ERR_NULL;
    if (n_pixels < 0 || K <= 0) return HAWQ_ERR_SHAPE;
    int64_t lo, hi;
    if (!dtype_range(m_dt, lo, hi) || !dtype_range(r_dt, lo, hi)) return HAWQ_ERR_DTYPE;
    hawq_status st = check_clamp(y_dt, y_lo, y_hi);
    if (st != HAWQ_OK) return st;
    if ((is4(m_dt) || is4(r_dt) || is4(y_dt)) && (K & 1)) return HAWQ_ERR_SHAPE;
    if (n_pixels * (int64_t)K >= kMaxBytes) return HAWQ_ERR_UNSUPPORTED;
    int32_t lo2 = (relu && y_lo < 0) ? 0 : y_lo, hi2 = y_hi;
    if (relu && y_hi < 0) lo2 = hi2 = y_hi;
    return launch_residual_add(n_pixels, K, m_dt, r_dt, y_dt, m, m_b, m_c, r, r_b, r_c, lo2, hi2, y, (hipStream_t)stream);
}

hawq_status hawq_avgpool_int(int32_t N, int32_t H, int32_t W, int32_t C, int32_t x_dt, int32_t y_dt, const void *x,
                             const int32_t *b, const uint8_t *c, int32_t y_lo, int32_t y_hi, void *y, void *stream) {
    if (!x || !b || !c || !y) return HAWQ_ERR_NULL;
    if (N < 0 || H <= 0 || W <= 0 || C <= 0) return HAWQ_ERR_SHAPE;
    if (!low_bit(x_dt)) return HAWQ_ERR_DTYPE;
    hawq_status st = check_clamp(y_dt, y_lo, y_hi);
    if (st != HAWQ_OK) return st;
    if ((is4(x_dt) || is4(y_dt)) && (C & 1)) return HAWQ_ERR_SHAPE;
    if ((int64_t)H * W * 255 >= kMaxBytes) return HAWQ_ERR_OVERFLOW;
    if ((int64_t)N * H * W * C >= kMaxBytes || N > 65535) return HAWQ_ERR_UNSUPPORTED;
    return launch_avgpool(N, H * W, C, x_dt, y_dt, x, b, c, y_lo, y_hi, y, (hipStream_t)stream);
}

hawq_status hawq_maxpool_int(int32_t N, int32_t H, int32_t W, int32_t C, int32_t x_dt, int32_t y_dt, const void *x,
                             int32_t y_lo, int32_t y_hi, void *y, void *stream) {
    if (!x || !y) return HAWQ_ERR_NULL;
    if (N < 0 || H <= 0 || W <= 0 || C <= 0) return HAWQ_ERR_SHAPE;
    if (!low_bit(x_dt) || !low_bit(y_dt)) return HAWQ_ERR_DTYPE;
    hawq_status st = check_clamp(y_dt, y_lo, y_hi);
    if (st != HAWQ_OK) return st;
    if ((is4(x_dt) || is4(y_dt)) && (C & 1)) return HAWQ_ERR_SHAPE;
    if ((int64_t)N * H * W * C >= kMaxBytes) return HAWQ_ERR_UNSUPPORTED;
    return launch_maxpool(N, H, W, C, x_dt, y_dt, x, y_lo, y_hi, y, (hipStream_t)stream);
}

hawq_status hawq_pool2d_sum_int(int32_t N, int32_t H, int32_t W, int32_t C, int32_t R, int32_t S, int32_t stride_h, int32_t stride_w,
                                int32_t pad_h, int32_t pad_w, int32_t x_dt, int32_t y_dt, const void *x, const int32_t *b,
                                const uint8_t *c, int32_t y_lo, int32_t y_hi, void *y, void *stream) {
    if (!x || !y) return HAWQ_ERR_NULL;
    if ((b == nullptr) != (c == nullptr)) return HAWQ_ERR_NULL;
    if (N < 0 || H <= 0 || W <= 0 || C <= 0 || R <= 0 || S <= 0 || stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0)
        return HAWQ_ERR_SHAPE;
    if ((int64_t)H + 2 * (int64_t)pad_h < R || (int64_t)W + 2 * (int64_t)pad_w < S) return HAWQ_ERR_SHAPE;
    int64_t lo, hi;
    if (!dtype_range(x_dt, lo, hi) || !dtype_range(y_dt, lo, hi)) return HAWQ_ERR_DTYPE;
    if (b == nullptr) {
        if (y_dt != HAWQ_S32) return HAWQ_ERR_DTYPE;   // raw window sums are INT32
        y_lo = INT32_MIN; y_hi = INT32_MAX;
    } else {
        hawq_status st = check_clamp(y_dt, y_lo, y_hi);
        if (st != HAWQ_OK) return st;
    }
    if ((is4(x_dt) || is4(y_dt)) && (C & 1)) return HAWQ_ERR_SHAPE;
    if (x_dt != HAWQ_S32 && (int64_t)R * S * 255 >= kMaxBytes) return HAWQ_ERR_OVERFLOW;
    const int64_t P = ((int64_t)H + 2 * pad_h - R) / stride_h + 1, Q = ((int64_t)W + 2 * pad_w - S) / stride_w + 1;
    if (tensor_bytes((int64_t)N * H * W * C, x_dt) >= kMaxBytes || tensor_bytes((int64_t)N * P * Q * C, y_dt) >= kMaxBytes)
        return HAWQ_ERR_UNSUPPORTED;
    return launch_pool_sum(N, H, W, C, R, S, stride_h, stride_w, pad_h, pad_w, x_dt, y_dt, x, b, c, y_lo, y_hi, y, (hipStream_t)stream);
}

hawq_status hawq_concat_dyadic(int64_t n_pixels, int32_t n_branches, const hawq_concat_branch *branches, int32_t y_dt,
                               int32_t y_lo, int32_t y_hi, void *y, void *stream) {
    if (!branches || !y) return HAWQ_ERR_NULL;
    if (n_pixels < 0 || n_branches <= 0) return HAWQ_ERR_SHAPE;
    hawq_status st = check_clamp(y_dt, y_lo, y_hi);
    if (st != HAWQ_OK) return st;
    int64_t Kt = 0;
    for (int32_t i = 0; i < n_branches; ++i) {
        const hawq_concat_branch &br = branches[i];
        if (!br.q || !br.b || !br.c) return HAWQ_ERR_NULL;
        if (br.K <= 0) return HAWQ_ERR_SHAPE;
        int64_t lo, hi;
        if (!dtype_range(br.dtype, lo, hi)) return HAWQ_ERR_DTYPE;
        if ((is4(br.dtype) || is4(y_dt)) && (br.K & 1)) return HAWQ_ERR_SHAPE;
        if (tensor_bytes(n_pixels * br.K, br.dtype) >= kMaxBytes) return HAWQ_ERR_UNSUPPORTED;
        Kt += br.K;
    }
    if (Kt > INT32_MAX || tensor_bytes(n_pixels * Kt, y_dt) >= kMaxBytes) return HAWQ_ERR_UNSUPPORTED;
    int64_t off = 0;
    for (int32_t i = 0; i < n_branches; ++i) {
        const hawq_concat_branch &br = branches[i];
        st = launch_concat_branch(n_pixels, br.K, (int)Kt, (int)off, br.dtype, y_dt, br.q, br.b, br.c, y_lo, y_hi, y, (hipStream_t)stream);
        if (st != HAWQ_OK) return st;
        off += br.K;
    }
    return HAWQ_OK;
}

void hawq_tune_set_tile(int32_t tile) { set_tile_override(tile); }

const char *hawq_status_string(hawq_status s) {
    switch (s) {
    case HAWQ_OK: return "ok";
    case HAWQ_ERR_NULL: return "required pointer is NULL";
    case HAWQ_ERR_SHAPE: return "invalid shape";
    case HAWQ_ERR_DTYPE: return "invalid dtype combination";
    case HAWQ_ERR_RANGE: return "value outside the allowed range";
    case HAWQ_ERR_OVERFLOW: return "INT32 accumulator could overflow";
    case HAWQ_ERR_UNSUPPORTED: return "unsupported request";
    case HAWQ_ERR_DEVICE: return "HIP call failed";
    case HAWQ_ERR_WORKSPACE: return "workspace too small";
    default: return "unknown status";
    }
}

}  // extern "C"
