// Direct quantised convolution: one thread per output element (per pair of channels for 4-bit
// outputs), scalar integer multiply-accumulate.  Serves every shape and type combination the
// interface accepts that the matrix-core kernel does not (channel counts that are not a
// multiple of 64, unsigned 8-bit inputs above 127, unaligned buffers), with or without a second
// convolution on the shortcut branch.  Same arithmetic, same epilogue order as the fast kernels.
#include "common.h"

namespace hawq {

__global__ void __launch_bounds__(256) conv_direct_kernel(const ConvArgs a, const int64_t units, const int per_unit) {
    const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= units) return;
    const int kunits = a.K / per_unit;
    const int64_t m = u / kunits;
    const int kq = (int)(u - m * kunits) * per_unit;
    const int PQ = a.P * a.Q;
    const int n = (int)(m / PQ);
    const int pq = (int)(m - (int64_t)n * PQ);
    const int p = pq / a.Q, q = pq - p * a.Q;
    const bool has_rq = a.b != nullptr, has_res = a.res != nullptr;
    int32_t out[2] = {0, 0};
    for (int e = 0; e < per_unit; ++e) {
        const int k = kq + e;
        int32_t acc = 0;
        for (int r = 0; r < a.R; ++r) {
            const int ih = p * a.stride_h - a.pad_h + r;
            if (ih < 0 || ih >= a.H) continue;
            for (int s = 0; s < a.S; ++s) {
                const int iw = q * a.stride_w - a.pad_w + s;
                if (iw < 0 || iw >= a.W) continue;
                const int64_t xo = (((int64_t)n * a.H + ih) * a.W + iw) * a.C;
                const int64_t wo = (((int64_t)k * a.R + r) * a.S + s) * a.C;
                for (int c = 0; c < a.C; ++c) acc += load_elem(a.x, a.x_dt, xo + c) * load_elem(a.w, a.w_dt, wo + c);
            }
        }
        const int32_t t = acc + a.bias[k];
        if (!has_rq) {
            out[e] = t;
        } else {
            int64_t v = rq64(t, a.b[k], a.c[k]);
            if (has_res) v += rq64(load_elem(a.res, a.res_dt, m * a.K + k), a.res_b[k], a.res_c[k]);
            if (a.xs != nullptr) {   // shortcut convolution (1x1, unpadded): its own accumulator, bias and dyadic number
                int32_t acc_s = 0;
                const int64_t xo = (((int64_t)n * a.Hs + p * a.stride_sh) * a.Ws + q * a.stride_sw) * a.Cs;
                const int64_t wo = (int64_t)k * a.Cs;
                for (int c = 0; c < a.Cs; ++c) acc_s += load_elem(a.xs, a.xs_dt, xo + c) * load_elem(a.ws, a.ws_dt, wo + c);
                int64_t sc = rq64(acc_s + a.bias_s[k], a.b_s[k], a.c_s[k]);
                if (a.mid_s8) sc = rq64(clamp64(sc, -128, 127), a.res_b[k], a.res_c[k]);
                v += sc;
            }
            out[e] = clamp64(v, a.lo, a.hi);
        }
    }
    const int64_t o = m * a.K + kq;
    if (a.y_dt == HAWQ_S32) ((int32_t *)a.y)[o] = out[0];
    else if (is4(a.y_dt)) a.y[o >> 1] = (uint8_t)((out[0] & 0xf) | ((out[1] & 0xf) << 4));
    else a.y[o] = (uint8_t)out[0];
}

hawq_status launch_conv_direct(const ConvArgs &a, hipStream_t s) {
    const int per_unit = is4(a.y_dt) ? 2 : 1;
    const int64_t units = (int64_t)a.M * (a.K / per_unit);
    if (units == 0) return HAWQ_OK;
    const int64_t blocks = (units + 255) / 256;
    if (blocks > 0x7fffffff) return HAWQ_ERR_UNSUPPORTED;
    conv_direct_kernel<<<(uint32_t)blocks, 256, 0, s>>>(a, units, per_unit);
    return check_launch();
}

}  // namespace hawq
