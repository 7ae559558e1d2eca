// Memory-bound integer kernels: stand-alone dyadic residual add, global average pool,
// 3x3/2 max pool, INT32 window-sum pool, per-branch dyadic concatenation.  One thread handles 4 consecutive channels of one pixel when the channel
// count allows it (dword loads/stores of packed 8-bit data), else one unit of 1 or 2 channels.
#include "common.h"

namespace hawq {

// ---- residual add (Section 3.3): y = clamp(rq(m) + rq(r)) ----
__global__ void __launch_bounds__(256)
residual_add_kernel(const int64_t units, const int K, const int per, const int m_dt, const int r_dt, const int y_dt,
                    const void *m, const int32_t *__restrict__ m_b, const uint8_t *__restrict__ m_c,
                    const void *r, const int32_t *__restrict__ r_b, const uint8_t *__restrict__ r_c,
                    const int lo, const int hi, void *y) {   // (m, r, y unqualified: y may alias m or r when the types match)
    const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= units) return;
    const int64_t e0 = u * per;
    const int k0 = (int)(e0 % K);
    int32_t out[4];
    for (int j = 0; j < per; ++j) {
        const int k = k0 + j;
        const int64_t v = rq64(load_elem(m, m_dt, e0 + j), m_b[k], m_c[k]) + rq64(load_elem(r, r_dt, e0 + j), r_b[k], r_c[k]);
        out[j] = clamp64(v, lo, hi);
    }
    if (y_dt == HAWQ_S32) {
        for (int j = 0; j < per; ++j) ((int32_t *)y)[e0 + j] = out[j];
    } else if (is4(y_dt)) {
        for (int j = 0; j < per; j += 2) ((uint8_t *)y)[(e0 + j) >> 1] = (uint8_t)((out[j] & 0xf) | ((out[j + 1] & 0xf) << 4));
    } else if (per == 4) {
        ((uint32_t *)y)[e0 >> 2] = (out[0] & 0xff) | ((out[1] & 0xff) << 8) | ((out[2] & 0xff) << 16) | ((uint32_t)out[3] << 24);
    } else {
        for (int j = 0; j < per; ++j) ((uint8_t *)y)[e0 + j] = (uint8_t)out[j];
    }
}

hawq_status launch_residual_add(int64_t n_pixels, int K, int m_dt, int r_dt, int y_dt, const void *m, const int32_t *m_b,
                                const uint8_t *m_c, const void *r, const int32_t *r_b, const uint8_t *r_c, int lo, int hi,
                                void *y, hipStream_t s) {
    const bool any4 = is4(m_dt) || is4(r_dt) || is4(y_dt);
    int per = (K % 4 == 0 && ((uintptr_t)y & 3) == 0) ? 4 : (any4 ? 2 : 1);
    const int64_t units = n_pixels * K / per;
    if (units == 0) return HAWQ_OK;
    const int64_t blocks = (units + 255) / 256;
    if (blocks > 0x7fffffff) return HAWQ_ERR_UNSUPPORTED;
    residual_add_kernel<<<(uint32_t)blocks, 256, 0, s>>>(units, K, per, m_dt, r_dt, y_dt, m, m_b, m_c, r, r_b, r_c, lo, hi, y);
    return check_launch();
}

// ---- global average pool (Appendix E): INT32 sum over H*W, then one dyadic rescale ----
// grid: (ceil(C/per/64), N); one thread sums `per` adjacent channels over all pixels, so a
// wave reads 64*per consecutive bytes of every pixel.
__global__ void __launch_bounds__(64)
avgpool_kernel(const int HW, const int C, const int per, const int x_dt, const int y_dt, const void *__restrict__ x,
               const int32_t *__restrict__ b, const uint8_t *__restrict__ c, const int lo, const int hi, void *__restrict__ y) {
    const int n = blockIdx.y;
    const int k0 = (blockIdx.x * 64 + threadIdx.x) * per;
    if (k0 >= C) return;
    int32_t sum[4] = {0, 0, 0, 0};
    const int64_t base = (int64_t)n * HW * C + k0;
    if (per == 4 && !is4(x_dt)) {
        const uint8_t *xp = (const uint8_t *)x + base;
        for (int i = 0; i < HW; ++i) {
            const uint32_t v = *(const uint32_t *)(xp + (int64_t)i * C);
            if (x_dt == HAWQ_U8) {
                sum[0] += v & 0xff; sum[1] += (v >> 8) & 0xff; sum[2] += (v >> 16) & 0xff; sum[3] += v >> 24;
            } else {
                sum[0] += (int8_t)(v & 0xff); sum[1] += (int8_t)((v >> 8) & 0xff);
                sum[2] += (int8_t)((v >> 16) & 0xff); sum[3] += (int8_t)(v >> 24);
            }
        }
    } else {
        for (int i = 0; i < HW; ++i)
            for (int j = 0; j < per; ++j) sum[j] += load_elem(x, x_dt, base + (int64_t)i * C + j);
    }
    int32_t out[4];
    for (int j = 0; j < per; ++j) out[j] = clamp64(rq64(sum[j], b[k0 + j], c[k0 + j]), lo, hi);
    const int64_t o = (int64_t)n * C + k0;
    if (y_dt == HAWQ_S32) {
        for (int j = 0; j < per; ++j) ((int32_t *)y)[o + j] = out[j];
    } else if (is4(y_dt)) {
        for (int j = 0; j < per; j += 2) ((uint8_t *)y)[(o + j) >> 1] = (uint8_t)((out[j] & 0xf) | ((out[j + 1] & 0xf) << 4));
    } else {
        for (int j = 0; j < per; ++j) ((uint8_t *)y)[o + j] = (uint8_t)out[j];
    }
}

// fast path: unsigned 8-bit input, 8-bit output, C % 256 == 0.  A workgroup owns 256 channels of one image:
// 16 channel groups (16 bytes each) x 16 pixel slices; every thread adds up its slice's pixels with 16-byte
// loads, the 16 partial sums of a channel group meet in LDS, one thread per channel requantises.
__global__ void __launch_bounds__(256)
avgpool_u8_kernel(const int HW, const int C, const uint8_t *__restrict__ x, const int32_t *__restrict__ b,
                  const uint8_t *__restrict__ c, const int lo, const int hi, uint8_t *__restrict__ y) {
    __shared__ int32_t part[16][256 + 8];
    const int n = blockIdx.y, cbase = blockIdx.x * 256;
    const int g = threadIdx.x & 15, sl = threadIdx.x >> 4;
    int32_t sum[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) sum[j] = 0;
    const uint8_t *xp = x + (int64_t)n * HW * C + cbase + g * 16;
    for (int i = sl; i < HW; i += 16) {
        const uint4 v = *(const uint4 *)(xp + (int64_t)i * C);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            sum[4 * d + 0] += w[d] & 0xff; sum[4 * d + 1] += (w[d] >> 8) & 0xff;
            sum[4 * d + 2] += (w[d] >> 16) & 0xff; sum[4 * d + 3] += w[d] >> 24;
        }
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) part[sl][g * 16 + j] = sum[j];
    __syncthreads();
    const int k = threadIdx.x;   // one channel per thread
    int32_t t = 0;
#pragma unroll
    for (int s2 = 0; s2 < 16; ++s2) t += part[s2][k];
    y[(int64_t)n * C + cbase + k] = (uint8_t)clamp64(rq64(t, b[cbase + k], c[cbase + k]), lo, hi);
}

hawq_status launch_avgpool(int N, int HW, int C, int x_dt, int y_dt, const void *x, const int32_t *b, const uint8_t *c,
                           int lo, int hi, void *y, hipStream_t s) {
    if (N == 0) return HAWQ_OK;
    if (x_dt == HAWQ_U8 && (y_dt == HAWQ_U8 || y_dt == HAWQ_S8) && C % 256 == 0 && ((uintptr_t)x & 15) == 0) {
        dim3 grid(C / 256, N);
        avgpool_u8_kernel<<<grid, 256, 0, s>>>(HW, C, (const uint8_t *)x, b, c, lo, hi, (uint8_t *)y);
        return check_launch();
    }
    const bool any4 = is4(x_dt) || is4(y_dt);
    const int per = (C % 4 == 0 && ((uintptr_t)x & 3) == 0) ? 4 : (any4 ? 2 : 1);
    dim3 grid((C / per + 63) / 64, N);
    avgpool_kernel<<<grid, 64, 0, s>>>(HW, C, per, x_dt, y_dt, x, b, c, lo, hi, y);
    return check_launch();
}

// ---- max pool 3x3 / 2, pad 1 ----

// fast path: U8 in, C % 16 == 0; one thread = 16 channels of one output pixel
__global__ void __launch_bounds__(256)
maxpool_u8_kernel(const int64_t units, const int H, const int W, const int C, const int P, const int Q,
                  const uint8_t *__restrict__ x, const int lo, const int hi, const int y_dt, uint8_t *__restrict__ y) {
    const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= units) return;
    const int cg = C / 16;
    const int g = (int)(u % cg);
    int64_t t = u / cg;
    const int q = (int)(t % Q); t /= Q;
    const int p = (int)(t % P);
    const int n = (int)(t / P);
    uint4 best = make_uint4(0, 0, 0, 0);   // unsigned data: 0 is the identity, padding never wins
    for (int r = 0; r < 3; ++r) {
        const int ih = 2 * p - 1 + r;
        if (ih < 0 || ih >= H) continue;
        for (int s = 0; s < 3; ++s) {
            const int iw = 2 * q - 1 + s;
            if (iw < 0 || iw >= W) continue;
            const uint4 v = *(const uint4 *)(x + (((int64_t)n * H + ih) * W + iw) * C + g * 16);
            best.x = max_u8x4(best.x, v.x); best.y = max_u8x4(best.y, v.y);
            best.z = max_u8x4(best.z, v.z); best.w = max_u8x4(best.w, v.w);
        }
    }
    uint32_t wv[4] = {best.x, best.y, best.z, best.w};
    uint32_t ov[4];
    uint32_t nib[2] = {0, 0};
    for (int d = 0; d < 4; ++d) {
        uint32_t o = 0, h = 0;
        for (int j = 0; j < 4; ++j) {
            int32_t v = (int32_t)((wv[d] >> (8 * j)) & 0xff);
            v = v < lo ? lo : (v > hi ? hi : v);
            o |= (uint32_t)(v & 0xff) << (8 * j);
            h |= (uint32_t)(v & 0xf) << (4 * j);
        }
        ov[d] = o;
        nib[d >> 1] |= h << (16 * (d & 1));
    }
    const int64_t oe = (((int64_t)n * P + p) * Q + q) * C + g * 16;
    if (is4(y_dt)) *(uint2 *)(y + (oe >> 1)) = make_uint2(nib[0], nib[1]);
    else *(uint4 *)(y + oe) = make_uint4(ov[0], ov[1], ov[2], ov[3]);
}

__global__ void __launch_bounds__(256)
maxpool_generic_kernel(const int64_t units, const int per, const int H, const int W, const int C, const int P, const int Q,
                       const int x_dt, const int y_dt, const void *__restrict__ x, const int lo, const int hi,
                       void *__restrict__ y) {
    const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= units) return;
    const int cu = C / per;
    const int k0 = (int)(u % cu) * per;
    int64_t t = u / cu;
    const int q = (int)(t % Q); t /= Q;
    const int p = (int)(t % P);
    const int n = (int)(t / P);
    int32_t out[2];
    for (int j = 0; j < per; ++j) {
        int32_t best = INT32_MIN;
        for (int r = 0; r < 3; ++r) {
            const int ih = 2 * p - 1 + r;
            if (ih < 0 || ih >= H) continue;
            for (int s = 0; s < 3; ++s) {
                const int iw = 2 * q - 1 + s;
                if (iw < 0 || iw >= W) continue;
                const int32_t v = load_elem(x, x_dt, (((int64_t)n * H + ih) * W + iw) * C + k0 + j);
                best = v > best ? v : best;
            }
        }
        out[j] = best < lo ? lo : (best > hi ? hi : best);
    }
    const int64_t oe = (((int64_t)n * P + p) * Q + q) * C + k0;
    if (is4(y_dt)) ((uint8_t *)y)[oe >> 1] = (uint8_t)((out[0] & 0xf) | ((out[1] & 0xf) << 4));
    else
        for (int j = 0; j < per; ++j) ((uint8_t *)y)[oe + j] = (uint8_t)out[j];   // (per = 2 with a 4-bit input and an 8-bit output)
}

hawq_status launch_maxpool(int N, int H, int W, int C, int x_dt, int y_dt, const void *x, int lo, int hi, void *y,
                           hipStream_t s) {
    const int P = (H - 1) / 2 + 1, Q = (W - 1) / 2 + 1;
    if (N == 0) return HAWQ_OK;
    const bool fast = x_dt == HAWQ_U8 && (y_dt == HAWQ_U8 || y_dt == HAWQ_U4) && C % 16 == 0 &&
                      (((uintptr_t)x | (uintptr_t)y) & 15) == 0 && lo >= 0;
    if (fast) {
        const int64_t units = (int64_t)N * P * Q * (C / 16);
        const int64_t blocks = (units + 255) / 256;
        if (blocks > 0x7fffffff) return HAWQ_ERR_UNSUPPORTED;
        maxpool_u8_kernel<<<(uint32_t)blocks, 256, 0, s>>>(units, H, W, C, P, Q, (const uint8_t *)x, lo, hi, y_dt, (uint8_t *)y);
    } else {
        const int per = (is4(x_dt) || is4(y_dt)) ? 2 : 1;
        const int64_t units = (int64_t)N * P * Q * (C / per);
        const int64_t blocks = (units + 255) / 256;
        if (blocks > 0x7fffffff) return HAWQ_ERR_UNSUPPORTED;
        maxpool_generic_kernel<<<(uint32_t)blocks, 256, 0, s>>>(units, per, H, W, C, P, Q, x_dt, y_dt, x, lo, hi, y);
    }
    return check_launch();
}

// ---- window-sum pool carried in INT32 (Appendix E) ----
// one thread = `per` adjacent channels of one output pixel; the in-image taps are added in INT32 (64-bit while adding,
// the caller's contract keeps the sum inside INT32), then either stored raw or rescaled by one dyadic number and clamped
__global__ void __launch_bounds__(256)
pool_sum_kernel(const int64_t units, const int H, const int W, const int C, const int R, const int S, const int sh, const int sw,
                const int ph, const int pw, const int P, const int Q, const int per, const int x_dt, const int y_dt,
                const void *__restrict__ x, const int32_t *__restrict__ b, const uint8_t *__restrict__ c, const int lo, const int hi,
                void *__restrict__ y) {
    const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= units) return;
    const int cg = C / per;
    const int k0 = (int)(u % cg) * per;
    int64_t t = u / cg;
    const int q = (int)(t % Q); t /= Q;
    const int p = (int)(t % P);
    const int n = (int)(t / P);
    int64_t sum[4] = {0, 0, 0, 0};
    for (int r = 0; r < R; ++r) {
        const int ih = p * sh - ph + r;
        if (ih < 0 || ih >= H) continue;
        for (int s = 0; s < S; ++s) {
            const int iw = q * sw - pw + s;
            if (iw < 0 || iw >= W) continue;
            const int64_t e = (((int64_t)n * H + ih) * W + iw) * C + k0;
            if (per == 4 && x_dt == HAWQ_S32) {
                const v4i v = *(const v4i *)((const int32_t *)x + e);
                sum[0] += v[0]; sum[1] += v[1]; sum[2] += v[2]; sum[3] += v[3];
            } else if (per == 4 && x_dt == HAWQ_U8) {
                const uint32_t v = *(const uint32_t *)((const uint8_t *)x + e);
                sum[0] += v & 0xff; sum[1] += (v >> 8) & 0xff; sum[2] += (v >> 16) & 0xff; sum[3] += v >> 24;
            } else {
                for (int j = 0; j < per; ++j) sum[j] += load_elem(x, x_dt, e + j);
            }
        }
    }
    int32_t out[4];
    for (int j = 0; j < per; ++j)
        out[j] = b != nullptr ? clamp64(rq64((int32_t)sum[j], b[k0 + j], c[k0 + j]), lo, hi) : (int32_t)sum[j];
    const int64_t o = (((int64_t)n * P + p) * Q + q) * C + k0;
    if (y_dt == HAWQ_S32) {
        for (int j = 0; j < per; ++j) ((int32_t *)y)[o + j] = out[j];
    } else if (is4(y_dt)) {
        for (int j = 0; j < per; j += 2) ((uint8_t *)y)[(o + j) >> 1] = (uint8_t)((out[j] & 0xf) | ((out[j + 1] & 0xf) << 4));
    } else if (per == 4) {
        ((uint32_t *)y)[o >> 2] = (out[0] & 0xff) | ((out[1] & 0xff) << 8) | ((out[2] & 0xff) << 16) | ((uint32_t)out[3] << 24);
    } else {
        for (int j = 0; j < per; ++j) ((uint8_t *)y)[o + j] = (uint8_t)out[j];
    }
}

// patch of output pixels per thread (measured at 128 x 35 x 35 x 288 INT32: 4x4 73.8 us, 4x8 76.8, 8x4 77.4, 8x8 78.2;
// one row of eight, the previous form, 117.6 us)
#define POOL_QT 4
#define POOL_PT 4
// fast path for the Inception pooling branch: 3x3 / stride 1 / pad 1 on INT32 (or unsigned 8-bit) data, C % 4 == 0.  One
// thread = 4 channels of a QT-wide, PT-high patch of output pixels.  It walks the PT + 2 input rows under the patch once:
// per row QT + 2 loads and the QT horizontal three-sums; an output row is the sum of the last three rows' horizontal sums
// (kept in a ring of three).  (PT + 2)(QT + 2) loads for PT QT outputs -- 2.25 per output at 4 x 4 instead of 9, which is
// what the vector-memory path, not HBM, limits in the general kernel.
template <bool X32, int QT, int PT>
__global__ void __launch_bounds__(256)
pool_sum3x3_kernel(const int64_t units, const int H, const int W, const int C, const int y_dt, const void *__restrict__ x,
                   const int32_t *__restrict__ b, const uint8_t *__restrict__ c, const int lo, const int hi, void *__restrict__ y) {
    const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= units) return;
    const int cg = C / 4, qb = (W + QT - 1) / QT, pb = (H + PT - 1) / PT;
    const int k0 = (int)(u % cg) * 4;
    int64_t t = u / cg;
    const int q0 = (int)(t % qb) * QT; t /= qb;
    const int p0 = (int)(t % pb) * PT;
    const int n = (int)(t / pb);
    int32_t bb[4] = {0, 0, 0, 0}, cc[4] = {1, 1, 1, 1};
    if (b != nullptr)
        for (int j = 0; j < 4; ++j) { bb[j] = b[k0 + j]; cc[j] = c[k0 + j]; }
    int32_t hs[3][QT][4];   // horizontal three-sums of the last three input rows
    static_for<0, PT + 2>([&](auto rc) {
        constexpr int rr = decltype(rc)::value;
        constexpr int slot = rr % 3;
        const int ih = p0 - 1 + rr;
        int32_t v[QT + 2][4];
#pragma unroll
        for (int j = 0; j < QT + 2; ++j) {
            const int iw = q0 - 1 + j;
            v[j][0] = v[j][1] = v[j][2] = v[j][3] = 0;
            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
            const int64_t e = (((int64_t)n * H + ih) * W + iw) * C + k0;
            if (X32) {
                const v4i w4 = *(const v4i *)((const int32_t *)x + e);
                v[j][0] = w4[0]; v[j][1] = w4[1]; v[j][2] = w4[2]; v[j][3] = w4[3];
            } else {
                const uint32_t w1 = *(const uint32_t *)((const uint8_t *)x + e);
                v[j][0] = w1 & 0xff; v[j][1] = (w1 >> 8) & 0xff; v[j][2] = (w1 >> 16) & 0xff; v[j][3] = w1 >> 24;
            }
        }
#pragma unroll
        for (int i = 0; i < QT; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) hs[slot][i][j] = v[i][j] + v[i + 1][j] + v[i + 2][j];
        if constexpr (rr >= 2) {
            const int p = p0 + rr - 2;
            if (p < H) {
#pragma unroll
                for (int i = 0; i < QT; ++i) {
                    if (q0 + i >= W) break;
                    int32_t out[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int32_t sum = hs[0][i][j] + hs[1][i][j] + hs[2][i][j];
                        out[j] = b != nullptr ? clamp64(rq64(sum, bb[j], cc[j]), lo, hi) : sum;
                    }
                    const int64_t o = (((int64_t)n * H + p) * W + q0 + i) * C + k0;
                    if (y_dt == HAWQ_S32) *(v4i *)((int32_t *)y + o) = (v4i){out[0], out[1], out[2], out[3]};
                    else if (is4(y_dt)) *(uint16_t *)((uint8_t *)y + (o >> 1)) = (uint16_t)((out[0] & 0xf) | ((out[1] & 0xf) << 4) | ((out[2] & 0xf) << 8) | ((out[3] & 0xf) << 12));
                    else ((uint32_t *)y)[o >> 2] = (out[0] & 0xff) | ((out[1] & 0xff) << 8) | ((out[2] & 0xff) << 16) | ((uint32_t)out[3] << 24);
                }
            }
        }
    });
}

hawq_status launch_pool_sum(int N, int H, int W, int C, int R, int S, int sh, int sw, int ph, int pw, int x_dt, int y_dt,
                            const void *x, const int32_t *b, const uint8_t *c, int lo, int hi, void *y, hipStream_t s) {
    const int P = (H + 2 * ph - R) / sh + 1, Q = (W + 2 * pw - S) / sw + 1;
    const bool any4 = is4(x_dt) || is4(y_dt);
    if (R == 3 && S == 3 && sh == 1 && sw == 1 && ph == 1 && pw == 1 && C % 4 == 0 && (x_dt == HAWQ_S32 || x_dt == HAWQ_U8) &&
        (((uintptr_t)x | (uintptr_t)y) & 15) == 0) {
        constexpr int QT = POOL_QT, PT = POOL_PT;
        const int64_t units = (int64_t)N * ((H + PT - 1) / PT) * ((W + QT - 1) / QT) * (C / 4);
        if (units == 0) return HAWQ_OK;
        const int64_t blocks = (units + 255) / 256;
        if (blocks > 0x7fffffff) return HAWQ_ERR_UNSUPPORTED;
        if (x_dt == HAWQ_S32) pool_sum3x3_kernel<true, QT, PT><<<(uint32_t)blocks, 256, 0, s>>>(units, H, W, C, y_dt, x, b, c, lo, hi, y);
        else pool_sum3x3_kernel<false, QT, PT><<<(uint32_t)blocks, 256, 0, s>>>(units, H, W, C, y_dt, x, b, c, lo, hi, y);
        return check_launch();
    }
    const int per = (C % 4 == 0 && (((uintptr_t)x | (uintptr_t)y) & 15) == 0) ? 4 : (any4 ? 2 : 1);
    const int64_t units = (int64_t)N * P * Q * (C / per);
    if (units == 0) return HAWQ_OK;
    const int64_t blocks = (units + 255) / 256;
    if (blocks > 0x7fffffff) return HAWQ_ERR_UNSUPPORTED;
    pool_sum_kernel<<<(uint32_t)blocks, 256, 0, s>>>(units, H, W, C, R, S, sh, sw, ph, pw, P, Q, per, x_dt, y_dt, x, b, c, lo, hi, y);
    return check_launch();
}

// ---- concatenation with one dyadic number per branch (Appendix E) ----
// one launch per branch: branch elements [n_pixels][K] -> channels off .. off + K of the [n_pixels][Kt] output
__global__ void __launch_bounds__(256)
concat_branch_kernel(const int64_t units, const int K, const int Kt, const int off, const int per, const int q_dt, const int y_dt,
                     const void *__restrict__ q, const int32_t *__restrict__ b, const uint8_t *__restrict__ c, const int lo, const int hi,
                     void *__restrict__ y) {
    const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= units) return;
    const int kg = K / per;
    const int64_t px = u / kg;
    const int k0 = (int)(u - px * kg) * per;
    const int64_t e = px * K + k0;
    int32_t out[4];
    if (per == 4 && q_dt == HAWQ_S32) {
        const v4i v = *(const v4i *)((const int32_t *)q + e);
        for (int j = 0; j < 4; ++j) out[j] = clamp64(rq64(v[j], b[k0 + j], c[k0 + j]), lo, hi);
    } else {
        for (int j = 0; j < per; ++j) out[j] = clamp64(rq64(load_elem(q, q_dt, e + j), b[k0 + j], c[k0 + j]), lo, hi);
    }
    const int64_t o = px * Kt + off + k0;
    if (y_dt == HAWQ_S32) {
        for (int j = 0; j < per; ++j) ((int32_t *)y)[o + j] = out[j];
    } else if (is4(y_dt)) {
        for (int j = 0; j < per; j += 2) ((uint8_t *)y)[(o + j) >> 1] = (uint8_t)((out[j] & 0xf) | ((out[j + 1] & 0xf) << 4));
    } else if (per == 4) {
        ((uint32_t *)y)[o >> 2] = (out[0] & 0xff) | ((out[1] & 0xff) << 8) | ((out[2] & 0xff) << 16) | ((uint32_t)out[3] << 24);
    } else {
        for (int j = 0; j < per; ++j) ((uint8_t *)y)[o + j] = (uint8_t)out[j];
    }
}

hawq_status launch_concat_branch(int64_t n_pixels, int K, int Kt, int off, int q_dt, int y_dt, const void *q, const int32_t *b,
                                 const uint8_t *c, int lo, int hi, void *y, hipStream_t s) {
    const bool any4 = is4(q_dt) || is4(y_dt);
    // four channels per thread need dword-aligned output positions (and 16-byte aligned INT32 rows)
    const bool vec = K % 4 == 0 && Kt % 4 == 0 && off % 4 == 0 && (((uintptr_t)q | (uintptr_t)y) & 15) == 0;
    const int per = vec ? 4 : (any4 ? 2 : 1);
    const int64_t units = n_pixels * (K / per);
    if (units == 0) return HAWQ_OK;
    const int64_t blocks = (units + 255) / 256;
    if (blocks > 0x7fffffff) return HAWQ_ERR_UNSUPPORTED;
    concat_branch_kernel<<<(uint32_t)blocks, 256, 0, s>>>(units, K, Kt, off, per, q_dt, y_dt, q, b, c, lo, hi, y);
    return check_launch();
}

// ---- weights into the blocked order of the implicit-GEMM kernel: one thread per 16-byte chunk of the copy ----
__global__ void __launch_bounds__(256)
block_weights_kernel(const uint8_t *__restrict__ w, uint8_t *__restrict__ out, const int K, const int64_t row, const int64_t chunks) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= chunks) return;
    const int64_t steps = row / 64;
    const int ch = (int)(i & 3);
    const int kk = (int)((i >> 2) & 63);
    const int64_t blk = i >> 8;                  // (k / 64) * steps + step
    const int64_t st = blk % steps;
    const int k = (int)(blk / steps) * 64 + kk;
    v4i v = {0, 0, 0, 0};
    if (k < K) v = *(const v4i *)(w + (int64_t)k * row + st * 64 + ch * 16);
    *(v4i *)(out + i * 16) = v;
}

hawq_status launch_block_weights(const void *w, void *w_blocked, int K, int64_t row, hipStream_t s) {
    const int64_t chunks = (int64_t)((K + 63) / 64) * (row / 64) * 256;
    if (chunks == 0) return HAWQ_OK;
    const int64_t blocks = (chunks + 255) / 256;
    if (blocks > 0x7fffffff) return HAWQ_ERR_UNSUPPORTED;
    block_weights_kernel<<<(uint32_t)blocks, 256, 0, s>>>((const uint8_t *)w, (uint8_t *)w_blocked, K, row, chunks);
    return check_launch();
}

}  // namespace hawq
