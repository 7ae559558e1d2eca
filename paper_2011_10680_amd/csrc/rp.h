// Pieces shared by the resident-pixel kernels (conv_rp.hip: 3x3, conv_rp1.hip: 1x1): the per-channel parameters as staged
// in LDS and the integer epilogue of one lane (Section 3.1's requantisation, Section 3.3's rescaled shortcut).
#pragma once
#include "common.h"

namespace hawq {

// Per-channel parameters as staged in LDS.  narrow evaluation (c <= 32, b < 2^(c-1)):  rq(acc + bias, b, c) = high word of
// acc * bs + Rs  with bs = b << (32-c), Rs = (bias*b + 2^(c-1)) << (32-c); any other channel makes the whole workgroup
// take the exact 64-bit evaluation from (bias, b, c).
struct RpChan { int32_t bs, b, c, bias; int64_t Rs; };
struct RpRes { int32_t rb, rc; };

// Epilogue of one lane: NT (1 or 2) of its pixels (MFMA column tiles T0, T0 + 1) x 16 consecutive channels.  pc / pr: the
// lane's first channel's entries.  resw[t]: the 16 shortcut bytes of pixel T0 + t (only read when has_res).  Result:
// out[t] = the 16 output bytes.  (Two pixels per call: a channel's parameters are read once for both, and the
// intermediate values of all pixels at once would not fit the register budget next to the accumulators and the
// prefetched weights.)
template <int NT>
__device__ __forceinline__ void rp_epilogue(const v16i &acc0, const v16i &acc1, const RpChan *pc, const RpRes *pr, const bool has_res,
                                            const bool res_signed, const uint32_t (&resw)[2][4], const int wide, const int lo_,
                                            const int hi_, uint32_t (&out)[2][4]) {
    if (wide) {
        // Exact general form (64-bit products, shifts and clamp), written as a compact loop because it is cold: every round
        // handles element 0 of the accumulators and the low shortcut byte, then rotates both by one element, and shifts the
        // new output byte in from the top of the 128-bit result (after sixteen rounds everything is back in place).
        const uint32_t sgn = res_signed ? 0x80u : 0u;   // signed bytes: subtract 256 where bit 7 is set
        v16i t0 = acc0, t1 = acc1;
        uint32_t r0[4] = {resw[0][0], resw[0][1], resw[0][2], resw[0][3]};
        uint32_t r1[4] = {resw[1][0], resw[1][1], resw[1][2], resw[1][3]};
        uint32_t o0[4] = {0, 0, 0, 0}, o1[4] = {0, 0, 0, 0};
#pragma unroll 1
        for (int i = 0; i < 16; ++i) {
            const RpChan p = pc[i];
            const RpRes q = has_res ? pr[i] : RpRes{0, 1};   // (no shortcut: the bytes are zero and rq(0, 0, 1) = 0)
            const uint32_t w0 = r0[0] & 0xff, w1 = r1[0] & 0xff;
            const int64_t v0 = rq64(t0[0] + p.bias, p.b, p.c) + rq64((int32_t)w0 - (int32_t)((w0 & sgn) << 1), q.rb, q.rc);
            const int64_t v1 = rq64(t1[0] + p.bias, p.b, p.c) + rq64((int32_t)w1 - (int32_t)((w1 & sgn) << 1), q.rb, q.rc);
            const uint32_t b0 = (uint32_t)clamp64(v0, lo_, hi_) & 0xff, b1 = (uint32_t)clamp64(v1, lo_, hi_) & 0xff;
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                o0[j] = (o0[j] >> 8) | (o0[j + 1] << 24); o1[j] = (o1[j] >> 8) | (o1[j + 1] << 24);
                r0[j] = (r0[j] >> 8) | (r0[j + 1] << 24); r1[j] = (r1[j] >> 8) | (r1[j + 1] << 24);
            }
            o0[3] = (o0[3] >> 8) | (b0 << 24); o1[3] = (o1[3] >> 8) | (b1 << 24);
            r0[3] >>= 8; r1[3] >>= 8;
            t0 = __builtin_shufflevector(t0, t0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 0);
            t1 = __builtin_shufflevector(t1, t1, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 0);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) { out[0][j] = o0[j]; out[1][j] = o1[j]; }
        return;
    }
    int32_t lo = lo_, hi = hi_;
    asm volatile("" : "+v"(lo), "+v"(hi));   // in vector registers: the clamp is then one three-operand median
    int32_t y[2][16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int32_t bs = pc[i].bs;
        const int64_t Rs = pc[i].Rs;
        y[0][i] = (int32_t)(((int64_t)acc0[i] * (int64_t)bs + Rs) >> 32);
        if (NT == 2) y[1][i] = (int32_t)(((int64_t)acc1[i] * (int64_t)bs + Rs) >> 32);
    }
    if (has_res) {
        auto add_res = [&](auto sc) {
            constexpr bool S = decltype(sc)::value;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const RpRes p = pr[i];
                const int32_t rr = (int32_t)(1u << ((p.rc - 1) & 31));
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const int32_t r = S ? __builtin_amdgcn_sbfe((int32_t)resw[t][i >> 2], 8 * (i & 3), 8)
                                        : (int32_t)__builtin_amdgcn_ubfe(resw[t][i >> 2], 8 * (i & 3), 8);
                    y[t][i] += (__mul24(r, p.rb) + rr) >> p.rc;
                }
            }
        };
        if (res_signed) add_res(std::true_type{});
        else add_res(std::false_type{});
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            int32_t v;
            asm("v_med3_i32 %0, %1, %2, %3" : "=v"(v) : "v"(y[t][i]), "v"(lo), "v"(hi));
            y[t][i] = v;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {   // low bytes of 4 values -> one dword
            const uint32_t t0 = __builtin_amdgcn_perm((uint32_t)y[t][4 * q + 1], (uint32_t)y[t][4 * q], 0x0c0c0400u);
            const uint32_t t1 = __builtin_amdgcn_perm((uint32_t)y[t][4 * q + 3], (uint32_t)y[t][4 * q + 2], 0x04000c0cu);
            out[t][q] = t0 | t1;
        }
    }
    if (NT == 1) out[1][0] = out[1][1] = out[1][2] = out[1][3] = 0;   // (every element written on every path keeps the array in registers)
}

}  // namespace hawq
