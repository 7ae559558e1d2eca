// Internal declarations shared by the kernels and the C interface (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "../../include/hawq.h"

namespace hawq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Everything a convolution kernel needs; passed by value as the kernel argument.
struct ConvArgs {
    const uint8_t *x;        // activations (bytes; 4-bit: packed)
    const uint8_t *w;        // weights [K][R*S*C] (bytes; 4-bit: packed)
    const int32_t *bias;     // [K]
    const int32_t *b;        // [K] or nullptr (raw output)
    const uint8_t *c;        // [K]
    const uint8_t *res;      // shortcut tensor [M][K] or nullptr
    const int32_t *res_b;
    const uint8_t *res_c;
    uint8_t *y;              // output [M][K]
    int32_t N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, P, Q;
    int32_t M;               // N*P*Q output pixels
    int32_t x_dt, w_dt, y_dt, res_dt;
    int32_t lo, hi;          // clamp with ReLU already folded in (lo = max(lo,0))
    // Optional second convolution on the shortcut branch (xs != nullptr; 1x1, unpadded, same N, P, Q, K): its INT32
    // accumulator plus bias_s is rescaled by (b_s, c_s) and added to the rescaled main branch.  res is null then.
    const uint8_t *xs;       // shortcut activations [N][Hs][Ws][Cs]
    const uint8_t *ws;       // shortcut weights [K][Cs]
    const int32_t *bias_s, *b_s;
    const uint8_t *c_s;
    int32_t Hs, Ws, Cs, stride_sh, stride_sw, xs_dt, ws_dt;
    // mid_s8: the shortcut accumulator is first requantised by (b_s, c_s) and clamped to the signed 8-bit tensor a separate
    // transition layer would store, and that value enters the sum rescaled by (res_b, res_c) -- the two-launch result
    // without the tensor's round trip through memory
    int32_t mid_s8;
    // w_t / ws_t (optional, the network plan provides them): the same weights as w / ws in blocked order for the
    // implicit-GEMM kernel -- [ceil(K/64)][row bytes / 64][64 channels][64 bytes], i.e. the [K][R*S*C] byte matrix cut
    // into 64-channel x 64-byte blocks, rows past K zero -- so that one K-step of a channel tile is contiguous memory
    const void *w_t, *ws_t;
    // w_f (optional): the weights in MFMA fragment order for the resident-pixel 3x3 kernel (launch_fragment_weights)
    const void *w_f;
    // ws_f (optional): the shortcut convolution's weights in the same fragment order (two-convolution form of conv_rp1.hip)
    const void *ws_f;
    // corun: kernels of another stream share the chip with this launch (the forward's two half-batches): configurations
    // meant for a launch that is alone (small tiles with a deep LDS ring when there are few tiles) are not chosen
    int32_t corun;
    // dual16 (two-convolution form, set by the network plan from host data): every (b, c) and (b_s, c_s) is in the narrow
    // evaluation's range and |rq(acc + bias, b, c)| of the main branch cannot exceed 32767 for any input
    int32_t dual16;
};

// Arguments of the resident-pixel 3x3 kernel (conv_rp.hip), with or without the fused 1x1 that ends a bottleneck block.
struct RpArgs {
    const uint8_t *x;        // input [N,H,W,C], 8-bit (signed operand range), or packed 4-bit when pk
    int32_t N, H, W, C;
    int32_t M;               // N*H*W pixels (the 3x3 convolution is stride 1, pad 1: as many output pixels)
    // stage 1: 3x3, C -> K1
    const uint8_t *w1f;      // weights in MFMA fragment order (launch_fragment_weights)
    const int32_t *bias1, *b1;
    const uint8_t *c1;
    int32_t K1, lo1, hi1;    // clamp with ReLU folded in
    // shortcut and output of the stage that stores to memory (stage 1 alone, or stage 2 when fused): [M][K] 8-bit
    const uint8_t *res;      // nullptr: none (plain form only; the fused form requires one)
    const int32_t *res_b;
    const uint8_t *res_c;
    int32_t res_dt;          // HAWQ_U8 | HAWQ_S8
    uint8_t *y;
    // stage 2 (fused form): 1x1, K1 -> K2
    const uint8_t *w2f;
    const int32_t *bias2, *b2;
    const uint8_t *c2;
    int32_t K2, lo2, hi2;
    int32_t corun;           // kernels of another stream share the chip (see ConvArgs::corun)
    int32_t pk;              // operands are packed 4-bit (unsigned activations, signed weights); plain form only, no shortcut
    int32_t y4;              // pk: the output is packed unsigned 4-bit (else one byte per channel)
#ifdef HAWQ_RP_TIMING
    long long *timing;       // measurement build only: [workgroup][wave][6] cycle stamps
#endif
};

// Arguments of the resident-pixel 1x1 kernel (conv_rp1.hip): one convolution with an optional shortcut tensor, or a block
// output with a convolution on both branches (xs != nullptr).
struct Rp1Args {
    const uint8_t *x;        // main operand [M][C], 8-bit (signed operand range)
    int32_t M, C;
    const uint8_t *wf;       // [K][C] weights in MFMA fragment order (launch_fragment_weights)
    const int32_t *bias, *b;
    const uint8_t *c;
    int32_t K, lo, hi;       // clamp with ReLU folded in
    const uint8_t *res;      // shortcut tensor [M][K] 8-bit or nullptr (one-convolution form only)
    const int32_t *res_b;    // its rescale -- or, two-convolution form with mid_s8, the stored shortcut's
    const uint8_t *res_c;
    int32_t res_dt;          // HAWQ_U8 | HAWQ_S8
    uint8_t *y;              // [M][K] 8-bit
    // shortcut convolution: 1x1, unpadded, strides (sh, sw) over [N][Hs][Ws][Cs]; output pixel m = (n P + p) Q + q
    const uint8_t *xs;
    const uint8_t *wsf;      // [K][Cs] weights in fragment order
    const int32_t *bias_s, *b_s;
    const uint8_t *c_s;
    int32_t Cs, PQ, Q, Hs, Ws, sh, sw;
    int32_t mid_s8;          // see ConvArgs::mid_s8
    int64_t xs_bytes;        // bytes of the xs tensor
    int32_t corun;           // see ConvArgs::corun
    int32_t npass;           // set by the launcher: groups of 256 output channels a workgroup walks
};

__host__ __device__ inline bool is4(int dt) { return dt == HAWQ_U4 || dt == HAWQ_S4; }
// bytes of `n` elements of a dense tensor of type dt (n even for 4-bit types)
__host__ __device__ inline int64_t tensor_bytes(int64_t n, int dt) {
    return dt == HAWQ_S32 ? n * 4 : (is4(dt) ? n / 2 : n);
}

// ---- dyadic requantisation: rq(t,b,c) = floor(t*b/2^c + 1/2), exact in 64-bit ----
__device__ __forceinline__ int64_t rq64(int32_t t, int32_t b, int32_t c) {
    return ((int64_t)t * (int64_t)b + ((int64_t)1 << (c - 1))) >> c;
}

__device__ __forceinline__ int32_t clamp64(int64_t v, int32_t lo, int32_t hi) {
    v = v < (int64_t)lo ? (int64_t)lo : v;
    v = v > (int64_t)hi ? (int64_t)hi : v;
    return (int32_t)v;
}

// Read logical element i of a dense tensor (slow path / element-wise kernels).
__device__ __forceinline__ int32_t load_elem(const void *p, int dt, int64_t i) {
    switch (dt) {
    case HAWQ_U8: return ((const uint8_t *)p)[i];
    case HAWQ_S8: return ((const int8_t *)p)[i];
    case HAWQ_S32: return ((const int32_t *)p)[i];
    case HAWQ_U4: {
        uint32_t v = ((const uint8_t *)p)[i >> 1];
        return (int32_t)((i & 1) ? (v >> 4) : (v & 0xF));
    }
    default: {
        uint32_t v = ((const uint8_t *)p)[i >> 1];
        int32_t n = (int32_t)((i & 1) ? (v >> 4) : (v & 0xF));
        return n >= 8 ? n - 16 : n;
    }
    }
}

// Compile-time loop: indices into register arrays stay constants even when the body is large.
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// Per-byte unsigned maximum / minimum of packed dwords through the packed 16-bit ALU: the even bytes and the odd
// bytes of a dword are compared as two 16-bit lanes each (odd bytes in place, in the high byte of a lane whose low
// byte is zero).
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b)));
}
__device__ __forceinline__ uint32_t pk_min_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b)));
}
__device__ __forceinline__ uint32_t max_u8x4(uint32_t a, uint32_t b) {
    return pk_max_u16(a & 0x00ff00ffu, b & 0x00ff00ffu) | pk_max_u16(a & 0xff00ff00u, b & 0xff00ff00u);
}
// per-byte clamp of packed unsigned bytes to [lo, hi] (0 <= lo <= hi <= 255)
__device__ __forceinline__ uint32_t clamp_u8x4(uint32_t a, uint32_t lo, uint32_t hi) {
    const uint32_t le = lo * 0x00010001u, he = hi * 0x00010001u;
    const uint32_t e = pk_min_u16(pk_max_u16(a & 0x00ff00ffu, le), he);
    const uint32_t o = pk_min_u16(pk_max_u16(a & 0xff00ff00u, le << 8), he << 8);
    return e | o;
}

// XCD-aware remap of a linear workgroup id.  Workgroups are dealt round-robin to the 8 XCDs
// (each with its own L2); this gives every XCD one contiguous range of logical tile ids so
// neighbouring tiles (shared input halo, shared activation rows) meet in the same L2.
__device__ __forceinline__ uint32_t xcd_remap(uint32_t bid, uint32_t nblocks) {
    const uint32_t per = nblocks >> 3, rem = nblocks & 7u;
    const uint32_t xcd = bid & 7u, idx = bid >> 3;
    return xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
}

// ---- launchers (host) ----
hawq_status launch_conv_mfma(const ConvArgs &a, hipStream_t s);     // requires conv_mfma_eligible
bool conv_mfma_eligible(const ConvArgs &a, int x_hi);
void set_tile_override(int t);
int tile_override();
// 3x3 / stride 1 / pad 1, 64 -> 64 channels, INT8: weights resident in LDS, pixel operand kept across the taps
bool conv3x3_c64_eligible(const ConvArgs &a, int x_hi);
hawq_status launch_conv3x3_c64(const ConvArgs &a, hipStream_t s);
hawq_status launch_conv_direct(const ConvArgs &a, hipStream_t s);   // any valid shape (also with a shortcut convolution)
// matrix-core kernel for a block output with a convolution on both branches (ConvArgs::xs set)
bool conv_mfma_dual_eligible(const ConvArgs &a, int x_hi, int xs_hi);
hawq_status launch_conv_mfma_dual(const ConvArgs &a, hipStream_t s);
// persistent streaming form of the same for 1x1 main branches: (C, Cs) = (64, 64) or (128, 256), many pixels
bool conv_pws_dual_shape_ok(int C, int Cs, int K, int64_t M);
bool conv_pws_dual_eligible(const ConvArgs &a, int x_hi, int xs_hi);
hawq_status launch_conv_pws_dual(const ConvArgs &a, hipStream_t s);
// persistent streaming kernel for 1x1 convolutions with C = 64 / 128 (/ 256 with few output channels) and many pixels
bool conv_pw_eligible(const ConvArgs &a, int x_hi);
hawq_status launch_conv_pw(const ConvArgs &a, hipStream_t s);
// same, for C = 256 with K >= 256 a multiple of 128: the activation stage is shared by a workgroup's four waves
bool conv_pws_eligible(const ConvArgs &a, int x_hi);
hawq_status launch_conv_pws(const ConvArgs &a, hipStream_t s);
// few rows, long reduction (the fully connected layer): eight waves split the reduction, partial tiles meet in LDS
bool gemm_splitk_eligible(const ConvArgs &a);
hawq_status launch_gemm_splitk(const ConvArgs &a, int x_hi, hipStream_t s);
// conv1 of the networks: 7x7/2 pad 3, C=3 -> 64, weights re-tiled to [64][8][8][4] and the
// bias corrected for the -128 input offset by the host (see net.hip)
hawq_status launch_conv_stem(const ConvArgs &a, hipStream_t s);
// conv1 fused with the 3x3/2 max pool: writes only the pooled tensor (U8 or packed U4)
hawq_status launch_conv_stem_pool(const ConvArgs &a, int pool_y_dt, int pool_lo, int pool_hi, void *pool_y, hipStream_t s);
hawq_status launch_residual_add(int64_t n_pixels, int K, int m_dt, int r_dt, int y_dt, const void *m,
                                const int32_t *m_b, const uint8_t *m_c, const void *r, const int32_t *r_b,
                                const uint8_t *r_c, int lo, int hi, void *y, hipStream_t s);
hawq_status launch_avgpool(int N, int HW, int C, int x_dt, int y_dt, const void *x, const int32_t *b,
                           const uint8_t *c, int lo, int hi, void *y, hipStream_t s);
hawq_status launch_maxpool(int N, int H, int W, int C, int x_dt, int y_dt, const void *x, int lo, int hi, void *y,
                           hipStream_t s);

hawq_status launch_pool_sum(int N, int H, int W, int C, int R, int S, int sh, int sw, int ph, int pw, int x_dt, int y_dt,
                            const void *x, const int32_t *b, const uint8_t *c, int lo, int hi, void *y, hipStream_t s);
hawq_status launch_concat_branch(int64_t n_pixels, int K, int Kt, int off, int q_dt, int y_dt, const void *q, const int32_t *b,
                                 const uint8_t *c, int lo, int hi, void *y, hipStream_t s);

// resident-pixel 3x3 (+ fused 1x1) kernel: shape test and launch (operand types / alignment are the caller's to check)
bool conv_rp_shape_ok(const RpArgs &a, bool fused);
// RpArgs from a validated 3x3 layer (and, fused, the 1x1 layer that follows it); false if types, alignment or shape do not fit
bool make_rp_args(const ConvArgs &a1, int x_hi, const ConvArgs *a2, const void *w2f, RpArgs &r);
hawq_status launch_conv_rp(const RpArgs &a, bool fused, hipStream_t s);
// resident-pixel 1x1 kernel (one convolution + optional shortcut tensor, or two convolutions when a.xs is set and the
// caller vouches for a.dual16): Rp1Args from validated requests; false if types, alignment or shape do not fit
bool conv_rp1_shape_ok(const Rp1Args &a);
bool make_rp1_args(const ConvArgs &a, int x_hi, int xs_hi, Rp1Args &r);
hawq_status launch_conv_rp1(const Rp1Args &a, hipStream_t s);
// [K][row bytes] weights -> MFMA fragment order for that kernel (four: packed 4-bit rows, expanded to bytes on the way);
// out: ceil(K/32) * 32 * (bytes of an expanded row)
hawq_status launch_fragment_weights(const void *w, void *w_frag, int K, int64_t row, bool four, hipStream_t s);

// [K][row bytes] weights -> the implicit-GEMM kernel's blocked order (ConvArgs::w_t); row a multiple of 64
hawq_status launch_block_weights(const void *w, void *w_blocked, int K, int64_t row, hipStream_t s);

inline hawq_status check_launch() { return hipGetLastError() == hipSuccess ? HAWQ_OK : HAWQ_ERR_DEVICE; }

}  // namespace hawq
