// Fused epilogue of the matrix-core convolution kernels: bias add, dyadic requantisation,
// dyadic-rescaled shortcut add, ReLU / clamp, packing and the NHWC store.
//
// Register layout it expects: a lane owns, for one output pixel, GROUPS*16 consecutive output
// channels starting at `ch0`; acc[g][i] is channel ch0 + 16*g + i.  That makes every store a
// contiguous 16-byte (8-bit outputs), 8-byte (4-bit) or 64-byte (INT32) run per group.
#pragma once
#include "common.h"

namespace hawq {

struct EpiParams4 {  // parameters of 4 consecutive channels
    int32_t bias[4], b[4], c[4], rb[4], rc[4];
};

template <bool VEC>
__device__ __forceinline__ void load_params4(const ConvArgs &a, int ch, bool has_rq, bool has_res, EpiParams4 &p) {
    if (VEC) {
        const v4i bv = *(const v4i *)(a.bias + ch);
        p.bias[0] = bv[0]; p.bias[1] = bv[1]; p.bias[2] = bv[2]; p.bias[3] = bv[3];
        if (has_rq) {
            const v4i mv = *(const v4i *)(a.b + ch);
            const uint32_t cv = *(const uint32_t *)(a.c + ch);
            p.b[0] = mv[0]; p.b[1] = mv[1]; p.b[2] = mv[2]; p.b[3] = mv[3];
            p.c[0] = cv & 0xff; p.c[1] = (cv >> 8) & 0xff; p.c[2] = (cv >> 16) & 0xff; p.c[3] = cv >> 24;
        }
        if (has_res) {
            const v4i mv = *(const v4i *)(a.res_b + ch);
            const uint32_t cv = *(const uint32_t *)(a.res_c + ch);
            p.rb[0] = mv[0]; p.rb[1] = mv[1]; p.rb[2] = mv[2]; p.rb[3] = mv[3];
            p.rc[0] = cv & 0xff; p.rc[1] = (cv >> 8) & 0xff; p.rc[2] = (cv >> 16) & 0xff; p.rc[3] = cv >> 24;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool ok = ch + j < a.K;
            p.bias[j] = ok ? a.bias[ch + j] : 0;
            p.b[j] = (ok && has_rq) ? a.b[ch + j] : 0;
            p.c[j] = (ok && has_rq) ? a.c[ch + j] : 1;
            p.rb[j] = (ok && has_res) ? a.res_b[ch + j] : 0;
            p.rc[j] = (ok && has_res) ? a.res_c[ch + j] : 1;
        }
    }
}

// value of shortcut element j (0..3) of a group of 4 channels held in `word`
// (8-bit: 4 bytes in one dword; 4-bit: 4 nibbles in the low 16 bits)
__device__ __forceinline__ int32_t res_elem(uint32_t word, int j, int res_dt) {
    switch (res_dt) {
    case HAWQ_U8: return (int32_t)((word >> (8 * j)) & 0xff);
    case HAWQ_S8: return (int32_t)(int8_t)((word >> (8 * j)) & 0xff);
    case HAWQ_U4: return (int32_t)((word >> (4 * j)) & 0xf);
    default: {
        int32_t n = (int32_t)((word >> (4 * j)) & 0xf);
        return n >= 8 ? n - 16 : n;
    }
    }
}

// One output value: accumulator -> stored integer.
__device__ __forceinline__ int32_t finish(int32_t acc, const EpiParams4 &p, int j, bool has_rq, bool has_res, int32_t r,
                                          int32_t lo, int32_t hi) {
    const int32_t t = acc + p.bias[j];
    if (!has_rq) return t;
    int64_t v = rq64(t, p.b[j], p.c[j]);
    if (has_res) v += rq64(r, p.rb[j], p.rc[j]);
    return clamp64(v, lo, hi);
}

// Epilogue for one pixel `m` and GROUPS*16 channels starting at ch0 (ch0 % 16 == 0).
// VEC: K % 16 == 0 and all arrays 16-byte aligned -> vector loads/stores; otherwise a guarded
// element-wise path (still one lane per pixel x 16-channel group).
template <int GROUPS, bool VEC>
__device__ __forceinline__ void epilogue_pixel(const ConvArgs &a, int64_t m, int ch0, const v16i (&acc)[GROUPS]) {
    const bool has_rq = a.b != nullptr;
    const bool has_res = a.res != nullptr;
    const int y_dt = a.y_dt, res_dt = a.res_dt;
    const int64_t o = m * (int64_t)a.K + ch0;  // element offset of the lane's first channel
    static_for<0, GROUPS>([&](auto gc) {
        constexpr int g = decltype(gc)::value;
        const int chg = ch0 + 16 * g;
        if (chg >= a.K) return;
        // shortcut values of the 16 channels, as 4 words of 4 channels
        uint32_t rw[4] = {0, 0, 0, 0};
        if (has_res) {
            if (VEC) {
                if (is4(res_dt)) {
                    const uint2 t = *(const uint2 *)(a.res + ((o + 16 * g) >> 1));
                    rw[0] = t.x & 0xffff; rw[1] = t.x >> 16; rw[2] = t.y & 0xffff; rw[3] = t.y >> 16;
                } else {
                    const uint4 t = *(const uint4 *)(a.res + (o + 16 * g));
                    rw[0] = t.x; rw[1] = t.y; rw[2] = t.z; rw[3] = t.w;
                }
            }
        }
        uint32_t out8[4];   // 8-bit outputs: 4 dwords;  4-bit outputs: out8[0..1]
        uint32_t out4[2] = {0, 0};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            EpiParams4 p;
            load_params4<VEC>(a, chg + 4 * q, has_rq, has_res, p);
            int32_t v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int32_t r = 0;
                if (has_res) {
                    if (VEC) r = res_elem(rw[q], j, res_dt);
                    else if (chg + 4 * q + j < a.K) r = load_elem(a.res, res_dt, o + 16 * g + 4 * q + j);
                }
                v[j] = finish(acc[g][4 * q + j], p, j, has_rq, has_res, r, a.lo, a.hi);
            }
            if (VEC) {
                if (y_dt == HAWQ_S32) {
                    v4i t = {v[0], v[1], v[2], v[3]};
                    *(v4i *)(a.y + 4 * (o + 16 * g + 4 * q)) = t;
                } else if (is4(y_dt)) {
                    const uint32_t h = (v[0] & 0xf) | ((v[1] & 0xf) << 4) | ((v[2] & 0xf) << 8) | ((v[3] & 0xf) << 12);
                    out4[q >> 1] |= h << (16 * (q & 1));
                } else {
                    out8[q] = (v[0] & 0xff) | ((v[1] & 0xff) << 8) | ((v[2] & 0xff) << 16) | ((uint32_t)v[3] << 24);
                }
            } else {
                // guarded element-wise stores; 4-bit outputs are written a byte (2 channels) at a time,
                // K is even for them so a pair never straddles the channel edge
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int ch = chg + 4 * q + j;
                    if (ch >= a.K) continue;
                    const int64_t e = o + 16 * g + 4 * q + j;
                    if (y_dt == HAWQ_S32) ((int32_t *)a.y)[e] = v[j];
                    else if (is4(y_dt)) {
                        if ((j & 1) == 0) a.y[e >> 1] = (uint8_t)((v[j] & 0xf) | ((v[j + 1] & 0xf) << 4));
                    } else a.y[e] = (uint8_t)v[j];
                }
            }
        }
        if (VEC) {
            if (is4(y_dt)) {
                *(uint2 *)(a.y + ((o + 16 * g) >> 1)) = make_uint2(out4[0], out4[1]);
            } else if (y_dt != HAWQ_S32) {
                *(uint4 *)(a.y + (o + 16 * g)) = make_uint4(out8[0], out8[1], out8[2], out8[3]);
            }
        }
    });
}


// ------------------------------------------------------------------------------------------
// Tile epilogue with per-channel parameters staged in LDS (the hot variant).
//
// stage_channel() prepares one channel as
//     main: { b, c, R = bias*b + 2^(c-1) }                   so that  rq(acc+bias) = (acc*b + R) >> c
//           { bs = b << (32-c), Rs = R << (32-c) }            so that  rq(acc+bias) = high word of acc*bs + Rs
//     res : { rb, rc, 2^(rc-1) }
// and reports whether the channel allows the narrow evaluation:
//     main: c <= 32 and b < 2^(c-1)  -> bs fits a signed 32-bit operand, the result fits int32 and the
//                                        shift disappears into "take the high word"
//     res : rc <= 31 and rb < 2^22   -> |r| <= 255 keeps r*rb + 2^(rc-1) inside int32
// A workgroup (or wave) with any other channel takes the general path: 64-bit shift and clamp.
// Both paths compute the same exact integer.
struct ChanMain { int32_t b, c; int64_t R; int32_t bs, bias; int64_t Rs; };
struct ChanRes { int32_t rb, rc, rround, rbs; };   // rbs: res_b << (T - res_c) for the register-resident form's wave-uniform T

__device__ __forceinline__ int stage_channel(const ConvArgs &a, int k, ChanMain &m, ChanRes &r) {
    int wide = 0;
    m = ChanMain{0, 1, 0, 0, 0, 0};
    r = ChanRes{0, 1, 1, 0};
    if (k < a.K) {
        m.b = a.b[k]; m.c = a.c[k]; m.bias = a.bias[k];
        m.R = (int64_t)a.bias[k] * (int64_t)m.b + ((int64_t)1 << (m.c - 1));
        if (m.c > 32 || ((int64_t)m.b >> (m.c - 1)) != 0) {
            wide = 1;
        } else {
            m.bs = (int32_t)((uint32_t)m.b << (32 - m.c));
            m.Rs = (int64_t)((uint64_t)m.R << (32 - m.c));
        }
        if (a.res != nullptr) {
            r.rb = a.res_b[k]; r.rc = a.res_c[k];
            if (r.rc > 31 || r.rb >= (1 << 22)) wide = 1;
            r.rround = (int32_t)(1u << ((r.rc - 1) & 31));
        }
    }
    return wide;
}

// One branch of a two-convolution block output: { bias, b, c } of channel k in ChanMain form.
__device__ __forceinline__ int stage_branch(const int32_t *bias, const int32_t *b, const uint8_t *c, int k, int K, ChanMain &m) {
    int wide = 0;
    m = ChanMain{0, 1, 0, 0, 0, 0};
    if (k < K) {
        m.b = b[k]; m.c = c[k];
        m.R = (int64_t)bias[k] * (int64_t)m.b + ((int64_t)1 << (m.c - 1));
        if (m.c > 32 || ((int64_t)m.b >> (m.c - 1)) != 0) {
            wide = 1;
        } else {
            m.bs = (int32_t)((uint32_t)m.b << (32 - m.c));
            m.Rs = (int64_t)((uint64_t)m.R << (32 - m.c));
        }
    }
    return wide;
}

// The stored-shortcut form's second rescaling { res_b, res_c } of channel k; wide if outside the narrow evaluation's range.
__device__ __forceinline__ int stage_res(const int32_t *res_b, const uint8_t *res_c, int k, int K, ChanRes &r) {
    int wide = 0;
    r = ChanRes{0, 1, 1, 0};
    if (k < K) {
        r.rb = res_b[k]; r.rc = res_c[k];
        if (r.rc > 31 || r.rb >= (1 << 22)) wide = 1;
        r.rround = (int32_t)(1u << ((r.rc - 1) & 31));
    }
    return wide;
}

// pr != nullptr: also stage res_b / res_c (the shortcut passes through a signed 8-bit value)
__device__ __forceinline__ int stage_params_dual(const ConvArgs &a, int k0, int n_ch, ChanMain *pm, ChanMain *ps, ChanRes *pr) {
    int wide = 0;
    const int i = threadIdx.x;
    if (i < n_ch) {
        ChanMain m, r;
        wide = stage_branch(a.bias, a.b, a.c, k0 + i, a.K, m) | stage_branch(a.bias_s, a.b_s, a.c_s, k0 + i, a.K, r);
        pm[i] = m;
        ps[i] = r;
        if (pr != nullptr) {
            ChanRes q;
            wide |= stage_res(a.res_b, a.res_c, k0 + i, a.K, q);
            pr[i] = q;
        }
    }
    return wide;
}

__device__ __forceinline__ int stage_params(const ConvArgs &a, int k0, int n_ch, ChanMain *pm, ChanRes *pr) {
    int wide = 0;
    const int i = threadIdx.x;
    if (i < n_ch && a.b != nullptr) {
        ChanMain m;
        ChanRes r;
        wide = stage_channel(a, k0 + i, m, r);
        pm[i] = m;
        pr[i] = r;
    }
    return wide;
}

// Epilogue of one lane: TP pixels (m[tp], valid[tp]) x TC*16 consecutive channels starting at
// workgroup-relative channel `chl` (absolute ch0 = k0 + chl).  8-bit or packed 4-bit outputs,
// requantising, vector stores; requires K % 16 == 0.
// `pre` holds the lane's shortcut data already fetched by the caller when PRE is set
// (pre[tp][tc][0..3]: the 16 bytes, or 8 bytes for 4-bit data in [0..1], of channel group tc);
// arrays are taken by reference so they stay in registers.
//
// Exact general form (64-bit shift, 64-bit clamp, every type combination); also the wide path.
template <int TC, int TP, bool PRE>
__device__ __forceinline__ void epilogue_tile_general(const ConvArgs &a, const ChanMain *pm, const ChanRes *pr,
                                                      const int64_t (&m)[TP], const bool (&valid)[TP], int k0, int chl,
                                                      const v16i (&acc_in)[TP][TC], const uint32_t (&pre)[TP][TC][4]) {
    const int y_dt = a.y_dt, res_dt = a.res_dt;
    const bool y4 = is4(y_dt), r4 = is4(res_dt), has_res = a.res != nullptr;
    const int32_t lo = a.lo, hi = a.hi;
    static_for<0, TC>([&](auto gc) {
        constexpr int g = decltype(gc)::value;
        const int chg = k0 + chl + 16 * g;
        if (chg >= a.K) return;
        static_for<0, TP>([&](auto tpc) {
            constexpr int tp = decltype(tpc)::value;
            if (!valid[tp]) return;
            const int64_t o = m[tp] * (int64_t)a.K + chg;
            uint32_t ow[4] = {0, 0, 0, 0};
            static_for<0, 16>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                const ChanMain pmv = pm[chl + 16 * g + i];
                int32_t av = acc_in[tp][g][i];
                // opaque copy: keeps this cold path's products from being merged with (and hoisted above) the
                // narrow path's identical expressions
                asm volatile("" : "+v"(av));
                int64_t w64 = ((int64_t)av * (int64_t)pmv.b + pmv.R) >> pmv.c;
                if (has_res) {
                    const ChanRes prv = pr[chl + 16 * g + i];
                    int32_t r;
                    if (PRE) {
                        const uint32_t w = r4 ? (pre[tp][g][i >> 3] >> (4 * (i & 7))) & 0xf : (pre[tp][g][i >> 2] >> (8 * (i & 3))) & 0xff;
                        r = (int32_t)w;
                        if (res_dt == HAWQ_S8) r = (int32_t)(int8_t)w;
                        if (res_dt == HAWQ_S4) r = (r ^ 8) - 8;
                    } else {
                        r = load_elem(a.res, res_dt, o + i);
                    }
                    w64 += rq64(r, prv.rb, prv.rc);
                }
                const int32_t y = clamp64(w64, lo, hi);
                if (y4) ow[i >> 3] |= (uint32_t)(y & 0xf) << (4 * (i & 7));
                else ow[i >> 2] |= (uint32_t)(y & 0xff) << (8 * (i & 3));
            });
            if (y4) *(uint2 *)(a.y + (o >> 1)) = make_uint2(ow[0], ow[1]);
            else *(uint4 *)(a.y + o) = make_uint4(ow[0], ow[1], ow[2], ow[3]);
        });
    });
}

// Hot form.  Runs in three passes over the lane's outputs so that every type / path decision is one
// uniform branch per pass instead of several per output:
//   1. y = (acc * b + R) >> c        one 64-bit multiply-add and one funnel shift per output
//   2. y += (r * rb + 2^(rc-1)) >> rc  per shortcut type (u8 / s8 / u4), 24-bit multiply-add
//   3. clamp, pack 4 (or 8) outputs per dword, 16-byte (8-byte) store per 16 channels
// `wide` (a channel outside the narrow range) or a signed 4-bit tensor take the general form.
// YMODE 0: plain global stores of the valid pixels.  1: a.y points into LDS (a kernel that keeps the requantised
// tile on chip, 64 channels per pixel, chunk-swizzled -- see the store below); stores use LDS instructions.  2: every lane issues its store as a buffer store, invalid pixels
// with an out-of-range offset that the hardware drops -- the number of memory instructions is then the same
// for every wave, which lets a caller count outstanding operations exactly.
template <int TC, int TP, bool PRE, int YMODE = 0>
__device__ __forceinline__ void epilogue_tile(const ConvArgs &a, const ChanMain *pm, const ChanRes *pr, const int64_t (&m)[TP],
                                              const bool (&valid)[TP], int k0, int chl, const v16i (&acc)[TP][TC], int wide,
                                              const uint32_t (&pre)[TP][TC][4]) {
    const int y_dt = a.y_dt, res_dt = a.res_dt;
    const bool has_res = a.res != nullptr;
    if (wide || y_dt == HAWQ_S4 || (has_res && res_dt == HAWQ_S4)) {
        epilogue_tile_general<TC, TP, PRE>(a, pm, pr, m, valid, k0, chl, acc, pre);
        return;
    }
    const bool y4 = is4(y_dt);
    const __amdgpu_buffer_rsrc_t yrs = __builtin_amdgcn_make_buffer_rsrc(
        (void *)a.y, 0, YMODE == 2 ? (int)tensor_bytes((int64_t)a.M * a.K, y_dt) : 0, 0x00020000);
    // clamp bounds in vector registers so the clamp is a single three-operand median
    int32_t lo = a.lo, hi = a.hi;
    asm volatile("" : "+v"(lo), "+v"(hi));
    static_for<0, TC>([&](auto gc) {
        constexpr int g = decltype(gc)::value;
        const int chg = k0 + chl + 16 * g;
        if (chg >= a.K) return;
        int32_t y[TP][16];
        // ---- pass 1: main branch ----
        static_for<0, 16>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            const ChanMain &pc = pm[chl + 16 * g + i];
            const int32_t bs = pc.bs;
            const int64_t Rs = pc.Rs;
#pragma unroll
            for (int tp = 0; tp < TP; ++tp) y[tp][i] = (int32_t)(((int64_t)acc[tp][g][i] * (int64_t)bs + Rs) >> 32);
        });
        // ---- pass 2: shortcut ----
        if (has_res) {
            uint32_t rw[TP][4];
#pragma unroll
            for (int tp = 0; tp < TP; ++tp) {
                rw[tp][0] = rw[tp][1] = rw[tp][2] = rw[tp][3] = 0;
                if (PRE) {
                    rw[tp][0] = pre[tp][g][0]; rw[tp][1] = pre[tp][g][1]; rw[tp][2] = pre[tp][g][2]; rw[tp][3] = pre[tp][g][3];
                } else if (valid[tp]) {
                    const int64_t o = m[tp] * (int64_t)a.K + chg;
                    if (res_dt == HAWQ_U4) {
                        const uint2 t = *(const uint2 *)(a.res + (o >> 1));
                        rw[tp][0] = t.x; rw[tp][1] = t.y;
                    } else {
                        const uint4 t = *(const uint4 *)(a.res + o);
                        rw[tp][0] = t.x; rw[tp][1] = t.y; rw[tp][2] = t.z; rw[tp][3] = t.w;
                    }
                }
            }
            auto add_res = [&](auto kindc) {
                constexpr int kind = decltype(kindc)::value;   // 0: u8, 1: s8, 2: u4
                static_for<0, 16>([&](auto ic) {
                    constexpr int i = decltype(ic)::value;
                    const ChanRes prv = pr[chl + 16 * g + i];
#pragma unroll
                    for (int tp = 0; tp < TP; ++tp) {
                        int32_t r;
                        if (kind == 0) r = (int32_t)__builtin_amdgcn_ubfe(rw[tp][i >> 2], 8 * (i & 3), 8);
                        else if (kind == 1) r = __builtin_amdgcn_sbfe((int32_t)rw[tp][i >> 2], 8 * (i & 3), 8);
                        else r = (int32_t)__builtin_amdgcn_ubfe(rw[tp][i >> 3], 4 * (i & 7), 4);
                        y[tp][i] += (__mul24(r, prv.rb) + prv.rround) >> prv.rc;
                    }
                });
            };
            if (res_dt == HAWQ_U8) add_res(std::integral_constant<int, 0>{});
            else if (res_dt == HAWQ_S8) add_res(std::integral_constant<int, 1>{});
            else add_res(std::integral_constant<int, 2>{});
        }
        // ---- pass 3: clamp, pack, store ----
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                int32_t t;   // lo <= hi is validated by the interface, so the median is the clamp
                asm("v_med3_i32 %0, %1, %2, %3" : "=v"(t) : "v"(y[tp][i]), "v"(lo), "v"(hi));
                y[tp][i] = t;
            }
        }
        if (y4) {
#pragma unroll
            for (int tp = 0; tp < TP; ++tp) {
                uint32_t w0 = 0, w1 = 0;
#pragma unroll
                for (int i = 0; i < 8; ++i) {   // values are within 0..15 after the clamp (unsigned 4-bit output)
                    w0 |= (uint32_t)y[tp][i] << (4 * i);
                    w1 |= (uint32_t)y[tp][8 + i] << (4 * i);
                }
                if (YMODE == 2) {
                    const uint32_t off = valid[tp] ? (uint32_t)((m[tp] * (int64_t)a.K + chg) >> 1) : 0x80000000u;
                    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(v2i, make_uint2(w0, w1)), yrs, (int)off, 0, 0);
                } else if (valid[tp]) {
                    *(uint2 *)(a.y + ((m[tp] * (int64_t)a.K + chg) >> 1)) = make_uint2(w0, w1);
                }
            }
        } else {
#pragma unroll
            for (int tp = 0; tp < TP; ++tp) {
                uint32_t w[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {   // low bytes of 4 values -> one dword (works for signed outputs too)
                    const uint32_t t0 = __builtin_amdgcn_perm((uint32_t)y[tp][4 * q + 1], (uint32_t)y[tp][4 * q], 0x0c0c0400u);
                    const uint32_t t1 = __builtin_amdgcn_perm((uint32_t)y[tp][4 * q + 3], (uint32_t)y[tp][4 * q + 2], 0x04000c0cu);
                    w[q] = t0 | t1;
                }
                if (YMODE == 2) {
                    const uint32_t off = valid[tp] ? (uint32_t)(m[tp] * (int64_t)a.K + chg) : 0x80000000u;
                    __builtin_amdgcn_raw_buffer_store_b128((v4i){(int)w[0], (int)w[1], (int)w[2], (int)w[3]}, yrs, (int)off, 0, 0);
                } else if (valid[tp]) {
                    if (YMODE == 1) {
                        // LDS tile of 64-byte pixels: the four 16-byte chunks of a pixel are XOR-swizzled with
                        // (pixel >> 2) & 3, so that the sixteen lanes of a store phase (consecutive pixels, one
                        // chunk) fall into different banks
                        typedef __attribute__((address_space(3))) v4i lds_v4i;
                        const int pix = (int)m[tp];
                        *(lds_v4i *)(a.y + (pix * 64 + ((((chg >> 4) ^ (pix >> 2)) & 3) << 4))) = (v4i){(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
                    } else {
                        *(uint4 *)(a.y + (m[tp] * (int64_t)a.K + chg)) = make_uint4(w[0], w[1], w[2], w[3]);
                    }
                }
            }
        }
    });
}

// ------------------------------------------------------------------------------------------
// Register-resident form for the persistent kernels (a wave keeps its 32 output channels for its whole life, so the
// parameters of a lane's 16 channels can stay in registers; read from LDS per output they cost as much LDS bandwidth as the
// epilogue costs VALU time).  Two rewritings make three registers per channel enough:
//   * the accumulator starts at bias[k] instead of 0, and  rq(t, b, c) = high word of  t * (b << (32-c)) + 2^31 :
//     the per-channel 64-bit rounding term becomes one constant;
//   * the shortcut's shifts are aligned to one wave-uniform T:  (r*rb + 2^(rc-1)) >> rc = (r*(rb << (T-rc)) + 2^(T-1)) >> T.
// Conditions (else the caller takes the LDS-staged exact path with a zero-initialised accumulator): c <= 32,
// b < 2^(c-1); a T with  max rc <= T <= min(rc + 22 - bits(rb)), T <= 30  exists (|r| <= 255 keeps r*rbs + 2^(T-1) in INT32).
struct LaneParams {
    int32_t bias[16];   // start value of the accumulator
    int32_t bs[16];     // b << (32 - c)
    int32_t rbs[16];    // res_b << (T - res_c), where the register budget allows (else read from ChanRes::rbs)
    int32_t T;          // wave-uniform shift of the shortcut term
};

// Whether channel k allows the form, and its bounds for T (the lane that stages channel k calls this; the wave then
// combines: any bad -> staged form; T_lo = max, T_hi = min over its channels; T_lo <= T_hi needed).
template <bool RES>
__device__ __forceinline__ int lane_form_check(const ConvArgs &a, int k, int &T_lo, int &T_hi) {
    T_lo = 1; T_hi = 30;
    if (k >= a.K) return 0;
    const int32_t b = a.b[k], c = a.c[k];
    const int bad = (c > 32 || ((int64_t)b >> (c - 1)) != 0) ? 1 : 0;
    if (RES) {
        const int32_t rb = a.res_b[k], rc = a.res_c[k];
        const int bits = rb == 0 ? 0 : 32 - __builtin_clz((uint32_t)rb);
        T_lo = rc;
        T_hi = rc + 22 - bits < 30 ? rc + 22 - bits : 30;
    }
    return bad;
}

// The lane's 16 channels from the staged copy (pm / pr: the lane's first entries) into registers.
__device__ __forceinline__ void load_lane_params(const ChanMain *pm, const ChanRes *pr, LaneParams &p) {
#pragma unroll
    for (int i = 0; i < 16; ++i) { p.bias[i] = pm[i].bias; p.bs[i] = pm[i].bs; p.rbs[i] = pr[i].rbs; }
}

// The staged shortcut entry of channel k for shift T (call for every staged channel once T is known).
__device__ __forceinline__ void finish_res(const ConvArgs &a, int k, int T, ChanRes &r) {
    r.rbs = k < a.K ? (int32_t)((uint32_t)a.res_b[k] << ((T - a.res_c[k]) & 31)) : 0;
}

// Epilogue of one lane with register-resident parameters: TP pixels x 16 channels starting at absolute channel chg
// (a whole group: chg + 16 <= K is not required, chg < K is); acc already holds bias + the products.  8-bit or unsigned
// 4-bit outputs; shortcut bytes in pre[tp][0..3] (u8 / s8 / u4).  Stores are unconditional buffer stores (invalid pixels
// out of range), as in epilogue_tile's YMODE 2.
// pr: the lane's 16 staged shortcut entries -- with a shortcut the shifted multipliers are read from there (one dword per
// channel instead of the 32 bytes of the staged form) because the registers do not hold a third array.
// RREG: the shifted shortcut multipliers are taken from p.rbs instead.
template <int TP, bool RES, bool RREG = false>
__device__ __forceinline__ void epilogue_lane(const ConvArgs &a, const LaneParams &p, const ChanRes *pr, const int64_t (&m)[TP],
                                              const bool (&valid)[TP], int chg, const v16i (&acc)[TP][1], const uint32_t (&pre)[TP][1][4]) {
    const int y_dt = a.y_dt, res_dt = a.res_dt;
    const bool y4 = is4(y_dt);
    const __amdgpu_buffer_rsrc_t yrs = __builtin_amdgcn_make_buffer_rsrc((void *)a.y, 0, (int)tensor_bytes((int64_t)a.M * a.K, y_dt), 0x00020000);
    int32_t lo = a.lo, hi = a.hi;
    asm volatile("" : "+v"(lo), "+v"(hi));
    const bool chan_ok = chg < a.K;   // (no early exit: every lane takes part in the same store instructions)
    int64_t half = (int64_t)1 << 31;
    asm volatile("" : "+v"(half));   // opaque, in vector registers: with a known addend the compiler splits the 64-bit multiply-add into three multiplies
    int32_t y[TP][16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        // opaque copy: otherwise the sign extension of the loop-invariant multiplier is hoisted out of the caller's loop as a
        // 64-bit value (two registers per channel) and the product becomes a 64 x 32 multiply instead of one v_mad_i64_i32
        int32_t bsv = p.bs[i];
        asm volatile("" : "+v"(bsv));
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) y[tp][i] = (int32_t)(((int64_t)acc[tp][0][i] * (int64_t)bsv + half) >> 32);
    }
    if (RES) {
        const int32_t rround = (int32_t)(1u << ((p.T - 1) & 31));
        auto add_res = [&](auto kindc) {
            constexpr int kind = decltype(kindc)::value;   // 0: u8, 1: s8, 2: u4
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int32_t rbs = RREG ? p.rbs[i] : pr[i].rbs;
#pragma unroll
                for (int tp = 0; tp < TP; ++tp) {
                    int32_t r;
                    if (kind == 0) r = (int32_t)__builtin_amdgcn_ubfe(pre[tp][0][i >> 2], 8 * (i & 3), 8);
                    else if (kind == 1) r = __builtin_amdgcn_sbfe((int32_t)pre[tp][0][i >> 2], 8 * (i & 3), 8);
                    else r = (int32_t)__builtin_amdgcn_ubfe(pre[tp][0][i >> 3], 4 * (i & 7), 4);
                    y[tp][i] += (__mul24(r, rbs) + rround) >> p.T;
                }
            }
        };
        if (res_dt == HAWQ_U8) add_res(std::integral_constant<int, 0>{});
        else if (res_dt == HAWQ_S8) add_res(std::integral_constant<int, 1>{});
        else add_res(std::integral_constant<int, 2>{});
    }
#pragma unroll
    for (int tp = 0; tp < TP; ++tp) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            int32_t t;
            asm("v_med3_i32 %0, %1, %2, %3" : "=v"(t) : "v"(y[tp][i]), "v"(lo), "v"(hi));
            y[tp][i] = t;
        }
        if (y4) {
            uint32_t w0 = 0, w1 = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                w0 |= (uint32_t)y[tp][i] << (4 * i);
                w1 |= (uint32_t)y[tp][8 + i] << (4 * i);
            }
            const uint32_t off = (valid[tp] && chan_ok) ? (uint32_t)((m[tp] * (int64_t)a.K + chg) >> 1) : 0x80000000u;
            __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(v2i, make_uint2(w0, w1)), yrs, (int)off, 0, 0);
        } else {
            uint32_t w[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t t0 = __builtin_amdgcn_perm((uint32_t)y[tp][4 * q + 1], (uint32_t)y[tp][4 * q], 0x0c0c0400u);
                const uint32_t t1 = __builtin_amdgcn_perm((uint32_t)y[tp][4 * q + 3], (uint32_t)y[tp][4 * q + 2], 0x04000c0cu);
                w[q] = t0 | t1;
            }
            const uint32_t off = (valid[tp] && chan_ok) ? (uint32_t)(m[tp] * (int64_t)a.K + chg) : 0x80000000u;
            __builtin_amdgcn_raw_buffer_store_b128((v4i){(int)w[0], (int)w[1], (int)w[2], (int)w[3]}, yrs, (int)off, 0, 0);
        }
    }
}

// Epilogue of a block output with a convolution on both branches (Section 3.3's residual equation with two INT32
// accumulators), same lane layout as epilogue_tile, K % 16 == 0.  pm / ps: the two branches' staged parameters.
//   MID == false:  y = clamp( rq(accm + bias, b, c) + rq(accs + bias_s, b_s, c_s) )
//   MID == true :  the shortcut accumulator first becomes the signed 8-bit tensor a separate transition layer would have
//                  stored, sc = clamp(rq(accs + bias_s, b_s, c_s), -128, 127), and enters the sum as rq(sc, res_b, res_c)
//                  (pr: staged res_b / res_c) -- bit for bit the result of the two-launch form, without the round trip.
// The two-accumulator block output when the main branch's rescaled term is known (from the weights, on the host) to fit
// 16 bits and every parameter is in the narrow evaluation's range: the caller has already turned the finished main
// accumulators into t = rq(accm + bias, b, c) and keeps them as packed 16-bit pairs (t16[.][8 (tp*TC+tc) + i/2], low half
// first), which frees half the registers of a second accumulator set.  y = clamp(t + rq(accs + bias_s, b_s, c_s)); MID: the
// stored-shortcut arithmetic, y = clamp(t + rq(clamp(rq(accs + bias_s, b_s, c_s), -128, 127), res_b, res_c)).
template <int TC, int TP, bool MID = false>
__device__ __forceinline__ void epilogue_tile_dual16(const ConvArgs &a, const ChanMain *ps, const ChanRes *pr, const int64_t (&m)[TP],
                                                     const bool (&valid)[TP], int k0, int chl,
                                                     const uint32_t (&t16)[TP * TC * 8], const v16i (&accs)[TP][TC]) {
    const bool y4 = is4(a.y_dt);
    int32_t lo = a.lo, hi = a.hi, m128 = -128, p127 = 127;
    asm volatile("" : "+v"(lo), "+v"(hi), "+v"(m128), "+v"(p127));
    static_for<0, TC>([&](auto gc) {
        constexpr int g = decltype(gc)::value;
        const int chg = k0 + chl + 16 * g;
        if (chg >= a.K) return;
        int32_t y[TP][16];
        static_for<0, 16>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            const ChanMain &p2 = ps[chl + 16 * g + i];
            const int32_t bs2 = p2.bs;
            const int64_t Rs2 = p2.Rs;
            ChanRes p3 = ChanRes{0, 1, 1, 0};
            if (MID) p3 = pr[chl + 16 * g + i];
#pragma unroll
            for (int tp = 0; tp < TP; ++tp) {
                const uint32_t w = t16[8 * (tp * TC + g) + i / 2];
                const int32_t t = (i & 1) ? ((int32_t)w >> 16) : (int32_t)(int16_t)(w & 0xffffu);
                int32_t sc = (int32_t)(((int64_t)accs[tp][g][i] * (int64_t)bs2 + Rs2) >> 32);
                if (MID) {
                    int32_t s8;
                    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(s8) : "v"(sc), "v"(m128), "v"(p127));
                    sc = (__mul24(s8, p3.rb) + p3.rround) >> p3.rc;
                }
                const int32_t v = t + sc;
                int32_t r;
                asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
                y[tp][i] = r;
            }
        });
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) {
            if (!valid[tp]) continue;
            if (y4) {
                uint32_t w0 = 0, w1 = 0;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    w0 |= (uint32_t)y[tp][i] << (4 * i);
                    w1 |= (uint32_t)y[tp][8 + i] << (4 * i);
                }
                *(uint2 *)(a.y + ((m[tp] * (int64_t)a.K + chg) >> 1)) = make_uint2(w0, w1);
            } else {
                uint32_t w[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t t0 = __builtin_amdgcn_perm((uint32_t)y[tp][4 * q + 1], (uint32_t)y[tp][4 * q], 0x0c0c0400u);
                    const uint32_t t1 = __builtin_amdgcn_perm((uint32_t)y[tp][4 * q + 3], (uint32_t)y[tp][4 * q + 2], 0x04000c0cu);
                    w[q] = t0 | t1;
                }
                *(uint4 *)(a.y + (m[tp] * (int64_t)a.K + chg)) = make_uint4(w[0], w[1], w[2], w[3]);
            }
        }
    });
}

// YMODE 0: plain global stores of the valid pixels; 2: every lane issues a buffer store (invalid pixels out of range).
template <int TC, int TP, int YMODE = 0, bool MID = false>
__device__ __forceinline__ void epilogue_tile_dual(const ConvArgs &a, const ChanMain *pm, const ChanMain *ps, const ChanRes *pr,
                                                   const int64_t (&m)[TP], const bool (&valid)[TP], int k0, int chl,
                                                   const v16i (&accm)[TP][TC], const v16i (&accs)[TP][TC], int wide) {
    const int y_dt = a.y_dt;
    const bool y4 = is4(y_dt);
    int32_t lo = a.lo, hi = a.hi;
    const __amdgpu_buffer_rsrc_t yrs = __builtin_amdgcn_make_buffer_rsrc(
        (void *)a.y, 0, YMODE == 2 ? (int)tensor_bytes((int64_t)a.M * a.K, y_dt) : 0, 0x00020000);
    if (wide || y_dt == HAWQ_S4) {
        // exact general form: 64-bit products, shifts and clamp
        static_for<0, TC>([&](auto gc) {
            constexpr int g = decltype(gc)::value;
            const int chg = k0 + chl + 16 * g;
            if (chg >= a.K) return;
            static_for<0, TP>([&](auto tpc) {
                constexpr int tp = decltype(tpc)::value;
                if (!valid[tp]) return;
                const int64_t o = m[tp] * (int64_t)a.K + chg;
                uint32_t ow[4] = {0, 0, 0, 0};
                static_for<0, 16>([&](auto ic) {
                    constexpr int i = decltype(ic)::value;
                    const ChanMain p1 = pm[chl + 16 * g + i], p2 = ps[chl + 16 * g + i];
                    int32_t av = accm[tp][g][i], sv = accs[tp][g][i];
                    asm volatile("" : "+v"(av), "+v"(sv));   // keeps this cold path's products apart from the narrow path's
                    int64_t sc = ((int64_t)sv * (int64_t)p2.b + p2.R) >> p2.c;
                    if (MID) {
                        const ChanRes p3 = pr[chl + 16 * g + i];
                        sc = rq64(clamp64(sc, -128, 127), p3.rb, p3.rc);
                    }
                    const int64_t w64 = (((int64_t)av * (int64_t)p1.b + p1.R) >> p1.c) + sc;
                    const int32_t y = clamp64(w64, lo, hi);
                    if (y4) ow[i >> 3] |= (uint32_t)(y & 0xf) << (4 * (i & 7));
                    else ow[i >> 2] |= (uint32_t)(y & 0xff) << (8 * (i & 3));
                });
                if (y4) *(uint2 *)(a.y + (o >> 1)) = make_uint2(ow[0], ow[1]);
                else *(uint4 *)(a.y + o) = make_uint4(ow[0], ow[1], ow[2], ow[3]);
            });
        });
        return;
    }
    int32_t m128 = -128, p127 = 127;
    asm volatile("" : "+v"(lo), "+v"(hi), "+v"(m128), "+v"(p127));
    static_for<0, TC>([&](auto gc) {
        constexpr int g = decltype(gc)::value;
        const int chg = k0 + chl + 16 * g;
        if (chg >= a.K) return;
        int32_t y[TP][16];
        static_for<0, 16>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            const ChanMain &p1 = pm[chl + 16 * g + i];
            const ChanMain &p2 = ps[chl + 16 * g + i];
            const int32_t bs1 = p1.bs, bs2 = p2.bs;
            const int64_t Rs1 = p1.Rs, Rs2 = p2.Rs;
            ChanRes p3 = ChanRes{0, 1, 1, 0};
            if (MID) p3 = pr[chl + 16 * g + i];
#pragma unroll
            for (int tp = 0; tp < TP; ++tp) {
                int32_t sc = (int32_t)(((int64_t)accs[tp][g][i] * (int64_t)bs2 + Rs2) >> 32);
                if (MID) {
                    int32_t s8;
                    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(s8) : "v"(sc), "v"(m128), "v"(p127));
                    sc = (__mul24(s8, p3.rb) + p3.rround) >> p3.rc;
                }
                const int32_t v = (int32_t)(((int64_t)accm[tp][g][i] * (int64_t)bs1 + Rs1) >> 32) + sc;
                int32_t t;
                asm("v_med3_i32 %0, %1, %2, %3" : "=v"(t) : "v"(v), "v"(lo), "v"(hi));
                y[tp][i] = t;
            }
        });
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) {
            if (y4) {
                uint32_t w0 = 0, w1 = 0;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    w0 |= (uint32_t)y[tp][i] << (4 * i);
                    w1 |= (uint32_t)y[tp][8 + i] << (4 * i);
                }
                if (YMODE == 2) {
                    const uint32_t off = valid[tp] ? (uint32_t)((m[tp] * (int64_t)a.K + chg) >> 1) : 0x80000000u;
                    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(v2i, make_uint2(w0, w1)), yrs, (int)off, 0, 0);
                } else if (valid[tp]) {
                    *(uint2 *)(a.y + ((m[tp] * (int64_t)a.K + chg) >> 1)) = make_uint2(w0, w1);
                }
            } else {
                uint32_t w[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t t0 = __builtin_amdgcn_perm((uint32_t)y[tp][4 * q + 1], (uint32_t)y[tp][4 * q], 0x0c0c0400u);
                    const uint32_t t1 = __builtin_amdgcn_perm((uint32_t)y[tp][4 * q + 3], (uint32_t)y[tp][4 * q + 2], 0x04000c0cu);
                    w[q] = t0 | t1;
                }
                if (YMODE == 2) {
                    const uint32_t off = valid[tp] ? (uint32_t)(m[tp] * (int64_t)a.K + chg) : 0x80000000u;
                    __builtin_amdgcn_raw_buffer_store_b128((v4i){(int)w[0], (int)w[1], (int)w[2], (int)w[3]}, yrs, (int)off, 0, 0);
                } else if (valid[tp]) {
                    *(uint4 *)(a.y + (m[tp] * (int64_t)a.K + chg)) = make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
        }
    });
}

}  // namespace hawq
