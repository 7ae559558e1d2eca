// 1x1 / stride 1 / unpadded quantised convolution with the pixel operand resident in LDS -- the layer that closes a
// bottleneck block (Section 3.3: requantise + rescaled shortcut) or opens one, and the block output with a convolution on
// both branches (Figure 2, Section 3.3's residual equation with two INT32 accumulators) in one launch.
//
// Same division of labour as the 3x3 kernel of conv_rp.hip (Section 3.1's integer convolution as  D[k][m] = sum_c W[k][c] X[m][c]):
//   * Pixels.  A workgroup owns a tile of 32 TP consecutive output pixels and keeps every input channel of them in LDS
//     (rows of C + 16 bytes, so that the sixteen lanes of a 128-bit LDS access fall into different banks) -- fetched once,
//     read by all eight waves, for every pass.
//   * Weights.  The eight waves split the output channels, 32 each (one MFMA row tile x TP column tiles), and stream
//     their weight fragments from the fragment-ordered copy (launch_fragment_weights) straight from global memory into
//     registers, four K-steps ahead; no barrier in the K loop.
//   * Passes.  A workgroup walks `npass` groups of 256 output channels over its resident pixels: few pixels with many
//     channels (7x7 and 14x14 images) then fill the chip with one round of workgroups, and the activations are fetched
//     once per npass * 256 channels.
//   * Two convolutions (DUAL): the shortcut convolution's pixels -- the strided samples of the block input -- sit in a
//     second LDS patch.  A pass first runs the main branch's K-steps, rescales the finished accumulators at once to
//     16-bit values (the caller guarantees from the weights that they fit), then runs the shortcut branch's K-steps into
//     the same accumulators; the epilogue rescales those and adds.  The weight stream runs through both without a gap.
#include "rp.h"

namespace hawq {

// narrow evaluation of rq(acc + bias, b, c): high word of acc * bs + Rs (see RpChan)
struct Rp1Narrow { int64_t Rs; int32_t bs; int32_t pad; };

// Epilogue of one lane of the two-convolution form: NT (1 or 2) pixels x 16 consecutive channels.  t16: the main
// branch's rescaled terms as packed 16-bit pairs (element i in half i & 1 of word i / 2).  acc: the shortcut
// convolution's accumulators.  MID: the shortcut term is first rounded and clamped to the signed 8-bit value a separate
// transition layer would store and enters the sum rescaled by (rb, rc); otherwise the rescaled accumulator enters directly.
template <int NT, bool MID>
__device__ __forceinline__ void rp1_epilogue_dual(const v16i &acc0, const v16i &acc1, const uint32_t (&t0)[8], const uint32_t (&t1)[8],
                                                  const Rp1Narrow *ps, const RpRes *pr, const int lo_, const int hi_,
                                                  uint32_t (&out)[2][4]) {
    int32_t lo = lo_, hi = hi_, m128 = -128, p127 = 127;
    asm volatile("" : "+v"(lo), "+v"(hi), "+v"(m128), "+v"(p127));
    int32_t y[2][16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int32_t bs = ps[i].bs;
        const int64_t Rs = ps[i].Rs;
        RpRes q = RpRes{0, 1};
        if (MID) q = pr[i];
        const int32_t rr = (int32_t)(1u << ((q.rc - 1) & 31));
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const uint32_t w = t == 0 ? t0[i / 2] : t1[i / 2];
            const int32_t m = (i & 1) ? ((int32_t)w >> 16) : (int32_t)(int16_t)(w & 0xffffu);
            int32_t sc = (int32_t)(((int64_t)(t == 0 ? acc0[i] : acc1[i]) * (int64_t)bs + Rs) >> 32);
            if (MID) {
                int32_t s8;
                asm("v_med3_i32 %0, %1, %2, %3" : "=v"(s8) : "v"(sc), "v"(m128), "v"(p127));
                sc = (__mul24(s8, q.rb) + rr) >> q.rc;
            }
            const int32_t v = m + sc;
            int32_t r;
            asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
            y[t][i] = r;
        }
    }
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int q = 0; q < 4; ++q) {   // low bytes of 4 values -> one dword
            const uint32_t u0 = __builtin_amdgcn_perm((uint32_t)y[t][4 * q + 1], (uint32_t)y[t][4 * q], 0x0c0c0400u);
            const uint32_t u1 = __builtin_amdgcn_perm((uint32_t)y[t][4 * q + 3], (uint32_t)y[t][4 * q + 2], 0x04000c0cu);
            out[t][q] = u0 | u1;
        }
    if (NT == 1) out[1][0] = out[1][1] = out[1][2] = out[1][3] = 0;
}

// CCH / CCS: input channels / 64 of the main / the shortcut convolution (CCS = 0: one convolution, optional shortcut
// tensor).  TP: MFMA column tiles (of 32 pixels) per wave = per workgroup.  NPMAX: passes the static parameter arrays hold.
template <int CCH, int CCS, int TP, int NPMAX>
__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
conv_rp1_kernel(const Rp1Args a) {
    constexpr bool DUAL = CCS > 0;
    constexpr int T = 512;
    constexpr int BP = 32 * TP;                      // pixels per tile
    constexpr int C = 64 * CCH, CS = 64 * CCS;
    constexpr int PITCH = C + 16, PITCHS = CS + 16;  // bytes per LDS row
    constexpr int S1 = CCH, S2 = CCS, SS = S1 + S2;  // K-steps of a pass: main branch, then shortcut branch
    constexpr int KW = 256 * NPMAX;                  // channels of a workgroup at most
    constexpr int D = 4;                             // K-steps the weight fragments are requested ahead
    static_assert(SS % D == 0 && SS >= D, "the weight ring keeps its phase from pass to pass");
    __shared__ __attribute__((aligned(16))) uint8_t patch[BP * PITCH];
    __shared__ __attribute__((aligned(16))) uint8_t patchs[DUAL ? BP * PITCHS : 16];
    __shared__ RpChan par[DUAL ? 1 : KW];
    __shared__ Rp1Narrow parm[DUAL ? KW : 1];
    __shared__ Rp1Narrow pars[DUAL ? KW : 1];
    __shared__ RpRes pres[KW];
    __shared__ uint32_t xo[DUAL ? BP : 1];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rho = lane & 31, khalf = lane >> 5;
    const int npass = a.npass;
    const int kw = npass * 256;                              // channels of this workgroup
    const int ncg = a.K / kw;                                // channel groups (workgroups per tile)
    const uint32_t L = xcd_remap(blockIdx.x, gridDim.x);
    const int tile_i = (int)(L / (uint32_t)ncg), cg = (int)(L % (uint32_t)ncg);
    const int m0 = tile_i * BP;
    const int kbase = cg * kw;
    const bool has_res = !DUAL && a.res != nullptr;
    const bool mid = DUAL && a.mid_s8 != 0;

    // ---- prologue: every global load of it is issued before the first one is waited for ----
    if constexpr (DUAL) {
        // byte offset of each tile pixel's shortcut-branch sample: output pixel (n, p, q) reads (n, p sh, q sw)
        if (tid < BP) {
            const int64_t m = (int64_t)m0 + tid;
            uint32_t o = 0x80000000u;   // no such pixel: out of range, zeros
            if (m < a.M) {
                const int n = (int)(m / a.PQ), rem = (int)(m % a.PQ);
                const int pp = rem / a.Q, qq = rem - pp * a.Q;
                o = (uint32_t)((((int64_t)n * a.Hs + (int64_t)pp * a.sh) * a.Ws + (int64_t)qq * a.sw) * CS);
            }
            xo[tid] = o;
        }
    }
    constexpr int CPR = C / 16;                      // 16-byte chunks per pixel
    constexpr int NIT = BP * CPR / T;
    static_assert(BP * CPR % T == 0, "whole rounds of patch loads");
    v4i pv[NIT];
    {
        const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, (int)((int64_t)a.M * C), 0x00020000);
        const int64_t src0 = (int64_t)m0 * C;        // the tile's pixels are one contiguous range; past the tensor: zeros
#pragma unroll
        for (int j = 0; j < NIT; ++j) {
            const int64_t o = src0 + (int64_t)(tid + j * T) * 16;
            pv[j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, (int)(o < (int64_t)0x7fffffff ? (uint32_t)o : 0x80000000u), 0, 0);
        }
    }
    // weight streams of this wave: channel group (kbase + pass * 256) / 32 + wave of each branch, K-steps in order
    const int G = a.K / 32;
    const __amdgpu_buffer_rsrc_t rsrc_w1 = __builtin_amdgcn_make_buffer_rsrc((void *)a.wf, 0, (int)((int64_t)G * S1 * 2048), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_w2 = __builtin_amdgcn_make_buffer_rsrc((void *)(DUAL ? a.wsf : a.wf), 0, DUAL ? (int)((int64_t)G * S2 * 2048) : 0, 0x00020000);
    const int lane16 = lane * 16;
    const int g0 = __builtin_amdgcn_readfirstlane(kbase / 32 + wave);   // channel group of pass 0
    v4i af[D][2];
    // fragments of unified K-step u (0 .. SS - 1: main branch first) of the pass whose channel group is g
    auto load_w = [&](auto uc, int g, v4i (&dst)[2]) {
        constexpr int u = decltype(uc)::value;
        if constexpr (u < S1) {
            const int o = (g * S1 + u) * 2048;
            dst[0] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w1, lane16, o, 0);
            dst[1] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w1, lane16, o + 1024, 0);
        } else {
            const int o = (g * S2 + (u - S1)) * 2048;
            dst[0] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w2, lane16, o, 0);
            dst[1] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w2, lane16, o + 1024, 0);
        }
    };
    static_for<0, D>([&](auto dc) { load_w(dc, g0, af[decltype(dc)::value]); });
    // per-channel parameters: thread i stages channels i, i + 512 of the workgroup's range
    constexpr int NPT = (KW + T - 1) / T;
    int32_t qb[NPT], qc[NPT], qbias[NPT], qrb[NPT], qrc[NPT], qbs[NPT], qcs[NPT], qbiass[NPT];
#pragma unroll
    for (int j = 0; j < NPT; ++j) {
        const int k = tid + j * T;
        const bool ok = k < kw;
        qb[j] = ok ? a.b[kbase + k] : 0; qc[j] = ok ? a.c[kbase + k] : 1; qbias[j] = ok ? a.bias[kbase + k] : 0;
        qrb[j] = 0; qrc[j] = 1; qbs[j] = 0; qcs[j] = 1; qbiass[j] = 0;
        if ((has_res || mid) && ok) { qrb[j] = a.res_b[kbase + k]; qrc[j] = a.res_c[kbase + k]; }
        if (DUAL && ok) { qbs[j] = a.b_s[kbase + k]; qcs[j] = a.c_s[kbase + k]; qbiass[j] = a.bias_s[kbase + k]; }
    }
    constexpr int CPRS = DUAL ? CS / 16 : 1;
    constexpr int NITS = DUAL ? BP * CPRS / T : 1;
    v4i pvs[NITS];
    if constexpr (DUAL) {
        __syncthreads();   // the sample offsets are in LDS
        const __amdgpu_buffer_rsrc_t rsrc_xs = __builtin_amdgcn_make_buffer_rsrc((void *)a.xs, 0, (int)a.xs_bytes, 0x00020000);
#pragma unroll
        for (int j = 0; j < NITS; ++j) {
            const int i = tid + j * T;
            const uint32_t o = xo[i / CPRS];
            pvs[j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_xs, (int)(o == 0x80000000u ? o : o + (uint32_t)(i % CPRS) * 16), 0, 0);
        }
    }

    // ---- the lane's pixels ----
    int base[TP], bases[TP];
    uint32_t yoff[TP];   // byte offset of the pixel's first channel in the output tensor (out of range: no such pixel)
#pragma unroll
    for (int tp = 0; tp < TP; ++tp) {
        const int p = tp * 32 + rho;
        const int64_t m = (int64_t)m0 + p;
        yoff[tp] = m < a.M ? (uint32_t)(m * a.K) : 0x80000000u;
        base[tp] = p * PITCH + khalf * 16;
        bases[tp] = p * PITCHS + khalf * 16;
    }

    // ---- LDS: patches, parameters ----
#pragma unroll
    for (int j = 0; j < NIT; ++j) {
        const int i = tid + j * T;
        *(v4i *)(patch + (i / CPR) * PITCH + (i % CPR) * 16) = pv[j];
    }
    int wide = 0;
    auto stage = [&](int32_t bias, int32_t b, int32_t c, RpChan &o) {
        o.b = b; o.c = c; o.bias = bias; o.bs = 0; o.Rs = 0;
        if (c > 32 || ((int64_t)b >> (c - 1)) != 0) { wide = 1; return; }
        const int64_t R = (int64_t)bias * (int64_t)b + ((int64_t)1 << (c - 1));
        o.bs = (int32_t)((uint32_t)b << (32 - c));
        o.Rs = (int64_t)((uint64_t)R << (32 - c));
    };
#pragma unroll
    for (int j = 0; j < NPT; ++j) {
        const int k = tid + j * T;
        if (k < kw) {
            RpChan p;
            stage(qbias[j], qb[j], qc[j], p);
            if constexpr (DUAL) {
                // (the caller vouches for the narrow range of both branches' parameters: `wide` is not consulted)
                parm[k] = Rp1Narrow{p.Rs, p.bs, 0};
                stage(qbiass[j], qbs[j], qcs[j], p);
                pars[k] = Rp1Narrow{p.Rs, p.bs, 0};
                pres[k] = RpRes{qrb[j], qrc[j]};
            } else {
                par[k] = p;
                if (has_res) {
                    if (qrc[j] > 31 || qrb[j] >= (1 << 22)) wide = 1;
                    pres[k] = RpRes{qrb[j], qrc[j]};
                }
            }
        }
    }
    if constexpr (DUAL) {
#pragma unroll
        for (int j = 0; j < NITS; ++j) {
            const int i = tid + j * T;
            *(v4i *)(patchs + (i / CPRS) * PITCHS + (i % CPRS) * 16) = pvs[j];
        }
    }
    wide = __syncthreads_or(wide);   // patches and parameters are in LDS

    v16i acc[TP];
    v4i bf[2][TP];   // pixel fragments: [buffer][pixel tile], one half K-step (32 reduction elements) each
    uint32_t t16[DUAL ? TP : 1][8];
    auto mfma_row = [&](auto bufc, const v4i &aw) {
        constexpr int buf = decltype(bufc)::value;
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) acc[tp] = __builtin_amdgcn_mfma_i32_32x32x32_i8(aw, bf[buf][tp], acc[tp], 0, 0, 0);
    };
    const __amdgpu_buffer_rsrc_t rsrc_y = __builtin_amdgcn_make_buffer_rsrc((void *)a.y, 0, (int)((int64_t)a.M * a.K), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_r = __builtin_amdgcn_make_buffer_rsrc((void *)(has_res ? a.res : a.x), 0, has_res ? (int)((int64_t)a.M * a.K) : 0, 0x00020000);
    const bool res_signed = a.res_dt == HAWQ_S8;
    // The lane's shortcut bytes are requested a whole pass ahead of their use: two buffers where there is more than one pass.
    constexpr int RB = (!DUAL && NPMAX > 1) ? 2 : 1;
    uint32_t resw[RB][TP + 1][4] = {};   // (one spare row: the last epilogue call of an odd TP reads a pair)
    auto load_res = [&](auto bc, int ch) {   // 16 shortcut bytes of each of the lane's pixels, channels ch .. ch + 15
        constexpr int rb = decltype(bc)::value;
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) {
            const v4i t = __builtin_amdgcn_raw_buffer_load_b128(rsrc_r, (int)(yoff[tp] + (uint32_t)ch), 0, 0);
            resw[rb][tp][0] = (uint32_t)t[0]; resw[rb][tp][1] = (uint32_t)t[1]; resw[rb][tp][2] = (uint32_t)t[2]; resw[rb][tp][3] = (uint32_t)t[3];
        }
    };
    using R0 = std::integral_constant<int, 0>;
    const int chl0 = wave * 32 + khalf * 16;   // the lane's first channel of pass 0 within the workgroup's range
    if (has_res) load_res(R0{}, kbase + chl0);
    // With several passes a wave alternates a burst of MFMAs with a long integer epilogue.  Waves w and w + 4 share a SIMD
    // and leave the barrier together; delaying one of them by about half a burst makes its MFMAs fall into the other's
    // epilogue instead of both queueing for the matrix pipe and then for the vector ALU.
    if (NPMAX > 1 && npass > 1 && wave >= 4) __builtin_amdgcn_s_sleep(TP * SS * 2 * 32 / 64 / 2);

    auto one_pass = [&](auto bc, int pass) {
        constexpr int rb = decltype(bc)::value;
        const int gnext = g0 + (pass + 1) * 8;
        const bool more = pass + 1 < npass;
        const int chl = pass * 256 + chl0;
        if (RB == 2 && has_res && more) load_res(std::integral_constant<int, (rb + 1) % RB>{}, kbase + chl + 256);
#pragma unroll
        for (int tp = 0; tp < TP; ++tp)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[tp][i] = 0;
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) bf[0][tp] = *(const v4i *)(patch + base[tp]);
        // Half-step h (32 reduction elements) = K-step h / 2, half h % 2.  While half-step h is multiplied, the pixel
        // fragments of half-step h + 1 are read into the other buffer; the weight fragments of K-step t + D (of this pass or
        // the next) are requested as soon as K-step t has issued.
        static_for<0, 2 * SS>([&](auto hc) {
            constexpr int h = decltype(hc)::value;
            constexpr int t = h / 2, kk = h % 2;
            constexpr int hn = h + 1, tn = hn / 2, kn = hn % 2;
            if constexpr (hn < 2 * SS) {
#pragma unroll
                for (int tp = 0; tp < TP; ++tp) {
                    if constexpr (tn < S1) bf[hn % 2][tp] = *(const v4i *)(patch + base[tp] + tn * 64 + kn * 32);
                    else bf[hn % 2][tp] = *(const v4i *)(patchs + bases[tp] + (tn - S1) * 64 + kn * 32);
                }
            }
            if constexpr (DUAL && h == 2 * S1) {
                // the main branch is complete: rescale it to packed 16-bit terms, start the shortcut branch from zero
                const Rp1Narrow *pm = parm + chl;
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    const int32_t bs0 = pm[i].bs, bs1 = pm[i + 1].bs;
                    const int64_t Rs0 = pm[i].Rs, Rs1 = pm[i + 1].Rs;
#pragma unroll
                    for (int tp = 0; tp < TP; ++tp) {
                        const int32_t v0 = (int32_t)(((int64_t)acc[tp][i] * (int64_t)bs0 + Rs0) >> 32);
                        const int32_t v1 = (int32_t)(((int64_t)acc[tp][i + 1] * (int64_t)bs1 + Rs1) >> 32);
                        t16[tp][i / 2] = __builtin_amdgcn_perm((uint32_t)v1, (uint32_t)v0, 0x05040100u);
                    }
                }
#pragma unroll
                for (int tp = 0; tp < TP; ++tp)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[tp][i] = 0;
            }
            mfma_row(std::integral_constant<int, h % 2>{}, af[t % D][kk]);
            if constexpr (kk == 1) {
                if constexpr (t + D < SS) load_w(std::integral_constant<int, t + D>{}, g0 + pass * 8, af[t % D]);
                else if (more) load_w(std::integral_constant<int, t + D - SS>{}, gnext, af[t % D]);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        // epilogue of all the lane's pixels, two at a time
        const int ch = kbase + chl;
        static_for<0, (TP + 1) / 2>([&](auto jc) {
            constexpr int t0 = 2 * decltype(jc)::value;
            constexpr int nt = t0 + 1 < TP ? 2 : 1;
            constexpr int t1 = nt == 2 ? t0 + 1 : t0;
            uint32_t o[2][4];
            if constexpr (DUAL) {
                if (mid) rp1_epilogue_dual<nt, true>(acc[t0], acc[t1], t16[t0], t16[t1], pars + chl, pres + chl, a.lo, a.hi, o);
                else rp1_epilogue_dual<nt, false>(acc[t0], acc[t1], t16[t0], t16[t1], pars + chl, pres + chl, a.lo, a.hi, o);
            } else {
                const uint32_t rw[2][4] = {{resw[rb][t0][0], resw[rb][t0][1], resw[rb][t0][2], resw[rb][t0][3]},
                                           {resw[rb][t0 + 1][0], resw[rb][t0 + 1][1], resw[rb][t0 + 1][2], resw[rb][t0 + 1][3]}};
                rp_epilogue<nt>(acc[t0], acc[t1], par + chl, pres + chl, has_res, res_signed, rw, wide, a.lo, a.hi, o);
            }
            __builtin_amdgcn_raw_buffer_store_b128((v4i){(int)o[0][0], (int)o[0][1], (int)o[0][2], (int)o[0][3]}, rsrc_y, (int)(yoff[t0] + (uint32_t)ch), 0, 0);
            if constexpr (nt == 2)
                __builtin_amdgcn_raw_buffer_store_b128((v4i){(int)o[1][0], (int)o[1][1], (int)o[1][2], (int)o[1][3]}, rsrc_y, (int)(yoff[t1] + (uint32_t)ch), 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        });
        if (RB == 1 && has_res && more) load_res(R0{}, ch + 256);
    };
    for (int pass = 0; pass < npass; pass += 2) {
        one_pass(R0{}, pass);
        if (pass + 1 < npass) one_pass(std::integral_constant<int, 1 % RB>{}, pass + 1);
    }
}

// ---- host side ----

// Which instantiation serves the request; 0 = none.
//   1: C = 256 + shortcut convolution over 512 channels (block output of the 14 x 14 stage), tiles of 128 pixels
//   2: C = 512 + shortcut convolution over 1024 channels (7 x 7 stage), tiles of 64 pixels (the two patches fill LDS)
//   3: C = 512, one convolution (7 x 7 stage's closing layer), tiles of 128 pixels
//   4: C = 1024, one convolution (14 x 14 stage's opening layer), tiles of 128 pixels, one pass
//   5: C = 2048, one convolution (7 x 7 stage's opening layer), tiles of 64 pixels, one pass
static int rp1_variant(const Rp1Args &a) {
    if (a.M <= 0 || a.K <= 0 || a.K % 256 != 0) return 0;
    if (a.xs != nullptr) {
        if (a.C == 256 && a.Cs == 512) return 1;
        if (a.C == 512 && a.Cs == 1024) return 2;
        return 0;
    }
    if (a.C == 512) return 3;
    if (a.C == 1024) return 4;
    if (a.C == 2048) return 5;
    return 0;
}

// A workgroup of this kernel takes a compute unit to itself (LDS and registers), also while it waits for its pixels.
// Alone on the chip that costs nothing, and the kernel beats the tiled ones on every shape above (ResNet50 at batch 128
// on one stream: 37 -> 29 us for the 14 x 14 block output, 16 -> 12.5 us for the 7 x 7 opening layer, 1.135 -> 1.094 ms
// per forward).  When the forward runs as two half-batches on two streams, the tiled kernels' smaller workgroups
// interleave with the other stream's better: measured per variant, the kernel then pays only with full-size parts (two
// parts of 128 images: +1.3 % together) and never for the 7 x 7 closing layer.
bool conv_rp1_shape_ok(const Rp1Args &a) {
    const int v = rp1_variant(a);
    if (v == 0) return false;
    if (!a.corun) return true;
    if (v == 3) return false;
    const int bp = (v == 2 || v == 5) ? 64 : 128;
    return ((int64_t)a.M + bp - 1) / bp >= (bp == 64 ? 75 : 150);
}

hawq_status launch_conv_rp1(const Rp1Args &a0, hipStream_t s) {
    const int v = rp1_variant(a0);
    if (v == 0) return HAWQ_ERR_UNSUPPORTED;
    Rp1Args a = a0;
    const int bp = (v == 2 || v == 5) ? 64 : 128;
    const int npmax = v >= 4 ? 1 : 4;
    const uint32_t tiles = (uint32_t)(((int64_t)a.M + bp - 1) / bp);
    // channel groups per tile: as few as fill the chip in one round of workgroups (counting the twin launch of the other
    // half-batch when the forward runs as two parts) -- every group fetches the tile's pixels again
    const int g256 = a.K / 256;
    const uint32_t want = a.corun ? 80 : 160;
    int ncg = g256;   // (no smaller choice fills the chip: one pass per workgroup, the most workgroups)
    for (int d = 1; d < g256; ++d)
        if (g256 % d == 0 && g256 / d <= npmax && tiles * (uint32_t)d >= want) { ncg = d; break; }
    a.npass = g256 / ncg;
    const uint32_t grid = tiles * (uint32_t)ncg;
    switch (v) {
    case 1: conv_rp1_kernel<4, 8, 4, 4><<<grid, 512, 0, s>>>(a); break;
    case 2: conv_rp1_kernel<8, 16, 2, 4><<<grid, 512, 0, s>>>(a); break;
    case 3: conv_rp1_kernel<8, 0, 4, 4><<<grid, 512, 0, s>>>(a); break;
    case 4: conv_rp1_kernel<16, 0, 4, 1><<<grid, 512, 0, s>>>(a); break;
    default: conv_rp1_kernel<32, 0, 2, 1><<<grid, 512, 0, s>>>(a); break;
    }
    return check_launch();
}

}  // namespace hawq
