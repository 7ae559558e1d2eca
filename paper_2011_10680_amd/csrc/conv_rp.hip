// 3x3 / stride 1 / pad 1 quantised convolution with the pixel operand resident in LDS, optionally followed -- in the same
// launch, on the same pixels -- by the 1x1 convolution that ends a bottleneck block and adds the shortcut (Figure 2,
// Section 3.3: conv -> requantise -> conv -> requantise + rescaled shortcut; the tensor between the two convolutions
// never leaves the compute unit).
//
// Section 3.1's integer convolution as an implicit GEMM  D[k][m] = sum_kg Wt[k][kg] X[m][kg]  (k output channel, m output
// pixel, kg = (r, s, c)), arranged around what is scarce on a gfx950 compute unit:
//   * Pixels.  With stride 1 and pad 1 the input pixel of output pixel m under tap (r, s) is flat pixel
//     m + (r-1) W + (s-1) of the NHWC tensor, so the nine pixel operands of a tile of BP consecutive output pixels are nine
//     shifted windows of ONE run of BP + 2W + 2 input pixels.  That run ("patch") is fetched once per tile into LDS, every
//     channel of it, in rows of C + 16 bytes (the 16 bytes of padding put the sixteen lanes of a 128-bit LDS access, which
//     hold sixteen consecutive pixels, into different banks).  Taps that fall into the zero padding (or across an image
//     boundary) are redirected, per lane, to a row of zeros.
//   * Weights.  A wave owns 32 output channels x 128 pixels (one MFMA row tile, four column tiles): its weight fragment of a
//     K-step is 2 KB and no other wave of the workgroup needs it.  The weights are therefore read from a copy laid out in
//     MFMA fragment order ([channel group of 32][K-step][half][lane][16 bytes], made once per layer), straight from global
//     memory into registers with fully coalesced 1 KB loads, three K-steps ahead.  Nothing is written to LDS in the K loop,
//     so the loop needs no barrier: waves run decoupled and hide each other's waits.
//   * The fused second convolution takes the requantised tile of the first one (written to LDS by its epilogue, same row
//     layout) as its pixel operand; its weights stream the same way.
// INT32 accumulators never leave the register file; the epilogue is bias, dyadic requantisation, rescaled shortcut, clamp,
// pack, 16-byte NHWC stores, with the per-channel parameters staged once per workgroup in LDS.
#include "common.h"

namespace hawq {

// Per-channel parameters as staged in LDS.  narrow evaluation (c <= 32, b < 2^(c-1)):  rq(acc + bias, b, c) = high word of
// acc * bs + Rs  with bs = b << (32-c), Rs = (bias*b + 2^(c-1)) << (32-c); any other channel makes the whole workgroup
// take the exact 64-bit evaluation from (bias, b, c).
struct RpChan { int32_t bs, b, c, bias; int64_t Rs; };
struct RpRes { int32_t rb, rc; };

__device__ __forceinline__ int rp_stage_chan(const int32_t *bias, const int32_t *b, const uint8_t *c, int k, RpChan &o) {
    o.b = b[k]; o.c = c[k]; o.bias = bias[k];
    o.bs = 0; o.Rs = 0;
    if (o.c > 32 || ((int64_t)o.b >> (o.c - 1)) != 0) return 1;
    const int64_t R = (int64_t)o.bias * (int64_t)o.b + ((int64_t)1 << (o.c - 1));
    o.bs = (int32_t)((uint32_t)o.b << (32 - o.c));
    o.Rs = (int64_t)((uint64_t)R << (32 - o.c));
    return 0;
}

// Epilogue of one lane: pixels T0, T0 + 1 of its four (MFMA column tiles) x 16 consecutive channels.  pc / pr: the lane's
// first channel's entries.  resw[tp]: the 16 shortcut bytes of pixel tp (only read when has_res).  Result: out[tp] = the
// 16 output bytes.  (Two pixels per call: a channel's parameters are read once for both, and the intermediate values of
// all four pixels at once would not fit the register budget next to the accumulators and the prefetched weights.)
template <int T0>
__device__ __forceinline__ void rp_epilogue(const v16i (&acc)[4], const RpChan *pc, const RpRes *pr, const bool has_res,
                                            const bool res_signed, const uint32_t (&resw)[4][4], const int wide, const int lo_,
                                            const int hi_, uint32_t (&out)[4][4]) {
    if (wide) {   // exact general form: 64-bit products, shifts and clamp
        const uint32_t sgn = res_signed ? 0x80u : 0u;   // signed bytes: subtract 256 where bit 7 is set
#pragma unroll
        for (int tp = T0; tp < T0 + 2; ++tp) {
            uint32_t ow[4] = {0, 0, 0, 0};
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const RpChan p = pc[i];
                int64_t v = rq64(acc[tp][i] + p.bias, p.b, p.c);
                // (no shortcut: the word is zero and so is its term -- rq(0, rb, rc) = 0 for rb < 2^31)
                const uint32_t w = (resw[tp][i >> 2] >> (8 * (i & 3))) & 0xff;
                const int32_t r = (int32_t)w - (int32_t)((w & sgn) << 1);
                const RpRes q = has_res ? pr[i] : RpRes{0, 1};
                v += rq64(r, q.rb, q.rc);
                ow[i >> 2] |= (uint32_t)(clamp64(v, lo_, hi_) & 0xff) << (8 * (i & 3));
            }
            out[tp][0] = ow[0]; out[tp][1] = ow[1]; out[tp][2] = ow[2]; out[tp][3] = ow[3];
        }
        return;
    }
    int32_t lo = lo_, hi = hi_;
    asm volatile("" : "+v"(lo), "+v"(hi));   // in vector registers: the clamp is then one three-operand median
    int32_t y[4][16];   // (only rows T0, T0 + 1 are used)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int32_t bs = pc[i].bs;
        const int64_t Rs = pc[i].Rs;
#pragma unroll
        for (int tp = T0; tp < T0 + 2; ++tp) y[tp][i] = (int32_t)(((int64_t)acc[tp][i] * (int64_t)bs + Rs) >> 32);
    }
    if (has_res) {
        auto add_res = [&](auto sc) {
            constexpr bool S = decltype(sc)::value;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const RpRes p = pr[i];
                const int32_t rr = (int32_t)(1u << ((p.rc - 1) & 31));
#pragma unroll
                for (int tp = T0; tp < T0 + 2; ++tp) {
                    const int32_t r = S ? __builtin_amdgcn_sbfe((int32_t)resw[tp][i >> 2], 8 * (i & 3), 8)
                                        : (int32_t)__builtin_amdgcn_ubfe(resw[tp][i >> 2], 8 * (i & 3), 8);
                    y[tp][i] += (__mul24(r, p.rb) + rr) >> p.rc;
                }
            }
        };
        if (res_signed) add_res(std::true_type{});
        else add_res(std::false_type{});
    }
#pragma unroll
    for (int tp = T0; tp < T0 + 2; ++tp) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            int32_t t;
            asm("v_med3_i32 %0, %1, %2, %3" : "=v"(t) : "v"(y[tp][i]), "v"(lo), "v"(hi));
            y[tp][i] = t;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {   // low bytes of 4 values -> one dword
            const uint32_t t0 = __builtin_amdgcn_perm((uint32_t)y[tp][4 * q + 1], (uint32_t)y[tp][4 * q], 0x0c0c0400u);
            const uint32_t t1 = __builtin_amdgcn_perm((uint32_t)y[tp][4 * q + 3], (uint32_t)y[tp][4 * q + 2], 0x04000c0cu);
            out[tp][q] = t0 | t1;
        }
    }
}

// CCH: input channels / 64 of the 3x3 convolution.  WC x WP = 8 waves: WC along channels (32 each per pass), WP along
// pixels (128 each).  WMAX: largest image width the static LDS patch is sized for.  FUSED: second phase (1x1 on the
// requantised tile, K1 == 64 CCH channels wide, + shortcut).  Without it a workgroup computes `kg` channels of the 3x3
// convolution's output (grid: tiles x K1 / kg) and its epilogue stores to memory (optionally adding a shortcut).
template <int CCH, int WC, int WP, int WMAX, bool FUSED>
__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
conv_rp_kernel(const RpArgs a) {
    static_assert(WC * WP == 8, "eight waves");
    static_assert(CCH >= 2, "the double-buffered fragment registers assume an even number of K-steps per filter row");
    constexpr int T = 512;
    constexpr int BP = 128 * WP;              // output pixels per tile
    constexpr int C = 64 * CCH;
    constexpr int PITCH = C + 16;             // bytes per LDS row (patch and, fused, the intermediate tile: K1 == C)
    constexpr int ROWS = BP + 2 * WMAX + 2;   // patch rows; row ROWS is the row of zeros
    constexpr int S1 = 9 * CCH;               // K-steps of the 3x3 convolution
    constexpr int S2 = CCH;                   // K-steps of the fused 1x1 convolution (K1 / 64)
    constexpr int NCH1 = FUSED ? C : 512;     // stage-1 channels a workgroup can own
    constexpr int NCH2 = FUSED ? 4 * C : 1;   // stage-2 channels (at most)
    __shared__ __attribute__((aligned(16))) uint8_t patch[(ROWS + 1) * PITCH];
    __shared__ __attribute__((aligned(16))) uint8_t tile[FUSED ? BP * PITCH : 16];
    __shared__ RpChan par1[NCH1];
    __shared__ RpChan par2[NCH2];
    __shared__ RpRes pres[FUSED ? NCH2 : NCH1];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wc = wave % WC, wp = wave / WC;
    const int rho = lane & 31, khalf = lane >> 5;

    const int ncg = FUSED ? 1 : a.K1 / a.kg;                        // channel groups (workgroups per tile)
    const uint32_t L = xcd_remap(blockIdx.x, gridDim.x);
    const int tile_i = (int)(L / (uint32_t)ncg), cg = (int)(L % (uint32_t)ncg);
    const int m0 = tile_i * BP;
    const int W = a.W, H = a.H, HW = a.H * a.W;
    const int kg = FUSED ? C : a.kg;                                 // stage-1 channels of this workgroup
    const int kbase1 = cg * kg;
    const int npass1 = kg / (32 * WC);

    // ---- patch: flat input pixels m0 - W - 1 ... m0 + BP + W of every channel, one contiguous range of memory ----
    const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, (int)((int64_t)a.M * C), 0x00020000);
    {
        constexpr int CPR = C / 16;                                  // 16-byte chunks per pixel
        constexpr int NIT = (ROWS * CPR + T - 1) / T;
        const int nchunk = (BP + 2 * W + 2) * CPR;
        const int64_t src0 = ((int64_t)m0 - W - 1) * C;
        v4i v[NIT];
#pragma unroll
        for (int j = 0; j < NIT; ++j) {
            const int i = tid + j * T;
            // outside the tensor (before the first or after the last pixel) the offset is out of range: zeros
            const int64_t o = src0 + (int64_t)i * 16;
            const uint32_t off = (i < nchunk && o >= 0) ? (uint32_t)o : 0x80000000u;
            v[j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, (int)off, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < NIT; ++j) {
            const int i = tid + j * T;
            if (i < nchunk) *(v4i *)(patch + (i / CPR) * PITCH + (i % CPR) * 16) = v[j];
        }
        if (tid < CPR) *(v4i *)(patch + ROWS * PITCH + tid * 16) = (v4i){0, 0, 0, 0};
    }
    // ---- per-channel parameters ----
    int wide = 0;
    const bool has_res1 = !FUSED && a.res != nullptr;
    for (int i = tid; i < kg; i += T) {
        RpChan p;
        wide |= rp_stage_chan(a.bias1, a.b1, a.c1, kbase1 + i, p);
        par1[i] = p;
        if (has_res1) {
            RpRes q;
            q.rb = a.res_b[kbase1 + i]; q.rc = a.res_c[kbase1 + i];
            if (q.rc > 31 || q.rb >= (1 << 22)) wide = 1;
            pres[i] = q;
        }
    }
    if constexpr (FUSED) {
        for (int i = tid; i < a.K2; i += T) {
            RpChan p;
            wide |= rp_stage_chan(a.bias2, a.b2, a.c2, i, p);
            par2[i] = p;
            RpRes q;
            q.rb = a.res_b[i]; q.rc = a.res_c[i];
            if (q.rc > 31 || q.rb >= (1 << 22)) wide = 1;
            pres[i] = q;
        }
    }

    // ---- the lane's four pixels: LDS row offsets, and which of the nine taps lie inside the image ----
    int base[4];
    uint32_t vmask[4];
    uint32_t yoff[4];   // byte offset of the pixel's first channel in the tensor this launch stores (out of range: no such pixel)
    const int Ky = FUSED ? a.K2 : a.K1;
#pragma unroll
    for (int tp = 0; tp < 4; ++tp) {
        const int p = wp * 128 + tp * 32 + rho;
        const int64_t m = (int64_t)m0 + p;
        const bool pvalid = m < a.M;
        yoff[tp] = pvalid ? (uint32_t)(m * Ky) : 0x80000000u;
        const int rem = pvalid ? (int)(m % HW) : 0;
        const int yy = rem / W, xx = rem - yy * W;
        uint32_t mask = 0;
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int s = 0; s < 3; ++s)
                if (pvalid && (unsigned)(yy + r - 1) < (unsigned)H && (unsigned)(xx + s - 1) < (unsigned)W) mask |= 1u << (r * 3 + s);
        vmask[tp] = mask;
        base[tp] = p * PITCH + khalf * 16;
    }
    const int zaddr = ROWS * PITCH + khalf * 16;

    // ---- weight stream of this wave: channel groups  (kbase1 / 32) + wc * npass1 + pass,  K-steps in order ----
    const int G1 = (a.K1 + 31) / 32;
    __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void *)a.w1f, 0, (int)((int64_t)G1 * S1 * 2048), 0x00020000);
    const int lane16 = lane * 16;
    int woff = __builtin_amdgcn_readfirstlane((kbase1 / 32 + wc * npass1) * S1 * 2048);   // byte offset of the next K-step to fetch
    v4i af[3][2];
#pragma unroll
    for (int d = 0; d < 3; ++d) {
        af[d][0] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, lane16, woff, 0);
        af[d][1] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, lane16, woff + 1024, 0);
        woff += 2048;
    }

    wide = __syncthreads_or(wide);   // patch and parameters are in LDS

    v16i acc[4];
    v4i bf[2][2][4];   // [buffer][half of the K-step][pixel tile]
    int sel[4];
    // row offsets of tap (r, s) for the lane's four pixels (the zero row where the tap is outside the image)
    auto set_tap = [&](int r, int s) {
        const int tapoff = (r * W + s) * PITCH;
        const int bit = r * 3 + s;
#pragma unroll
        for (int tp = 0; tp < 4; ++tp) sel[tp] = ((vmask[tp] >> bit) & 1u) ? base[tp] + tapoff : zaddr;
    };
    auto read_b1 = [&](auto bufc, auto ccc) {
        constexpr int buf = decltype(bufc)::value, cc = decltype(ccc)::value;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int tp = 0; tp < 4; ++tp) bf[buf][kk][tp] = *(const v4i *)(patch + sel[tp] + cc * 64 + kk * 32);
    };
    auto mfma8 = [&](auto bufc, const v4i(&aw)[2]) {
        constexpr int buf = decltype(bufc)::value;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int tp = 0; tp < 4; ++tp) acc[tp] = __builtin_amdgcn_mfma_i32_32x32x32_i8(aw[kk], bf[buf][kk][tp], acc[tp], 0, 0, 0);
    };
    using B0 = std::integral_constant<int, 0>;
    using B1 = std::integral_constant<int, 1>;

    // y of the stage whose epilogue stores to memory
    const __amdgpu_buffer_rsrc_t rsrc_y = __builtin_amdgcn_make_buffer_rsrc((void *)a.y, 0, (int)((int64_t)a.M * Ky), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_r = __builtin_amdgcn_make_buffer_rsrc((void *)(a.res ? a.res : a.x), 0, a.res ? (int)((int64_t)a.M * Ky) : 0, 0x00020000);
    const bool res_signed = a.res_dt == HAWQ_S8;
    uint32_t resw[4][4] = {};
    auto load_res = [&](int ch) {   // the lane's 16 shortcut bytes of each of its pixels, channels ch .. ch + 15
#pragma unroll
        for (int tp = 0; tp < 4; ++tp) {
            // (an out-of-range pixel stays out of range: the tensors are below 2 GiB, ch below 2^16)
            const v4i t = __builtin_amdgcn_raw_buffer_load_b128(rsrc_r, (int)(yoff[tp] + (uint32_t)ch), 0, 0);
            resw[tp][0] = (uint32_t)t[0]; resw[tp][1] = (uint32_t)t[1]; resw[tp][2] = (uint32_t)t[2]; resw[tp][3] = (uint32_t)t[3];
        }
    };
    auto store_y = [&](int ch, const uint32_t (&o)[4][4]) {
#pragma unroll
        for (int tp = 0; tp < 4; ++tp) {
            __builtin_amdgcn_raw_buffer_store_b128((v4i){(int)o[tp][0], (int)o[tp][1], (int)o[tp][2], (int)o[tp][3]}, rsrc_y, (int)(yoff[tp] + (uint32_t)ch), 0, 0);
        }
    };

    // ================= phase 1: the 3x3 convolution =================
    if (has_res1) load_res(kbase1 + wc * npass1 * 32 + khalf * 16);
    for (int it = 0; it < 3 * npass1; ++it) {
        const int r = it % 3, pass = it / 3;
        if (r == 0) {
#pragma unroll
            for (int tp = 0; tp < 4; ++tp)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[tp][i] = 0;
            // (the pixel fragments of a pass's first step are not prefetched across the previous pass's epilogue: the
            // epilogue needs the registers)
            set_tap(0, 0);
            read_b1(B0{}, std::integral_constant<int, 0>{});
        }
        // one filter row: taps (r, 0..2) x CCH channel chunks; the pixel fragments of step i + 1 are read while step i
        // is multiplied, the weight fragments of step i + 3 are requested as soon as step i has issued
        static_for<0, 3 * CCH>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            constexpr int slot = i % 3;
            constexpr int cur = i % 2, nxt = (i + 1) % 2;
            constexpr int jn = i + 1;                              // the step to prefetch pixel fragments for
            if constexpr (jn < 3 * CCH) {
                if constexpr (jn % CCH == 0) set_tap(r, jn / CCH);
                read_b1(std::integral_constant<int, nxt>{}, std::integral_constant<int, jn % CCH>{});
            } else if (r != 2) {
                set_tap(r + 1, 0);
                read_b1(std::integral_constant<int, nxt>{}, std::integral_constant<int, 0>{});
            }
            mfma8(std::integral_constant<int, cur>{}, af[slot]);
            af[slot][0] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, lane16, woff, 0);
            af[slot][1] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, lane16, woff + 1024, 0);
            woff += 2048;
            __builtin_amdgcn_sched_barrier(0);
        });
        if (r == 2) {
            const int chl = (wc * npass1 + pass) * 32 + khalf * 16;   // the lane's first channel within the workgroup's range
            uint32_t o[4][4];
            __builtin_amdgcn_sched_barrier(0);
            rp_epilogue<0>(acc, par1 + chl, pres + chl, has_res1, res_signed, resw, wide, a.lo1, a.hi1, o);
            __builtin_amdgcn_sched_barrier(0);
            rp_epilogue<2>(acc, par1 + chl, pres + chl, has_res1, res_signed, resw, wide, a.lo1, a.hi1, o);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (FUSED) {
#pragma unroll
                for (int tp = 0; tp < 4; ++tp)
                    *(v4i *)(tile + (wp * 128 + tp * 32 + rho) * PITCH + chl) = (v4i){(int)o[tp][0], (int)o[tp][1], (int)o[tp][2], (int)o[tp][3]};
            } else {
                if (has_res1 && pass + 1 < npass1) load_res(kbase1 + chl + 32);
                store_y(kbase1 + chl, o);
            }
        }
    }

    // ================= phase 2: 1x1 on the requantised tile, + shortcut =================
    if constexpr (FUSED) {
        const int npass2 = a.K2 / (32 * WC);
        const int G2 = a.K2 / 32;
        rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void *)a.w2f, 0, (int)((int64_t)G2 * S2 * 2048), 0x00020000);
        woff = __builtin_amdgcn_readfirstlane(wc * npass2 * S2 * 2048);
        v4i ag[S2][2];
#pragma unroll
        for (int d = 0; d < S2; ++d) {
            ag[d][0] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, lane16, woff, 0);
            ag[d][1] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, lane16, woff + 1024, 0);
            woff += 2048;
        }
        load_res(wc * npass2 * 32 + khalf * 16);
        __syncthreads();   // every wave's part of the tile is written
        auto read_b2 = [&](auto bufc, auto stc) {
            constexpr int buf = decltype(bufc)::value, st = decltype(stc)::value;
#pragma unroll
            for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                for (int tp = 0; tp < 4; ++tp) bf[buf][kk][tp] = *(const v4i *)(tile + base[tp] + st * 64 + kk * 32);
        };
        for (int pass = 0; pass < npass2; ++pass) {
#pragma unroll
            for (int tp = 0; tp < 4; ++tp)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[tp][i] = 0;
            read_b2(B0{}, std::integral_constant<int, 0>{});
            static_for<0, S2>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                constexpr int cur = i % 2, nxt = (i + 1) % 2;
                if constexpr (i + 1 < S2) read_b2(std::integral_constant<int, nxt>{}, std::integral_constant<int, i + 1>{});
                mfma8(std::integral_constant<int, cur>{}, ag[i]);
                ag[i][0] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, lane16, woff, 0);
                ag[i][1] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, lane16, woff + 1024, 0);
                woff += 2048;
                __builtin_amdgcn_sched_barrier(0);
            });
            const int ch = (wc * npass2 + pass) * 32 + khalf * 16;
            uint32_t o[4][4];
            __builtin_amdgcn_sched_barrier(0);
            rp_epilogue<0>(acc, par2 + ch, pres + ch, true, res_signed, resw, wide, a.lo2, a.hi2, o);
            __builtin_amdgcn_sched_barrier(0);
            rp_epilogue<2>(acc, par2 + ch, pres + ch, true, res_signed, resw, wide, a.lo2, a.hi2, o);
            __builtin_amdgcn_sched_barrier(0);
            if (pass + 1 < npass2) load_res(ch + 32);
            store_y(ch, o);
        }
    }
}

// ---- host side ----

// Which instantiation serves the request; 0 = none.  C = 128: tiles of 256 pixels (4 waves along channels x 2 along
// pixels), image widths up to 28; C = 256: tiles of 128 pixels (8 x 1), widths up to 14 (fused) or 28 (plain).
static int rp_variant(const RpArgs &a, bool fused) {
    if (a.C % 64 != 0 || a.M <= 0 || a.H <= 0 || a.W <= 0) return 0;
    const int cch = a.C / 64;
    if (fused) {
        if (a.K1 != a.C || a.K2 > 4 * a.C) return 0;
        if (cch == 2 && a.W <= 28 && a.K2 % 128 == 0) return 1;
        if (cch == 4 && a.W <= 14 && a.K2 % 256 == 0) return 2;
        return 0;
    }
    if (cch == 2 && a.W <= 28 && a.K1 % 128 == 0) return 3;
    if (cch == 4 && a.W <= 28 && a.K1 % 256 == 0) return 4;
    return 0;
}

bool conv_rp_shape_ok(const RpArgs &a, bool fused) { return rp_variant(a, fused) != 0; }

hawq_status launch_conv_rp(const RpArgs &a_in, bool fused, hipStream_t s) {
    RpArgs a = a_in;
    const int v = rp_variant(a, fused);
    if (v == 0) return HAWQ_ERR_UNSUPPORTED;
    auto tiles = [&](int bp) { return (uint32_t)(((int64_t)a.M + bp - 1) / bp); };
    switch (v) {
    case 1: a.kg = a.C; conv_rp_kernel<2, 4, 2, 28, true><<<tiles(256), 512, 0, s>>>(a); break;
    case 2: a.kg = a.C; conv_rp_kernel<4, 8, 1, 14, true><<<tiles(128), 512, 0, s>>>(a); break;
    case 3: a.kg = 128; conv_rp_kernel<2, 4, 2, 28, false><<<tiles(256) * (uint32_t)(a.K1 / a.kg), 512, 0, s>>>(a); break;
    default: a.kg = 256; conv_rp_kernel<4, 8, 1, 28, false><<<tiles(128) * (uint32_t)(a.K1 / a.kg), 512, 0, s>>>(a); break;
    }
    return check_launch();
}

// Fragment-ordered copy of a weight matrix [K][row bytes] (row = R*S*C, a multiple of 64):
//   out[g][t][kk][lane][16]  with  g = channel group of 32 (rows past K are zero), t = K-step of 64 bytes,
//   lane = khalf * 32 + rho  holding bytes  t*64 + (kk*2 + khalf)*16 .. + 16  of channel
//   32 g + ((rho >> 2) & 1) * 16 + (rho >> 3) * 4 + (rho & 3)
// -- the channel whose accumulator the 32x32x32 MFMA leaves in register (rho >> 3) * 4 + (rho & 3) of lane half
// (rho >> 2) & 1, so that a lane ends up with 16 consecutive channels.
__global__ void __launch_bounds__(256) fragment_weights_kernel(const uint8_t *__restrict__ w, uint8_t *__restrict__ out, const int K,
                                                               const int64_t row, const int64_t chunks) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // index of a 16-byte chunk of the output
    if (i >= chunks) return;
    const int lane = (int)(i & 63), kk = (int)((i >> 6) & 1);
    const int64_t gt = i >> 7;
    const int64_t steps = row / 64;
    const int64_t t = gt % steps, g = gt / steps;
    const int rho = lane & 31, khalf = lane >> 5;
    const int k = (int)g * 32 + ((rho >> 2) & 1) * 16 + (rho >> 3) * 4 + (rho & 3);
    v4i v = {0, 0, 0, 0};
    if (k < K) v = *(const v4i *)(w + (int64_t)k * row + t * 64 + (kk * 2 + khalf) * 16);
    *(v4i *)(out + i * 16) = v;
}

hawq_status launch_fragment_weights(const void *w, void *w_frag, int K, int64_t row, hipStream_t s) {
    const int64_t chunks = (int64_t)((K + 31) / 32) * (row / 64) * 128;
    if (chunks == 0) return HAWQ_OK;
    const int64_t blocks = (chunks + 255) / 256;
    if (blocks > 0x7fffffff) return HAWQ_ERR_UNSUPPORTED;
    fragment_weights_kernel<<<(uint32_t)blocks, 256, 0, s>>>((const uint8_t *)w, (uint8_t *)w_frag, K, row, chunks);
    return check_launch();
}

}  // namespace hawq
