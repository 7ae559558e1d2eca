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
#include "rp.h"

namespace hawq {

// CCH: input channels / 64 of the 3x3 convolution.  WC x WP = 8 waves: WC along channels (32 each), WP along pixels
// (32 TP each: TP MFMA column tiles per wave).  WMAX: largest image width the static LDS patch is sized for.  FUSED:
// second phase (1x1 on the requantised tile, K1 == 64 CCH == 32 WC channels wide, + shortcut).  Without it a workgroup
// computes 32 WC channels of the 3x3 convolution's output (grid: tiles x K1 / (32 WC)) and its epilogue stores to memory
// (optionally adding a shortcut).
// PK: packed 4-bit operands (Section 3.5's storage: two elements per byte).  There is no 4-bit matrix instruction, so the
// nibbles become bytes before the MFMA; here that happens at the edges only.  The patch fill splits every 16 packed bytes
// (32 channels) into the 16 low-nibble bytes (even channels) and the 16 high-nibble bytes (odd channels) and writes them
// as two adjacent 16-byte LDS chunks; the weight fragments were expanded once, on the way into the fragment copy, with
// the same even / odd order (launch_fragment_weights), so both operands see the same permutation of the reduction
// index.  The K loop is the 8-bit loop, instruction for instruction: a 4-bit layer costs what its 8-bit twin costs, minus
// half the activation and output bytes.
template <int CCH, int WC, int WP, int TP, int WMAX, bool FUSED, bool PK = false>
__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
conv_rp_kernel(const RpArgs a) {
    static_assert(WC * WP == 8, "eight waves");
    static_assert(!(FUSED && PK), "the fused form takes 8-bit operands");
    static_assert(!FUSED || 32 * WC == 64 * CCH, "fused: the workgroup owns every channel of the intermediate tile");
    constexpr int T = 512;
    constexpr int WPX = 32 * TP;              // pixels per wave
    constexpr int BP = WPX * WP;              // output pixels per tile
    constexpr int C = 64 * CCH;
    constexpr int KG = 32 * WC;               // stage-1 channels of a workgroup
    constexpr int PITCH = C + 16;             // bytes per LDS row (patch and, fused, the intermediate tile: K1 == C)
    constexpr int ROWS = (BP + 2 * WMAX + 2 + 15) / 16 * 16;   // patch rows (rounded up); rows ROWS .. ROWS + 15 hold zeros
    constexpr int S1 = 9 * CCH;               // K-steps of the 3x3 convolution
    constexpr int S2 = CCH;                   // K-steps of the fused 1x1 convolution (K1 / 64)
    constexpr int NCH2 = FUSED ? 4 * C : 1;   // stage-2 channels (at most)
    __shared__ __attribute__((aligned(16))) uint8_t patch[(ROWS + 16) * PITCH];
    __shared__ __attribute__((aligned(16))) uint8_t tile[FUSED ? BP * PITCH : 16];
    __shared__ RpChan par1[KG];
    __shared__ RpChan par2[NCH2];
    __shared__ RpRes pres[FUSED ? NCH2 : KG];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wc = wave % WC, wp = wave / WC;
    const int rho = lane & 31, khalf = lane >> 5;
#ifdef HAWQ_RP_TIMING
    long long tstamp[6] = {0, 0, 0, 0, 0, 0};
    long long pstamp[4] = {0, 0, 0, 0};
#define RP_STAMP(i) tstamp[i] = (long long)__builtin_readcyclecounter()
#define RP_PSTAMP(i) pstamp[i] = (long long)__builtin_readcyclecounter()
#define RP_STAMP_OUT() do { if (a.timing && lane == 0) { for (int q_ = 0; q_ < 6; ++q_) a.timing[((long long)blockIdx.x * 8 + wave) * 10 + q_] = tstamp[q_]; for (int q_ = 0; q_ < 4; ++q_) a.timing[((long long)blockIdx.x * 8 + wave) * 10 + 6 + q_] = pstamp[q_]; } } while (0)
#else
#define RP_STAMP(i) do { } while (0)
#define RP_PSTAMP(i) do { } while (0)
#define RP_STAMP_OUT() do { } while (0)
#endif
    RP_STAMP(0);

    const int ncg = FUSED ? 1 : a.K1 / KG;                           // channel groups (workgroups per tile)
    const uint32_t L = xcd_remap(blockIdx.x, gridDim.x);
    const int tile_i = (int)(L / (uint32_t)ncg), cg = (int)(L % (uint32_t)ncg);
    const int m0 = tile_i * BP;
    const int W = a.W;
    const int kbase1 = cg * KG;
    const bool has_res1 = !FUSED && a.res != nullptr;

    // ---- prologue: every global load of it is issued before the first one is waited for ----
    // patch: flat input pixels m0 - W - 1 ... m0 + BP + W of every channel, one contiguous range of memory
    constexpr int CPR = PK ? C / 32 : C / 16;                    // 16-byte chunks per pixel in memory
    constexpr int NIT = (ROWS * CPR + T - 1) / T;
    const int nchunk = (BP + 2 * W + 2) * CPR;
    v4i pv[NIT];
    {
        const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, (int)((int64_t)a.M * CPR * 16), 0x00020000);
        const int64_t src0 = ((int64_t)m0 - W - 1) * (CPR * 16);
#pragma unroll
        for (int j = 0; j < NIT; ++j) {
            const int i = tid + j * T;
            // outside the tensor (before the first or after the last pixel) the offset is out of range: zeros
            const int64_t o = src0 + (int64_t)i * 16;
            const uint32_t off = (i < nchunk && o >= 0) ? (uint32_t)o : 0x80000000u;
            pv[j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, (int)off, 0, 0);
        }
    }
    // weight stream of this wave: channel group  kbase1 / 32 + wc,  K-steps in order, three steps ahead
    const int G1 = (a.K1 + 31) / 32;
    __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void *)a.w1f, 0, (int)((int64_t)G1 * S1 * 2048), 0x00020000);
    const int lane16 = lane * 16;
    int woff = __builtin_amdgcn_readfirstlane((kbase1 / 32 + wc) * S1 * 2048);   // byte offset of the next K-step to fetch
    constexpr int D = 3;            // K-steps the weight fragments are requested ahead
    v4i af[D][2];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        af[d][0] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, lane16, woff, 0);
        af[d][1] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, lane16, woff + 1024, 0);
        woff += 2048;
    }
    // per-channel parameters: thread i stages channel i of stage 1 and channels i, i + 512, ... of stage 2
    constexpr int NP2 = FUSED ? (NCH2 + T - 1) / T : 0;
    int32_t q1b = 0, q1c = 1, q1bias = 0, q1rb = 0, q1rc = 1;
    int32_t q2b[NP2 + 1], q2c[NP2 + 1], q2bias[NP2 + 1], q2rb[NP2 + 1], q2rc[NP2 + 1];
    if (tid < KG) {
        q1b = a.b1[kbase1 + tid]; q1c = a.c1[kbase1 + tid]; q1bias = a.bias1[kbase1 + tid];
        if (has_res1) { q1rb = a.res_b[kbase1 + tid]; q1rc = a.res_c[kbase1 + tid]; }
    }
    if constexpr (FUSED) {
#pragma unroll
        for (int j = 0; j < NP2; ++j) {
            const int k = tid + j * T;
            const bool ok = k < a.K2;
            q2b[j] = ok ? a.b2[k] : 0; q2c[j] = ok ? a.c2[k] : 1; q2bias[j] = ok ? a.bias2[k] : 0;
            q2rb[j] = ok ? a.res_b[k] : 0; q2rc[j] = ok ? a.res_c[k] : 1;
        }
    }

    RP_PSTAMP(0);
    // ---- the lane's pixels: LDS row offsets, and which of the nine taps lie inside the image ----
    // A tap outside the image reads zeros: its lane is redirected to one of sixteen rows of zeros, the one congruent to the
    // row it would have read (mod 16) -- the sixteen lanes of an LDS access then still fall into sixteen different banks.
    int base[TP];
    uint32_t vmask[TP];
    uint32_t yoff[TP];   // byte offset of the pixel's first channel in the tensor this launch stores (out of range: no such pixel)
    const int Ky = FUSED ? a.K2 : a.K1;
    const int ysh = (PK && a.y4) ? 1 : 0;   // a packed 4-bit output holds two channels per byte
    {
        const int H = a.H, HW = a.H * a.W;
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) {
            const int p = wp * WPX + tp * 32 + rho;
            const int64_t m = (int64_t)m0 + p;
            const bool pvalid = m < a.M;
            yoff[tp] = pvalid ? (uint32_t)((m * Ky) >> ysh) : 0x80000000u;
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
    }

    // ---- LDS: patch, rows of zeros, parameters ----
    RP_PSTAMP(1);
#pragma unroll
    for (int j = 0; j < NIT; ++j) {
        const int i = tid + j * T;
        if (i < nchunk) {
            if constexpr (PK) {   // 16 packed bytes -> low nibbles (even channels), high nibbles (odd channels): two chunks
                v4i lo, hi;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t u = (uint32_t)pv[j][e];
                    lo[e] = (int)(u & 0x0F0F0F0Fu);
                    hi[e] = (int)((u >> 4) & 0x0F0F0F0Fu);
                }
                *(v4i *)(patch + (i / CPR) * PITCH + (i % CPR) * 32) = lo;
                *(v4i *)(patch + (i / CPR) * PITCH + (i % CPR) * 32 + 16) = hi;
            } else {
                *(v4i *)(patch + (i / CPR) * PITCH + (i % CPR) * 16) = pv[j];
            }
        }
    }
    RP_PSTAMP(2);
    for (int i = tid; i < 16 * (C / 16); i += T) *(v4i *)(patch + (ROWS + i / (C / 16)) * PITCH + (i % (C / 16)) * 16) = (v4i){0, 0, 0, 0};
    int wide = 0;
    auto stage = [&](int32_t bias, int32_t b, int32_t c, RpChan &o) {
        o.b = b; o.c = c; o.bias = bias; o.bs = 0; o.Rs = 0;
        if (c > 32 || ((int64_t)b >> (c - 1)) != 0) { wide = 1; return; }
        const int64_t R = (int64_t)bias * (int64_t)b + ((int64_t)1 << (c - 1));
        o.bs = (int32_t)((uint32_t)b << (32 - c));
        o.Rs = (int64_t)((uint64_t)R << (32 - c));
    };
    if (tid < KG) {
        RpChan p;
        stage(q1bias, q1b, q1c, p);
        par1[tid] = p;
        if (has_res1) {
            if (q1rc > 31 || q1rb >= (1 << 22)) wide = 1;
            pres[tid] = RpRes{q1rb, q1rc};
        }
    }
    if constexpr (FUSED) {
#pragma unroll
        for (int j = 0; j < NP2; ++j) {
            const int k = tid + j * T;
            if (k < a.K2) {
                RpChan p;
                stage(q2bias[j], q2b[j], q2c[j], p);
                par2[k] = p;
                if (q2rc[j] > 31 || q2rb[j] >= (1 << 22)) wide = 1;
                pres[k] = RpRes{q2rb[j], q2rc[j]};
            }
        }
    }
    RP_PSTAMP(3);
    wide = __syncthreads_or(wide);   // patch and parameters are in LDS
    RP_STAMP(1);

    v16i acc[TP];
#pragma unroll
    for (int tp = 0; tp < TP; ++tp)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[tp][i] = 0;
    v4i bf[2][TP];   // pixel fragments: [buffer][pixel tile], one half K-step (32 reduction elements) each
    int sel[TP];
    // row offsets of tap (r, s) for the lane's pixels
    auto set_tap = [&](int r, int s) {
        const int shift = r * W + s;
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) {
            const int p = wp * WPX + tp * 32 + rho;
            sel[tp] = ((vmask[tp] >> (r * 3 + s)) & 1u) ? base[tp] + shift * PITCH : (ROWS + ((p + shift) & 15)) * PITCH + khalf * 16;
        }
    };
    auto mfma_row = [&](auto bufc, const v4i &aw) {
        constexpr int buf = decltype(bufc)::value;
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) acc[tp] = __builtin_amdgcn_mfma_i32_32x32x32_i8(aw, bf[buf][tp], acc[tp], 0, 0, 0);
    };

    const __amdgpu_buffer_rsrc_t rsrc_y = __builtin_amdgcn_make_buffer_rsrc((void *)a.y, 0, (int)(((int64_t)a.M * Ky) >> ysh), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_r = __builtin_amdgcn_make_buffer_rsrc((void *)(a.res ? a.res : a.x), 0, a.res ? (int)((int64_t)a.M * Ky) : 0, 0x00020000);
    const bool res_signed = a.res_dt == HAWQ_S8;
    // The lane's shortcut bytes, fetched a whole pass of the second convolution ahead of their use: two buffers where the
    // registers allow it (RB = 2), else one, refilled right after the epilogue that read it.
    constexpr int RB = (FUSED && TP <= 4) ? 2 : 1;
    uint32_t resw[RB][TP + 1][4] = {};   // (one spare row: the last epilogue call of an odd TP reads a pair)
    auto load_res = [&](auto bc, int ch) {   // 16 shortcut bytes of each of the lane's pixels, channels ch .. ch + 15
        constexpr int rb = decltype(bc)::value;
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) {
            // (an out-of-range pixel stays out of range: the tensors are below 2 GiB, ch below 2^16)
            const v4i t = __builtin_amdgcn_raw_buffer_load_b128(rsrc_r, (int)(yoff[tp] + (uint32_t)ch), 0, 0);
            resw[rb][tp][0] = (uint32_t)t[0]; resw[rb][tp][1] = (uint32_t)t[1]; resw[rb][tp][2] = (uint32_t)t[2]; resw[rb][tp][3] = (uint32_t)t[3];
        }
    };
    using R0 = std::integral_constant<int, 0>;
    // epilogue of all the lane's pixels, two at a time; `put(tp, bytes)` stores one pixel's 16 bytes
    auto epilogue = [&](auto bc, const RpChan *pc, const RpRes *pr, bool has_res, int lo, int hi, auto put) {
        constexpr int rb = decltype(bc)::value;
        static_for<0, (TP + 1) / 2>([&](auto jc) {
            constexpr int t0 = 2 * decltype(jc)::value;
            constexpr int nt = t0 + 1 < TP ? 2 : 1;
            const uint32_t rw[2][4] = {{resw[rb][t0][0], resw[rb][t0][1], resw[rb][t0][2], resw[rb][t0][3]},
                                       {resw[rb][t0 + 1][0], resw[rb][t0 + 1][1], resw[rb][t0 + 1][2], resw[rb][t0 + 1][3]}};
            uint32_t o[2][4];
            rp_epilogue<nt>(acc[t0], acc[nt == 2 ? t0 + 1 : t0], pc, pr, has_res, res_signed, rw, wide, lo, hi, o);
            put(std::integral_constant<int, t0>{}, o[0]);
            if constexpr (nt == 2) put(std::integral_constant<int, t0 + 1>{}, o[1]);
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    // ================= phase 1: the 3x3 convolution, 9 CCH K-steps, fully unrolled =================
    // Half-step h (32 reduction elements) = K-step h / 2, half h % 2.  While half-step h is multiplied, the pixel fragments
    // of half-step h + 1 are read into the other buffer; the weight fragments of K-step t + D are requested as soon as
    // K-step t has issued.
    const int chl = wc * 32 + khalf * 16;   // the lane's first channel within the workgroup's range
    if (has_res1) load_res(R0{}, kbase1 + chl);
    set_tap(0, 0);
#pragma unroll
    for (int tp = 0; tp < TP; ++tp) bf[0][tp] = *(const v4i *)(patch + sel[tp]);
    static_for<0, 2 * S1>([&](auto hc) {
        constexpr int h = decltype(hc)::value;
        constexpr int t = h / 2, kk = h % 2;
        constexpr int hn = h + 1, tn = hn / 2, kn = hn % 2;          // the half-step to prefetch
        if constexpr (hn < 2 * S1) {
            if constexpr (kn == 0 && tn % CCH == 0) set_tap((tn / CCH) / 3, (tn / CCH) % 3);
#pragma unroll
            for (int tp = 0; tp < TP; ++tp) bf[hn % 2][tp] = *(const v4i *)(patch + sel[tp] + (tn % CCH) * 64 + kn * 32);
        }
        mfma_row(std::integral_constant<int, h % 2>{}, af[t % D][kk]);
        if constexpr (kk == 1) {
            if constexpr (t + D < S1) {
                af[t % D][0] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, lane16, woff, 0);
                af[t % D][1] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, lane16, woff + 1024, 0);
                woff += 2048;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    });
    RP_STAMP(2);

    auto put_y = [&](int ch) {
        return [&, ch](auto tpc, const uint32_t (&o)[4]) {
            constexpr int tp = decltype(tpc)::value;
            if (PK && a.y4) {
                // sixteen values 0..15, one per byte -> sixteen nibbles, even channel in the low nibble
                auto nib = [](uint32_t d) { return (d & 0xfu) | ((d >> 4) & 0xf0u) | ((d >> 8) & 0xf00u) | ((d >> 12) & 0xf000u); };
                const v2i w = {(int)(nib(o[0]) | (nib(o[1]) << 16)), (int)(nib(o[2]) | (nib(o[3]) << 16))};
                __builtin_amdgcn_raw_buffer_store_b64(w, rsrc_y, (int)(yoff[tp] + (uint32_t)(ch >> 1)), 0, 0);
            } else {
                __builtin_amdgcn_raw_buffer_store_b128((v4i){(int)o[0], (int)o[1], (int)o[2], (int)o[3]}, rsrc_y, (int)(yoff[tp] + (uint32_t)ch), 0, 0);
            }
        };
    };
    if constexpr (!FUSED) {
        epilogue(R0{}, par1 + chl, pres + chl, has_res1, a.lo1, a.hi1, put_y(kbase1 + chl));
    } else {
        // ================= phase 2: 1x1 on the requantised tile, + shortcut =================
        // the second convolution's first weights and shortcut bytes travel while the first one's epilogue runs
        const int npass2 = a.K2 / KG;
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
        __builtin_amdgcn_sched_barrier(0);
        epilogue(R0{}, par1 + chl, pres, false, a.lo1, a.hi1, [&](auto tpc, const uint32_t (&o)[4]) {
            constexpr int tp = decltype(tpc)::value;
            *(v4i *)(tile + (wp * WPX + tp * 32 + rho) * PITCH + chl) = (v4i){(int)o[0], (int)o[1], (int)o[2], (int)o[3]};
        });
        const int ch0 = wc * npass2 * 32 + khalf * 16;   // the lane's first channel of pass 0
        load_res(R0{}, ch0);
        __syncthreads();   // every wave's part of the tile is written
        RP_STAMP(3);
        // Phase 2 alternates a short burst of MFMAs with a long integer epilogue.  Waves w and w + 4 share a SIMD and leave
        // the barrier together; delaying one of them by about one burst makes its MFMAs fall into the other's epilogue
        // instead of both queueing for the matrix pipe and then for the vector ALU.
        if (wave >= 4) __builtin_amdgcn_s_sleep(TP * S2 * 2 * 32 / 64);
        // one pass: 32 output channels per wave; `bc`: which shortcut buffer this pass reads
        auto pass2 = [&](auto bc, int pass) {
            constexpr int rb = decltype(bc)::value;
            // with two buffers the next pass's shortcut bytes are requested before this pass's MFMAs
            if (RB == 2 && pass + 1 < npass2) load_res(std::integral_constant<int, (rb + 1) % RB>{}, ch0 + (pass + 1) * 32);
#pragma unroll
            for (int tp = 0; tp < TP; ++tp)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[tp][i] = 0;
#pragma unroll
            for (int tp = 0; tp < TP; ++tp) bf[0][tp] = *(const v4i *)(tile + base[tp]);
            static_for<0, 2 * S2>([&](auto hc) {
                constexpr int h = decltype(hc)::value;
                constexpr int t = h / 2, kk = h % 2;
                constexpr int hn = h + 1, tn = hn / 2, kn = hn % 2;
                if constexpr (hn < 2 * S2) {
#pragma unroll
                    for (int tp = 0; tp < TP; ++tp) bf[hn % 2][tp] = *(const v4i *)(tile + base[tp] + tn * 64 + kn * 32);
                }
                mfma_row(std::integral_constant<int, h % 2>{}, ag[t][kk]);
                if constexpr (kk == 1) {   // the same K-step of the next pass
                    if (pass + 1 < npass2) {
                        ag[t][0] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, lane16, woff, 0);
                        ag[t][1] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, lane16, woff + 1024, 0);
                        woff += 2048;
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            });
            const int ch = ch0 + pass * 32;
            epilogue(bc, par2 + ch, pres + ch, true, a.lo2, a.hi2, put_y(ch));
            if (RB == 1 && pass + 1 < npass2) load_res(R0{}, ch + 32);
            if (pass == 0) RP_STAMP(4);
        };
        for (int pass = 0; pass < npass2; pass += 2) {
            pass2(R0{}, pass);
            if (pass + 1 < npass2) pass2(std::integral_constant<int, 1 % RB>{}, pass + 1);
        }
    }
    RP_STAMP(5);
    RP_STAMP_OUT();
}

// ---- host side ----

// Which instantiation serves the request; 0 = none.  C = 128: tiles of 448 pixels (4 waves along channels x 2 along
// pixels x 7 MFMA column tiles), image widths up to 28; C = 256: tiles of 128 pixels (8 x 1 x 4), widths up to 14 (fused)
// or 28 (plain); C = 512 (plain only): tiles of 64 pixels (8 x 1 x 2), widths up to 14.  (A 28 x 28 layer at batch 128 has 100352 pixels: 224 tiles of 448 keep every tile in one round on 256
// compute units, where 392 tiles of 256 need two.)
static int rp_variant(const RpArgs &a, bool fused) {
    if (a.C % 64 != 0 || a.M <= 0 || a.H <= 0 || a.W <= 0) return 0;
    const int cch = a.C / 64;
    if (a.pk && (fused || a.res != nullptr)) return 0;
    if (fused) {
        if (a.K1 != a.C || a.K2 > 4 * a.C) return 0;
        if (cch == 2 && a.W <= 28 && a.K2 % 128 == 0) return 1;
        if (cch == 4 && a.W <= 14 && a.K2 % 256 == 0) return 2;
        return 0;
    }
    // (128 channels: below some forty 256-pixel tiles the tiled kernel's 128 x 128 tiles put more compute units to work --
    // 28 x 28 at batch 8: 8.8 us there, 10.9 us here)
    if (cch == 2 && a.W <= 28 && a.K1 % 128 == 0 && a.M >= 40 * 256) return 3;
    if (cch == 4 && a.W <= 28 && a.K1 % 256 == 0) return 4;
    if (cch == 8 && a.W <= 14 && a.K1 % 256 == 0) return 5;
    return 0;
}

bool conv_rp_shape_ok(const RpArgs &a, bool fused) { return rp_variant(a, fused) != 0; }

hawq_status launch_conv_rp(const RpArgs &a, bool fused, hipStream_t s) {
    const int v = rp_variant(a, fused);
    if (v == 0) return HAWQ_ERR_UNSUPPORTED;
    auto tiles = [&](int bp) { return (uint32_t)(((int64_t)a.M + bp - 1) / bp); };
    // few tiles and the chip to itself (14 x 14 at batch 64: 98 tiles of 128 pixels): half the channels per workgroup,
    // twice the workgroups (14x14 256 -> 256 at batch 64: 15.7 -> 11.1 us); with another stream's kernels on the chip the
    // larger workgroups are the better neighbours
    const bool few = !a.corun && tiles(128) * (uint32_t)(a.K1 / 256) < 160;
    // 128 channels: 448-pixel tiles once they cover most of the chip in one round -- counting the other stream's twin launch
    // when the forward runs as two half-batches (2 x 112 tiles then share the 256 compute units)
    const bool wide_tiles = a.M >= 448 * (a.corun ? 80 : 160);
    switch (v) {
    case 1:   // small problems: narrower tiles put more compute units to work
        if (wide_tiles) conv_rp_kernel<2, 4, 2, 7, 28, true><<<tiles(448), 512, 0, s>>>(a);
        else conv_rp_kernel<2, 4, 2, 4, 28, true><<<tiles(256), 512, 0, s>>>(a);
        break;
    case 2: conv_rp_kernel<4, 8, 1, 4, 14, true><<<tiles(128), 512, 0, s>>>(a); break;
    case 3:
        if (a.pk) {
            if (wide_tiles) conv_rp_kernel<2, 4, 2, 7, 28, false, true><<<tiles(448) * (uint32_t)(a.K1 / 128), 512, 0, s>>>(a);
            else conv_rp_kernel<2, 4, 2, 4, 28, false, true><<<tiles(256) * (uint32_t)(a.K1 / 128), 512, 0, s>>>(a);
        } else {
            if (wide_tiles) conv_rp_kernel<2, 4, 2, 7, 28, false><<<tiles(448) * (uint32_t)(a.K1 / 128), 512, 0, s>>>(a);
            else conv_rp_kernel<2, 4, 2, 4, 28, false><<<tiles(256) * (uint32_t)(a.K1 / 128), 512, 0, s>>>(a);
        }
        break;
    case 4:
        if (a.pk) {
            if (few) conv_rp_kernel<4, 4, 2, 2, 28, false, true><<<tiles(128) * (uint32_t)(a.K1 / 128), 512, 0, s>>>(a);
            else conv_rp_kernel<4, 8, 1, 4, 28, false, true><<<tiles(128) * (uint32_t)(a.K1 / 256), 512, 0, s>>>(a);
        } else {
            if (few) conv_rp_kernel<4, 4, 2, 2, 28, false><<<tiles(128) * (uint32_t)(a.K1 / 128), 512, 0, s>>>(a);
            else conv_rp_kernel<4, 8, 1, 4, 28, false><<<tiles(128) * (uint32_t)(a.K1 / 256), 512, 0, s>>>(a);
        }
        break;
    // 512 channels (7 x 7 images: few pixels, long reduction): 64-pixel tiles, so that pixel tiles x channel halves fill the chip
    default:
        if (a.pk) conv_rp_kernel<8, 8, 1, 2, 14, false, true><<<tiles(64) * (uint32_t)(a.K1 / 256), 512, 0, s>>>(a);
        else conv_rp_kernel<8, 8, 1, 2, 14, false><<<tiles(64) * (uint32_t)(a.K1 / 256), 512, 0, s>>>(a);
        break;
    }
    return check_launch();
}

// Fragment-ordered copy of a weight matrix [K][row bytes] of signed bytes (row = R*S*C, a multiple of 64):
//   out[g][t][kk][lane][16]  with  g = channel group of 32 (rows past K are zero), t = K-step of 64 bytes,
//   lane = khalf * 32 + rho  holding bytes  t*64 + (kk*2 + khalf)*16 .. + 16  of channel
//   32 g + ((rho >> 2) & 1) * 16 + (rho >> 3) * 4 + (rho & 3)
// -- the channel whose accumulator the 32x32x32 MFMA leaves in register (rho >> 3) * 4 + (rho & 3) of lane half
// (rho >> 2) & 1, so that a lane ends up with 16 consecutive channels.
// FOUR: the source rows are packed 4-bit (row bytes = R*S*C / 2, a multiple of 32) and are expanded to signed bytes on
// the way: 16-byte chunk 2q of the expanded row holds the sign-extended low nibbles of packed bytes 16q .. 16q + 15 (the
// even elements), chunk 2q + 1 their high nibbles (the odd elements) -- the order in which the kernel's patch fill
// splits the packed activations.  The copy then has the size and the layout of an 8-bit layer's.
template <bool FOUR>
__global__ void __launch_bounds__(256) fragment_weights_kernel(const uint8_t *__restrict__ w, uint8_t *__restrict__ out, const int K,
                                                               const int64_t row, const int64_t chunks) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // index of a 16-byte chunk of the output
    if (i >= chunks) return;
    const int lane = (int)(i & 63), kk = (int)((i >> 6) & 1);
    const int64_t gt = i >> 7;
    const int64_t steps = (FOUR ? 2 * row : row) / 64;
    const int64_t t = gt % steps, g = gt / steps;
    const int rho = lane & 31, khalf = lane >> 5;
    const int k = (int)g * 32 + ((rho >> 2) & 1) * 16 + (rho >> 3) * 4 + (rho & 3);
    v4i v = {0, 0, 0, 0};
    if (k < K) {
        const int64_t ci = t * 4 + kk * 2 + khalf;   // 16-byte chunk of the (expanded) row
        if (FOUR) {
            const v4i p = *(const v4i *)(w + (int64_t)k * row + (ci >> 1) * 16);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                uint32_t u = (uint32_t)p[e];
                u = (ci & 1) ? (u >> 4) & 0x0F0F0F0Fu : u & 0x0F0F0F0Fu;
                v[e] = (int)(u | ((u & 0x08080808u) * 0x1Eu));   // sign-extend each nibble to its byte
            }
        } else {
            v = *(const v4i *)(w + (int64_t)k * row + ci * 16);
        }
    }
    *(v4i *)(out + i * 16) = v;
}

// row: bytes of a weight row as stored (packed 4-bit when four)
hawq_status launch_fragment_weights(const void *w, void *w_frag, int K, int64_t row, bool four, hipStream_t s) {
    const int64_t chunks = (int64_t)((K + 31) / 32) * ((four ? 2 * row : row) / 64) * 128;
    if (chunks == 0) return HAWQ_OK;
    const int64_t blocks = (chunks + 255) / 256;
    if (blocks > 0x7fffffff) return HAWQ_ERR_UNSUPPORTED;
    if (four) fragment_weights_kernel<true><<<(uint32_t)blocks, 256, 0, s>>>((const uint8_t *)w, (uint8_t *)w_frag, K, row, chunks);
    else fragment_weights_kernel<false><<<(uint32_t)blocks, 256, 0, s>>>((const uint8_t *)w, (uint8_t *)w_frag, K, row, chunks);
    return check_launch();
}

}  // namespace hawq
