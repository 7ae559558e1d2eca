// Implicit-GEMM quantised convolution on the gfx950 INT8 matrix cores.
//
// GEMM view (Section 3.1's integer convolution): D[k][m] = sum_kg Wt[k][kg] * X[m][kg] with
// m = (n,p,q) an output pixel, k an output channel and kg = (r,s,c).  With NHWC activations and
// KRSC weights both operands are contiguous along kg inside one filter tap, so a K-step is
// "one tap, 64 input channels": 64 bytes per row for INT8, 32 bytes for packed INT4.
//
// Weights are the MFMA "row" operand and pixels the "column" operand, and the rows of a wave's
// tile are assigned to channels through a fixed permutation such that every lane ends up
// holding 16 (or 32) *consecutive* output channels of one pixel: the epilogue then requantises
// in registers and writes 16-byte runs straight into the NHWC output.  INT32 never leaves the
// register file.
//
// INT4 operands stay packed in HBM.  With C a multiple of 128 they also stay packed in LDS (same LDS-DMA
// pipeline as INT8, a K-step then covers 128 channels) and are split into nibbles between the fragment
// read and the MFMA (template parameter PK).  Otherwise the loader passes them through registers, splits
// each 16-byte chunk into low and high nibbles (weights sign-extended) and writes two INT8 chunks to LDS.
// Both operands always use the same nibble de-interleave, i.e. the same permutation of kg, which leaves
// the dot product unchanged.  gfx950 has no 4-bit integer MFMA: a 4-bit layer runs at the INT8 rate.
#include "common.h"
#include "epilogue.h"

namespace hawq {

// XOR swizzle of the four 16-byte chunks of a 64-byte tile row: with this choice of row bits every
// 128-bit LDS fragment read of the MFMA layouts below (both operands, every tile shape) is free of bank
// conflicts (checked with the LDS bank-conflict counter).
__device__ __forceinline__ int swz(int row) { return (row >> 2) & 3; }

constexpr int kMaxSteps = 320;   // K-steps (R*S*C/64, plus the pipeline's run-out) the step table holds

// Minimum waves per SIMD the register allocation must leave room for, by the wave's share of the tile:
// 2 for 64x64 per wave (64 accumulator registers per lane), 3-4 for 64x32, 6 for 32x32 (the latency-bound
// shapes live on occupancy).
// NBUF: LDS buffers in the operand ring (4, or 8 for the 64x64 tile of the LDS-DMA path: few tiles, long reductions)
// DUALM != 0: block output with a convolution on both branches (Section 3.3's residual equation with two INT32
// accumulators, Figure 2): after the main convolution's K-steps the same pipeline runs on through the K-steps of the 1x1
// shortcut convolution (other tensors, same tile) into a second set of accumulators, and the epilogue rescales and adds
// both (DUALM = 1) -- or first rounds the shortcut accumulator to the signed 8-bit value a separate transition layer would
// have stored (DUALM = 2: the bits of the two-launch form without the tensor's round trip; see epilogue_tile_dual).
// DUALM = 3 is DUALM = 1 for callers that know (from the weights and parameters, on the host) that the main branch's
// rescaled term fits 16 bits and that every parameter is in the narrow range: when the main convolution is complete its
// accumulators are rescaled at once and kept as packed 16-bit pairs, half the registers of a second accumulator set,
// which is what lets this form run as eight waves like the plain kernel (see epilogue_tile_dual16).  DUALM = 4: the same
// for the stored-shortcut arithmetic of DUALM = 2.
// PK (4-bit operands whose channel count is a multiple of 128): the packed bytes take the LDS-DMA path unchanged -- a
// K-step is then one tap and 128 input channels, still 64 bytes per row -- and are split into nibbles only between the
// LDS fragment read and the MFMA (see unpack_pk below): per multiply-accumulate half the operand traffic of the INT8
// form at every level above the register file.
template <int BC, int BP, int WC, int WP, bool INT4, int NBUF = 4, int DUALM = 0, bool PK = false>
__global__ void __launch_bounds__(WC *WP * 64) __attribute__((amdgpu_waves_per_eu(BC * BP / (WC * WP) >= 64 * 64 ? 2 : (BC * BP / (WC * WP) >= 64 * 32 ? (WC * WP == 8 ? 4 : 3) : 6))))
conv_mfma_kernel(const ConvArgs a, const uint32_t n_ctiles, const uint32_t nblocks, const int vec_epilogue) {
    constexpr bool DUAL = DUALM != 0;
    constexpr int T = WC * WP * 64;
    static_assert(!PK || INT4, "the packed LDS-DMA form is a 4-bit form");
    constexpr int CPR = (INT4 && !PK) ? 2 : 4;  // 16-byte global chunks per tile row per K-step
    constexpr int BKB = (INT4 && !PK) ? 32 : 64;   // bytes of one K-step in memory
    constexpr int CPS = PK ? 128 : 64;          // input channels of one K-step
    constexpr int NA = (BC * CPR + T - 1) / T;  // chunks per thread, weight tile
    constexpr int NB = (BP * CPR + T - 1) / T;  // chunks per thread, pixel tile
    constexpr int TC = BC / WC / 32;            // 32x32 MFMA tiles per wave along channels
    constexpr int TP = BP / WP / 32;            //                        ... along pixels
    static_assert(BC % (WC * 32) == 0 && BP % (WP * 32) == 0, "tile shape");

    constexpr int kBufBytes = (BC + BP) * 64;
    // INT8 operands go global -> LDS directly (LDS-DMA buffer loads); packed INT4 operands pass through
    // registers to be unpacked.  The four pipeline buffers are separate objects so that the compiler's
    // wait-count tracking of the asynchronous LDS writes is per buffer.
    constexpr bool DMA = !INT4 || PK;
    __shared__ __attribute__((aligned(1024))) uint8_t lds0[kBufBytes];
    __shared__ __attribute__((aligned(1024))) uint8_t lds1[kBufBytes];
    __shared__ __attribute__((aligned(1024))) uint8_t lds2[kBufBytes];
    __shared__ __attribute__((aligned(1024))) uint8_t lds3[kBufBytes];
    static_assert(NBUF == 4 || (NBUF == 8 && !INT4), "ring depth");   // (the deep ring measured slower with packed 4-bit operands)
    static_assert(!DUAL || !INT4, "the two-convolution form takes 8-bit operands");
    __shared__ __attribute__((aligned(1024))) uint8_t lds4[NBUF == 8 ? kBufBytes : 16];
    __shared__ __attribute__((aligned(1024))) uint8_t lds5[NBUF == 8 ? kBufBytes : 16];
    __shared__ __attribute__((aligned(1024))) uint8_t lds6[NBUF == 8 ? kBufBytes : 16];
    __shared__ __attribute__((aligned(1024))) uint8_t lds7[NBUF == 8 ? kBufBytes : 16];
    auto ldsbuf = [&](auto nc) -> uint8_t * {
        constexpr int n = decltype(nc)::value;
        if constexpr (n == 0) return lds0;
        else if constexpr (n == 1) return lds1;
        else if constexpr (n == 2) return lds2;
        else if constexpr (n == 3) return lds3;
        else if constexpr (n == 4) return lds4;
        else if constexpr (n == 5) return lds5;
        else if constexpr (n == 6) return lds6;
        else return lds7;
    };
    __shared__ ChanMain par_m[BC];
    __shared__ ChanRes par_r[(DUALM == 1 || DUALM == 3) ? 1 : BC];   // (two-convolution forms: only the stored-shortcut ones use it)
    __shared__ ChanMain par_s[DUAL ? BC : 1];   // the shortcut convolution's staged parameters
    // Per K-step addressing, tabulated once per workgroup: {weight offset, activation tap offset, r | s << 16}.
    // Deriving these in the loop costs each wave some twenty scalar instructions per step, and the one scalar
    // unit of a CU serves all its waves: with sixteen waves resident that alone approaches the duration of
    // the step's MFMAs.
    __shared__ int4 steptab[kMaxSteps];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: LDS-DMA bases stay in SGPRs
    const int wc = wave % WC, wp = wave / WC;

    const uint32_t L = xcd_remap(blockIdx.x, nblocks);
    const int m0 = (int)(L / n_ctiles) * BP;
    const int k0 = (int)(L % n_ctiles) * BC;

    const int Cb = INT4 ? a.C / 2 : a.C;          // bytes per pixel
    const int cchunks = a.C / CPS;                // K-steps per tap
    const int steps1 = a.R * a.S * cchunks;             // K-steps of the (main) convolution
    const int steps = steps1 + (DUAL ? a.Cs / 64 : 0);  // ... followed by those of the shortcut convolution
    const int64_t wrow_bytes = (int64_t)a.R * a.S * Cb;
    // Weights in blocked order (see ConvArgs::w_t): a channel tile's K-step is 4 KB (64 channels) or 8 KB of contiguous
    // memory instead of 64-byte pieces a filter apart -- whole cache lines, and fewer of them, per LDS-DMA instruction.
    const bool tiled = DMA && a.w_t != nullptr && (!DUAL || a.ws_t != nullptr);
    const int wstep = tiled ? 4096 : BKB;          // bytes from one K-step to the next
    // (the rounded-up loop fetches at most 2*NBUF - 2 entries past the last step)
    for (int i = tid; i < steps + 2 * NBUF; i += T) {
        const int st = i < steps ? i : steps - 1;      // past the last step the activation address stays put ...
        // ... and the weight offset leaves the buffer: the weights read as zeros, padded iterations add nothing
        if (DUAL && st >= steps1) {
            steptab[i] = make_int4(i < steps ? (st - steps1) * wstep : 0x40000000, (st - steps1) * 64, 0, 0);
        } else {
            const int cc = st % cchunks, t = st / cchunks;
            const int s_ = t % a.S, r_ = t / a.S;
            steptab[i] = make_int4(i < steps ? i * wstep : 0x40000000, (r_ * a.W + s_) * Cb + cc * BKB,
                                   r_ | (s_ << 16), 0);
        }
    }
    __syncthreads();

    // ---- per-thread load bookkeeping ----
    // Operands are fetched with buffer loads: a lane whose row is past the tensor edge, or whose
    // filter tap falls into the zero padding, presents an offset beyond num_records and the
    // hardware returns zeros -- no branch, no select, and the address is one 32-bit add.
    constexpr uint32_t kInvalid = 0x80000000u;     // >= any tensor size the interface accepts
    // (not const: the two-convolution form switches descriptors and offsets to the shortcut's tensors once)
    __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(tiled ? a.w_t : a.w), 0, (int)(tiled ? (int64_t)((a.K + 63) / 64) * steps1 * 4096 : (int64_t)a.K * wrow_bytes), 0x00020000);
    __amdgpu_buffer_rsrc_t rsrc_x =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, (int)((int64_t)a.N * a.H * a.W * Cb), 0x00020000);
    int a_row[NA], a_ch[NA];
    uint32_t a_voff[NA];
#pragma unroll
    for (int j = 0; j < NA; ++j) {
        const int i = tid + j * T;
        a_row[j] = i / CPR;
        // LDS-DMA: lane i of the workgroup writes LDS chunk i, so it must fetch the logical chunk that the
        // XOR swizzle places there; register path: lane i fetches logical chunk i%CPR and swizzles on write
        a_ch[j] = DMA ? ((i % CPR) ^ swz(a_row[j])) : (i % CPR);
        const int k = k0 + a_row[j];
        const bool ok = (i < BC * CPR) && (k < a.K);
        a_voff[j] = !ok ? kInvalid
                        : tiled ? (uint32_t)((k >> 6) * steps1 * 4096 + (k & 63) * 64 + a_ch[j] * 16)
                                : (uint32_t)(k * (int)wrow_bytes + a_ch[j] * 16);
    }
    int b_row[NB], b_ch[NB], b_ih0[NB], b_iw0[NB];
    uint32_t b_voff[NB];   // offset of tap (0,0), channel chunk 0 (may be "negative" inside the padding)
    bool b_ok[NB];
    const int PQ = a.P * a.Q;
    bool padded = (a.pad_h | a.pad_w) != 0;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int i = tid + j * T;
        b_row[j] = i / CPR;
        b_ch[j] = DMA ? ((i % CPR) ^ swz(b_row[j])) : (i % CPR);
        const int m = m0 + b_row[j];
        b_ok[j] = (i < BP * CPR) && (m < a.M);
        const int mm = b_ok[j] ? m : 0;
        const int n = mm / PQ, pq = mm - n * PQ;
        const int p = pq / a.Q, q = pq - p * a.Q;
        b_ih0[j] = p * a.stride_h - a.pad_h;
        b_iw0[j] = q * a.stride_w - a.pad_w;
        b_voff[j] = (uint32_t)(((n * a.H + b_ih0[j]) * a.W + b_iw0[j]) * Cb + b_ch[j] * 16);
        if (!b_ok[j] && !padded) b_voff[j] = kInvalid;   // unpadded: validity never changes with the tap
    }

    v16i acc[TP][TC];
    constexpr bool D16 = DUALM >= 3;
    // two-convolution form: the finished main-branch accumulators (D16: their rescaled values, two per register)
    v16i accm[DUAL ? (D16 ? 1 : TP) : 1][DUAL ? (D16 ? (TP * TC + 1) / 2 : TC) : 1];
    const int chl_early = wc * (BC / WC) + (lane >> 5) * 16 * TC;   // the lane's first channel within the tile (as in the epilogue)
#pragma unroll
    for (int tp = 0; tp < TP; ++tp)
#pragma unroll
        for (int tc = 0; tc < TC; ++tc)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[tp][tc][i] = 0;
    if constexpr (DUAL) {
        // The same rows' offsets into the shortcut convolution's weights and (strided, unpadded) activations.  They are
        // needed once, when the fetches switch over, which is always before the main accumulators are parked in accm:
        // until then they live in accm's registers instead of adding to the loop's register pressure.
        static_assert(NA + NB <= 16, "parking space");
#pragma unroll
        for (int j = 0; j < NA; ++j) {
            const int k = k0 + a_row[j];
            accm[0][0][j] = (int)(k >= a.K ? kInvalid
                                           : tiled ? (uint32_t)((k >> 6) * (a.Cs / 64) * 4096 + (k & 63) * 64 + a_ch[j] * 16)
                                                   : (uint32_t)(k * a.Cs + a_ch[j] * 16));
        }
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int mm = b_ok[j] ? m0 + b_row[j] : 0;
            const int n = mm / PQ, pq = mm - n * PQ;
            const int p = pq / a.Q, q = pq - p * a.Q;
            accm[0][0][NA + j] = (int)(b_ok[j] ? (uint32_t)(((n * a.Hs + p * a.stride_sh) * a.Ws + q * a.stride_sw) * a.Cs + b_ch[j] * 16) : kInvalid);
        }
    }

    // Two register sets: while K-step t is multiplied out of LDS, step t+1 sits in one set (issued one
    // iteration ago, written to LDS at the end of this one) and step t+2 is being fetched into the other,
    // so a global load has two iterations to land.  Loads are issued unconditionally in the steady state
    // (past the last step they re-read it): under a branch the compiler could not count outstanding loads
    // and would wait for all of them before every LDS write.
    v4i ra[2][NA], rb[2][NB];
    // K-steps are fetched strictly in order; `ent` is the table entry of the next step to fetch, itself read
    // one fetch ahead so that its LDS latency is never waited for
    int tab_i = 0;
    int4 ent = steptab[0];
    // gload(step, set): register path -- fetch K-step `step` into register set `set`.
    // gload(step, buf) with DMA -- fetch K-step `step` straight into LDS buffer `buf`: every wave-instruction
    // fills 64 consecutive 16-byte chunks (16 tile rows), the destination base is wave-uniform.
    auto gload = [&](int step, auto setc) {
        constexpr int set = decltype(setc)::value;
        (void)step;
        if constexpr (DUAL) {
            if (tab_i == steps1) {   // first K-step of the shortcut convolution: from here on its tensors are fetched
                rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void *)(tiled ? a.ws_t : a.ws), 0,
                                                           (int)(tiled ? (int64_t)((a.K + 63) / 64) * (a.Cs / 64) * 4096 : (int64_t)a.K * a.Cs), 0x00020000);
                rsrc_x = __builtin_amdgcn_make_buffer_rsrc((void *)a.xs, 0, (int)((int64_t)a.N * a.Hs * a.Ws * a.Cs), 0x00020000);
                // the shortcut's offsets were parked in the not yet used second accumulator set (see below)
#pragma unroll
                for (int j = 0; j < NA; ++j) a_voff[j] = (uint32_t)accm[0][0][j];
#pragma unroll
                for (int j = 0; j < NB; ++j) b_voff[j] = (uint32_t)accm[0][0][NA + j];
                padded = false;
            }
        }
        const uint32_t a_off = (uint32_t)ent.x, tapoff = (uint32_t)ent.y;
        const int r = ent.z & 0xffff, s = ent.z >> 16;
#pragma unroll
        for (int j = 0; j < NA; ++j) {
            if constexpr (DMA) {
                if (NA * T != BC * CPR && tid + j * T >= BC * CPR) continue;   // (never for INT8: tiles divide evenly)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    rsrc_w, (__attribute__((address_space(3))) void *)(ldsbuf(setc) + (j * (T / 64) + wave) * 1024), 16,
                    (int)(a_voff[j] + a_off), 0, 0, 0);
            } else {
                ra[set][j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, (int)(a_voff[j] + a_off), 0, 0);
            }
        }
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            uint32_t off = b_voff[j] + tapoff;
            if (padded) {
                const bool ok = b_ok[j] & ((unsigned)(b_ih0[j] + r) < (unsigned)a.H) & ((unsigned)(b_iw0[j] + s) < (unsigned)a.W);
                off = ok ? off : kInvalid;
            }
            if constexpr (DMA) {
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    rsrc_x, (__attribute__((address_space(3))) void *)(ldsbuf(setc) + BC * 64 + (j * (T / 64) + wave) * 1024), 16,
                    (int)off, 0, 0, 0);
            } else {
                rb[set][j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, (int)off, 0, 0);
            }
        }
        ent = steptab[++tab_i];
    };

    // LDS write addresses in buffer 0 (per chunk; INT4 writes two 16-byte pieces)
    int a_wo[NA][2], b_wo[NB][2];
#pragma unroll
    for (int j = 0; j < NA; ++j) {
        const int row = a_row[j], sw = swz(row);
        a_wo[j][0] = row * 64 + (((INT4 ? 2 * a_ch[j] : a_ch[j]) ^ sw) << 4);
        a_wo[j][1] = row * 64 + (((2 * a_ch[j] + 1) ^ sw) << 4);
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int row = b_row[j], sw = swz(row);
        b_wo[j][0] = BC * 64 + row * 64 + (((INT4 ? 2 * b_ch[j] : b_ch[j]) ^ sw) << 4);
        b_wo[j][1] = BC * 64 + row * 64 + (((2 * b_ch[j] + 1) ^ sw) << 4);
    }
    // Write chunk `idx` (0..NA-1: weights, NA..NA+NB-1: pixels) of register set `set` to LDS buffer `buf`.
    auto lstore_one = [&](auto bufc, auto setc, auto idxc) {
        constexpr int set = decltype(setc)::value;
        constexpr int idx = decltype(idxc)::value;
        constexpr bool isA = idx < NA;
        constexpr int j = isA ? idx : idx - NA;
        constexpr int rows = isA ? BC : BP;
        if ((isA ? NA : NB) * T != rows * CPR && tid + j * T >= rows * CPR) return;
        uint8_t *p0, *p1;
        v4i v;
        if constexpr (isA) { p0 = ldsbuf(bufc) + a_wo[j][0]; p1 = ldsbuf(bufc) + a_wo[j][1]; v = ra[set][j]; }
        else { p0 = ldsbuf(bufc) + b_wo[j][0]; p1 = ldsbuf(bufc) + b_wo[j][1]; v = rb[set][j]; }
        if (INT4 && !PK) {
            v4i lo, hi;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                uint32_t u = (uint32_t)v[e];
                uint32_t l = u & 0x0F0F0F0Fu, h = (u >> 4) & 0x0F0F0F0Fu;
                if (isA) {   // weights: sign-extend each nibble to a byte
                    l |= (l & 0x08080808u) * 0x1Eu;
                    h |= (h & 0x08080808u) * 0x1Eu;
                }
                lo[e] = (int)l; hi[e] = (int)h;
            }
            *(v4i *)p0 = lo;
            *(v4i *)p1 = hi;
        } else {
            *(v4i *)p0 = v;
        }
    };
    auto lstore = [&](auto bufc, auto setc) {
        static_for<0, NA + NB>([&](auto ic) { lstore_one(bufc, setc, ic); });
    };

    // ---- MFMA fragment addresses (loop invariant) ----
    // Row operand: MFMA row rho = lane%32 of channel tile tc is output register i = (rho>>3)*4 + (rho&3)
    // of lane half h = (rho>>2)&1; we want that register to be channel  h*16*TC + tc*16 + i  of the wave.
    const int rho = lane & 31, khalf = lane >> 5;
    const int hsel = (rho >> 2) & 1, isel = (rho >> 3) * 4 + (rho & 3);
    // byte offsets of the lane's fragments inside a buffer (the buffer's base is a link-time constant that
    // folds into the instruction's immediate offset)
    int a_fo[TC][2], b_fo[TP][2];
#pragma unroll
    for (int tc = 0; tc < TC; ++tc) {
        const int row = wc * (BC / WC) + hsel * 16 * TC + tc * 16 + isel;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) a_fo[tc][kk] = row * 64 + (((kk * 2 + khalf) ^ swz(row)) << 4);
    }
#pragma unroll
    for (int tp = 0; tp < TP; ++tp) {
        const int row = wp * (BP / WP) + tp * 32 + rho;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) b_fo[tp][kk] = BC * 64 + row * 64 + (((kk * 2 + khalf) ^ swz(row)) << 4);
    }

    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    using S2 = std::integral_constant<int, 2>;
    using S3 = std::integral_constant<int, 3>;
    if constexpr (DMA) {
        static_for<0, NBUF - 1>([&](auto ic) { gload(decltype(ic)::value, ic); });
    } else {
        gload(0, S0{});
        gload(1, S1{});
    }
    // hot epilogue: 8-bit / 4-bit requantised outputs with whole 16-channel groups
    const bool tile_epi = vec_epilogue && a.b != nullptr && a.y_dt != HAWQ_S32;
    int wide = 0;
    if constexpr (DUAL) wide = stage_params_dual(a, k0, BC, par_m, par_s, (DUALM == 2 || DUALM == 4) ? par_r : nullptr);
    else if (tile_epi) wide = stage_params(a, k0, BC, par_m, par_r);
    // the lane's shortcut bytes are fetched now, a whole K loop ahead of their use in the epilogue
    uint32_t resw[TP][TC][4] = {};
    const bool has_res = tile_epi && a.res != nullptr;
    if (has_res) {
        const bool r4 = is4(a.res_dt);
        const __amdgpu_buffer_rsrc_t rsrc_r =
            __builtin_amdgcn_make_buffer_rsrc((void *)a.res, 0, (int)tensor_bytes((int64_t)a.M * a.K, a.res_dt), 0x00020000);
        const int chq = k0 + wc * (BC / WC) + khalf * 16 * TC;
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) {
            const int64_t m = m0 + wp * (BP / WP) + tp * 32 + rho;
#pragma unroll
            for (int tc = 0; tc < TC; ++tc) {
                const int64_t e = m * (int64_t)a.K + chq + 16 * tc;
                const uint32_t ro = (m < a.M && chq + 16 * tc < a.K) ? (uint32_t)(r4 ? (e >> 1) : e) : kInvalid;
                if (r4) {
                    const uint2 t = __builtin_bit_cast(uint2, __builtin_amdgcn_raw_buffer_load_b64(rsrc_r, (int)ro, 0, 0));
                    resw[tp][tc][0] = t.x; resw[tp][tc][1] = t.y; resw[tp][tc][2] = 0; resw[tp][tc][3] = 0;
                } else {
                    const v4i t = __builtin_amdgcn_raw_buffer_load_b128(rsrc_r, (int)ro, 0, 0);
                    resw[tp][tc][0] = (uint32_t)t[0]; resw[tp][tc][1] = (uint32_t)t[1];
                    resw[tp][tc][2] = (uint32_t)t[2]; resw[tp][tc][3] = (uint32_t)t[3];
                }
            }
        }
    }
    // ---- software pipeline over a ring of LDS buffers (described for the ring of four) ----
    // Register path (INT4), iteration t (LDS buffer t%4 is multiplied):
    //   * K-step t+2, requested two iterations ago, is written from register set t%2 to buffer (t+2)%4
    //     (last read in iteration t-2); K-step t+4 is requested into the freed register set.
    // LDS-DMA path (INT8), iteration t:
    //   * K-step t+3 is requested straight into buffer (t+3)%4 (last read in iteration t-1); before the closing
    //     barrier every wave waits until its own requests of iteration t-1 have landed, so after the barrier
    //     step t+2 is complete for all waves.
    // Both: the first-half fragments of step t+1 are read while this step's MFMAs run, so after the closing
    // barrier the next MFMAs issue at once.  One barrier per K-step.  The loop is unrolled four times with a
    // single exit (the trip count is rounded up; padded steps multiply zero weights), so buffer and
    // register-set indices are compile-time constants and the accumulators stay in place.
    if constexpr (DMA) {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NBUF - 3) * (NA + NB)) : "memory");   // steps 0 and 1 have landed (later ones may fly)
    } else {
        lstore(S0{}, S0{});
        lstore(S1{}, S1{});
        gload(2, S0{});
        gload(3, S1{});
    }
    wide = __syncthreads_or(wide);
    v4i af0[TC], bf0[TP];   // first-half fragments of the step about to be multiplied
#pragma unroll
    for (int tc = 0; tc < TC; ++tc) af0[tc] = *(const v4i *)(lds0 + a_fo[tc][0]);
#pragma unroll
    for (int tp = 0; tp < TP; ++tp) bf0[tp] = *(const v4i *)(lds0 + b_fo[tp][0]);

    // Packed 4-bit fragments: a lane's 16 bytes hold 32 channels of its row.  Low and high nibbles go to two MFMAs; both
    // operands are split the same way, i.e. the reduction index is permuted identically on both sides.  Activations
    // (unsigned) become bytes 0..15.  Weights (two's complement nibbles) are left in the upper half of their byte -- the
    // byte then reads as 16 w, with the sign in place and no sign extension to compute -- so the accumulators hold
    // 16 times the convolution and are shifted back once, after the K loop (exact; 16 * 15 * 8 * R*S*C is far inside
    // INT32 for every reduction length the step table admits).
    auto mfma_pk = [&](const v4i(&af)[TC], const v4i(&bf)[TP], auto between) {
        v4i al[TC], ah[TC], bl[TP], bh[TP];
#pragma unroll
        for (int tc = 0; tc < TC; ++tc)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t u = (uint32_t)af[tc][e];
                al[tc][e] = (int)((u << 4) & 0xF0F0F0F0u);
                ah[tc][e] = (int)(u & 0xF0F0F0F0u);
            }
#pragma unroll
        for (int tp = 0; tp < TP; ++tp)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t u = (uint32_t)bf[tp][e];
                bl[tp][e] = (int)(u & 0x0F0F0F0Fu);
                bh[tp][e] = (int)((u >> 4) & 0x0F0F0F0Fu);
            }
        static_for<0, TP * TC>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            constexpr int tp = i / TC, tc = i % TC;
            acc[tp][tc] = __builtin_amdgcn_mfma_i32_32x32x32_i8(al[tc], bl[tp], acc[tp][tc], 0, 0, 0);
            if constexpr (i == 0) between();
            acc[tp][tc] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ah[tc], bh[tp], acc[tp][tc], 0, 0, 0);
        });
        __builtin_amdgcn_sched_barrier(0);
    };
    auto iteration = [&](int step, auto phasec) {
        constexpr int phase = decltype(phasec)::value;            // step % 4
        using Cur = std::integral_constant<int, phase>;
        using Nxt = std::integral_constant<int, (phase + 1) % NBUF>;
        using Wr = std::integral_constant<int, (phase + 2) % 4>;
        using Dma = std::integral_constant<int, (phase + NBUF - 1) % NBUF>;
        using Set = std::integral_constant<int, phase % 2>;
        if constexpr (DUAL) {
            if (step == steps1) {   // the main convolution is complete: park its accumulators, start the shortcut's at zero
#pragma unroll
                for (int tp = 0; tp < TP; ++tp)
#pragma unroll
                    for (int tc = 0; tc < TC; ++tc) {
                        if constexpr (D16) {
                            // t = rq(acc + bias, b, c) in the narrow evaluation (high word of acc * (b << (32-c)) + rounding)
#pragma unroll
                            for (int i = 0; i < 16; i += 2) {
                                const ChanMain &p0 = par_m[chl_early + 16 * tc + i], &p1 = par_m[chl_early + 16 * tc + i + 1];
                                const int32_t t0 = (int32_t)(((int64_t)acc[tp][tc][i] * (int64_t)p0.bs + p0.Rs) >> 32);
                                const int32_t t1 = (int32_t)(((int64_t)acc[tp][tc][i + 1] * (int64_t)p1.bs + p1.Rs) >> 32);
                                accm[0][(tp * TC + tc) / 2][((tp * TC + tc) % 2) * 8 + i / 2] = (int)(((uint32_t)t0 & 0xffffu) | ((uint32_t)t1 << 16));
                            }
                        } else {
                            accm[tp][tc] = acc[tp][tc];
                        }
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc[tp][tc][i] = 0;
                    }
            }
        }
        v4i af1[TC], bf1[TP];
#pragma unroll
        for (int tc = 0; tc < TC; ++tc) af1[tc] = *(const v4i *)(ldsbuf(Cur{}) + a_fo[tc][1]);
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) bf1[tp] = *(const v4i *)(ldsbuf(Cur{}) + b_fo[tp][1]);
        if constexpr (DMA) gload(step + NBUF - 1, Dma{});
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (PK) {
            mfma_pk(af0, bf0, [] {});
        } else {
        // first-half MFMAs (register path: each followed by one LDS write of step+2)
        static_for<0, TP * TC>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            constexpr int tp = i / TC, tc = i % TC;
            acc[tp][tc] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af0[tc], bf0[tp], acc[tp][tc], 0, 0, 0);
            if constexpr (!DMA && i < NA + NB) lstore_one(Wr{}, Set{}, ic);
            __builtin_amdgcn_sched_barrier(0);
        });
        }
        if constexpr (!DMA) {
            static_for<TP * TC, NA + NB>([&](auto ic) { lstore_one(Wr{}, Set{}, ic); });
            gload(step + 4, Set{});
            __builtin_amdgcn_sched_barrier(0);
        }
        // second-half MFMAs with the next step's first-half fragment reads in between
        if constexpr (PK) {
            mfma_pk(af1, bf1, [&] {
#pragma unroll
                for (int t2 = 0; t2 < TC; ++t2) af0[t2] = *(const v4i *)(ldsbuf(Nxt{}) + a_fo[t2][0]);
#pragma unroll
                for (int t2 = 0; t2 < TP; ++t2) bf0[t2] = *(const v4i *)(ldsbuf(Nxt{}) + b_fo[t2][0]);
            });
        } else
        static_for<0, TP * TC>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            constexpr int tp = i / TC, tc = i % TC;
            acc[tp][tc] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af1[tc], bf1[tp], acc[tp][tc], 0, 0, 0);
            if constexpr (i == 0) {
#pragma unroll
                for (int t2 = 0; t2 < TC; ++t2) af0[t2] = *(const v4i *)(ldsbuf(Nxt{}) + a_fo[t2][0]);
#pragma unroll
                for (int t2 = 0; t2 < TP; ++t2) bf0[t2] = *(const v4i *)(ldsbuf(Nxt{}) + b_fo[t2][0]);
            }
        });
        if constexpr (DMA) {
            // Wait until this wave's requests of the previous iteration are in LDS (the NA+NB just issued may
            // still fly) and its LDS reads are done, then meet the other waves.  A plain barrier instruction
            // is used instead of __syncthreads(): that one carries a workgroup fence, which would wait for
            // *all* outstanding LDS-DMA writes and expose their full latency every K-step.  The memory clobber
            // keeps the compiler from moving LDS accesses across it.
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"((NBUF - 3) * (NA + NB)) : "memory");
        } else {
            __syncthreads();
        }
    };
    for (int step = 0; step < steps; step += NBUF)
        static_for<0, NBUF>([&](auto ic) { iteration(step + decltype(ic)::value, ic); });

    if constexpr (PK) {
#pragma unroll
        for (int tp = 0; tp < TP; ++tp)
#pragma unroll
            for (int tc = 0; tc < TC; ++tc)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[tp][tc][i] >>= 4;
    }
    // ---- epilogue: lane owns pixel (tile tp, column rho) and channels ch0 .. ch0 + 16*TC ----
    const int chl = wc * (BC / WC) + khalf * 16 * TC;
    const int ch0 = k0 + chl;
    if (ch0 >= a.K) return;
    if constexpr (DUAL) {
        int64_t mm[TP];
        bool valid[TP];
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) {
            mm[tp] = m0 + wp * (BP / WP) + tp * 32 + rho;
            valid[tp] = mm[tp] < a.M;
        }
        if constexpr (D16) {
            uint32_t t16[TP * TC * 8];
#pragma unroll
            for (int j = 0; j < TP * TC * 8; ++j) t16[j] = (uint32_t)accm[0][j / 16][j % 16];
            epilogue_tile_dual16<TC, TP, DUALM == 4>(a, par_s, par_r, mm, valid, k0, chl, t16, acc);
        } else {
            epilogue_tile_dual<TC, TP, 0, DUALM == 2>(a, par_m, par_s, par_r, mm, valid, k0, chl, accm, acc, wide);
        }
    } else {
    if (tile_epi) {
        int64_t mm[TP];
        bool valid[TP];
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) {
            mm[tp] = m0 + wp * (BP / WP) + tp * 32 + rho;
            valid[tp] = mm[tp] < a.M;
        }
        epilogue_tile<TC, TP, true>(a, par_m, par_r, mm, valid, k0, chl, acc, wide, resw);
        return;
    }
    static_for<0, TP>([&](auto tpc) {
        constexpr int tp = decltype(tpc)::value;
        const int m = m0 + wp * (BP / WP) + tp * 32 + rho;
        if (m >= a.M) return;
        if (vec_epilogue) epilogue_pixel<TC, true>(a, m, ch0, acc[tp]);
        else epilogue_pixel<TC, false>(a, m, ch0, acc[tp]);
    });
    }
}

// 4-bit operands take the packed LDS-DMA form when a tap's channels fill whole 128-channel K-steps
static bool conv_mfma_packed(const ConvArgs &a) { return is4(a.x_dt) && a.C % 128 == 0; }

bool conv_mfma_eligible(const ConvArgs &a, int x_hi) {
    if (a.C % 64 != 0) return false;
    const bool four = is4(a.x_dt);
    if (four != is4(a.w_dt)) return false;
    if (four) {
        if (a.x_dt != HAWQ_U4 || a.w_dt != HAWQ_S4) return false;
    } else {
        if (a.w_dt != HAWQ_S8) return false;
        if (a.x_dt == HAWQ_U8 && x_hi > 127) return false;   // needs the signed INT8 operand range
        if (a.x_dt != HAWQ_U8 && a.x_dt != HAWQ_S8) return false;
    }
    if (((uintptr_t)a.x | (uintptr_t)a.w) & 15) return false;
    if ((int64_t)a.R * a.S * (a.C / (conv_mfma_packed(a) ? 128 : 64)) + 16 > kMaxSteps) return false;   // the per-step address table is in LDS
    // the pipeline's padded K-steps present the weight offset 2^30 and rely on it lying outside the weights (so that they
    // read as zeros): the weight matrix, also in its blocked order (channels rounded up to 64), must end below it
    if ((int64_t)((a.K + 63) / 64 * 64) * a.R * a.S * (is4(a.w_dt) ? a.C / 2 : a.C) >= ((int64_t)1 << 30)) return false;
    return true;
}

bool conv_mfma_dual_eligible(const ConvArgs &a, int x_hi, int xs_hi) {
    if (a.xs == nullptr || a.res != nullptr || a.b == nullptr) return false;
    if (a.mid_s8 && (a.res_b == nullptr || a.res_c == nullptr)) return false;
    if (!conv_mfma_eligible(a, x_hi) || is4(a.x_dt)) return false;
    if (a.Cs % 64 != 0 || a.ws_dt != HAWQ_S8) return false;
    if (a.xs_dt == HAWQ_U8 ? xs_hi > 127 : a.xs_dt != HAWQ_S8) return false;
    if ((int64_t)a.R * a.S * (a.C / 64) + a.Cs / 64 + 16 > kMaxSteps) return false;
    if ((int64_t)((a.K + 63) / 64 * 64) * a.Cs >= ((int64_t)1 << 30)) return false;   // (as above, for the shortcut's weights)
    // every array 16-byte aligned, whole 16-channel groups (the epilogue's vector form), 8-bit or unsigned 4-bit output
    uintptr_t al = (uintptr_t)a.xs | (uintptr_t)a.ws | (uintptr_t)a.y | (uintptr_t)a.bias | (uintptr_t)a.b | (uintptr_t)a.bias_s |
                   (uintptr_t)a.b_s | (uintptr_t)a.c | (uintptr_t)a.c_s;
    if ((al & 15) || a.K % 16 != 0 || a.y_dt == HAWQ_S32) return false;
    return true;
}

hawq_status launch_conv_mfma_dual(const ConvArgs &a, hipStream_t s) {
    if (a.M == 0) return HAWQ_OK;
    const uint32_t n_ctiles = (a.K + 127) / 128, n_mtiles = (a.M + 127) / 128;
    // four waves of 64 channels x 64 pixels: two accumulator sets of that size need the register budget of two waves per
    // SIMD (the eight-wave form would spill inside the K loop, and a reload there waits for every operand in flight)
    if (a.dual16) {
        // the eight-wave form (the caller vouches for the 16-bit bound and the narrow parameters)
        const int steps16 = a.R * a.S * (a.C / 64) + a.Cs / 64;
        if (!a.corun && a.K >= 512 && n_ctiles * n_mtiles <= 112 && steps16 >= 32) {
            const uint32_t nc = (a.K + 63) / 64, nm = (a.M + 63) / 64;
            if (a.mid_s8) conv_mfma_kernel<64, 64, 2, 2, false, 4, 4><<<nc * nm, 256, 0, s>>>(a, nc, nc * nm, 1);
            else conv_mfma_kernel<64, 64, 2, 2, false, 4, 3><<<nc * nm, 256, 0, s>>>(a, nc, nc * nm, 1);
        } else if (a.mid_s8) {
            conv_mfma_kernel<128, 128, 4, 2, false, 4, 4><<<n_ctiles * n_mtiles, 512, 0, s>>>(a, n_ctiles, n_ctiles * n_mtiles, 1);
        } else {
            conv_mfma_kernel<128, 128, 4, 2, false, 4, 3><<<n_ctiles * n_mtiles, 512, 0, s>>>(a, n_ctiles, n_ctiles * n_mtiles, 1);
        }
        return check_launch();
    }
    // few tiles, long reduction, the chip to itself: quarter-size tiles (see launch_conv_mfma; 40.4 -> 36.6 us for the 7x7
    // 3x3 512 -> 512 + 1x1 256 -> 512 block output at batch 64; a ring of eight changes nothing here)
    const int steps = a.R * a.S * (a.C / 64) + a.Cs / 64;
    if (!a.corun && a.K >= 512 && n_ctiles * n_mtiles <= 112 && steps >= 32) {
        const uint32_t nc = (a.K + 63) / 64, nm = (a.M + 63) / 64;
        if (a.mid_s8) conv_mfma_kernel<64, 64, 2, 2, false, 4, 2><<<nc * nm, 256, 0, s>>>(a, nc, nc * nm, 1);
        else conv_mfma_kernel<64, 64, 2, 2, false, 4, 1><<<nc * nm, 256, 0, s>>>(a, nc, nc * nm, 1);
        return check_launch();
    }
    if (a.mid_s8) conv_mfma_kernel<128, 128, 2, 2, false, 4, 2><<<n_ctiles * n_mtiles, 256, 0, s>>>(a, n_ctiles, n_ctiles * n_mtiles, 1);
    else conv_mfma_kernel<128, 128, 2, 2, false, 4, 1><<<n_ctiles * n_mtiles, 256, 0, s>>>(a, n_ctiles, n_ctiles * n_mtiles, 1);
    return check_launch();
}

template <int BC, int BP, int WC, int WP>
static hawq_status launch_cfg(const ConvArgs &a, int vec, hipStream_t s, bool deep = false) {
    const uint32_t n_ctiles = (a.K + BC - 1) / BC;
    const uint32_t n_mtiles = (a.M + BP - 1) / BP;
    const uint32_t nblocks = n_ctiles * n_mtiles;
    if constexpr (BC == 64 && BP == 64) {
        if (deep && !is4(a.x_dt)) {
            conv_mfma_kernel<BC, BP, WC, WP, false, 8><<<nblocks, WC * WP * 64, 0, s>>>(a, n_ctiles, nblocks, vec);
            return check_launch();
        }
    }
    if (conv_mfma_packed(a))
        conv_mfma_kernel<BC, BP, WC, WP, true, 4, 0, true><<<nblocks, WC * WP * 64, 0, s>>>(a, n_ctiles, nblocks, vec);
    else if (is4(a.x_dt))
        conv_mfma_kernel<BC, BP, WC, WP, true><<<nblocks, WC * WP * 64, 0, s>>>(a, n_ctiles, nblocks, vec);
    else
        conv_mfma_kernel<BC, BP, WC, WP, false><<<nblocks, WC * WP * 64, 0, s>>>(a, n_ctiles, nblocks, vec);
    return check_launch();
}

static int g_tile_override = 0;   // 0: heuristic; 1..3: force a tile shape (measurement hook)
void set_tile_override(int t) { g_tile_override = (t >= 1 && t <= 3) ? t : 0; }
int tile_override() { return g_tile_override; }

hawq_status launch_conv_mfma(const ConvArgs &a, hipStream_t s) {
    if (a.M == 0) return HAWQ_OK;
    // vector epilogue needs 16-channel groups to be whole and every array 16-byte aligned
    uintptr_t al = (uintptr_t)a.y | (uintptr_t)a.bias | (uintptr_t)a.b | (uintptr_t)a.res_b | (uintptr_t)a.res;
    al |= ((uintptr_t)a.c | (uintptr_t)a.res_c) & 3;
    const int vec = (a.K % 16 == 0) && ((al & 15) == 0);
    if (g_tile_override == 1) return launch_cfg<128, 128, 2, 2>(a, vec, s);
    if (g_tile_override == 2) return launch_cfg<64, 128, 1, 4>(a, vec, s);
    if (g_tile_override == 3) return launch_cfg<64, 64, 2, 2>(a, vec, s);
    // Measured on MI355X over the ResNet layer shapes: with at least 128 output channels the 128x128 tile
    // wins (operand reuse: a CU's vector-memory path delivers ~60 B/clk and its LDS accepts ~70 B/clk of
    // writes, which a 128x128x64 step of INT8 MFMA consumes in exactly the time it takes to multiply), in
    // its 8-wave form (a wave owns 32 channels x 64 pixels: half the accumulators, four waves per SIMD, and every
    // per-channel parameter read in the epilogue serves two pixels); 64-channel layers take 64x128,
    // tiny problems 64x64.
    if (a.K >= 128 && a.M >= 1024) {
        const int64_t nblocks = (int64_t)((a.K + 127) / 128) * ((a.M + 127) / 128);
        const int steps = a.R * a.S * (a.C / (conv_mfma_packed(a) ? 128 : 64));
        // Few tiles and a long reduction (the 7x7 layers of a ResNet at batch 64: 100 tiles of 128x128 for 256 CUs, 72
        // K-steps): every workgroup is alone on its CU and advances one memory latency per ring depth.  Quarter-size
        // tiles put a workgroup on every CU, with the ring of eight (20.0 -> 17.3 us for 7x7 3x3 512 -> 512 at batch 64).
        // Not when another stream's kernels share the chip: they fill the idle CUs better (measured).
        if (!a.corun && a.K >= 512 && nblocks <= 112 && steps >= 32) return launch_cfg<64, 64, 2, 2>(a, vec, s, true);
        // (A ring of eight for the 128x128 tile, for launches with at most one workgroup per CU, paid off while the
        // weights came as 64-byte pieces; with the blocked copy it measures the same or slower, and it is gone.)
        return launch_cfg<128, 128, 4, 2>(a, vec, s);
    }
    if (a.M >= 4096) return launch_cfg<64, 128, 1, 4>(a, vec, s);
    // a few small tiles with a long reduction (the fully connected layer: 32 tiles x 32 K-steps at batch 128) advance one
    // memory latency per ring depth: the ring of eight there too
    return launch_cfg<64, 64, 2, 2>(a, vec, s, (int64_t)((a.K + 63) / 64) * ((a.M + 63) / 64) <= 512 && a.R * a.S * (a.C / (conv_mfma_packed(a) ? 128 : 64)) >= 16);
}

}  // namespace hawq
