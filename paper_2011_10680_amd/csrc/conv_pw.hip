// Pointwise (1x1) quantised convolution for shallow reductions (C = 64, 128 or 256), streaming form.
//
// These layers (the expanding 1x1 of a bottleneck with its residual, the stride-1 transition
// convolution, the first reducing 1x1) do a handful of MFMAs per output tile and are bound by HBM
// traffic and by the integer epilogue.  A tile-per-workgroup kernel spends its life in start-up
// latency there.  Here a wave is persistent instead: it keeps the weights of its 32 output channels in
// registers (they are only C/8 registers per lane) and its channels' requantisation parameters in
// registers too (epilogue_lane; a wave-private LDS slot holds the staged copy for parameters outside
// that form's range), then walks over pixel tiles with the next tiles' activations and shortcut
// bytes already in flight while the current tile is multiplied, requantised and stored.  No
// workgroup barrier.
//
// Activations travel global -> LDS (LDS-DMA buffer loads into a wave-private ring) -> MFMA fragments.
// Fetching them straight into the MFMA operand layout would make every lane of a load instruction touch
// its own cache line, which the vector memory path serves at a quarter of its rate (measured: ~16 instead
// of ~60 bytes per clock per CU); the DMA form reads 64 contiguous bytes per four lanes.
#include "common.h"
#include "epilogue.h"

namespace hawq {

// KC: 64-element chunks of the reduction (C / 64); TP: 32-pixel tiles per group; NS: groups in flight per wave
// (ring of LDS stages); WPE: waves per SIMD the register allocation is held to; RES: a shortcut is added.
template <int KC, int TP, int NS, int WPE, bool RES, bool INT4>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(WPE)))
conv_pw_kernel(const ConvArgs a, const int n_ct, const int n_seq, const int n_groups) {
    static_assert(NS == 2 || NS == 3, "ring depth");
    constexpr bool RREG = WPE <= 3;                 // room for the shortcut multipliers (and the biases) in registers too
    constexpr int BKB = INT4 ? 32 : 64;             // bytes of 64 reduction elements in memory = LDS row length
    constexpr int SUB = 32 * BKB;                   // one 32-pixel x 64-element sub-tile
    constexpr int STAGE = TP * KC * SUB;            // LDS bytes of one group of one wave
    constexpr int ND = INT4 ? 1 : 2;                // DMA instructions (1 KB each) per sub-tile
    // vector-memory instructions every wave issues per group, in program order: D loads into LDS and R
    // shortcut loads (issue), later S stores (process).  The counts are the same for every wave and group,
    // so the wait for a stage's arrival is an exact outstanding-operations count.
    constexpr int D = TP * KC * ND, R = RES ? TP : 0, S = TP;
    constexpr uint32_t kInvalid = 0x80000000u;
    __shared__ ChanMain par_m[4][32];
    __shared__ ChanRes par_r[4][32];
    // one array per ring slot: the compiler tracks asynchronous LDS writes per object
    __shared__ __attribute__((aligned(1024))) uint8_t xs0[4 * STAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t xs1[4 * STAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t xs2[NS >= 3 ? 4 * STAGE : 1024];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // workgroups that share pixels (consecutive channel tiles of one sequence) stay on one XCD and its L2
    const int g = (int)xcd_remap(blockIdx.x, gridDim.x) * 4 + wave;
    const int ct = g % n_ct, seq = g / n_ct;
    if (seq >= n_seq) return;                        // whole wave; the kernel has no workgroup barrier
    const int rho = lane & 31, khalf = lane >> 5;
    const int k0 = ct * 32;
    const int Cb = INT4 ? a.C / 2 : a.C;

    // ---- parameters of this wave's 32 channels -> wave-private LDS ----
    int wide = 0;
    {
        ChanMain m;
        ChanRes r;
        if (khalf == 0) {
            wide = stage_channel(a, k0 + rho, m, r);
            par_m[wave][rho] = m;
            par_r[wave][rho] = r;
        }
        wide = __any(wide);
    }
    // the same parameters in registers, in the form the register-resident epilogue takes (falls back to the staged ones)
    LaneParams lp;
    bool fast;
    {
        int T_lo, T_hi;
        const int bad = lane_form_check<RES>(a, k0 + rho, T_lo, T_hi);   // lanes rho and rho + 32 look at the same channel
#pragma unroll
        for (int sft = 1; sft < 32; sft <<= 1) {
            T_lo = max(T_lo, __shfl_xor(T_lo, sft));
            T_hi = min(T_hi, __shfl_xor(T_hi, sft));
        }
        fast = !__any(bad) && !wide && T_lo <= T_hi && a.y_dt != HAWQ_S4 && !(RES && a.res_dt == HAWQ_S4);
        lp.T = T_hi;
        if (RES && fast && khalf == 0) finish_res(a, k0 + rho, T_hi, par_r[wave][rho]);
        load_lane_params(par_m[wave] + khalf * 16, par_r[wave] + khalf * 16, lp);   // (wave-private slots, written by this wave's own lanes above)
    }

    // ---- weights of the 32 channels, in MFMA row-operand layout, resident in registers ----
    // row rho of the tile is channel  hsel*16 + isel  (so that a lane ends up with 16 consecutive channels)
    const int hsel = (rho >> 2) & 1, isel = (rho >> 3) * 4 + (rho & 3);
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void *)a.w, 0, (int)((int64_t)a.K * Cb), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_x =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, (int)((int64_t)a.N * a.H * a.W * Cb), 0x00020000);
    v4i A[KC][2];
    {
        const int k = k0 + hsel * 16 + isel;
        const uint32_t base = k < a.K ? (uint32_t)(k * Cb) : kInvalid;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            if (INT4) {
                const v4i v = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, (int)(base + kc * BKB + khalf * 16), 0, 0);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    uint32_t u = (uint32_t)v[e];
                    uint32_t l = u & 0x0F0F0F0Fu, h = (u >> 4) & 0x0F0F0F0Fu;
                    l |= (l & 0x08080808u) * 0x1Eu;
                    h |= (h & 0x08080808u) * 0x1Eu;
                    A[kc][0][e] = (int)l; A[kc][1][e] = (int)h;
                }
            } else {
#pragma unroll
                for (int kk = 0; kk < 2; ++kk)
                    A[kc][kk] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, (int)(base + kc * 64 + kk * 32 + khalf * 16), 0, 0);
            }
        }
    }

    const bool r4 = is4(a.res_dt);
    const __amdgpu_buffer_rsrc_t rsrc_r = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(RES ? a.res : a.x), 0, RES ? (int)tensor_bytes((int64_t)a.M * a.K, a.res_dt) : 0, 0x00020000);
    const bool unit = a.stride_h == 1 && a.stride_w == 1;   // 1x1, no padding: output pixel m reads input pixel m
    const int PQ = a.P * a.Q;
    auto pixel_offset = [&](int grp, int64_t m) -> uint32_t {   // byte offset of output pixel m's input row
        if (grp >= n_groups || m >= a.M) return kInvalid;
        if (unit) return (uint32_t)m * (uint32_t)Cb;
        const int mi = (int)m;
        const int n = mi / PQ, pq = mi - n * PQ;
        const int p = pq / a.Q, q = pq - p * a.Q;
        return (uint32_t)(((n * a.H + p * a.stride_h) * a.W + q * a.stride_w) * Cb);
    };

    // LDS layout of a sub-tile: 32 rows (pixels) of BKB bytes.  INT8: the four 16-byte chunks of a row are
    // XOR-swizzled with (row >> 2) & 3, which makes the fragment reads below free of bank conflicts; a DMA
    // instruction fills 16 rows, lane i writing slot i (row i/4, chunk i%4) with the chunk that belongs there.
    // INT4: 32-byte rows, one instruction fills all 32 rows.
    const int d_row = INT4 ? lane >> 1 : lane >> 2;                     // row within the instruction's rows
    const int d_chunk = INT4 ? (lane & 1) : ((lane & 3) ^ ((d_row >> 2) & 3));
    // (row >> 2) & 3 is the same for row and row + 16, so one chunk index serves both halves
    struct Stage {
        uint32_t r[TP][1][4];   // the lane's 16 shortcut bytes per tile
    };
    auto issue = [&](int grp, uint8_t *xs, Stage &st) {
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) {
            const int64_t mbase = ((int64_t)grp * TP + tp) * 32;
#pragma unroll
            for (int h = 0; h < ND; ++h) {
                const uint32_t po = pixel_offset(grp, mbase + h * 16 + d_row);
#pragma unroll
                for (int kc = 0; kc < KC; ++kc) {
                    const uint32_t off = po == kInvalid ? kInvalid : po + kc * BKB + d_chunk * 16;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        rsrc_x, (__attribute__((address_space(3))) void *)(xs + wave * STAGE + (tp * KC + kc) * SUB + h * 1024),
                        16, (int)off, 0, 0, 0);
                }
            }
            if (RES) {
                // the lane's 16 channels of pixel m: 16 bytes (8 for 4-bit data)
                const int64_t m = mbase + rho;
                const bool ok = grp < n_groups && m < a.M;
                const int64_t e = m * (int64_t)a.K + k0 + khalf * 16;
                const uint32_t ro = (ok && k0 + khalf * 16 < a.K) ? (uint32_t)(r4 ? (e >> 1) : e) : kInvalid;
                // one 16-byte load for either width (4-bit data uses the first 8 bytes; bytes past the end of the
                // buffer read as zero), so that the count of outstanding operations is static
                const v4i t = __builtin_amdgcn_raw_buffer_load_b128(rsrc_r, (int)ro, 0, 0);
                st.r[tp][0][0] = (uint32_t)t[0]; st.r[tp][0][1] = (uint32_t)t[1];
                st.r[tp][0][2] = (uint32_t)t[2]; st.r[tp][0][3] = (uint32_t)t[3];
            } else {
                st.r[tp][0][0] = st.r[tp][0][1] = st.r[tp][0][2] = st.r[tp][0][3] = 0;
            }
        }
    };

    // the exact general epilogue issues a data-dependent number of stores; after it everything is drained,
    // which keeps the static operation counts below valid
    const bool slow_epilogue = !fast && (wide || a.y_dt == HAWQ_S4 || (RES && a.res_dt == HAWQ_S4));
    const int swz = (rho >> 2) & 3;
    auto process = [&](auto fastc, int grp, const uint8_t *xs, const Stage &st, auto nwaitc) {
        constexpr bool FAST = decltype(fastc)::value;
        // wait until at most NWAIT vector-memory operations issued after this stage's loads are outstanding
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(decltype(nwaitc)::value) : "memory");
        v16i acc[TP][1];
        int64_t mm[TP];
        bool valid[TP];
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[tp][0][i] = FAST ? ((RES && !RREG) ? par_m[wave][khalf * 16 + i].bias : lp.bias[i]) : 0;   // (four waves per SIMD with a shortcut: the registers are short, the bias comes from the staged copy)
            mm[tp] = ((int64_t)grp * TP + tp) * 32 + rho;
            valid[tp] = mm[tp] < a.M;
        }
#pragma unroll
        for (int tp = 0; tp < TP; ++tp)
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) {
                const uint8_t *sub = xs + wave * STAGE + (tp * KC + kc) * SUB + rho * BKB;
                v4i b0, b1;
                if (INT4) {
                    const v4i raw = *(const v4i *)(sub + khalf * 16);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint32_t u = (uint32_t)raw[e];
                        b0[e] = (int)(u & 0x0F0F0F0Fu);
                        b1[e] = (int)((u >> 4) & 0x0F0F0F0Fu);
                    }
                } else {
                    b0 = *(const v4i *)(sub + ((khalf ^ swz) << 4));
                    b1 = *(const v4i *)(sub + (((2 + khalf) ^ swz) << 4));
                }
                acc[tp][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[kc][0], b0, acc[tp][0], 0, 0, 0);
                acc[tp][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[kc][1], b1, acc[tp][0], 0, 0, 0);
            }
        if constexpr (FAST) {
            epilogue_lane<TP, RES, RREG>(a, lp, par_r[wave] + khalf * 16, mm, valid, k0 + khalf * 16, acc, st.r);
        } else {
            epilogue_tile<1, TP, true, 2>(a, par_m[wave], par_r[wave], mm, valid, k0, khalf * 16, acc, wide, st.r);
            if (slow_epilogue) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
    };

    // Ring of NS stages: while group i is processed, groups i + n_seq .. i + (NS-1) n_seq are landing
    // (issue() past the last group presents out-of-range offsets and fetches nothing, but still counts).
    // Operations issued after a stage's own loads when its turn comes: the loads of the NS-1 later stages and
    // the stores of the groups processed since -- none for the first group, up to NS-1 groups' worth later.
    // (the walk exists twice, once per epilogue form, so that neither form's registers burden the other's loop)
    auto walk = [&](auto fastc) {
    Stage st0, st1, st2;   // separate named objects so that each stays in registers
    using W0 = std::integral_constant<int, (NS - 1) * (D + R)>;
    using W1 = std::integral_constant<int, (NS - 1) * (D + R) + S>;
    using WN = std::integral_constant<int, (NS - 1) * (D + R) + (NS - 1) * S>;
    int grp = seq;
    if constexpr (NS == 2) {
        issue(grp, xs0, st0);
        issue(grp + n_seq, xs1, st1);
        process(fastc, grp, xs0, st0, W0{});
        grp += n_seq;
        while (grp < n_groups) {
            issue(grp + n_seq, xs0, st0);
            process(fastc, grp, xs1, st1, WN{});
            grp += n_seq;
            if (grp >= n_groups) break;
            issue(grp + n_seq, xs1, st1);
            process(fastc, grp, xs0, st0, WN{});
            grp += n_seq;
        }
    } else {
        issue(grp, xs0, st0);
        issue(grp + n_seq, xs1, st1);
        issue(grp + 2 * n_seq, xs2, st2);
        process(fastc, grp, xs0, st0, W0{});
        grp += n_seq;
        if (grp >= n_groups) return;
        issue(grp + 2 * n_seq, xs0, st0);
        process(fastc, grp, xs1, st1, W1{});
        grp += n_seq;
        while (grp < n_groups) {
            issue(grp + 2 * n_seq, xs1, st1);
            process(fastc, grp, xs2, st2, WN{});
            grp += n_seq;
            if (grp >= n_groups) break;
            issue(grp + 2 * n_seq, xs2, st2);
            process(fastc, grp, xs0, st0, WN{});
            grp += n_seq;
            if (grp >= n_groups) break;
            issue(grp + 2 * n_seq, xs0, st0);
            process(fastc, grp, xs1, st1, WN{});
            grp += n_seq;
        }
    }
    };
    if (fast) walk(std::true_type{});
    else walk(std::false_type{});
}

// Variant for C = 256 with many output channels: the four waves of a workgroup work on
// four consecutive channel tiles of the *same* pixels, so the activation stage is fetched once per workgroup
// (each wave a quarter of it) into a ring of four shared LDS stages, three groups ahead.  With a stage per wave
// the LDS budget allows a ring of two only, and a wave's walk then advances one memory latency per group.
// One workgroup barrier per group (a stage's arrival; it also orders the stage's reuse).  INT8 operands.
template <int KC, int WPE, bool RES>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(WPE)))
conv_pws_kernel(const ConvArgs a, const int n_ct, const int n_seq, const int n_groups) {
    constexpr int NS = 4;
    constexpr int STAGE = KC * 2048;                // 32 pixels x C bytes
    constexpr int DW = KC * 2 / 4;                  // LDS-DMA instructions (1 KB) per wave and stage
    static_assert(KC % 2 == 0, "stage split");
    constexpr int R = RES ? 1 : 0, S = 1;           // shortcut loads, stores per wave and group
    constexpr uint32_t kInvalid = 0x80000000u;
    __shared__ ChanMain par_m[4][32];
    __shared__ ChanRes par_r[4][32];
    __shared__ __attribute__((aligned(1024))) uint8_t xs0[STAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t xs1[STAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t xs2[STAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t xs3[STAGE];

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // the launch makes n_ct a multiple of 4 and the grid exactly n_seq * n_ct / 4 workgroups: the four waves
    // of a workgroup share `seq` (so every wave reaches every barrier the same number of times)
    const int g = (int)xcd_remap(blockIdx.x, gridDim.x) * 4 + wave;
    const int ct = g % n_ct, seq = g / n_ct;
    const int rho = lane & 31, khalf = lane >> 5;
    const int k0 = ct * 32;
    const int Cb = a.C;

    int wide = 0;
    {
        ChanMain m;
        ChanRes r;
        if (khalf == 0) {
            wide = stage_channel(a, k0 + rho, m, r);
            par_m[wave][rho] = m;
            par_r[wave][rho] = r;
        }
        wide = __any(wide);
    }
    LaneParams lp;   // the same parameters in registers (see conv_pw_kernel)
    bool fast;
    {
        int T_lo, T_hi;
        const int bad = lane_form_check<RES>(a, k0 + rho, T_lo, T_hi);   // lanes rho and rho + 32 look at the same channel
#pragma unroll
        for (int sft = 1; sft < 32; sft <<= 1) {
            T_lo = max(T_lo, __shfl_xor(T_lo, sft));
            T_hi = min(T_hi, __shfl_xor(T_hi, sft));
        }
        fast = !__any(bad) && !wide && T_lo <= T_hi && a.y_dt != HAWQ_S4 && !(RES && a.res_dt == HAWQ_S4);
        lp.T = T_hi;
        if (RES && fast && khalf == 0) finish_res(a, k0 + rho, T_hi, par_r[wave][rho]);
        load_lane_params(par_m[wave] + khalf * 16, par_r[wave] + khalf * 16, lp);   // (wave-private slots, written by this wave's own lanes above)
    }
    const int hsel = (rho >> 2) & 1, isel = (rho >> 3) * 4 + (rho & 3);
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void *)a.w, 0, (int)((int64_t)a.K * Cb), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_x =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, (int)((int64_t)a.N * a.H * a.W * Cb), 0x00020000);
    // The wave's 32 x C weight bytes reach its registers through LDS: fetched with coalesced LDS-DMA loads into
    // the stage buffer of the same number as the wave (a stage is exactly 32 rows x C bytes), then read as MFMA
    // row fragments.  Loading them straight into the fragment layout makes every lane touch its own cache line,
    // and with a dozen waves per CU starting at once that alone costs microseconds.
    v4i A[KC][2];
    {
        uint8_t *wst = wave == 0 ? xs0 : (wave == 1 ? xs1 : (wave == 2 ? xs2 : xs3));
        const int w_row = lane >> 2;
        const int w_chunk = (lane & 3) ^ ((w_row >> 2) & 3);
#pragma unroll
        for (int inst = 0; inst < 2 * KC; ++inst) {
            const int kc = inst >> 1, h = inst & 1;
            const int k = k0 + h * 16 + w_row;
            const uint32_t off = k < a.K ? (uint32_t)(k * Cb + kc * 64 + w_chunk * 16) : kInvalid;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_w, (__attribute__((address_space(3))) void *)(wst + inst * 1024), 16,
                                                     (int)off, 0, 0, 0);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        const int row = hsel * 16 + isel;
        const int sw = (row >> 2) & 3;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc)
#pragma unroll
            for (int kk = 0; kk < 2; ++kk)
                A[kc][kk] = *(const v4i *)(wst + kc * 2048 + row * 64 + (((kk * 2 + khalf) ^ sw) << 4));
        __syncthreads();    // every wave has its weights (and parameters) before the stage buffers are reused
    }
    const bool r4 = is4(a.res_dt);
    const __amdgpu_buffer_rsrc_t rsrc_r = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(RES ? a.res : a.x), 0, RES ? (int)tensor_bytes((int64_t)a.M * a.K, a.res_dt) : 0, 0x00020000);
    const bool unit = a.stride_h == 1 && a.stride_w == 1;
    const int PQ = a.P * a.Q;
    auto pixel_offset = [&](int grp, int64_t m) -> uint32_t {
        if (grp >= n_groups || m >= a.M) return kInvalid;
        if (unit) return (uint32_t)m * (uint32_t)Cb;
        const int mi = (int)m;
        const int n = mi / PQ, pq = mi - n * PQ;
        const int p = pq / a.Q, q = pq - p * a.Q;
        return (uint32_t)(((n * a.H + p * a.stride_h) * a.W + q * a.stride_w) * Cb);
    };
    // stage layout: KC sub-tiles of 32 rows x 64 B (chunks XOR-swizzled with (row >> 2) & 3); the 2 KC fetch
    // instructions of a stage (16 rows of one sub-tile each) are dealt round-robin to the four waves
    const int d_row = lane >> 2;
    const int d_chunk = (lane & 3) ^ ((d_row >> 2) & 3);
    struct Stage {
        uint32_t r[1][1][4];
    };
    auto issue = [&](int grp, uint8_t *xs, Stage &st) {
        const int64_t mbase = (int64_t)grp * 32;
#pragma unroll
        for (int j = 0; j < DW; ++j) {
            const int inst = wave + 4 * j;            // 0 .. 2 KC - 1: sub-tile inst / 2, row half inst % 2
            const int kc = inst >> 1, h = inst & 1;
            const uint32_t po = pixel_offset(grp, mbase + h * 16 + d_row);
            const uint32_t off = po == kInvalid ? kInvalid : po + kc * 64 + d_chunk * 16;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_x, (__attribute__((address_space(3))) void *)(xs + inst * 1024), 16,
                                                     (int)off, 0, 0, 0);
        }
        if (RES) {
            const int64_t m = mbase + rho;
            const bool ok = grp < n_groups && m < a.M;
            const int64_t e = m * (int64_t)a.K + k0 + khalf * 16;
            const uint32_t ro = (ok && k0 + khalf * 16 < a.K) ? (uint32_t)(r4 ? (e >> 1) : e) : kInvalid;
            const v4i t = __builtin_amdgcn_raw_buffer_load_b128(rsrc_r, (int)ro, 0, 0);
            st.r[0][0][0] = (uint32_t)t[0]; st.r[0][0][1] = (uint32_t)t[1];
            st.r[0][0][2] = (uint32_t)t[2]; st.r[0][0][3] = (uint32_t)t[3];
        } else {
            st.r[0][0][0] = st.r[0][0][1] = st.r[0][0][2] = st.r[0][0][3] = 0;
        }
    };
    const bool slow_epilogue = !fast && (wide || a.y_dt == HAWQ_S4 || (RES && a.res_dt == HAWQ_S4));
    const int swz = (rho >> 2) & 3;
    auto compute = [&](auto fastc, int grp, const uint8_t *xs, const Stage &st) {
        constexpr bool FAST = decltype(fastc)::value;
        v16i acc[1][1];
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[0][0][i] = FAST ? ((RES && WPE > 2) ? par_m[wave][khalf * 16 + i].bias : lp.bias[i]) : 0;
        const int64_t mm[1] = {(int64_t)grp * 32 + rho};
        const bool valid[1] = {mm[0] < a.M};
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            const uint8_t *sub = xs + kc * 2048 + rho * 64;
            const v4i b0 = *(const v4i *)(sub + ((khalf ^ swz) << 4));
            const v4i b1 = *(const v4i *)(sub + (((2 + khalf) ^ swz) << 4));
            acc[0][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[kc][0], b0, acc[0][0], 0, 0, 0);
            acc[0][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[kc][1], b1, acc[0][0], 0, 0, 0);
        }
        if constexpr (FAST) {
            epilogue_lane<1, RES, (WPE <= 2)>(a, lp, par_r[wave] + khalf * 16, mm, valid, k0 + khalf * 16, acc, st.r);
        } else {
            epilogue_tile<1, 1, true, 2>(a, par_m[wave], par_r[wave], mm, valid, k0, khalf * 16, acc, wide, st.r);
            if (slow_epilogue) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
    };
    // Per group and wave, in program order: [wait for the stage] [barrier] DW stage loads + R shortcut loads for
    // the group three ahead, then this group's S stores.  Operations issued after a stage's own loads when its turn
    // comes: the loads of the two later stages and the stores of the groups processed since (none for the first
    // group, up to three groups' worth from the fourth on).
    auto arrive = [&](int it) {
        constexpr int L = (NS - 2) * (DW + R);
        if (it == 0) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(L) : "memory");
        else if (it == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(L + S) : "memory");
        else if (it == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(L + 2 * S) : "memory");
        else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(L + 3 * S) : "memory");
        __builtin_amdgcn_s_barrier();
    };
    auto walk = [&](auto fastc) {   // once per epilogue form (see conv_pw_kernel)
    Stage st0, st1, st2, st3;
    int grp = seq, it = 0;
    issue(grp, xs0, st0);
    issue(grp + n_seq, xs1, st1);
    issue(grp + 2 * n_seq, xs2, st2);
#define HAWQ_PWS_STEP(curx, curs, nxtx, nxts)        \
    arrive(it);                                      \
    issue(grp + 3 * n_seq, nxtx, nxts);              \
    compute(fastc, grp, curx, curs);                 \
    grp += n_seq;                                    \
    ++it;                                            \
    if (grp >= n_groups) break;
    while (grp < n_groups) {
        HAWQ_PWS_STEP(xs0, st0, xs3, st3)
        HAWQ_PWS_STEP(xs1, st1, xs0, st0)
        HAWQ_PWS_STEP(xs2, st2, xs1, st1)
        HAWQ_PWS_STEP(xs3, st3, xs2, st2)
    }
#undef HAWQ_PWS_STEP
    };
    if (fast) walk(std::true_type{});
    else walk(std::false_type{});
}

// Block output with a convolution on both branches, streaming form: the shared-stage kernel above with the pixels of
// BOTH 1x1 convolutions in a stage -- KC1 sub-tiles of the main branch's input followed by KC2 of the shortcut's
// (strided) input -- two weight sets in registers and two accumulators per wave.  MID: the shortcut accumulator is first
// rounded to the signed 8-bit value a separate transition layer would store (see epilogue_tile_dual).  The transition
// tensor is never written or read, and one launch replaces two.
template <int KC1, int KC2, int WPE, bool MID>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(WPE)))
conv_pws_dual_kernel(const ConvArgs a, const int n_ct, const int n_seq, const int n_groups) {
    constexpr int NS = 4;
    constexpr int KC = KC1 + KC2;
    constexpr int STAGE = KC * 2048;                // 32 pixels x (C + Cs) bytes
    constexpr int DW = KC * 2 / 4;                  // LDS-DMA instructions (1 KB) per wave and stage
    static_assert(KC % 2 == 0, "stage split");
    constexpr int S = 1;                            // stores per wave and group
    constexpr uint32_t kInvalid = 0x80000000u;
    __shared__ ChanMain par_m[4][32];
    __shared__ ChanMain par_s[4][32];
    __shared__ ChanRes par_r[4][32];
    __shared__ __attribute__((aligned(1024))) uint8_t xs0[STAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t xs1[STAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t xs2[STAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t xs3[STAGE];

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = (int)xcd_remap(blockIdx.x, gridDim.x) * 4 + wave;
    const int ct = g % n_ct, seq = g / n_ct;        // the four waves of a workgroup share `seq` (n_ct is a multiple of 4)
    const int rho = lane & 31, khalf = lane >> 5;
    const int k0 = ct * 32;

    int wide = 0;
    if (khalf == 0) {
        ChanMain m, r;
        wide = stage_branch(a.bias, a.b, a.c, k0 + rho, a.K, m) | stage_branch(a.bias_s, a.b_s, a.c_s, k0 + rho, a.K, r);
        par_m[wave][rho] = m;
        par_s[wave][rho] = r;
        ChanRes q = ChanRes{0, 1, 1, 0};
        if (MID) wide |= stage_res(a.res_b, a.res_c, k0 + rho, a.K, q);
        par_r[wave][rho] = q;
    }
    wide = __any(wide);
    const int hsel = (rho >> 2) & 1, isel = (rho >> 3) * 4 + (rho & 3);
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void *)a.w, 0, (int)((int64_t)a.K * a.C), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_ws = __builtin_amdgcn_make_buffer_rsrc((void *)a.ws, 0, (int)((int64_t)a.K * a.Cs), 0x00020000);
    // both weight sets (32 rows x (C + Cs) bytes: exactly one stage) reach the registers through LDS, coalesced
    v4i A[KC][2];
    {
        uint8_t *wst = wave == 0 ? xs0 : (wave == 1 ? xs1 : (wave == 2 ? xs2 : xs3));
        const int w_row = lane >> 2;
        const int w_chunk = (lane & 3) ^ ((w_row >> 2) & 3);
#pragma unroll
        for (int inst = 0; inst < 2 * KC; ++inst) {
            const int kc = inst >> 1, h = inst & 1;
            const int k = k0 + h * 16 + w_row;
            if (kc < KC1) {
                const uint32_t off = k < a.K ? (uint32_t)(k * a.C + kc * 64 + w_chunk * 16) : kInvalid;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_w, (__attribute__((address_space(3))) void *)(wst + inst * 1024), 16,
                                                         (int)off, 0, 0, 0);
            } else {
                const uint32_t off = k < a.K ? (uint32_t)(k * a.Cs + (kc - KC1) * 64 + w_chunk * 16) : kInvalid;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_ws, (__attribute__((address_space(3))) void *)(wst + inst * 1024), 16,
                                                         (int)off, 0, 0, 0);
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        const int row = hsel * 16 + isel;
        const int sw = (row >> 2) & 3;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc)
#pragma unroll
            for (int kk = 0; kk < 2; ++kk)
                A[kc][kk] = *(const v4i *)(wst + kc * 2048 + row * 64 + (((kk * 2 + khalf) ^ sw) << 4));
        __syncthreads();    // every wave has its weights (and parameters) before the stage buffers are reused
    }
    // A wave's fetch instructions of a stage: sub-tile (wave + 4 j) / 2, row half (wave + 4 j) % 2 -- which tensor an
    // instruction reads is fixed per wave and j, so its descriptor and per-pixel stride are chosen once, here.
    const int PQ = a.P * a.Q;
    const int d_row = lane >> 2;
    const int d_chunk = (lane & 3) ^ ((d_row >> 2) & 3);
    // Where a lane's shortcut fetch reads (image, row, column of its output pixel) is found by division once, for the wave's
    // first group; successive calls of issue() are one sequence stride (32 n_seq pixels) apart, so the byte offset then
    // advances by wave-uniform increments with two carries -- no division in the loop.
    const int step_px = 32 * n_seq;
    const int dn = step_px / PQ, drem = step_px - dn * PQ, dp = drem / a.Q, dq = drem - dp * a.Q;
    const uint32_t row_b = (uint32_t)(a.stride_sh * a.Ws * a.Cs), col_b = (uint32_t)(a.stride_sw * a.Cs);
    const uint32_t inc_q = (uint32_t)dq * col_b, inc_p = (uint32_t)dp * row_b;
    const uint32_t inc_n = (uint32_t)dn * (uint32_t)(a.Hs * a.Ws * a.Cs);
    const uint32_t wrap_q = row_b - (uint32_t)a.Q * col_b;                              // next row, first column
    const uint32_t wrap_p = (uint32_t)(a.Hs * a.Ws * a.Cs) - (uint32_t)a.P * row_b;     // next image, first row
    int s_p[DW], s_q[DW];
    uint32_t s_off[DW];
#pragma unroll
    for (int j = 0; j < DW; ++j) {
        const int inst = wave + 4 * j;
        const int kc = inst >> 1, h = inst & 1;
        const int mi = seq * 32 + h * 16 + d_row;
        const int n = mi / PQ, pq = mi - n * PQ;
        s_p[j] = pq / a.Q;
        s_q[j] = pq - s_p[j] * a.Q;
        s_off[j] = (uint32_t)(((n * a.Hs + s_p[j] * a.stride_sh) * a.Ws + s_q[j] * a.stride_sw) * a.Cs) +
                   (uint32_t)((kc - KC1) * 64 + d_chunk * 16);
    }
    const __amdgpu_buffer_rsrc_t rsrc_xm = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, (int)((int64_t)a.N * a.H * a.W * a.C), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_xs = __builtin_amdgcn_make_buffer_rsrc((void *)a.xs, 0, (int)((int64_t)a.N * a.Hs * a.Ws * a.Cs), 0x00020000);
    // (calls must come in the order of the walk below: grp = seq, seq + n_seq, seq + 2 n_seq, ...)
    auto issue = [&](int grp, uint8_t *xs) {
        const int64_t mbase = (int64_t)grp * 32;
#pragma unroll
        for (int j = 0; j < DW; ++j) {
            const int inst = wave + 4 * j;
            const int kc = inst >> 1, h = inst & 1;
            const bool main_branch = kc < KC1;      // wave-uniform
            const int64_t m = mbase + h * 16 + d_row;
            const bool ok = grp < n_groups && m < a.M;
            auto *dst = (__attribute__((address_space(3))) void *)(xs + inst * 1024);
            if (main_branch) {                      // a scalar branch: each side names its own descriptor
                const uint32_t off = ok ? (uint32_t)m * (uint32_t)a.C + kc * 64 + d_chunk * 16 : kInvalid;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_xm, dst, 16, (int)off, 0, 0, 0);
            } else {
                const uint32_t off = ok ? s_off[j] : kInvalid;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_xs, dst, 16, (int)off, 0, 0, 0);
                s_q[j] += dq;
                s_off[j] += inc_q + inc_p + inc_n;
                if (s_q[j] >= a.Q) { s_q[j] -= a.Q; s_p[j] += 1; s_off[j] += wrap_q; }
                s_p[j] += dp;
                if (s_p[j] >= a.P) { s_p[j] -= a.P; s_off[j] += wrap_p; }
            }
        }
    };
    const bool slow_epilogue = wide || a.y_dt == HAWQ_S4;
    const int swz = (rho >> 2) & 3;
    auto compute = [&](int grp, const uint8_t *xs) {
        v16i acc[1][1], acc2[1][1];
#pragma unroll
        for (int i = 0; i < 16; ++i) { acc[0][0][i] = 0; acc2[0][0][i] = 0; }
        const int64_t mm[1] = {(int64_t)grp * 32 + rho};
        const bool valid[1] = {mm[0] < a.M};
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            const uint8_t *sub = xs + kc * 2048 + rho * 64;
            const v4i b0 = *(const v4i *)(sub + ((khalf ^ swz) << 4));
            const v4i b1 = *(const v4i *)(sub + (((2 + khalf) ^ swz) << 4));
            if (kc < KC1) {
                acc[0][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[kc][0], b0, acc[0][0], 0, 0, 0);
                acc[0][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[kc][1], b1, acc[0][0], 0, 0, 0);
            } else {
                acc2[0][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[kc][0], b0, acc2[0][0], 0, 0, 0);
                acc2[0][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[kc][1], b1, acc2[0][0], 0, 0, 0);
            }
        }
        epilogue_tile_dual<1, 1, 2, MID>(a, par_m[wave], par_s[wave], par_r[wave], mm, valid, k0, khalf * 16, acc, acc2, wide);
        if (slow_epilogue) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    };
    // outstanding-operation counts as in the kernel above, without shortcut loads
    auto arrive = [&](int it) {
        constexpr int L = (NS - 2) * DW;
        if (it == 0) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(L) : "memory");
        else if (it == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(L + S) : "memory");
        else if (it == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(L + 2 * S) : "memory");
        else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(L + 3 * S) : "memory");
        __builtin_amdgcn_s_barrier();
    };
    int grp = seq, it = 0;
    issue(grp, xs0);
    issue(grp + n_seq, xs1);
    issue(grp + 2 * n_seq, xs2);
#define HAWQ_PWSD_STEP(curx, nxtx)                   \
    arrive(it);                                      \
    issue(grp + 3 * n_seq, nxtx);                    \
    compute(grp, curx);                              \
    grp += n_seq;                                    \
    ++it;                                            \
    if (grp >= n_groups) break;
    while (grp < n_groups) {
        HAWQ_PWSD_STEP(xs0, xs3)
        HAWQ_PWSD_STEP(xs1, xs0)
        HAWQ_PWSD_STEP(xs2, xs1)
        HAWQ_PWSD_STEP(xs3, xs2)
    }
#undef HAWQ_PWSD_STEP
}

bool conv_pw_eligible(const ConvArgs &a, int x_hi) {
    if (!conv_mfma_eligible(a, x_hi)) return false;
    if (a.R != 1 || a.S != 1 || a.pad_h != 0 || a.pad_w != 0) return false;
    // measured: at C = 256 this form wins for narrow outputs (few channel tiles re-read the pixels); from
    // K = 256 on the tiled kernel is as fast or faster
    if (a.C != 64 && a.C != 128 && !(a.C == 256 && a.K <= 128)) return false;
    if (a.b == nullptr || a.y_dt == HAWQ_S32) return false;
    if (a.K % 16 != 0) return false;
    uintptr_t al = (uintptr_t)a.y | (uintptr_t)a.res;
    if (al & 15) return false;
    if (((uintptr_t)a.bias | (uintptr_t)a.b | (uintptr_t)a.res_b) & 3) return false;
    return (int64_t)a.M >= 8192;   // enough pixels for persistent waves to reach a steady state
}

template <int KC, int TP, int NS, int WPE, bool RES>
static hawq_status launch_pw_res(const ConvArgs &a, hipStream_t s) {
    const int n_ct = (a.K + 31) / 32;
    const int n_groups = (a.M + 32 * TP - 1) / (32 * TP);
    // fill every SIMD of the 256 CUs with as many waves as the register budget allows, each walking over
    // several pixel groups
    int n_seq = (WPE * 4 * 256 + n_ct - 1) / n_ct;
    if (n_seq > n_groups) n_seq = n_groups;
    const int waves = n_seq * n_ct;
    const uint32_t blocks = (uint32_t)((waves + 3) / 4);
    if (is4(a.x_dt)) conv_pw_kernel<KC, TP, NS, WPE, RES, true><<<blocks, 256, 0, s>>>(a, n_ct, n_seq, n_groups);
    else conv_pw_kernel<KC, TP, NS, WPE, RES, false><<<blocks, 256, 0, s>>>(a, n_ct, n_seq, n_groups);
    return check_launch();
}

template <int KC, int TP, int NS, int WPE>
static hawq_status launch_pw(const ConvArgs &a, hipStream_t s) {
    return a.res != nullptr ? launch_pw_res<KC, TP, NS, WPE, true>(a, s) : launch_pw_res<KC, TP, NS, WPE, false>(a, s);
}

bool conv_pws_eligible(const ConvArgs &a, int x_hi) {
    if (!conv_mfma_eligible(a, x_hi) || is4(a.x_dt)) return false;
    if (a.R != 1 || a.S != 1 || a.pad_h != 0 || a.pad_w != 0) return false;
    if (a.C != 256) return false;                        // measured: at C = 512 the tiled kernel is faster
    if (a.K % 128 != 0 || a.K < 256) return false;       // four channel tiles per workgroup share the pixels
    if (a.b == nullptr || a.y_dt == HAWQ_S32) return false;
    uintptr_t al = (uintptr_t)a.y | (uintptr_t)a.res;
    if (al & 15) return false;
    if (((uintptr_t)a.bias | (uintptr_t)a.b | (uintptr_t)a.res_b) & 3) return false;
    return (int64_t)a.M >= 8192;
}

template <int KC, int WPE>
static hawq_status launch_pws(const ConvArgs &a, hipStream_t s) {
    const int n_ct = a.K / 32;                           // a multiple of 4
    const int n_groups = (a.M + 31) / 32;
    int n_seq = (WPE * 4 * 256) / n_ct;
    if (n_seq < 1) n_seq = 1;
    if (n_seq > n_groups) n_seq = n_groups;
    const uint32_t blocks = (uint32_t)(n_seq * (n_ct / 4));   // exactly: every wave of the grid has work
    if (a.res != nullptr) conv_pws_kernel<KC, WPE, true><<<blocks, 256, 0, s>>>(a, n_ct, n_seq, n_groups);
    else conv_pws_kernel<KC, WPE, false><<<blocks, 256, 0, s>>>(a, n_ct, n_seq, n_groups);
    return check_launch();
}

bool conv_pws_dual_shape_ok(int C, int Cs, int K, int64_t M) {
    // (at (256, 512) the stage ring and the weight registers leave one workgroup per CU: the separate launches win)
    const bool pair = (C == 64 && Cs == 64) || (C == 128 && Cs == 256);
    return pair && K % 128 == 0 && K >= 256 && M >= 8192;
}

bool conv_pws_dual_eligible(const ConvArgs &a, int x_hi, int xs_hi) {
    if (a.xs == nullptr || a.res != nullptr || a.b == nullptr) return false;
    if (!conv_mfma_eligible(a, x_hi) || is4(a.x_dt)) return false;
    if (a.R != 1 || a.S != 1 || a.pad_h != 0 || a.pad_w != 0 || a.stride_h != 1 || a.stride_w != 1) return false;
    if (a.ws_dt != HAWQ_S8 || (a.xs_dt == HAWQ_U8 ? xs_hi > 127 : a.xs_dt != HAWQ_S8)) return false;
    if (!conv_pws_dual_shape_ok(a.C, a.Cs, a.K, a.M)) return false;
    if (a.y_dt == HAWQ_S32) return false;
    if (a.mid_s8 && (a.res_b == nullptr || a.res_c == nullptr)) return false;
    uintptr_t al = (uintptr_t)a.y | (uintptr_t)a.xs | (uintptr_t)a.ws;
    if (al & 15) return false;
    if (((uintptr_t)a.bias | (uintptr_t)a.b | (uintptr_t)a.bias_s | (uintptr_t)a.b_s | (uintptr_t)a.res_b) & 3) return false;
    return true;
}

template <int KC1, int KC2, int WPE>
static hawq_status launch_pws_dual(const ConvArgs &a, hipStream_t s) {
    const int n_ct = a.K / 32;                           // a multiple of 4
    const int n_groups = (a.M + 31) / 32;
    int n_seq = (WPE * 4 * 256) / n_ct;
    if (n_seq < 1) n_seq = 1;
    if (n_seq > n_groups) n_seq = n_groups;
    const uint32_t blocks = (uint32_t)(n_seq * (n_ct / 4));
    if (a.mid_s8) conv_pws_dual_kernel<KC1, KC2, WPE, true><<<blocks, 256, 0, s>>>(a, n_ct, n_seq, n_groups);
    else conv_pws_dual_kernel<KC1, KC2, WPE, false><<<blocks, 256, 0, s>>>(a, n_ct, n_seq, n_groups);
    return check_launch();
}

hawq_status launch_conv_pws_dual(const ConvArgs &a, hipStream_t s) {
    if (a.M == 0) return HAWQ_OK;
    if (a.C == 64) return launch_pws_dual<1, 1, 4>(a, s);
    return launch_pws_dual<2, 4, 2>(a, s);
}

hawq_status launch_conv_pws(const ConvArgs &a, hipStream_t s) {
    if (a.M == 0) return HAWQ_OK;
    // measured: three waves per SIMD (a fourth spills registers); with a shortcut two, whose register budget holds all of a
    // lane's epilogue parameters
    return a.res != nullptr ? launch_pws<4, 2>(a, s) : launch_pws<4, 3>(a, s);
}

hawq_status launch_conv_pw(const ConvArgs &a, hipStream_t s) {
    if (a.M == 0) return HAWQ_OK;
    // measured: at C = 64 one pixel tile per group and four waves per SIMD hide the epilogue's integer work
    // behind the memory stream best; at C = 128 two tiles per group (two waves per SIMD) are as good as any
    // deeper or wider arrangement
    // (with a shortcut: three waves per SIMD, whose register budget holds all of a lane's epilogue parameters -- 52 -> 47.5 us
    // for 56x56x64 -> 256 at batch 128 against four waves that read bias and shortcut multiplier from LDS)
    if (a.C == 64) return a.res != nullptr ? launch_pw<1, 1, 2, 3>(a, s) : launch_pw<1, 1, 2, 4>(a, s);
    if (a.C == 256) return launch_pw<4, 1, 2, 2>(a, s);
    return launch_pw<2, 2, 2, 2>(a, s);
}

}  // namespace hawq
