// Pointwise (1x1) quantised convolution for shallow reductions (C = 64 or 128), streaming form.
//
// These layers (the expanding 1x1 of a bottleneck with its residual, the stride-1 transition
// convolution, the first reducing 1x1) do a handful of MFMAs per output tile and are bound by HBM
// traffic and by the integer epilogue.  A tile-per-workgroup kernel spends its life in start-up
// latency there.  Here a wave is persistent instead: it keeps the weights of its 32 output channels in
// registers (they are only C/8 registers per lane) and its channels' requantisation parameters in a
// wave-private LDS slot, then walks over pixel tiles with the next tile's activations and shortcut
// bytes already in flight while the current tile is multiplied, requantised and stored.  No
// workgroup barrier, no LDS staging of operands; every activation byte is fetched straight into the
// MFMA operand layout.
#include "common.h"
#include "epilogue.h"

namespace hawq {

// KC: 64-element chunks of the reduction (C / 64); TP: 32-pixel tiles per group; NS: groups in flight per wave
// (ring of register stages); WPE: waves per SIMD the register allocation is held to.
template <int KC, int TP, int NS, int WPE, bool INT4>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(WPE)))
conv_pw_kernel(const ConvArgs a, const int n_ct, const int n_seq, const int n_groups) {
    constexpr int BKB = INT4 ? 32 : 64;             // bytes of 64 reduction elements in memory
    constexpr int NL = INT4 ? 1 : 2;                // 16-byte loads per lane per 64 elements
    constexpr uint32_t kInvalid = 0x80000000u;
    __shared__ ChanMain par_m[4][32];
    __shared__ ChanRes par_r[4][32];

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

    const bool has_res = a.res != nullptr;
    const bool r4 = is4(a.res_dt);
    const __amdgpu_buffer_rsrc_t rsrc_r = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(has_res ? a.res : a.x), 0, has_res ? (int)tensor_bytes((int64_t)a.M * a.K, a.res_dt) : 0, 0x00020000);
    const bool unit = a.stride_h == 1 && a.stride_w == 1;   // 1x1, no padding: output pixel m reads input pixel m
    const int PQ = a.P * a.Q;

    // raw operand loads of one group of TP pixel tiles (NL x 16 bytes per 64 elements) and its shortcut bytes
    struct Stage {
        v4i b[TP][KC][NL];
        uint32_t r[TP][1][4];
    };
    auto issue = [&](int grp, Stage &st) {
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) {
            const int64_t m = ((int64_t)grp * TP + tp) * 32 + rho;
            const bool ok = grp < n_groups && m < a.M;
            uint32_t off = kInvalid;
            if (ok) {
                if (unit) {
                    off = (uint32_t)m * (uint32_t)Cb;
                } else {
                    const int mi = (int)m;
                    const int n = mi / PQ, pq = mi - n * PQ;
                    const int p = pq / a.Q, q = pq - p * a.Q;
                    off = (uint32_t)(((n * a.H + p * a.stride_h) * a.W + q * a.stride_w) * Cb);
                }
            }
#pragma unroll
            for (int kc = 0; kc < KC; ++kc)
#pragma unroll
                for (int l = 0; l < NL; ++l)
                    st.b[tp][kc][l] = __builtin_amdgcn_raw_buffer_load_b128(
                        rsrc_x, (int)(off + kc * BKB + (INT4 ? khalf * 16 : l * 32 + khalf * 16)), 0, 0);
            st.r[tp][0][0] = st.r[tp][0][1] = st.r[tp][0][2] = st.r[tp][0][3] = 0;
            if (has_res) {
                // the lane's 16 channels of pixel m: 16 bytes (8 for 4-bit data)
                const int64_t e = m * (int64_t)a.K + k0 + khalf * 16;
                const uint32_t ro = (ok && k0 + khalf * 16 < a.K) ? (uint32_t)(r4 ? (e >> 1) : e) : kInvalid;
                if (r4) {
                    const uint2 t = __builtin_bit_cast(uint2, __builtin_amdgcn_raw_buffer_load_b64(rsrc_r, (int)ro, 0, 0));
                    st.r[tp][0][0] = t.x; st.r[tp][0][1] = t.y; st.r[tp][0][2] = 0; st.r[tp][0][3] = 0;
                } else {
                    const v4i t = __builtin_amdgcn_raw_buffer_load_b128(rsrc_r, (int)ro, 0, 0);
                    st.r[tp][0][0] = (uint32_t)t[0]; st.r[tp][0][1] = (uint32_t)t[1];
                    st.r[tp][0][2] = (uint32_t)t[2]; st.r[tp][0][3] = (uint32_t)t[3];
                }
            }
        }
    };

    auto process = [&](int grp, const Stage &st) {
        v16i acc[TP][1];
        int64_t mm[TP];
        bool valid[TP];
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[tp][0][i] = 0;
            mm[tp] = ((int64_t)grp * TP + tp) * 32 + rho;
            valid[tp] = mm[tp] < a.M;
        }
#pragma unroll
        for (int tp = 0; tp < TP; ++tp)
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) {
                v4i b0, b1;
                if (INT4) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint32_t u = (uint32_t)st.b[tp][kc][0][e];
                        b0[e] = (int)(u & 0x0F0F0F0Fu);
                        b1[e] = (int)((u >> 4) & 0x0F0F0F0Fu);
                    }
                } else {
                    b0 = st.b[tp][kc][0];
                    b1 = st.b[tp][kc][NL - 1];
                }
                acc[tp][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[kc][0], b0, acc[tp][0], 0, 0, 0);
                acc[tp][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[kc][1], b1, acc[tp][0], 0, 0, 0);
            }
        epilogue_tile<1, TP, true>(a, par_m[wave], par_r[wave], mm, valid, k0, khalf * 16, acc, wide, st.r);
    };

    // NS - 1 groups in flight: while group i is processed, groups i + n_seq .. i + (NS-1) n_seq are landing
    // (issue() past the last group presents out-of-range offsets and fetches nothing)
    static_assert(NS >= 2 && NS <= 4, "ring depth");
    Stage st0, st1, st2, st3;   // separate objects, named explicitly, so that each stays in registers
    int grp = seq;
    issue(grp, st0);
    if constexpr (NS >= 3) issue(grp + n_seq, st1);
    if constexpr (NS >= 4) issue(grp + 2 * n_seq, st2);
#define HAWQ_PW_STEP(cur, nxt)                      \
    issue(grp + (NS - 1) * n_seq, nxt);             \
    process(grp, cur);                              \
    grp += n_seq;                                   \
    if (grp >= n_groups) break;
    while (grp < n_groups) {
        if constexpr (NS == 2) {
            HAWQ_PW_STEP(st0, st1)
            HAWQ_PW_STEP(st1, st0)
        } else if constexpr (NS == 3) {
            HAWQ_PW_STEP(st0, st2)
            HAWQ_PW_STEP(st1, st0)
            HAWQ_PW_STEP(st2, st1)
        } else {
            HAWQ_PW_STEP(st0, st3)
            HAWQ_PW_STEP(st1, st0)
            HAWQ_PW_STEP(st2, st1)
            HAWQ_PW_STEP(st3, st2)
        }
    }
#undef HAWQ_PW_STEP
}

bool conv_pw_eligible(const ConvArgs &a, int x_hi) {
    if (!conv_mfma_eligible(a, x_hi)) return false;
    if (a.R != 1 || a.S != 1 || a.pad_h != 0 || a.pad_w != 0) return false;
    if (a.C != 64 && a.C != 128) return false;   // measured: at C = 256 the tiled kernel is as fast or faster
    if (a.b == nullptr || a.y_dt == HAWQ_S32) return false;
    if (a.K % 16 != 0) return false;
    uintptr_t al = (uintptr_t)a.y | (uintptr_t)a.res;
    if (al & 15) return false;
    if (((uintptr_t)a.bias | (uintptr_t)a.b | (uintptr_t)a.res_b) & 3) return false;
    return (int64_t)a.M >= 8192;   // enough pixels for persistent waves to reach a steady state
}

template <int KC, int TP, int NS, int WPE>
static hawq_status launch_pw(const ConvArgs &a, hipStream_t s) {
    const int n_ct = (a.K + 31) / 32;
    const int n_groups = (a.M + 32 * TP - 1) / (32 * TP);
    // fill every SIMD of the 256 CUs with as many waves as the register budget allows, each walking over
    // several pixel groups
    int n_seq = (WPE * 4 * 256 + n_ct - 1) / n_ct;
    if (n_seq > n_groups) n_seq = n_groups;
    const int waves = n_seq * n_ct;
    const uint32_t blocks = (uint32_t)((waves + 3) / 4);
    if (is4(a.x_dt)) conv_pw_kernel<KC, TP, NS, WPE, true><<<blocks, 256, 0, s>>>(a, n_ct, n_seq, n_groups);
    else conv_pw_kernel<KC, TP, NS, WPE, false><<<blocks, 256, 0, s>>>(a, n_ct, n_seq, n_groups);
    return check_launch();
}

hawq_status launch_conv_pw(const ConvArgs &a, hipStream_t s) {
    if (a.M == 0) return HAWQ_OK;
    // measured: at C = 64 one pixel tile per group and four waves per SIMD hide the epilogue's integer work
    // behind the memory stream best; at C = 128 two tiles per group (two waves per SIMD) are as good as any
    // deeper or wider arrangement
    if (a.C == 64) return launch_pw<1, 1, 2, 4>(a, s);
    return launch_pw<2, 2, 2, 2>(a, s);
}

}  // namespace hawq
