// First layer of the networks: 7x7 stride-2 pad-3 convolution of a 3-channel uint8 image to 64
// channels (Appendix H keeps this layer at 8 bits), on the INT8 matrix cores.
//
// The image holds 0..255, which does not fit the signed INT8 operand.  The kernel feeds x - 128
// (x XOR 0x80) and the host adds 128 * sum(w[k]) to the bias; out-of-image taps are filled with
// raw 0, i.e. -128 after the offset, so the correction is the same at every pixel.  Exact.
//
// K layout: pixels are widened to 4 bytes (RGB0) while staging, a filter row becomes 8 pixels x
// 4 bytes = 32 bytes = one 32x32x32 MFMA K-step, and the 7 rows plus one zero row give K = 256.
// Weights arrive re-tiled by the host as [64][8][8][4] with zeros in the padding positions.
// A workgroup computes a 16x16 tile of output pixels for all 64 channels from a 37x40-pixel
// input patch staged once in LDS; each input byte is read from HBM once per workgroup.
#include "common.h"
#include "epilogue.h"

namespace hawq {

constexpr int STEM_TILE = 16;                    // output tile edge
constexpr int STEM_ROWS = 2 * STEM_TILE + 5;     // 37 input rows
constexpr int STEM_COLS = 40;                    // patch width in pixels (38 used), origin = 2*q0 - 3
constexpr int STEM_W_BYTES = 64 * 256;

__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3))) conv_stem_kernel(const ConvArgs a, const int tiles_q, const int tiles_p) {
    __shared__ __attribute__((aligned(16))) uint8_t lw[STEM_W_BYTES];
    __shared__ __attribute__((aligned(16))) uint32_t lx[STEM_ROWS * STEM_COLS];
    __shared__ ChanMain par_m[64];
    __shared__ ChanRes par_r[64];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int bid = blockIdx.x;
    const int tq = bid % tiles_q; bid /= tiles_q;
    const int tp_ = bid % tiles_p;
    const int n = bid / tiles_p;
    const int p0 = tp_ * STEM_TILE, q0 = tq * STEM_TILE;

    // ---- stage weights: 1024 16-byte chunks, swizzled by channel ----
    for (int i = tid; i < STEM_W_BYTES / 16; i += 256) {
        const int row = i >> 4, ch = i & 15;
        *(v4i *)(lw + row * 256 + ((ch ^ (row & 15)) << 4)) = *(const v4i *)(a.w + i * 16);
    }
    // ---- stage the input patch: groups of 4 pixels (12 bytes, dword aligned) -> 4 RGB0 dwords ----
    const uint8_t *img = a.x + (int64_t)n * a.H * a.W * 3;
    for (int i = tid; i < STEM_ROWS * 10; i += 256) {
        const int rl = i / 10, g = i - rl * 10;
        const int ih = 2 * p0 - 3 + rl;
        const int iw = 2 * q0 - 4 + 4 * g;       // first pixel of the group; patch column = 4g - 1
        uint32_t px[4] = {0, 0, 0, 0};
        if ((unsigned)ih < (unsigned)a.H && iw >= 0 && iw + 3 < a.W) {
            const uint32_t *src = (const uint32_t *)(img + ((int64_t)ih * a.W + iw) * 3);
            const uint32_t d0 = src[0], d1 = src[1], d2 = src[2];
            px[0] = d0 & 0x00ffffffu;
            px[1] = ((d0 >> 24) | (d1 << 8)) & 0x00ffffffu;
            px[2] = ((d1 >> 16) | (d2 << 16)) & 0x00ffffffu;
            px[3] = d2 >> 8;
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int col = 4 * g - 1 + k;
            if (col >= 0 && col < STEM_COLS) lx[rl * STEM_COLS + col] = px[k] ^ 0x00808080u;
        }
    }
    const bool tile_epi = a.y_dt != HAWQ_S32;
    int wide = 0;
    if (tile_epi) wide = stage_params(a, 0, 64, par_m, par_r);
    wide = __syncthreads_or(wide);

    // ---- MFMA: wave w owns output rows 4w..4w+3 of the tile (2 pixel tiles of 2 rows x 16 cols) ----
    const int rho = lane & 31, khalf = lane >> 5;
    const int hsel = (rho >> 2) & 1, isel = (rho >> 3) * 4 + (rho & 3);
    int a_row[2];
#pragma unroll
    for (int tc = 0; tc < 2; ++tc) a_row[tc] = hsel * 32 + tc * 16 + isel;
    int b_base[2];
#pragma unroll
    for (int tp = 0; tp < 2; ++tp) {
        const int pr = wave * 4 + tp * 2 + (rho >> 4), pc = rho & 15;
        b_base[tp] = (2 * pr) * STEM_COLS + 2 * pc + 4 * khalf;   // dword index; K-step r adds r*STEM_COLS
    }
    v16i acc[2][2];
#pragma unroll
    for (int tp = 0; tp < 2; ++tp)
#pragma unroll
        for (int tc = 0; tc < 2; ++tc)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[tp][tc][i] = 0;

#pragma unroll
    for (int r = 0; r < 7; ++r) {   // the 8th K-step multiplies zero weights: skipped
        v4i af[2], bf[2];
#pragma unroll
        for (int tc = 0; tc < 2; ++tc) {
            const int row = a_row[tc];
            af[tc] = *(const v4i *)(lw + row * 256 + (((2 * r + khalf) ^ (row & 15)) << 4));
        }
#pragma unroll
        for (int tp = 0; tp < 2; ++tp) {
            const uint2 lo = *(const uint2 *)(lx + b_base[tp] + r * STEM_COLS);
            const uint2 hi = *(const uint2 *)(lx + b_base[tp] + r * STEM_COLS + 2);
            bf[tp] = (v4i){(int)lo.x, (int)lo.y, (int)hi.x, (int)hi.y};
        }
#pragma unroll
        for (int tp = 0; tp < 2; ++tp)
#pragma unroll
            for (int tc = 0; tc < 2; ++tc)
                acc[tp][tc] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[tc], bf[tp], acc[tp][tc], 0, 0, 0);
    }

    const int ch0 = khalf * 32;
    if (tile_epi) {
        int64_t mm[2];
        bool valid[2];
#pragma unroll
        for (int tp = 0; tp < 2; ++tp) {
            const int p = p0 + wave * 4 + tp * 2 + (rho >> 4), q = q0 + (rho & 15);
            valid[tp] = p < a.P && q < a.Q;
            mm[tp] = ((int64_t)n * a.P + p) * a.Q + q;
        }
        const uint32_t none[2][2][4] = {};
        epilogue_tile<2, 2, false>(a, par_m, par_r, mm, valid, 0, ch0, acc, wide, none);
        return;
    }
    static_for<0, 2>([&](auto tpc) {
        constexpr int tp = decltype(tpc)::value;
        const int p = p0 + wave * 4 + tp * 2 + (rho >> 4), q = q0 + (rho & 15);
        if (p >= a.P || q >= a.Q) return;
        const int64_t m = ((int64_t)n * a.P + p) * a.Q + q;
        epilogue_pixel<2, true>(a, m, ch0, acc[tp]);
    });
}

// Re-tile [64][7][7][3] int8 weights to [64][8][8][4] (zeros in the padding) -- host helper.
void stem_pack_weights(const int8_t *w, int8_t *out) {
    for (int k = 0; k < 64; ++k)
        for (int r = 0; r < 8; ++r)
            for (int s = 0; s < 8; ++s)
                for (int c = 0; c < 4; ++c)
                    out[((k * 8 + r) * 8 + s) * 4 + c] = (r < 7 && s < 7 && c < 3) ? w[((k * 7 + r) * 7 + s) * 3 + c] : 0;
}

bool conv_stem_eligible(const ConvArgs &a) {
    return a.C == 3 && a.K == 64 && a.R == 7 && a.S == 7 && a.stride_h == 2 && a.stride_w == 2 && a.pad_h == 3 &&
           a.pad_w == 3 && a.x_dt == HAWQ_U8 && a.w_dt == HAWQ_S8 && a.W % 4 == 0 && a.res == nullptr && a.b != nullptr &&
           (((uintptr_t)a.x | (uintptr_t)a.w | (uintptr_t)a.y | (uintptr_t)a.bias | (uintptr_t)a.b) & 15) == 0 &&
           ((uintptr_t)a.c & 3) == 0;
}

hawq_status launch_conv_stem(const ConvArgs &a, hipStream_t s) {
    if (a.M == 0) return HAWQ_OK;
    const int tiles_p = (a.P + STEM_TILE - 1) / STEM_TILE, tiles_q = (a.Q + STEM_TILE - 1) / STEM_TILE;
    const int64_t blocks = (int64_t)a.N * tiles_p * tiles_q;
    if (blocks > 0x7fffffff) return HAWQ_ERR_UNSUPPORTED;
    conv_stem_kernel<<<(uint32_t)blocks, 256, 0, s>>>(a, tiles_q, tiles_p);
    return check_launch();
}

}  // namespace hawq
