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

// ---------------------------------------------------------------------------------------------------
// conv1 fused with the 3x3/2 max pool that follows it in every ResNet.
//
// A workgroup produces a 7x8 tile of *pooled* pixels: it computes the 15x17 = 255 conv1 outputs under them
// (exactly eight 32-pixel MFMA tiles, two per wave; same scheme as above, from a 35x44-pixel input patch),
// requantises them with conv1's own epilogue into an LDS tile instead of HBM, and then takes the 3x3 maxima
// from LDS over the taps that lie inside the conv image.  The conv1 tensor (the largest of the network) is
// never written to or read from HBM.
constexpr int FUSE_PR = 7, FUSE_PC = 8;            // pooled tile: rows x columns
constexpr int FUSE_CR = 2 * FUSE_PR + 1;           // 15 conv rows
constexpr int FUSE_CC = 2 * FUSE_PC + 1;           // 17 conv columns
constexpr int FUSE_ROWS = 2 * FUSE_CR + 5;         // 35 input rows
constexpr int FUSE_COLS = 44;                      // patch width in pixels (origin = 4*pq0 - 5)
constexpr int FUSE_NPX = FUSE_CR * FUSE_CC;        // 255 conv pixels

__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3)))
conv_stem_pool_kernel(const ConvArgs a, const int pool_P, const int pool_Q, const int pool_y_dt, const int pool_lo,
                      const int pool_hi, uint8_t *__restrict__ pool_y, const int tiles_q, const int tiles_p) {
    __shared__ __attribute__((aligned(16))) uint8_t lw[STEM_W_BYTES];
    __shared__ __attribute__((aligned(16))) uint32_t lx[FUSE_ROWS * FUSE_COLS];
    __shared__ __attribute__((aligned(16))) uint8_t lc[256 * 64];   // requantised conv1 tile [pixel][channel]
    __shared__ ChanMain par_m[64];
    __shared__ ChanRes par_r[64];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int bid = blockIdx.x;
    const int tq = bid % tiles_q; bid /= tiles_q;
    const int tp_ = bid % tiles_p;
    const int n = bid / tiles_p;
    const int pp0 = tp_ * FUSE_PR, pq0 = tq * FUSE_PC;       // pooled tile origin
    const int cp0 = 2 * pp0 - 1, cq0 = 2 * pq0 - 1;          // conv tile origin (may be -1)

    for (int i = tid; i < STEM_W_BYTES / 16; i += 256) {
        const int row = i >> 4, ch = i & 15;
        *(v4i *)(lw + row * 256 + ((ch ^ (row & 15)) << 4)) = *(const v4i *)(a.w + i * 16);
    }
    // input patch: row rl <-> image row 2*cp0 - 3 + rl, column col <-> image column 2*cq0 - 3 + col;
    // groups of 4 pixels start at image column 4*pq0 - 8 + 4g, i.e. patch column 4g - 3
    const uint8_t *img = a.x + (int64_t)n * a.H * a.W * 3;
    for (int i = tid; i < FUSE_ROWS * 12; i += 256) {
        const int rl = i / 12, g = i - rl * 12;
        const int ih = 2 * cp0 - 3 + rl;
        const int iw = 4 * pq0 - 8 + 4 * g;
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
            const int col = 4 * g - 3 + k;
            if (col >= 0 && col < FUSE_COLS) lx[rl * FUSE_COLS + col] = px[k] ^ 0x00808080u;
        }
    }
    int wide = stage_params(a, 0, 64, par_m, par_r);
    wide = __syncthreads_or(wide);

    // ---- conv1 on the 255 pixels of the tile: wave w takes MFMA pixel tiles 2w and 2w+1 ----
    const int rho = lane & 31, khalf = lane >> 5;
    const int hsel = (rho >> 2) & 1, isel = (rho >> 3) * 4 + (rho & 3);
    int a_row[2];
#pragma unroll
    for (int tc = 0; tc < 2; ++tc) a_row[tc] = hsel * 32 + tc * 16 + isel;
    int b_base[2], ci[2];
#pragma unroll
    for (int tp = 0; tp < 2; ++tp) {
        ci[tp] = (2 * wave + tp) * 32 + rho;                       // 0..255; 255 is the one padding slot
        const int cix = ci[tp] < FUSE_NPX ? ci[tp] : 0;
        const int cr = cix / FUSE_CC, cc = cix - cr * FUSE_CC;
        b_base[tp] = (2 * cr) * FUSE_COLS + 2 * cc + 4 * khalf;
    }
    v16i acc[2][2];
#pragma unroll
    for (int tp = 0; tp < 2; ++tp)
#pragma unroll
        for (int tc = 0; tc < 2; ++tc)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[tp][tc][i] = 0;
#pragma unroll
    for (int r = 0; r < 7; ++r) {
        v4i af[2], bf[2];
#pragma unroll
        for (int tc = 0; tc < 2; ++tc) {
            const int row = a_row[tc];
            af[tc] = *(const v4i *)(lw + row * 256 + (((2 * r + khalf) ^ (row & 15)) << 4));
        }
#pragma unroll
        for (int tp = 0; tp < 2; ++tp) {
            const uint2 lo = *(const uint2 *)(lx + b_base[tp] + r * FUSE_COLS);
            const uint2 hi = *(const uint2 *)(lx + b_base[tp] + r * FUSE_COLS + 2);
            bf[tp] = (v4i){(int)lo.x, (int)lo.y, (int)hi.x, (int)hi.y};
        }
#pragma unroll
        for (int tp = 0; tp < 2; ++tp)
#pragma unroll
            for (int tc = 0; tc < 2; ++tc)
                acc[tp][tc] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[tc], bf[tp], acc[tp][tc], 0, 0, 0);
    }
    {
        ConvArgs lds_out = a;             // the epilogue stores into the LDS conv tile: [pixel][64 channels]
        lds_out.y = lc;
        lds_out.K = 64;
        const int64_t mm[2] = {ci[0], ci[1]};
        const bool valid[2] = {true, true};   // every slot is inside lc; out-of-image pixels are skipped when pooling
        const uint32_t none[2][2][4] = {};
        epilogue_tile<2, 2, false, true>(lds_out, par_m, par_r, mm, valid, 0, khalf * 32, acc, wide, none);
    }
    __syncthreads();

    // ---- 3x3/2 max pool out of LDS: thread = 16 channels of one pooled pixel ----
    const int g = tid & 3, j = (tid >> 2) & 7, i = tid >> 5;
    const int pp = pp0 + i, pq = pq0 + j;
    if (i >= FUSE_PR || pp >= pool_P || pq >= pool_Q) return;
    uint4 best = make_uint4(0, 0, 0, 0);   // unsigned data: zero is the identity of the maximum
#pragma unroll
    for (int dr = 0; dr < 3; ++dr) {
        const int cp = cp0 + 2 * i + dr;
        if ((unsigned)cp >= (unsigned)a.P) continue;
#pragma unroll
        for (int dc = 0; dc < 3; ++dc) {
            const int cq = cq0 + 2 * j + dc;
            if ((unsigned)cq >= (unsigned)a.Q) continue;
            const uint4 v = *(const uint4 *)(lc + ((2 * i + dr) * FUSE_CC + 2 * j + dc) * 64 + g * 16);
            best.x = max_u8x4(best.x, v.x); best.y = max_u8x4(best.y, v.y);
            best.z = max_u8x4(best.z, v.z); best.w = max_u8x4(best.w, v.w);
        }
    }
    const uint32_t wv[4] = {best.x, best.y, best.z, best.w};
    uint32_t ov[4], nib[2] = {0, 0};
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        uint32_t o = 0, h = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            int32_t v = (int32_t)((wv[d] >> (8 * e)) & 0xff);
            v = v < pool_lo ? pool_lo : (v > pool_hi ? pool_hi : v);
            o |= (uint32_t)(v & 0xff) << (8 * e);
            h |= (uint32_t)(v & 0xf) << (4 * e);
        }
        ov[d] = o;
        nib[d >> 1] |= h << (16 * (d & 1));
    }
    const int64_t oe = (((int64_t)n * pool_P + pp) * pool_Q + pq) * 64 + g * 16;
    if (is4(pool_y_dt)) *(uint2 *)(pool_y + (oe >> 1)) = make_uint2(nib[0], nib[1]);
    else *(uint4 *)(pool_y + oe) = make_uint4(ov[0], ov[1], ov[2], ov[3]);
}

hawq_status launch_conv_stem_pool(const ConvArgs &a, int pool_y_dt, int pool_lo, int pool_hi, void *pool_y, hipStream_t s) {
    if (a.M == 0) return HAWQ_OK;
    const int pool_P = (a.P - 1) / 2 + 1, pool_Q = (a.Q - 1) / 2 + 1;
    const int tiles_p = (pool_P + FUSE_PR - 1) / FUSE_PR, tiles_q = (pool_Q + FUSE_PC - 1) / FUSE_PC;
    const int64_t blocks = (int64_t)a.N * tiles_p * tiles_q;
    if (blocks > 0x7fffffff) return HAWQ_ERR_UNSUPPORTED;
    conv_stem_pool_kernel<<<(uint32_t)blocks, 256, 0, s>>>(a, pool_P, pool_Q, pool_y_dt, pool_lo, pool_hi, (uint8_t *)pool_y,
                                                           tiles_q, tiles_p);
    return check_launch();
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
