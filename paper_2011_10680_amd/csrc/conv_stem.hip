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
                      const int pool_hi, uint8_t *__restrict__ pool_y, const int tiles_q, const int tiles_p, const int n_tiles) {
    __shared__ __attribute__((aligned(16))) uint8_t lw[STEM_W_BYTES];
    __shared__ __attribute__((aligned(16))) uint32_t lx[FUSE_ROWS * FUSE_COLS];
    __shared__ __attribute__((aligned(16))) uint8_t lc[256 * 64];   // requantised conv1 tile [pixel][channel]
    __shared__ ChanMain par_m[64];
    __shared__ ChanRes par_r[64];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // The workgroup is persistent: weights and parameters are staged once, then it walks over tiles
    // blockIdx.x, + gridDim.x, ...; the raw input bytes of the next tile are fetched into registers while the
    // current tile is multiplied, requantised and pooled.
    for (int i = tid; i < STEM_W_BYTES / 16; i += 256) {
        const int row = i >> 4, ch = i & 15;
        *(v4i *)(lw + row * 256 + ((ch ^ (row & 15)) << 4)) = *(const v4i *)(a.w + i * 16);
    }
    int wide = stage_params(a, 0, 64, par_m, par_r);
    wide = __syncthreads_or(wide);

    // input patch of a tile: row rl <-> image row 2*cp0 - 3 + rl, column col <-> image column 2*cq0 - 3 + col;
    // groups of 4 pixels (12 bytes) start at image column 4*pq0 - 8 + 4g, i.e. patch column 4g - 3.  A thread
    // owns work items tid and tid + 256 of the FUSE_ROWS * 12 groups.
    constexpr int NITEM = (FUSE_ROWS * 12 + 255) / 256;
    uint32_t raw[NITEM][3];
    auto fetch = [&](int tile) {
        int t = tile;
        const int tq = t % tiles_q; t /= tiles_q;
        const int tp_ = t % tiles_p;
        const int n = t / tiles_p;
        const int cp0 = 2 * tp_ * FUSE_PR - 1, pq0 = tq * FUSE_PC;       // conv row origin, pooled column origin
        const uint8_t *img = a.x + (int64_t)n * a.H * a.W * 3;
#pragma unroll
        for (int it = 0; it < NITEM; ++it) {
            const int i = tid + it * 256;
            const int rl = i / 12, g = i - rl * 12;
            const int ih = 2 * cp0 - 3 + rl;
            const int iw = 4 * pq0 - 8 + 4 * g;
            raw[it][0] = raw[it][1] = raw[it][2] = 0;
            if (tile < n_tiles && i < FUSE_ROWS * 12 && (unsigned)ih < (unsigned)a.H && iw >= 0 && iw + 3 < a.W) {
                const uint32_t *src = (const uint32_t *)(img + ((int64_t)ih * a.W + iw) * 3);
                raw[it][0] = src[0]; raw[it][1] = src[1]; raw[it][2] = src[2];
            }
        }
    };
    // widen the fetched RGB triples to RGB0 dwords, offset by -128 (XOR 0x80 per byte), into the LDS patch;
    // out-of-image positions are raw zeros and get the same offset (the bias correction assumes it everywhere)
    auto stage = [&]() {
#pragma unroll
        for (int it = 0; it < NITEM; ++it) {
            const int i = tid + it * 256;
            const int rl = i / 12, g = i - rl * 12;
            const uint32_t d0 = raw[it][0], d1 = raw[it][1], d2 = raw[it][2];
            const uint32_t p0 = d0 & 0x00ffffffu;
            const uint32_t p1 = ((d0 >> 24) | (d1 << 8)) & 0x00ffffffu;
            const uint32_t p2 = ((d1 >> 16) | (d2 << 16)) & 0x00ffffffu;
            const uint32_t p3 = d2 >> 8;
            const int col = 4 * g - 3;          // -3, 1, 5, ... 41: patch columns col .. col + 3
            if (i < FUSE_ROWS * 12) {
                uint32_t *dst = lx + rl * FUSE_COLS + col;
                if (col >= 0) { dst[0] = p0 ^ 0x00808080u; dst[1] = p1 ^ 0x00808080u; dst[2] = p2 ^ 0x00808080u; }
                if (col + 3 < FUSE_COLS) dst[3] = p3 ^ 0x00808080u;
            }
        }
    };
    const int rho = lane & 31, khalf = lane >> 5;
    const int hsel = (rho >> 2) & 1, isel = (rho >> 3) * 4 + (rho & 3);
    int a_row[2];
#pragma unroll
    for (int tc = 0; tc < 2; ++tc) a_row[tc] = hsel * 32 + tc * 16 + isel;
    ConvArgs lds_out = a;             // the epilogue stores into the LDS conv tile: [pixel][64 channels]
    lds_out.y = lc;
    lds_out.K = 64;
    const int pg = tid & 3, pj = (tid >> 2) & 7, pi = tid >> 5;   // pool phase: 16 channels of one pooled pixel

    int tile = blockIdx.x;            // < n_tiles by construction of the grid
    fetch(tile);
    for (; tile < n_tiles; tile += gridDim.x) {
        int t = tile;
        const int tq = t % tiles_q; t /= tiles_q;
        const int tp_ = t % tiles_p;
        const int n = t / tiles_p;
        const int pp0 = tp_ * FUSE_PR, pq0 = tq * FUSE_PC;       // pooled tile origin
        const int cp0 = 2 * pp0 - 1, cq0 = 2 * pq0 - 1;          // conv tile origin (may be -1)
        stage();
        fetch(tile + gridDim.x);
        __syncthreads();              // patch complete; the previous tile's pool reads are done

        // ---- conv1 on the 255 pixels of the tile: wave w takes MFMA pixel tiles 2w and 2w+1, one after the
        // other (kept as a rolled loop: both at once would need twice the accumulators and spill) ----
#pragma nounroll
        for (int tp = 0; tp < 2; ++tp) {
            const int cidx = (2 * wave + tp) * 32 + rho;               // 0..255; 255 is the one padding slot
            const int cix = cidx < FUSE_NPX ? cidx : 0;
            const int cr = cix / FUSE_CC, cc = cix - cr * FUSE_CC;
            const int bb = (2 * cr) * FUSE_COLS + 2 * cc + 4 * khalf;
            v16i acc[1][2];
#pragma unroll
            for (int tc = 0; tc < 2; ++tc)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[0][tc][i] = 0;
#pragma unroll
            for (int r = 0; r < 7; ++r) {
                v4i af[2];
#pragma unroll
                for (int tc = 0; tc < 2; ++tc) {
                    const int row = a_row[tc];
                    af[tc] = *(const v4i *)(lw + row * 256 + (((2 * r + khalf) ^ (row & 15)) << 4));
                }
                const uint2 lo = *(const uint2 *)(lx + bb + r * FUSE_COLS);
                const uint2 hi = *(const uint2 *)(lx + bb + r * FUSE_COLS + 2);
                const v4i bf = (v4i){(int)lo.x, (int)lo.y, (int)hi.x, (int)hi.y};
#pragma unroll
                for (int tc = 0; tc < 2; ++tc)
                    acc[0][tc] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[tc], bf, acc[0][tc], 0, 0, 0);
            }
            const int64_t mm[1] = {cidx};
            const bool valid[1] = {true};   // every slot is inside lc; out-of-image pixels are skipped when pooling
            const uint32_t none[1][2][4] = {};
            epilogue_tile<2, 1, false, 1>(lds_out, par_m, par_r, mm, valid, 0, khalf * 32, acc, wide, none);
        }
        __syncthreads();              // conv tile complete; patch reads are done

        // ---- 3x3/2 max pool out of LDS ----
        const int pp = pp0 + pi, pq = pq0 + pj;
        if (pi < FUSE_PR && pp < pool_P && pq < pool_Q) {
            // running per-byte maxima, even and odd bytes kept apart (two 16-bit lanes each); unsigned data:
            // zero is the identity of the maximum
            uint32_t be[4] = {0, 0, 0, 0}, bo[4] = {0, 0, 0, 0};
#pragma unroll
            for (int dr = 0; dr < 3; ++dr) {
                const int cp = cp0 + 2 * pi + dr;
                if ((unsigned)cp >= (unsigned)a.P) continue;
#pragma unroll
                for (int dc = 0; dc < 3; ++dc) {
                    const int cq = cq0 + 2 * pj + dc;
                    if ((unsigned)cq >= (unsigned)a.Q) continue;
                    const int pix = (2 * pi + dr) * FUSE_CC + 2 * pj + dc;
                    // chunk swizzle of the tile (the exact general epilogue writes the plain layout)
                    const int chunk = wide ? pg : ((pg ^ (pix >> 2)) & 3);
                    const uint4 v = *(const uint4 *)(lc + pix * 64 + (chunk << 4));
                    const uint32_t vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        be[d] = pk_max_u16(be[d], vv[d] & 0x00ff00ffu);
                        bo[d] = pk_max_u16(bo[d], vv[d] & 0xff00ff00u);
                    }
                }
            }
            uint32_t ov[4], nib[2] = {0, 0};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                ov[d] = clamp_u8x4(be[d] | bo[d], (uint32_t)pool_lo, (uint32_t)pool_hi);
                // low nibbles of the four bytes -> 16 bits (only used for a packed 4-bit output, values <= 15)
                const uint32_t h = (ov[d] & 0xf) | ((ov[d] >> 4) & 0xf0) | ((ov[d] >> 8) & 0xf00) | ((ov[d] >> 12) & 0xf000);
                nib[d >> 1] |= h << (16 * (d & 1));
            }
            const int64_t oe = (((int64_t)n * pool_P + pp) * pool_Q + pq) * 64 + pg * 16;
            if (is4(pool_y_dt)) *(uint2 *)(pool_y + (oe >> 1)) = make_uint2(nib[0], nib[1]);
            else *(uint4 *)(pool_y + oe) = make_uint4(ov[0], ov[1], ov[2], ov[3]);
        }
    }
}

hawq_status launch_conv_stem_pool(const ConvArgs &a, int pool_y_dt, int pool_lo, int pool_hi, void *pool_y, hipStream_t s) {
    if (a.M == 0) return HAWQ_OK;
    const int pool_P = (a.P - 1) / 2 + 1, pool_Q = (a.Q - 1) / 2 + 1;
    const int tiles_p = (pool_P + FUSE_PR - 1) / FUSE_PR, tiles_q = (pool_Q + FUSE_PC - 1) / FUSE_PC;
    const int64_t n_tiles = (int64_t)a.N * tiles_p * tiles_q;
    if (n_tiles > 0x7fffffff) return HAWQ_ERR_UNSUPPORTED;
    const int64_t grid = n_tiles < 3 * 256 ? n_tiles : 3 * 256;    // persistent: three workgroups per CU
    // the pooled bytes are unsigned: bounds outside 0..255 never bind
    pool_lo = pool_lo < 0 ? 0 : pool_lo;
    pool_hi = pool_hi > 255 ? 255 : pool_hi;
    conv_stem_pool_kernel<<<(uint32_t)grid, 256, 0, s>>>(a, pool_P, pool_Q, pool_y_dt, pool_lo, pool_hi, (uint8_t *)pool_y,
                                                          tiles_q, tiles_p, (int)n_tiles);
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
