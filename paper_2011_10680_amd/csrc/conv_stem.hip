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
// conv1 fused with the 3x3/2 max pool that follows it in every ResNet: the conv1 tensor (the largest of the network) is
// never written to or read from HBM -- and never requantised either.  Requantisation (Section 3.1) and the clamps are
// non-decreasing in the accumulator for every multiplier the interface admits (b >= 0), so the maximum commutes with
// them exactly: the kernel takes the maximum over a window's INT32 accumulators (+ the channel's bias, the same for every
// pixel) and requantises once per *pooled* output, 4.5 times fewer quarter-rate 64-bit multiplies than conv1 has outputs.
//
// For that a pooling window's nine accumulators must meet in one lane.  The MFMA leaves a lane with one column and
// sixteen rows of the 32x32 result, so here the *pixels* are the row operand and the channels the column operand (the
// other way round from every other kernel of the library): lane (n, h) ends up with channel n and the sixteen pixels in
// rows {8j + 4h + q}.  Which conv1 pixel feeds which row is the kernel's choice: the sixteen rows of a lane half hold a
// block of 3 x 5 conv1 outputs (one slot spare) -- the windows of two horizontally adjacent pooled pixels, which share
// their middle column.  One MFMA tile thus yields four pooled pixels per channel; 15 conv1 outputs per two pooled pixels
// instead of the 9 of perfect sharing is 1.7 times the multiply-accumulates of the plain tiling, on matrix pipes that
// were one fifth busy, in exchange for a quarter of the vector arithmetic and no pooling pass over LDS.
//
// A workgroup (four waves) makes 8 x 8 tiles of pooled pixels from a 39 x 40 input patch staged once in LDS (pixels
// widened to RGB0 dwords; a filter row = 8 pixels x 4 B = one K = 32 MFMA step): sixteen MFMA tiles, four per wave.  The
// 64 x 7 x 32 weight bytes a lane needs as column operand (two channels) stay in registers for the life of the
// (persistent) workgroup.  Results go through a 4 KB LDS tile to become 16-byte NHWC stores.
constexpr int FUSE_PT = 8;                         // pooled tile edge
constexpr int FUSE_CT = 2 * FUSE_PT + 1;           // 17 conv rows / columns under it
constexpr int FUSE_ROWS = 2 * FUSE_CT + 5;         // 39 input rows
// patch width in pixels (41 used; origin = image column 4*pq0 - 5).  42: the 32 lanes of one pass of a fragment read touch
// three conv1 rows (two patch rows apart) x 18 consecutive dwords each; 2 x 42 = 20 (mod 64 banks) lays the three spans side
// by side, where 44 wrapped the third onto the first (every pass a two-way conflict: half of all LDS cycles)
constexpr int FUSE_COLS = 42;
constexpr int FUSE_GROUPS = 11;                    // 4-pixel groups fetched per patch row (patch columns -3 .. 40)

__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3)))
conv_stem_pool_kernel(const ConvArgs a, const int pool_P, const int pool_Q, const int pool_y_dt, const int pool_lo,
                      const int pool_hi, uint8_t *__restrict__ pool_y, const int tiles_q, const int tiles_p, const int n_tiles) {
    __shared__ __attribute__((aligned(16))) uint32_t lx[FUSE_ROWS * FUSE_COLS];
    __shared__ __attribute__((aligned(16))) uint8_t lp[FUSE_PT * FUSE_PT * 64];   // pooled tile [row][column][channel]
    __shared__ ChanMain par_m[64];
    __shared__ ChanRes par_r[64];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    int wide = stage_params(a, 0, 64, par_m, par_r);
    wide = __syncthreads_or(wide);
    // column operand: channel col + 32 tc, K-step r (filter row), this lane half's 16 bytes (filter columns 4 half .. + 3)
    v4i wf[7][2];
#pragma unroll
    for (int r = 0; r < 7; ++r)
#pragma unroll
        for (int tc = 0; tc < 2; ++tc) wf[r][tc] = *(const v4i *)(a.w + (((col + 32 * tc) * 8 + r) * 8 + 4 * half) * 4);
    // the two channels' requantisation: narrow form  high word of t * bs + Rs  (bias inside Rs), else the exact 64-bit form
    int32_t q_bs[2], q_b[2], q_c[2], q_bias[2];
    int64_t q_Rs[2];
#pragma unroll
    for (int tc = 0; tc < 2; ++tc) {
        const ChanMain m = par_m[col + 32 * tc];
        q_bs[tc] = m.bs; q_Rs[tc] = m.Rs; q_b[tc] = m.b; q_c[tc] = m.c; q_bias[tc] = m.bias;
    }

    // input patch of a tile: row rl <-> image row 4*pp0 - 5 + rl, column c <-> image column 4*pq0 - 5 + c; groups of 4
    // pixels (12 bytes) start at image column 4*pq0 - 8 + 4g, i.e. patch column 4g - 3.  A thread owns work items tid
    // and tid + 256 of the FUSE_ROWS * FUSE_GROUPS groups.
    constexpr int NITEM = (FUSE_ROWS * FUSE_GROUPS + 255) / 256;
    uint32_t raw[NITEM][3];
    auto fetch = [&](int tile) {
        int t = tile;
        const int tq = t % tiles_q; t /= tiles_q;
        const int tp_ = t % tiles_p;
        const int n = t / tiles_p;
        const uint8_t *img = a.x + (int64_t)n * a.H * a.W * 3;
#pragma unroll
        for (int it = 0; it < NITEM; ++it) {
            const int i = tid + it * 256;
            const int rl = i / FUSE_GROUPS, g = i - rl * FUSE_GROUPS;
            const int ih = 4 * tp_ * FUSE_PT - 5 + rl;
            const int iw = 4 * tq * FUSE_PT - 8 + 4 * g;
            raw[it][0] = raw[it][1] = raw[it][2] = 0;
            if (tile < n_tiles && i < FUSE_ROWS * FUSE_GROUPS && (unsigned)ih < (unsigned)a.H && iw >= 0 && iw + 3 < a.W) {
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
            const int rl = i / FUSE_GROUPS, g = i - rl * FUSE_GROUPS;
            const uint32_t d0 = raw[it][0], d1 = raw[it][1], d2 = raw[it][2];
            const uint32_t p0 = d0 & 0x00ffffffu;
            const uint32_t p1 = ((d0 >> 24) | (d1 << 8)) & 0x00ffffffu;
            const uint32_t p2 = ((d1 >> 16) | (d2 << 16)) & 0x00ffffffu;
            const uint32_t p3 = d2 >> 8;
            const int c0 = 4 * g - 3;          // -3, 1, 5, ... 37: patch columns c0 .. c0 + 3
            if (i < FUSE_ROWS * FUSE_GROUPS) {
                uint32_t *dst = lx + rl * FUSE_COLS + c0;
                if (c0 >= 0) { dst[0] = p0 ^ 0x00808080u; dst[1] = p1 ^ 0x00808080u; dst[2] = p2 ^ 0x00808080u; }
                dst[3] = p3 ^ 0x00808080u;
            }
        }
    };
    // row operand: MFMA row rho of a tile is slot 4 (rho >> 3) + (rho & 3) of the block of lane half (rho >> 2) & 1;
    // slot s < 15 is conv1 pixel (s / 5, s % 5) of the 3 x 5 block (slot 15 repeats slot 14 and is never looked at)
    const int a_h = (col >> 2) & 1;
    const int a_s = min(4 * (col >> 3) + (col & 3), 14);
    const int a_br = a_s / 5, a_bc = a_s - 5 * a_br;
    int32_t lo_c = a.lo, hi_c = a.hi, lo_p = pool_lo, hi_p = pool_hi;
    asm volatile("" : "+v"(lo_c), "+v"(hi_c), "+v"(lo_p), "+v"(hi_p));

    int tile = blockIdx.x;            // < n_tiles by construction of the grid
    fetch(tile);
    for (; tile < n_tiles; tile += gridDim.x) {
        int t = tile;
        const int tq = t % tiles_q; t /= tiles_q;
        const int tp_ = t % tiles_p;
        const int n = t / tiles_p;
        const int pp0 = tp_ * FUSE_PT, pq0 = tq * FUSE_PT;       // pooled tile origin
        stage();
        fetch(tile + gridDim.x);
        __syncthreads();              // patch complete; the previous tile's output reads are done

        // ---- wave w: MFMA tiles 4w .. 4w + 3, one after the other; tile wt = pooled row wt / 2 of the pooled tile, column
        // pairs 2 (wt % 2) and 2 (wt % 2) + 1 (lane halves 0 and 1) ----
#pragma nounroll
        for (int it = 0; it < 4; ++it) {
            const int wt = 4 * wave + it;
            const int pr = wt >> 1;
            {
                // the row this lane feeds: conv1 pixel (2 pr + br, 4 pcp + bc) of the 17 x 17 under the pooled tile
                const int pcp = 2 * (wt & 1) + a_h;
                const int bb = (2 * (2 * pr + a_br)) * FUSE_COLS + 2 * (4 * pcp + a_bc) + 4 * half;
                v16i acc[2];
#pragma unroll
                for (int tc = 0; tc < 2; ++tc)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[tc][i] = 0;
#pragma unroll
                for (int r = 0; r < 7; ++r) {   // the 8th K-step multiplies zero weights: skipped
                    const uint2 l0 = *(const uint2 *)(lx + bb + r * FUSE_COLS);
                    const uint2 h0 = *(const uint2 *)(lx + bb + r * FUSE_COLS + 2);
                    const v4i pf = (v4i){(int)l0.x, (int)l0.y, (int)h0.x, (int)h0.y};
#pragma unroll
                    for (int tc = 0; tc < 2; ++tc) acc[tc] = __builtin_amdgcn_mfma_i32_32x32x32_i8(pf, wf[r][tc], acc[tc], 0, 0, 0);
                }
                // ---- this lane: channels col, col + 32 of the block (pr, pcp = 2 (wt % 2) + half): two pooled pixels ----
                const int pcq = 2 * (2 * (wt & 1) + half);            // first pooled column of the block within the tile
                const int cr0 = 2 * (pp0 + pr) - 1, cq0 = 2 * (pq0 + pcq) - 1;   // conv1 coordinates of block pixel (0, 0)
                bool rv[3], cv[5];
                bool all = true;
#pragma unroll
                for (int i = 0; i < 3; ++i) { rv[i] = (unsigned)(cr0 + i) < (unsigned)a.P; all = all && rv[i]; }
#pragma unroll
                for (int i = 0; i < 5; ++i) { cv[i] = (unsigned)(cq0 + i) < (unsigned)a.Q; all = all && cv[i]; }
                if (!__all(all)) {   // a window reaches over the image's edge: those taps do not take part
#pragma unroll
                    for (int tc = 0; tc < 2; ++tc)
#pragma unroll
                        for (int i = 0; i < 15; ++i)
                            if (!(rv[i / 5] && cv[i % 5])) acc[tc][i] = INT32_MIN;
                }
                uint32_t yb[2][2];
#pragma unroll
                for (int tc = 0; tc < 2; ++tc) {
                    // columns 0..2 -> first pooled pixel, 2..4 -> second; the shared middle column once
                    const int32_t mid = max(acc[tc][2], max(acc[tc][7], acc[tc][12]));
                    int32_t m0 = max(max(acc[tc][0], acc[tc][1]), max(acc[tc][5], acc[tc][6]));
                    m0 = max(max(m0, mid), max(acc[tc][10], acc[tc][11]));
                    int32_t m1 = max(max(acc[tc][3], acc[tc][4]), max(acc[tc][8], acc[tc][9]));
                    m1 = max(max(m1, mid), max(acc[tc][13], acc[tc][14]));
                    const int32_t mm[2] = {m0, m1};
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        int32_t y;
                        // (wrapping sum: a pooled pixel outside the tensor carries INT32_MIN and is never stored)
                        if (wide) y = clamp64(rq64((int32_t)((uint32_t)mm[j] + (uint32_t)q_bias[tc]), q_b[tc], q_c[tc]), lo_c, hi_c);
                        else {
                            const int32_t v = (int32_t)(((int64_t)mm[j] * (int64_t)q_bs[tc] + q_Rs[tc]) >> 32);
                            asm("v_med3_i32 %0, %1, %2, %3" : "=v"(y) : "v"(v), "v"(lo_c), "v"(hi_c));
                        }
                        int32_t z;
                        asm("v_med3_i32 %0, %1, %2, %3" : "=v"(z) : "v"(y), "v"(lo_p), "v"(hi_p));
                        yb[tc][j] = (uint32_t)z;
                    }
                }
#pragma unroll
                for (int tc = 0; tc < 2; ++tc)
#pragma unroll
                    for (int j = 0; j < 2; ++j) lp[(pr * FUSE_PT + pcq + j) * 64 + col + 32 * tc] = (uint8_t)yb[tc][j];
            }
        }
        __syncthreads();              // pooled tile complete; patch reads are done

        // ---- 16 channels of one pooled pixel per thread: 16-byte NHWC stores ----
        {
            const int pg = tid & 3, pi = tid >> 2;
            const int pp = pp0 + (pi >> 3), pq = pq0 + (pi & 7);
            if (pp < pool_P && pq < pool_Q) {
                const uint4 v = *(const uint4 *)(lp + pi * 64 + pg * 16);
                const int64_t oe = (((int64_t)n * pool_P + pp) * pool_Q + pq) * 64 + pg * 16;
                if (is4(pool_y_dt)) {
                    // low nibbles of the four bytes of a dword -> 16 bits (values <= 15 by the clamp)
                    auto nib = [](uint32_t d) { return (d & 0xfu) | ((d >> 4) & 0xf0u) | ((d >> 8) & 0xf00u) | ((d >> 12) & 0xf000u); };
                    *(uint2 *)(pool_y + (oe >> 1)) = make_uint2(nib(v.x) | (nib(v.y) << 16), nib(v.z) | (nib(v.w) << 16));
                } else {
                    *(uint4 *)(pool_y + oe) = v;
                }
            }
        }
    }
}

hawq_status launch_conv_stem_pool(const ConvArgs &a, int pool_y_dt, int pool_lo, int pool_hi, void *pool_y, hipStream_t s) {
    if (a.M == 0) return HAWQ_OK;
    const int pool_P = (a.P - 1) / 2 + 1, pool_Q = (a.Q - 1) / 2 + 1;
    const int tiles_p = (pool_P + FUSE_PT - 1) / FUSE_PT, tiles_q = (pool_Q + FUSE_PT - 1) / FUSE_PT;
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
