// 3x3, stride 1, pad 1 quantised convolution with 64 input and 64 output channels (INT8 operands): the
// integer convolution of Section 3.1 for the widest-image 3x3 layers of the ResNets (56x56 at 224 input).
//
// These layers have the lowest arithmetic intensity of all 3x3 convolutions (64 channels per pixel) and the
// general implicit-GEMM kernel spends its time moving operands: per 64-channel K-step it fetches a weight
// tile and a pixel tile through the CU's vector-memory path, which is slower than the step's MFMAs.  Here
//   * all 9 x 64 x 64 weights (36 KB) stay in LDS for the life of a persistent workgroup;
//   * for this filter shape output pixel m (flat index over n, p, q) reads input pixel  m + (r-1) W + (s-1)
//     for tap (r, s), so the nine pixel operands of a 128-pixel tile are nine shifted windows of one run of
//     128 + 2W + 2 input pixels (the "patch"), fetched once per tile by LDS-DMA into a double buffer; taps
//     that fall into the zero padding are redirected, per lane, to a zero-filled row of the patch buffer;
//   * there is one workgroup barrier per tile (the patch's arrival), none per K-step.
// A workgroup is four waves; a wave multiplies all 64 channels by 32 pixels of the tile (36 MFMAs), then
// requantises and stores its 64 x 32 outputs with the shared epilogue while the next patch is in flight.
#include "common.h"
#include "epilogue.h"

namespace hawq {

// RES: a shortcut is added.  INT4: packed 4-bit operands -- the weights are expanded to INT8 once, while they are
// staged into LDS; the pixels stay packed in the patch (32-byte rows) and are split into nibbles when a fragment
// is read: the low nibbles of a lane's 16 bytes form the first-half MFMA operand, the high nibbles the second
// half, and the weight staging applies the same split, which leaves every dot product unchanged.
template <bool RES, bool INT4>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2)))
conv3x3_c64_kernel(const ConvArgs a, const int n_tiles) {
    constexpr int BP = 128;                     // pixels per tile
    constexpr int PROWS = 256;                  // patch rows (input pixels) a patch buffer holds
    constexpr int ROWB = INT4 ? 32 : 64;        // bytes of a pixel (64 channels) in memory and in the patch
    constexpr int RPI = 1024 / ROWB;            // patch rows one fetch instruction (1 KB) fills
    constexpr int NPW = PROWS / RPI / 4;        // patch fetch instructions per wave
    constexpr int PB = PROWS * ROWB;
    constexpr int TC = 2, TP = 1;
    constexpr int R = RES ? TC * TP : 0, S = TC * TP;   // shortcut loads / stores per lane and tile (16 bytes each)
    constexpr uint32_t kInvalid = 0x80000000u;

    __shared__ __attribute__((aligned(1024))) uint8_t wl[9 * 64 * 64];      // weights: 9 taps x [64 channels][64 B]
    __shared__ __attribute__((aligned(1024))) uint8_t pa[PB];               // patch buffer, even tiles
    __shared__ __attribute__((aligned(1024))) uint8_t pb[PB];               // patch buffer, odd tiles
    __shared__ ChanMain par_m[64];
    __shared__ ChanRes par_r[64];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int W = a.W, HW = a.H * a.W;
    const int n_in = a.N * HW;                  // input pixels = output pixels
    const int prows = BP + 2 * W + 2;           // rows in use (<= PROWS - 1, checked by the host)

    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void *)a.w, 0, 64 * 9 * ROWB, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, n_in * ROWB, 0x00020000);
    constexpr bool has_res = RES;
    const bool r4 = is4(a.res_dt);
    const __amdgpu_buffer_rsrc_t rsrc_r = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(has_res ? a.res : a.x), 0, has_res ? (int)tensor_bytes((int64_t)a.M * 64, a.res_dt) : 0, 0x00020000);

    // ---- weights -> LDS, once: instruction j of wave w fills 1 KB = 16 channels of one tap; lane i writes chunk
    // i of that KB and therefore fetches the chunk the XOR swizzle places there ----
    if constexpr (!INT4) {
        const int row16 = lane >> 2;
#pragma unroll
        for (int j = 0; j < 9; ++j) {
            const int inst = wave + 4 * j;                 // 0..35: tap = inst / 4, channel quarter = inst % 4
            const int tap = inst >> 2, k = (inst & 3) * 16 + row16;
            const int ch = (lane & 3) ^ ((k >> 2) & 3);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rsrc_w, (__attribute__((address_space(3))) void *)(wl + inst * 1024), 16, k * 576 + tap * 64 + ch * 16, 0, 0, 0);
        }
    } else {
        // packed weights: a thread takes 16 packed bytes (half a tap row of one channel: the bytes a lane half
        // `kh` multiplies), expands them to the two 16-byte INT8 chunks (kk = 0: low nibbles, kk = 1: high nibbles,
        // sign-extended) and writes them where the INT8 layout keeps chunk 2 kk + kh
        for (int i = tid; i < 9 * 64 * 2; i += 256) {
            const int kh = i & 1, k = (i >> 1) & 63, tap = i >> 7;
            const v4i v = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, k * 288 + tap * 32 + kh * 16, 0, 0);
            v4i lo, hi;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t u = (uint32_t)v[e];
                uint32_t l = u & 0x0F0F0F0Fu, h = (u >> 4) & 0x0F0F0F0Fu;
                l |= (l & 0x08080808u) * 0x1Eu;
                h |= (h & 0x08080808u) * 0x1Eu;
                lo[e] = (int)l; hi[e] = (int)h;
            }
            const int sw = (k >> 2) & 3;
            *(v4i *)(wl + tap * 4096 + k * 64 + ((kh ^ sw) << 4)) = lo;
            *(v4i *)(wl + tap * 4096 + k * 64 + (((2 + kh) ^ sw) << 4)) = hi;
        }
    }
    int wide = stage_params(a, 0, 64, par_m, par_r);

    // ---- patch fetch: patch row j of tile t is flat input pixel  t*BP - W - 1 + j ----
    // (INT8: 64-byte rows, four lanes per row, chunks XOR-swizzled; INT4: 32-byte rows, two lanes per row, plain)
    const int p_row0 = INT4 ? lane >> 1 : lane >> 2;
    auto fetch_patch = [&](int tile, uint8_t *buf) {
        const int f0 = tile * BP - W - 1;
#pragma unroll
        for (int jj = 0; jj < NPW; ++jj) {
            const int inst = wave + 4 * jj;
            const int row = inst * RPI + p_row0;
            const int ch = INT4 ? (lane & 1) : ((lane & 3) ^ ((row >> 2) & 3));
            const int f = f0 + row;
            const bool ok = tile < n_tiles && row < prows && f >= 0 && f < n_in;   // other rows are filled with zeros
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rsrc_x, (__attribute__((address_space(3))) void *)(buf + inst * 1024), 16,
                ok ? f * ROWB + ch * 16 : (int)kInvalid, 0, 0, 0);
        }
    };
    // shortcut bytes of the lane's outputs of a tile (16 channels per load; 4-bit data uses the first 8 bytes)
    const int rho = lane & 31, khalf = lane >> 5;
    const int chl = khalf * 16 * TC;            // the lane's first channel
    auto fetch_res = [&](int tile, uint32_t (&rw)[TP][TC][4]) {
        const int64_t m = (int64_t)tile * BP + wave * 32 + rho;
#pragma unroll
        for (int tc = 0; tc < TC; ++tc) {
            const int64_t e = m * 64 + chl + 16 * tc;
            const uint32_t ro = (tile < n_tiles && m < a.M) ? (uint32_t)(r4 ? (e >> 1) : e) : kInvalid;
            const v4i t = __builtin_amdgcn_raw_buffer_load_b128(rsrc_r, (int)ro, 0, 0);
            rw[0][tc][0] = (uint32_t)t[0]; rw[0][tc][1] = (uint32_t)t[1];
            rw[0][tc][2] = (uint32_t)t[2]; rw[0][tc][3] = (uint32_t)t[3];
        }
    };

    // ---- MFMA fragment addresses ----
    const int hsel = (rho >> 2) & 1, isel = (rho >> 3) * 4 + (rho & 3);
    int a_fo[TC][2];    // within a tap's 4 KB weight tile
#pragma unroll
    for (int tc = 0; tc < TC; ++tc) {
        const int row = hsel * 16 * TC + tc * 16 + isel;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) a_fo[tc][kk] = row * 64 + (((kk * 2 + khalf) ^ ((row >> 2) & 3)) << 4);
    }
    const int ml64 = (wave * 32 + rho) * ROWB;  // byte offset of the lane's pixel in the tap-(0,0) window

    // One tile: wait for its patch, start the next patch and shortcut fetch, multiply, requantise, store.
    // Vector-memory operations a wave issues per tile, in program order: NPW patch loads and R shortcut loads
    // (for the next tile), then S stores (this tile).  When a tile's patch is waited for, the operations
    // issued after it are the R shortcut loads of the same fetch and the S stores of the tile before.
    auto do_tile = [&](int tile, const uint8_t *cur, uint8_t *nxt, uint32_t (&rw_cur)[TP][TC][4], uint32_t (&rw_nxt)[TP][TC][4],
                       int gstride, auto firstc) {
        constexpr bool first = decltype(firstc)::value;
        if (first) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(R) : "memory");
        else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(R + S) : "memory");
        __builtin_amdgcn_s_barrier();            // the patch (and, the first time, weights and parameters) of all waves
        fetch_patch(tile + gstride, nxt);
        if (has_res) fetch_res(tile + gstride, rw_nxt);

        // which of the nine taps of the lane's pixel are inside the image
        const int m = tile * BP + wave * 32 + rho;
        uint32_t mask = 0;
        if (m < a.M) {
            const int pq = m % HW;
            const int p = pq / W, q = pq - p * W;
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                const int ih = p + t / 3 - 1, iw = q + t % 3 - 1;
                if ((unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)W) mask |= 1u << t;
            }
        }
        v16i acc[TP][TC];
#pragma unroll
        for (int tc = 0; tc < TC; ++tc)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[0][tc][i] = 0;
        static_for<0, 9>([&](auto tc_) {
            constexpr int t = decltype(tc_)::value;
            constexpr int r = t / 3, s = t % 3;
            // bits 8-9 of the window row's byte offset are (row >> 2) & 3, its swizzle; the second-half chunk
            // index is the first-half one XOR 2
            const int v = ml64 + (r * W + s) * ROWB;
            const bool in = (mask >> t) & 1u;
            // a tap outside the image reads row PROWS-1 of the same buffer, which is beyond the rows in use and
            // therefore zero-filled by the fetch (plain offsets into the one buffer: the compiler then knows these
            // reads cannot touch the other patch buffer, whose asynchronous fill is in flight)
            v4i b0, b1;
            if constexpr (INT4) {
                const int off = in ? v + khalf * 16 : (PROWS - 1) * ROWB + khalf * 16;
                const v4i raw = *(const v4i *)(cur + off);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t u = (uint32_t)raw[e];
                    b0[e] = (int)(u & 0x0F0F0F0Fu);
                    b1[e] = (int)((u >> 4) & 0x0F0F0F0Fu);
                }
            } else {
                const int c0 = (((v >> 8) & 3) ^ khalf) << 4;
                const int off0 = in ? v + c0 : (PROWS - 1) * 64 + khalf * 16;
                b0 = *(const v4i *)(cur + off0);
                b1 = *(const v4i *)(cur + (off0 ^ 32));
            }
#pragma unroll
            for (int tc = 0; tc < TC; ++tc) {
                const v4i a0 = *(const v4i *)(wl + t * 4096 + a_fo[tc][0]);
                const v4i a1 = *(const v4i *)(wl + t * 4096 + a_fo[tc][1]);
                acc[0][tc] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b0, acc[0][tc], 0, 0, 0);
                acc[0][tc] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b1, acc[0][tc], 0, 0, 0);
            }
        });
        const int64_t mm[TP] = {m};
        const bool valid[TP] = {m < a.M};
        epilogue_tile<TC, TP, true, 2>(a, par_m, par_r, mm, valid, 0, chl, acc, wide, rw_cur);
        // the exact general epilogue issues a data-dependent number of stores: drain, so that the static counts
        // above stay valid (everything, the next patch included, is then complete)
        if (wide) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    };

    const int gstride = gridDim.x;
    int tile = blockIdx.x;                       // < n_tiles by construction of the grid
    uint32_t rw0[TP][TC][4] = {}, rw1[TP][TC][4] = {};
    fetch_patch(tile, pa);
    if (has_res) fetch_res(tile, rw0);
    wide = __syncthreads_or(wide);   // parameters staged by all waves; `wide` is workgroup-uniform from here
    do_tile(tile, pa, pb, rw0, rw1, gstride, std::true_type{});
    tile += gstride;
    while (tile < n_tiles) {
        do_tile(tile, pb, pa, rw1, rw0, gstride, std::false_type{});
        tile += gstride;
        if (tile >= n_tiles) break;
        do_tile(tile, pa, pb, rw0, rw1, gstride, std::false_type{});
        tile += gstride;
    }
}

bool conv3x3_c64_eligible(const ConvArgs &a, int x_hi) {
    if (!conv_mfma_eligible(a, x_hi)) return false;
    if (a.R != 3 || a.S != 3 || a.stride_h != 1 || a.stride_w != 1 || a.pad_h != 1 || a.pad_w != 1) return false;
    if (a.C != 64 || a.K != 64) return false;
    if (128 + 2 * a.W + 2 > 255) return false;      // the patch of a tile has to fit its LDS buffer
    if (a.M < 128 * 256) return false;              // enough tiles to put a persistent workgroup on every CU
    if (a.b == nullptr || a.y_dt == HAWQ_S32 || a.y_dt == HAWQ_S4) return false;
    if (a.res != nullptr && a.res_dt == HAWQ_S4) return false;
    uintptr_t al = (uintptr_t)a.y | (uintptr_t)a.bias | (uintptr_t)a.b | (uintptr_t)a.res_b | (uintptr_t)a.res;
    al |= ((uintptr_t)a.c | (uintptr_t)a.res_c) & 3;
    if ((al & 15) != 0) return false;
    if ((int64_t)a.N * a.H * a.W * 64 >= ((int64_t)1 << 31)) return false;
    if (is4(a.x_dt) && (((uintptr_t)a.x | (uintptr_t)a.w) & 15)) return false;
    return true;
}

hawq_status launch_conv3x3_c64(const ConvArgs &a, hipStream_t s) {
    if (a.M == 0) return HAWQ_OK;
    const int n_tiles = (a.M + 127) / 128;
    const int grid = n_tiles < 512 ? n_tiles : 512;   // two workgroups per CU
    const bool four = is4(a.x_dt);
    if (a.res != nullptr) {
        if (four) conv3x3_c64_kernel<true, true><<<grid, 256, 0, s>>>(a, n_tiles);
        else conv3x3_c64_kernel<true, false><<<grid, 256, 0, s>>>(a, n_tiles);
    } else {
        if (four) conv3x3_c64_kernel<false, true><<<grid, 256, 0, s>>>(a, n_tiles);
        else conv3x3_c64_kernel<false, false><<<grid, 256, 0, s>>>(a, n_tiles);
    }
    return check_launch();
}

}  // namespace hawq
