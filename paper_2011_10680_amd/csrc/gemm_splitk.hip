// Quantised matrix multiply with few rows (the fully connected layer that ends the network: Section 3.1's matmul, last
// layer 8-bit per Appendix H):  y[m][n] = epilogue( sum_k x[m][k] w[n][k] + bias[n] ),  M up to a few hundred.
//
// With so few rows a tiling over (m, n) gives a handful of workgroups that each walk the whole reduction serially -- at
// batch 128 the layer is 32 tiles of 32 K-steps on 256 compute units, all latency.  Here a workgroup owns 32 output
// channels x 128 rows and its eight waves split the REDUCTION: wave v multiplies K-steps v S/8 ... (v+1) S/8 - 1 into its own
// INT32 accumulators (MFMA 32x32x32, operands read straight from the row-major tensors into the fragment layout), the
// eight partial tiles meet in LDS, and every wave finishes one eighth of the outputs.  Integer addition is associative:
// the split changes no bit.
//
// XOR (unsigned bytes above 127, which the signed matrix operand cannot hold): the kernel multiplies x XOR 0x80 = x - 128
// and, with one more MFMA per half-step against a constant operand of -128, accumulates  -128 sum_k w[n][k]  next to it;
// their difference is the exact sum over the unsigned bytes.
#include "common.h"

namespace hawq {

template <bool XOR>
__global__ void __launch_bounds__(512)
gemm_splitk_kernel(const uint8_t *__restrict__ x, const uint8_t *__restrict__ w, const int32_t *__restrict__ bias,
                   const int32_t *__restrict__ b, const uint8_t *__restrict__ c, uint8_t *__restrict__ y, const int M, const int N,
                   const int K, const int y_dt, const int lo, const int hi) {
    __shared__ int32_t red[8][64][64];   // [wave][accumulator register][lane]: consecutive lanes, consecutive banks
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rho = lane & 31, khalf = lane >> 5;
    const int n0 = blockIdx.x * 32, m0 = blockIdx.y * 128;
    const int steps = (K / 64) / 8;                          // K-steps of this wave
    const int kbeg = wave * steps * 64;

    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void *)w, 0, (int)((int64_t)N * K), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc((void *)x, 0, (int)((int64_t)M * K), 0x00020000);
    // MFMA row rho holds the channel whose accumulator lands in register (rho >> 3) * 4 + (rho & 3) of lane half
    // (rho >> 2) & 1: a lane then owns 16 consecutive channels of one row of x
    const int n = n0 + ((rho >> 2) & 1) * 16 + (rho >> 3) * 4 + (rho & 3);
    const uint32_t woff = n < N ? (uint32_t)(n * K + kbeg + khalf * 16) : 0x80000000u;
    uint32_t xoff[4];
#pragma unroll
    for (int tp = 0; tp < 4; ++tp) {
        const int m = m0 + tp * 32 + rho;
        xoff[tp] = m < M ? (uint32_t)(m * K + kbeg + khalf * 16) : 0x80000000u;
    }
    v16i acc[4], corr;
#pragma unroll
    for (int i = 0; i < 16; ++i) { acc[0][i] = 0; acc[1][i] = 0; acc[2][i] = 0; acc[3][i] = 0; corr[i] = 0; }
    const v4i c80 = {(int)0x80808080u, (int)0x80808080u, (int)0x80808080u, (int)0x80808080u};
    for (int st = 0; st < steps; ++st) {
        v4i af[2], bf[2][4];
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            af[kk] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, (int)(woff + (uint32_t)(st * 64 + kk * 32)), 0, 0);
#pragma unroll
            for (int tp = 0; tp < 4; ++tp) {
                bf[kk][tp] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, (int)(xoff[tp] + (uint32_t)(st * 64 + kk * 32)), 0, 0);
                // (rows past M read zeros and stay zero: they are never stored)
                if (XOR) bf[kk][tp] ^= c80;
            }
        }
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
            for (int tp = 0; tp < 4; ++tp) acc[tp] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[kk], bf[kk][tp], acc[tp], 0, 0, 0);
            if (XOR) corr = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[kk], c80, corr, 0, 0, 0);
        }
    }
    // partial tiles -> LDS
#pragma unroll
    for (int tp = 0; tp < 4; ++tp)
#pragma unroll
        for (int i = 0; i < 16; ++i) red[wave][tp * 16 + i][lane] = XOR ? acc[tp][i] - corr[i] : acc[tp][i];
    __syncthreads();
    // wave v finishes registers 8v ... 8v + 7: row tile v / 2, channels (v % 2) * 8 ... + 7 of the lane's sixteen
    const int tp = wave >> 1, i0 = (wave & 1) * 8;
    const int m = m0 + tp * 32 + rho;
    const int ch = n0 + khalf * 16 + i0;
    int32_t sum[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        int32_t s = 0;
#pragma unroll
        for (int v = 0; v < 8; ++v) s += red[v][wave * 8 + j][lane];
        sum[j] = s;
    }
    if (m >= M) return;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int k = ch + j;
        if (k >= N) break;
        const int32_t t = sum[j] + bias[k];
        const int64_t o = (int64_t)m * N + k;
        if (b == nullptr) ((int32_t *)y)[o] = t;
        else if (y_dt == HAWQ_S32) ((int32_t *)y)[o] = clamp64(rq64(t, b[k], c[k]), lo, hi);
        else y[o] = (uint8_t)clamp64(rq64(t, b[k], c[k]), lo, hi);
    }
}

// 1x1 / stride 1 / unpadded request with 8-bit operands, few rows and a long reduction.  The fragment-layout reads put every
// lane in a cache line of its own, which the vector-memory path serves at a quarter of its rate: at the size of ResNet50's
// last layer (128 x 2048 -> 1000) the kernel measures 15 us against 13 us for the tiled kernel, so the dispatcher takes it
// only for what no other matrix-core kernel can do -- unsigned bytes above 127 (x_hi > 127), which otherwise fall to the
// one-thread-per-output kernel.
bool gemm_splitk_eligible(const ConvArgs &a) {
    if (a.R != 1 || a.S != 1 || a.stride_h != 1 || a.stride_w != 1 || a.pad_h != 0 || a.pad_w != 0) return false;
    if (a.res != nullptr || a.xs != nullptr) return false;
    if (a.w_dt != HAWQ_S8 || (a.x_dt != HAWQ_U8 && a.x_dt != HAWQ_S8)) return false;
    if (a.y_dt != HAWQ_S32 && a.y_dt != HAWQ_U8 && a.y_dt != HAWQ_S8) return false;
    if (a.C % 512 != 0 || a.M > 512 || a.M <= 0) return false;
    if (((uintptr_t)a.x | (uintptr_t)a.w) & 15) return false;
    if ((int64_t)a.K * a.C >= ((int64_t)1 << 31) || (int64_t)a.M * a.C >= ((int64_t)1 << 31)) return false;
    return true;
}

hawq_status launch_gemm_splitk(const ConvArgs &a, int x_hi, hipStream_t s) {
    const dim3 grid((a.K + 31) / 32, (a.M + 127) / 128);
    const bool xr = a.x_dt == HAWQ_U8 && x_hi > 127;
    if (xr) gemm_splitk_kernel<true><<<grid, 512, 0, s>>>(a.x, a.w, a.bias, a.b, a.c, a.y, a.M, a.K, a.C, a.y_dt, a.lo, a.hi);
    else gemm_splitk_kernel<false><<<grid, 512, 0, s>>>(a.x, a.w, a.bias, a.b, a.c, a.y, a.M, a.K, a.C, a.y_dt, a.lo, a.hi);
    return check_launch();
}

}  // namespace hawq
