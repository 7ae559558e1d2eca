// Measurement helper: what the chip's INT8 matrix cores sustain when nothing else is in the way.
//
// A register-only loop of independent v_mfma_i32_32x32x32_i8 (four accumulators per wave, four waves per SIMD, every CU
// occupied, no memory traffic inside the loop) -- the denominator next to the datasheet figure when a convolution's
// TOP/s are quoted as a fraction of peak.  The operands are not all zero, so the datapath toggles.
#include "common.h"

namespace hawq {

__global__ void __launch_bounds__(256) mfma_loop_kernel(int *out, int iters, int seed) {
    v16i acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0;
    const int t = (int)threadIdx.x;
    v4i a = {seed + t, seed * 3 + t, seed * 5, seed * 7 - t}, b = {seed * 11, seed * 13 + t, t * 0x01010101, seed};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[j], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[j][i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

}  // namespace hawq

extern "C" hawq_status hawq_probe_mfma_peak(int32_t iters, double *tops) {
    using namespace hawq;
    if (!tops) return HAWQ_ERR_NULL;
    if (iters < 1 || iters > 1000000) return HAWQ_ERR_RANGE;
    constexpr int kBlocks = 1024, kThreads = 256;   // four workgroups of four waves per CU
    int *out = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hawq_status rc = HAWQ_ERR_DEVICE;
    float ms = 0.f;
    if (hipMalloc(&out, (size_t)kBlocks * kThreads * sizeof(int)) != hipSuccess) return HAWQ_ERR_DEVICE;
    if (hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess) {
        mfma_loop_kernel<<<kBlocks, kThreads, 0, nullptr>>>(out, iters, 0x1b2d4f71);   // warm-up
        if (hipEventRecord(e0, nullptr) == hipSuccess) {
            mfma_loop_kernel<<<kBlocks, kThreads, 0, nullptr>>>(out, iters, 0x1b2d4f71);
            if (hipEventRecord(e1, nullptr) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
                hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms > 0.f && check_launch() == HAWQ_OK) {
                const double ops = 2.0 * 32 * 32 * 32 * 4 * (double)iters * kBlocks * (kThreads / 64);
                *tops = ops / ((double)ms * 1e-3) / 1e12;
                rc = HAWQ_OK;
            }
        }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(out);
    return rc;
}
