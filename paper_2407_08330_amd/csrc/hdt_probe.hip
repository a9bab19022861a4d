// A measuring stick for benchmarks, not part of the attention path: what this chip sustains when its matrix
// cores do nothing but the bf16 contraction instruction the attention kernels use.  Published peaks assume the
// nominal clock; under sustained MFMA load the clock is lower, and a kernel's MFMA share is better read
// against this figure as well.
#include "hdt_internal.h"
#include "hdt_mfma.h"

namespace {

constexpr int kProbeThreads = 256, kProbeChains = 4, kProbePerIter = 8;  // 8 MFMAs per chain visit: 32 per iteration

// every wave keeps kProbeChains independent accumulator chains going: 4 waves per workgroup, one per SIMD
__global__ __launch_bounds__(kProbeThreads) void k_probe_mfma(int iters, float *sink)
{
    const int lane = threadIdx.x & 63;
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; e++) {
        a[e] = (__bf16)(0.001f * (float)(lane + e));
        b[e] = (__bf16)(0.002f * (float)(lane - e));
    }
    f32x16 c[kProbeChains];
#pragma unroll
    for (int i = 0; i < kProbeChains; i++)
#pragma unroll
        for (int e = 0; e < 16; e++) c[i][e] = 0.f;
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int m = 0; m < kProbePerIter; m++)
#pragma unroll
            for (int i = 0; i < kProbeChains; i++) c[i] = mfma_32x32x16(a, b, c[i]);
    }
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < kProbeChains; i++)
#pragma unroll
        for (int e = 0; e < 16; e++) acc += c[i][e];
    if (acc == 12345.678f) sink[0] = acc;  // keeps the chains alive; never true for these operands
}

}  // namespace

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_probe_mfma_bf16(int32_t workgroups, int32_t iters,
                                                                                    float *d_sink, double *h_flop,
                                                                                    void *stream)
{
    if (workgroups <= 0 || iters <= 0 || d_sink == nullptr || h_flop == nullptr)
        return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_probe_mfma_bf16: workgroups and iters must be positive, pointers not NULL");
    hipLaunchKernelGGL(k_probe_mfma, dim3((unsigned)workgroups), dim3(kProbeThreads), 0, (hipStream_t)stream, iters, d_sink);
    HDT_HIP_TRY(hipGetLastError());
    *h_flop = (double)workgroups * (kProbeThreads / 64) * (double)iters * kProbePerIter * kProbeChains * (2.0 * 32 * 32 * 16);
    return HDT_OK;
}
