// Measurement aid, not part of the attention path: a kernel that issues nothing but bf16
// 32x32x16 MFMAs, so that a benchmark can report what the matrix pipes of the GPU it runs
// on sustain next to the nominal peak the roofline is quoted against.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/attn.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 512;        // 8 waves: two per SIMD, as in the attention kernels
constexpr int kMfmaPerIter = 16;     // four independent accumulator chains, four steps each

__global__ void __launch_bounds__(kThreads) probe_mfma_kernel(int iters, float *sink)
{
    const int l = threadIdx.x & 63;
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        // small operands (|x| <= 2^-6): the accumulators stay far from overflow
        a[i] = (__bf16)(0.0009765625f * (float)(1 + ((l + i) & 15)));
        b[i] = (__bf16)(0.0009765625f * (float)(1 + ((l * 3 + i) & 15)));
    }
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < kMfmaPerIter / 4; ++s)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) t += acc[j][i];
    sink[(size_t)blockIdx.x * kThreads + threadIdx.x] = t;
}

}  // namespace

extern "C" int attn_probe_mfma_bf16(int workgroups, int iters, float *sink, size_t sink_floats,
                                    double *flop, void *hip_stream)
{
    if (!sink) return ATTN_ERR_NULL;
    if (workgroups < 1 || iters < 1 || workgroups > (1 << 20)) return ATTN_ERR_SHAPE;
    if (sink_floats < (size_t)workgroups * kThreads) return ATTN_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(sink) & 3u) != 0) return ATTN_ERR_ALIGN;
    if (flop)  // 32x32x16 multiply-adds, two operations each
        *flop = (double)workgroups * (kThreads / 64) * (double)iters * kMfmaPerIter * 32768.0;
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(workgroups), dim3(kThreads), 0,
                       static_cast<hipStream_t>(hip_stream), iters, sink);
    return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}
