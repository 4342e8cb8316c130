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

// RANDOM: operands with random signs and mantissas, a different pair of fragments at every
// step, so that the operand buses toggle the way they do on real data (the power drawn, and
// with it the clock the GPU sustains, depends on it); otherwise constant small operands.
template <bool RANDOM>
__global__ void __launch_bounds__(kThreads) probe_mfma_kernel(int iters, float *sink)
{
    const int l = threadIdx.x & 63;
    bf16x8 a[4], b[4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (RANDOM) {
                // +-[0.5, 1): sign and 7 mantissa bits from a hash of (lane, fragment, element)
                uint32_t x = (uint32_t)(l * 64 + s * 8 + i) * 2654435761u;
                x ^= x >> 15; x *= 2246822519u; x ^= x >> 13;
                const uint32_t ua = 0x3F000000u | ((x & 0x7Fu) << 16) | ((x & 0x80u) << 24);
                const uint32_t ub = 0x3F000000u | ((x & 0x7F00u) << 8) | ((x & 0x8000u) << 16);
                a[s][i] = (__bf16)__builtin_bit_cast(float, ua);
                b[s][i] = (__bf16)__builtin_bit_cast(float, ub);
            } else {
                // small operands (|x| <= 2^-6): the accumulators stay far from overflow
                a[s][i] = (__bf16)(0.0009765625f * (float)(1 + ((l + i) & 15)));
                b[s][i] = (__bf16)(0.0009765625f * (float)(1 + ((l * 3 + i) & 15)));
            }
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
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(s + j) & 3], b[s], acc[j], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) t += acc[j][i];
    sink[(size_t)blockIdx.x * kThreads + threadIdx.x] = t;
}

}  // namespace

extern "C" int attn_probe_mfma_bf16(int workgroups, int iters, int random_operands, float *sink,
                                    size_t sink_floats, double *flop, void *hip_stream)
{
    if (!sink) return ATTN_ERR_NULL;
    if (workgroups < 1 || iters < 1 || workgroups > (1 << 20)) return ATTN_ERR_SHAPE;
    if (sink_floats < (size_t)workgroups * kThreads) return ATTN_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(sink) & 3u) != 0) return ATTN_ERR_ALIGN;
    if (flop)  // 32x32x16 multiply-adds, two operations each
        *flop = (double)workgroups * (kThreads / 64) * (double)iters * kMfmaPerIter * 32768.0;
    if (random_operands)
        hipLaunchKernelGGL(probe_mfma_kernel<true>, dim3(workgroups), dim3(kThreads), 0,
                           static_cast<hipStream_t>(hip_stream), iters, sink);
    else
        hipLaunchKernelGGL(probe_mfma_kernel<false>, dim3(workgroups), dim3(kThreads), 0,
                           static_cast<hipStream_t>(hip_stream), iters, sink);
    return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}
