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

// The traffic a one-kernel backward would put on fp32 global atomics: the work-group that owns
// key block kb of a head adds one 32 x 128 fp32 tile of partial dQ per 32-row query slot that
// sees its keys.  Nothing else runs, so the time is the ceiling of that path alone.  A lane
// addresses column l%32 of a row, as the accumulator layout of a dQ = dS K product would, so
// one instruction touches two rows of 128 contiguous bytes.
__global__ void __launch_bounds__(256) probe_atomic_kernel(float *acc, int S, int key_block,
                                                           int BH, int causal)
{
    // all key blocks of a head on one XCD (work-groups go to the 8 XCDs round-robin by id)
    const int id = blockIdx.x, x = id % 8, pos = id / 8, hpx = BH / 8;
    const int bh = x * hpx + pos % hpx, kb = pos / hpx;
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63, r = l & 31, h = l >> 5;
    float *base = acc + (size_t)bh * S * 128;
    const int nslot = S / 32, slot0 = causal ? min(nslot, (kb * key_block) / 32) : 0;
    for (int s = slot0 + w; s < nslot; s += 4) {
        float *tile = base + (size_t)s * 32 * 128;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                __hip_atomic_fetch_add(tile + (8 * (i / 4) + 4 * h + (i % 4)) * 128 + 32 * db + r, 1.0f,
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

}  // namespace

extern "C" int attn_probe_atomic_f32(int BH, int S, int key_block, int causal, float *acc,
                                     size_t acc_floats, double *bytes_added, void *hip_stream)
{
    if (!acc) return ATTN_ERR_NULL;
    if (BH < 8 || BH % 8 || BH > 4096 || S < 32 || S % 32 || S > (1 << 20) || key_block < 32 ||
        key_block % 32 || key_block > S)
        return ATTN_ERR_SHAPE;
    if (acc_floats < (size_t)BH * S * 128) return ATTN_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(acc) & 3u) != 0) return ATTN_ERR_ALIGN;
    const int nkb = (S + key_block - 1) / key_block, nslot = S / 32;
    if (bytes_added) {
        double tiles = 0;
        for (int kb = 0; kb < nkb; ++kb) tiles += nslot - (causal ? (kb * key_block) / 32 : 0);
        *bytes_added = tiles * BH * 32.0 * 128.0 * 4.0;
    }
    hipLaunchKernelGGL(probe_atomic_kernel, dim3(nkb * BH), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), acc, S, key_block, BH, causal);
    return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}

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
