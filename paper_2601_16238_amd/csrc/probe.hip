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

// What a work-group that only reads can stream: the ceiling for the decoding forward, whose time
// is the time to read K and V once.  Both kernels fold everything they read into one 32-bit XOR
// per work-group, so that a test can check that every byte was read.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t fold(u32x4 v) { return v.x ^ v.y ^ v.z ^ v.w; }

// XOR over the work-group's 256 threads; the result in thread 0.  red: 4 words of LDS.
__device__ __forceinline__ uint32_t group_xor(uint32_t x, uint32_t *red)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x ^= (uint32_t)__shfl_xor((int)x, d, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
    __syncthreads();
    return red[0] ^ red[1] ^ red[2] ^ red[3];
}

// Plain loads: the work-group walks its contiguous share in steps of 32 KB, eight 16-byte
// loads in flight per lane.
template <bool NT>
__global__ void __launch_bounds__(256) probe_stream_loads_kernel(const char *src, size_t per_wg,
                                                                 uint32_t *checksum)
{
    __shared__ uint32_t red[4];
    const u32x4 *p = (const u32x4 *)(src + (size_t)blockIdx.x * per_wg) + threadIdx.x;
    const size_t steps = per_wg / 32768;
    uint32_t acc = 0;
    for (size_t i = 0; i < steps; ++i) {
        u32x4 v[8];
#pragma unroll
        for (int n = 0; n < 8; ++n)
            v[n] = NT ? __builtin_nontemporal_load(p + i * 2048 + n * 256) : p[i * 2048 + n * 256];
#pragma unroll
        for (int n = 0; n < 8; ++n) acc ^= fold(v[n]);
    }
    acc = group_xor(acc, red);
    if (threadIdx.x == 0) checksum[blockIdx.x] = acc;
}

// Direct global -> LDS transfers in the shape of the decoding forward: the buffer is two tensors
// (its halves), a tile is 16 KB of each, a transfer moves 1 KB with neighbouring lanes fetching
// from neighbouring 256-byte rows (the attention kernels' piece order), two tile buffers, the
// next tile requested right after the barrier that publishes the current one.
template <bool NT>
__global__ void __launch_bounds__(256) probe_stream_direct_kernel(const char *src, uint32_t half_per_wg,
                                                                  size_t half_bytes, uint32_t *checksum)
{
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    __shared__ uint32_t red[4];
    const int tid = threadIdx.x, l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    auto make_desc = [](const char *base, uint32_t bytes) {
        const uint64_t a = (uint64_t)base;
        u32x4 d;
        d.x = __builtin_amdgcn_readfirstlane((uint32_t)a);
        d.y = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32) & 0xffffu);
        d.z = __builtin_amdgcn_readfirstlane(bytes);
        d.w = 0x00020000u;
        return d;
    };
    const u32x4 d0 = make_desc(src + (size_t)blockIdx.x * half_per_wg, half_per_wg);
    const u32x4 d1 = make_desc(src + half_bytes + (size_t)blockIdx.x * half_per_wg, half_per_wg);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char *)smem;
    const uint32_t voff = (l % 4) * 256 + (l / 4) * 16;
    const int n_tiles = (int)(half_per_wg / 16384);
    auto issue = [&](int t, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            const int ii = w + 4 * n;  // piece of the tile: 0..15 first tensor, 16..31 second
            if (NT)
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen nt lds"
                             ::"s"(__builtin_amdgcn_readfirstlane(lds0 + buf * 32768 + ii * 1024)), "v"(voff),
                             "s"(ii < 16 ? d0 : d1), "s"(__builtin_amdgcn_readfirstlane(t * 16384 + (ii & 15) * 1024))
                             : "memory", "m0");
            else
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                             ::"s"(__builtin_amdgcn_readfirstlane(lds0 + buf * 32768 + ii * 1024)), "v"(voff),
                             "s"(ii < 16 ? d0 : d1), "s"(__builtin_amdgcn_readfirstlane(t * 16384 + (ii & 15) * 1024))
                             : "memory", "m0");
        }
    };
    if (n_tiles > 0) issue(0, 0);
    uint32_t acc = 0;
    for (int t = 0; t < n_tiles; ++t) {
        const int buf = t & 1;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();  // tile t is in LDS; the other buffer was last read before this barrier
        if (t + 1 < n_tiles) issue(t + 1, buf ^ 1);
#pragma unroll
        for (int n = 0; n < 8; ++n) acc ^= fold(*(const u32x4 *)(smem + buf * 32768 + n * 4096 + tid * 16));
    }
    __syncthreads();
    acc = group_xor(acc, red);
    if (tid == 0) checksum[blockIdx.x] = acc;
}

}  // namespace

extern "C" int attn_probe_stream(const void *src, size_t bytes, int workgroups, int direct,
                                 uint32_t *checksum, void *hip_stream)
{
    if (!src || !checksum) return ATTN_ERR_NULL;
    if (workgroups < 1 || workgroups > (1 << 20) || bytes == 0 || bytes % ((size_t)workgroups * 32768) != 0 ||
        bytes / workgroups > (size_t)1 << 31)
        return ATTN_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) != 0 || (reinterpret_cast<uintptr_t>(checksum) & 3u) != 0)
        return ATTN_ERR_ALIGN;
    const size_t per_wg = bytes / workgroups;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const bool nt = (direct & 2) != 0;
    if (direct & 1) {
        const void *k = nt ? (const void *)probe_stream_direct_kernel<true> : (const void *)probe_stream_direct_kernel<false>;
        if (hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, 65536) != hipSuccess)
            return ATTN_ERR_LAUNCH;
        if (nt)
            hipLaunchKernelGGL(probe_stream_direct_kernel<true>, dim3(workgroups), dim3(256), 65536, st,
                               static_cast<const char *>(src), (uint32_t)(per_wg / 2), bytes / 2, checksum);
        else
            hipLaunchKernelGGL(probe_stream_direct_kernel<false>, dim3(workgroups), dim3(256), 65536, st,
                               static_cast<const char *>(src), (uint32_t)(per_wg / 2), bytes / 2, checksum);
    } else if (nt) {
        hipLaunchKernelGGL(probe_stream_loads_kernel<true>, dim3(workgroups), dim3(256), 0, st,
                           static_cast<const char *>(src), per_wg, checksum);
    } else {
        hipLaunchKernelGGL(probe_stream_loads_kernel<false>, dim3(workgroups), dim3(256), 0, st,
                           static_cast<const char *>(src), per_wg, checksum);
    }
    return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}

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
