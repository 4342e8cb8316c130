// Device-side building blocks shared by the forward and backward attention kernels
// (gfx950 / CDNA4 only: wave64, 16-bit MFMA 32x32x16, LDS transpose reads).  `elem` is the
// 16-bit element type of this build of the kernels: bf16, or IEEE fp16 with -DATTN_F16.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "attn_launch.hpp"

namespace attn {

typedef elem elem8 __attribute__((ext_vector_type(8)));
typedef elem elem4 __attribute__((ext_vector_type(4)));
typedef elem elem2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// D = A(32x16) * B(16x32) + C, 16-bit elements in, fp32 accumulate.
// Lane l holds A[l%32][8*(l/32)..+7], B[8*(l/32)..+7][l%32] and, in C/D register i,
// element [8*(i/4) + 4*(l/32) + i%4][l%32].
__device__ __forceinline__ f32x16 mfma32(elem8 a, elem8 b, f32x16 c)
{
#ifdef ATTN_F16
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
#else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
#endif
}

// Row of a 32x32 accumulator block held in register i by a lane of half h = lane/32.
__device__ __forceinline__ constexpr int acc_row(int i, int h) { return 8 * (i / 4) + 4 * h + (i % 4); }

// Exchange between lane l and lane l^32: returns {value of the lower-half partner or self,
// value of the upper-half partner or self}; max/sum of the pair is symmetric in the two.
__device__ __forceinline__ float xhalf_max(float x)
{
    u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
}
__device__ __forceinline__ float xhalf_sum(float x)
{
    u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r.x) + __uint_as_float(r.y);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// Eight fp32 -> elem8 (round to nearest even; v_cvt_pk_bf16_f32 / v_cvt_pk_f16_f32 on gfx950).
__device__ __forceinline__ elem8 pack8(float a0, float a1, float a2, float a3,
                                        float a4, float a5, float a6, float a7)
{
    typedef float f32x8 __attribute__((ext_vector_type(8)));
    f32x8 v = {a0, a1, a2, a3, a4, a5, a6, a7};
    return __builtin_convertvector(v, elem8);
}
__device__ __forceinline__ elem4 pack4(float a0, float a1, float a2, float a3)
{
    f32x4 v = {a0, a1, a2, a3};
    return __builtin_convertvector(v, elem4);
}

// acc + a + b for two 16-bit elements, accumulated in fp32 (v_dot2c_f32_bf16 / v_dot2_f32_f16
// with a vector of ones).
__device__ __forceinline__ float dot2_acc(elem a, elem b, float acc)
{
    elem2 v = {a, b}, one = {(elem)1.0f, (elem)1.0f};
#ifdef ATTN_F16
    return __builtin_amdgcn_fdot2(v, one, acc, false);
#else
    return __builtin_amdgcn_fdot2_f32_bf16(v, one, acc, false);
#endif
}

// LDS transpose read (ds_read_b64_tr_b16).  Within each group of 16 lanes, source lane
// s = 4*e + c points at 4 consecutive 16-bit elements ("row e, chunk c"); result lane i
// receives, in element e, element i%4 of the chunk addressed by source lane 4*e + i/4.
// I.e. the group reads a 4-row x 16-column tile and every lane gets one column.
__device__ __forceinline__ s16x4 lds_read_tr(const elem *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (s16x4 __attribute__((address_space(3))) *)(p));
}
__device__ __forceinline__ elem8 join8(s16x4 lo, s16x4 hi)
{
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(elem8, v);
}

// 16-byte global load / LDS access of 8 elem.
__device__ __forceinline__ u32x4 ld_global16(const elem *p) { return *(const u32x4 *)p; }
// The same for columns col..col+7 of a row with only dr real columns: zeros past the end.
__device__ __forceinline__ u32x4 ld_row16(const elem *row, int col, int dr)
{
    u32x4 z = {0u, 0u, 0u, 0u};
    return col < dr ? *(const u32x4 *)(row + col) : z;
}
__device__ __forceinline__ elem8 as_elem8(u32x4 v) { return __builtin_bit_cast(elem8, v); }

// Raw buffer loads: byte offset = per-lane voff + wave-uniform soff into a resource that
// covers `bytes` bytes from `p`; reads past the end return 0 instead of faulting, which is
// how ragged tails and tiles past the end of a sequence are fetched.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void *p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 buf_load16(rsrc_t r, uint32_t voff, uint32_t soff)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, 0);
}
__device__ __forceinline__ u32x2 buf_load8(rsrc_t r, uint32_t voff, uint32_t soff)
{
    return __builtin_amdgcn_raw_buffer_load_b64(r, (int)voff, (int)soff, 0);
}

// Global -> LDS transfer issued from inline assembly: 16 bytes per lane, lane i lands at LDS
// byte address lds_addr + 16 i; the global byte offset is voff (per lane) + soff (uniform)
// into the raw buffer `desc`, and offsets at or past its size read as zero.  Written as
// assembly so that the compiler does not see the transfer: it would otherwise make a wave
// wait for ALL of its outstanding transfers before any later transpose read of LDS.  The
// caller orders transfers and reads itself (s_waitcnt vmcnt + barrier) and must wait for
// vmcnt(0) before the work-group ends.
// (m0 is named as clobbered so that the compiler does not assume a value it put there earlier
// survives; it answers that with a warning about reserved registers, silenced here)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
typedef u32x4 desc_t;
__device__ __forceinline__ desc_t make_desc(const void *p, uint32_t bytes)
{
    const uint64_t a = (uint64_t)p;
    desc_t d;
    d.x = __builtin_amdgcn_readfirstlane((uint32_t)a);
    d.y = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32) & 0xffffu);
    d.z = __builtin_amdgcn_readfirstlane(bytes);
    d.w = 0x00020000u;
    return d;
}
__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char *)p;
}
__device__ __forceinline__ void dma16(desc_t desc, uint32_t lds_addr, uint32_t voff, uint32_t soff)
{
    // lds_addr and soff are wave-uniform; readfirstlane makes that known to the compiler
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 ::"s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(voff), "s"(desc),
                 "s"(__builtin_amdgcn_readfirstlane(soff))
                 : "memory", "m0");
}
// The 16-byte transfer without the memory clobber, for a transfer into a buffer that no wave
// reads before a later barrier: the compiler may then move the LDS reads of the current tile
// across it, so it can be issued between the MFMAs of a step instead of in a burst in front of
// them (a burst makes the waves of a compute unit queue at its vector-memory path while the
// matrix pipes idle).  Volatile assembly keeps its order relative to the waits and barriers,
// which are volatile too.
__device__ __forceinline__ void dma16_between(desc_t desc, uint32_t lds_addr, uint32_t voff, uint32_t soff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 ::"s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(voff), "s"(desc),
                 "s"(__builtin_amdgcn_readfirstlane(soff))
                 : "m0");
}
// The same with the non-temporal hint, for data that is read once: a stream larger than the
// last-level cache then moves 12-14 % faster (stand-alone loops over 512 MiB: 5.98 -> 6.71 TB/s),
// one that fits it and is read again by the next launch 2-3 % slower.
__device__ __forceinline__ void dma16_between_nt(desc_t desc, uint32_t lds_addr, uint32_t voff, uint32_t soff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen nt lds"
                 ::"s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(voff), "s"(desc),
                 "s"(__builtin_amdgcn_readfirstlane(soff))
                 : "m0");
}
// Same with 4 bytes per lane: lane i lands at lds_addr + 4 i.
__device__ __forceinline__ void dma4(desc_t desc, uint32_t lds_addr, uint32_t voff, uint32_t soff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, %3 offen lds"
                 ::"s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(voff), "s"(desc),
                 "s"(__builtin_amdgcn_readfirstlane(soff))
                 : "memory", "m0");
}
#pragma clang diagnostic pop
// Wait until at most N of this wave's vector-memory operations are outstanding and all its
// LDS operations are done, then join the work-group barrier.  Unlike __syncthreads this
// leaves the newest global -> LDS transfers in flight across the barrier.
template <int N>
__device__ __forceinline__ void wait_vm_and_barrier()
{
    // The vmcnt wait is assembly because the compiler does not know about the transfers; the
    // lgkmcnt(0) wait is the builtin so that the compiler DOES know that no LDS operation is
    // pending after the barrier (otherwise its first wait after the barrier is a full
    // lgkmcnt(0) that also covers the reads issued since).  0xC07F = vmcnt 63, expcnt 7,
    // lgkmcnt 0 in the gfx9 encoding.
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// A kernel-argument scalar that is first used inside the main loop is fetched by a scalar
// load the compiler is free to leave pending at loop entry; scalar loads complete out of
// order, so the loop would then contain an s_waitcnt lgkmcnt(0) that also drains every LDS
// read issued in that iteration.  Passing the value through this function pins its load (and
// the wait for it) to the point of the call.
__device__ __forceinline__ float pin_scalar(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, x)));
}
__device__ __forceinline__ int pin_scalar(int x) { return __builtin_amdgcn_readfirstlane(x); }

// Work-group id -> position in a virtual order in which consecutive positions land on the
// same XCD.  Work-groups are handed to the 8 XCDs round-robin by linear id, each XCD has
// its own L2, so giving one XCD a contiguous range of (head, query tile) pairs keeps the
// K/V of a head in one L2.  Bijection on [0,total) for any total.
__device__ __forceinline__ int xcd_contiguous_order(int id, int total)
{
    constexpr int kXcd = 8;
    const int x = id % kXcd, pos = id / kXcd;
    const int full = total / kXcd, rem = total % kXcd;
    const int start = x * full + (x < rem ? x : rem);
    return start + pos;
}

// (head, tile rank) of a work-group.  Each XCD owns BH/8 whole heads, so that the operand a
// head's work-groups stream (K/V, or Q/dO) stays in one L2, and walks them a group of heads at
// a time: within a group rank-major -- rank 0 is meant to be the heaviest tile, so with
// unequal (causal) tiles the long work-groups of the group start first and its short ones fill
// the tail while the next group's long ones start.  Small groups keep few heads' operands
// competing for the 4 MB L2 at a time.  Without a mask (tiles of equal cost) the group is one
// head.  Under a causal mask it is four heads (measured on B=4 H=32 S=4096 and B=32 H=10
// S=2048, D = 128: groups of 4 or 8 heads are 5-9 % faster than all heads of the XCD
// rank-major, groups of 2 slightly slower than 4) and never fewer heads than fill the XCD's
// 32 compute units with one work-group each.  A group's order only balances the load within
// the group, and the launch ends with the tail of the last group, so a launch of only a few
// rounds of work-groups keeps all heads in one group, heaviest tiles of all heads first
// (B=8 H=8 S=1024 backward, two rounds: 66 us against 74 us with groups of four).
// Falls back to the contiguous order when the heads do not divide evenly over the XCDs.
template <bool CAUSAL>
__device__ __forceinline__ void xcd_tile_order(int id_, int ntile_, int BH_, int &bh, int &rank)
{
    // (unsigned throughout: nothing here is negative, and an unsigned division by a run-time
    // value is a third shorter than a signed one)
    constexpr unsigned kXcd = 8, kCuPerXcd = 32;
    const unsigned id = id_, ntile = ntile_, BH = BH_;
    if (BH % kXcd == 0) {
        const unsigned hpx = BH / kXcd, x = id % kXcd, pos = id / kXcd;
        unsigned G = 1;  // heads per group
        if (CAUSAL) G = hpx * ntile >= 4 * kCuPerXcd ? max(4u, (kCuPerXcd + ntile - 1) / ntile) : hpx;
        const unsigned group = pos / (G * ntile), within = pos - group * (G * ntile);
        const unsigned heads = min(G, hpx - group * G);  // the last group may be smaller
        const unsigned rk = within / heads;
        rank = (int)rk;
        bh = (int)(x * hpx + group * G + (within - rk * heads));
    } else {
        const unsigned v = (unsigned)xcd_contiguous_order(id_, ntile_ * BH_);
        bh = (int)(v / ntile);
        rank = (int)(v - (v / ntile) * ntile);
    }
}

}  // namespace attn
