// Fused attention forward for head dimensions above 128 (up to 256) on gfx950: the same
// computation and the same orientation of the score tiles as the kernel for D <= 128 (S^T =
// K Q^T with one query per lane, O^T += V^T P^T, lazily moved reference max, two row sums), but
// a different budget: the Q fragments (64 registers) and the 256 x 32 fp32 accumulator of O^T
// (128 registers) leave room for one wave per SIMD only, and one K tile plus one V^T tile of 64
// keys take 70 KB of LDS, so both are double-buffered, not triple-buffered.
//
// Work-group = 4 waves = 128 query rows of one head; one barrier per tile of 64 keys.  With a
// single wave per SIMD the matrix pipe and the vector ALU can only overlap inside the wave, so a
// tile is processed in four steps whose independent halves sit in one basic block each:
//   A  S^T(0) = K Q^T                          (16 MFMAs)
//   B  S^T(1) = K Q^T   with   P(0) = exp2(c S(0) - m)
//   C  O^T += V^T P(0)^T   with   P(1) = exp2(c S(1) - m)
//   D  O^T += V^T P(1)^T                       (16 MFMAs)
// Nothing is carried from one tile to the next except the accumulators, which is what lets
// two K buffers do.
#include "attn_device.hpp"
#include "attn_launch.hpp"

namespace attn {

struct WideCfg {
    static constexpr int kD = 256;
    static constexpr int kNW = 4;
    static constexpr int kThreads = kNW * 64;
    static constexpr int kBR = kNW * 32;
    static constexpr int kBC = 64;
    // K tile: wave-wide transfers of 16 B per lane fill 1 KB pieces of two rows, chunk-major
    // inside a piece (chunk c of row r at 16 * (2 c + r % 2)), pieces 32 bytes further apart
    // than their size: the 16 rows a quarter wave reads at a fixed chunk fall into 16 different
    // 16-byte bank groups.
    static constexpr int kPR = 2;
    static constexpr int kKPieceBytes = 1024 + kPR * 16;
    static constexpr int kKPieces = kBC / kPR;
    static constexpr int kKTileBytes = kKPieces * kKPieceBytes;
    static constexpr int kKHalfBytes = kKTileBytes / 2;     // 32 rows further
    static constexpr int kKStepBytes = 2 * kPR * 16;        // next contraction step
    static constexpr int kKDmaPerWave = kKPieces / kNW;
    static constexpr int kLdV = kBC + 8;                    // V^T tile [d][key order], rows skewed
    static constexpr int kVTileBytes = kD * kLdV * 2;
    static constexpr int kVMicro = (kBC / 4) * (kD / 4);    // 4 keys x 4 d micro-tiles
    static constexpr int kVPerThread = kVMicro / kThreads;
    static constexpr int kOffV = 2 * kKTileBytes;
    static constexpr int kLdsBytes = 2 * (kKTileBytes + kVTileBytes);
    static_assert(kVMicro % kThreads == 0 && kKPieces % kNW == 0, "staging divides evenly");
    static_assert(kLdsBytes <= 160 * 1024, "LDS budget of a gfx950 CU exceeded");
};

constexpr float kWideOverflow = 1024.0f;   // a partial row sum above this moves the reference max
constexpr float kWideMinusHuge = -1.0e30f;

template <bool CAUSAL>
__global__ void __launch_bounds__(WideCfg::kThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
attn_fwd_wide_kernel(const FwdArgs a)
{
    using C = WideCfg;
    constexpr int D = C::kD, KS = D / 16, DB = D / 32, PR = C::kPR;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, l = tid & 63, r = l & 31, h = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int S = a.S, Dr = a.Dr, Sk = a.Sk, coff = a.Sk - a.S;

    int bh, rank;
    xcd_tile_order<CAUSAL>(blockIdx.x, a.nqt, a.BH, bh, rank);
    const int qt = CAUSAL ? a.nqt - 1 - rank : rank;  // heaviest tiles first
    const int64_t base = (int64_t)(bh / a.H) * a.stride_b + (int64_t)(bh % a.H) * a.stride_h;
    const int64_t base_kv = (int64_t)(bh / a.H) * a.kv_stride_b +
                            (int64_t)((bh % a.H) / a.group) * a.kv_stride_h;

    const int q0 = qt * C::kBR + w * 32;
    const int q = q0 + r;
    const int qc = q < S ? q : S - 1;  // clamped for loads; rows >= S are never stored
    const int q0e = q0 + coff;         // the wave's first row in key coordinates

    // Q fragments, B operand of K Q^T: lane holds Q[q][16 ks + 8 h .. +7]
    elem8 qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        qf[ks] = as_elem8(ld_row16(a.Q + base + (int64_t)qc * a.stride_s, ks * 16 + 8 * h, Dr));

    const int q_end = min(S, (qt + 1) * C::kBR);
    const int k_end = CAUSAL ? min(Sk, q_end + coff) : Sk;
    const int n_kt = (k_end + C::kBC - 1) / C::kBC;

    // ---- staging.  Rows past Sk-1, tiles past the last one and columns Dr..D-1 lie outside
    // the head's buffer resource and read as zero.
    const uint32_t head_bytes = (uint32_t)(((int64_t)(Sk - 1) * a.kv_stride_s + Dr) * 2);
    const rsrc_t Kr = make_rsrc(a.K + base_kv, head_bytes), Vr = make_rsrc(a.V + base_kv, head_bytes);
    const uint32_t row_bytes = (uint32_t)a.kv_stride_s * 2u;
    const uint32_t tile_bytes = C::kBC * row_bytes;
    // K: lane l of a transfer fetches chunk l / 2 of the piece's row l % 2
    const uint32_t k_voff = (l / PR) * 8 < Dr ? (l % PR) * row_bytes + ((l / PR) << 4) : head_bytes;
    auto dma_k = [&](int kt, int buf) {
#pragma unroll
        for (int n = 0; n < C::kKDmaPerWave; ++n) {
            const int ii = w + n * C::kNW;  // which piece of the tile: wave-uniform
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                Kr, (void __attribute__((address_space(3))) *)(smem + buf * C::kKTileBytes + ii * C::kKPieceBytes),
                16, (int)k_voff, kt * tile_bytes + ii * PR * row_bytes, 0, 0);
        }
    };
    // V: global -> registers -> transposed into LDS.  Micro-tile mt = 4 keys x 4 d; a wave
    // covers 32 keys x 32 d as 8 key groups x 8 d groups.
    auto v_coords = [&](int mt, int &key0, int &d0) {
        const int blk = mt >> 6;
        key0 = 32 * (blk & 1) + 4 * (mt & 7);
        d0 = 32 * (blk >> 1) + 4 * ((mt >> 3) & 7);
    };
    u32x2 vreg[C::kVPerThread][4];
    auto load_v = [&](int kt) {
#pragma unroll
        for (int n = 0; n < C::kVPerThread; ++n) {
            int key0, d0;
            v_coords(tid + n * C::kThreads, key0, d0);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                vreg[n][i] = buf_load8(Vr, d0 < Dr ? (key0 + i) * row_bytes + d0 * 2 : head_bytes,
                                       kt * tile_bytes);
        }
    };
    auto store_v = [&](int buf) {
#pragma unroll
        for (int n = 0; n < C::kVPerThread; ++n) {
            int key0, d0;
            v_coords(tid + n * C::kThreads, key0, d0);
            // position of key0 (a multiple of 4) in the MFMA contraction order:
            // key = 16 cc + 8 u + 4 hh + e  ->  16 cc + 8 hh + 4 u + e
            const int kpos = (key0 & ~15) | ((key0 & 4) << 1) | ((key0 & 8) >> 1);
            elem *dst = reinterpret_cast<elem *>(smem + C::kOffV + buf * C::kVTileBytes) + d0 * C::kLdV + kpos;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // column d0 + j of the 4 x 4 micro-tile: keys key0 .. key0 + 3
                const unsigned sel = (j & 1) ? 0x07060302u : 0x05040100u;
                const int hw = j >> 1;
                u32x2 col;
                col.x = __builtin_amdgcn_perm(vreg[n][1][hw], vreg[n][0][hw], sel);
                col.y = __builtin_amdgcn_perm(vreg[n][3][hw], vreg[n][2][hw], sel);
                *(u32x2 *)(dst + j * C::kLdV) = col;
            }
        }
    };

    float m = kWideMinusHuge;  // reference max of c*s (log2 units), the same in lanes l and l^32
    float lsum = 0.f;          // exact fp32 sum of this lane's half of the probabilities (for LSE)
    float hsum = 0.f;          // sum of the ROUNDED probabilities (O is divided by this one)
    f32x16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
    const float c = a.scale_log2e;

    const int k_lane = (r / PR) * C::kKPieceBytes + (h * PR + r % PR) * 16;
    const int v_lane = C::kOffV + (r * C::kLdV + 8 * h) * 2;

    // S^T of sub-tile u of the tile in buffer buf
    auto scores = [&](int buf, int u, f32x16 &s) __attribute__((always_inline)) {
        const char *Kt = smem + buf * C::kKTileBytes + u * C::kKHalfBytes + k_lane;
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            s = mfma32(*(const elem8 *)(Kt + ks * C::kKStepBytes), qf[ks], s);
    };
    // ragged tail and causal mask of sub-tile (kt, u); wave-uniform test whether any is needed
    auto mask = [&](int kt, int u, f32x16 &s) __attribute__((always_inline)) {
        const int kb = kt * C::kBC + 32 * u;
        if ((kb + 32 > Sk) || (CAUSAL && kb + 31 > q0e)) {
            const int lim = (CAUSAL ? min(qc + coff, Sk - 1) : Sk - 1) - kb - 4 * h;
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (8 * (i / 4) + (i % 4) > lim) s[i] = -INFINITY;
        }
    };
    auto softmax8 = [&](const f32x16 &t, int i0, float &psum) -> elem8 {
        float e[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            e[i] = fast_exp2(__builtin_fmaf(t[i0 + i], c, -m));
            psum += e[i];
        }
        return pack8(e[0], e[1], e[2], e[3], e[4], e[5], e[6], e[7]);
    };
    // The reference max moves to the true running max: rescale what has been accumulated and
    // redo the probabilities of the sub-tile whose scores are in s.
    auto move_reference = [&](const f32x16 &s, elem8 &p0, elem8 &p1, float &psum)
                              __attribute__((always_inline)) {
        float mx = s[0];
#pragma unroll
        for (int i = 1; i < 16; i += 3) mx = fmaxf(mx, fmaxf(s[i], fmaxf(s[i + 1], s[i + 2])));
        mx = xhalf_max(mx) * c;
        const float m_new = fmaxf(m, mx);
        const float alpha = fast_exp2(m - m_new);
        m = m_new;
        lsum *= alpha;
        hsum *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
        psum = 0.f;
        p0 = softmax8(s, 0, psum);
        p1 = softmax8(s, 8, psum);
    };
    // P of the sub-tile whose (masked) scores are in s, relative to the current reference; the
    // test whether the reference must move (settle) comes after the MFMAs that share the basic
    // block with this arithmetic
    auto probs = [&](const f32x16 &s, elem8 &p0, elem8 &p1, float &psum) __attribute__((always_inline)) {
        psum = 0.f;
        p0 = softmax8(s, 0, psum);
        p1 = softmax8(s, 8, psum);
    };
    auto settle = [&](const f32x16 &s, elem8 &p0, elem8 &p1, float &psum) __attribute__((always_inline)) {
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(psum > kWideOverflow) != 0, 0))
            move_reference(s, p0, p1, psum);
        lsum += psum;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            hsum = dot2_acc(p0[2 * i], p0[2 * i + 1], hsum);
            hsum = dot2_acc(p1[2 * i], p1[2 * i + 1], hsum);
        }
    };
    // O^T += V^T P^T for sub-tile u of the V tile in buffer buf
    auto pv = [&](int buf, int u, elem8 p0, elem8 p1) __attribute__((always_inline)) {
        const char *Vt = smem + buf * C::kVTileBytes + 64 * u + v_lane;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            o[db] = mfma32(*(const elem8 *)(Vt + 32 * db * C::kLdV * 2), p0, o[db]);
            o[db] = mfma32(*(const elem8 *)(Vt + 32 * db * C::kLdV * 2 + 32), p1, o[db]);
        }
    };
    // Start of iteration kt: V(kt) -> LDS (the buffer's previous tile, kt-2, was last read before
    // the barrier of iteration kt-1); K(kt) has been on its way since iteration kt-1.  After the
    // barrier the other buffers are free and take tile kt+1.
    auto stage = [&](int kt) __attribute__((always_inline)) {
        store_v(kt & 1);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (kt + 1 < n_kt) {
            dma_k(kt + 1, (kt & 1) ^ 1);
            load_v(kt + 1);
        }
    };

    if (n_kt > 0) {
        dma_k(0, 0);
        load_v(0);
    }
    // Tiles of which this wave sees some key come first; for the rest of the work-group's tiles
    // (under a causal mask, the waves with the earlier rows) it only takes part in the staging.
    // A second sub-tile that lies wholly above the wave's diagonal is computed with every score
    // masked: one code path, and it only happens on the diagonal tile.
    const int n_mine = CAUSAL ? __builtin_amdgcn_readfirstlane(min(n_kt, (q0e + 31) / C::kBC + 1)) : n_kt;
    for (int kt = 0; kt < n_mine; ++kt) {
        const int buf = kt & 1;
        stage(kt);
        f32x16 sA, sB;
        elem8 pA0, pA1, pB0, pB1;
        float sumA, sumB;
        scores(buf, 0, sA);                         // A
        mask(kt, 0, sA);
        scores(buf, 1, sB);                         // B
        probs(sA, pA0, pA1, sumA);
        __builtin_amdgcn_sched_barrier(0);
        settle(sA, pA0, pA1, sumA);
        mask(kt, 1, sB);
        pv(buf, 0, pA0, pA1);                       // C
        probs(sB, pB0, pB1, sumB);
        __builtin_amdgcn_sched_barrier(0);
        settle(sB, pB0, pB1, sumB);
        pv(buf, 1, pB0, pB1);                       // D
    }
    for (int kt = n_mine; kt < n_kt; ++kt) stage(kt);

    // Epilogue: O = O_acc / l, LSE = ln2 * (m + log2 l).
    const float lt = xhalf_sum(lsum);
    const float lr = xhalf_sum(hsum);
    const float inv = 1.0f / lr;
    if (q < S) {
        elem *Op = a.O + base + (int64_t)q * a.stride_s;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const elem4 ov = pack4(o[db][4 * g] * inv, o[db][4 * g + 1] * inv,
                                        o[db][4 * g + 2] * inv, o[db][4 * g + 3] * inv);
                if (32 * db + 8 * g + 4 * h < Dr) *(elem4 *)(Op + 32 * db + 8 * g + 4 * h) = ov;
            }
        if (h == 0) a.LSE[(int64_t)bh * S + q] = (m + fast_log2(lt)) * kLn2;
    }
}

template <bool CAUSAL>
static int launch_wide(FwdArgs a, hipStream_t st)
{
    using C = WideCfg;
    a.nqt = (a.S + C::kBR - 1) / C::kBR;
    if (hipFuncSetAttribute((const void *)attn_fwd_wide_kernel<CAUSAL>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, C::kLdsBytes) != hipSuccess)
        return -1;
    hipLaunchKernelGGL((attn_fwd_wide_kernel<CAUSAL>), dim3(a.nqt * a.BH), dim3(C::kThreads),
                       C::kLdsBytes, st, a);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Head dimensions 129..256 (D = 256 with the missing columns read as zeros); never split over
// the keys, no fused rotary embedding.
int launch_fwd_wide(const FwdArgs &a, bool causal, hipStream_t st)
{
    if (a.nsplit > 1 || a.rope_cos) return -1;
    return causal ? launch_wide<true>(a, st) : launch_wide<false>(a, st);
}

}  // namespace attn
