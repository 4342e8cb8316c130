// Fused attention forward for gfx950: O = softmax(scale * Q K^T [+ causal mask]) V and the
// per-row natural-log LSE, one pass over K/V with an online softmax (the
// "flash-attention-style formulation" the paper's debugging table refers to).
//
// Work decomposition
//   work-group = NW waves, one tile of BR = 32*NW query rows of one (batch, head);
//   wave       = 32 query rows; loops over key tiles of BC = 64 rows staged in LDS.
// The score tile is computed TRANSPOSED, S^T = K Q^T (keys x queries), with the
// 32x32x16 bf16 MFMA.  Its accumulator layout puts one query per lane (column l%32) and
// 16 keys per lane and 32-key block, so
//   - row max / row sum are in-lane reductions plus ONE exchange with lane l^32,
//   - the rescale factor alpha is a per-lane scalar,
//   - bf16(P^T) is already in the B-operand layout of the second MFMA,
//     O^T = V^T P^T (d x queries), once the contraction index is enumerated in the order
//     the accumulator holds it (key = 8*(t/4) + 4*(l/32) + t%4 within 16 keys).
// V^T fragments come from row-major V in LDS through the LDS transpose read.
#include "attn_device.hpp"
#include "attn_launch.hpp"

namespace attn {

template <int D, int NW>
struct FwdCfg {
    static constexpr int kThreads = NW * 64;
    static constexpr int kBR = NW * 32;
    static constexpr int kBC = 64;
    static constexpr int kLd = D + 8;               // LDS row stride (elements): +16 B skew
    static constexpr int kTileElems = kBC * kLd;    // one K or V tile
    static constexpr int kLdsBytes = 2 * 2 * kTileElems * 2;  // K,V double-buffered
    static constexpr int kChunks = kBC * D / 8;     // 16-byte chunks per tile
    static constexpr int kChunksPerThread = (kChunks + kThreads - 1) / kThreads;
    static_assert(kLdsBytes <= 160 * 1024, "LDS budget of a gfx950 CU exceeded");
};

template <int D, int NW, bool CAUSAL>
__global__ void __launch_bounds__(NW * 64) attn_fwd_kernel(const FwdArgs a)
{
    using C = FwdCfg<D, NW>;
    constexpr int KS = D / 16;  // contraction steps of K Q^T
    constexpr int DB = D / 32;  // 32-row blocks of O^T
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16 *Ks = reinterpret_cast<bf16 *>(smem);  // [2][BC][kLd]
    bf16 *Vs = Ks + 2 * C::kTileElems;          // [2][BC][kLd]

    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, r = l & 31, h = l >> 5;
    const int S = a.S;

    // (head, query tile) of this work-group; causal tiles are issued heaviest first.
    const int v = xcd_contiguous_order(blockIdx.x, a.nqt * a.BH);
    const int bh = v / a.nqt;
    const int qt = CAUSAL ? a.nqt - 1 - (v % a.nqt) : v % a.nqt;
    const int64_t base = (int64_t)(bh / a.H) * a.stride_b + (int64_t)(bh % a.H) * a.stride_h;
    const bf16 *Qp = a.Q + base, *Kp = a.K + base, *Vp = a.V + base;

    const int q0 = qt * C::kBR + w * 32;  // first query row of this wave
    const int q = q0 + r;                 // this lane's query row
    const int qc = q < S ? q : S - 1;     // clamped for loads; rows >= S are never stored

    // Q fragments, B operand of K Q^T: lane holds Q[q][16*ks + 8h .. +7].
    bf16x8 qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        qf[ks] = as_bf16x8(ld_global16(Qp + (int64_t)qc * a.stride_s + ks * 16 + 8 * h));

    // Key tiles this work-group visits.
    const int q_end = min(S, (qt + 1) * C::kBR);
    const int n_kt = ((CAUSAL ? q_end : S) + C::kBC - 1) / C::kBC;

    // Global -> register prefetch of one K and one V tile (rows clamped to S-1: finite
    // data, masked to probability 0 below).
    u32x4 kreg[C::kChunksPerThread], vreg[C::kChunksPerThread];
    auto prefetch = [&](int kt) {
#pragma unroll
        for (int n = 0; n < C::kChunksPerThread; ++n) {
            const int c = tid + n * C::kThreads;
            if (C::kChunks % C::kThreads == 0 || c < C::kChunks) {
                const int row = c / (D / 8), col = (c % (D / 8)) * 8;
                int kr = kt * C::kBC + row;
                kr = kr < S ? kr : S - 1;
                kreg[n] = ld_global16(Kp + (int64_t)kr * a.stride_s + col);
                vreg[n] = ld_global16(Vp + (int64_t)kr * a.stride_s + col);
            }
        }
    };
    auto commit = [&](int buf) {
#pragma unroll
        for (int n = 0; n < C::kChunksPerThread; ++n) {
            const int c = tid + n * C::kThreads;
            if (C::kChunks % C::kThreads == 0 || c < C::kChunks) {
                const int row = c / (D / 8), col = (c % (D / 8)) * 8;
                *(u32x4 *)(Ks + buf * C::kTileElems + row * C::kLd + col) = kreg[n];
                *(u32x4 *)(Vs + buf * C::kTileElems + row * C::kLd + col) = vreg[n];
            }
        }
    };

    float m = -INFINITY;  // running max of c*s (log2 units), identical in lanes l and l^32
    float lsum = 0.f;     // running sum of this lane's half of the keys
    f32x16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] = 0.f;

    const float c = a.scale_log2e;
    // transpose-read source role of this lane: row (l%16)/4 of a 4-row group, 4-element
    // chunk (l%4) of the 16 columns served by its 16-lane group.
    const int tr_row = 4 * h + ((l & 15) >> 2);
    const int tr_col = ((l >> 4) & 1) * 16 + (l & 3) * 4;

    prefetch(0);
    for (int kt = 0; kt < n_kt; ++kt) {
        const int buf = kt & 1;
        commit(buf);
        __syncthreads();
        if (kt + 1 < n_kt) prefetch(kt + 1);

        const int kb = kt * C::kBC;
        const bool active = !CAUSAL || kb <= q0 + 31;  // wave-uniform
        if (active) {
            const bf16 *Kt = Ks + buf * C::kTileElems;
            const bf16 *Vt = Vs + buf * C::kTileElems;
            f32x16 s0, s1;
#pragma unroll
            for (int i = 0; i < 16; ++i) { s0[i] = 0.f; s1[i] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 k0 = *(const bf16x8 *)(Kt + r * C::kLd + ks * 16 + 8 * h);
                const bf16x8 k1 = *(const bf16x8 *)(Kt + (32 + r) * C::kLd + ks * 16 + 8 * h);
                s0 = mfma32(k0, qf[ks], s0);
                s1 = mfma32(k1, qf[ks], s1);
            }
            // Ragged tail and causal mask: only tiles that touch the end or the diagonal.
            const bool need_mask = (kb + C::kBC > S) || (CAUSAL && kb + C::kBC - 1 > q0);
            if (need_mask) {
                const int lim = (CAUSAL ? qc : S - 1) - kb - 4 * h;  // last visible key offset
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int ko = 8 * (i / 4) + (i % 4);
                    if (ko > lim) s0[i] = -INFINITY;
                    if (ko + 32 > lim) s1[i] = -INFINITY;
                }
            }
            float mx = fmaxf(s0[0], s1[0]);
#pragma unroll
            for (int i = 1; i < 16; ++i) mx = fmaxf(mx, fmaxf(s0[i], s1[i]));
            mx = xhalf_max(mx);
            const float m_new = fmaxf(m, mx * c);
            const float alpha = fast_exp2(m - m_new);
            m = m_new;
            float psum = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                s0[i] = fast_exp2(__builtin_fmaf(s0[i], c, -m_new));
                s1[i] = fast_exp2(__builtin_fmaf(s1[i], c, -m_new));
                psum += s0[i] + s1[i];
            }
            lsum = lsum * alpha + psum;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[db][i] *= alpha;

            // bf16(P^T) as B operands: contraction step cc covers keys 16*cc .. 16*cc+15.
            bf16x8 pf[4];
            pf[0] = pack8(s0[0], s0[1], s0[2], s0[3], s0[4], s0[5], s0[6], s0[7]);
            pf[1] = pack8(s0[8], s0[9], s0[10], s0[11], s0[12], s0[13], s0[14], s0[15]);
            pf[2] = pack8(s1[0], s1[1], s1[2], s1[3], s1[4], s1[5], s1[6], s1[7]);
            pf[3] = pack8(s1[8], s1[9], s1[10], s1[11], s1[12], s1[13], s1[14], s1[15]);
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    // V^T fragment: lane (d = 32*db + l%32, half h) needs V[16cc + 4h + e][d]
                    // in elements 0..3 and V[16cc + 8 + 4h + e][d] in elements 4..7.
                    const bf16 *vp = Vt + (16 * cc + tr_row) * C::kLd + 32 * db + tr_col;
                    const bf16x8 vf = join8(lds_read_tr(vp), lds_read_tr(vp + 8 * C::kLd));
                    o[db] = mfma32(vf, pf[cc], o[db]);
                }
            }
        }
    }

    // Epilogue: O = O_acc / l, LSE = ln2 * (m + log2 l).
    const float lt = xhalf_sum(lsum);
    const float inv = 1.0f / lt;
    if (q < S) {
        bf16 *Op = a.O + base + (int64_t)q * a.stride_s;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const bf16x4 ov = pack4(o[db][4 * g] * inv, o[db][4 * g + 1] * inv,
                                        o[db][4 * g + 2] * inv, o[db][4 * g + 3] * inv);
                *(bf16x4 *)(Op + 32 * db + 8 * g + 4 * h) = ov;
            }
        if (h == 0) a.LSE[(int64_t)bh * S + q] = (m + fast_log2(lt)) * kLn2;
    }
}

template <int D, int NW>
static int launch_fwd_nw(const FwdArgs &a, bool causal, hipStream_t st)
{
    using C = FwdCfg<D, NW>;
    const dim3 grid(a.nqt * a.BH), block(C::kThreads);
    if (causal) {
        hipFuncSetAttribute((const void *)attn_fwd_kernel<D, NW, true>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, C::kLdsBytes);
        hipLaunchKernelGGL((attn_fwd_kernel<D, NW, true>), grid, block, C::kLdsBytes, st, a);
    } else {
        hipFuncSetAttribute((const void *)attn_fwd_kernel<D, NW, false>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, C::kLdsBytes);
        hipLaunchKernelGGL((attn_fwd_kernel<D, NW, false>), grid, block, C::kLdsBytes, st, a);
    }
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Waves per work-group: 8 (256 query rows) unless the sequence is too short to fill them.
int fwd_waves_for(int S)
{
    const int blocks32 = (S + 31) / 32;
    if (blocks32 >= 8) return 8;
    if (blocks32 >= 4) return 4;
    return blocks32;  // 1, 2 or 3
}

template <int D>
static int launch_fwd_d(FwdArgs a, bool causal, hipStream_t st)
{
    const int nw = fwd_waves_for(a.S);
    a.nqt = (a.S + nw * 32 - 1) / (nw * 32);
    switch (nw) {
        case 8: return launch_fwd_nw<D, 8>(a, causal, st);
        case 4: return launch_fwd_nw<D, 4>(a, causal, st);
        case 3: return launch_fwd_nw<D, 3>(a, causal, st);
        case 2: return launch_fwd_nw<D, 2>(a, causal, st);
        default: return launch_fwd_nw<D, 1>(a, causal, st);
    }
}

int launch_fwd(const FwdArgs &a, int D, bool causal, hipStream_t st)
{
    return D == 128 ? launch_fwd_d<128>(a, causal, st) : launch_fwd_d<64>(a, causal, st);
}

}  // namespace attn
