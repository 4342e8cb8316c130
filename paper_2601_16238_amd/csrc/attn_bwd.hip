// Fused attention backward for gfx950.  P is recomputed from Q, K and the forward's LSE;
// three kernels on one stream, no atomics, deterministic:
//   1. delta_i = sum_d dO_id O_id                                  (HBM-bound preprocess)
//   2. dK, dV : one work-group per block of keys, loops over query tiles, dK^T / dV^T
//               accumulate in registers                            (4 GEMMs per tile pair)
//   3. dQ     : one work-group per block of queries, loops over key tiles, dQ^T
//               accumulates in registers                           (3 GEMMs per tile pair)
// With dP = dO V^T and dS = P o (dP - delta):
//   dV = P^T dO,  dK = scale * dS^T Q,  dQ = scale * dS K.
//
// Layout trick shared with the forward: every 32x32 score block is produced in the
// orientation whose accumulator layout IS the B-operand layout of the GEMM that consumes
// it (contraction index enumerated in accumulator order), so P and dS never leave
// registers; the other operand of those GEMMs is a transposed tile read from LDS with
// the LDS transpose read.
//   kernel 2: S = Q K^T (queries x keys): lane owns a key; dV^T += dO^T P, dK^T += Q^T dS
//   kernel 3: S^T = K Q^T (keys x queries): lane owns a query; dQ^T += K^T dS^T
#include "attn_device.hpp"
#include "attn_launch.hpp"

namespace attn {

// ---------------------------------------------------------------------------------------
// 1. delta = rowsum(dO * O), fp32, contiguous [B,H,S].  D/8 lanes per row, 16-byte loads.
// ---------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(256) attn_bwd_delta_kernel(const BwdArgs a)
{
    constexpr int LPR = D / 8;          // lanes per row
    constexpr int RPB = 256 / LPR;      // rows per block
    const int64_t rows = (int64_t)a.BH * a.S;
    const int64_t row = (int64_t)blockIdx.x * RPB + threadIdx.x / LPR;
    const int sub = threadIdx.x % LPR;
    float acc = 0.f;
    if (row < rows) {
        const int bh = (int)(row / a.S), i = (int)(row % a.S);
        const int64_t off = (int64_t)(bh / a.H) * a.stride_b + (int64_t)(bh % a.H) * a.stride_h +
                            (int64_t)i * a.stride_s + sub * 8;
        const bf16x8 o = as_bf16x8(ld_global16(a.O + off));
        const bf16x8 g = as_bf16x8(ld_global16(a.dO + off));
#pragma unroll
        for (int t = 0; t < 8; ++t) acc += (float)o[t] * (float)g[t];
    }
#pragma unroll
    for (int s = LPR / 2; s >= 1; s >>= 1) acc += __shfl_xor(acc, s);
    if (row < rows && sub == 0) a.delta[row] = acc;
}

// ---------------------------------------------------------------------------------------
// Tile staging shared by kernels 2 and 3: two bf16 tiles of 64 rows x D (row-major, skewed
// rows) and, for kernel 2, the 64 LSE / delta values of the rows, double-buffered.
// ---------------------------------------------------------------------------------------
template <int D, int NW>
struct BwdCfg {
    static constexpr int kThreads = NW * 64;
    static constexpr int kBlk = NW * 32;            // rows owned by the work-group
    static constexpr int kTile = 64;                // rows streamed per iteration
    static constexpr int kLd = D + 8;
    static constexpr int kTileElems = kTile * kLd;
    static constexpr int kRowStatBytes = 2 * 2 * kTile * 4;   // lse2, delta double-buffered
    static constexpr int kLdsBytes = 2 * 2 * kTileElems * 2 + kRowStatBytes;
    static constexpr int kChunks = kTile * D / 8;
    static constexpr int kChunksPerThread = (kChunks + kThreads - 1) / kThreads;
    static_assert(kLdsBytes <= 160 * 1024, "LDS budget of a gfx950 CU exceeded");
};

// ---------------------------------------------------------------------------------------
// 2. dK, dV.  Work-group = NW waves, wave = 32 keys, loop over query tiles of 64 rows.
// ---------------------------------------------------------------------------------------
template <int D, int NW, bool CAUSAL>
__global__ void __launch_bounds__(NW * 64) attn_bwd_dkdv_kernel(const BwdArgs a)
{
    using C = BwdCfg<D, NW>;
    constexpr int KS = D / 16, DB = D / 32;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16 *Qs = reinterpret_cast<bf16 *>(smem);      // [2][64][kLd]
    bf16 *Gs = Qs + 2 * C::kTileElems;              // [2][64][kLd]  (dO)
    float *Ls = reinterpret_cast<float *>(Gs + 2 * C::kTileElems);  // [2][64] LSE*log2e
    float *Ds = Ls + 2 * C::kTile;                                  // [2][64] delta

    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, r = l & 31, h = l >> 5;
    const int S = a.S;
    ATTN_CYCLES_BEGIN();
    int bh, kt;  // causal: key block 0 is the heaviest
    xcd_heavy_first(blockIdx.x, a.ntile, a.BH, bh, kt);
    const int64_t base = (int64_t)(bh / a.H) * a.stride_b + (int64_t)(bh % a.H) * a.stride_h;
    const bf16 *Qp = a.Q + base, *Gp = a.dO + base;
    const float *Lp = a.LSE + (int64_t)bh * S, *Dp = a.delta + (int64_t)bh * S;

    const int k0 = kt * C::kBlk + w * 32;  // first key of this wave
    const int key = k0 + r;
    const int keyc = key < S ? key : S - 1;

    // K and V fragments (B operands): lane holds K[key][16ks + 8h .. +7].
    bf16x8 kf[KS], vf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        kf[ks] = as_bf16x8(ld_global16(a.K + base + (int64_t)keyc * a.stride_s + ks * 16 + 8 * h));
        vf[ks] = as_bf16x8(ld_global16(a.V + base + (int64_t)keyc * a.stride_s + ks * 16 + 8 * h));
    }

    const int n_qt = (S + C::kTile - 1) / C::kTile;
    const int qt_begin = CAUSAL ? (kt * C::kBlk) / C::kTile : 0;

    u32x4 qreg[C::kChunksPerThread], greg[C::kChunksPerThread];
    float lreg = 0.f, dreg = 0.f;
    auto prefetch = [&](int qt) {
#pragma unroll
        for (int n = 0; n < C::kChunksPerThread; ++n) {
            const int c = tid + n * C::kThreads;
            if (C::kChunks % C::kThreads == 0 || c < C::kChunks) {
                const int row = c / (D / 8), col = (c % (D / 8)) * 8;
                int qr = qt * C::kTile + row;
                qr = qr < S ? qr : S - 1;
                qreg[n] = ld_global16(Qp + (int64_t)qr * a.stride_s + col);
                greg[n] = ld_global16(Gp + (int64_t)qr * a.stride_s + col);
            }
        }
        if (tid < C::kTile) {
            int qr = qt * C::kTile + tid;
            qr = qr < S ? qr : S - 1;
            lreg = Lp[qr] * kLog2e;
            dreg = Dp[qr];
        }
    };
    auto commit = [&](int buf) {
#pragma unroll
        for (int n = 0; n < C::kChunksPerThread; ++n) {
            const int c = tid + n * C::kThreads;
            if (C::kChunks % C::kThreads == 0 || c < C::kChunks) {
                const int row = c / (D / 8), col = (c % (D / 8)) * 8;
                *(u32x4 *)(Qs + buf * C::kTileElems + row * C::kLd + col) = qreg[n];
                *(u32x4 *)(Gs + buf * C::kTileElems + row * C::kLd + col) = greg[n];
            }
        }
        if (tid < C::kTile) {
            Ls[buf * C::kTile + tid] = lreg;
            Ds[buf * C::kTile + tid] = dreg;
        }
    };

    f32x16 dv[DB], dk[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) { dv[db][i] = 0.f; dk[db][i] = 0.f; }

    const float c = a.scale_log2e;
    const int tr_row = 4 * h + ((l & 15) >> 2);
    const int tr_col = ((l >> 4) & 1) * 16 + (l & 3) * 4;

    if (qt_begin < n_qt) prefetch(qt_begin);
    for (int qt = qt_begin; qt < n_qt; ++qt) {
        const int buf = (qt - qt_begin) & 1;
        commit(buf);
        __syncthreads();
        if (qt + 1 < n_qt) prefetch(qt + 1);

        const bf16 *Qt = Qs + buf * C::kTileElems;
        const bf16 *Gt = Gs + buf * C::kTileElems;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const int q_lo = qt * C::kTile + qb * 32;
            // wave-uniform: some row of the block is a real row that sees some key of the wave
            const bool active = q_lo < S && (!CAUSAL || q_lo + 31 >= k0);
            if (!active) continue;
            f32x16 s, dp;
#pragma unroll
            for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 qa = *(const bf16x8 *)(Qt + (qb * 32 + r) * C::kLd + ks * 16 + 8 * h);
                const bf16x8 ga = *(const bf16x8 *)(Gt + (qb * 32 + r) * C::kLd + ks * 16 + 8 * h);
                s = mfma32(qa, kf[ks], s);
                dp = mfma32(ga, vf[ks], dp);
            }
            // register i <-> query row q_lo + 8*(i/4) + 4h + i%4; this lane's key is fixed
            const bool need_mask = (q_lo + 32 > S) || (CAUSAL && q_lo < k0 + 31);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 l4 = *(const f32x4 *)(Ls + buf * C::kTile + qb * 32 + 8 * g + 4 * h);
                const f32x4 d4 = *(const f32x4 *)(Ds + buf * C::kTile + qb * 32 + 8 * g + 4 * h);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int i = 4 * g + e;
                    float p = fast_exp2(__builtin_fmaf(s[i], c, -l4[e]));
                    if (need_mask) {
                        const int qi = q_lo + 8 * g + 4 * h + e;
                        if (qi >= S || (CAUSAL && key > qi)) p = 0.f;
                    }
                    s[i] = p;
                    dp[i] = p * (dp[i] - d4[e]);
                }
            }
            bf16x8 pb[2], sb[2];
            pb[0] = pack8(s[0], s[1], s[2], s[3], s[4], s[5], s[6], s[7]);
            pb[1] = pack8(s[8], s[9], s[10], s[11], s[12], s[13], s[14], s[15]);
            sb[0] = pack8(dp[0], dp[1], dp[2], dp[3], dp[4], dp[5], dp[6], dp[7]);
            sb[1] = pack8(dp[8], dp[9], dp[10], dp[11], dp[12], dp[13], dp[14], dp[15]);
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const int off = (qb * 32 + 16 * cc + tr_row) * C::kLd + 32 * db + tr_col;
                    const bf16x8 gT = join8(lds_read_tr(Gt + off), lds_read_tr(Gt + off + 8 * C::kLd));
                    dv[db] = mfma32(gT, pb[cc], dv[db]);
                    const bf16x8 qT = join8(lds_read_tr(Qt + off), lds_read_tr(Qt + off + 8 * C::kLd));
                    dk[db] = mfma32(qT, sb[cc], dk[db]);
                }
            }
        }
    }

    if (key < S) {
        bf16 *dKp = a.dK + base + (int64_t)key * a.stride_s;
        bf16 *dVp = a.dV + base + (int64_t)key * a.stride_s;
        const float sc = a.scale;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int col = 32 * db + 8 * g + 4 * h;
                *(bf16x4 *)(dVp + col) = pack4(dv[db][4 * g], dv[db][4 * g + 1],
                                               dv[db][4 * g + 2], dv[db][4 * g + 3]);
                *(bf16x4 *)(dKp + col) = pack4(dk[db][4 * g] * sc, dk[db][4 * g + 1] * sc,
                                               dk[db][4 * g + 2] * sc, dk[db][4 * g + 3] * sc);
            }
    }
    ATTN_CYCLES_END(1);
}

// ---------------------------------------------------------------------------------------
// 3. dQ.  Work-group = NW waves, wave = 32 queries, loop over key tiles of 64 rows.
// ---------------------------------------------------------------------------------------
template <int D, int NW, bool CAUSAL>
__global__ void __launch_bounds__(NW * 64) attn_bwd_dq_kernel(const BwdArgs a)
{
    using C = BwdCfg<D, NW>;
    constexpr int KS = D / 16, DB = D / 32;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16 *Ks = reinterpret_cast<bf16 *>(smem);  // [2][64][kLd]
    bf16 *Vs = Ks + 2 * C::kTileElems;          // [2][64][kLd]

    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, r = l & 31, h = l >> 5;
    const int S = a.S;
    ATTN_CYCLES_BEGIN();
    int bh, rank;
    xcd_heavy_first(blockIdx.x, a.ntile, a.BH, bh, rank);
    const int qt = CAUSAL ? a.ntile - 1 - rank : rank;  // heaviest first
    const int64_t base = (int64_t)(bh / a.H) * a.stride_b + (int64_t)(bh % a.H) * a.stride_h;
    const bf16 *Kp = a.K + base, *Vp = a.V + base;

    const int q0 = qt * C::kBlk + w * 32;
    const int q = q0 + r;
    const int qc = q < S ? q : S - 1;

    bf16x8 qf[KS], gf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        qf[ks] = as_bf16x8(ld_global16(a.Q + base + (int64_t)qc * a.stride_s + ks * 16 + 8 * h));
        gf[ks] = as_bf16x8(ld_global16(a.dO + base + (int64_t)qc * a.stride_s + ks * 16 + 8 * h));
    }
    const float lse2 = a.LSE[(int64_t)bh * S + qc] * kLog2e;
    const float delta = a.delta[(int64_t)bh * S + qc];

    const int q_end = min(S, (qt + 1) * C::kBlk);
    const int n_kt = ((CAUSAL ? q_end : S) + C::kTile - 1) / C::kTile;

    u32x4 kreg[C::kChunksPerThread], vreg[C::kChunksPerThread];
    auto prefetch = [&](int kt) {
#pragma unroll
        for (int n = 0; n < C::kChunksPerThread; ++n) {
            const int c = tid + n * C::kThreads;
            if (C::kChunks % C::kThreads == 0 || c < C::kChunks) {
                const int row = c / (D / 8), col = (c % (D / 8)) * 8;
                int kr = kt * C::kTile + row;
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

    f32x16 dq[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) dq[db][i] = 0.f;

    const float c = a.scale_log2e;
    const int tr_row = 4 * h + ((l & 15) >> 2);
    const int tr_col = ((l >> 4) & 1) * 16 + (l & 3) * 4;

    prefetch(0);
    for (int kt = 0; kt < n_kt; ++kt) {
        const int buf = kt & 1;
        commit(buf);
        __syncthreads();
        if (kt + 1 < n_kt) prefetch(kt + 1);

        const bf16 *Kt = Ks + buf * C::kTileElems;
        const bf16 *Vt = Vs + buf * C::kTileElems;
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2) {
            const int k_lo = kt * C::kTile + kb2 * 32;
            const bool active = k_lo < S && (!CAUSAL || k_lo <= q0 + 31);  // wave-uniform
            if (!active) continue;
            f32x16 s, dp;
#pragma unroll
            for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 ka = *(const bf16x8 *)(Kt + (kb2 * 32 + r) * C::kLd + ks * 16 + 8 * h);
                const bf16x8 va = *(const bf16x8 *)(Vt + (kb2 * 32 + r) * C::kLd + ks * 16 + 8 * h);
                s = mfma32(ka, qf[ks], s);
                dp = mfma32(va, gf[ks], dp);
            }
            // register i <-> key k_lo + 8*(i/4) + 4h + i%4; this lane's query is fixed
            const bool need_mask = (k_lo + 32 > S) || (CAUSAL && k_lo + 31 > q0);
            const int lim = (CAUSAL ? qc : S - 1) - k_lo - 4 * h;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float p = fast_exp2(__builtin_fmaf(s[i], c, -lse2));
                if (need_mask && (8 * (i / 4) + (i % 4) > lim)) p = 0.f;
                dp[i] = p * (dp[i] - delta);
            }
            bf16x8 sb[2];
            sb[0] = pack8(dp[0], dp[1], dp[2], dp[3], dp[4], dp[5], dp[6], dp[7]);
            sb[1] = pack8(dp[8], dp[9], dp[10], dp[11], dp[12], dp[13], dp[14], dp[15]);
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const int off = (kb2 * 32 + 16 * cc + tr_row) * C::kLd + 32 * db + tr_col;
                    const bf16x8 kT = join8(lds_read_tr(Kt + off), lds_read_tr(Kt + off + 8 * C::kLd));
                    dq[db] = mfma32(kT, sb[cc], dq[db]);
                }
            }
        }
    }

    if (q < S) {
        bf16 *dQp = a.dQ + base + (int64_t)q * a.stride_s;
        const float sc = a.scale;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                *(bf16x4 *)(dQp + 32 * db + 8 * g + 4 * h) =
                    pack4(dq[db][4 * g] * sc, dq[db][4 * g + 1] * sc,
                          dq[db][4 * g + 2] * sc, dq[db][4 * g + 3] * sc);
    }
    ATTN_CYCLES_END(2);
}

// ---------------------------------------------------------------------------------------
// Launch
// ---------------------------------------------------------------------------------------
template <typename K>
static void allow_lds(K kernel, int bytes)
{
    hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

template <int D, int NW, bool CAUSAL>
static int launch_bwd_main(BwdArgs a, hipStream_t st, unsigned stages)
{
    using C = BwdCfg<D, NW>;
    a.ntile = (a.S + C::kBlk - 1) / C::kBlk;
    const dim3 grid(a.ntile * a.BH), block(C::kThreads);
    if (stages & 2u) {
        allow_lds(attn_bwd_dkdv_kernel<D, NW, CAUSAL>, C::kLdsBytes);
        hipLaunchKernelGGL((attn_bwd_dkdv_kernel<D, NW, CAUSAL>), grid, block, C::kLdsBytes, st, a);
    }
    if (stages & 4u) {
        allow_lds(attn_bwd_dq_kernel<D, NW, CAUSAL>, C::kLdsBytes);
        hipLaunchKernelGGL((attn_bwd_dq_kernel<D, NW, CAUSAL>), grid, block, C::kLdsBytes, st, a);
    }
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <int D, int NW>
static int launch_bwd_nw(const BwdArgs &a, bool causal, hipStream_t st, unsigned stages)
{
    return causal ? launch_bwd_main<D, NW, true>(a, st, stages)
                  : launch_bwd_main<D, NW, false>(a, st, stages);
}

template <int D>
static int launch_bwd_d(const BwdArgs &a, bool causal, hipStream_t st, unsigned stages)
{
    if (stages & 1u) {
        constexpr int RPB = 256 / (D / 8);
        const int64_t rows = (int64_t)a.BH * a.S;
        hipLaunchKernelGGL((attn_bwd_delta_kernel<D>), dim3((unsigned)((rows + RPB - 1) / RPB)),
                           dim3(256), 0, st, a);
        if (hipGetLastError() != hipSuccess) return -1;
    }
    if (!(stages & 6u)) return 0;
    const int blocks32 = (a.S + 31) / 32;
    if (blocks32 >= 8) return launch_bwd_nw<D, 8>(a, causal, st, stages);
    if (blocks32 >= 4) return launch_bwd_nw<D, 4>(a, causal, st, stages);
    if (blocks32 == 3) return launch_bwd_nw<D, 3>(a, causal, st, stages);
    if (blocks32 == 2) return launch_bwd_nw<D, 2>(a, causal, st, stages);
    return launch_bwd_nw<D, 1>(a, causal, st, stages);
}

#ifdef ATTN_CYCLES
extern "C" void attn_debug_cycles_bwd(unsigned long long *out, int reset)
{
    hipMemcpyFromSymbol(out, HIP_SYMBOL(g_attn_cycles), sizeof(g_attn_cycles));
    if (reset) { unsigned long long z[4][4] = {}; hipMemcpyToSymbol(HIP_SYMBOL(g_attn_cycles), z, sizeof(z)); }
}
#endif

int launch_bwd(const BwdArgs &a, int D, bool causal, hipStream_t st, unsigned stages)
{
    return D == 128 ? launch_bwd_d<128>(a, causal, st, stages)
                    : launch_bwd_d<64>(a, causal, st, stages);
}

}  // namespace attn
