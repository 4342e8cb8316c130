// Fused attention backward for short sequences on gfx950: when a head's query rows and keys
// both fit 128, ONE work-group per head computes dQ, dK and dV in one launch.  The two-kernel
// backward of attn_bwd.hip spends most of its time on such shapes in two launches and in
// reading the head's tensors twice; here Q, K, V and dO are brought into LDS once (direct
// global -> LDS transfers), and nothing is exchanged between work-groups.
//
// Wave w (of up to four) owns query block w (32 rows) and key block w (32 keys):
//   as the owner of query block i (the dQ kernel's orientation, one query per lane):
//     for every key block j:  S^T = K_j Q_i^T,  dP^T = V_j dO_i^T - delta,  P, dS,
//                             dQ_i^T += K_j^T dS^T
//   as the owner of key block j (the dK/dV kernel's orientation, one key per lane):
//     for every query block i:  S = Q_i K_j^T,  dP = dO_i V_j^T - delta,  P, dS,
//                               dV_j^T += dO_i^T P,  dK_j^T += Q_i^T dS
// P and dS stay in registers in both parts (their accumulator layout is the B-operand layout of
// the GEMM that consumes them).  The row statistics (delta, LSE in log2 units) are formed by the
// owners of the query blocks and shared through LDS; that is the only barrier after the tiles
// have landed.  With grouped-query heads the work-group owns a K/V head and walks the query heads
// that read it one after the other (their Q and dO tiles replace each other in LDS; dK and dV
// accumulate across them).
#include "attn_device.hpp"
#include "attn_launch.hpp"

namespace attn {

template <int D, int NW>
struct SmallCfg {
    static constexpr int kWaves = NW;                          // 4, or 8 (D = 64 only)
    static constexpr int kMaxRows = 32 * NW;                   // query rows and keys per head
    static constexpr int kThreads = kWaves * 64;
    static constexpr int kRowBytes = D * 2;
    static constexpr int kCPR = D / 8;                         // 16-byte chunks per row
    static constexpr int kPieceRows = 1024 / kRowBytes;        // rows one 1 KB transfer fills
    // LDS: lse2[kMaxRows], -delta[kMaxRows], then Q, dO, K, V, each padded to whole 32-row blocks of the
    // longer of the two lengths (sized at launch: three work-groups of the 65-row shape fit a
    // compute unit that way).  Rows are stored unpadded with the 16-byte chunk index XOR-swizzled
    // by the row, as in the slots of the dK/dV kernel: conflict free for row reads and for
    // transpose reads.
    static constexpr int kStatBytes = 2 * kMaxRows * 4;
    static constexpr int lds_bytes(int rows_pad) { return kStatBytes + 4 * rows_pad * kRowBytes; }
    static_assert(lds_bytes(kMaxRows) <= 160 * 1024, "LDS budget of a gfx950 CU exceeded");
};

template <int D, int NW, bool CAUSAL, bool GQA>
// (D = 64, four waves, one query head per K/V head: at most 168 registers, so that three
// work-groups share a compute unit; with grouped heads the dK/dV accumulators stay live while dQ
// of the next query head is formed, which takes more)
__global__ void __launch_bounds__(NW * 64)
    __attribute__((amdgpu_waves_per_eu(D == 64 ? (NW == 4 && !GQA ? 3 : 2) : 1)))
attn_bwd_small_kernel(const BwdArgs a)
{
    using C = SmallCfg<D, NW>;
    constexpr int KS = D / 16, DB = D / 32, PR = C::kPieceRows, CPR = C::kCPR, RB = C::kRowBytes;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int tid = threadIdx.x, l = tid & 63, r = l & 31, h = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int S = a.S, Sk = a.Sk, Dr = a.Dr;
    const int coff = Sk - S;  // causal: query row i sees keys 0 .. i + coff
    // the work-group owns one K/V head and sums dK, dV over the `group` query heads that read it
    const int Hkv = a.H / a.group, bkv = blockIdx.x;
    const int64_t base_kv = (int64_t)(bkv / Hkv) * a.kv_stride_b + (int64_t)(bkv % Hkv) * a.kv_stride_h;
    const int bh0 = (bkv / Hkv) * a.H + (bkv % Hkv) * a.group;  // first query head of the group
    const int nqb = (S + 31) / 32, nkb = (Sk + 31) / 32;  // query / key blocks of the head
    const int tensor_bytes = 32 * max(nqb, nkb) * RB;
    const int offQ = C::kStatBytes, offG = offQ + tensor_bytes, offK = offG + tensor_bytes, offV = offK + tensor_bytes;
    // chunk position swizzle: rows 0..15 get 16 distinct values (row reads of 16 lanes hit 16
    // different 16-byte bank groups) and 4 consecutive rows differ in the upper two bits (the
    // 4 rows x 64 bytes of a transpose read spread over all banks)
    auto swz = [](int row) {
        return CPR >= 16 ? (((row & 3) << 2) | ((row >> 2) & 3))
                         : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
    };

    // ---- the four tensors -> LDS.  Rows past the end and columns Dr..D-1 lie outside the
    // buffer resources and read as zero.
    const uint32_t q_bytes = (uint32_t)(((int64_t)(S - 1) * a.stride_s + Dr) * 2);
    const uint32_t k_bytes = (uint32_t)(((int64_t)(Sk - 1) * a.kv_stride_s + Dr) * 2);
    const desc_t Kd = make_desc(a.K + base_kv, k_bytes), Vd = make_desc(a.V + base_kv, k_bytes);
    const uint32_t lds0 = lds_address(smem);
    const uint32_t q_row = (uint32_t)a.stride_s * 2u, k_row = (uint32_t)a.kv_stride_s * 2u;
    // a transfer fills 1 KB = PR rows in lane order: lane l lands in row l / CPR of the piece, at
    // chunk position l % CPR, and fetches the chunk that the swizzle puts there
    auto voff = [&](int piece, uint32_t row_bytes, uint32_t end) {
        const int row = piece * PR + l / CPR;
        const int chunk = (l % CPR) ^ swz(row);
        return chunk * 8 < Dr ? (uint32_t)(l / CPR) * row_bytes + ((uint32_t)chunk << 4) : end;
    };
    const int q_pieces = nqb * (32 / PR), k_pieces = nkb * (32 / PR);
    for (int i = w; i < k_pieces; i += C::kWaves) {
        const uint32_t vo = voff(i, k_row, k_bytes);
        dma16(Kd, lds0 + offK + i * 1024, vo, i * PR * k_row);
        dma16(Vd, lds0 + offV + i * 1024, vo, i * PR * k_row);
    }

    const int q = 32 * w + r, qc = q < S ? q : S - 1;
    const int key = 32 * w + r, keyc = key < Sk ? key : Sk - 1;
    f32x16 dk[DB], dv[DB];  // part 2's accumulators, summed over the query heads of the group
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) dk[db][i] = dv[db][i] = 0.f;

    const int n_heads = GQA ? a.group : 1;
    for (int gq = 0; gq < n_heads; ++gq) {
    const int bh = bh0 + gq;
    const int64_t base = (int64_t)(bh / a.H) * a.stride_b + (int64_t)(bh % a.H) * a.stride_h;
    // every wave is done with the previous query head's tiles and statistics
    if (GQA && gq > 0) __syncthreads();
    {
        const desc_t Qd = make_desc(a.Q + base, q_bytes), Gd = make_desc(a.dO + base, q_bytes);
        for (int i = w; i < q_pieces; i += C::kWaves) {
            const uint32_t vo = voff(i, q_row, q_bytes);
            dma16(Qd, lds0 + offQ + i * 1024, vo, i * PR * q_row);
            dma16(Gd, lds0 + offG + i * 1024, vo, i * PR * q_row);
        }
    }
    // ---- this wave's query block: Q and dO fragments (B operands: lane holds row q, columns
    // 16 ks + 8 h .. +7) and the row statistics, as in the dQ kernel
    elem8 qf[KS], gf[KS];
    float lse2 = 0.f, ndelta = 0.f;
    if (w < nqb) {
        float acc = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qf[ks] = as_elem8(ld_row16(a.Q + base + (int64_t)qc * a.stride_s, ks * 16 + 8 * h, Dr));
            gf[ks] = as_elem8(ld_row16(a.dO + base + (int64_t)qc * a.stride_s, ks * 16 + 8 * h, Dr));
            const elem8 of = as_elem8(ld_row16(a.O + base + (int64_t)qc * a.stride_s, ks * 16 + 8 * h, Dr));
#pragma unroll
            for (int t = 0; t < 8; ++t) acc += (float)of[t] * (float)gf[ks][t];
        }
        ndelta = -xhalf_sum(acc);
        lse2 = a.LSE[(int64_t)bh * S + qc] * kLog2e;
        if (h == 0) {
            float *st = reinterpret_cast<float *>(smem);
            st[q] = lse2;
            st[C::kMaxRows + q] = ndelta;
            if (q < S) {  // the workspace receives them as it does from the two-kernel backward
                a.delta[(int64_t)bh * 2 * S + q] = ndelta;
                a.delta[(int64_t)bh * 2 * S + S + q] = lse2;
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    const float c = a.scale_log2e;
    // per-lane LDS offsets within a 32-row block: row fragment = chunk 2 ks + h of row r (the
    // step enters by XOR: ^ (ks * 32)); transpose reads = rows 4h + e (+8), 64 bytes of d block 0
    // of each row (d block db flips bits 6.. of the swizzled offset)
    const int row_lane = r * RB + ((h ^ swz(r)) << 4);
    int tr_lane[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int row = 8 * j + 4 * h + ((l & 15) >> 2);
        const int chunk = 2 * ((l >> 4) & 1) + ((l >> 1) & 1);
        tr_lane[j] = row * RB + ((chunk ^ swz(row)) << 4) + (l & 1) * 8;
    }
    // A operand = rows [32 blk, 32 blk + 32) of a tensor, contraction step ks
    auto row_frag = [&](int tensor_off, int blk, int ks) {
        return *(const elem8 *)(smem + tensor_off + blk * 32 * RB + (row_lane ^ (ks * 32)));
    };
    // A operand = the transpose of 16 rows (16-row step cc of block blk), d block db
    auto tr_frag = [&](int tensor_off, int blk, int cc, int db) {
        const char *p = smem + tensor_off + (blk * 2 + cc) * 16 * RB;
        return join8(lds_read_tr((const elem *)(p + (tr_lane[0] ^ (db << 6)))),
                     lds_read_tr((const elem *)(p + (tr_lane[1] ^ (db << 6)))));
    };

    // ---- part 1: dQ of query block w
    if (w < nqb) {
        f32x16 nd, dq[DB];
#pragma unroll
        for (int i = 0; i < 16; ++i) nd[i] = ndelta;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) dq[db][i] = 0.f;
        const int q0e = 32 * w + coff;  // the wave's first row in key coordinates
        for (int j = 0; j < nkb; ++j) {
            const int k_lo = 32 * j;
            if (CAUSAL && k_lo > q0e + 31) break;  // wholly above the diagonal
            f32x16 s, dp = nd;  // register i <-> key k_lo + 8*(i/4) + 4h + i%4 (this lane's query is fixed)
#pragma unroll
            for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                s = mfma32(row_frag(offK, j, ks), qf[ks], s);
                dp = mfma32(row_frag(offV, j, ks), gf[ks], dp);  // ends as dP - delta
            }
            const int lim = (CAUSAL ? min(qc + coff, Sk - 1) : Sk - 1) - k_lo - 4 * h;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float p = fast_exp2(__builtin_fmaf(s[i], c, -lse2));
                dp[i] *= (8 * (i / 4) + (i % 4) > lim) ? 0.f : p;  // dS = P o (dP - delta)
            }
            const elem8 sb[2] = {pack8(dp[0], dp[1], dp[2], dp[3], dp[4], dp[5], dp[6], dp[7]),
                                 pack8(dp[8], dp[9], dp[10], dp[11], dp[12], dp[13], dp[14], dp[15])};
#pragma unroll
            for (int cc = 0; cc < 2; ++cc)
#pragma unroll
                for (int db = 0; db < DB; ++db) dq[db] = mfma32(tr_frag(offK, j, cc, db), sb[cc], dq[db]);
        }
        if (a.rope_cos) {
            // Q was rotated before the forward: what has been accumulated is the gradient of the
            // rotated rows; the gradient of the unrotated ones is its image under the transpose of
            // the rotation (head dimension == D; column d pairs with d + D/2, i.e. d block db with
            // db + DB/2, same register) -- as in the dQ kernel's epilogue
            const int64_t pos = (int64_t)(qc + a.rope_pos0) * (D / 2);
#pragma unroll
            for (int db = 0; db < DB / 2; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 c4 = *(const f32x4 *)(a.rope_cos + pos + 32 * db + 8 * g + 4 * h);
                    const f32x4 s4 = *(const f32x4 *)(a.rope_sin + pos + 32 * db + 8 * g + 4 * h);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float y1 = dq[db][4 * g + e], y2 = dq[db + DB / 2][4 * g + e];
                        dq[db][4 * g + e] = __builtin_fmaf(y1, c4[e], y2 * s4[e]);
                        dq[db + DB / 2][4 * g + e] = __builtin_fmaf(y2, c4[e], -(y1 * s4[e]));
                    }
                }
        }
        if (q < S) {
            elem *dQp = a.dQ + base + (int64_t)q * a.stride_s;
            const float sc = a.scale;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    if (32 * db + 8 * g + 4 * h < Dr)
                        *(elem4 *)(dQp + 32 * db + 8 * g + 4 * h) =
                            pack4(dq[db][4 * g] * sc, dq[db][4 * g + 1] * sc,
                                  dq[db][4 * g + 2] * sc, dq[db][4 * g + 3] * sc);
        }
    }

    // ---- part 2: dK and dV of key block w
    if (w < nkb) {
        elem8 kf[KS], vf[KS];  // B operands: lane holds row `key`, columns 16 ks + 8 h .. +7
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int o = keyc * RB + (((2 * ks + h) ^ swz(keyc)) << 4);
            kf[ks] = *(const elem8 *)(smem + offK + o);
            vf[ks] = *(const elem8 *)(smem + offV + o);
        }
        const float *st = reinterpret_cast<const float *>(smem);
        // first query block with a row that sees a key of this block (row >= key - coff)
        const int i0 = CAUSAL ? max(0, 32 * w - coff) / 32 : 0;
        for (int i = i0; i < nqb; ++i) {
            const int q_lo = 32 * i;
            // register t <-> query row q_lo + 8*(t/4) + 4h + t%4 (this lane's key is fixed); the
            // dP accumulator starts from -delta of its row
            f32x16 s, dp;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 d4 = *(const f32x4 *)(st + C::kMaxRows + q_lo + 8 * g + 4 * h);
#pragma unroll
                for (int e = 0; e < 4; ++e) { dp[4 * g + e] = d4[e]; s[4 * g + e] = 0.f; }
            }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                s = mfma32(row_frag(offQ, i, ks), kf[ks], s);
                dp = mfma32(row_frag(offG, i, ks), vf[ks], dp);
            }
            // visible row offsets: >= key - coff - q_lo (causal) and <= S - 1 - q_lo; keys past
            // the end see nothing
            const int lo = (CAUSAL ? key - coff - q_lo : -64) - 4 * h;
            const int hi = (key < Sk ? S - 1 - q_lo : -64) - 4 * h;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 l4 = *(const f32x4 *)(st + q_lo + 8 * g + 4 * h);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int ro = 8 * g + e;
                    const float p = fast_exp2(__builtin_fmaf(s[4 * g + e], c, -l4[e]));
                    s[4 * g + e] = (ro < lo || ro > hi) ? 0.f : p;
                }
            }
#pragma unroll
            for (int t = 0; t < 16; ++t) dp[t] *= s[t];  // dS = P o (dP - delta)
            const elem8 pb[2] = {pack8(s[0], s[1], s[2], s[3], s[4], s[5], s[6], s[7]),
                                 pack8(s[8], s[9], s[10], s[11], s[12], s[13], s[14], s[15])};
            const elem8 sb[2] = {pack8(dp[0], dp[1], dp[2], dp[3], dp[4], dp[5], dp[6], dp[7]),
                                 pack8(dp[8], dp[9], dp[10], dp[11], dp[12], dp[13], dp[14], dp[15])};
#pragma unroll
            for (int cc = 0; cc < 2; ++cc)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    dv[db] = mfma32(tr_frag(offG, i, cc, db), pb[cc], dv[db]);
                    dk[db] = mfma32(tr_frag(offQ, i, cc, db), sb[cc], dk[db]);
                }
        }
    }
    }  // query heads of the group

    // dK and dV.  The accumulators hold 4 consecutive columns of one key per register group, so a
    // direct store writes 8-byte pieces of 32 rows per instruction.  Where the registers allow
    // it (not the 168-register four-wave form at D = 64, nor the grouped-head forms, which spill
    // and measure slower with it) the rows of key block w go through block w of the Q tensor's
    // space, once every wave is done with the tensors in LDS, and leave whole, 16 bytes per lane
    // (same box: B=32 H=8 S=256 D=64 causal 25.7 -> 24.5 us, B=64 H=8 S=128 D=128 causal 48.2 ->
    // 45.9).
    constexpr bool kStageOut = !GQA && !(D == 64 && NW == 4);
    if constexpr (kStageOut) {
        __syncthreads();
        if (w < nkb) {
            constexpr int RPI = 64 / CPR;  // rows per store instruction
            char *stg = smem + offQ + w * 32 * RB;
            const int lr = l / CPR, lc = l % CPR;
            const float sc = a.scale;
#pragma unroll
            for (int t = 0; t < 2; ++t) {  // dK, then dV
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        *(elem4 *)(stg + r * RB + (((4 * db + g) ^ swz(r)) << 4) + 8 * h) =
                            t == 0 ? pack4(dk[db][4 * g] * sc, dk[db][4 * g + 1] * sc, dk[db][4 * g + 2] * sc,
                                           dk[db][4 * g + 3] * sc)
                                   : pack4(dv[db][4 * g], dv[db][4 * g + 1], dv[db][4 * g + 2], dv[db][4 * g + 3]);
                asm volatile("" ::: "memory");  // a wave's LDS accesses execute in order
                elem *out = (t == 0 ? a.dK : a.dV) + base_kv;
#pragma unroll
                for (int j = 0; j < 32 / RPI; ++j) {
                    const int row = RPI * j + lr;
                    const u32x4 v = *(const u32x4 *)(stg + row * RB + ((lc ^ swz(row)) << 4));
                    const int okey = 32 * w + row;
                    if (okey < Sk && lc * 8 < Dr) *(u32x4 *)(out + (int64_t)okey * a.kv_stride_s + lc * 8) = v;
                }
                asm volatile("" ::: "memory");
            }
        }
        return;
    }
    if (w < nkb) {
        if (key < Sk) {
            elem *dKp = a.dK + base_kv + (int64_t)key * a.kv_stride_s;
            elem *dVp = a.dV + base_kv + (int64_t)key * a.kv_stride_s;
            const float sc = a.scale;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    if (32 * db + 8 * g + 4 * h < Dr) {
                        *(elem4 *)(dKp + 32 * db + 8 * g + 4 * h) =
                            pack4(dk[db][4 * g] * sc, dk[db][4 * g + 1] * sc,
                                  dk[db][4 * g + 2] * sc, dk[db][4 * g + 3] * sc);
                        *(elem4 *)(dVp + 32 * db + 8 * g + 4 * h) =
                            pack4(dv[db][4 * g], dv[db][4 * g + 1], dv[db][4 * g + 2], dv[db][4 * g + 3]);
                    }
        }
    }
}

template <int D, int NW, bool CAUSAL, bool GQA>
static int launch_small_g(const BwdArgs &a, hipStream_t st)
{
    using C = SmallCfg<D, NW>;
    const int rows_pad = ((a.S > a.Sk ? a.S : a.Sk) + 31) / 32 * 32;
    if (hipFuncSetAttribute((const void *)attn_bwd_small_kernel<D, NW, CAUSAL, GQA>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, C::lds_bytes(C::kMaxRows)) != hipSuccess)
        return -1;
    hipLaunchKernelGGL((attn_bwd_small_kernel<D, NW, CAUSAL, GQA>), dim3(a.BH / a.group), dim3(C::kThreads),
                       C::lds_bytes(rows_pad), st, a);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <int D, int NW, bool CAUSAL>
static int launch_small(const BwdArgs &a, hipStream_t st)
{
    return a.group > 1 ? launch_small_g<D, NW, CAUSAL, true>(a, st) : launch_small_g<D, NW, CAUSAL, false>(a, st);
}

#ifndef ATTN_F16  // a function of the head dimension only: defined once, by the bf16 build
// Longest head (query rows and keys) the fused form takes at kernel head dimension D.
int bwd_small_max_rows(int D) { return D == 64 ? 256 : D == 128 ? 128 : 0; }
#endif

// Whole backward of a problem whose heads have at most bwd_small_max_rows(D) query rows and keys
// (the caller checks).
int launch_bwd_small(const BwdArgs &a, int D, bool causal, hipStream_t st)
{
    const int rows = a.S > a.Sk ? a.S : a.Sk;
    if (rows > bwd_small_max_rows(D)) return -1;
    if (D == 128) return causal ? launch_small<128, 4, true>(a, st) : launch_small<128, 4, false>(a, st);
    if (rows <= 128) return causal ? launch_small<64, 4, true>(a, st) : launch_small<64, 4, false>(a, st);
    return causal ? launch_small<64, 8, true>(a, st) : launch_small<64, 8, false>(a, st);
}

}  // namespace attn
