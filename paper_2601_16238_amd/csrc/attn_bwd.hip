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
// 1. Row statistics, fp32, workspace layout [B*H][2][S]: -delta = -rowsum(dO * O), then
// lse2 = LSE * log2(e) (the main kernels run the softmax on exp2).  delta is stored negated
// because the main kernels start the dP = dO V^T accumulation from it, which yields
// dP - delta without a subtraction per element.  D/8 lanes per row,
// 16-byte loads.
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
        if (sub * 8 < a.Dr) {  // lanes past the tensors' head dimension add nothing
            const elem8 o = as_elem8(ld_global16(a.O + off));
            const elem8 g = as_elem8(ld_global16(a.dO + off));
#pragma unroll
            for (int t = 0; t < 8; ++t) acc += (float)o[t] * (float)g[t];
        }
    }
#pragma unroll
    for (int s = LPR / 2; s >= 1; s >>= 1) acc += __shfl_xor(acc, s);
    if (row < rows && sub == 0) {
        const int64_t bh = row / a.S, i = row % a.S;
        a.delta[(2 * bh) * a.S + i] = -acc;  // negated: it seeds the dP accumulators
        a.delta[(2 * bh + 1) * a.S + i] = a.LSE[row] * kLog2e;
    }
}

// ---------------------------------------------------------------------------------------
// 2. dK, dV.  Work-group = 2P waves = P producers (waves 0 .. P-1) + P consumers (P = 4: two
// waves per SIMD; P = 6 at D = 128: three); it owns 32 P keys and streams the head's Q and dO
// rows through LDS in slots of 32 rows.
// The K/V fragments plus two 32 x D fp32 accumulators do not fit one wave's registers, and a
// wave alternating between the exp-heavy and the accumulate-heavy half cannot overlap them, so
// the halves go to different waves:
//   producer p, slot t:   32 keys; S = Q K^T, dP = dO V^T, P = exp2(c S - lse2),
//                         dS = P o (dP - delta); elem P and dS -> LDS exchange
//   consumer, slot t-1:   64 keys (two producers) and ONE output: even consumers
//                         dV^T += dO^T P, odd ones dK^T += Q^T dS; every transposed
//                         LDS fragment feeds two MFMAs (one per 32-key block)
// Both issue 16 MFMAs per slot (D = 128); the producers' VALU work overlaps the consumers'
// MFMAs on the shared SIMD.  One barrier per slot.
//
// Q/dO slots go global -> LDS directly, kAhead slots ahead, into a ring of kAhead + 2 slots
// (the producer's, the consumer's, and those in flight), requested by the consumers; rows are
// stored unpadded with the 16-byte chunk index XOR-swizzled by the row so that both the
// producer's row reads and the consumer's transpose reads are bank-conflict free.
// ---------------------------------------------------------------------------------------
template <int D, int P>
struct DkdvCfg {
    static constexpr int kPairs = P;                 // producer/consumer pairs: 4, or 6 (three waves per SIMD)
    static constexpr int kWaves = 2 * kPairs;
    static constexpr int kThreads = kWaves * 64;
    static constexpr int kBlk = kPairs * 32;         // keys owned by the work-group
    static constexpr int kRows = 32;                 // query rows per slot
    // slots requested ahead of the producer (a slot of D = 256 is 32 KB: one fewer fits)
    static constexpr int kAhead = D > 128 ? 2 : 3;
    static constexpr int kRing = kAhead + 2;
    static constexpr int kRowBytes = D * 2;
    static constexpr int kTensorBytes = kRows * kRowBytes;   // Q part of a slot; dO follows
    static constexpr int kSlotBytes = 2 * kTensorBytes;
    static constexpr int kStatBytes = 2 * kRows * 4;         // lse2[32], delta[32]
    static constexpr int kXchgBytes = 2 * kPairs * 4 * 1024; // [2][pair][P0,P1,dS0,dS1][64] x 16 B
    static constexpr int kOffStat = kRing * kSlotBytes;
    static constexpr int kOffXchg = kOffStat + kRing * kStatBytes;
    static constexpr int kLdsBytes = kOffXchg + kXchgBytes;
    static constexpr int kDmaPerTensor = kTensorBytes / 1024; // wave-wide 1 KB transfers
    // transfers of a slot that one consumer requests: its share of the Q pieces, then of the dO pieces
    static constexpr int kDmaPerWave = 2 * ((kDmaPerTensor + kPairs - 1) / kPairs);
    // the producer that also fetches the stats (six pairs: waves 2 and 3 are the only producers on
    // their SIMDs, waves 0/4 and 1/5 share one; -0.3..0.6 %)
    static constexpr int kStatWave = kPairs == 6 ? 3 : kPairs - 1;
    static_assert(kOffXchg % 16 == 0 && kLdsBytes <= 160 * 1024, "LDS layout");
};

template <int D, int P, bool CAUSAL>
__global__ void __launch_bounds__(P * 128) __attribute__((amdgpu_waves_per_eu(P >= 4 ? P / 2 : 1)))
attn_bwd_dkdv_kernel(const BwdArgs a)
{
    using C = DkdvCfg<D, P>;
    constexpr int KS = D / 16, DB = D / 32, CPR = D / 8, RB = C::kRowBytes;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int tid = threadIdx.x, l = tid & 63, r = l & 31, h = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool producer = w < C::kPairs;
    const int pair = w < C::kPairs ? w : w - C::kPairs;
    const int S = a.S;
    // The work-group owns 128 keys of one K/V head and sums over the `group` query heads that
    // read it (grouped-query attention; group == 1 is multi-head attention).
    const int Hkv = a.H / a.group;
    int bkv, kt;  // causal: key block 0 is the heaviest
    xcd_tile_order<CAUSAL>(blockIdx.x, a.ntile, a.BH / a.group, bkv, kt);
    const int64_t base_kv = (int64_t)(bkv / Hkv) * a.kv_stride_b + (int64_t)(bkv % Hkv) * a.kv_stride_h;
    const int bh0 = (bkv / Hkv) * a.H + (bkv % Hkv) * a.group;  // first query head of the group

    const int Sk = a.Sk;          // key/value rows; S is the number of query rows
    const int coff = Sk - S;      // causal: query row i sees keys 0 .. i + coff
    const int k0 = kt * C::kBlk + pair * 32;  // first key of this pair
    const int key = k0 + r;
    const int n_slot = (S + C::kRows - 1) / C::kRows;
    // first slot with a row that sees a key of this block (row >= key - coff)
    const int t0 = CAUSAL ? max(0, kt * C::kBlk - coff) / C::kRows : 0;
    const int n_seq = n_slot > t0 ? a.group * (n_slot - t0) : 0;  // slots of all heads of the group

    // chunk position swizzle: rows 0..15 get 16 distinct values (row reads of 16 lanes hit 16
    // different 16-byte bank groups) and 4 consecutive rows differ in the upper two bits (the
    // 4 rows x 64 bytes of a transpose read spread over all banks)
    auto swz = [](int row) {
        return CPR >= 16 ? (((row & 3) << 2) | ((row >> 2) & 3))
                         : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
    };

    // ---- global -> LDS streaming of slot t into ring position rs.  Rows past S-1 lie
    // outside the head's buffer resource and read as zero.
    // Columns Dr..D-1 (head dimensions below the kernel's D) are fetched at an offset past
    // the end of the resource, so they read as zero like everything else outside it.
    const int Dr = a.Dr;
    const uint32_t head_bytes = (uint32_t)(((int64_t)(S - 1) * a.stride_s + Dr) * 2);
    desc_t Qd, Gd;  // Q and dO of the current query head
    rsrc_t Wr;      // its row statistics
    const uint32_t lds0 = lds_address(smem);
    auto set_head = [&](int bh) {
        const int64_t base = (int64_t)(bh / a.H) * a.stride_b + (int64_t)(bh % a.H) * a.stride_h;
        Qd = make_desc(a.Q + base, head_bytes);
        Gd = make_desc(a.dO + base, head_bytes);
        Wr = make_rsrc(a.delta + (int64_t)bh * 2 * S, (uint32_t)S * 8u);
    };
    const uint32_t row_bytes = (uint32_t)a.stride_s * 2u;
    uint32_t dma_voff[C::kDmaPerWave];
#pragma unroll
    for (int n = 0; n < C::kDmaPerWave; ++n) {
        // (with a pair count that does not divide the pieces the last index wraps; dma_piece skips it)
        const int grp = (pair + (n % (C::kDmaPerWave / 2)) * C::kPairs) % C::kDmaPerTensor;
        const int row = grp * (64 / CPR) + l / CPR;
        const int chunk = (l % CPR) ^ swz(row);
        dma_voff[n] = chunk * 8 < Dr ? row * row_bytes + (chunk << 4) : head_bytes;
    }
    // stats: lanes 0-31 fetch lse2 (second half of the head's workspace), 32-63 delta
    const uint32_t stat_voff = (uint32_t)(h ? r : S + r) * 4u;
    // The statistics of a slot are requested by one producer, its Q and dO pieces by the
    // CONSUMERS, consumer c taking the pieces that pair c is assigned (they have no other vector
    // memory traffic and are the shorter chain of a slot; with the producers issuing them between
    // their MFMAs the kernel was 2-5 % slower), right after the slot barrier, into a ring position
    // that nobody reads before a later barrier.  (Spread between the consumers' MFMAs instead they
    // measured the same or up to 2.5 % slower.)
    auto dma_stat = [&](int t, int rs) __attribute__((always_inline)) {
        if (w == C::kStatWave)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                Wr, (void __attribute__((address_space(3))) *)(smem + C::kOffStat + rs * C::kStatBytes),
                4, (int)stat_voff, t * C::kRows * 4, 0, 0);
    };
    // (With a pair count that does not divide the pieces of a tensor -- six pairs, eight pieces --
    // the first producers take two pieces of each tensor and the others one: `extra`.)
    const bool extra = pair + (C::kDmaPerWave / 2 - 1) * C::kPairs < C::kDmaPerTensor;
    auto dma_piece = [&](int t, int rs, int n) __attribute__((always_inline)) {
        const int tensor = n / (C::kDmaPerWave / 2);  // Q transfers first, then dO
        if (C::kDmaPerTensor % C::kPairs != 0 && n % (C::kDmaPerWave / 2) == C::kDmaPerWave / 2 - 1 && !extra) return;
        const int grp = (pair + (n % (C::kDmaPerWave / 2)) * C::kPairs) % C::kDmaPerTensor;  // 1 KB piece
        const uint32_t dst = lds0 + rs * C::kSlotBytes + tensor * C::kTensorBytes + grp * 1024;
        dma16_between(tensor == 0 ? Qd : Gd, dst, dma_voff[n], (uint32_t)(t * C::kRows * row_bytes));
    };
    auto dma_pieces = [&](int t, int rs) __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < C::kDmaPerWave; ++n) dma_piece(t, rs, n);
    };
    // Before slot t is used: this wave's transfers of slot t must have landed (those of the
    // kAhead-1 newer slots may stay in flight) and everyone must be done with slot t-2.
    auto slot_barrier = [&]() {
        if (producer) {
            if (w == C::kStatWave) wait_vm_and_barrier<C::kAhead - 1>();
            else wait_vm_and_barrier<0>();
        } else if (C::kDmaPerTensor % C::kPairs != 0 && !extra) {
            wait_vm_and_barrier<(C::kAhead - 1) * (C::kDmaPerWave - 2)>();
        } else {
            wait_vm_and_barrier<(C::kAhead - 1) * C::kDmaPerWave>();
        }
    };
    // slot and head of the next transfer (both roles keep count: the producers for the statistics,
    // the consumers for the rows): the slots of the group's query heads form ONE sequence (head
    // after head, slots t0 .. n_slot-1 of each), so that the ring stays full across the change of
    // head; past the last head the rows lie beyond S and read as zero
    int tf = t0, gqf = 0;
    auto advance_fetch = [&]() __attribute__((always_inline)) {
        ++tf;
        if (tf == n_slot && gqf + 1 < a.group) {
            tf = t0;
            set_head(bh0 + ++gqf);
        }
    };
    // wave-uniform: does slot t hold a real row that sees some key of the pair
    auto active = [&](int t) {
        return t * C::kRows < S && (!CAUSAL || t * C::kRows + 31 + coff >= k0);
    };
    auto ring_next = [](int x) { return x + 1 == C::kRing ? 0 : x + 1; };

    elem8 *const Xs = reinterpret_cast<elem8 *>(smem + C::kOffXchg) + pair * 256 + l;

    if (producer) {
        // The statistics of the first kAhead slots are requested before anything else (the
        // consumers request the rows meanwhile).
        set_head(bh0);
#pragma unroll
        for (int i = 0; i < C::kAhead; ++i) {
            dma_stat(tf, i);
            advance_fetch();
        }
        // K and V fragments (B operands): lane holds K[key][16ks + 8h .. +7].
        // The 32 rows are fetched whole (an instruction covers 64 / (D/8) consecutive rows instead
        // of 16 bytes of each of 32) and sorted into the fragment layout through LDS that nobody
        // else touches before the first barrier of the slot loop: at D <= 128 the producer's own
        // two slices of the exchange buffer (2 x 4 KB: rows 0-15 and 16-31), at D = 256 (two
        // producers, 16 KB each) the two tensors of the first ring slot that no transfer has been
        // issued for; chunks XOR-swizzled by the row like the slots.
        elem8 kf[KS], vf[KS];
        {
            constexpr int RPI = 64 / CPR;  // rows per load instruction
            const int lr = l / CPR, lc = l % CPR;
            u32x4 tk[KS], tv[KS];
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                const int64_t off = base_kv + (int64_t)min(k0 + RPI * j + lr, Sk - 1) * a.kv_stride_s;
                tk[j] = ld_row16(a.K + off, lc * 8, Dr);
                tv[j] = ld_row16(a.V + off, lc * 8, Dr);
            }
            static_assert(D <= 128 || C::kPairs <= 2, "staging space of the producers");
            char *const mine = D <= 128 ? smem + C::kOffXchg + pair * 4096
                                        : smem + C::kAhead * C::kSlotBytes + pair * C::kTensorBytes;
            auto slot_of = [&](int row, int chunk) {  // byte offset of a chunk of a staged row
                return D <= 128 ? (row >> 4) * (C::kPairs * 4096) + (row & 15) * RB + ((chunk ^ swz(row & 15)) << 4)
                                : row * RB + ((chunk ^ swz(row)) << 4);
            };
            auto sort_rows = [&](const u32x4 (&t)[KS], elem8 (&f)[KS]) __attribute__((always_inline)) {
#pragma unroll
                for (int j = 0; j < KS; ++j) *(u32x4 *)(mine + slot_of(RPI * j + lr, lc)) = t[j];
                asm volatile("" ::: "memory");  // a wave's LDS accesses execute in order
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) f[ks] = *(const elem8 *)(mine + slot_of(r, 2 * ks + h));
                asm volatile("" ::: "memory");
            };
            sort_rows(tk, kf);
            sort_rows(tv, vf);
        }
        // make sure no register load is counted among the streamed transfers any more
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        const float c = a.scale_log2e;
        const int lane_off = r * RB + ((h ^ swz(r)) << 4);  // chunk 2ks+h of row r: ^ (ks*32)

        int rs = 0;  // ring position of the current slot
        int t = t0;  // its rows: slot t of the current head
        for (int g = 0; g < n_seq; ++g) {
            slot_barrier();
            int rd = rs + C::kAhead;
            rd = rd >= C::kRing ? rd - C::kRing : rd;
            dma_stat(tf, rd);
            if (active(t)) {
                const char *Qt = smem + rs * C::kSlotBytes;
                const float *st = reinterpret_cast<const float *>(smem + C::kOffStat + rs * C::kStatBytes);
                const int q_lo = t * C::kRows;
                f32x16 s, dp;
                {
                    // register i <-> query row q_lo + 8*(i/4) + 4h + i%4.  The dP accumulator
                    // starts from -delta of its row, so that it ends as dP - delta.
                    f32x16 zero, nd;
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const f32x4 d4 = *(const f32x4 *)(st + 32 + 8 * g + 4 * h);
#pragma unroll
                        for (int e = 0; e < 4; ++e) nd[4 * g + e] = d4[e];
                    }
#pragma unroll
                    for (int i = 0; i < 16; ++i) zero[i] = 0.f;
                    s = mfma32(*(const elem8 *)(Qt + lane_off), kf[0], zero);
                    dp = mfma32(*(const elem8 *)(Qt + C::kTensorBytes + lane_off), vf[0], nd);
                }
#pragma unroll
                for (int ks = 1; ks < KS; ++ks) {
                    const int off = lane_off ^ (ks * 32);
                    s = mfma32(*(const elem8 *)(Qt + off), kf[ks], s);
                    dp = mfma32(*(const elem8 *)(Qt + C::kTensorBytes + off), vf[ks], dp);
                }
                // the lane's key is fixed; P = exp2(c S - lse2) per row
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 l4 = *(const f32x4 *)(st + 8 * g + 4 * h);
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        s[4 * g + e] = fast_exp2(__builtin_fmaf(s[4 * g + e], c, -l4[e]));
                }
                if ((q_lo + 32 > S) || (CAUSAL && q_lo + coff < k0 + 31)) {
                    // visible row offsets: >= key - coff - q_lo (causal) and <= S - 1 - q_lo
                    const int lo = (CAUSAL ? key - coff - q_lo : -64) - 4 * h;
                    const int hi = S - 1 - q_lo - 4 * h;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int ro = 8 * (i / 4) + (i % 4);
                        if (ro < lo || ro > hi) s[i] = 0.f;
                    }
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) dp[i] *= s[i];  // dS = P o (dP - delta)
                elem8 *x = Xs + (g & 1) * (C::kPairs * 256);
                x[0] = pack8(s[0], s[1], s[2], s[3], s[4], s[5], s[6], s[7]);
                x[64] = pack8(s[8], s[9], s[10], s[11], s[12], s[13], s[14], s[15]);
                x[128] = pack8(dp[0], dp[1], dp[2], dp[3], dp[4], dp[5], dp[6], dp[7]);
                x[192] = pack8(dp[8], dp[9], dp[10], dp[11], dp[12], dp[13], dp[14], dp[15]);
            }
            advance_fetch();
            rs = ring_next(rs);
            if (++t == n_slot) t = t0;
        }
        wait_vm_and_barrier<0>();  // the consumers' last slot
    } else {
        // Consumers.  Wave 4+cw accumulates ONE output for the 64 keys of two producers
        // (2*(cw>>1) and the next): dV^T += dO^T P for even cw, dK^T += Q^T dS for odd cw.
        // Each transposed fragment read from LDS then feeds two MFMAs (one per key block),
        // which halves the consumers' LDS traffic against one wave per 32 keys and both
        // outputs.
        const int cw = w - C::kPairs;
        const int kind = cw & 1, half = cw >> 1;
        const int kA = kt * C::kBlk + half * 64, kB = kA + 32;  // first keys of the two blocks
        f32x16 acc[2][DB];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[kb][db][i] = 0.f;
        // transpose-read addresses: the 16-lane group reads rows 4h+e (e = 0..3), +8 for the
        // second read, 64 bytes of d block db per row; byte offset within a slot tensor
        int tr_off[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int row = 8 * j + 4 * h + ((l & 15) >> 2);
            const int chunk = 2 * ((l >> 4) & 1) + ((l >> 1) & 1);
            tr_off[j] = row * RB + ((chunk ^ swz(row)) << 4) + (l & 1) * 8;
        }
        // wave-uniform: does slot t hold a real row that sees some key of the block at kfirst
        auto block_active = [&](int t, int kfirst) {
            return t * C::kRows < S && (!CAUSAL || t * C::kRows + 31 + coff >= kfirst);
        };
        const elem8 *const Xc = reinterpret_cast<const elem8 *>(smem + C::kOffXchg) +
                                 (2 * half) * 256 + kind * 128 + l;
        auto consume = [&](int t, int g, int rs) {
            const bool actA = block_active(t, kA), actB = block_active(t, kB);
            if (!actA) return;  // kA < kB: then the second block is not active either
            const char *Tt = smem + rs * C::kSlotBytes + (kind ? 0 : C::kTensorBytes);
            const elem8 *x = Xc + (g & 1) * (C::kPairs * 256);
            const elem8 opA[2] = {x[0], x[64]};
            // Slots above the diagonal of the second key block: its producer wrote nothing,
            // so the block gets zero operands (a second code path without its MFMAs makes
            // the compiler spill the accumulators).
            elem8 opB[2];
#pragma unroll
            for (int i = 0; i < 8; ++i) opB[0][i] = opB[1][i] = 0;
            if (actB) { opB[0] = x[256]; opB[1] = x[256 + 64]; }
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    // d block db = chunks 4db..4db+3: flips bits 6.. of the swizzled offset
                    const int o0 = (tr_off[0] ^ (db << 6)) + cc * 16 * RB;
                    const int o1 = (tr_off[1] ^ (db << 6)) + cc * 16 * RB;
                    const elem8 T = join8(lds_read_tr((const elem *)(Tt + o0)),
                                           lds_read_tr((const elem *)(Tt + o1)));
                    acc[0][db] = mfma32(T, opA[cc], acc[0][db]);
                    acc[1][db] = mfma32(T, opB[cc], acc[1][db]);
                }
            }
        };

        // the rows of the first kAhead slots
        set_head(bh0);
#pragma unroll
        for (int i = 0; i < C::kAhead; ++i) {
            dma_pieces(tf, i);
            advance_fetch();
        }
        int rs = 0;  // ring position of the producers' slot; the consumers' is one behind
        int t = t0, tp = t0;  // rows of the producers' slot and of the one before it
        for (int g = 0; g < n_seq; ++g) {
            slot_barrier();
            // slot g + kAhead goes into the ring position that slot g - 2 has left
            int rd = rs + C::kAhead;
            rd = rd >= C::kRing ? rd - C::kRing : rd;
            dma_pieces(tf, rd);
            advance_fetch();
            if (g > 0) consume(tp, g - 1, rs == 0 ? C::kRing - 1 : rs - 1);
            rs = ring_next(rs);
            tp = t;
            if (++t == n_slot) t = t0;
        }
        wait_vm_and_barrier<0>();
        if (n_seq > 0) consume(tp, n_seq - 1, rs == 0 ? C::kRing - 1 : rs - 1);

        // The accumulators hold 4 consecutive columns of one key per register group: stored
        // directly, every instruction writes 8-byte pieces of 32 rows (32 such stores per wave).
        // The rows of a key block go through LDS instead and leave whole, 16 bytes per lane: each
        // consumer takes one tensor's worth of a ring slot other than the last one, which other
        // consumers may still be reading (the producers have issued their last transfer and all
        // of them have landed), in the slots' swizzled row layout.
        elem *const out = kind ? a.dK : a.dV;
        const float sc = kind ? a.scale : 1.f;
        {
            constexpr int RPI = 64 / CPR;  // rows per store instruction
            const int last = rs == 0 ? C::kRing - 1 : rs - 1;  // ring position of the last slot
            int slot = cw >> 1;
            slot += slot >= last ? 1 : 0;
            char *stg = smem + slot * C::kSlotBytes + (cw & 1) * C::kTensorBytes;
            const int lr = l / CPR, lc = l % CPR;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        *(elem4 *)(stg + r * RB + (((4 * db + g) ^ swz(r)) << 4) + 8 * h) =
                            pack4(acc[kb][db][4 * g] * sc, acc[kb][db][4 * g + 1] * sc,
                                  acc[kb][db][4 * g + 2] * sc, acc[kb][db][4 * g + 3] * sc);
                asm volatile("" ::: "memory");  // a wave's LDS accesses execute in order
#pragma unroll
                for (int j = 0; j < 32 / RPI; ++j) {
                    const int row = RPI * j + lr;
                    const u32x4 v = *(const u32x4 *)(stg + row * RB + ((lc ^ swz(row)) << 4));
                    const int okey = kA + 32 * kb + row;
                    if (okey < Sk && lc * 8 < Dr)
                        *(u32x4 *)(out + base_kv + (int64_t)okey * a.kv_stride_s + lc * 8) = v;
                }
                asm volatile("" ::: "memory");
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// 3. dQ.  Work-group = NW waves, wave = 32 queries (Q, dO fragments and the 32 x D fp32
// accumulator in registers), loop over key tiles of 64 rows.  K and V tiles go global -> LDS
// directly, two tiles ahead, into a ring of three.
//
// LDS layout of a tile tensor.  One wave-wide transfer fills 1 KB in lane order, and a lane
// may fetch any 16-byte chunk, so within such a piece (P rows of a tile: 4 at D = 128, 8 at
// D = 64) the chunks are stored chunk-major: chunk c of row r sits at 16 * (c * P + r % P),
// and consecutive pieces are P * 16 bytes apart more than their size.  Then
//  - the address of a fragment is a per-lane constant plus compile-time terms for the
//    contraction step, the d block, the sub-tile and the ring position: with the loop unrolled
//    over the ring positions every LDS access is one register plus an immediate offset and the
//    loop has no vector instruction for addressing (it had 16 per sub-tile with a row-major,
//    XOR-swizzled tile);
//  - 16 consecutive rows at a fixed chunk fall into 16 different 16-byte bank groups (the row
//    reads for S^T = K Q^T and dP^T = V dO^T), and the 64 lanes of a transpose read (4 rows x
//    4 chunks x 2 halves per half-wave, for dQ^T += K^T dS^T) cover 512 contiguous bytes:
//    both are conflict free.
// ---------------------------------------------------------------------------------------
template <int D, int NW>
struct DqCfg {
    static constexpr int kThreads = NW * 64;
    static constexpr int kBlk = NW * 32;             // queries owned by the work-group
    static constexpr int kTile = D > 128 ? 32 : 64;  // keys per tile (a ring of three must fit the LDS)
    static constexpr int kSub = kTile / 32;          // 32-key sub-tiles per tile
    static constexpr int kRing = 3;
    static constexpr int kRowBytes = D * 2;
    static constexpr int kPieceRows = 1024 / kRowBytes;       // rows one 1 KB transfer fills
    static constexpr int kPieceBytes = 1024 + kPieceRows * 16;
    static constexpr int kPieces = kTile / kPieceRows;        // per tensor
    // D = 256 (two rows per piece): the uniform piece distance that spreads the row reads over
    // the banks puts the four rows of a transpose read into overlapping banks.  Pieces are laid
    // out in pairs instead: the second of a pair 1024 + 128 bytes after the first (the two pieces
    // a transpose read touches then fall into different halves of the banks), pairs 2 * 1024 +
    // 128 + 160 bytes apart (16 consecutive rows at a fixed chunk: 16 different 16-byte bank groups).
    static constexpr int kPairBytes = 2 * 1024 + 128 + 160;
    static constexpr int piece_base(int piece)
    {
        return D > 128 ? (piece >> 1) * kPairBytes + (piece & 1) * (1024 + 128) : piece * kPieceBytes;
    }
    static constexpr int kTensorBytes = piece_base(kPieces);     // K part of a tile; V follows
    static constexpr int kTileBytes = 2 * kTensorBytes;
    // D <= 128: the rows of Q, dO and O reach the fragment registers through a per-wave staging
    // area of 32 rows in the tile tensors' layout (see the kernel's prologue).  The areas start
    // at ring position 2, which is free until the first barrier of the key loop.
    static constexpr bool kStageRows = true;
    static constexpr int kStageBytes = kStageRows ? piece_base(32 / kPieceRows) : 0;
    static constexpr int kLdsBytes = kRing * kTileBytes > 2 * kTileBytes + NW * kStageBytes
                                         ? kRing * kTileBytes : 2 * kTileBytes + NW * kStageBytes;
    static constexpr int kDmaPerTile = 2 * kPieces;           // wave-wide 1 KB transfers
    static constexpr int kDmaPerWave = (kDmaPerTile + NW - 1) / NW;
    static constexpr int kChunkStep = kPieceRows * 16;        // next 16-byte chunk of a row
    static constexpr int kRows16 = piece_base(16 / kPieceRows);      // 16 rows further
    static_assert(16 % kPieceRows == 0, "sub-tiles start at piece boundaries");
    static_assert(kLdsBytes <= 160 * 1024, "LDS budget of a gfx950 CU exceeded");
};

template <int D, int NW, bool CAUSAL, bool SPLIT>
__global__ void __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(D > 128 ? 1 : 2)))
attn_bwd_dq_kernel(const BwdArgs a)
{
    using C = DqCfg<D, NW>;
    constexpr int KS = D / 16, DB = D / 32, PR = C::kPieceRows;
    // A wave's transfers per tile are issued between the MFMAs of the tile's first step instead of
    // in a burst after the barrier wherever their number divides that of the MFMAs (measured at
    // D = 128: long causal shapes 2-3 % faster)
    constexpr bool kBetween = KS % C::kDmaPerWave == 0;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int tid = threadIdx.x, l = tid & 63, r = l & 31, h = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int S = a.S;
    int bh, rank;
    xcd_tile_order<CAUSAL>(blockIdx.x, a.ntile, a.BH, bh, rank);
    const int qt = CAUSAL ? a.ntile - 1 - rank : rank;  // heaviest first
    const int64_t base = (int64_t)(bh / a.H) * a.stride_b + (int64_t)(bh % a.H) * a.stride_h;
    // grouped-query heads: query head h reads K/V head h / group
    const int64_t base_kv = (int64_t)(bh / a.H) * a.kv_stride_b +
                            (int64_t)((bh % a.H) / a.group) * a.kv_stride_h;

    const int q0 = qt * C::kBlk + w * 32;
    const int q = q0 + r;
    const int qc = q < S ? q : S - 1;
    // Keys seen by this work-group: all Sk of them, or one split's range (then K and V are
    // simply re-based to the range and the causal offset moves with them; the row statistics
    // belong to the whole row, so the partial dQ of the ranges just add up).
    int Sk = a.Sk;      // key/value rows; S is the number of query rows
    int coff = Sk - S;  // causal: query row i sees keys 0 .. i + coff
    int64_t kv_first = 0;
    if (SPLIT) {
        const int k_begin = blockIdx.y * a.dq_kps;  // < Sk by the launcher's plan
        kv_first = (int64_t)k_begin * a.kv_stride_s;
        Sk = min(Sk - k_begin, a.dq_kps);
        coff -= k_begin;
    }
    const int q0e = q0 + coff;
    const int q_end = min(S, (qt + 1) * C::kBlk);
    // (a split that lies wholly above the work-group's diagonal has no tile)
    const int n_kt = max(0, (CAUSAL ? min(Sk, q_end + coff) : Sk) + C::kTile - 1) / C::kTile;

    // byte offset of 16-byte chunk `chunk` of row `row` within a tile tensor
    auto at = [](int row, int chunk) {
        return C::piece_base(row / PR) + (chunk * PR + row % PR) * 16;
    };

    // ---- streaming of tile kt into ring position pos; rows past S-1 read as zero
    const int Dr = a.Dr;  // columns Dr..D-1 read as zero (offset past the end of the resource)
    const uint32_t head_bytes = (uint32_t)(((int64_t)(Sk - 1) * a.kv_stride_s + Dr) * 2);
    const desc_t Kd0 = make_desc(a.K + base_kv + kv_first, head_bytes),
                 Vd0 = make_desc(a.V + base_kv + kv_first, head_bytes);
    const uint32_t row_bytes = (uint32_t)a.kv_stride_s * 2u;
    const uint32_t lds0 = lds_address(smem);
    // (the descriptors are passed by value: captured by reference through two levels of
    // lambdas the compiler no longer proves them wave-uniform)
    // lane l lands at byte 16 * l of a piece: chunk l / PR of the piece's row l % PR.  The
    // piece's first row goes into the scalar offset (which takes part in the range check like
    // the per-lane one), so one per-lane offset serves every transfer.
    const uint32_t voff = (l / PR) * 8 < Dr ? (l % PR) * row_bytes + ((l / PR) << 4) : head_bytes;
    auto dma_piece = [&](int kt, int pos, int n, desc_t Kd, desc_t Vd) __attribute__((always_inline)) {
        // wave-uniform 1 KB piece; a wave with nothing left repeats an earlier piece so
        // that every wave has the same number of transfers in flight
        const int i = (w + n * NW) % C::kDmaPerTile;
        const int tensor = i / C::kPieces, piece = i % C::kPieces;
        const uint32_t dst = lds0 + pos * C::kTileBytes + tensor * C::kTensorBytes + C::piece_base(piece);
        const uint32_t soff = (kt * C::kTile + piece * PR) * row_bytes;
        if (kBetween) dma16_between(tensor ? Vd : Kd, dst, voff, soff);
        else dma16(tensor ? Vd : Kd, dst, voff, soff);
    };
    auto dma_tile = [&](int kt, int pos, desc_t Kd, desc_t Vd) __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < C::kDmaPerWave; ++n) dma_piece(kt, pos, n, Kd, Vd);
    };
    if (n_kt > 0) dma_tile(0, 0, Kd0, Vd0);
    if (n_kt > 1) dma_tile(1, 1, Kd0, Vd0);

    // Q and dO fragments (B operands: lane holds row q, columns 16 ks + 8 h .. +7) and, in a full
    // backward, the O rows for the row statistics.  A load in which every lane fetches 16 bytes
    // of its own row touches 32 rows per instruction, and a work-group issues 192 of them here:
    // measured in the forward, 64 such loads alone took the last wave 5000-7000 cycles to get
    // issued, with the compute unit idle.  At D <= 128 the rows are therefore fetched whole (an
    // instruction covers 64 / (D/8) consecutive rows), all in flight together, and sorted into
    // the fragment layout through the wave's staging area in LDS, one tensor after the other.
    elem8 qf[KS], gf[KS], of[KS];
    if constexpr (C::kStageRows) {
        constexpr int CPR = D / 8, RPI = 64 / CPR;  // chunks per row; rows per load instruction
        const int lr = l / CPR, lc = l % CPR;
        u32x4 tq[KS], tg[KS], to[KS];
#pragma unroll
        for (int j = 0; j < KS; ++j) {
            const int64_t off = base + (int64_t)min(q0 + RPI * j + lr, S - 1) * a.stride_s;
            tq[j] = ld_row16(a.Q + off, lc * 8, Dr);
            tg[j] = ld_row16(a.dO + off, lc * 8, Dr);
            if (a.stats_in_dq) to[j] = ld_row16(a.O + off, lc * 8, Dr);
        }
        char *stage = smem + 2 * C::kTileBytes + w * C::kStageBytes;
        const int rd = at(r, h);  // chunk h of row r; contraction step ks: 2 ks chunks further
        auto sort_rows = [&](const u32x4 (&t)[KS], elem8 (&f)[KS]) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < KS; ++j) *(u32x4 *)(stage + at(RPI * j + lr, lc)) = t[j];
            asm volatile("" ::: "memory");  // a wave's LDS accesses execute in order
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) f[ks] = *(const elem8 *)(stage + rd + ks * 2 * C::kChunkStep);
            asm volatile("" ::: "memory");
        };
        sort_rows(tq, qf);
        sort_rows(tg, gf);
        if (a.stats_in_dq) sort_rows(to, of);
    } else {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qf[ks] = as_elem8(ld_row16(a.Q + base + (int64_t)qc * a.stride_s, ks * 16 + 8 * h, Dr));
            gf[ks] = as_elem8(ld_row16(a.dO + base + (int64_t)qc * a.stride_s, ks * 16 + 8 * h, Dr));
        }
        if (a.stats_in_dq) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                of[ks] = as_elem8(ld_row16(a.O + base + (int64_t)qc * a.stride_s, ks * 16 + 8 * h, Dr));
        }
    }
    // Row statistics of this lane's query: lse2 = LSE * log2(e) and -delta = -rowsum(dO * O).
    // In a full backward this kernel runs first and forms them itself (the dO row is in
    // registers anyway; lanes l and l^32 hold the two halves of a row) and stores them for the
    // dK/dV kernel, which saves the separate kernel's launch; called alone it reads them.
    float lse2, ndelta;
    if (a.stats_in_dq) {
        float acc = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
            for (int t = 0; t < 8; ++t) acc += (float)of[ks][t] * (float)gf[ks][t];
        }
        ndelta = -xhalf_sum(acc);
        lse2 = a.LSE[(int64_t)bh * S + qc] * kLog2e;
        if (q < S && h == 0 && (!SPLIT || blockIdx.y == 0)) {
            a.delta[(int64_t)bh * 2 * S + q] = ndelta;
            a.delta[(int64_t)bh * 2 * S + S + q] = lse2;
        }
    } else {
        lse2 = a.delta[(int64_t)bh * 2 * S + S + qc];
        ndelta = a.delta[(int64_t)bh * 2 * S + qc];
    }
    // -delta replicated: the dP accumulators start from it
    f32x16 nd;
#pragma unroll
    for (int i = 0; i < 16; ++i) nd[i] = ndelta;

    f32x16 dq[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) dq[db][i] = 0.f;

    const float c = a.scale_log2e;
    // Per-lane LDS addresses within ring position 0 (lo) and 2 (hi): row fragment = chunk h of
    // row r (contraction step ks: 2 ks chunks further); transpose reads = rows 4h+e (+8), the
    // 64 bytes of d block 0 of each row (d block db: 4 db chunks further).  Everything else --
    // ring position, tensor, sub-tile, 16-row step -- is a compile-time offset.  Position 2
    // gets registers of its own because an LDS instruction's immediate reaches 64 KB and the
    // ring is longer than that at D = 128.  The values are made opaque so that the compiler
    // keeps exactly these six registers instead of re-deriving addresses in the loop.
    int row_lo = at(r, h), tr_lo[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
        tr_lo[j] = at(8 * j + 4 * h + ((l & 15) >> 2), 2 * ((l >> 4) & 1) + ((l >> 1) & 1)) + (l & 1) * 8;
    int row_hi = row_lo + 2 * C::kTileBytes, tr_hi[2] = {tr_lo[0] + 2 * C::kTileBytes,
                                                          tr_lo[1] + 2 * C::kTileBytes};
    asm volatile("" : "+v"(row_lo), "+v"(tr_lo[0]), "+v"(tr_lo[1]));
    if (NW == 8) asm volatile("" : "+v"(row_hi), "+v"(tr_hi[0]), "+v"(tr_hi[1]));

    // All register loads above must be complete before the loop: the compiler would otherwise
    // place its own vmcnt waits for them at their first use inside the loop, where they would
    // also wait for the tile transfers (which it does not see) in every iteration.
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)

    // One tile of 64 keys at ring position `pos`; Kt + rowa / tra0 / tra1 address its K tensor.
    // The steps of one 32-key sub-tile kb2 of the tile whose K tensor Kt + rowa / tra0 / tra1
    // address; register i of s and dp <-> key k_lo + 8*(i/4) + 4h + i%4 (this lane's query is
    // fixed).
    auto step_s = [&](const char *Kt, int rowa, int kb2, f32x16 &s) __attribute__((always_inline)) {
        f32x16 zero;
#pragma unroll
        for (int i = 0; i < 16; ++i) zero[i] = 0.f;
        s = mfma32(*(const elem8 *)(Kt + kb2 * 2 * C::kRows16 + rowa), qf[0], zero);
#pragma unroll
        for (int ks = 1; ks < KS; ++ks)
            s = mfma32(*(const elem8 *)(Kt + kb2 * 2 * C::kRows16 + ks * 2 * C::kChunkStep + rowa), qf[ks], s);
    };
    // the same with the transfers of tile kt_next (into ring position pos_next) between the MFMAs
    auto step_s_fetch = [&](const char *Kt, int rowa, f32x16 &s, int kt_next, int pos_next, desc_t Kd,
                            desc_t Vd) __attribute__((always_inline)) {
        constexpr int kEvery = kBetween ? KS / C::kDmaPerWave : 1;
        f32x16 zero;
#pragma unroll
        for (int i = 0; i < 16; ++i) zero[i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            s = mfma32(*(const elem8 *)(Kt + ks * 2 * C::kChunkStep + rowa), qf[ks], ks ? s : zero);
            if ((ks + 1) % kEvery == 0) dma_piece(kt_next, pos_next, (ks + 1) / kEvery - 1, Kd, Vd);
        }
    };
    auto step_dp = [&](const char *Kt, int rowa, int kb2, f32x16 &dp) __attribute__((always_inline)) {
        const char *Vt = Kt + C::kTensorBytes;
        dp = mfma32(*(const elem8 *)(Vt + kb2 * 2 * C::kRows16 + rowa), gf[0], nd);  // ends as dP - delta
#pragma unroll
        for (int ks = 1; ks < KS; ++ks)
            dp = mfma32(*(const elem8 *)(Vt + kb2 * 2 * C::kRows16 + ks * 2 * C::kChunkStep + rowa), gf[ks], dp);
    };
    auto step_p = [&](int k_lo, f32x16 &s) __attribute__((always_inline)) {  // S -> P
        const bool need_mask = (k_lo + 32 > Sk) || (CAUSAL && k_lo + 31 > q0e);
        const int lim = (CAUSAL ? qc + coff : Sk - 1) - k_lo - 4 * h;
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] = fast_exp2(__builtin_fmaf(s[i], c, -lse2));
        if (need_mask) {  // wave-uniform: only blocks on the diagonal or at the ragged end
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (8 * (i / 4) + (i % 4) > lim) s[i] = 0.f;
        }
    };
    auto step_ds = [&](const f32x16 &s, f32x16 &dp, elem8 (&sb)[2]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 16; ++i) dp[i] *= s[i];  // dS = P o (dP - delta)
        sb[0] = pack8(dp[0], dp[1], dp[2], dp[3], dp[4], dp[5], dp[6], dp[7]);
        sb[1] = pack8(dp[8], dp[9], dp[10], dp[11], dp[12], dp[13], dp[14], dp[15]);
    };
    auto step_dq = [&](const char *Kt, int tra0, int tra1, int kb2, const elem8 (&sb)[2])
                       __attribute__((always_inline)) {
#pragma unroll
        for (int cc = 0; cc < 2; ++cc) {
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const int off = (kb2 * 2 + cc) * C::kRows16 + db * 4 * C::kChunkStep;
                const elem8 kT = join8(lds_read_tr((const elem *)(Kt + off + tra0)),
                                       lds_read_tr((const elem *)(Kt + off + tra1)));
                dq[db] = mfma32(kT, sb[cc], dq[db]);
            }
        }
    };
    // One tile at ring position `pos`.
    auto tile = [&](int kt, int pos, const char *Kt, int rowa, int tra0, int tra1, desc_t Kd,
                    desc_t Vd) __attribute__((always_inline)) {
        // tile kt must have landed; tile kt+1 (if any) may stay in flight
        if (kt + 1 < n_kt) wait_vm_and_barrier<C::kDmaPerWave>();
        else wait_vm_and_barrier<0>();
        const bool fetch = kt + 2 < n_kt;  // tile kt + 2 goes into the ring position freed by the barrier
        if (fetch && !kBetween) dma_tile(kt + 2, pos == 0 ? 2 : pos - 1, Kd, Vd);

        const int k0 = kt * C::kTile;
        // wave-uniform: does this wave see any key of the first / second sub-tile
        const bool act0 = k0 < Sk && (!CAUSAL || k0 <= q0e + 31);
        const bool act1 = k0 + 32 < Sk && (!CAUSAL || k0 + 32 <= q0e + 31);
        if (kBetween && fetch && !act0) dma_tile(kt + 2, pos == 0 ? 2 : pos - 1, Kd, Vd);
#pragma unroll
        for (int kb2 = 0; kb2 < C::kSub; ++kb2) {
            if (!(kb2 ? act1 : act0)) continue;
            f32x16 s, dp;
            elem8 sb[2];
            if (kBetween && kb2 == 0 && fetch) step_s_fetch(Kt, rowa, s, kt + 2, pos == 0 ? 2 : pos - 1, Kd, Vd);
            else step_s(Kt, rowa, kb2, s);
            step_dp(Kt, rowa, kb2, dp);
            step_p(k0 + kb2 * 32, s);
            step_ds(s, dp, sb);
            step_dq(Kt, tra0, tra1, kb2, sb);
        }
    };
    if constexpr (NW == 8) {
        // unrolled over the three ring positions, which makes them compile-time constants;
        // n_kt is the same for every wave of the work-group
        for (int kt = 0; kt < n_kt; kt += 3) {
            tile(kt, 0, smem, row_lo, tr_lo[0], tr_lo[1], Kd0, Vd0);
            if (kt + 1 < n_kt)
                tile(kt + 1, 1, smem + C::kTileBytes, row_lo, tr_lo[0], tr_lo[1], Kd0, Vd0);
            if (kt + 2 < n_kt) tile(kt + 2, 2, smem, row_hi, tr_hi[0], tr_hi[1], Kd0, Vd0);
        }
    } else {
        // fewer waves issue more transfers each and have no registers to spare for the unrolled
        // form: the ring position advances at run time (three additions per tile)
        int pos = 0;
        for (int kt = 0; kt < n_kt; ++kt) {
            const int o = pos * C::kTileBytes;
            tile(kt, pos, smem, row_lo + o, tr_lo[0] + o, tr_lo[1] + o, Kd0, Vd0);
            pos = pos == 2 ? 0 : pos + 1;
        }
    }
    // no transfer may still be in flight when the work-group's LDS is released
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // Output rows leave through the wave's staging area in LDS (see the end of the kernel).  The
    // areas that lie in ring position 2 move to the position that the last two tiles did not use
    // (other waves may still be reading those).
    constexpr int CPR = D / 8, RPI = 64 / CPR;  // chunks per bf16 row; rows per store instruction
    char *const stg = smem + ((w + 1) * C::kStageBytes <= C::kTileBytes
                                  ? (n_kt % 3) * C::kTileBytes + w * C::kStageBytes
                                  : 2 * C::kTileBytes + w * C::kStageBytes);
    const int lr = l / CPR, lc = l % CPR;
    if (SPLIT) {
        // unscaled fp32 partial of this key range (zeros if the range had no visible key); an
        // fp32 row is twice as long as the staging area's, so it goes in two halves
        const int64_t row0 = ((int64_t)blockIdx.y * a.BH + bh) * S;
#pragma unroll
        for (int hp = 0; hp < 2; ++hp) {
#pragma unroll
            for (int db = hp * (DB / 2); db < (hp + 1) * (DB / 2); ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f32x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = dq[db][4 * g + e];
                    *(f32x4 *)(stg + at(r, (db % (DB / 2)) * 8 + 2 * g + h)) = v;
                }
            asm volatile("" ::: "memory");  // a wave's LDS accesses execute in order
#pragma unroll
            for (int j = 0; j < 32 / RPI; ++j) {
                const f32x4 v = *(const f32x4 *)(stg + at(RPI * j + lr, lc));
                const int row = q0 + RPI * j + lr;
                if (row < S) *(f32x4 *)(a.dQpart + (row0 + row) * D + hp * (D / 2) + lc * 4) = v;
            }
            asm volatile("" ::: "memory");
        }
        return;
    }
    if (a.rope_cos) {
        // Q was rotated before the forward: what has been accumulated is the gradient of the
        // rotated rows; the gradient of the unrotated ones is its image under the transpose of
        // the rotation (head dimension == D only; column d pairs with d + D/2, i.e. d block db
        // with db + DB/2, same register).
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
    {
        // The accumulator holds 4 consecutive columns of one row per register group: stored
        // directly, every instruction writes 8-byte pieces of 32 rows.  The rows go through the
        // wave's staging area in LDS instead and leave whole, 16 bytes per lane.  The areas that
        // lie in ring position 2 move to the position that the last two tiles did not use (other
        // waves may still be reading those).
        const float sc = a.scale;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                *(elem4 *)(stg + at(r, 4 * db + g) + 8 * h) =
                    pack4(dq[db][4 * g] * sc, dq[db][4 * g + 1] * sc, dq[db][4 * g + 2] * sc, dq[db][4 * g + 3] * sc);
        asm volatile("" ::: "memory");  // a wave's LDS accesses execute in order
#pragma unroll
        for (int j = 0; j < 32 / RPI; ++j) {
            const u32x4 v = *(const u32x4 *)(stg + at(RPI * j + lr, lc));
            const int row = q0 + RPI * j + lr;
            if (row < S && lc * 8 < Dr) *(u32x4 *)(a.dQ + base + (int64_t)row * a.stride_s + lc * 8) = v;
        }
    }
}

// Sum of the per-split partial dQ, times scale, rounded: one thread per (row, 4 consecutive d);
// HBM-bound and small.
template <int D>
__global__ void __launch_bounds__(256) attn_bwd_dq_merge_kernel(const BwdArgs a)
{
    constexpr int TPR = D / 4;  // threads per row
    const int64_t rows = (int64_t)a.BH * a.S;
    const int64_t row = (int64_t)blockIdx.x * (256 / TPR) + threadIdx.x / TPR;
    if (row >= rows) return;
    const int d0 = (threadIdx.x % TPR) * 4;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    // four splits per step, their loads issued together (one dependent load per split costs a
    // memory latency each); added in the order of the splits
    const int n = a.dq_nsplit;
    for (int z0 = 0; z0 < n; z0 += 4) {
        f32x4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            v[k] = *(const f32x4 *)(a.dQpart + ((int64_t)(z0 + k < n ? z0 + k : z0) * rows + row) * D + d0);
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (z0 + k < n) {
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] += v[k][e];
            }
    }
    const int bh = (int)(row / a.S), q = (int)(row % a.S);
    elem *dQp = a.dQ + (int64_t)(bh / a.H) * a.stride_b + (int64_t)(bh % a.H) * a.stride_h +
                (int64_t)q * a.stride_s + d0;
    const float sc = a.scale;
    if (d0 < a.Dr) *(elem4 *)dQp = pack4(acc[0] * sc, acc[1] * sc, acc[2] * sc, acc[3] * sc);
}

// ---------------------------------------------------------------------------------------
// Launch
// ---------------------------------------------------------------------------------------
template <typename K>
static bool allow_lds(K kernel, int bytes)
{
    return hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                               bytes) == hipSuccess;
}

template <int D, int P, bool CAUSAL>
static int launch_dkdv_p(BwdArgs a, hipStream_t st)
{
    using C = DkdvCfg<D, P>;
    a.ntile = (a.Sk + C::kBlk - 1) / C::kBlk;
    if (!allow_lds(attn_bwd_dkdv_kernel<D, P, CAUSAL>, C::kLdsBytes)) return -1;
    hipLaunchKernelGGL((attn_bwd_dkdv_kernel<D, P, CAUSAL>), dim3(a.ntile * (a.BH / a.group)),
                       dim3(C::kThreads), C::kLdsBytes, st, a);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Work-groups of four producer/consumer pairs (128 keys, two waves per SIMD), or, at D = 128
// on launches of at least two rounds of work-groups, of six (192 keys, 12 waves at 168
// registers: three per SIMD hide more of each other's latencies).  Measured: -2.5..4 % on the
// large shapes; slower on small launches (more of a 192-key block is padding) and at D = 64
// (the larger work-group no longer fits a compute unit twice).
template <int D, bool CAUSAL>
static int launch_dkdv(const BwdArgs &a, hipStream_t st)
{
    // D = 256: two pairs, one wave per SIMD (a consumer's two 32 x 256 accumulators alone are
    // 256 registers), 64 keys per work-group
    if constexpr (D > 128) return launch_dkdv_p<D, 2, CAUSAL>(a, st);
    else {
        if constexpr (D == 128) {
            const int64_t wgs6 = (int64_t)(a.BH / a.group) * ((a.Sk + 191) / 192);
            if (wgs6 >= 512) return launch_dkdv_p<D, 6, CAUSAL>(a, st);
        }
        return launch_dkdv_p<D, 4, CAUSAL>(a, st);
    }
}

template <int D, int NW, bool CAUSAL>
static int launch_dq(BwdArgs a, hipStream_t st)
{
    using C = DqCfg<D, NW>;
    a.ntile = (a.S + C::kBlk - 1) / C::kBlk;
    if (!allow_lds(attn_bwd_dq_kernel<D, NW, CAUSAL, false>, C::kLdsBytes)) return -1;
    hipLaunchKernelGGL((attn_bwd_dq_kernel<D, NW, CAUSAL, false>), dim3(a.ntile * a.BH),
                       dim3(C::kThreads), C::kLdsBytes, st, a);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Split over the keys: 256-row work-groups, one grid row per split, then the merge.
template <int D, bool CAUSAL>
static int launch_dq_split(BwdArgs a, hipStream_t st)
{
    using C = DqCfg<D, 8>;
    a.ntile = (a.S + C::kBlk - 1) / C::kBlk;
    if (!allow_lds(attn_bwd_dq_kernel<D, 8, CAUSAL, true>, C::kLdsBytes)) return -1;
    hipLaunchKernelGGL((attn_bwd_dq_kernel<D, 8, CAUSAL, true>), dim3(a.ntile * a.BH, a.dq_nsplit),
                       dim3(C::kThreads), C::kLdsBytes, st, a);
    if (hipGetLastError() != hipSuccess) return -1;
    const int64_t rows = (int64_t)a.BH * a.S;
    constexpr int RPB = 256 / (D / 4);
    hipLaunchKernelGGL((attn_bwd_dq_merge_kernel<D>), dim3((unsigned)((rows + RPB - 1) / RPB)),
                       dim3(256), 0, st, a);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <int D, bool CAUSAL>
static int launch_dq_for(const BwdArgs &a, hipStream_t st)
{
    // D = 256: always four waves, one per SIMD (Q and dO fragments plus the accumulator are
    // 256 registers); never split
    if constexpr (D > 128) return a.dq_nsplit > 1 ? -1 : launch_dq<D, 4, CAUSAL>(a, st);
    else {
    if (a.dq_nsplit > 1) return launch_dq_split<D, CAUSAL>(a, st);
    const int blocks32 = (a.S + 31) / 32;
    // 256-row work-groups unless they would leave compute units (256) idle while 128-row
    // ones would not (few heads and rows against many keys, e.g. chunked prefill).  Under a
    // causal mask 128-row work-groups also balance the unequal tiles better as long as the
    // launch is small: at D = 128 (one work-group per compute unit either way) up to one
    // 256-row work-group per unit (B=1 H=16 S=4096: 135 -> 117 us, B=1 H=8 S=8192: 256 -> 220 us;
    // with 1.25 per unit already 15 % slower), at D = 64 (two fit a unit) up to four
    // (B=8 H=8 S=1024: 28.9 -> 26.6 us, B=4 H=8 S=2048: 45.4 -> 42.0 us).
    const int64_t wgs8 = (int64_t)a.BH * ((a.S + 255) / 256);
    const bool prefer4 = CAUSAL && (D == 64 ? wgs8 < 1024 : wgs8 <= 256);
    if (blocks32 >= 8 && wgs8 >= 256 && !prefer4) return launch_dq<D, 8, CAUSAL>(a, st);
    if (blocks32 >= 4) return launch_dq<D, 4, CAUSAL>(a, st);
    if (blocks32 == 3) return launch_dq<D, 3, CAUSAL>(a, st);
    if (blocks32 == 2 || D == 128) return launch_dq<D, 2, CAUSAL>(a, st);
    // one wave: only D = 64 (with D = 128 a lone wave would spill while it streams tiles)
    if constexpr (D < 128) return launch_dq<D, 1, CAUSAL>(a, st);
    return -1;
    }
}

// Order of a full backward: dQ (which also forms the row statistics and stores them), then
// dK/dV (which reads them).  The separate statistics kernel runs only when they are asked for
// without dQ.
template <int D>
static int launch_bwd_d(BwdArgs a, bool causal, hipStream_t st, unsigned stages)
{
    a.stats_in_dq = (stages & 5u) == 5u;
    if (stages & 4u) {
        if (causal ? launch_dq_for<D, true>(a, st) : launch_dq_for<D, false>(a, st)) return -1;
    } else if (stages & 1u) {
        constexpr int RPB = 256 / (D / 8);
        const int64_t rows = (int64_t)a.BH * a.S;
        hipLaunchKernelGGL((attn_bwd_delta_kernel<D>), dim3((unsigned)((rows + RPB - 1) / RPB)),
                           dim3(256), 0, st, a);
        if (hipGetLastError() != hipSuccess) return -1;
    }
    if (stages & 2u) return causal ? launch_dkdv<D, true>(a, st) : launch_dkdv<D, false>(a, st);
    return 0;
}

// Split the dQ kernel over the keys when its 256-row work-groups would leave compute units
// (256) idle: aim at one work-group per unit, every split at least eight 64-key tiles (the
// merge reads and writes one fp32 partial per split and row).  Needs at least 256 query rows
// per head (a 256-row work-group must have rows to work on) -- decoding shapes have one row per
// head and many heads, and are not split.
#ifndef ATTN_F16  // a function of the shape only: defined once, by the bf16 build
int dq_split_plan(int BH, int S, int Sk, int D, bool causal, int *kps)
{
    (void)causal;
    if (D > 128) {  // the kernel for head dimensions above 128 is not split
        if (kps) *kps = (Sk + 63) / 64 * 64;
        return 1;
    }
    const int64_t wgs = (int64_t)BH * ((S + 255) / 256);
    const int tiles = (Sk + 63) / 64;
    int nsplit = 1;
    if (S >= 256 && wgs < 256 && tiles >= 16) {
        nsplit = (int)((256 + wgs - 1) / wgs);
        if (nsplit > tiles / 8) nsplit = tiles / 8;
        if (nsplit > 16) nsplit = 16;
    }
    const int tiles_per = (tiles + nsplit - 1) / nsplit;
    nsplit = (tiles + tiles_per - 1) / tiles_per;  // no empty split
    if (kps) *kps = tiles_per * 64;
    return nsplit;
}
#endif

int launch_bwd(const BwdArgs &a, int D, bool causal, hipStream_t st, unsigned stages)
{
    // short heads, the full backward: one fused launch.  With grouped-query heads its work-group
    // walks the query heads of a K/V head one after the other, which pays once there is a K/V
    // head for every compute unit (measured: 10-26 % faster from 256 K/V heads on, slower below,
    // where the two-kernel form spreads the query heads over the chip)
    if (stages == 7u && (a.S > a.Sk ? a.S : a.Sk) <= bwd_small_max_rows(D) &&
        (a.group == 1 || a.BH / a.group >= 256))
        return launch_bwd_small(a, D, causal, st);
    return D == 256 ? launch_bwd_d<256>(a, causal, st, stages)
         : D == 128 ? launch_bwd_d<128>(a, causal, st, stages)
                    : launch_bwd_d<64>(a, causal, st, stages);
}

}  // namespace attn
