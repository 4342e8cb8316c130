// Fused attention forward for gfx950: O = softmax(scale * Q K^T [+ causal mask]) V and the
// per-row natural-log LSE, one pass over K/V with an online softmax (the
// "flash-attention-style formulation" the paper's debugging table refers to).
//
// Work decomposition
//   work-group = NW waves, one tile of BR = 32*NW query rows of one (batch, head);
//   wave       = 32 query rows; loops over key tiles of BC = 64 rows staged in LDS.
// The score tile is computed TRANSPOSED, S^T = K Q^T (keys x queries), with the
// 32x32x16 elem MFMA.  Its accumulator layout puts one query per lane (column l%32) and
// 16 keys per lane and 32-key block, so
//   - row max / row sum are in-lane reductions plus ONE exchange with lane l^32,
//   - the rescale factor alpha is a per-lane scalar,
//   - elem(P^T) is already in the B-operand layout of the second MFMA,
//     O^T = V^T P^T (d x queries), once the contraction index is enumerated in the order
//     the accumulator holds it (key = 8*(t/4) + 4*(l/32) + t%4 within 16 keys).
// K and V tiles reach LDS by direct global -> LDS transfers, both row-major.  The K operand is a
// plain 16-byte read; V^T is produced by the reads themselves (two LDS transpose reads per
// fragment, which deliver the keys in exactly that order).  Staging V through registers with a
// 4x4 register transpose, so that its operand is a plain read as well, costs more vector
// instructions than the slower transpose reads do (measured in the kernel: 3-5 % slower).
//
// Software pipeline (per wave): the MFMAs of S^T(j+1) are issued in the same block as the
// softmax arithmetic of tile j, so the matrix pipe and the vector ALU overlap inside one
// wave as well as across the two waves of a SIMD.  The vector ALU issue port is the scarce
// resource (it also carries the MFMA issue and the LDS read returns), so the common path
// does no max reduction at all: probabilities are taken relative to a reference max that is
// only moved when a partial row sum shows that some probability outgrew 2^10 (the O
// accumulator and row sum are then rescaled and the sub-tile redone).  Any reference gives
// the same O and LSE after the final division by the row sum.
#include "attn_device.hpp"
#include "attn_launch.hpp"

namespace attn {

template <int D, int NW>
struct FwdCfg {
    static constexpr int kThreads = NW * 64;
    static constexpr int kBR = NW * 32;
    static constexpr int kBC = 64;
    // K tile: one wave-wide transfer of 16 B per lane fills a 1 KB piece of kKRowsPerDma
    // rows; within a piece the 16-byte chunks are stored chunk-major (chunk c of row r at
    // 16 * (c * rows + r % rows)) and consecutive pieces lie 16 * rows bytes further apart than
    // their size.  The fragment a lane needs for contraction step ks is then at a per-lane
    // constant plus ks * kKStep -- one address register instead of one per step -- and the 16
    // rows that one quarter of a wave reads at a fixed chunk fall into 16 different 16-byte
    // bank groups.
    static constexpr int kKRowsPerDma = 1024 / (D * 2);        // rows one wave-wide 16 B/lane load fills
    static constexpr int kKPieceBytes = 1024 + kKRowsPerDma * 16;
    static constexpr int kKDmas = kBC / kKRowsPerDma;          // such loads per tile
    static constexpr int kKTile = kKDmas * kKPieceBytes / 2;   // in elements
    static constexpr int kKHalf = kKTile / 2;                  // 32 rows further
    static constexpr int kKStep = 2 * kKRowsPerDma * 16 / 2;   // next contraction step, in elements
    static constexpr int kKDmaPerWave = (kKDmas + NW - 1) / NW;
    // V tile: the same transfers and layout as the K tile (row-major rows in chunk-major pieces);
    // it is transposed by the reads (LDS transpose read), whose 64 lanes fetch 4 rows x 4 chunks
    // x 2 halves = 512 contiguous bytes of a piece.
    static constexpr int kVTile = kKTile;                                  // in elements
    static constexpr int kVRows16 = (16 / kKRowsPerDma) * kKPieceBytes;   // 16 rows further, in bytes
    // V tiles: two, or three for the eight-wave kernel, whose main loop multiplies P of a
    // sub-tile by V one sub-tile later and therefore still reads tile kt-1 while tile kt+1 is
    // arriving
    static constexpr int kVBufs = NW == 8 ? 3 : 2;
    // Eight waves: the query rows reach the registers through LDS (see the kernel's prologue):
    // the 64 rows of a pair of waves are staged like a K tile, pair 0 in K buffer 2, pair 1 in
    // V buffer 1 (both free until the first tile barrier), pairs 2 and 3 behind the V buffers.
    static constexpr int kQStage = NW == 8 ? 2 * kKTile : 0;
    static constexpr int kLdsBytes = (3 * kKTile + kVBufs * kVTile + kQStage) * 2;
    static_assert(kLdsBytes <= 160 * 1024, "LDS budget of a gfx950 CU exceeded");
};

// A sub-tile's probabilities are taken relative to a reference max that is only moved when
// one lane's partial row sum (16 keys) exceeds this bound, i.e. some exp2 argument > ~10.
constexpr float kOverflow = 1024.0f;
constexpr float kMinusHuge = -1.0e30f;  // initial reference: finite, so masked -inf scores give 0

template <int D, int NW, bool CAUSAL, bool SPLIT>
__global__ void __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2)))
attn_fwd_kernel(const FwdArgs a)
{
    using C = FwdCfg<D, NW>;
    constexpr int KS = D / 16;  // contraction steps of K Q^T
    constexpr int DB = D / 32;  // 32-row blocks of O^T
    extern __shared__ __attribute__((aligned(16))) char smem[];
    elem *Ks = reinterpret_cast<elem *>(smem);  // [3][64][D] swizzled
    elem *Vs = Ks + 3 * C::kKTile;              // [kVBufs] tiles in the K tile's layout

    const int tid = threadIdx.x, l = tid & 63, r = l & 31, h = l >> 5;
    const int w = tid >> 6;
    const int S = a.S, Dr = a.Dr;

    // (head, query tile) of this work-group; causal tiles are issued heaviest first.
    int bh, rank;
    xcd_tile_order<CAUSAL>(blockIdx.x, a.nqt, a.BH, bh, rank);
    const int qt = CAUSAL ? a.nqt - 1 - rank : rank;
    const int64_t base = (int64_t)(bh / a.H) * a.stride_b + (int64_t)(bh % a.H) * a.stride_h;
    // grouped-query heads: query head h reads K/V head h / group
    const int64_t base_kv = (int64_t)(bh / a.H) * a.kv_stride_b +
                            (int64_t)((bh % a.H) / a.group) * a.kv_stride_h;
    const elem *Qp = a.Q + base, *Kp = a.K + base_kv, *Vp = a.V + base_kv;
    // Keys seen by this work-group: all Sk of them, or one split's range (then K and V are
    // simply re-based to the range and the causal offset moves with them).  Query row i sees
    // key j iff j <= i + coff.
    int Sk = a.Sk, coff = a.Sk - S;
    if (SPLIT) {
        const int k_begin = blockIdx.y * a.kps;  // < Sk by the launcher's plan
        Kp += (int64_t)k_begin * a.kv_stride_s;
        Vp += (int64_t)k_begin * a.kv_stride_s;
        Sk = min(Sk - k_begin, a.kps);
        coff -= k_begin;
    }

    const int q0 = qt * C::kBR + w * 32;  // first query row of this wave
    const int q = q0 + r;                 // this lane's query row
    const int qc = q < S ? q : S - 1;     // clamped for loads; rows >= S are never stored

    // Q fragments, B operand of K Q^T: lane holds Q[q][16*ks + 8h .. +7].  Fewer than eight
    // waves load them straight from memory.  Eight waves take them through LDS (below): a load
    // in which every lane fetches 16 bytes of its own row touches 32 rows per instruction, and
    // the 64 such instructions of a work-group took its last wave 5000-7000 cycles to get issued
    // (measured) -- time in which the compute unit, which holds one such work-group, does nothing.
    elem8 qf[KS];
    if constexpr (NW != 8) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qf[ks] = as_elem8(ld_row16(Qp + (int64_t)qc * a.stride_s, ks * 16 + 8 * h, Dr));
    }

    // Key tiles this work-group visits.
    const int q_end = min(S, (qt + 1) * C::kBR);
    const int k_end = CAUSAL ? min(Sk, q_end + coff) : Sk;  // <= 0: nothing visible (splits only)
    const int n_kt = k_end > 0 ? (k_end + C::kBC - 1) / C::kBC : 0;
    const int q0e = q0 + coff;  // the wave's first row in key coordinates

    // ---- staging: global -> LDS.  Rows past S-1 and tiles past the last one
    // lie outside the head's buffer resource and read as zero (masked to probability 0).
    // Columns Dr..D-1 (head dimensions below the kernel's D) are fetched at an offset past the
    // end of the resource, so they read as zero like everything else outside it.
    const uint32_t head_bytes = (uint32_t)(((int64_t)(Sk - 1) * a.kv_stride_s + Dr) * 2);
    const desc_t Kd = make_desc(Kp, head_bytes), Vd = make_desc(Vp, head_bytes);
    const uint32_t lds0 = lds_address(smem);
    const uint32_t row_bytes = (uint32_t)a.kv_stride_s * 2u;
    const uint32_t tile_bytes = C::kBC * row_bytes;
    // K and V go global -> LDS directly (no registers): one wave-wide transfer of 16 B per lane
    // fills 1 KB of LDS in lane order; lane l fetches the chunk that belongs at its position of the
    // piece, chunk l / rows of row l % rows.  The piece's first row goes into the scalar
    // offset (which takes part in the range check like the per-lane one).  The transfers are
    // issued from assembly, out of the compiler's sight (it would otherwise make the wave wait for
    // all of them before its next transpose read of LDS); tile_barrier() orders them against the
    // reads.  They fill buffers that nobody reads before the next barrier.
    constexpr int PR = C::kKRowsPerDma;
    const uint32_t k_voff = (l / PR) * 8 < Dr ? (l % PR) * row_bytes + ((l / PR) << 4) : head_bytes;
    auto dma_tile = [&](desc_t desc, uint32_t lds_tile, int kt) __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < C::kKDmaPerWave; ++n) {
            // which 1 KB piece of the tile: wave-uniform
            const int ii = __builtin_amdgcn_readfirstlane(w) + n * NW;
            if (C::kKDmas % NW == 0 || ii < C::kKDmas)
                dma16_between(desc, lds_tile + ii * C::kKPieceBytes, k_voff, kt * tile_bytes + ii * PR * row_bytes);
        }
    };
    auto dma_k = [&](int kt, int buf) __attribute__((always_inline)) {
        dma_tile(Kd, lds0 + buf * (C::kKTile * 2), kt);
    };
    auto dma_v = [&](int kt, int buf) __attribute__((always_inline)) {
        dma_tile(Vd, lds0 + (3 * C::kKTile + buf * C::kVTile) * 2, kt);
    };

    float m = kMinusHuge;  // reference max of c*s (log2 units), identical in lanes l and l^32
    float lsum = 0.f;     // running sum of this lane's half of the keys
    f32x16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
    const float c = a.scale_log2e;

    // ---- MFMA steps and their LDS operand fetches.  Work proceeds in sub-tiles of 32 keys
    // (one 32x32 score block per wave).  One step is four (D=128) MFMAs whose A fragments
    // are fetched a step ahead into the other of two fragment sets, so the LDS latency hides
    // behind the previous step's MFMAs.
    constexpr int NKQ = KS / 4;  // K Q^T steps per sub-tile, four contraction steps each
    // element offset of this lane's fragment for contraction step 0 within a 32-row half
    // tile: chunk h of row r
    // The per-lane parts of the LDS addresses are kept in one register each and made opaque to
    // the compiler, so that buffer, sub-tile and step are folded into the 16-bit immediate
    // offset of the LDS instruction instead of into further address registers.  (The V region
    // starts beyond what an immediate reaches from zero, so its registers include its base.)
    int k_lane = ((r / PR) * (C::kKPieceBytes / 2) + (h * PR + r % PR) * 8) * 2;
    // transpose reads of a V tile: the 16-lane group reads rows 4h + e (e = 0..3; +8 for the
    // second read), 64 bytes of d block 0 of each row -- the keys of contraction half h in the
    // order the accumulator of S^T holds them
    auto v_at = [](int row, int chunk) {
        return (row / PR) * C::kKPieceBytes + (chunk * PR + row % PR) * 16;
    };
    int v_lane0 = 3 * C::kKTile * 2 + v_at(4 * h + ((l & 15) >> 2), 2 * ((l >> 4) & 1) + ((l >> 1) & 1)) + (l & 1) * 8;
    int v_lane1 = 3 * C::kKTile * 2 + v_at(8 + 4 * h + ((l & 15) >> 2), 2 * ((l >> 4) & 1) + ((l >> 1) & 1)) + (l & 1) * 8;
    asm volatile("" : "+v"(k_lane), "+v"(v_lane0), "+v"(v_lane1));
    auto ld_k = [&](const elem *Kt, int kq, elem8 (&f)[4]) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
            f[t] = *(const elem8 *)((const char *)(Kt + (4 * kq + t) * C::kKStep) + k_lane);
    };
    auto mm_k = [&](int kq, const elem8 (&f)[4], f32x16 &t0) {
#pragma unroll
        for (int t = 0; t < 4; ++t) t0 = mfma32(f[t], qf[4 * kq + t], t0);
    };
    // V^T fragment: lane (d = 32*db + l%32, half h) gets the 8 keys of contraction step cc
    // that its half owns, from two transpose reads.  Vt: byte offset of tile and sub-tile
    // within the V region.
    auto ld_v = [&](int Vt, int cc, elem8 (&f)[4]) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const char *p = smem + Vt + cc * C::kVRows16 + db * 4 * PR * 16;  // d block db: four chunks further
            f[db] = join8(lds_read_tr((const elem *)(p + v_lane0)), lds_read_tr((const elem *)(p + v_lane1)));
        }
    };
    // Row sums of the ROUNDED probabilities (one packed dot product with a vector of ones per
    // element pair; this lane's half of the keys, both halves are added at the end like the
    // exact sum).  O is divided by this sum, so that the rounding of P cancels between
    // numerator and denominator: the reference max is not the true row max, so the dominant
    // probability of a peaked row is in general not exactly representable, and dividing by the
    // exact sum would leave its rounding error (up to 2^-9 relative) in O.  LSE is still made
    // from the exact fp32 sum.
    float hsum = 0.f;
    auto mm_v = [&](const elem8 (&f)[4], elem8 p) {
#pragma unroll
        for (int db = 0; db < DB; ++db) o[db] = mfma32(f[db], p, o[db]);
#pragma unroll
        for (int i = 0; i < 4; ++i) hsum = dot2_acc(p[2 * i], p[2 * i + 1], hsum);
    };
    // exp2 of eight scores against the reference max, fp32 row-sum, and elem pack
    auto softmax8 = [&](const f32x16 &t, int i0, float &psum) -> elem8 {
        float e[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            e[i] = fast_exp2(__builtin_fmaf(t[i0 + i], c, -m));
            psum += e[i];
        }
        return pack8(e[0], e[1], e[2], e[3], e[4], e[5], e[6], e[7]);
    };
#define ATTN_FENCE() __builtin_amdgcn_sched_barrier(0)

    // One 32-key sub-tile g = 2*kt + u for an active wave: softmax and P V of sub-tile g
    // (scores in cur) overlapped with S^T of sub-tile g+1 (into nxt; one sub-tile past the
    // end reads zero rows and is unused).  Four fragment sets rotate through the steps
    //   K0 (f0), K1 (f1): S^T(g+1) += K Q^T      V0 (f2), V1 (f3): O^T += V^T P^T(g)
    // and every set is fetched two steps before it is consumed; the K fragments of sub-tile
    // g+2 (tile kt+1, resident since the previous iteration) are fetched during V0/V1.
    elem8 f0[4], f1[4], f2[4], f3[4];
    // The reference max moves to the true running max: rescale what has been accumulated and
    // redo the probabilities of the sub-tile whose scores are in cur.
    auto move_reference = [&](const f32x16 &cur, elem8 &p0, elem8 &p1, float &psum)
                              __attribute__((always_inline)) {
        float mx = cur[0];
#pragma unroll
        for (int i = 1; i < 16; i += 3)
            mx = fmaxf(mx, fmaxf(cur[i], fmaxf(cur[i + 1], cur[i + 2])));
        mx = xhalf_max(mx) * c;
        const float m_new = fmaxf(m, mx);
        const float alpha = fast_exp2(m - m_new);
        m = m_new;
        lsum *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
        hsum *= alpha;
        psum = 0.f;
        p0 = softmax8(cur, 0, psum);
        p1 = softmax8(cur, 8, psum);
    };
    // vb: buffer of V(kt); vb_fill: buffer that takes V(kt+1)
    auto subtile = [&](int kt, int u, int kbuf_next, int kbuf_fill, int vb, int vb_fill, bool masked,
                       f32x16 &cur, f32x16 &nxt) __attribute__((always_inline)) {
        const elem *Kn = Ks + kbuf_next * C::kKTile + u * C::kKHalf;  // rows of sub-tile g+2
        const int Vt = vb * (C::kVTile * 2) + 2 * u * C::kVRows16;
        // ---- K0
        ld_v(Vt, 0, f2);
        if (NKQ == 1) ld_v(Vt, 1, f3);
        if (u == 0) dma_k(kt + 2, kbuf_fill);  // K(kt+2) -> the buffer freed at the last barrier
#pragma unroll
        for (int i = 0; i < 16; ++i) nxt[i] = 0.f;
        if (masked) {
            // Ragged tail and causal mask: only sub-tiles that touch the end or the diagonal.
            const int lim = (CAUSAL ? min(qc + coff, Sk - 1) : Sk - 1) - (kt * C::kBC + 32 * u) - 4 * h;
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (8 * (i / 4) + (i % 4) > lim) cur[i] = -INFINITY;
        }
        float psum = 0.f;
        elem8 p0 = softmax8(cur, 0, psum);
        mm_k(0, f0, nxt);
        ATTN_FENCE();
        // ---- K1
        if (NKQ > 1) {
            ld_v(Vt, 1, f3);
            mm_k(1, f1, nxt);
        }
        elem8 p1 = softmax8(cur, 8, psum);
        // Rare path: some probability outgrew 2^10 relative to the reference max (always so
        // for a wave's first sub-tile).  Move the reference to the true running max, rescale
        // what has been accumulated, and redo this sub-tile's probabilities.
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(psum > kOverflow) != 0, 0)) move_reference(cur, p0, p1, psum);
        ATTN_FENCE();
        // ---- V0 (first sub-tile: V(kt+1) -> the buffer freed at the last barrier)
        ld_k(Kn, 0, f0);
        mm_v(f2, p0);
        if (u == 0) dma_v(kt + 1, vb_fill);
        ATTN_FENCE();
        // ---- V1
        if (NKQ > 1) ld_k(Kn, 1, f1);
        mm_v(f3, p1);
        lsum += psum;
        ATTN_FENCE();
    };

    // ---- prologue: K(0), K(1), V(0) resident; V(1) in flight; first S^T block computed and
    // the K fragments of the second sub-tile on their way.
    // Eight waves: the wave's 32 query rows as half of a K-layout tile, by the same direct
    // transfers (whole rows of four per instruction), issued before those of K and V.  Rows past
    // S-1 and columns Dr..D-1 read as zero.
    uint32_t q_stage = 0;
    if constexpr (NW == 8) {
        const int pair = __builtin_amdgcn_readfirstlane(w) >> 1, half = __builtin_amdgcn_readfirstlane(w) & 1;
        q_stage = (pair == 0 ? 2 * C::kKTile : pair == 1 ? 3 * C::kKTile + C::kVTile
                                                          : 3 * C::kKTile + 3 * C::kVTile + (pair - 2) * C::kKTile) * 2 +
                  half * (C::kKHalf * 2);
        const int row0 = qt * C::kBR + pair * 64;
        const int rows = min(64, S - row0);
        const uint32_t q_bytes = rows > 0 ? (uint32_t)(((int64_t)(rows - 1) * a.stride_s + Dr) * 2) : 0u;
        const desc_t Qd = make_desc(Qp + (int64_t)(rows > 0 ? row0 : 0) * a.stride_s, q_bytes);
        const uint32_t q_row_bytes = (uint32_t)a.stride_s * 2u;
        const uint32_t q_voff = (l / PR) * 8 < Dr ? (l % PR) * q_row_bytes + ((l / PR) << 4) : q_bytes;
#pragma unroll
        for (int n = 0; n < C::kKDmas / 2; ++n)
            dma16_between(Qd, lds0 + q_stage + n * C::kKPieceBytes, q_voff,
                          (half * (C::kKDmas / 2) + n) * PR * q_row_bytes);
    }
    dma_k(0, 0);
    dma_k(1, 1);
    dma_v(0, 0);
    // Rotary embedding of the query rows, fused into their load (head dimension == D only):
    // column d pairs with d + D/2, i.e. fragment ks with ks + KS/2, element by element, in this
    // lane; fp32 arithmetic on the widened values, rounded once -- what a separate rotary pass
    // would have written to memory as bf16.  The table rows are requested here, after the first
    // K and V tiles, so that all of them are in flight together, and used further down.
    f32x4 rc[KS][2], rs[KS][2];  // [ks][half of the 8 columns]; only ks < KS/2 is used
    if (a.rope_cos) {
        const int64_t pos = (int64_t)(qc * a.rope_row_step + a.rope_pos0) * (D / 2);
#pragma unroll
        for (int ks = 0; ks < KS / 2; ++ks)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                rc[ks][j] = *(const f32x4 *)(a.rope_cos + pos + 16 * ks + 8 * h + 4 * j);
                rs[ks][j] = *(const f32x4 *)(a.rope_sin + pos + 16 * ks + 8 * h + 4 * j);
            }
    }
    if constexpr (NW == 8) {
        // the wave's own query rows have landed once at most the later transfers (K(0), K(1),
        // V(0)) are outstanding; with the rotary table rows in flight as well, whose place in the
        // order of issue is the compiler's choice, everything is awaited
        if (a.rope_cos) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(3 * C::kKDmaPerWave) : "memory");
        const char *Qs = smem + q_stage + ((r / PR) * C::kKPieceBytes + (h * PR + r % PR) * 16);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = *(const elem8 *)(Qs + ks * (C::kKStep * 2));
        // ... and are in registers before anybody may overwrite the staging space
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    if (a.rope_cos) {
        elem *qr = a.Qrot ? a.Qrot + base + (int64_t)qc * a.stride_s : nullptr;
#pragma unroll
        for (int ks = 0; ks < KS / 2; ++ks) {
            float lo[8], hi[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const float x1 = (float)qf[ks][t], x2 = (float)qf[ks + KS / 2][t];
                const float cc = rc[ks][t >> 2][t & 3], ss = rs[ks][t >> 2][t & 3];
                lo[t] = __builtin_fmaf(x1, cc, -(x2 * ss));
                hi[t] = __builtin_fmaf(x2, cc, x1 * ss);
            }
            qf[ks] = pack8(lo[0], lo[1], lo[2], lo[3], lo[4], lo[5], lo[6], lo[7]);
            qf[ks + KS / 2] = pack8(hi[0], hi[1], hi[2], hi[3], hi[4], hi[5], hi[6], hi[7]);
            if (qr && q < S && (!SPLIT || blockIdx.y == 0)) {
                *(elem8 *)(qr + 16 * ks + 8 * h) = qf[ks];
                *(elem8 *)(qr + 16 * (ks + KS / 2) + 8 * h) = qf[ks + KS / 2];
            }
        }
    }
    if constexpr (NW == 8) {
        // The main loop's first iteration multiplies an all-zero P by the second half of V
        // buffer 2, which nothing has written yet: give it finite contents.
        const u32x4 z = {0u, 0u, 0u, 0u};
        for (int i = tid; i < C::kVTile / 8; i += C::kThreads)
            *(u32x4 *)(Vs + 2 * C::kVTile + 8 * i) = z;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // K(0), K(1), V(0) have landed
    __syncthreads();
    f32x16 sa, sb;
    {
#pragma unroll
        for (int i = 0; i < 16; ++i) sa[i] = 0.f;
        ld_k(Ks, 0, f0);
        if (NKQ > 1) ld_k(Ks, 1, f1);
        mm_k(0, f0, sa);
        if (NKQ > 1) mm_k(1, f1, sa);
        ATTN_FENCE();
        ld_k(Ks + C::kKHalf, 0, f0);
        if (NKQ > 1) ld_k(Ks + C::kKHalf, 1, f1);
    }

    // Main-loop form of a sub-tile (eight-wave kernel, sub-tiles that the wave sees in full):
    // the probabilities of sub-tile g are multiplied by V one sub-tile LATER.  The iteration
    // then holds three independent pieces of work -- S^T(g+1) = K Q^T, the softmax arithmetic
    // of g, and O^T += V^T P^T(g-1) -- in one basic block with nothing to mask, and the test
    // whether the reference max must move sits at its end instead of between the softmax and
    // the second MFMA phase, where it made every wave wait for its last exp2 before it could
    // issue the next MFMA (measured: the same arithmetic without that branch in the middle
    // runs 15 % faster).  pp0/pp1 carry P(g-1) into the iteration; vprev is the buffer that
    // holds the V rows of sub-tile g-1 (tile kt-1 for u == 0, tile kt for u == 1).
    elem8 pp0, pp1;
#pragma unroll
    for (int i = 0; i < 8; ++i) pp0[i] = pp1[i] = (elem)0.f;
    auto subtile_main = [&](int kt, int u, int kbuf_next, int kbuf_fill, int vprev, int vb_fill,
                            f32x16 &cur, f32x16 &nxt) __attribute__((always_inline)) {
        const elem *Kn = Ks + kbuf_next * C::kKTile + u * C::kKHalf;  // rows of sub-tile g+2
        const int Vt = vprev * (C::kVTile * 2) + 2 * (1 - u) * C::kVRows16;  // rows of sub-tile g-1
        // The softmax arithmetic of g is spread evenly over the four MFMA steps (four scores
        // each), so that every step has about three quarters as many vector-ALU cycles as
        // matrix-pipe cycles.
        float e[16], psum = 0.f;
        auto exp4 = [&](int i0) __attribute__((always_inline)) {
#pragma unroll
            for (int i = i0; i < i0 + 4; ++i) {
                e[i] = fast_exp2(__builtin_fmaf(cur[i], c, -m));
                psum += e[i];
            }
        };
        auto hsum4 = [&](elem8 p) __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < 4; ++i) hsum = dot2_acc(p[2 * i], p[2 * i + 1], hsum);
        };
        auto mm_o = [&](const elem8 (&f)[4], elem8 p) __attribute__((always_inline)) {
#pragma unroll
            for (int db = 0; db < DB; ++db) o[db] = mfma32(f[db], p, o[db]);
        };
        // ---- K0
        ld_v(Vt, 0, f2);
        if (NKQ == 1) ld_v(Vt, 1, f3);
        // (both tiles' transfers right after the barrier: the V buffer being filled was last read
        // before the previous barrier; measured the same or up to 1 % faster than V two steps later)
        if (u == 0) {
            dma_k(kt + 2, kbuf_fill);
            dma_v(kt + 1, vb_fill);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) nxt[i] = 0.f;
        exp4(0);
        hsum4(pp0);
        mm_k(0, f0, nxt);
        ATTN_FENCE();
        // ---- K1
        if (NKQ > 1) {
            ld_v(Vt, 1, f3);
            mm_k(1, f1, nxt);
        }
        exp4(4);
        hsum4(pp1);
        elem8 p0 = pack8(e[0], e[1], e[2], e[3], e[4], e[5], e[6], e[7]);
        ATTN_FENCE();
        // ---- V0
        ld_k(Kn, 0, f0);
        mm_o(f2, pp0);
        exp4(8);
        ATTN_FENCE();
        // ---- V1
        if (NKQ > 1) ld_k(Kn, 1, f1);
        mm_o(f3, pp1);
        exp4(12);
        elem8 p1 = pack8(e[8], e[9], e[10], e[11], e[12], e[13], e[14], e[15]);
        ATTN_FENCE();
        // rare: some probability of g outgrew 2^10 (always so for a wave's first sub-tile);
        // what has been accumulated (up to g-1) is rescaled, P(g) redone
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(psum > kOverflow) != 0, 0)) move_reference(cur, p0, p1, psum);
        lsum += psum;
        pp0 = p0;
        pp1 = p1;
    };
    // Every transfer this wave issued during the tile (its pieces of K(kt+2) and V(kt+1)) must
    // have landed before the other waves are let past the barrier to read them.
    auto tile_barrier = [&]() {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    };

    // One loop iteration = one staged tile of 64 keys = two sub-tiles.  Staging is folded
    // into the first sub-tile's steps.  During iteration kt the waves read K(kt) (second
    // half) and K(kt+1) (first half), so K is triple-buffered and K(kt+2) streams into the
    // third buffer; V(kt+1) replaces the oldest V tile, whose last readers finished before the
    // previous barrier.
    int kt0 = 0;  // first tile of the generic loop below
    if constexpr (NW == 8) {
        // Tiles that this wave sees in full (no key past the end, none above its diagonal), in
        // whole groups of three: the loop is unrolled over the three K (and V) buffers so that
        // the buffer of every access is a compile-time constant and the LDS addresses of the
        // fragments are a loop-invariant register plus an immediate offset.
        const int seen = CAUSAL ? min(Sk, q0e + 1) : Sk;  // keys 0 .. seen-1 are visible to every row of the wave
        // (rows past S: never more than n_kt; the same in every lane of the wave, and said so,
        // so that the loop is controlled by scalar registers)
        const int n_main = __builtin_amdgcn_readfirstlane(min(max(seen, 0) / C::kBC, n_kt) / 3 * 3);
        for (int kt = 0; kt < n_main; kt += 3) {
            subtile_main(kt, 0, 1, 2, 2, 1, sa, sb);
            subtile_main(kt, 1, 1, 2, 0, 1, sb, sa);
            tile_barrier();
            subtile_main(kt + 1, 0, 2, 0, 0, 2, sa, sb);
            subtile_main(kt + 1, 1, 2, 0, 1, 2, sb, sa);
            tile_barrier();
            subtile_main(kt + 2, 0, 0, 1, 1, 0, sa, sb);
            subtile_main(kt + 2, 1, 0, 1, 2, 0, sb, sa);
            tile_barrier();
        }
        if (n_main > 0) {
            // the last sub-tile's P V is still owed: second half of V(n_main - 1), buffer 2
            const int Vt = 2 * (C::kVTile * 2) + 2 * C::kVRows16;
            ld_v(Vt, 0, f2);
            ld_v(Vt, 1, f3);
            mm_v(f2, pp0);
            mm_v(f3, pp1);
        }
        kt0 = n_main;  // a multiple of three: K(kt0) and V(kt0) are in buffer 0 again
    }
    // Generic form of a tile (the tiles at the diagonal and the ragged end of the eight-wave
    // kernel; every tile with fewer waves).  kb1, kb2: buffers of K(kt+1), K(kt+2); vb, vb1:
    // buffers of V(kt), V(kt+1).
    auto tile = [&](int kt, int kb1, int kb2, int vb, int vb1) __attribute__((always_inline)) {
        const int kb = kt * C::kBC;
        // wave-uniform: does the wave see any key of the sub-tile / must it mask some
        if (!CAUSAL || kb <= q0e + 31) {
            subtile(kt, 0, kb1, kb2, vb, vb1, (kb + 32 > Sk) || (CAUSAL && kb + 31 > q0e), sa, sb);
        } else {
            dma_k(kt + 2, kb2);
            dma_v(kt + 1, vb1);
        }
        if (!CAUSAL || kb + 32 <= q0e + 31)
            subtile(kt, 1, kb1, kb2, vb, vb1, (kb + 64 > Sk) || (CAUSAL && kb + 63 > q0e), sb, sa);
        tile_barrier();
    };
    if constexpr (NW == 8) {
        // unrolled over the three buffers like the main loop (kt0 is a multiple of three)
        for (int kt = kt0; kt < n_kt; kt += 3) {  // n_kt is the same for every wave of the work-group
            tile(kt, 1, 2, 0, 1);
            if (kt + 1 < n_kt) tile(kt + 1, 2, 0, 1, 2);
            if (kt + 2 < n_kt) tile(kt + 2, 0, 1, 2, 0);
        }
    } else {
        // fewer waves stage more of each tile per wave and have no registers to spare for the
        // unrolled form: the buffer indices rotate at run time
        int kb1 = 1, kb2 = 2, kb0 = 0;
        for (int kt = kt0; kt < n_kt; ++kt) {
            tile(kt, kb1, kb2, kt & 1, (kt + 1) & 1);
            const int t = kb0; kb0 = kb1; kb1 = kb2; kb2 = t;
        }
    }
#undef ATTN_FENCE

    // Epilogue: O = O_acc / l, LSE = ln2 * (m + log2 l).
    const float lt = xhalf_sum(lsum);
    const float lr = xhalf_sum(hsum);  // sum of the rounded probabilities
    // Eight waves.  The accumulator holds 4 consecutive columns of one row per register group, so
    // a direct store writes 16 bytes to each of 32 rows per instruction, sixteen times per wave.
    // The rows go through LDS instead and leave whole, 16 bytes per lane and four (D = 128) or
    // eight rows per instruction: half as many stores, each over contiguous memory.  The wave's
    // staging space (32 rows in the K tile's layout) lies in the K buffers and the query staging
    // space, which nobody reads after the last tile barrier.
    constexpr int kWaveBytes = C::kKHalf * 2;
    char *const stg = smem + (NW != 8 ? 0 : w < 6 ? w * kWaveBytes
                                                  : (3 * C::kKTile + 3 * C::kVTile) * 2 + (w - 6) * kWaveBytes);
    auto at = [](int row, int chunk) {
        return (row / PR) * C::kKPieceBytes + (chunk * PR + row % PR) * 16;
    };
    if (SPLIT) {
        // normalised fp32 partial result of this key range; a row that saw no key of the
        // range contributes O = 0 with LSE = -inf
        const float inv = lr > 0.f ? 1.0f / lr : 0.f;
        const int64_t row0 = ((int64_t)blockIdx.y * a.BH + bh) * S;
        if constexpr (NW == 8) {
            // through LDS like O below; an fp32 row is twice as long, so it goes in two halves
            constexpr int CPR = D / 8, RPI = 64 / CPR;
            const int lr_ = l / CPR, lc = l % CPR;
#pragma unroll
            for (int hp = 0; hp < 2; ++hp) {
#pragma unroll
                for (int db = hp * (DB / 2); db < (hp + 1) * (DB / 2); ++db)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        f32x4 ov;
#pragma unroll
                        for (int e = 0; e < 4; ++e) ov[e] = o[db][4 * g + e] * inv;
                        *(f32x4 *)(stg + at(r, (db % (DB / 2)) * 8 + 2 * g + h)) = ov;
                    }
                asm volatile("" ::: "memory");  // a wave's LDS accesses execute in order
#pragma unroll
                for (int j = 0; j < 32 / RPI; ++j) {
                    const f32x4 v = *(const f32x4 *)(stg + at(RPI * j + lr_, lc));
                    const int row = q0 + RPI * j + lr_;
                    if (row < S) *(f32x4 *)(a.Opart + (row0 + row) * D + hp * (D / 2) + lc * 4) = v;
                }
                asm volatile("" ::: "memory");
            }
            if (q < S && h == 0) a.LSEpart[row0 + q] = lt > 0.f ? (m + fast_log2(lt)) * kLn2 : -INFINITY;
        } else if (q < S) {
            float *Op = a.Opart + (row0 + q) * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f32x4 ov;
#pragma unroll
                    for (int e = 0; e < 4; ++e) ov[e] = o[db][4 * g + e] * inv;
                    *(f32x4 *)(Op + 32 * db + 8 * g + 4 * h) = ov;
                }
            if (h == 0) a.LSEpart[row0 + q] = lt > 0.f ? (m + fast_log2(lt)) * kLn2 : -INFINITY;
        }
        return;
    }
    const float inv = 1.0f / lr;
    if constexpr (NW == 8) {
        constexpr int CPR = D / 8, RPI = 64 / CPR;  // chunks per row; rows per store instruction
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                *(elem4 *)(stg + at(r, 4 * db + g) + 8 * h) =
                    pack4(o[db][4 * g] * inv, o[db][4 * g + 1] * inv, o[db][4 * g + 2] * inv, o[db][4 * g + 3] * inv);
        asm volatile("" ::: "memory");  // a wave's LDS accesses execute in order
        const int lr = l / CPR, lc = l % CPR;
#pragma unroll
        for (int j = 0; j < 32 / RPI; ++j) {
            const u32x4 v = *(const u32x4 *)(stg + at(RPI * j + lr, lc));
            const int row = q0 + RPI * j + lr;
            if (row < S && lc * 8 < Dr) *(u32x4 *)(a.O + base + (int64_t)row * a.stride_s + lc * 8) = v;
        }
        if (q < S && h == 0) a.LSE[(int64_t)bh * S + q] = (m + fast_log2(lt)) * kLn2;
    } else if (q < S) {
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

// Combine the per-split partial results: LSE = log sum_z exp(LSE_z), O = sum_z exp(LSE_z - LSE) O_z.
// A thread owns 4 consecutive d of one row and every ZG-th split, four splits per step with their
// loads issued together (a thread that walks all splits one load after the other spends a memory
// latency per split: 21 us for 32 splits of 32 rows), as a running (max, sum, weighted O) triple;
// the ZG triples of a row are then combined through LDS.  The order of the sums is a function of
// the shape only.  HBM-bound and small.
template <int D, int ZG>
__global__ void __launch_bounds__(256) attn_fwd_merge_kernel(const FwdArgs a)
{
    constexpr int TPR = D / 4;               // threads per row and split group
    constexpr int RPB = 256 / (TPR * ZG);    // rows per work-group
    static_assert(RPB >= 1, "a row's threads fit the work-group");
    const int64_t rows = (int64_t)a.BH * a.S;
    const int t = threadIdx.x;
    const int d0 = (t % TPR) * 4, zg = (t / TPR) % ZG;
    const int64_t row_raw = (int64_t)blockIdx.x * RPB + t / (TPR * ZG);
    const bool live = row_raw < rows;
    const int64_t row = live ? row_raw : rows - 1;  // clamped: every thread reaches the barrier
    const int nsplit = a.nsplit;
    float m = -INFINITY, den = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int z0 = zg; z0 < nsplit; z0 += 4 * ZG) {
        float lz[4];
        f32x4 oz[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int z = z0 + k * ZG;
            const int64_t at = (int64_t)(z < nsplit ? z : z0) * rows + row;
            lz[k] = a.LSEpart[at];
            oz[k] = *(const f32x4 *)(a.Opart + at * D + d0);
            if (z >= nsplit) lz[k] = -INFINITY;
        }
        const float mk = fmaxf(fmaxf(m, fmaxf(lz[0], lz[1])), fmaxf(lz[2], lz[3]));
        if (mk > -INFINITY) {  // (an empty split has LSE = -inf and weight 0)
            const float sc = expf(m - mk);
            den *= sc;
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] *= sc;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float wz = expf(lz[k] - mk);
                den += wz;
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] += wz * oz[k][e];
            }
            m = mk;
        }
    }
    if constexpr (ZG > 1) {
        __shared__ float red[256 * 6];
        red[t] = m;
        red[256 + t] = den;
#pragma unroll
        for (int e = 0; e < 4; ++e) red[(2 + e) * 256 + t] = acc[e];
        __syncthreads();
        if (zg != 0) return;
        float mm = m;
#pragma unroll
        for (int g = 1; g < ZG; ++g) mm = fmaxf(mm, red[t + g * TPR]);
        const float s0 = mm > -INFINITY ? expf(m - mm) : 0.f;
        den *= s0;
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] *= s0;
#pragma unroll
        for (int g = 1; g < ZG; ++g) {
            const int u = t + g * TPR;
            const float sg = mm > -INFINITY ? expf(red[u] - mm) : 0.f;
            den += sg * red[256 + u];
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] += sg * red[(2 + e) * 256 + u];
        }
        m = mm;
    }
    if (!live) return;
    const float inv = 1.0f / den;
    const int bh = (int)(row / a.S), q = (int)(row % a.S);
    elem *Op = a.O + (int64_t)(bh / a.H) * a.stride_b + (int64_t)(bh % a.H) * a.stride_h +
               a.row_offset(q) + d0;
    if (d0 < a.Dr) *(elem4 *)Op = pack4(acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv);
    if (d0 == 0) a.LSE[row] = m + logf(den);
}

template <int D, int ZG>
static int launch_fwd_merge_zg(const FwdArgs &a, hipStream_t st)
{
    const int64_t rows = (int64_t)a.BH * a.S;
    constexpr int RPB = 256 / ((D / 4) * ZG);
    hipLaunchKernelGGL((attn_fwd_merge_kernel<D, ZG>), dim3((unsigned)((rows + RPB - 1) / RPB)),
                       dim3(256), 0, st, a);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Up to four splits: one thread per (row, 4 d) takes them all in one step.  More: a row's splits
// are spread over as many thread groups as fit the work-group with it.
template <int D>
static int launch_fwd_merge(const FwdArgs &a, hipStream_t st)
{
    if (a.nsplit <= 4) return launch_fwd_merge_zg<D, 1>(a, st);
    return launch_fwd_merge_zg<D, (D > 128 ? 4 : 8)>(a, st);
}

template <int D, int NW, bool CAUSAL, bool SPLIT>
static int launch_fwd_kernel(const FwdArgs &a, hipStream_t st)
{
    using C = FwdCfg<D, NW>;
    if (hipFuncSetAttribute((const void *)attn_fwd_kernel<D, NW, CAUSAL, SPLIT>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, C::kLdsBytes) != hipSuccess)
        return -1;
    hipLaunchKernelGGL((attn_fwd_kernel<D, NW, CAUSAL, SPLIT>),
                       dim3(a.nqt * a.BH, SPLIT ? a.nsplit : 1), dim3(C::kThreads),
                       C::kLdsBytes, st, a);
    if (hipGetLastError() != hipSuccess) return -1;
    if (SPLIT) return launch_fwd_merge<D>(a, st);
    return 0;
}

template <int D, int NW>
static int launch_fwd_nw(const FwdArgs &a, bool causal, hipStream_t st)
{
    if (a.nsplit > 1)
        return causal ? launch_fwd_kernel<D, NW, true, true>(a, st)
                      : launch_fwd_kernel<D, NW, false, true>(a, st);
    return causal ? launch_fwd_kernel<D, NW, true, false>(a, st)
                  : launch_fwd_kernel<D, NW, false, false>(a, st);
}

// Waves per work-group: 8 (256 query rows) unless the sequence is too short to fill them.
// With D = 128 at least 4 (waves whose rows lie past the end compute and store nothing useful,
// but still take part in the staging): the one- and two-wave forms are only built for D = 64,
// and short problems at D = 128 go to the kernel of attn_fwd_wide.hip unless the rotary
// embedding is fused into the call.
static int fwd_waves_for(int S, int D, int BH, bool causal)
{
    const int blocks32 = (S + 31) / 32;
    // D = 64 under a causal mask with fewer than four 256-row work-groups per compute unit:
    // 128-row work-groups (three fit a compute unit at D = 64) balance the unequal tiles
    // better.  Measured: B=8 H=8 S=1024 26.5 -> 24.3 us, B=16 H=16 S=512 29.5 -> 27.6 us; not
    // so without a mask (+5 %), at D = 128 (+4..33 % on mid-size shapes) or on large problems.
    if (blocks32 >= 8 && D == 64 && causal && (int64_t)BH * ((S + 255) / 256) < 1024) return 4;
    if (blocks32 >= 8) return 8;
    // Three 32-row blocks also take four waves; the fourth has no rows and only stages K and V.
    // Measured at B=128 H=6 S=65: 13.6 -> 10.4 us, S=96: 15.4 -> 12.5 us.  The three-wave
    // kernel needs 177 registers at D = 64 (two waves per SIMD, two work-groups per compute
    // unit) against 150 for four waves (three work-groups), but capping it at 168 registers
    // (with 48 bytes of spills) did not make it faster, so the shorter staging per wave counts
    // as well.  Four waves for two blocks change nothing.
    if (blocks32 >= 3 || D == 128) return 4;
    return blocks32;  // 1 or 2
}

template <int D>
static int launch_fwd_d(FwdArgs a, bool causal, hipStream_t st)
{
    const int nw = fwd_waves_for(a.S, D, a.BH, causal);
    a.nqt = (a.S + nw * 32 - 1) / (nw * 32);
    if (nw == 8) return launch_fwd_nw<D, 8>(a, causal, st);
    if (nw == 4) return launch_fwd_nw<D, 4>(a, causal, st);
    if constexpr (D < 128) {
        if (nw == 2) return launch_fwd_nw<D, 2>(a, causal, st);
        return launch_fwd_nw<D, 1>(a, causal, st);
    }
    return -1;
}

// Split the keys when the unsplit launch would leave compute units (256) idle: aim at one
// work-group per unit.  (Measured on the decode shape: 256 work-groups with long key ranges
// beat 512 or 1024 shorter ones, 0.060 ms against 0.071 and 0.086 -- a work-group streams
// best when it stays in its pipelined loop, and a second round of work-groups only adds
// prologues.)  Every split keeps at least four 64-key tiles (the merge reads and writes one
// fp32 partial result per split and row).
#ifndef ATTN_F16  // a function of the shape only: defined once, by the bf16 build
int fwd_split_plan(int BH, int S, int Sk, int D, bool causal, int *kps)
{
    // (head dimensions above 128: four waves, 128 rows per work-group)
    const int nw = D > 128 ? 4 : fwd_waves_for(S, D, BH, causal);
    const int64_t wgs = (int64_t)BH * ((S + nw * 32 - 1) / (nw * 32));
    const int64_t target = 256;
    const int tiles = (Sk + 63) / 64;
    int nsplit = 1;
    if (wgs < target && tiles >= 8) {
        nsplit = (int)((target + wgs - 1) / wgs);
        if (nsplit > tiles / 4) nsplit = tiles / 4;
        if (nsplit > 128) nsplit = 128;
    }
    // Decoding (at most 32 rows per head) runs in the streaming kernel, of which two work-groups
    // fit a compute unit: aim at two per unit as far as that leaves every split 8 tiles or more
    // (B=8 Hkv=8 Sk=8192: 8 splits, 55.0 -> 49.5 us; B=16 H=16 Sk=4096: 2 splits, 111 -> 103 us;
    // B=1 Hkv=8 Sk=32768: 64 splits of 8 tiles 28.2 us against 30.0 with 32 of 16; four work-groups
    // per unit are 4-5 % slower again).
    if (S <= 32 && D <= 128 && wgs < 512) {
        int n2 = (int)((512 + wgs - 1) / wgs);
        if (n2 > tiles / 8) n2 = tiles / 8;
        if (n2 > 128) n2 = 128;
        if (n2 > nsplit) nsplit = n2;
    }
    const int tiles_per = (tiles + nsplit - 1) / nsplit;
    nsplit = (tiles + tiles_per - 1) / tiles_per;  // no empty split
    if (kps) *kps = tiles_per * 64;
    return nsplit;
}
#endif

// Which problems of D <= 128 go to the kernel of attn_fwd_wide.hip (128-row work-groups, two K/V
// buffers, two work-groups per compute unit at D = 128) instead of the one above.  Measured,
// forward only, graph replay, same box:
//  - at most 32 query rows per head (decoding; one wave of four has rows, the problem is K/V
//    streaming): B=8 Hq=32 Hkv=8 Sk=8192 66.7 -> 49.7 us, B=16 H=16 Sk=4096 143 -> 103;
//  - D = 128 and at most 128 rows: S=96 causal 18.8 -> 14.3 us (the kernel above needs four waves
//    at D = 128 whatever the length); 128 rows on 1024 keys the same either way.
// Everything else is faster above: mid-size causal D = 64 launches by 3-5 % (B=8 H=8 S=1024 22.5
// against 23.6 us), large launches by 7-12 %.
static bool prefer_streaming_forward(const FwdArgs &a, int D)
{
    if (a.S <= 32 || a.pack_sq) return true;  // (packed rows: only that kernel knows their positions)
    return D == 128 && a.S <= 128;
}

int launch_fwd(const FwdArgs &a, int D, bool causal, hipStream_t st)
{
    if (D == 256 || prefer_streaming_forward(a, D)) {
        if (launch_fwd_wide(a, D, causal, st)) return -1;
        if (a.nsplit <= 1) return 0;
        return D == 256 ? launch_fwd_merge<256>(a, st)
             : D == 128 ? launch_fwd_merge<128>(a, st) : launch_fwd_merge<64>(a, st);
    }
    return D == 128 ? launch_fwd_d<128>(a, causal, st) : launch_fwd_d<64>(a, causal, st);
}

}  // namespace attn
