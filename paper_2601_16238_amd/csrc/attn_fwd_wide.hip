// Fused attention forward, the form in which BOTH the K and the V tile reach LDS by direct
// global -> LDS transfers (V row-major, transposed by the LDS reads), four waves = 128 query rows
// per work-group, K and V double-buffered.  The same computation and the same orientation of the
// score tiles as the kernel in attn_fwd.hip (S^T = K Q^T with one query per lane, O^T += V^T P^T,
// lazily moved reference max, two row sums).  It serves
//  - head dimensions above 128 (D = 256): the Q fragments (64 registers) and the 256 x 32 fp32
//    accumulator of O^T (128 registers) leave room for one wave per SIMD only, and one K tile plus
//    one V tile of 64 keys take 70 KB of LDS;
//  - D = 64 and 128 on problems with few query rows against many keys (decoding, short chunks),
//    which only stream K and V: the transfers move a tile with a quarter of the vector-memory
//    instructions of the register-staged V path and none of its transposing arithmetic.
//    Decoding proper (at most 32 rows per head, so that only the first wave holds rows; the rows
//    may be the query heads of one K/V head, times a few new positions each, packed into one head
//    by the caller of the launcher) runs in the NT form of the kernel: K and V, which the launch
//    reads exactly once, come by non-temporal transfers, and those are requested by the three waves
//    without rows, so that the computing wave never delays a tile.
//
// One barrier per tile of 64 keys.  A tile is processed in four steps whose independent halves
// sit in one basic block each, so that the matrix pipe and the vector ALU overlap inside a wave:
//   A  S^T(0) = K Q^T                          (D/16 MFMAs)
//   B  S^T(1) = K Q^T   with   P(0) = exp2(c S(0) - m)
//   C  O^T += V^T P(0)^T   with   P(1) = exp2(c S(1) - m)
//   D  O^T += V^T P(1)^T
// Nothing is carried from one tile to the next except the accumulators, which is what lets
// two K buffers do.
#include "attn_device.hpp"
#include "attn_launch.hpp"

namespace attn {

template <int D>
struct WideCfg {
    static constexpr int kD = D;
    static constexpr int kNW = 4;
    static constexpr int kThreads = kNW * 64;
    static constexpr int kBR = kNW * 32;
    static constexpr int kBC = 64;
    // K tile: wave-wide transfers of 16 B per lane fill 1 KB pieces of kPR rows, chunk-major
    // inside a piece (chunk c of row r at 16 * (kPR c + r % kPR)), pieces 16 kPR bytes further
    // apart than their size: the 16 rows a quarter wave reads at a fixed chunk fall into 16
    // different 16-byte bank groups.
    static constexpr int kPR = 1024 / (D * 2);
    static constexpr int kKPieceBytes = 1024 + kPR * 16;
    static constexpr int kKPieces = kBC / kPR;
    static constexpr int kKTileBytes = kKPieces * kKPieceBytes;
    static constexpr int kKHalfBytes = kKTileBytes / 2;     // 32 rows further
    static constexpr int kKStepBytes = 2 * kPR * 16;        // next contraction step
    static constexpr int kKDmaPerWave = kKPieces / kNW;
    // V tile: the same transfers and chunk-major pieces.  The tile is only read with the LDS
    // transpose read (the A operand of O^T += V^T P^T is V^T), whose 32 lanes per half wave fetch
    // 4 rows x 64 bytes.  With four or eight rows per piece those lie in one piece and the K
    // tile's piece distance serves; with two rows per piece (D = 256) they are 128 contiguous
    // bytes in each of two neighbouring pieces, which a distance of 1024 + 128 bytes puts into
    // disjoint banks.
    static constexpr int kVPieceBytes = D > 128 ? 1024 + 128 : kKPieceBytes;
    static constexpr int kVTileBytes = kKPieces * kVPieceBytes;
    static constexpr int kVRows16 = (16 / kPR) * kVPieceBytes;   // 16 rows further
    static constexpr int kOffV = 2 * kKTileBytes;
    static constexpr int kLdsBytes = 2 * (kKTileBytes + kVTileBytes);
    static_assert(kKPieces % kNW == 0 && 2 * kKDmaPerWave == D / 16, "staging divides evenly");
    static_assert(kLdsBytes <= 160 * 1024, "LDS budget of a gfx950 CU exceeded");
};

constexpr float kWideOverflow = 1024.0f;   // a partial row sum above this moves the reference max
constexpr float kWideMinusHuge = -1.0e30f;

// NT: K and V are read once by the whole launch (decoding: one query tile per K/V head) and
// are more than the last-level cache holds: their transfers carry the non-temporal hint.
template <int D, bool CAUSAL, bool SPLIT, bool NT = false>
__global__ void __launch_bounds__(WideCfg<D>::kThreads)
    __attribute__((amdgpu_waves_per_eu(D > 128 ? 1 : 2, D > 128 ? 1 : 2)))
attn_fwd_wide_kernel(const FwdArgs a)
{
    using C = WideCfg<D>;
    constexpr int KS = D / 16, DB = D / 32, PR = C::kPR;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, l = tid & 63, r = l & 31, h = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int S = a.S, Dr = a.Dr;

    int bh, rank;
    xcd_tile_order<CAUSAL>(blockIdx.x, a.nqt, a.BH, bh, rank);
    const int qt = CAUSAL ? a.nqt - 1 - rank : rank;  // heaviest tiles first
    const int64_t base = (int64_t)(bh / a.H) * a.stride_b + (int64_t)(bh % a.H) * a.stride_h;
    const int64_t base_kv = (int64_t)(bh / a.H) * a.kv_stride_b +
                            (int64_t)((bh % a.H) / a.group) * a.kv_stride_h;

    // Keys seen by this work-group: all Sk of them, or one split's range (then K and V are
    // simply re-based to the range and the causal offset moves with them).  Query row i sees
    // key j iff j <= i + coff.
    int Sk = a.Sk, coff = a.Sk - (a.pack_sq ? a.pack_sq : S);  // (packed rows: Sq positions per head)
    int64_t kv_first = 0;
    if (SPLIT) {
        const int k_begin = blockIdx.y * a.kps;  // < Sk by the launcher's plan
        kv_first = (int64_t)k_begin * a.kv_stride_s;
        Sk = min(Sk - k_begin, a.kps);
        coff -= k_begin;
    }

    const int q0 = qt * C::kBR + w * 32;
    const int q = q0 + r;
    const int qc = q < S ? q : S - 1;  // clamped for loads; rows >= S are never stored
    // the wave's first row in key coordinates (packed rows: every wave holds a row at position 0)
    const int q0e = (a.pack_sq ? 0 : q0) + coff;
    // position of the lane's row among the new rows of its sequence (packed heads: row r is
    // position r % Sq, so the wave's rows see at least the keys that q0e says and at most 31 more)
    const int qpos = a.pack_sq ? qc % a.pack_sq : qc;

    // Q fragments, B operand of K Q^T: lane holds Q[q][16 ks + 8 h .. +7].  At D = 256 they come
    // through LDS (further down, where the transfers are set up): sixteen loads per wave in
    // which every lane fetches 16 bytes of its own row touch 32 rows per instruction and keep
    // the work-group's last wave from even issuing its K and V transfers for thousands of cycles.
    constexpr bool kStageQ = D > 128;
    elem8 qf[KS];
    if constexpr (!kStageQ) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qf[ks] = as_elem8(ld_row16(a.Q + base + a.row_offset(qc), ks * 16 + 8 * h, Dr));
    }

    // Rotary embedding of the query rows, fused into their load (D <= 128, head dimension == D):
    // column d pairs with d + D/2, i.e. fragment ks with ks + KS/2, element by element, in this
    // lane; the same two fused multiply-adds per pair as the rotary kernel and the forward of
    // attn_fwd.hip, so that all three give the same bits.
    if constexpr (D <= 128) {
        if (a.rope_cos) {
            // (packed rows: row r sits at position r % Sq of the new rows)
            const int rpos = a.pack_sq ? qc % a.pack_sq : qc * a.rope_row_step;
            const int64_t pos = (int64_t)(rpos + a.rope_pos0) * (D / 2);
            elem *qr = a.Qrot ? a.Qrot + base + a.row_offset(qc) : nullptr;
#pragma unroll
            for (int ks = 0; ks < KS / 2; ++ks) {
                float lo[8], hi[8];
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const f32x4 c4 = *(const f32x4 *)(a.rope_cos + pos + 16 * ks + 8 * h + 4 * j);
                    const f32x4 s4 = *(const f32x4 *)(a.rope_sin + pos + 16 * ks + 8 * h + 4 * j);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int t = 4 * j + e;
                        const float x1 = (float)qf[ks][t], x2 = (float)qf[ks + KS / 2][t];
                        lo[t] = __builtin_fmaf(x1, c4[e], -(x2 * s4[e]));
                        hi[t] = __builtin_fmaf(x2, c4[e], x1 * s4[e]);
                    }
                }
                qf[ks] = pack8(lo[0], lo[1], lo[2], lo[3], lo[4], lo[5], lo[6], lo[7]);
                qf[ks + KS / 2] = pack8(hi[0], hi[1], hi[2], hi[3], hi[4], hi[5], hi[6], hi[7]);
                if (qr && q < S && (!SPLIT || blockIdx.y == 0)) {
                    *(elem8 *)(qr + 16 * ks + 8 * h) = qf[ks];
                    *(elem8 *)(qr + 16 * (ks + KS / 2) + 8 * h) = qf[ks + KS / 2];
                }
            }
        }
    }

    const int q_end = min(S, (qt + 1) * C::kBR);
    const int k_end = CAUSAL ? min(Sk, q_end + coff) : Sk;  // <= 0: nothing visible (splits only)
    const int n_kt = k_end > 0 ? (k_end + C::kBC - 1) / C::kBC : 0;

    // ---- staging.  Rows past Sk-1, tiles past the last one and columns Dr..D-1 lie outside
    // the head's buffer resource and read as zero.
    const uint32_t head_bytes = (uint32_t)(((int64_t)(Sk - 1) * a.kv_stride_s + Dr) * 2);
    const desc_t Kd = make_desc(a.K + base_kv + kv_first, head_bytes),
                 Vd = make_desc(a.V + base_kv + kv_first, head_bytes);
    const uint32_t lds0 = lds_address(smem);
    const uint32_t row_bytes = (uint32_t)a.kv_stride_s * 2u;
    const uint32_t tile_bytes = C::kBC * row_bytes;
    // lane l of a transfer fetches chunk l / kPR of the piece's row l % kPR
    const uint32_t k_voff = (l / PR) * 8 < Dr ? (l % PR) * row_bytes + ((l / PR) << 4) : head_bytes;
    // (The transfers are issued from assembly, out of the compiler's sight: it would otherwise
    // make the wave wait for all of them before its next transpose read of LDS.  stage() orders
    // them against the reads.)
    // piece n of this wave's share of tile kt; tensor 0: K, 1: V
    auto dma_piece = [&](int tensor, int kt, int buf, int n) __attribute__((always_inline)) {
        const int ii = w + n * C::kNW;  // which piece of the tile: wave-uniform
        const uint32_t lds = tensor ? lds0 + C::kOffV + buf * C::kVTileBytes + ii * C::kVPieceBytes
                                    : lds0 + buf * C::kKTileBytes + ii * C::kKPieceBytes;
        if constexpr (NT) dma16_between_nt(tensor ? Vd : Kd, lds, k_voff, kt * tile_bytes + ii * PR * row_bytes);
        else dma16_between(tensor ? Vd : Kd, lds, k_voff, kt * tile_bytes + ii * PR * row_bytes);
    };
    auto dma_k = [&](int kt, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < C::kKDmaPerWave; ++n) dma_piece(0, kt, buf, n);
    };
    auto dma_v = [&](int kt, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < C::kKDmaPerWave; ++n) dma_piece(1, kt, buf, n);
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
    // transpose reads of the V tile: the 16-lane group reads rows 4h + e (e = 0..3; +8 for the
    // second read), 64 bytes of d block 0 of each row -- the keys of contraction half h in the
    // order the accumulator of S^T holds them
    auto v_at = [](int row, int chunk) {
        return (row / PR) * C::kVPieceBytes + (chunk * PR + row % PR) * 16;
    };
    int v_lane[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
        v_lane[j] = C::kOffV + v_at(8 * j + 4 * h + ((l & 15) >> 2), 2 * ((l >> 4) & 1) + ((l >> 1) & 1)) + (l & 1) * 8;

    // S^T of sub-tile u of the tile in buffer buf
    // Per-lane LDS addresses of the current tile's fragments, set once per tile and made opaque
    // to the compiler, so that sub-tile, contraction step and d block are folded into the 16-bit
    // immediate offsets of the LDS instructions instead of into further address arithmetic.
    int k_base = 0, v_base0 = 0, v_base1 = 0;
    auto set_bases = [&](int buf) __attribute__((always_inline)) {
        k_base = k_lane + buf * C::kKTileBytes;
        v_base0 = v_lane[0] + buf * C::kVTileBytes;
        v_base1 = v_lane[1] + buf * C::kVTileBytes;
        asm volatile("" : "+v"(k_base), "+v"(v_base0), "+v"(v_base1));
    };
    // (fetch: -1, or the tensor of tile kt + 1 whose transfers are issued between the MFMAs,
    // one per two of them -- the chain of dependent MFMAs leaves the issue slots for it)
    auto scores = [&](int u, f32x16 &s, int fetch = -1, int kt = 0) __attribute__((always_inline)) {
        const char *Kt = smem + u * C::kKHalfBytes + k_base;
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            s = mfma32(*(const elem8 *)(Kt + ks * C::kKStepBytes), qf[ks], s);
            if (!NT && fetch >= 0 && (ks & 1) && kt + 1 < n_kt) dma_piece(fetch, kt + 1, (kt & 1) ^ 1, ks >> 1);
        }
    };
    // ragged tail and causal mask of sub-tile (kt, u); wave-uniform test whether any is needed
    auto mask = [&](int kt, int u, f32x16 &s) __attribute__((always_inline)) {
        const int kb = kt * C::kBC + 32 * u;
        if ((kb + 32 > Sk) || (CAUSAL && kb + 31 > q0e)) {
            const int lim = (CAUSAL ? min(qpos + coff, Sk - 1) : Sk - 1) - kb - 4 * h;
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
    auto pv = [&](int u, elem8 p0, elem8 p1) __attribute__((always_inline)) {
        const char *Vt = smem + 2 * u * C::kVRows16;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const char *Vd = Vt + db * 4 * PR * 16;  // d block db: four chunks further
            const elem8 f0 = join8(lds_read_tr((const elem *)(Vd + v_base0)),
                                    lds_read_tr((const elem *)(Vd + v_base1)));
            const elem8 f1 = join8(lds_read_tr((const elem *)(Vd + C::kVRows16 + v_base0)),
                                    lds_read_tr((const elem *)(Vd + C::kVRows16 + v_base1)));
            o[db] = mfma32(f0, p0, o[db]);
            o[db] = mfma32(f1, p1, o[db]);
        }
    };
    // Start of iteration kt: K(kt) and V(kt) have been on their way since iteration kt-1.  After
    // the barrier the other buffers (tile kt-1, last read before the barrier) are free and take
    // tile kt+1.  Its transfers are issued between the MFMAs of the two score steps (see scores):
    // issued in one burst after the barrier, the waves all queue at the compute unit's
    // vector-memory path while the matrix pipes idle (measured: +35 % on the whole kernel).
    auto stage = [&](int kt) __attribute__((always_inline)) {
        (void)kt;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    };
    // (waves that only take part in the staging: part 0 K(kt+1), part 1 V(kt+1))
    auto fetch_next = [&](int kt, int part) __attribute__((always_inline)) {
        if (kt + 1 >= n_kt) return;
        if constexpr (NT) {
            // decoding: the wave with the query rows (wave 0) requests nothing in the loop; the
            // 2 kKPieces pieces of a tile are dealt to the three waves that only stage
            if (part != 0 || w == 0) return;
            constexpr int kN = (2 * C::kKPieces + 2) / 3;
#pragma unroll
            for (int n = 0; n < kN; ++n) {
                const int pc = (w - 1) + 3 * n;  // wave-uniform
                if (pc >= 2 * C::kKPieces) continue;
                const int tensor = pc / C::kKPieces, ii = pc % C::kKPieces, buf = (kt & 1) ^ 1;
                const uint32_t lds = tensor ? lds0 + C::kOffV + buf * C::kVTileBytes + ii * C::kVPieceBytes
                                            : lds0 + buf * C::kKTileBytes + ii * C::kKPieceBytes;
                dma16_between_nt(tensor ? Vd : Kd, lds, k_voff, (kt + 1) * tile_bytes + ii * PR * row_bytes);
            }
        } else {
            if (part == 0) dma_k(kt + 1, (kt & 1) ^ 1);
            if (part == 1) dma_v(kt + 1, (kt & 1) ^ 1);
        }
    };
    auto commit = [&](elem8 p0, elem8 p1, float psum) __attribute__((always_inline)) {
        lsum += psum;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            hsum = dot2_acc(p0[2 * i], p0[2 * i + 1], hsum);
            hsum = dot2_acc(p1[2 * i], p1[2 * i + 1], hsum);
        }
    };
    auto overflow = [&](float psum) { return __builtin_amdgcn_ballot_w64(psum > kWideOverflow) != 0; };

    // D = 256: the wave's 32 query rows as half of a K-layout tile, by the same direct transfers
    // (whole rows, two per instruction), into the second buffer pair, which takes tile 1 only
    // after the first barrier: waves 0 and 1 into the K buffer, 2 and 3 into the V buffer.  Rows
    // past S-1 and columns Dr..D-1 read as zero.
    uint32_t q_stage = 0;
    if constexpr (kStageQ) {
        const int pair = w >> 1, half = w & 1;
        q_stage = (pair == 0 ? C::kKTileBytes : C::kOffV + C::kVTileBytes) + half * C::kKHalfBytes;
        const int row0 = qt * C::kBR + pair * 64;
        const int rows = min(64, S - row0);
        const uint32_t q_bytes = rows > 0 ? (uint32_t)(((int64_t)(rows - 1) * a.stride_s + Dr) * 2) : 0u;
        const desc_t Qd = make_desc(a.Q + base + (int64_t)(rows > 0 ? row0 : 0) * a.stride_s, q_bytes);
        const uint32_t q_row_bytes = (uint32_t)a.stride_s * 2u;
        const uint32_t q_voff = (l / PR) * 8 < Dr ? (l % PR) * q_row_bytes + ((l / PR) << 4) : q_bytes;
#pragma unroll
        for (int n = 0; n < C::kKPieces / 2; ++n)
            dma16_between(Qd, lds0 + q_stage + n * C::kKPieceBytes, q_voff,
                          (half * (C::kKPieces / 2) + n) * PR * q_row_bytes);
    }
    if (n_kt > 0) {
        dma_k(0, 0);
        dma_v(0, 0);
    }
    if constexpr (kStageQ) {
        // the query rows have landed once at most the transfers of K(0) and V(0) are outstanding
        if (n_kt > 0) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * C::kKDmaPerWave) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        const char *Qs = smem + q_stage + ((r / PR) * C::kKPieceBytes + (h * PR + r % PR) * 16);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = *(const elem8 *)(Qs + ks * C::kKStepBytes);
        // ... and are in registers before anybody may overwrite the staging space
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    // Tiles of which this wave sees some key come first; for the rest of the work-group's tiles
    // (under a causal mask, the waves with the earlier rows) it only takes part in the staging.
    // A second sub-tile that lies wholly above the wave's diagonal is computed with every score
    // masked: one code path, and it only happens on the diagonal tile.
    // A wave whose rows all lie past the end of the head computes nothing either.
    const int n_seen = !CAUSAL ? n_kt : q0e + 31 < 0 ? 0 : min(n_kt, (q0e + 31) / C::kBC + 1);
    const int n_mine = __builtin_amdgcn_readfirstlane(q0 < S ? n_seen : 0);
    // The loop over the tiles is written twice.  The inner, fast form never touches the O^T
    // accumulators with the vector ALU: when a sub-tile's probabilities show that the reference
    // max must move, it leaves the loop before that sub-tile is added, and the slow form below
    // finishes the tile (rescaling what has been accumulated) and hands back.  With the rescaling
    // inside the one loop the register allocator moved all 128 accumulator registers between the
    // two halves of the register file in every iteration.
    int kt = 0;
    while (kt < n_mine) {
        int redo = -1;  // first sub-tile of tile kt that the slow form has to take over
        for (; kt < n_mine; ++kt) {
            stage(kt);
            set_bases(kt & 1);
            f32x16 sA, sB;
            elem8 pA0, pA1, pB0, pB1;
            float sumA, sumB;
            scores(0, sA, 0, kt);                       // A
            mask(kt, 0, sA);
            scores(1, sB, 1, kt);                       // B
            probs(sA, pA0, pA1, sumA);
            __builtin_amdgcn_sched_barrier(0);
            if (__builtin_expect(overflow(sumA), 0)) { redo = 0; break; }
            commit(pA0, pA1, sumA);
            mask(kt, 1, sB);
            pv(0, pA0, pA1);                            // C
            probs(sB, pB0, pB1, sumB);
            __builtin_amdgcn_sched_barrier(0);
            if (__builtin_expect(overflow(sumB), 0)) { redo = 1; break; }
            commit(pB0, pB1, sumB);
            pv(1, pB0, pB1);                            // D
            __builtin_amdgcn_sched_barrier(0);
        }
        if (redo >= 0) {
            set_bases(kt & 1);
            for (int u = redo; u < 2; ++u) {
                f32x16 sx;
                elem8 p0, p1;
                float psum;
                if (u == 0) scores(0, sx); else scores(1, sx);
                mask(kt, u, sx);
                probs(sx, p0, p1, psum);
                settle(sx, p0, p1, psum);
                if (u == 0) pv(0, p0, p1); else pv(1, p0, p1);
            }
            ++kt;
        }
    }
    for (kt = n_mine; kt < n_kt; ++kt) {
        stage(kt);
        fetch_next(kt, 0);
        fetch_next(kt, 1);
    }

    // no transfer may still be in flight when the work-group's LDS is released
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // Epilogue: O = O_acc / l, LSE = ln2 * (m + log2 l).
    const float lt = xhalf_sum(lsum);
    const float lr = xhalf_sum(hsum);
    if (SPLIT) {
        // normalised fp32 partial result of this key range; a row that saw no key of the
        // range contributes O = 0 with LSE = -inf
        const float inv = lr > 0.f ? 1.0f / lr : 0.f;
        if (q < S) {
            const int64_t row = ((int64_t)blockIdx.y * a.BH + bh) * S + q;
            float *Op = a.Opart + row * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f32x4 ov;
#pragma unroll
                    for (int e = 0; e < 4; ++e) ov[e] = o[db][4 * g + e] * inv;
                    *(f32x4 *)(Op + 32 * db + 8 * g + 4 * h) = ov;
                }
            if (h == 0) a.LSEpart[row] = lt > 0.f ? (m + fast_log2(lt)) * kLn2 : -INFINITY;
        }
        return;
    }
    const float inv = 1.0f / lr;
    {
        // The accumulator holds 4 consecutive columns of one row per register group: stored
        // directly, every instruction writes 8-byte pieces of 32 rows.  The rows go through LDS
        // instead and leave whole, 16 bytes per lane: the wave's 32 rows as half of a K-layout
        // tile in the buffer pair that the last tile did not use (other waves may still be
        // reading that one), waves 0 and 1 in its K buffer, 2 and 3 in its V buffer.
        constexpr int CPR = D / 8, RPI = 64 / CPR;  // chunks per row; rows per store instruction
        const int b = n_kt & 1;
        char *stg = smem + ((w >> 1) == 0 ? b * C::kKTileBytes : C::kOffV + b * C::kVTileBytes) +
                    (w & 1) * C::kKHalfBytes;
        auto at = [](int row, int chunk) {
            return (row / PR) * C::kKPieceBytes + (chunk * PR + row % PR) * 16;
        };
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                *(elem4 *)(stg + at(r, 4 * db + g) + 8 * h) =
                    pack4(o[db][4 * g] * inv, o[db][4 * g + 1] * inv, o[db][4 * g + 2] * inv, o[db][4 * g + 3] * inv);
        asm volatile("" ::: "memory");  // a wave's LDS accesses execute in order
        const int lr_ = l / CPR, lc = l % CPR;
#pragma unroll
        for (int j = 0; j < 32 / RPI; ++j) {
            const u32x4 v = *(const u32x4 *)(stg + at(RPI * j + lr_, lc));
            const int row = q0 + RPI * j + lr_;
            if (row < S && lc * 8 < Dr) *(u32x4 *)(a.O + base + a.row_offset(row) + lc * 8) = v;
        }
        if (q < S && h == 0) a.LSE[(int64_t)bh * S + q] = (m + fast_log2(lt)) * kLn2;
    }
}

template <int D, bool CAUSAL, bool SPLIT, bool NT = false>
static int launch_wide(FwdArgs a, hipStream_t st)
{
    using C = WideCfg<D>;
    a.nqt = (a.S + C::kBR - 1) / C::kBR;
    if (hipFuncSetAttribute((const void *)attn_fwd_wide_kernel<D, CAUSAL, SPLIT, NT>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, C::kLdsBytes) != hipSuccess)
        return -1;
    hipLaunchKernelGGL((attn_fwd_wide_kernel<D, CAUSAL, SPLIT, NT>), dim3(a.nqt * a.BH, SPLIT ? a.nsplit : 1),
                       dim3(C::kThreads), C::kLdsBytes, st, a);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <int D>
static int launch_wide_d(const FwdArgs &a, bool causal, hipStream_t st)
{
    // Decoding: every K/V head is read by one query tile only, once per call, and the next call
    // of a model reads another layer's cache: non-temporal transfers.  Measured with the timing loop
    // rotating over K/V sets that together exceed the last-level cache (256 MB), as a model's
    // layers do: 6-10 % faster at every size (B=8 Hkv=8 Sk=8192: 55 -> 50 us); with every byte from
    // HBM in one call (B=16 H=16 Sk=4096, 512 MiB) 98.6 -> 86.5 us.  A loop that re-reads ONE set
    // that fits the cache is 2-3 % slower for it.
    {
        // (not for an unsplit launch of few work-groups, i.e. a caller without a workspace: B=8
        // Hkv=8 Sk=8192 in 64 work-groups 156 -> 180 us with the hint)
        if (a.S <= 32 && a.group == 1 && (a.nsplit > 1 || a.BH >= 256)) {
            if (a.nsplit > 1)
                return causal ? launch_wide<D, true, true, true>(a, st) : launch_wide<D, false, true, true>(a, st);
            return causal ? launch_wide<D, true, false, true>(a, st) : launch_wide<D, false, false, true>(a, st);
        }
    }
    if (a.nsplit > 1)
        return causal ? launch_wide<D, true, true>(a, st) : launch_wide<D, false, true>(a, st);
    return causal ? launch_wide<D, true, false>(a, st) : launch_wide<D, false, false>(a, st);
}

// The main kernel only: with a split over the keys the caller launches the merge of the partial
// results afterwards.  The rotary embedding can be fused at D = 64 and 128.
int launch_fwd_wide(const FwdArgs &a, int D, bool causal, hipStream_t st)
{
    if (a.rope_cos && D > 128) return -1;
    return D == 256 ? launch_wide_d<256>(a, causal, st)
         : D == 128 ? launch_wide_d<128>(a, causal, st)
                    : launch_wide_d<64>(a, causal, st);
}

}  // namespace attn
