// Host-side kernel argument blocks and launch entry points (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace attn {

// The library is built twice from the same kernel sources: once with bf16 elements (the
// default) and once with IEEE fp16 (-DATTN_F16).  `elem` is the element type of the
// translation unit; the argument blocks are templates so that both builds can live in one
// library (kernels and launchers are distinguished by their argument type).
#ifdef ATTN_F16
typedef _Float16 elem;
#else
typedef __bf16 elem;
#endif

// One small block of arguments per kernel, passed by value: no per-tensor stride lists
// (the paper's debugging table records a crash from too many explicit stride arguments).
// Q, O, dO, dQ have H heads, S rows and the strides stride_*; K, V, dK, dV have H / group
// heads, Sk rows and the strides kv_stride_* (grouped-query attention; group == 1 is
// multi-head attention; Sk == S is the square problem).  With a causal mask query row i sees
// keys 0 .. i + Sk - S (aligned to the bottom-right corner).
template <typename E>
struct FwdArgsT {
    const E *Q, *K, *V;
    E *O;
    float *LSE;
    int64_t stride_b, stride_h, stride_s;
    int64_t kv_stride_b, kv_stride_h, kv_stride_s;
    int S, H, BH;
    int Sk;             // key/value rows
    int Dr;             // head dimension of the tensors (a multiple of 8); the kernels run at
                        // D = 64, 128 or 256 and treat columns Dr..D-1 as zeros
    int group;          // query heads per K/V head
    int pack_sq;        // 0, or: the S rows of a head are G query heads x pack_sq positions of one
                        // K/V head (row r is position r % pack_sq of S_q = pack_sq new rows); only
                        // the mask needs to know
    int64_t pack_stride_g;  // packed rows that are NOT at one distance (e.g. [B,S,H,D] tensors): row r lies
                        // (r / pack_sq) * pack_stride_g + (r % pack_sq) * stride_s past the head; 0: r * stride_s
    int nqt;            // query tiles per head (set by the launcher)
    float scale_log2e;  // scale * log2(e): the softmax runs on exp2
    // Split over the keys (small problems that would leave most of the chip idle): split z
    // (grid y) covers keys [z*kps, (z+1)*kps) and writes a normalised fp32 partial O and its
    // LSE; attn_fwd_merge_kernel combines them.  nsplit == 1: O and LSE are written directly.
    int nsplit, kps;    // kps is a multiple of the 64-key tile
    float *Opart;       // [nsplit][B*H][S][D]
    float *LSEpart;     // [nsplit][B*H][S]
    // Rotary embedding fused into the Q load (NULL tables: none).  Query row i is rotated by the
    // table row i * rope_row_step + rope_pos0 (step 1; step 0 when the rows of a head are the query
    // heads of one decoding position, which all sit at position rope_pos0) ("rotate-half" pairing of column d with d + D/2; tables fp32
    // [positions][D/2]); Qrot, if not NULL, receives the rotated rows (same strides as Q).
    const float *rope_cos, *rope_sin;
    E *Qrot;
    int rope_pos0, rope_row_step;
    // element offset of query row r from its head's first row (Q, O, Qrot share the strides)
    __host__ __device__ int64_t row_offset(int r) const
    {
        return pack_stride_g ? (int64_t)(r / pack_sq) * pack_stride_g + (int64_t)(r % pack_sq) * stride_s
                             : (int64_t)r * stride_s;
    }
};

template <typename E>
struct BwdArgsT {
    const E *Q, *K, *V, *O, *dO;
    const float *LSE;
    float *delta;       // workspace [B*H][2][S]: -delta, then LSE * log2(e)
    E *dQ, *dK, *dV;
    int64_t stride_b, stride_h, stride_s;
    int64_t kv_stride_b, kv_stride_h, kv_stride_s;
    int S, H, BH;
    int Sk;             // key/value rows
    int Dr;             // head dimension of the tensors; columns Dr..D-1 are zeros (see FwdArgsT)
    int group;          // query heads per K/V head
    int ntile;          // tiles per head of the launched kernel (set by the launcher)
    int stats_in_dq;    // the dQ kernel forms the row statistics itself and stores them to
                        // `delta` for the dK/dV kernel (set by the launcher)
    float scale, scale_log2e;
    // dQ kernel split over the keys (few query tiles against many keys would leave most of the
    // chip idle): split z (grid y) covers keys [z*dq_kps, (z+1)*dq_kps) and writes an unscaled
    // fp32 partial dQ; attn_bwd_dq_merge_kernel adds the splits, scales and rounds.
    // dq_nsplit == 1: dQ is written directly.
    int dq_nsplit, dq_kps;   // dq_kps is a multiple of the 64-key tile
    float *dQpart;           // [dq_nsplit][B*H][S][D]
    // Rotary embedding: Q holds ROTATED rows; dQ is rotated back (by the transpose of the
    // rotation) before it is stored, so that it is the gradient of the unrotated rows.  NULL
    // tables: none.
    const float *rope_cos, *rope_sin;
    int rope_pos0;
};

typedef FwdArgsT<elem> FwdArgs;
typedef BwdArgsT<elem> BwdArgs;

// Each returns 0 on success, -1 if the HIP runtime reported a launch error.  One overload per
// element type; each is defined by the build of the kernel sources for that type.
int launch_fwd(const FwdArgsT<__bf16> &a, int D, bool causal, hipStream_t st);
int launch_fwd(const FwdArgsT<_Float16> &a, int D, bool causal, hipStream_t st);
// The forward that streams both K and V by direct transfers (attn_fwd_wide.hip; D = 64, 128 or
// 256; called by launch_fwd, which also launches the merge of a split).
int launch_fwd_wide(const FwdArgsT<__bf16> &a, int D, bool causal, hipStream_t st);
int launch_fwd_wide(const FwdArgsT<_Float16> &a, int D, bool causal, hipStream_t st);
// Number of key splits the forward would use for this problem (1: none), and the keys per
// split; a pure host function of the shape.
int fwd_split_plan(int BH, int S, int Sk, int D, bool causal, int *kps);
// `stages`: bit 0 row statistics, bit 1 dK/dV, bit 2 dQ.  With bits 0 and 2 the dQ kernel
// forms the statistics (and runs first); bit 0 without bit 2 runs the separate kernel.
// Number of key splits the dQ kernel would use for this problem (1: none) and the keys per
// split; a pure host function of the shape.
int dq_split_plan(int BH, int S, int Sk, int D, bool causal, int *kps);
// The whole backward in one launch for heads of at most bwd_small_max_rows(D) query rows and keys
// (attn_bwd_small.hip; called by launch_bwd when all three stages are asked for).
int bwd_small_max_rows(int D);
int launch_bwd_small(const BwdArgsT<__bf16> &a, int D, bool causal, hipStream_t st);
int launch_bwd_small(const BwdArgsT<_Float16> &a, int D, bool causal, hipStream_t st);
int launch_bwd(const BwdArgsT<__bf16> &a, int D, bool causal, hipStream_t st, unsigned stages);
int launch_bwd(const BwdArgsT<_Float16> &a, int D, bool causal, hipStream_t st, unsigned stages);

}  // namespace attn
