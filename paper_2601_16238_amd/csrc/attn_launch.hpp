// Host-side kernel argument blocks and launch entry points (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace attn {

typedef __bf16 bf16;

// One small block of arguments per kernel, passed by value: no per-tensor stride lists
// (the paper's debugging table records a crash from too many explicit stride arguments).
// Q, O, dO, dQ have H heads, S rows and the strides stride_*; K, V, dK, dV have H / group
// heads, Sk rows and the strides kv_stride_* (grouped-query attention; group == 1 is
// multi-head attention; Sk == S is the square problem).  With a causal mask query row i sees
// keys 0 .. i + Sk - S (aligned to the bottom-right corner).
struct FwdArgs {
    const bf16 *Q, *K, *V;
    bf16 *O;
    float *LSE;
    int64_t stride_b, stride_h, stride_s;
    int64_t kv_stride_b, kv_stride_h, kv_stride_s;
    int S, H, BH;
    int Sk;             // key/value rows
    int group;          // query heads per K/V head
    int nqt;            // query tiles per head (set by the launcher)
    float scale_log2e;  // scale * log2(e): the softmax runs on exp2
    // Split over the keys (small problems that would leave most of the chip idle): split z
    // (grid y) covers keys [z*kps, (z+1)*kps) and writes a normalised fp32 partial O and its
    // LSE; attn_fwd_merge_kernel combines them.  nsplit == 1: O and LSE are written directly.
    int nsplit, kps;    // kps is a multiple of the 64-key tile
    float *Opart;       // [nsplit][B*H][S][D]
    float *LSEpart;     // [nsplit][B*H][S]
};

struct BwdArgs {
    const bf16 *Q, *K, *V, *O, *dO;
    const float *LSE;
    float *delta;       // workspace [B*H][2][S]: -delta, then LSE * log2(e)
    bf16 *dQ, *dK, *dV;
    int64_t stride_b, stride_h, stride_s;
    int64_t kv_stride_b, kv_stride_h, kv_stride_s;
    int S, H, BH;
    int Sk;             // key/value rows
    int group;          // query heads per K/V head
    int ntile;          // tiles per head of the launched kernel (set by the launcher)
    float scale, scale_log2e;
};

// Each returns 0 on success, -1 if the HIP runtime reported a launch error.
int launch_fwd(const FwdArgs &a, int D, bool causal, hipStream_t st);
// Number of key splits the forward would use for this problem (1: none), and the keys per
// split; a pure host function of the shape.
int fwd_split_plan(int BH, int S, int Sk, int D, int *kps);
// `stages`: bit 0 delta, bit 1 dK/dV, bit 2 dQ.
int launch_bwd(const BwdArgs &a, int D, bool causal, hipStream_t st, unsigned stages);

}  // namespace attn
