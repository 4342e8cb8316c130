// Host-side kernel argument blocks and launch entry points (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace attn {

typedef __bf16 bf16;

// One small block of arguments per kernel, passed by value: no per-tensor stride lists
// (the paper's debugging table records a crash from too many explicit stride arguments).
// Q, O, dO, dQ have H heads and the strides stride_*; K, V, dK, dV have H / group heads and
// the strides kv_stride_* (grouped-query attention; group == 1 is multi-head attention).
struct FwdArgs {
    const bf16 *Q, *K, *V;
    bf16 *O;
    float *LSE;
    int64_t stride_b, stride_h, stride_s;
    int64_t kv_stride_b, kv_stride_h, kv_stride_s;
    int S, H, BH;
    int group;          // query heads per K/V head
    int nqt;            // query tiles per head (set by the launcher)
    float scale_log2e;  // scale * log2(e): the softmax runs on exp2
};

struct BwdArgs {
    const bf16 *Q, *K, *V, *O, *dO;
    const float *LSE;
    float *delta;       // workspace [B*H][2][S]: -delta, then LSE * log2(e)
    bf16 *dQ, *dK, *dV;
    int64_t stride_b, stride_h, stride_s;
    int64_t kv_stride_b, kv_stride_h, kv_stride_s;
    int S, H, BH;
    int group;          // query heads per K/V head
    int ntile;          // tiles per head of the launched kernel (set by the launcher)
    float scale, scale_log2e;
};

// Each returns 0 on success, -1 if the HIP runtime reported a launch error.
int launch_fwd(const FwdArgs &a, int D, bool causal, hipStream_t st);
// `stages`: bit 0 delta, bit 1 dK/dV, bit 2 dQ.
int launch_bwd(const BwdArgs &a, int D, bool causal, hipStream_t st, unsigned stages);

}  // namespace attn
