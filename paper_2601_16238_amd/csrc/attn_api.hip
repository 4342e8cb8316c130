// C ABI of the attention library: host-side validation and dispatch only.
#include "../../include/attn.h"
#include "attn_launch.hpp"

#include <cmath>
#include <limits>
#include <mutex>

namespace {

constexpr size_t kWsAlign = 256;

int check_strides(int32_t S, int32_t D, int64_t sb, int64_t sh, int64_t ss)
{
    if (ss < D || sh < 1 || sb < 1) return ATTN_ERR_STRIDE;
    if (ss % 8 || sh % 8 || sb % 8) return ATTN_ERR_STRIDE;
    // One head's rows (plus the look-ahead tiles the kernels fetch past the end, which read
    // as zero) are addressed with 32-bit byte offsets.
    // (half the 32-bit range: an offset one resource length past a row must not wrap either)
    if (((int64_t)S + 512) * ss * 2 >= ((int64_t)1 << 31)) return ATTN_ERR_STRIDE;
    return ATTN_OK;
}

// Every entry point funnels into the rectangular, grouped-query form.
int check_params(const attn_rect_params_t *p)
{
    if (!p) return ATTN_ERR_NULL;
    if (p->B < 1 || p->Hq < 1 || p->Hkv < 1 || p->Sq < 1 || p->Sk < 1) return ATTN_ERR_SHAPE;
    if (p->Hq % p->Hkv != 0) return ATTN_ERR_SHAPE;
    if (p->D < 8 || p->D > 256 || p->D % 8 != 0) return ATTN_ERR_SHAPE;
    // the causal mask is aligned bottom-right: with fewer keys than rows some rows see none
    if (p->causal && p->Sk < p->Sq) return ATTN_ERR_SHAPE;
    // B*Hq*Sq and B*Hkv*Sk rows must be indexable with int32 (LSE / workspace offsets, grids).
    const int64_t lim = (int64_t)std::numeric_limits<int32_t>::max();
    if ((int64_t)p->B * p->Hq * p->Sq > lim || (int64_t)p->B * p->Hkv * p->Sk > lim)
        return ATTN_ERR_SHAPE;
    int rc = check_strides(p->Sq, p->D, p->q_stride_b, p->q_stride_h, p->q_stride_s);
    if (rc != ATTN_OK) return rc;
    rc = check_strides(p->Sk, p->D, p->kv_stride_b, p->kv_stride_h, p->kv_stride_s);
    if (rc != ATTN_OK) return rc;
    if (!std::isfinite(p->scale) || !(p->scale > 0.0f)) return ATTN_ERR_SCALE;
    return ATTN_OK;
}

attn_rect_params_t as_rect(const attn_gqa_params_t &p)
{
    attn_rect_params_t g;
    g.B = p.B; g.Hq = p.Hq; g.Hkv = p.Hkv; g.Sq = p.S; g.Sk = p.S; g.D = p.D;
    g.q_stride_b = p.q_stride_b; g.q_stride_h = p.q_stride_h; g.q_stride_s = p.q_stride_s;
    g.kv_stride_b = p.kv_stride_b; g.kv_stride_h = p.kv_stride_h; g.kv_stride_s = p.kv_stride_s;
    g.scale = p.scale; g.causal = p.causal;
    return g;
}

// Multi-head parameters as the grouped-query ones with one query head per K/V head.
attn_gqa_params_t as_gqa(const attn_params_t &p)
{
    attn_gqa_params_t g;
    g.B = p.B; g.Hq = p.H; g.Hkv = p.H; g.S = p.S; g.D = p.D;
    g.q_stride_b = g.kv_stride_b = p.stride_b;
    g.q_stride_h = g.kv_stride_h = p.stride_h;
    g.q_stride_s = g.kv_stride_s = p.stride_s;
    g.scale = p.scale; g.causal = p.causal;
    return g;
}

// The kernels exist for D = 64, 128 and 256; other head dimensions (multiples of 8) run in the
// next larger one with the missing columns read as zeros.
int kernel_d(int D) { return D <= 64 ? 64 : D <= 128 ? 128 : 256; }

size_t round_ws(size_t bytes) { return (bytes + kWsAlign - 1) / kWsAlign * kWsAlign; }

// The forward's view of a problem: (B*H) independent heads of S query rows each.
struct FwdView {
    int BH, H, S, group;
    bool packed;  // decoding: the rows of a head are the query heads of one K/V head
    int pack_sq;  // ... times this many new positions each (0: not packed, or one position)
    int64_t pack_stride_g;  // distance between the packed query heads when their rows are not at one distance
    int64_t stride_b, stride_h, stride_s;
    bool causal;
};

// Decoding (Sq == 1) with grouped-query heads: the G query heads that share a K/V head are
// G rows at a uniform distance (the head stride), so they are presented to the kernel as ONE
// head of G rows.  K and V are then streamed once per K/V head instead of once per query
// head.  A single row sees every key, so the mask drops out.  LSE [B,Hq,1] is the same
// memory as [B,Hkv,G].
// A few new positions per sequence (Sq = 2 .. 32, G x Sq <= 128 rows: one query tile, e.g. speculative decoding): with the rows of
// a query head contiguous to the next head's (q_stride_h == Sq * q_stride_s) the G x Sq rows of
// a K/V head are again rows at one uniform distance and are packed the same way; row r is
// position r % Sq, which the causal mask and the fused rotary embedding need to know.
FwdView fwd_view(const attn_rect_params_t &p, bool rope)
{
    (void)rope;  // the plan is the same with and without the fused rotary embedding
    FwdView v;
    v.pack_sq = 0; v.pack_stride_g = 0;
    const int G = p.Hq / p.Hkv;
    if (p.Sq == 1 && G > 1 &&
        check_strides(G, p.D, p.q_stride_b, G * p.q_stride_h, p.q_stride_h) == ATTN_OK) {
        v.BH = p.B * p.Hkv; v.H = p.Hkv; v.S = G; v.group = 1;
        v.stride_b = p.q_stride_b; v.stride_h = G * p.q_stride_h; v.stride_s = p.q_stride_h;
        v.causal = false; v.packed = true;
    } else if (p.Sq > 1 && p.Sq <= 32 && G > 1 &&
               G * p.Sq <= 128 &&  // one query tile of the streaming kernel
               // rows of a head contiguous to the next head's: one distance; otherwise (e.g. [B,S,H,D]
               // tensors) the kernels address a packed row by (head, position); not at D = 256, whose
               // query rows arrive by direct transfers of whole tiles
               (p.q_stride_h == (int64_t)p.Sq * p.q_stride_s || kernel_d(p.D) <= 128) &&
               check_strides(G * p.Sq, p.D, p.q_stride_b, G * p.q_stride_h, p.q_stride_s) == ATTN_OK) {
        v.BH = p.B * p.Hkv; v.H = p.Hkv; v.S = G * p.Sq; v.group = 1;
        v.stride_b = p.q_stride_b; v.stride_h = G * p.q_stride_h; v.stride_s = p.q_stride_s;
        v.causal = p.causal != 0; v.packed = true; v.pack_sq = p.Sq;
        if (p.q_stride_h != (int64_t)p.Sq * p.q_stride_s) v.pack_stride_g = p.q_stride_h;
    } else {
        v.BH = p.B * p.Hq; v.H = p.Hq; v.S = p.Sq; v.group = G;
        v.stride_b = p.q_stride_b; v.stride_h = p.q_stride_h; v.stride_s = p.q_stride_s;
        v.causal = p.causal != 0; v.packed = false;
    }
    return v;
}

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace

// E: element type of Q, K, V, O (__bf16 or _Float16)
// Workspace of the forward's split over the keys for this problem (0: it would not split).
static size_t fwd_workspace_bytes(const attn_rect_params_t *p, bool rope)
{
    if (check_params(p) != ATTN_OK) return 0;
    const FwdView v = fwd_view(*p, rope);
    const int nsplit = attn::fwd_split_plan(v.BH, v.S, p->Sk, kernel_d(p->D), v.causal, nullptr);
    if (nsplit <= 1) return 0;
    const size_t rows = (size_t)p->B * p->Hq * p->Sq;
    return round_ws((size_t)nsplit * rows * (kernel_d(p->D) + 1) * sizeof(float));
}

// The backward's row statistics: two fp32 values per query row.
static size_t bwd_stats_bytes(const attn_rect_params_t *p)
{
    return round_ws(2 * (size_t)p->B * p->Hq * p->Sq * sizeof(float));
}

// Rotary embedding fused into the call (both tables NULL: none).
struct Rope {
    const float *cos_table = nullptr, *sin_table = nullptr;
    void *Qrot = nullptr;  // forward only, optional
};

// The fused rotary embedding pairs column d with d + D/2 inside one lane's registers, which
// the kernels can do at their native head dimensions only; positions need Sk >= Sq.
static int check_rope(const attn_rect_params_t *p, const Rope &r)
{
    if (!r.cos_table || !r.sin_table) return ATTN_ERR_NULL;
    if ((p->D != 64 && p->D != 128) || p->Sk < p->Sq) return ATTN_ERR_SHAPE;
    if (!aligned(r.cos_table, 16) || !aligned(r.sin_table, 16) || !aligned(r.Qrot, 16))
        return ATTN_ERR_ALIGN;
    return ATTN_OK;
}

template <typename E>
static int fwd_impl(const void *Q, const void *K, const void *V, void *O, float *LSE,
                    void *workspace, size_t workspace_bytes,
                    const attn_rect_params_t *p, void *hip_stream, const Rope *rope = nullptr)
{
    if (!Q || !K || !V || !O || !LSE) return ATTN_ERR_NULL;
    int rc = check_params(p);
    if (rc != ATTN_OK) return rc;
    if (rope && (rc = check_rope(p, *rope)) != ATTN_OK) return rc;
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(O, 16) ||
        !aligned(LSE, 4))
        return ATTN_ERR_ALIGN;
    // No workspace at all: run unsplit.  A workspace that is there must be usable.
    const FwdView v = fwd_view(*p, rope != nullptr);
    int kps = 0;
    int nsplit = workspace ? attn::fwd_split_plan(v.BH, v.S, p->Sk, kernel_d(p->D), v.causal, &kps) : 1;
    if (workspace && (!aligned(workspace, kWsAlign) ||
                      workspace_bytes < fwd_workspace_bytes(p, rope != nullptr)))
        return ATTN_ERR_WORKSPACE;
    attn::FwdArgsT<E> a;
    a.nsplit = nsplit; a.kps = kps;
    a.Opart = static_cast<float *>(workspace);
    a.LSEpart = a.Opart ? a.Opart + (size_t)nsplit * p->B * p->Hq * p->Sq * kernel_d(p->D) : nullptr;
    a.Q = static_cast<const E *>(Q);
    a.K = static_cast<const E *>(K);
    a.V = static_cast<const E *>(V);
    a.O = static_cast<E *>(O);
    a.LSE = LSE;
    a.stride_b = v.stride_b; a.stride_h = v.stride_h; a.stride_s = v.stride_s;
    a.kv_stride_b = p->kv_stride_b; a.kv_stride_h = p->kv_stride_h; a.kv_stride_s = p->kv_stride_s;
    a.S = v.S; a.Sk = p->Sk; a.H = v.H; a.BH = v.BH; a.group = v.group; a.pack_sq = v.pack_sq; a.pack_stride_g = v.pack_stride_g;
    a.Dr = p->D;
    a.nqt = 0;
    a.scale_log2e = p->scale * 1.4426950408889634f;
    a.rope_cos = rope ? rope->cos_table : nullptr;
    a.rope_sin = rope ? rope->sin_table : nullptr;
    a.Qrot = rope ? static_cast<E *>(rope->Qrot) : nullptr;
    a.rope_pos0 = p->Sk - p->Sq;
    a.rope_row_step = v.packed ? 0 : 1;  // packed decoding heads all sit at the last position
    return attn::launch_fwd(a, kernel_d(p->D), v.causal, static_cast<hipStream_t>(hip_stream)) == 0
               ? ATTN_OK : ATTN_ERR_LAUNCH;
}

template <typename E>
static int bwd_impl(const void *Q, const void *K, const void *V, const void *O, const void *dO,
                    const float *LSE, void *dQ, void *dK, void *dV,
                    void *workspace, size_t workspace_bytes,
                    const attn_rect_params_t *p, void *hip_stream, uint32_t stages,
                    const Rope *rope = nullptr)
{
    if (!Q || !K || !V || !O || !dO || !LSE || !dQ || !dK || !dV) return ATTN_ERR_NULL;
    int rc = check_params(p);
    if (rc != ATTN_OK) return rc;
    if (rope && (rc = check_rope(p, *rope)) != ATTN_OK) return rc;
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(O, 16) ||
        !aligned(dO, 16) || !aligned(dQ, 16) || !aligned(dK, 16) || !aligned(dV, 16) ||
        !aligned(LSE, 4))
        return ATTN_ERR_ALIGN;
    // The row statistics always; the partial dQ of a key split only if they fit as well (a
    // smaller workspace runs the dQ kernel unsplit).  No split with rotary tables: the merge
    // does not rotate back.
    const size_t stats_bytes = bwd_stats_bytes(p);
    if (!workspace || !aligned(workspace, kWsAlign) || workspace_bytes < stats_bytes)
        return ATTN_ERR_WORKSPACE;
    if (stages == 0 || (stages & ~7u)) return ATTN_ERR_SHAPE;
    int dq_kps = 0;
    int dq_nsplit = attn::dq_split_plan(p->B * p->Hq, p->Sq, p->Sk, kernel_d(p->D), p->causal != 0, &dq_kps);
    if (rope || workspace_bytes < attn_bwd_rect_workspace_bytes(p)) dq_nsplit = 1;
    attn::BwdArgsT<E> a;
    a.Q = static_cast<const E *>(Q);
    a.K = static_cast<const E *>(K);
    a.V = static_cast<const E *>(V);
    a.O = static_cast<const E *>(O);
    a.dO = static_cast<const E *>(dO);
    a.LSE = LSE;
    a.delta = static_cast<float *>(workspace);
    a.dq_nsplit = dq_nsplit; a.dq_kps = dq_kps;
    a.dQpart = reinterpret_cast<float *>(static_cast<char *>(workspace) + stats_bytes);
    a.dQ = static_cast<E *>(dQ);
    a.dK = static_cast<E *>(dK);
    a.dV = static_cast<E *>(dV);
    a.stride_b = p->q_stride_b; a.stride_h = p->q_stride_h; a.stride_s = p->q_stride_s;
    a.kv_stride_b = p->kv_stride_b; a.kv_stride_h = p->kv_stride_h; a.kv_stride_s = p->kv_stride_s;
    a.S = p->Sq; a.Sk = p->Sk; a.H = p->Hq; a.BH = p->B * p->Hq; a.group = p->Hq / p->Hkv;
    a.Dr = p->D;
    a.ntile = 0;
    a.scale = p->scale;
    a.scale_log2e = p->scale * 1.4426950408889634f;
    a.rope_cos = rope ? rope->cos_table : nullptr;
    a.rope_sin = rope ? rope->sin_table : nullptr;
    a.rope_pos0 = p->Sk - p->Sq;
    return attn::launch_bwd(a, kernel_d(p->D), p->causal != 0, static_cast<hipStream_t>(hip_stream),
                            stages) == 0
               ? ATTN_OK : ATTN_ERR_LAUNCH;
}

extern "C" {

void attn_params_contiguous(attn_params_t *p, int32_t B, int32_t H, int32_t S, int32_t D,
                            float scale, int32_t causal)
{
    if (!p) return;
    p->B = B; p->H = H; p->S = S; p->D = D;
    p->stride_s = D;
    p->stride_h = (int64_t)S * D;
    p->stride_b = (int64_t)H * S * D;
    p->scale = scale;
    p->causal = causal;
}

void attn_gqa_params_contiguous(attn_gqa_params_t *p, int32_t B, int32_t Hq, int32_t Hkv,
                                int32_t S, int32_t D, float scale, int32_t causal)
{
    if (!p) return;
    p->B = B; p->Hq = Hq; p->Hkv = Hkv; p->S = S; p->D = D;
    p->q_stride_s = p->kv_stride_s = D;
    p->q_stride_h = p->kv_stride_h = (int64_t)S * D;
    p->q_stride_b = (int64_t)Hq * S * D;
    p->kv_stride_b = (int64_t)Hkv * S * D;
    p->scale = scale;
    p->causal = causal;
}

void attn_rect_params_contiguous(attn_rect_params_t *p, int32_t B, int32_t Hq, int32_t Hkv,
                                 int32_t Sq, int32_t Sk, int32_t D, float scale, int32_t causal)
{
    if (!p) return;
    p->B = B; p->Hq = Hq; p->Hkv = Hkv; p->Sq = Sq; p->Sk = Sk; p->D = D;
    p->q_stride_s = p->kv_stride_s = D;
    p->q_stride_h = (int64_t)Sq * D;
    p->kv_stride_h = (int64_t)Sk * D;
    p->q_stride_b = (int64_t)Hq * Sq * D;
    p->kv_stride_b = (int64_t)Hkv * Sk * D;
    p->scale = scale;
    p->causal = causal;
}

size_t attn_fwd_rect_workspace_bytes(const attn_rect_params_t *p) { return fwd_workspace_bytes(p, false); }

size_t attn_fwd_rope_workspace_bytes(const attn_rect_params_t *p) { return fwd_workspace_bytes(p, true); }

int attn_fwd_rope(const void *Q, const void *K_rot, const void *V, const float *cos_table,
                  const float *sin_table, void *O, float *LSE, void *Q_rot, void *workspace,
                  size_t workspace_bytes, const attn_rect_params_t *p, void *hip_stream)
{
    Rope r;
    r.cos_table = cos_table; r.sin_table = sin_table; r.Qrot = Q_rot;
    return fwd_impl<__bf16>(Q, K_rot, V, O, LSE, workspace, workspace_bytes, p, hip_stream, &r);
}

int attn_bwd_rope(const void *Q_rot, const void *K_rot, const void *V, const void *O,
                  const void *dO, const float *LSE, const float *cos_table, const float *sin_table,
                  void *dQ, void *dK_rot, void *dV, void *workspace, size_t workspace_bytes,
                  const attn_rect_params_t *p, void *hip_stream)
{
    Rope r;
    r.cos_table = cos_table; r.sin_table = sin_table;
    return bwd_impl<__bf16>(Q_rot, K_rot, V, O, dO, LSE, dQ, dK_rot, dV, workspace, workspace_bytes, p,
                            hip_stream,
                            ATTN_BWD_STAGE_DELTA | ATTN_BWD_STAGE_DKDV | ATTN_BWD_STAGE_DQ, &r);
}

int attn_fwd_rect(const void *Q, const void *K, const void *V, void *O, float *LSE,
                  void *workspace, size_t workspace_bytes,
                  const attn_rect_params_t *p, void *hip_stream)
{
    return fwd_impl<__bf16>(Q, K, V, O, LSE, workspace, workspace_bytes, p, hip_stream);
}

int attn_fwd_rect_f16(const void *Q, const void *K, const void *V, void *O, float *LSE,
                      void *workspace, size_t workspace_bytes,
                      const attn_rect_params_t *p, void *hip_stream)
{
    return fwd_impl<_Float16>(Q, K, V, O, LSE, workspace, workspace_bytes, p, hip_stream);
}

int attn_fwd_gqa(const void *Q, const void *K, const void *V, void *O, float *LSE,
                 const attn_gqa_params_t *p, void *hip_stream)
{
    if (!p) return ATTN_ERR_NULL;
    const attn_rect_params_t g = as_rect(*p);
    return attn_fwd_rect(Q, K, V, O, LSE, nullptr, 0, &g, hip_stream);
}

int attn_fwd(const void *Q, const void *K, const void *V, void *O, float *LSE,
             const attn_params_t *p, void *hip_stream)
{
    if (!p) return ATTN_ERR_NULL;
    const attn_gqa_params_t g = as_gqa(*p);
    return attn_fwd_gqa(Q, K, V, O, LSE, &g, hip_stream);
}

size_t attn_bwd_rect_workspace_bytes(const attn_rect_params_t *p)
{
    if (check_params(p) != ATTN_OK) return 0;
    const size_t rows = (size_t)p->B * p->Hq * p->Sq;
    const int nsplit = attn::dq_split_plan(p->B * p->Hq, p->Sq, p->Sk, kernel_d(p->D), p->causal != 0, nullptr);
    const size_t part = nsplit > 1 ? round_ws((size_t)nsplit * rows * kernel_d(p->D) * sizeof(float)) : 0;
    return bwd_stats_bytes(p) + part;
}

size_t attn_bwd_gqa_workspace_bytes(const attn_gqa_params_t *p)
{
    if (!p) return 0;
    const attn_rect_params_t g = as_rect(*p);
    return attn_bwd_rect_workspace_bytes(&g);
}

size_t attn_bwd_workspace_bytes(const attn_params_t *p)
{
    if (!p) return 0;
    const attn_gqa_params_t g = as_gqa(*p);
    return attn_bwd_gqa_workspace_bytes(&g);
}

int attn_bwd_rect(const void *Q, const void *K, const void *V, const void *O, const void *dO,
                  const float *LSE, void *dQ, void *dK, void *dV,
                  void *workspace, size_t workspace_bytes,
                  const attn_rect_params_t *p, void *hip_stream)
{
    return bwd_impl<__bf16>(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, p,
                            hip_stream,
                            ATTN_BWD_STAGE_DELTA | ATTN_BWD_STAGE_DKDV | ATTN_BWD_STAGE_DQ);
}

int attn_bwd_rect_f16(const void *Q, const void *K, const void *V, const void *O, const void *dO,
                      const float *LSE, void *dQ, void *dK, void *dV,
                      void *workspace, size_t workspace_bytes,
                      const attn_rect_params_t *p, void *hip_stream)
{
    return bwd_impl<_Float16>(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, p,
                              hip_stream,
                              ATTN_BWD_STAGE_DELTA | ATTN_BWD_STAGE_DKDV | ATTN_BWD_STAGE_DQ);
}

int attn_bwd_gqa(const void *Q, const void *K, const void *V, const void *O, const void *dO,
                 const float *LSE, void *dQ, void *dK, void *dV,
                 void *workspace, size_t workspace_bytes,
                 const attn_gqa_params_t *p, void *hip_stream)
{
    return attn_bwd_gqa_stages(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, p,
                               hip_stream,
                               ATTN_BWD_STAGE_DELTA | ATTN_BWD_STAGE_DKDV | ATTN_BWD_STAGE_DQ);
}

int attn_bwd_gqa_stages(const void *Q, const void *K, const void *V, const void *O,
                        const void *dO, const float *LSE, void *dQ, void *dK, void *dV,
                        void *workspace, size_t workspace_bytes,
                        const attn_gqa_params_t *p, void *hip_stream, uint32_t stages)
{
    if (!p) return ATTN_ERR_NULL;
    const attn_rect_params_t g = as_rect(*p);
    return bwd_impl<__bf16>(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, &g,
                            hip_stream, stages);
}

int attn_bwd(const void *Q, const void *K, const void *V, const void *O, const void *dO,
             const float *LSE, void *dQ, void *dK, void *dV,
             void *workspace, size_t workspace_bytes,
             const attn_params_t *p, void *hip_stream)
{
    return attn_bwd_stages(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, p,
                           hip_stream,
                           ATTN_BWD_STAGE_DELTA | ATTN_BWD_STAGE_DKDV | ATTN_BWD_STAGE_DQ);
}

int attn_bwd_stages(const void *Q, const void *K, const void *V, const void *O, const void *dO,
                    const float *LSE, void *dQ, void *dK, void *dV,
                    void *workspace, size_t workspace_bytes,
                    const attn_params_t *p, void *hip_stream, uint32_t stages)
{
    if (!p) return ATTN_ERR_NULL;
    const attn_gqa_params_t g = as_gqa(*p);
    return attn_bwd_gqa_stages(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, &g,
                               hip_stream, stages);
}

}  // extern "C"

// Scratch of attn_bwd_rect_noalloc: the backward's row statistics, in an array that lives in
// the library's device image instead of in memory the caller allocates.  Every GPU the library
// runs on holds its own copy at its own address, so the address is looked up once per device
// (with that device current) and kept; host code uses that pointer, never the array's name.
static __device__ __align__(256) unsigned char scratch[ATTN_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];  // guarded by g_scratch_mutex; nullptr = not looked up yet
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device, or nullptr if the runtime refuses.
void *scratch_of_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

extern "C" {

int attn_bwd_rect_noalloc(const void *Q, const void *K, const void *V, const void *O,
                          const void *dO, const float *LSE, void *dQ, void *dK, void *dV,
                          const attn_rect_params_t *p, void *hip_stream)
{
    // the same checks as attn_bwd_rect, before anything touches the device
    if (!Q || !K || !V || !O || !dO || !LSE || !dQ || !dK || !dV) return ATTN_ERR_NULL;
    const int rc = check_params(p);
    if (rc != ATTN_OK) return rc;
    const size_t need = bwd_stats_bytes(p);
    if (need > (size_t)ATTN_NOALLOC_SCRATCH_BYTES) return ATTN_ERR_WORKSPACE;
    void *ws = scratch_of_current_device();
    if (!ws) return ATTN_ERR_LAUNCH;
    // Every value of the scratch that a kernel reads is written earlier in the same call (the
    // dQ kernel stores the statistics of every query row, the dK/dV kernel reads only those),
    // so nothing has to be cleared although the array keeps the last call's contents.
    return bwd_impl<__bf16>(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ATTN_NOALLOC_SCRATCH_BYTES, p,
                            hip_stream,
                            ATTN_BWD_STAGE_DELTA | ATTN_BWD_STAGE_DKDV | ATTN_BWD_STAGE_DQ);
}

const char *attn_status_string(int status)
{
    switch (status) {
        case ATTN_OK: return "ok";
        case ATTN_ERR_NULL: return "a required pointer is NULL";
        case ATTN_ERR_SHAPE: return "unsupported shape (B,H,S >= 1, D a multiple of 8 up to 256, Hkv divides Hq, B*H*S < 2^31, causal needs Sk >= Sq)";
        case ATTN_ERR_STRIDE: return "bad stride (D contiguous, strides multiples of 8 elements, stride_s >= D)";
        case ATTN_ERR_ALIGN: return "tensor pointer not 16-byte aligned";
        case ATTN_ERR_WORKSPACE: return "workspace missing, misaligned (256 B) or too small";
        case ATTN_ERR_SCALE: return "scale must be finite and > 0";
        case ATTN_ERR_LAUNCH: return "HIP kernel launch failed";
        default: return "unknown status";
    }
}

int attn_version(void) { return 1005; }

}  // extern "C"
