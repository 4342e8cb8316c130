/*
 * attn.h -- C ABI of the MI355X (gfx950) fused scaled-dot-product attention library.
 *
 * The operator is the fused attention kernel that the paper's kernel suite benchmarks
 * against SDPA/FlashAttention (kernel-suite section; attention rows of the microbenchmark
 * table, shape written there as (B,Hq,Hkv,S,D), bf16, causal) in the natural-log,
 * max-stabilised "flash-attention-style" form its debugging table prescribes:
 *
 *     s_ij = scale * sum_d Q_id K_jd          j <= i only if causal (diagonal included)
 *     LSE_i = ln sum_j exp(s_ij)              natural log
 *     O_id  = sum_j exp(s_ij - LSE_i) V_jd
 *
 * and its gradient for an upstream gradient dO on O (LSE carries no gradient).
 *
 * Conventions common to every call
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library never
 *     allocates, frees, synchronises or changes the current device; it only enqueues
 *     kernels on `hip_stream` (a hipStream_t passed as void*, NULL = default stream) and
 *     returns.  The caller keeps the buffers alive until that work has completed.
 *   - Q, K, V, O, dO, dQ, dK, dV hold bf16 elements and all use the same element strides
 *     (stride_b, stride_h, stride_s) with the D axis contiguous.  A contiguous [B,H,S,D]
 *     tensor has stride_s = D, stride_h = S*D, stride_b = H*S*D; [B,S,H,D] storage is
 *     expressible too.  Strides must be multiples of 8 elements and base pointers 16-byte
 *     aligned (the kernels use 16-byte loads).
 *   - LSE (and the backward's internal delta) are fp32, contiguous [B,H,S].
 *   - Outputs are fully overwritten; nothing is accumulated into caller buffers and no
 *     buffer's previous contents are ever relied on (the paper's debugging table lists
 *     uninitialised reused gradient buffers as a bug class).
 *   - Outputs must not alias inputs.
 *   - Every entry point validates its arguments on the host before launching anything and
 *     returns ATTN_OK (0) or a negative attn_status.  No exceptions, no abort, no logging.
 *     Validation needs no GPU.  The calls are re-entrant; there is no global mutable state.
 */
#ifndef MI355_ATTN_H
#define MI355_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ATTN_OK = 0,
    ATTN_ERR_NULL = -1,      /* a required pointer is NULL                                  */
    ATTN_ERR_SHAPE = -2,     /* B,H,S < 1, D not a multiple of 8 in 8..256, Hkv not dividing Hq, or a size
                                overflows int32                                             */
    ATTN_ERR_STRIDE = -3,    /* a stride is < its minimum, not a multiple of 8 elements, or
                                (S + 512) * stride_s * 2 bytes does not fit in 32 bits        */
    ATTN_ERR_ALIGN = -4,     /* a tensor pointer is not 16-byte aligned (LSE: 4-byte)        */
    ATTN_ERR_WORKSPACE = -5, /* workspace NULL/misaligned or smaller than required           */
    ATTN_ERR_SCALE = -6,     /* scale is not a finite number > 0                             */
    ATTN_ERR_LAUNCH = -7     /* the HIP runtime refused a launch (hipGetLastError != 0)      */
} attn_status;

/* Problem description shared by forward and backward (host memory, read during the call). */
typedef struct {
    int32_t B, H, S, D;   /* batch, heads, sequence length (S_q == S_k), head dim: a multiple of
                             8, at most 256.  The kernels are built for 64, 128 and 256; any other
                             value runs in the next larger one, the missing columns read as zeros
                             (never loaded from or stored to memory)                          */
    int64_t stride_b;     /* element strides of all bf16 tensors; the D axis has stride 1     */
    int64_t stride_h;
    int64_t stride_s;
    float scale;          /* multiplies Q.K^T before the softmax; finite and > 0              */
    int32_t causal;       /* 0: every key visible; otherwise key j visible to query i iff j<=i */
} attn_params_t;

/* Fill strides for a contiguous [B,H,S,D] tensor.  Pure host function. */
void attn_params_contiguous(attn_params_t *p, int32_t B, int32_t H, int32_t S, int32_t D,
                            float scale, int32_t causal);

/*
 * Forward (paper: fused attention forward row of the microbenchmark table).
 *   Q,K,V : in,  bf16 device [B,H,S,D] by strides
 *   O     : out, bf16 device, same strides
 *   LSE   : out, fp32 device, contiguous [B,H,S], natural log of sum_j exp(s_ij)
 * Enqueues one kernel on hip_stream.
 */
int attn_fwd(const void *Q, const void *K, const void *V, void *O, float *LSE,
             const attn_params_t *p, void *hip_stream);

/*
 * Bytes of device workspace attn_bwd asks for: two fp32 values per query row ([B*H][2][S]:
 * -rowsum(dO*O), and LSE rescaled to base 2), rounded up to 256 bytes, plus -- for problems
 * with so few query tiles that the dQ kernel is split over the keys, see
 * attn_bwd_rect_workspace_bytes -- the fp32 partial results of that split.
 * Pure host function; returns 0 for an invalid problem.
 */
size_t attn_bwd_workspace_bytes(const attn_params_t *p);

/*
 * Backward (paper: fused attention backward row of the microbenchmark table).  P is
 * recomputed from Q, K and the forward's LSE; dK/dV are accumulated per key block in
 * registers, dQ per query block, so no atomics are used and results are deterministic.
 *   Q,K,V,O,dO : in,  bf16 device (O and LSE as produced by attn_fwd)
 *   LSE        : in,  fp32 device [B,H,S]
 *   dQ,dK,dV   : out, bf16 device, same strides as the inputs
 *   workspace  : device scratch of at least attn_bwd_workspace_bytes(p) bytes, 256-byte
 *                aligned; contents undefined on entry and on exit (the library initialises
 *                everything it reads)
 * Enqueues two kernels on hip_stream: dQ (which also forms the row statistics delta and
 * rescaled LSE and stores them in the workspace), then dK/dV (which reads them).
 */
int attn_bwd(const void *Q, const void *K, const void *V, const void *O, const void *dO,
             const float *LSE, void *dQ, void *dK, void *dV,
             void *workspace, size_t workspace_bytes,
             const attn_params_t *p, void *hip_stream);

/*
 * Profiling aid: attn_bwd restricted to a subset of its stages, so that each can be timed
 * on its own with events on the caller's stream.  `stages` is a bit mask of
 * ATTN_BWD_STAGE_*; attn_bwd is attn_bwd_stages with all three bits.  With DELTA and DQ
 * together the dQ kernel forms the row statistics itself, as in attn_bwd; DELTA without DQ
 * runs a separate kernel for them.  DKDV, and DQ without DELTA, read the statistics from the
 * workspace, so it must hold those of an earlier call on the same problem.  Validation and
 * errors as attn_bwd; stages == 0 or unknown bits give ATTN_ERR_SHAPE.
 */
#define ATTN_BWD_STAGE_DELTA 1u
#define ATTN_BWD_STAGE_DKDV 2u
#define ATTN_BWD_STAGE_DQ 4u
int attn_bwd_stages(const void *Q, const void *K, const void *V, const void *O, const void *dO,
                    const float *LSE, void *dQ, void *dK, void *dV,
                    void *workspace, size_t workspace_bytes,
                    const attn_params_t *p, void *hip_stream, uint32_t stages);

/*
 * Grouped-query variant (paper: the microbenchmark table writes the attention shape as
 * (B,Hq,Hkv,S,D) and the kernel-suite discussion is about grouped-query prefill).  Q, O, dO,
 * dQ have Hq heads and share the q_* strides; K, V, dK, dV have Hkv heads and share the kv_*
 * strides; Hq must be a multiple of Hkv and query head h reads K/V head h / (Hq/Hkv).  dK and
 * dV of a K/V head are summed over the Hq/Hkv query heads that read it, inside the kernel
 * (no atomics, deterministic).  LSE and the workspace are per QUERY head: LSE is [B,Hq,S].
 * Hkv == Hq is ordinary multi-head attention: attn_fwd / attn_bwd are exactly these calls
 * with both stride sets equal.  Everything else (pointers, alignment, ownership, errors,
 * stream semantics) is as for attn_fwd / attn_bwd; a head count that does not divide gives
 * ATTN_ERR_SHAPE, the stride rules apply to both stride sets.
 */
typedef struct {
    int32_t B, Hq, Hkv, S, D;
    int64_t q_stride_b, q_stride_h, q_stride_s;     /* Q, O, dO, dQ: element strides, D contiguous */
    int64_t kv_stride_b, kv_stride_h, kv_stride_s;  /* K, V, dK, dV                               */
    float scale;
    int32_t causal;
} attn_gqa_params_t;

/* Fill strides for contiguous [B,Hq,S,D] and [B,Hkv,S,D] tensors.  Pure host function. */
void attn_gqa_params_contiguous(attn_gqa_params_t *p, int32_t B, int32_t Hq, int32_t Hkv,
                                int32_t S, int32_t D, float scale, int32_t causal);

int attn_fwd_gqa(const void *Q, const void *K, const void *V, void *O, float *LSE,
                 const attn_gqa_params_t *p, void *hip_stream);

/* As attn_bwd_rect_workspace_bytes with Sq == Sk == S; 0 if invalid. */
size_t attn_bwd_gqa_workspace_bytes(const attn_gqa_params_t *p);

int attn_bwd_gqa(const void *Q, const void *K, const void *V, const void *O, const void *dO,
                 const float *LSE, void *dQ, void *dK, void *dV,
                 void *workspace, size_t workspace_bytes,
                 const attn_gqa_params_t *p, void *hip_stream);

/* Profiling aid, as attn_bwd_stages. */
int attn_bwd_gqa_stages(const void *Q, const void *K, const void *V, const void *O,
                        const void *dO, const float *LSE, void *dQ, void *dK, void *dV,
                        void *workspace, size_t workspace_bytes,
                        const attn_gqa_params_t *p, void *hip_stream, uint32_t stages);

/*
 * Rectangular variant: Sq query rows against Sk key/value rows (decoding or chunked prefill
 * against a longer key/value cache, cross attention; paper: the kernel-suite discussion of
 * small-batch grouped-query prefill, the case its table reports as slower than the library
 * baseline).  Q, O, dO, dQ are [B,Hq,Sq,D] by the q_* strides, K, V, dK, dV are [B,Hkv,Sk,D]
 * by the kv_* strides, LSE is [B,Hq,Sq].  With causal != 0 the mask is aligned to the
 * bottom-right corner: query row i sees keys 0 .. i + Sk - Sq, i.e. the rows are the LAST Sq
 * positions of a causal sequence of length Sk; causal with Sk < Sq is ATTN_ERR_SHAPE.
 * Sq == Sk is the grouped-query call above.
 *
 * Forward, split over the keys: when B*Hq*ceil(Sq/256) work-groups would leave most of the
 * chip idle (decoding: Sq = 1), the key range is cut into splits that run as separate
 * work-groups and write fp32 partial results to `workspace`; a second small kernel merges
 * them (log-sum-exp weights).  attn_fwd_rect_workspace_bytes returns what that needs for the
 * problem, 0 when it would not split.  workspace == NULL (with any size) is allowed and
 * means: do not split.  A non-NULL workspace must be 256-byte aligned and at least that
 * large, else ATTN_ERR_WORKSPACE; its contents are undefined on entry and exit.  The split
 * plan depends only on the shape and the strides, so results are deterministic.
 *
 * Backward: as attn_bwd_gqa.  Keys that no row sees get zero gradients.  Workspace: the row
 * statistics (two fp32 per query row, rounded up to 256 bytes) and, when B*Hq*ceil(Sq/256)
 * work-groups of the dQ kernel would leave most of the chip idle (Sq >= 256, at least 1024
 * keys), the fp32 partial dQ of a split of that kernel over the keys ([splits][B*Hq*Sq][64 or
 * 128]); a third small kernel adds them.  attn_bwd_rect_workspace_bytes(p) is the sum.  A
 * workspace that holds the statistics but not the partial results is accepted too: the dQ
 * kernel then runs unsplit.  Either way the plan depends only on the shape and the workspace
 * size, so results are deterministic.
 */
typedef struct {
    int32_t B, Hq, Hkv, Sq, Sk, D;
    int64_t q_stride_b, q_stride_h, q_stride_s;     /* Q, O, dO, dQ: element strides, D contiguous */
    int64_t kv_stride_b, kv_stride_h, kv_stride_s;  /* K, V, dK, dV                               */
    float scale;
    int32_t causal;
} attn_rect_params_t;

/* Fill strides for contiguous [B,Hq,Sq,D] and [B,Hkv,Sk,D] tensors.  Pure host function. */
void attn_rect_params_contiguous(attn_rect_params_t *p, int32_t B, int32_t Hq, int32_t Hkv,
                                 int32_t Sq, int32_t Sk, int32_t D, float scale, int32_t causal);

size_t attn_fwd_rect_workspace_bytes(const attn_rect_params_t *p);

int attn_fwd_rect(const void *Q, const void *K, const void *V, void *O, float *LSE,
                  void *workspace, size_t workspace_bytes,
                  const attn_rect_params_t *p, void *hip_stream);

size_t attn_bwd_rect_workspace_bytes(const attn_rect_params_t *p);

int attn_bwd_rect(const void *Q, const void *K, const void *V, const void *O, const void *dO,
                  const float *LSE, void *dQ, void *dK, void *dV,
                  void *workspace, size_t workspace_bytes,
                  const attn_rect_params_t *p, void *hip_stream);

/*
 * Rotary position embedding fused into the attention calls (paper: the "Rotary (fwd)" row of
 * the kernel-suite microbenchmark table next to its attention rows; "rotate-half" pairing as
 * rowops_rotary_fwd of rowops.h: column d pairs with d + D/2, tables fp32 [Sk][D/2] indexed by
 * the absolute position).  D must be 64 or 128 and Sk >= Sq, else ATTN_ERR_SHAPE; query row i
 * has position i + Sk - Sq, key row j position j.
 *
 * The contract is: K is rotated where it is written (once, e.g. into the key/value cache, by
 * rowops_rotary_fwd) and comes in rotated; Q comes in UNROTATED and is rotated in registers as
 * the kernel loads it -- the result is, bit for bit, that of rowops_rotary_fwd on Q followed by
 * attn_fwd_rect, without the pass over Q.  (K is not rotated in the kernel: every query tile of
 * a head would repeat that work.)
 *   attn_fwd_rope: Q in (unrotated), K_rot, V in; cos_table, sin_table in; O, LSE out as
 *     attn_fwd_rect; Q_rot: optional out (NULL: not stored), the rotated query rows, same
 *     strides as Q -- what attn_bwd_rope needs.  Workspace as attn_fwd_rect, sized by
 *     attn_fwd_rope_workspace_bytes (the same plan as attn_fwd_rect: when decoding, Sq == 1, the
 *     query heads of a K/V head are handled as rows of one head, all at the last position).
 *   attn_bwd_rope: Q_rot, K_rot, V, O, dO, LSE in as attn_bwd_rect (with the ROTATED Q and K);
 *     dQ out: gradient of the UNROTATED query rows (the accumulated gradient is rotated back in
 *     registers before it is stored); dK_rot out: gradient of the rotated K rows (rotate it
 *     back with rowops_rotary_fwd and a negated sin table if the unrotated one is wanted);
 *     dV out.  Workspace of attn_bwd_rect_workspace_bytes(p) bytes.
 * Tables must be 16-byte aligned; everything else as the rectangular calls.
 */
size_t attn_fwd_rope_workspace_bytes(const attn_rect_params_t *p);

int attn_fwd_rope(const void *Q, const void *K_rot, const void *V, const float *cos_table,
                  const float *sin_table, void *O, float *LSE, void *Q_rot, void *workspace,
                  size_t workspace_bytes, const attn_rect_params_t *p, void *hip_stream);

int attn_bwd_rope(const void *Q_rot, const void *K_rot, const void *V, const void *O,
                  const void *dO, const float *LSE, const float *cos_table, const float *sin_table,
                  void *dQ, void *dK_rot, void *dV, void *workspace, size_t workspace_bytes,
                  const attn_rect_params_t *p, void *hip_stream);

/*
 * attn_bwd_rect for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * backward's scratch (two fp32 values per query row) lives in an array inside the library's
 * device image, ATTN_NOALLOC_SCRATCH_BYTES long; each GPU the library runs on holds its own
 * copy until the process ends.  Arguments, validation and stream semantics are those of
 * attn_bwd_rect without the workspace pair; results are bit for bit those of attn_bwd_rect
 * called with a workspace of ATTN_NOALLOC_SCRATCH_BYTES bytes.
 *   - Problems with more than ATTN_NOALLOC_SCRATCH_BYTES / 8 query rows (B*Hq*Sq) give
 *     ATTN_ERR_WORKSPACE; nothing is launched.
 *   - The call allocates and frees nothing.  The first call on a device asks the runtime for
 *     the array's address on that device (make that call outside graph capture); failure to
 *     obtain it gives ATTN_ERR_LAUNCH.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU
 *     (different streams, or threads) race on it and give wrong results.  Calls on one stream,
 *     one after the other, are safe; nothing has to be cleared between them.
 */
#define ATTN_NOALLOC_SCRATCH_BYTES (8u << 20)
int attn_bwd_rect_noalloc(const void *Q, const void *K, const void *V, const void *O,
                          const void *dO, const float *LSE, void *dQ, void *dK, void *dV,
                          const attn_rect_params_t *p, void *hip_stream);

/*
 * IEEE fp16 variant of the rectangular entry points (an extension: the paper's microbenchmark
 * table names bf16 only): Q, K, V, O, dO, dQ, dK, dV hold fp16 instead of bf16; LSE, the
 * workspaces (same sizes, same *_workspace_bytes functions), parameters, errors and stream
 * semantics are unchanged.  Accumulation is fp32; P and dS are rounded to fp16 for the
 * second matrix product of each stage.
 */
int attn_fwd_rect_f16(const void *Q, const void *K, const void *V, void *O, float *LSE,
                      void *workspace, size_t workspace_bytes,
                      const attn_rect_params_t *p, void *hip_stream);

int attn_bwd_rect_f16(const void *Q, const void *K, const void *V, const void *O, const void *dO,
                      const float *LSE, void *dQ, void *dK, void *dV,
                      void *workspace, size_t workspace_bytes,
                      const attn_rect_params_t *p, void *hip_stream);

/* Measurement aid, not a step of the method: enqueues a kernel that executes nothing but bf16
 * 32x32x16 MFMAs (the instruction the attention kernels are built on): the figure the matrix
 * pipes of THIS device sustain, to print beside the nominal peak.  (The paper's microbenchmark
 * table prints latencies only; the fraction of peak is this build's own yardstick.)
 * `workgroups` work-groups of 512 threads each run `iters` iterations of 16 MFMAs per wave.
 * random_operands: 0 = the same small constant operands at every step; non-zero = operands
 * with random signs and mantissas that change from step to step, as real data does (the
 * clock a GPU sustains depends on how much the operand buses toggle).
 * sink: DEVICE, at least workgroups * 512 floats (sink_floats = its size), fully overwritten;
 * flop: HOST, optional; receives the floating-point operations one launch executes.
 * Errors: ATTN_ERR_NULL (sink), ATTN_ERR_SHAPE (workgroups or iters < 1, workgroups > 2^20),
 * ATTN_ERR_WORKSPACE (sink too small), ATTN_ERR_ALIGN, ATTN_ERR_LAUNCH.  Asynchronous. */
int attn_probe_mfma_bf16(int workgroups, int iters, int random_operands, float *sink,
                         size_t sink_floats, double *flop, void *hip_stream);

/* Measurement aid, not a step of the method: the fp32 atomic traffic of a backward that would
 * form dQ inside the key-block kernel (one launch, five matrix products per tile pair instead
 * of the seven that the two-kernel backward executes), with nothing else running.  For BH heads
 * of S rows and key blocks of key_block keys, the work-group of key block kb adds a 32 x 128
 * fp32 tile (16 KiB) to acc[head][32 s .. 32 s + 31][0..127] for every 32-row slot s that sees
 * the block (all slots, or with causal != 0 those from the block's diagonal on).  acc must be
 * zeroed by the caller; afterwards element (head, row, d) holds the number of key blocks that
 * see the row's slot.
 * acc: DEVICE, at least BH * S * 128 floats (acc_floats = its size); bytes_added: HOST,
 * optional, receives the bytes one launch adds.  BH a multiple of 8 up to 4096, S and
 * key_block multiples of 32, key_block <= S <= 2^20, else ATTN_ERR_SHAPE; ATTN_ERR_NULL,
 * ATTN_ERR_WORKSPACE (acc too small), ATTN_ERR_ALIGN, ATTN_ERR_LAUNCH.  Asynchronous. */
int attn_probe_atomic_f32(int BH, int S, int key_block, int causal, float *acc,
                          size_t acc_floats, double *bytes_added, void *hip_stream);

/* Measurement aid, not a step of the method: what work-groups that only read can stream from
 * device memory -- the ceiling for decoding, whose forward reads K and V once and does little
 * else (the paper reports its kernel's weak spot on small-batch prefill and decode shapes
 * without a bandwidth figure; this is the build's own yardstick for them).
 * `workgroups` work-groups of 256 threads read `bytes` bytes from src, each a contiguous share,
 * and write the XOR of all 32-bit words they read to checksum[work-group].
 * direct bit 0 clear: plain 16-byte loads, eight in flight per lane, work-group g reads
 *   [g * bytes/workgroups, (g+1) * bytes/workgroups).
 * direct bit 1: the loads or transfers carry the non-temporal hint.
 * direct bit 0 set: direct global -> LDS transfers in the shape of the decoding forward: src is taken
 *   as two tensors (its halves); work-group g reads its contiguous share of each, in tiles of
 *   16 KB per tensor, two tile buffers, one tile in flight, one barrier per tile, 1 KB per
 *   transfer with neighbouring lanes on neighbouring 256-byte rows.
 * src: DEVICE, 16-byte aligned, bytes a multiple of workgroups * 32768 and at most 2 GiB per
 * work-group; checksum: DEVICE, workgroups uint32, fully overwritten.
 * Errors: ATTN_ERR_NULL, ATTN_ERR_SHAPE, ATTN_ERR_ALIGN, ATTN_ERR_LAUNCH.  Asynchronous. */
int attn_probe_stream(const void *src, size_t bytes, int workgroups, int direct,
                      uint32_t *checksum, void *hip_stream);

/* Static, NUL-terminated description of a status code.  Never NULL. */
const char *attn_status_string(int status);

/* ABI version: major*1000 + minor. */
int attn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MI355_ATTN_H */
