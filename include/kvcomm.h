/*
 * kvcomm.h - C ABI of the MI355X (gfx950) implementation of KVComm's cache-reuse step
 * (arxiv 2510.12872, Sec. 3.4 "Anchor-based Cache Update" and the reuse branch of
 * Algorithm 1): instead of re-prefilling a shared segment (a placeholder sample such as
 * a peer agent's message) under a new agent-specific prefix, its base KV-cache is
 *   1. re-positioned: keys rotated by the RoPE position delta (Sec. 3.1, "Positional
 *      Alignment"),
 *   2. matched against the segment's anchor pool: l2 distance of base keys, softmax of
 *      the negative distance across anchors (Eq. "pred", Eq. "ph_update"),
 *   3. corrected by the weighted sum of the anchors' stored key/value deviations
 *      (Eq. "ph_update"; Eq. "pf_update" for the neighbouring prefix segment),
 *   4. written into the agent's contiguous cache (the concatenation of workflow step 4),
 * after which the remaining non-shared query tokens attend causally over that cache.
 *
 * General conventions
 *   - All tensor data lives in DEVICE memory.  Small metadata arrays (anchor pointer
 *     lists, anchor lengths, anchor position deltas) live in HOST memory and are read
 *     during the call; they may be freed or changed as soon as the call returns.
 *   - Ownership: the caller owns every buffer.  The library never allocates, frees or
 *     keeps device memory and retains no pointer after a call returns.
 *   - Asynchrony: a call only enqueues kernels on `stream` (a hipStream_t, passed as
 *     void*; NULL is the default stream).  It never synchronises.  Buffers must stay
 *     valid until the stream has passed the enqueued work.
 *   - Errors: every entry point returns a kvcomm_status (0 = OK, negative = error).
 *     Arguments are validated on the host before anything is enqueued; on an argument
 *     error nothing is launched and no output is touched.  A failed launch returns
 *     KVCOMM_EHIP.  No C++ exception crosses this boundary.
 *   - Thread safety: no mutable global state; calls from several host threads are safe
 *     as long as they do not write the same buffers.
 *   - Tensors are described by kvcomm_tensor: a base pointer plus strides in ELEMENTS for
 *     the layer, head and token axes; the channel axis (length head_dim) is contiguous.
 *     Base pointers must be 16-byte aligned and every stride a multiple of
 *     16 / sizeof(element) so that each row can be moved with 16-byte accesses.
 *   - Supported: dtype f32 or bf16; head_dim in {64, 128, 256};
 *     n_q_heads a multiple of n_kv_heads; 0 <= n_anchors <= KVCOMM_MAX_ANCHORS.
 *     Anything else returns KVCOMM_EUNSUPPORTED.
 */
#ifndef KVCOMM_H
#define KVCOMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KVCOMM_MAX_ANCHORS 64
#define KVCOMM_MAX_BATCH 8   /* segments per batched launch */

typedef enum {
    KVCOMM_OK = 0,
    KVCOMM_EINVAL = -1,        /* null / misaligned pointer, non-positive size or temperature, bad enum */
    KVCOMM_EUNSUPPORTED = -2,  /* valid request outside the supported shapes / dtypes */
    KVCOMM_EWORKSPACE = -3,    /* workspace missing or smaller than the matching *_workspace() size */
    KVCOMM_EHIP = -4           /* the HIP runtime refused a launch */
} kvcomm_status;

typedef enum { KVCOMM_F32 = 0, KVCOMM_BF16 = 1 } kvcomm_dtype;

/* What the norm ||h_phi - h_psi|| of the weighting rule is reduced over, i.e. how many
 * independent softmaxes one segment gets.  The paper's appendix on long-context anchor
 * matching states the per-token shape [m,1,1,seq_len,1]; that is the default.        */
typedef enum {
    KVCOMM_W_TOKEN = 0,            /* n = seg_len;               slot j = t               */
    KVCOMM_W_LAYER_HEAD_TOKEN = 1, /* n = L*Hkv*seg_len;         slot j = (l*Hkv+h)*S + t */
    KVCOMM_W_SEGMENT = 2           /* n = 1 (one scalar weight per anchor, as the entropy of Eq. "pred" uses) */
} kvcomm_wgran;

typedef struct {
    int32_t n_layers;    /* L   */
    int32_t n_kv_heads;  /* Hkv */
    int32_t n_q_heads;   /* Hq, a multiple of Hkv; query head hq reads kv head hq / (Hq/Hkv) */
    int32_t head_dim;    /* D   */
    int32_t dtype;       /* kvcomm_dtype of every cache / query / output tensor */
    double rope_theta;   /* RoPE base: channel pair (i, i + D/2) turns by pos * theta^(-2i/D) */
} kvcomm_model;

typedef struct {
    void *ptr;             /* device pointer to element (layer 0, head 0, token 0, channel 0) */
    int64_t stride_layer;  /* in elements */
    int64_t stride_head;
    int64_t stride_token;
} kvcomm_tensor;

/* Number of weight slots n for a granularity (see kvcomm_wgran); 0 on bad arguments. */
size_t kvcomm_weight_slots(const kvcomm_model *model, int32_t seg_len, int32_t gran);

/* --------------------------------------------------------------------------------------
 * Anchor matching: distances and weights (Eq. "pred" for the selection of anchors at
 * least as long as the sample; Eq. "ph_update" and the weight step of Algorithm 1 for
 *   w = softmax over anchors of  -||k_segment - k_anchor|| / temperature ).
 *
 *   seg_base_k     [L, Hkv, seg_len, D] base keys of the segment (base positions, unrotated).
 *   anchor_base_k  HOST array [n_anchors] of DEVICE pointers; anchor a's base keys are laid
 *                  out by `anchor_layout` (its ptr field is ignored) and hold anchor_len[a]
 *                  valid tokens.  Only the first seg_len tokens of a longer anchor are read.
 *   anchor_len     HOST array [n_anchors].  Anchor a is selected iff anchor_len[a] >= seg_len;
 *                  unselected anchors are never read.
 *   temperature    > 0; the paper's rule is 1.
 *   weights_out    DEVICE [n, n_anchors] fp32 (n = kvcomm_weight_slots): selected anchors of a
 *                  slot sum to 1, unselected anchors get exactly 0; all 0 if none is selected.
 *   nearest_out    DEVICE [n] int32 or NULL: selected anchor of smallest distance (lowest
 *                  index among equals), -1 if none is selected.
 *   selected_out   DEVICE [n_anchors] int32 (0/1) or NULL.
 *   workspace      DEVICE scratch of at least kvcomm_anchor_weights_workspace() bytes,
 *                  256-byte aligned; contents are undefined afterwards.
 * Distances are accumulated in double precision in a fixed order (two deterministic
 * stages, no floating-point atomics), so results are reproducible run to run.
 * Errors: KVCOMM_EINVAL for null/misaligned pointers, seg_len <= 0, n_anchors <= 0,
 * temperature <= 0 or NaN, negative anchor_len, bad granularity; KVCOMM_EWORKSPACE.     */
size_t kvcomm_anchor_weights_workspace(const kvcomm_model *model, int32_t seg_len,
                                       int32_t n_anchors, int32_t gran);

int kvcomm_anchor_weights(const kvcomm_model *model, int32_t gran, float temperature,
                          kvcomm_tensor seg_base_k, int32_t seg_len,
                          const void *const *anchor_base_k, kvcomm_tensor anchor_layout,
                          const int32_t *anchor_len, int32_t n_anchors,
                          float *weights_out, int32_t *nearest_out, int32_t *selected_out,
                          void *workspace, size_t workspace_bytes, void *stream);

/* --------------------------------------------------------------------------------------
 * kvcomm_anchor_weights for callers that cannot allocate device memory or size a workspace:
 * code recorded into a HIP graph, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results (bit for bit) and errors as kvcomm_anchor_weights, without the workspace:
 * the partial sums live in a fixed array of KVCOMM_STATIC_SCRATCH_BYTES that is part of the
 * library image (each GPU that runs the library holds one copy until the process ends).  The
 * call allocates and frees nothing.  A request whose kvcomm_anchor_weights_workspace() exceeds
 * the array returns KVCOMM_EWORKSPACE and launches nothing (16 MiB covers every per-token and
 * per-segment request of up to 32768 tokens and 64 anchors; per-(layer, head, token) weights
 * need 8 bytes per layer, head, token and anchor and fit only for short segments).
 * All calls on one GPU share that GPU's array: two calls whose kernels may overlap (different
 * streams, different host threads) race on it and must be ordered by the caller.  The array's
 * contents after a call are undefined; no call relies on what an earlier one left.  The first
 * call on a GPU looks up the array's address (hipGetSymbolAddress); make that call outside
 * stream capture.                                                                         */
#define KVCOMM_STATIC_SCRATCH_BYTES (16u << 20)

size_t kvcomm_anchor_weights_static_capacity(void);   /* = KVCOMM_STATIC_SCRATCH_BYTES */

int kvcomm_anchor_weights_static(const kvcomm_model *model, int32_t gran, float temperature,
                                 kvcomm_tensor seg_base_k, int32_t seg_len,
                                 const void *const *anchor_base_k, kvcomm_tensor anchor_layout,
                                 const int32_t *anchor_len, int32_t n_anchors,
                                 float *weights_out, int32_t *nearest_out, int32_t *selected_out,
                                 void *stream);

/* --------------------------------------------------------------------------------------
 * Offset approximation fused with positional alignment (Eq. "ph_update"; with the
 * prefix segment's tensors and the placeholder's weights it is Eq. "pf_update"):
 *   out_k[l,h,t,:] = R(delta_pos) base_k[l,h,t,:]
 *                    + sum_a w[j,a] * R(delta_pos - anchor_delta_pos[a]) anchor_dk[a][l,h,t,:]
 *   out_v[l,h,t,:] =              base_v[l,h,t,:] + sum_a w[j,a] * anchor_dv[a][l,h,t,:]
 * where R(p) is the RoPE rotation by p positions and the sums run over selected anchors
 * (anchor_len[a] >= seg_len).  Accumulation is fp32 in anchor order after the rotated base
 * term; bf16 outputs are rounded to nearest even once, at the store.
 *
 *   base_k, base_v     [L, Hkv, seg_len, D] base cache of the segment.
 *   anchor_dk/dv       HOST arrays [n_anchors] of DEVICE pointers to the stored deviations,
 *                      laid out by `anchor_layout` (ptr ignored), anchor_len[a] valid tokens.
 *   weights            DEVICE [n, n_anchors] fp32 as written by kvcomm_anchor_weights.
 *   delta_pos          new start position minus base start position of the segment.
 *   anchor_delta_pos   HOST [n_anchors] or NULL.  Position delta at which anchor a's key
 *                      deviation was recorded; NULL means "recorded at delta_pos", i.e. the
 *                      deviation is added unrotated (rotate the base key, then add the offset).
 *   out_k, out_v       [L, Hkv, seg_len, D] destination, normally a view into the agent's
 *                      cache at the segment's token offset (so concatenation costs nothing).
 *                      out_k may be exactly base_k, and out_v exactly base_v (in place: same
 *                      pointer and strides).  Any other sharing of bytes between an output and
 *                      another tensor of the call (the other output, a base tensor, a selected
 *                      anchor's deviations, the weights) returns KVCOMM_EINVAL; the check works
 *                      on the byte runs of whole (layer, head) blocks, first to last token.
 * n_anchors may be 0 (pure re-positioning; weights may then be NULL).
 * Errors: KVCOMM_EINVAL / KVCOMM_EUNSUPPORTED as above.                                  */
int kvcomm_align_kv(const kvcomm_model *model, int32_t gran,
                    kvcomm_tensor base_k, kvcomm_tensor base_v, int32_t seg_len,
                    const void *const *anchor_dk, const void *const *anchor_dv,
                    kvcomm_tensor anchor_layout, const int32_t *anchor_len, int32_t n_anchors,
                    const float *weights, int32_t delta_pos, const int32_t *anchor_delta_pos,
                    kvcomm_tensor out_k, kvcomm_tensor out_v, void *stream);

/* --------------------------------------------------------------------------------------
 * The same update for several segments in ONE launch (the reuse branch of Algorithm 1 treats
 * the placeholders of a prompt, and the prefix segments that follow them (Eq. "pf_update"),
 * independently and "in parallel").  Job j has exactly the arguments of kvcomm_align_kv; all
 * jobs share `anchor_layout` and the weight granularity.  For a prefix segment pass its own
 * base cache and stored deviations with the PLACEHOLDER's weights: per-segment weights
 * (KVCOMM_W_SEGMENT) apply to a segment of any length, per-token weights need equal lengths:
 * each job states the rows of its weight buffer (weights_slots), and a job whose rows differ from
 * kvcomm_weight_slots(seg_len, gran) is refused with KVCOMM_EINVAL before anything is read.
 * Limits: n_jobs <= KVCOMM_MAX_BATCH; over all jobs at most KVCOMM_MAX_ANCHORS selected anchors
 * and KVCOMM_MAX_ANCHORS + 1 distinct rotations; beyond them KVCOMM_EUNSUPPORTED (split the call).
 * Results are bit-identical to n_jobs separate kvcomm_align_kv calls.  The aliasing rule of
 * kvcomm_align_kv holds across jobs too: an output that shares bytes with another job's output
 * or inputs returns KVCOMM_EINVAL.                                                        */
typedef struct {
    kvcomm_tensor base_k, base_v;       /* [L, Hkv, seg_len, D] */
    kvcomm_tensor out_k, out_v;
    int32_t seg_len;
    int32_t delta_pos;
    const void *const *anchor_dk;       /* HOST [n_anchors] of DEVICE pointers */
    const void *const *anchor_dv;
    const int32_t *anchor_len;          /* HOST [n_anchors] */
    const int32_t *anchor_delta_pos;    /* HOST [n_anchors] or NULL */
    int32_t n_anchors;
    const float *weights;               /* DEVICE [weights_slots, n_anchors] */
    int64_t weights_slots;              /* rows of `weights`; must equal kvcomm_weight_slots(seg_len, gran) */
} kvcomm_align_job;

int kvcomm_align_kv_batch(const kvcomm_model *model, int32_t gran, kvcomm_tensor anchor_layout,
                          const kvcomm_align_job *jobs, int32_t n_jobs, void *stream);

/* --------------------------------------------------------------------------------------
 * Causal attention of the tq non-shared suffix queries over the assembled cache (workflow
 * step 4; q, k, v as defined in Sec. 3.1).  Suffix query i sits at cache position
 * n_ctx + i and attends to cache tokens 0 .. n_ctx + i:
 *   out[l,hq,i,:] = softmax_j( scale * <q[l,hq,i,:], k[l,hq/G,j,:]> ) v[l,hq/G,j,:]
 *
 *   q, out          [L, Hq, tq, D]; queries already carry their rotary position.
 *   cache_k/v       [L, Hkv, n_ctx + tq, D]; the suffix tokens' own K/V are already stored at
 *                   positions n_ctx .. n_ctx+tq-1.
 *   softmax_scale   <= 0 selects 1/sqrt(D).
 *   lse_out         DEVICE [L, Hq, tq] fp32 natural-log-sum-exp of the scaled scores, or NULL.
 *   workspace       kvcomm_suffix_attn_workspace() bytes (may be 0, then NULL is accepted).
 * bf16 tensors use bf16 MFMA with fp32 accumulation and an fp32 online softmax; f32 tensors
 * use fp32 arithmetic throughout.
 * Errors: KVCOMM_EINVAL for null/misaligned pointers, tq <= 0, n_ctx < 0;
 * KVCOMM_EUNSUPPORTED for bf16 caches whose token stride is D * 2^21 elements or more
 * (the kernel addresses a group of 512 / D rows with a 32-bit byte offset).                 */
size_t kvcomm_suffix_attn_workspace(const kvcomm_model *model, int32_t n_ctx, int32_t tq);

int kvcomm_suffix_attn(const kvcomm_model *model, kvcomm_tensor q,
                       kvcomm_tensor cache_k, kvcomm_tensor cache_v,
                       int32_t n_ctx, int32_t tq, float softmax_scale,
                       kvcomm_tensor out, float *lse_out,
                       void *workspace, size_t workspace_bytes, void *stream);

/* The same attention (workflow step 4), same arguments, results bit-identical to kvcomm_suffix_attn, launched
 * as at most `max_blocks` thread blocks that each walk a fixed share of the (layer, kv head, query tile) work
 * items.  A block of the bf16 kernel fills a compute unit, so the launch occupies max_blocks of the GPU's 256
 * compute units and leaves the others to kernels that run beside it on another stream: the memory-bound
 * alignment of the next agent next to the matrix-core-bound attention of the current one.  (Under the chip's
 * power limit the attention loses less than its share of compute units: measured 0.82 ms on 160 of 256 against
 * 0.66 ms on all of them.)  max_blocks is spread over the 8 XCDs in launch order; values of at least the number
 * of work items give the plain launch.  f32 tensors ignore max_blocks (their kernel is small-block and never fills
 * the chip's registers).
 * Errors: as kvcomm_suffix_attn; KVCOMM_EINVAL for max_blocks < 8 (one block per XCD is the minimum).          */
int kvcomm_suffix_attn_confined(const kvcomm_model *model, kvcomm_tensor q,
                                kvcomm_tensor cache_k, kvcomm_tensor cache_v,
                                int32_t n_ctx, int32_t tq, float softmax_scale,
                                kvcomm_tensor out, float *lse_out,
                                int32_t max_blocks, void *stream);

/* --------------------------------------------------------------------------------------
 * Weighting variants of the appendix on the approximation method: the default rule
 * (softmax of the negative l2 distance), "nearest" (all weight on the selected anchor of
 * smallest l2 distance) and "cosine" (softmax across anchors of the cosine similarity of
 * the base keys, reduced over the same axes as the distance).
 * Same arguments, outputs and errors as kvcomm_anchor_weights, plus `rule`; for
 * KVCOMM_RULE_COSINE nearest_out holds the anchor of LARGEST similarity.  The workspace
 * must hold kvcomm_anchor_weights_rule_workspace() bytes for the same rule.              */
typedef enum {
    KVCOMM_RULE_L2_SOFTMAX = 0,
    KVCOMM_RULE_NEAREST = 1,
    KVCOMM_RULE_COSINE_SOFTMAX = 2
} kvcomm_rule;

size_t kvcomm_anchor_weights_rule_workspace(const kvcomm_model *model, int32_t seg_len,
                                            int32_t n_anchors, int32_t gran, int32_t rule);

int kvcomm_anchor_weights_rule(const kvcomm_model *model, int32_t gran, int32_t rule, float temperature,
                               kvcomm_tensor seg_base_k, int32_t seg_len,
                               const void *const *anchor_base_k, kvcomm_tensor anchor_layout,
                               const int32_t *anchor_len, int32_t n_anchors,
                               float *weights_out, int32_t *nearest_out, int32_t *selected_out,
                               void *workspace, size_t workspace_bytes, void *stream);

/* --------------------------------------------------------------------------------------
 * Anchor matching of several segments in ONE launch of each stage (see kvcomm_align_kv_batch for
 * the reason).  Job j has the per-segment arguments of kvcomm_anchor_weights_rule; all jobs share
 * `anchor_layout`, the granularity, the rule and the temperature.  The workspace holds
 * kvcomm_anchor_weights_batch_workspace() bytes for the same segment lengths and pool sizes.
 * Limits: n_jobs <= KVCOMM_MAX_BATCH and at most KVCOMM_MAX_ANCHORS selected anchors over all jobs
 * (else KVCOMM_EUNSUPPORTED).  Each segment's result is what the single-segment call would give up
 * to the rounding of the double-precision partial sums (the cut into chunks may differ).        */
typedef struct {
    kvcomm_tensor seg_base_k;           /* [L, Hkv, seg_len, D] */
    int32_t seg_len;
    const void *const *anchor_base_k;   /* HOST [n_anchors] of DEVICE pointers */
    const int32_t *anchor_len;          /* HOST [n_anchors] */
    int32_t n_anchors;
    float *weights_out;                 /* DEVICE [n, n_anchors] */
    int32_t *nearest_out;               /* DEVICE [n] or NULL */
    int32_t *selected_out;              /* DEVICE [n_anchors] or NULL */
} kvcomm_weights_job;

size_t kvcomm_anchor_weights_batch_workspace(const kvcomm_model *model, int32_t gran, int32_t rule,
                                             const int32_t *seg_lens, const int32_t *n_anchors,
                                             int32_t n_jobs);

int kvcomm_anchor_weights_batch(const kvcomm_model *model, int32_t gran, int32_t rule, float temperature,
                                kvcomm_tensor anchor_layout, const kvcomm_weights_job *jobs, int32_t n_jobs,
                                void *workspace, size_t workspace_bytes, void *stream);

/* --------------------------------------------------------------------------------------
 * Anchor prediction (Eq. "pred"): should a sample become a new anchor?  Yes (1) when it is
 * longer than every anchor of the pool, when no anchor is at least as long, or when the
 * entropy of its weights over the candidate anchors, H = -sum_a w log w (the printed formula
 * lacks the minus sign), exceeds gamma * log(number of candidates).  With more than one
 * weight slot the mean entropy over the slots is compared.
 *
 *   weights        DEVICE [n_slots, n_anchors] fp32 from kvcomm_anchor_weights*.
 *   anchor_len     HOST [n_anchors]; candidates are the anchors with anchor_len >= seg_len.
 *   entropy_out    DEVICE [n_slots] fp32 or NULL.
 *   result_out     DEVICE float[2]: [0] = decision (1.0 new anchor / 0.0 shareable),
 *                  [1] = mean entropy.
 *   workspace      DEVICE scratch of kvcomm_anchor_predict_workspace(n_slots) bytes, 8-byte aligned.
 * Two small kernels; sums are taken in double in a fixed order.
 * Errors: KVCOMM_EINVAL for null pointers, n_slots <= 0, n_anchors <= 0, seg_len <= 0,
 * negative anchor_len, gamma < 0 or NaN; KVCOMM_EWORKSPACE.                              */
size_t kvcomm_anchor_predict_workspace(int64_t n_slots);

int kvcomm_anchor_predict(const float *weights, int64_t n_slots, const int32_t *anchor_len,
                          int32_t n_anchors, int32_t seg_len, float gamma,
                          float *entropy_out, float *result_out,
                          void *workspace, size_t workspace_bytes, void *stream);

/* --------------------------------------------------------------------------------------
 * Offset capture (fallback branch of Algorithm 1: after a dense generation, the offset
 * between the real and the base KV-cache fills a new anchor).  Inverse of kvcomm_align_kv
 * for a single anchor of weight 1 recorded at delta_pos:
 *   out_dk[l,h,t,:] = real_k[l,h,t,:] - R(delta_pos) base_k[l,h,t,:]
 *   out_dv[l,h,t,:] = real_v[l,h,t,:] -              base_v[l,h,t,:]
 * All six tensors are [L, Hkv, seg_len, D]; real_k / real_v are normally views into the
 * agent's cache at the segment's token offset.  fp32 arithmetic, one rounding at the store.
 * Errors as for kvcomm_align_kv.                                                         */
int kvcomm_capture_offsets(const kvcomm_model *model, kvcomm_tensor base_k, kvcomm_tensor base_v,
                           kvcomm_tensor real_k, kvcomm_tensor real_v, int32_t seg_len, int32_t delta_pos,
                           kvcomm_tensor out_dk, kvcomm_tensor out_dv, void *stream);

/* --------------------------------------------------------------------------------------
 * Compressed anchor deviations (the appendix on memory cost observes that the deviation
 * tensors are small in magnitude and names their compression as future work).  Storage:
 * one byte per element in the OCP 8-bit floating-point format E4M3 (1 sign, 4 exponent bits
 * with bias 7, 3 mantissa bits, no infinities, largest finite value 448) times a power-of-two
 * scale per tensor:  value = scale * e4m3(byte).  LOSSY: relative error at most 2^-4 for
 * |x| >= scale * 2^-6, absolute error at most scale * 2^-10 below; |x| > 448 * scale saturates.
 * Byte tensors are described by kvcomm_tensor with strides in bytes; pointers 16-byte aligned,
 * strides multiples of 16.
 *
 * kvcomm_quantize_deltas: in [L, Hkv, n_tokens, D] of the model dtype -> out, same shape, E4M3
 * bytes of in / scale rounded to nearest (ties to even); a NaN becomes the code 0x7f, +-infinity
 * saturates like any value beyond +-448 * scale.  scale must be a normal power of two, 2^-126 ...
 * 2^127 (else KVCOMM_EINVAL): the division is then exact and the codes are reproducible bit for bit.
 *
 * kvcomm_align_kv_q8: kvcomm_align_kv with anchor_dk / anchor_dv pointing at E4M3 tensors laid
 * out by `anchor_layout` (bytes) and HOST arrays anchor_scale_k / anchor_scale_v [n_anchors] of
 * their scales.  Everything else (selection, rotation of deviations recorded elsewhere, fp32
 * accumulation in anchor order, one rounding at the store) is as in kvcomm_align_kv.          */
int kvcomm_quantize_deltas(const kvcomm_model *model, kvcomm_tensor in, int32_t n_tokens, float scale,
                           kvcomm_tensor out, void *stream);

int kvcomm_align_kv_q8(const kvcomm_model *model, int32_t gran,
                       kvcomm_tensor base_k, kvcomm_tensor base_v, int32_t seg_len,
                       const void *const *anchor_dk, const void *const *anchor_dv,
                       kvcomm_tensor anchor_layout, const int32_t *anchor_len,
                       const float *anchor_scale_k, const float *anchor_scale_v, int32_t n_anchors,
                       const float *weights, int32_t delta_pos, const int32_t *anchor_delta_pos,
                       kvcomm_tensor out_k, kvcomm_tensor out_v, void *stream);

/* The compressed update for several segments in ONE launch: kvcomm_align_kv_batch with E4M3
 * deviations.  Job j has the per-segment arguments of kvcomm_align_kv_q8; limits, aliasing rule
 * and the weights_slots check are those of kvcomm_align_kv_batch; results are bit-identical to
 * n_jobs separate kvcomm_align_kv_q8 calls.                                                   */
typedef struct {
    kvcomm_tensor base_k, base_v;       /* [L, Hkv, seg_len, D], model dtype */
    kvcomm_tensor out_k, out_v;
    int32_t seg_len;
    int32_t delta_pos;
    const void *const *anchor_dk;       /* HOST [n_anchors] of DEVICE pointers to E4M3 tensors */
    const void *const *anchor_dv;
    const int32_t *anchor_len;          /* HOST [n_anchors] */
    const int32_t *anchor_delta_pos;    /* HOST [n_anchors] or NULL */
    const float *anchor_scale_k;        /* HOST [n_anchors], powers of two */
    const float *anchor_scale_v;
    int32_t n_anchors;
    const float *weights;               /* DEVICE [weights_slots, n_anchors] */
    int64_t weights_slots;
} kvcomm_align_q8_job;

int kvcomm_align_kv_q8_batch(const kvcomm_model *model, int32_t gran, kvcomm_tensor anchor_layout,
                             const kvcomm_align_q8_job *jobs, int32_t n_jobs, void *stream);

/* Human-readable name of a kvcomm_status; never NULL. */
const char *kvcomm_status_string(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int kvcomm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVCOMM_H */
