/*
 * mvla.h -- C ABI of the MI355X (gfx950) pruned-prefill library.
 *
 * The library runs the prefill of a LLaMA-2-shaped multi-visual-modal VLA
 * backbone over the token sequence [2D image tokens | 3D point tokens |
 * language tokens] (paper App. C "MVLA Models", Sec. 5.1 "Setup") with the
 * token-pruning step placed inside it: attention-score salience of every
 * visual token (Sec. 3.2, Eq. 3), a 2D:3D split of one keep budget by the
 * modality mass ratio (Eq. 5), per-modality top-k selection, and compaction of
 * the kept tokens, which alone go on to the later layers (Sec. 4.4, Eq. 10).
 *
 * Conventions that hold for every call unless a comment says otherwise:
 *  - Every pointer marked "device" is a DEVICE pointer owned by the caller
 *    (normally PyTorch tensor storage).  The library never allocates, frees or
 *    keeps caller buffers; its only memory is the workspace handed to
 *    mvla_create(), which the caller also owns and must keep alive until
 *    mvla_destroy().
 *  - Calls enqueue work on the context's HIP stream and return without waiting
 *    for it.  Calls on one context are stream-ordered; two contexts sharing a
 *    workspace must not run concurrently.
 *  - Arguments are validated on the host before anything is launched.  On any
 *    error nothing is launched and no output is written.
 *  - Return value: MVLA_OK (0) or a negative mvla_status.
 *  - Row-major everywhere; "bf16" is the 16-bit brain-float storage format.
 */
#ifndef MVLA_H_
#define MVLA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MVLA_OK = 0,
    MVLA_EINVAL = -1,       /* null pointer, bad shape, bad alignment             */
    MVLA_ENOMEM = -2,       /* workspace too small for the requested shape        */
    MVLA_EHIP = -3,         /* HIP runtime / launch failure                       */
    MVLA_EUNSUPPORTED = -4, /* shape outside what the kernels are built for       */
    MVLA_ELIMIT = -5        /* shape beyond the fixed scratch of mvla_salience_noalloc */
} mvla_status;

typedef struct mvla_ctx mvla_ctx; /* opaque */

/* Library version, "major.minor.patch". */
const char* mvla_version(void);
/* Static, human-readable text for a status code. */
const char* mvla_strerror(int code);

/* Bytes of workspace needed for batches up to [B, S] with the given layer
 * shape (D hidden, H heads, F MLP width) and up to n_query_tail scoring rows.
 * Covers every call below.  Returns 0 for non-positive arguments. */
size_t mvla_workspace_bytes(int B, int S, int D, int H, int F, int n_query_tail);

/* Create a context bound to `device`, a borrowed HIP stream (NULL = the
 * default stream) and a caller-owned device workspace (256-byte aligned).
 * Enqueues a clear of the workspace's counter area on the stream. */
int mvla_create(mvla_ctx** out, int device, void* hip_stream, void* workspace /*device*/,
                size_t workspace_bytes);
/* Rebind to another borrowed stream (previous work must have completed or be
 * ordered before it by the caller). */
int mvla_set_stream(mvla_ctx* ctx, void* hip_stream);
/* Frees host-side state only.  Does not synchronise. */
void mvla_destroy(mvla_ctx* ctx);

/* ------------------------------------------------------------------------ */
/* Pruning step                                                             */
/* ------------------------------------------------------------------------ */

/* Attention-score salience (Sec. 3.2: the attention matrix is partitioned by
 * token modality and each visual token is scored by the L1 norm of its
 * attention column, Eq. 3 / numerators of Eq. 5; probabilities are >= 0 so the
 * norm is a sum; "avg" is the mean over the H*Nq rows):
 *     sal[b, j] = (1 / (H*Nq)) * sum_h sum_q attn[b, h, q, j],   0 <= j < n_vis.
 * attn: device, fp32 [B, H, Nq, S], rows already softmaxed; n_vis <= S.
 * sal : device, fp32 [B, n_vis], fully overwritten.
 * Summation order is fixed, so results are bit-reproducible run to run. */
int mvla_salience(mvla_ctx* ctx, const float* attn, int B, int H, int Nq, int S, int n_vis,
                  float* sal);

/* mvla_salience for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Takes no context: the kernel's scratch (row-split partial
 * sums and arrival counters) is a fixed array inside the library, 16 MiB +
 * 32 KiB on each GPU the call is used on, held until the process ends.  The
 * call allocates nothing, enqueues two kernels on hip_stream (borrowed; NULL =
 * default stream) of the current device and returns; results are identical to
 * mvla_salience.  Shapes whose scratch need exceeds the array -- more than
 * (n_vis + 64) * (H*Nq/32 + 2) * B floats of partial sums in 16 MiB, or more
 * than 8192 (sample, 64-column chunk) pairs -- are rejected with MVLA_ELIMIT
 * (all five workload shapes of the paper's setup fit).  All calls on one GPU
 * share the array: calls that overlap in time on one GPU (two streams, two
 * threads) race; issue them on one stream or order them yourself. */
int mvla_salience_noalloc(void* hip_stream, const float* attn, int B, int H, int Nq, int S,
                          int n_vis, float* sal);

/* Split the visual keep budget between modalities by salience mass (Eq. 5:
 * m2 = |a_2D|_1 / (|a_2D|_1 + |a_3D|_1); Sec. 5.2: per-modality pruning
 * rates).  Per sample, masses are summed in fp64;
 *     K2 = floor(k_total*m2 + 0.5) clamped to [max(min2, k_total-n3), min(n2, k_total-min3)],
 *     K3 = k_total - K2;   zero total mass -> m2 = n2/(n2+n3).
 * sal : device, fp32 [B, n2+n3] (2D segment first).
 * k2k3: device, int32 [B, 2] = (K2, K3).
 * mass: device, fp32 [B, 2] = (m2, 1-m2), or NULL.
 * Requires 0 <= k_total <= n2+n3, min2+min3 <= k_total, min2 <= n2, min3 <= n3. */
int mvla_modality_budget(mvla_ctx* ctx, const float* sal, int B, int n2, int n3, int k_total,
                         int min2, int min3, int32_t* k2k3, float* mass);

/* Per-modality top-k (replaces the thresholded masks of Algorithm 1 by an
 * exact budget; mask semantics as Eq. 10).  In the 2D segment keep the K2
 * tokens of highest salience, in the 3D segment the K3 highest; equal scores:
 * the lower index is kept; -0 equals +0.  Indices are written ascending, then
 * all n_text language-token indices n2+n3 .. n2+n3+n_text-1 (never pruned).
 * sal     : device, fp32 [B, n2+n3]; NaN/Inf are invalid input (result then
 *           unspecified but in bounds).
 * k2k3    : device, int32 [B, 2], each row summing to k_total with
 *           0 <= K2 <= n2, 0 <= K3 <= n3 (as mvla_modality_budget writes);
 *           rows violating this are clamped on the device.
 * kept_idx: device, int32 [B, k_total + n_text], strictly increasing per row.
 * n2, n3 <= 16384 each (segment staged in LDS), else MVLA_EUNSUPPORTED. */
int mvla_select_topk(mvla_ctx* ctx, const float* sal, const int32_t* k2k3, int B, int n2, int n3,
                     int n_text, int k_total, int32_t* kept_idx);

/* Gather-compaction of the kept tokens (Sec. 4.4: tokens with mask 1 proceed
 * to later layers, mask 0 are discarded):
 *     h_out[b, i, :] = h[b, kept_idx[b, i], :],  pos_out[b, i] = pos[b, kept_idx[b, i]].
 * h, h_out: device, bf16 [B, S, D] / [B, S_out, D]; D % 8 == 0; must not overlap.
 * pos, pos_out: device, int32 [B, S] / [B, S_out].
 * kept_idx: device, int32 [B, S_out]; values outside [0, S) are clamped into
 * range on the device (never read out of bounds). */
int mvla_compact(mvla_ctx* ctx, const void* h, const int32_t* pos, const int32_t* kept_idx, int B,
                 int S, int S_out, int D, void* h_out, int32_t* pos_out);

/* Salience, budget, selection and compaction in one call (same results as the
 * four calls above in sequence; fewer launches).  sal, k2k3 are outputs too. */
int mvla_prune_step(mvla_ctx* ctx, const float* attn, int H, int Nq, const void* h,
                    const int32_t* pos, int B, int S, int D, int n2, int n3, int n_text,
                    int k_total, int min2, int min3, float* sal, int32_t* k2k3,
                    int32_t* kept_idx, void* h_out, int32_t* pos_out);

/* Per-patch modality indicators of the semantic stage (Sec. 3.2, Eqs. 4-6).
 * Patch p owns 2D token p and 3D token n_patch + p (needs as many 3D as 2D
 * tokens, as in the paper's 256 + 256 setup); its attention vectors a2, a3 run
 * over the H*Nq (head, query) rows.  a3 is split into its projection on a2 and
 * the orthogonal rest (Eq. 4):
 *     m2d[b,p] = |a2|_1 / (|a2|_1 + |a3|_1)                          (Eq. 5)
 *     m3d[b,p] = |a3 - (<a3,a2>/<a2,a2>) a2|_1 / (|a2|_1 + |a3|_1)     (Eq. 6)
 * (a2 = 0 leaves a3 whole; zero denominator -> 0).  These are the per-patch
 * indicators M^{S2}_{2D,p}, M^{S2}_{3D,p} of Algorithm 1; their means over
 * patches are its baselines.
 * attn: device fp32 [B, H, Nq, S] with 2*n_patch <= S; m2d, m3d: device fp32
 * [B, n_patch]. */
int mvla_modality_decompose(mvla_ctx* ctx, const float* attn, int B, int H, int Nq, int S,
                            int n_patch, float* m2d, float* m3d);

/* Temporal smoothing of a per-token (or per-patch) indicator across action
 * iterations (Sec. 4.3 Eq. 7; Sec. 4.4 Eqs. 8-9; Algorithm 1 "Action Iteration
 * Stage"), t counted from 1:
 *     t == 1      : x_hat = x_t                    (cold start: no history)
 *     1 < t < k   : x_hat = ((t-1)/t) x_hat + x_t/t    (running mean, Eq. 8)
 *     t >= k      : x_hat = beta x_hat + (1-beta) x_t  (Eq. 9)
 * x_t: device fp32 [n]; x_hat: device fp32 [n], read (t > 1) and overwritten.
 * Paper defaults: k = 7, beta = 0.85.  Requires 0 < beta < 1, t >= 1, k >= 1. */
int mvla_temporal_smooth(mvla_ctx* ctx, const float* x_t, float* x_hat, size_t n, int t, int k,
                         double beta);

/* Data-preprocessing indicators per patch (Sec. 3.1, Eq. 1): with l2, l3 the
 * L1 norms of the patch's 2D and 3D token features,
 *     m2d[b,p] = l2 / (l2 + l3),   m3d[b,p] = l3 / (l2 + l3)   (0 if l2+l3 == 0).
 * Patch p owns token rows p and n_patch + p.
 * feat: device bf16 [B, S, D], D % 8 == 0, 2*n_patch <= S (which layer's
 * output serves as "features" is the caller's choice); m2d, m3d: device fp32
 * [B, n_patch].  fp32 accumulation. */
int mvla_feature_share(mvla_ctx* ctx, const void* feat, int B, int S, int D, int n_patch,
                       float* m2d, float* m3d);

/* Constants of the mask rules of Algorithm 1.  tau_2d, tau_3d: the dual
 * threshold on the smoothed 3D feature share (Sec. 4.1; paper: 0.08, 0.20).
 * bg_drop: probability with which a background patch is discarded (Sec. 4.2:
 * 0.9).  obj_2d_min, obj_3d_max: an object patch keeps only its 2D token
 * when M2D^S2 > obj_2d_min and M3D^S2 < obj_3d_max (the paper says "far above
 * 0" and "near 0" without numbers).  kmeans_max_iter: cap on the Lloyd
 * assignments. */
typedef struct mvla_mask_rules {
    float tau_2d, tau_3d, bg_drop, obj_2d_min, obj_3d_max;
    int32_t kmeans_max_iter;
} mvla_mask_rules;
/* Fills *r (host) with 0.08, 0.20, 0.9, 0.9, 0.01, 32. */
void mvla_mask_rules_default(mvla_mask_rules* r);

/* Candidate sets, their fusion and the retention masks of Algorithm 1 for a
 * step t > 1 (Sec. 4.1, 4.2, 4.4; Eq. 10), one sample at a time:
 *  - patch score = sal[b,p] + sal[b,n_patch+p] (fp32); Lloyd's 1-D k-means
 *    with 3 centres started at (min, mid-range, max), nearest centre with the
 *    lower-numbered one on equal distance, centres as fp64 means, a centre
 *    without points unchanged, stopping when an assignment repeats or after
 *    kmeans_max_iter assignments; lowest centre = background (sem 0), middle =
 *    robot (1), highest = object (2);
 *  - baselines mu2, mu3: fp64 means over the sample's patches of M2D^S2, M3D^S2;
 *  - C1 = {2D} if M3D^S1 < tau_2d, {3D} if > tau_3d, else {2D,3D};
 *  - C2: background: {} if u < bg_drop else {2D,3D}; robot: {2D,3D} if
 *    M3D^S2 > mu3, else {2D} if M2D^S2 > mu2, else {}; object: {2D} under
 *    the exception above, else {2D,3D};
 *  - C2 = {} drops the patch; otherwise C = C1 & C2, or C2 when that is empty.
 * x_hat : device fp32 [4, B, n_patch], smoothed indicators in the order
 *         M2D^S1, M3D^S1, M2D^S2, M3D^S2 (row 0 is not read).
 * sal   : device fp32 [B, 2*n_patch] (as mvla_salience writes for n_vis = 2*n_patch).
 * u     : device fp32 [B, n_patch], caller-drawn uniforms in [0, 1).
 * rules : host.
 * mask2d, mask3d: device uint8 [B, n_patch], 1 = keep; sem: device uint8
 *         [B, n_patch] or NULL; kept_len: device int32 [B] = kept visual
 *         tokens + n_text.
 * n_patch <= 16384, else MVLA_EUNSUPPORTED.  NaN/Inf are invalid input. */
int mvla_candidate_masks(mvla_ctx* ctx, const float* x_hat, const float* sal, const float* u, int B,
                         int n_patch, int n_text, const mvla_mask_rules* rules, uint8_t* mask2d,
                         uint8_t* mask3d, uint8_t* sem, int32_t* kept_len);

/* Masks to token indices (Eq. 10: tokens with mask 1 go on): per sample the
 * kept 2D token indices ascending, then the kept 3D ones (n_patch + p), then
 * the n_text language tokens 2*n_patch ..; entries from kept_len[b] up to
 * S_pad repeat the last token's index so that every row has S_pad entries
 * (padding rows sit after all real rows, where causal attention never looks
 * back at them).  A row with more than S_pad kept tokens is cut at S_pad:
 * pass S_pad >= max_b kept_len[b].
 * kept_idx: device int32 [B, S_pad], usable by mvla_compact with S_out = S_pad. */
int mvla_mask_indices(mvla_ctx* ctx, const uint8_t* mask2d, const uint8_t* mask3d, int B,
                      int n_patch, int n_text, int S_pad, int32_t* kept_idx);

/* ------------------------------------------------------------------------ */
/* Backbone layer                                                           */
/* ------------------------------------------------------------------------ */

typedef struct {
    int D;         /* hidden size, multiple of 64, at most 8192                */
    int H;         /* attention heads                                          */
    int dh;        /* head dim: 64 or 128; H*dh == D                           */
    int F;         /* MLP width, multiple of 64, at most 2^20                  */
    float rms_eps; /* RMSNorm epsilon                                          */
} mvla_layer_cfg;

/* Weights of one decoder layer; all device pointers, bf16 unless noted.
 * Matrices are stored [out_features, in_features] row-major (y = x * W^T), so
 * both GEMM operands are contiguous along the contraction axis.
 *   wqkv     [3D, D]  rows 0..D-1 = query, D..2D-1 = key, 2D..3D-1 = value projection
 *   wo       [D, D]
 *   w_gateup [2F, D]  gate and up projections interleaved in blocks of 32 rows:
 *                     rows 64*i .. 64*i+31 = gate rows 32*i .. 32*i+31,
 *                     rows 64*i+32 .. 64*i+63 = up rows 32*i .. 32*i+31
 *   w_down   [D, F]
 *   g_attn, g_mlp [D] RMSNorm gains
 *   rope_cos, rope_sin: fp32 [rope_len, dh/2]; row = position id (see
 *                     mvla_rope_table); every pos value must be < rope_len. */
typedef struct {
    const void* wqkv;
    const void* wo;
    const void* w_gateup;
    const void* w_down;
    const void* g_attn;
    const void* g_mlp;
    const float* rope_cos;
    const float* rope_sin;
    int rope_len;
} mvla_layer_weights;

/* Fill a rotary table: cos/sin of pos * base^(-2i/dh), i < dh/2, evaluated in
 * fp64 and rounded to fp32.  cos_out, sin_out: device fp32 [rope_len, dh/2]. */
int mvla_rope_table(mvla_ctx* ctx, double base, int rope_len, int dh, float* cos_out,
                    float* sin_out);

/* One decoder layer of the backbone (App. C: LLaMA-2 7B; public layer maths:
 * RMSNorm -> q,k,v -> rotate-half RoPE by position id -> causal softmax
 * attention -> output projection + residual -> RMSNorm -> SiLU-gated MLP +
 * residual).  Causality follows row order, RoPE follows pos (so kept tokens
 * keep their original positions after compaction).
 * x, y : device, bf16 [B, S, D]; y may alias x.
 * pos  : device, int32 [B, S].
 * n_query_tail > 0: additionally write the attention probabilities of the
 * last n_query_tail rows (the language-token queries, Sec. 3.2) to
 * probs_out (device, fp32 [B, H, n_query_tail, S]); key_bias (device, fp32
 * [B, S] or NULL) is added to those scoring logits only, never to the layer's
 * own attention.  n_query_tail == 0: key_bias/probs_out ignored.
 * This call and the other layer and pruning calls only enqueue kernels on the
 * context's stream (no memset, no synchronisation, no allocation): with the
 * per-kernel timing off they may be recorded into a HIP graph and replayed. */
int mvla_prefill_layer(mvla_ctx* ctx, const mvla_layer_cfg* cfg, const mvla_layer_weights* w,
                       const void* x, const int32_t* pos, int B, int S, void* y, int n_query_tail,
                       const float* key_bias, float* probs_out);

/* The same layer with the scoring rows reduced on the fly (Sec. 3.2, Eq. 3):
 * instead of the probabilities it writes sal[b, j], j < n_vis, as
 * mvla_salience would from them; the [B, H, n_query_tail, S] tensor is never
 * materialised (column sums are formed per 32-query tile in registers, then
 * reduced over heads and tiles in a fixed order).  Differs from the two-call
 * route only in summation order.  n_query_tail >= 1, 1 <= n_vis <= S.
 * sal: device fp32 [B, n_vis].  Other arguments as mvla_prefill_layer. */
int mvla_prefill_layer_salience(mvla_ctx* ctx, const mvla_layer_cfg* cfg,
                                const mvla_layer_weights* w, const void* x, const int32_t* pos,
                                int B, int S, void* y, int n_query_tail, const float* key_bias,
                                int n_vis, float* sal);

/* The last full-sequence layer and the whole pruning step in one call: the
 * layer as above on S = n2 + n3 + n_text tokens with the n_text language
 * rows as scoring queries, salience reduced on the fly, budget split and
 * per-modality top-k (as mvla_modality_budget / mvla_select_topk), then the
 * gather of the kept rows of the layer output y and of pos (as mvla_compact).
 * y: device bf16 [B, S, D] (the full layer output, also an output); h_out:
 * device bf16 [B, k_total + n_text, D], must not overlap y; pos_out, sal, k2k3,
 * kept_idx as in mvla_prune_step. */
int mvla_prefill_layer_prune(mvla_ctx* ctx, const mvla_layer_cfg* cfg, const mvla_layer_weights* w,
                             const void* x, const int32_t* pos, int B, int S, void* y, int n2, int n3,
                             int n_text, int k_total, int min2, int min3, const float* key_bias,
                             float* sal, int32_t* k2k3, int32_t* kept_idx, void* h_out,
                             int32_t* pos_out);

/* Optional set-up step: times every tile configuration / K-split policy of
 * the four projections of a layer at M = B*S rows on this device, cycling
 * through the n_layers weight sets so that weights come from HBM as in real
 * use, and records the fastest per shape in the context; later layer calls at
 * that shape use it instead of the built-in cost model.  Results of the layer
 * calls change only in fp32 summation order.  Uses the context's workspace,
 * runs on and SYNCHRONISES the context's stream (not for use under graph
 * capture); takes a few tens of milliseconds.
 * layers: HOST array of n_layers weight descriptors (device pointers inside). */
int mvla_tune_layers(mvla_ctx* ctx, const mvla_layer_cfg* cfg, const mvla_layer_weights* layers,
                     int n_layers, int B, int S);
/* Record a choice by hand (e.g. one measured in an earlier run, for identical
 * summation order across runs): configuration index 0 .. 6 (256x256 on eight waves,
 * 256x128, 128x128 two per CU, 128x128 on eight waves, 256x256 on four waves, 192x128,
 * 288x192 on four waves; the 288x192 shape runs whole tiles only and ignores the K-split
 * threshold, the four-wave 256x256 shape hands a K-split last round to the eight-wave
 * kernel of the same tile size in a second launch; a shape whose tiles do not hold whole heads is not used for the
 * q/k/v projection, whatever is recorded) and the K-split
 * threshold in percent (0 never, 101 whenever the last round of tiles is not
 * full); cfg < 0 removes the record.  Host-side only, nothing is launched. */
int mvla_set_gemm_choice(mvla_ctx* ctx, int M, int N, int K, int epilogue, int cfg, int split_pct);
/* The recorded choice for a projection shape: *cfg_out = configuration index
 * or -1 when none is recorded, *split_pct_out its K-split threshold.
 * epilogue: 0 q/k/v, 1 attention output, 2 MLP down, 3 gate/up. */
int mvla_tuned_choice(mvla_ctx* ctx, int M, int N, int K, int epilogue, int* cfg_out,
                      int* split_pct_out);

/* Scoring pass alone, for pruning before any layer has run -- the variant in
 * which the masks go back to the encoder output and every layer sees kept tokens
 * only (Algorithm 1, last line: "return Mask_2D, Mask_3D to network encoder"):
 * RMSNorm, key projection of all rows, query projection of the last
 * n_query_tail rows only, RoPE, causal softmax (+ key_bias).  Uses the norm
 * gain and the q, k rows of w->wqkv.  Writes probs_out as above. */
int mvla_score_only(mvla_ctx* ctx, const mvla_layer_cfg* cfg, const mvla_layer_weights* w,
                    const void* x, const int32_t* pos, int B, int S, int n_query_tail,
                    const float* key_bias, float* probs_out);

/* ------------------------------------------------------------------------ */
/* Whole path                                                               */
/* ------------------------------------------------------------------------ */

/* What one pruned prefill runs (Sec. 4.4 and Algorithm 1 for the order of the
 * steps; App. C for the backbone): p layers on all S = n2 + n3 + n_text tokens,
 * the pruning step on the language-query attention of layer p-1, then the
 * remaining n_layers - p layers on the k_total + n_text kept tokens.  p = 0:
 * a scoring pass with layer 0's weights (mvla_score_only), the pruning step
 * on the input itself, then every layer on kept tokens.
 * smooth_step = t > 0 makes the call timestep t of an action-iteration episode
 * (Algorithm 1, "Action Iteration Stage"; Eqs. 8-9): the salience of the step
 * updates the smoothed state sal_hat (mvla_temporal_smooth with smooth_k,
 * smooth_beta), budget and selection read sal_hat; at t = 1 (cold start) nothing
 * is pruned: all layers run on all tokens and the state is seeded. */
typedef struct {
    int B, n2, n3, n_text;
    int k_total, min2, min3;      /* as mvla_modality_budget                            */
    int n_layers, p;
    int smooth_step, smooth_k;    /* 0 = no smoothing; paper: k = 7                     */
    double smooth_beta;           /* paper: 0.85                                        */
    int materialise_probs;        /* != 0: write the probabilities and reduce them in a
                                     second kernel; 0: reduce them inside the scoring
                                     kernel (p >= 1; p = 0 always materialises)        */
    int separate_prune_calls;     /* != 0: salience, budget, selection, gather as four
                                     launches instead of the fused ones                 */
} mvla_prefill_desc;

/* Device buffers of mvla_prefill, caller-owned, pairwise disjoint and disjoint
 * from x.  Outputs of the pruning step land in sal, k2k3, kept_idx, pos_kept
 * as the single calls define them. */
typedef struct {
    void* h_full[2];     /* bf16 [B, S, D] each: layer outputs on all tokens             */
    void* h_kept[2];     /* bf16 [B, k_total + n_text, D] each: gathered tokens, outputs  */
    float* probs;        /* fp32 [B, H, n_text, S]; may be NULL unless materialise_probs
                            or p == 0                                                     */
    float* sal;          /* fp32 [B, n2 + n3]: salience of this call                      */
    float* sal_hat;      /* fp32 [B, n2 + n3]: smoothed state (read and updated), or NULL
                            when smooth_step == 0                                         */
    int32_t* k2k3;       /* int32 [B, 2]                                                  */
    int32_t* kept_idx;   /* int32 [B, k_total + n_text]                                   */
    int32_t* pos_kept;   /* int32 [B, k_total + n_text]                                   */
} mvla_prefill_buffers;

/* Enqueue one whole pruned prefill: exactly the sequence of the calls above
 * that the description selects (no arithmetic of its own, same results as
 * issuing them one by one).  layers: HOST array of n_layers descriptors;
 * x: device bf16 [B, S, D]; pos: device int32 [B, S]; key_bias: device fp32
 * [B, S] or NULL (added to the scoring logits only).
 * *y_out (host) receives the device pointer of the final hidden states -- one
 * of the h_kept buffers, or one of the h_full buffers at a cold start -- and
 * *rows_out their rows per sample (k_total + n_text, or S).
 * Everything (description, every layer descriptor, workspace size) is checked
 * before the first launch. */
int mvla_prefill(mvla_ctx* ctx, const mvla_layer_cfg* cfg, const mvla_layer_weights* layers,
                 const mvla_prefill_desc* desc, const void* x, const int32_t* pos,
                 const float* key_bias, const mvla_prefill_buffers* buffers, void** y_out,
                 int* rows_out);

/* One action-iteration step of the paper's own mask generation (Algorithm 1,
 * all three stages; needs one 3D token per 2D token: S = 2 n_patch + n_text,
 * and p >= 1): p layers on all tokens (the p-th scores the language queries),
 * the salience and the four per-patch indicators of this step (Eq. 1 on the
 * output of layer p-1; Eqs. 5-6), their smoothing over steps (Eqs. 8-9), and
 * for t > 1 the candidate sets, fusion and masks (Sec. 4.1, 4.2, 4.4, Eq. 10),
 * the index scan, the gather, and the remaining layers on the kept tokens.
 * t = 1 is the cold start: nothing is pruned.  The kept length differs per
 * sample; rows are padded at the end up to the longest sample of the step. */
typedef struct {
    int B, n_patch, n_text, n_layers, p;
    int t;                        /* timestep, from 1                                   */
    int smooth_k;                 /* paper: 7                                           */
    double smooth_beta;           /* paper: 0.85                                        */
    mvla_mask_rules rules;
} mvla_masked_desc;

/* Device buffers of mvla_masked_prefill_step, caller-owned, pairwise disjoint. */
typedef struct {
    void* h_full[2];     /* bf16 [B, S, D] each                                          */
    void* h_kept[2];     /* bf16 [B, S, D] each (used as [B, S_pad, D])                   */
    float* probs;        /* fp32 [B, H, n_text, S]                                        */
    float* sal;          /* fp32 [B, 2 n_patch]                                           */
    float* x_t;          /* fp32 [4, B, n_patch]: this step's M2D^S1, M3D^S1, M2D^S2, M3D^S2 */
    float* x_hat;        /* fp32 [4, B, n_patch]: smoothed state, read (t > 1) and updated */
    uint8_t* mask2d;     /* uint8 [B, n_patch]                                            */
    uint8_t* mask3d;     /* uint8 [B, n_patch]                                            */
    uint8_t* sem;        /* uint8 [B, n_patch] or NULL                                    */
    int32_t* kept_len;   /* int32 [B]                                                     */
    int32_t* kept_idx;   /* int32 [B * S] (used as [B, S_pad])                            */
    int32_t* pos_kept;   /* int32 [B * S] (used as [B, S_pad])                            */
} mvla_masked_buffers;

/* Enqueue the step: exactly the sequence of the single calls above, no
 * arithmetic of its own.  u: device fp32 [B, n_patch] uniform draws of this
 * step (unused at t = 1).  For t > 1 the call copies the B kept lengths to
 * lengths_out (HOST int32 [B]) and SYNCHRONISES the stream once, because the
 * padded length S_pad = max_b length sizes the launches that follow; it cannot
 * be captured into a graph.  *y_out (host): device pointer of the final hidden
 * states, [B, *rows_out, D] with *rows_out = S_pad (S at t = 1); row i of sample
 * b is valid for i < lengths_out[b].  Everything is checked before the first
 * launch. */
int mvla_masked_prefill_step(mvla_ctx* ctx, const mvla_layer_cfg* cfg,
                             const mvla_layer_weights* layers, const mvla_masked_desc* desc,
                             const void* x, const int32_t* pos, const float* key_bias,
                             const float* u, const mvla_masked_buffers* buffers, void** y_out,
                             int* rows_out, int32_t* lengths_out);

/* ------------------------------------------------------------------------ */
/* Measurement (the paper's overhead study, Table 4, reports the pruning    */
/* method's own cost apart from the step latency; these calls give the same */
/* split per kernel)                                                        */
/* ------------------------------------------------------------------------ */

/* Bracket every launch whose kernel id bit is set in kernel_mask with a pair
 * of HIP events on the context's stream (ids: see mvla_kernel_name).  Creates
 * up to max_records event pairs on first use (host objects; no device
 * memory); further launches beyond max_records are not timed.  Mask 0 turns
 * timing off.  Discards records not yet read. */
int mvla_profile_enable(mvla_ctx* ctx, uint32_t kernel_mask, int max_records);
/* Wait for the recorded launches and copy out up to `capacity` records:
 * kernel id, tag (the launch's row count M, or batch for the pruning
 * kernels) and elapsed milliseconds; *n_out = records written.  HOST arrays.
 * Clears the record list. */
int mvla_profile_read(mvla_ctx* ctx, int capacity, int32_t* ids, int32_t* tags, float* ms,
                      int32_t* n_out);
/* Name of kernel id 0..18 ("rmsnorm", "gemm_qkv", "score_probs",
 * "attention", "gemm_o", "rmsnorm_mlp", "gemm_gateup", "gemm_down", "salience",
 * "budget", "select", "compact", "rope_table", "prune_fused", "smooth",
 * "decompose", "feature_share", "candidate_masks", "mask_indices"), "?"
 * otherwise. */
const char* mvla_kernel_name(int id);

/* Rates the device sustains on the simplest kernels, so that a kernel's time
 * can be quoted against what the part delivers as well as against its
 * datasheet.  Runs one untimed and `reps` timed launches on the context's
 * stream between two HIP events and SYNCHRONISES the stream.
 *   MVLA_PROBE_READ   streams `bytes` of buf once per launch        -> GB/s
 *   MVLA_PROBE_COPY   copies the first half of buf to the second    -> GB/s (bytes read + written)
 *   MVLA_PROBE_MFMA   every wave (four per compute unit) runs a loop of the sixteen
 *                     independent 32x32x16 bf16 products of a 128x128 register tile on
 *                     operands taken from the first 8 KiB of buf (all zeros, or random
 *                     values: the part's clock under matrix load depends on the data)
 *                                                                   -> TFLOP/s
 *   MVLA_PROBE_LAUNCH empty kernels back to back (buf unused)       -> microseconds per launch
 * buf: device, 16-byte aligned; bytes >= 1 MiB for READ/COPY, >= 8 KiB for MFMA.
 * result: HOST. */
enum { MVLA_PROBE_READ = 0, MVLA_PROBE_COPY = 1, MVLA_PROBE_MFMA = 2, MVLA_PROBE_LAUNCH = 3 };
int mvla_peak_probe(mvla_ctx* ctx, int kind, void* buf, size_t bytes, int reps, double* result);

#ifdef __cplusplus
}
#endif
#endif /* MVLA_H_ */
