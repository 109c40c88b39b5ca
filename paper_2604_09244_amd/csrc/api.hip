// C ABI of the pruned-prefill library: argument validation, workspace carving
// and launch sequencing.  No computation happens on the host.
#include <new>

#include "common.h"

using namespace mvla;

namespace {

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

struct LayerBuffers {
    bf16_t *u, *qkv, *vt, *attn, *act;
    float* x1;  // residual stream after attention, kept in fp32
    int S_pad;
    size_t bytes;  // total scratch needed
};

// carve the layer's intermediates out of the scratch area (base may be null: size query)
LayerBuffers layer_buffers(char* base, int B, int S, int D, int F) {
    LayerBuffers lb;
    const size_t M = (size_t)B * S;
    lb.S_pad = (S + 63) / 64 * 64;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char* p = base ? base + off : nullptr;
        off += align_up(bytes, 256);
        return reinterpret_cast<bf16_t*>(p);
    };
    lb.u = take(M * D * 2);
    lb.qkv = take(M * 3 * D * 2);
    lb.vt = take((size_t)B * D * lb.S_pad * 2);
    lb.attn = take(M * D * 2);
    lb.x1 = reinterpret_cast<float*>(take(M * D * 4));
    lb.act = take(M * F * 2);
    lb.bytes = off;
    return lb;
}

int check_layer_args(const mvla_ctx* ctx, const mvla_layer_cfg* cfg, const mvla_layer_weights* w,
                     const void* x, const int32_t* pos, int B, int S, int n_query_tail,
                     const float* probs_out, bool need_full) {
    if (!ctx || !cfg || !w || !x || !pos) return MVLA_EINVAL;
    if (B <= 0 || S <= 0) return MVLA_EINVAL;
    if (cfg->D <= 0 || cfg->H <= 0 || cfg->dh <= 0 || cfg->F <= 0) return MVLA_EINVAL;
    if (cfg->H * cfg->dh != cfg->D) return MVLA_EINVAL;
    if (cfg->dh != 64 && cfg->dh != 128) return MVLA_EUNSUPPORTED;
    if (cfg->D % 64 != 0 || cfg->F % 64 != 0 || cfg->D > 8192) return MVLA_EUNSUPPORTED;
    if (!(cfg->rms_eps >= 0.f)) return MVLA_EINVAL;
    if (!w->wqkv || !w->g_attn || !w->rope_cos || !w->rope_sin || w->rope_len <= 0)
        return MVLA_EINVAL;
    if (need_full && (!w->wo || !w->w_gateup || !w->w_down || !w->g_mlp)) return MVLA_EINVAL;
    if (!aligned(x, 16) || !aligned(w->wqkv, 16) || !aligned(w->g_attn, 16) ||
        !aligned(w->rope_cos, 16) || !aligned(w->rope_sin, 16))
        return MVLA_EINVAL;
    if (need_full && (!aligned(w->wo, 16) || !aligned(w->w_gateup, 16) ||
                      !aligned(w->w_down, 16) || !aligned(w->g_mlp, 16)))
        return MVLA_EINVAL;
    if (n_query_tail < 0 || n_query_tail > S) return MVLA_EINVAL;
    if (n_query_tail > 0 && !probs_out) return MVLA_EINVAL;
    return MVLA_OK;
}

#define GEMM_WS(ctx) (ctx)->gemm_partial, (ctx)->gemm_partial_bytes, (ctx)->counters + kCounterWords / 2, kCounterWords / 2

// measured choice for this shape, or (-1, 0): let the cost model decide
struct GemmPick {
    int cfg, split_pct;
};
GemmPick gemm_pick(const mvla_ctx* ctx, int M, int N, int K, int epi) {
    for (const auto& t : ctx->tuned)
        if (t.M == M && t.N == N && t.K == K && t.epi == epi) return {t.cfg, t.split_pct};
    return {-1, 0};
}
#define GEMM_PICK(ctx, M, N, K, epi) gemm_pick(ctx, M, N, K, epi).cfg, gemm_pick(ctx, M, N, K, epi).split_pct

// Brackets one launch with a pair of pre-created events when its kernel id is selected.
struct Timed {
    mvla_ctx* c;
    ProfRecord* r = nullptr;
    Timed(mvla_ctx* ctx, int id, int tag) : c(ctx) {
        if ((ctx->prof_mask >> id) & 1u) {
            if (ctx->prof_used < ctx->prof_pool.size()) {
                r = &ctx->prof_pool[ctx->prof_used++];
                r->id = id;
                r->tag = tag;
                (void)hipEventRecord(r->start, ctx->stream);
            }
        }
    }
    ~Timed() {
        if (r) (void)hipEventRecord(r->stop, c->stream);
    }
};
#define TIMED(ctx, id, tag, call)   \
    do {                            \
        Timed t_(ctx, id, tag);     \
        rc = (call);                \
    } while (0);                    \
    if (rc) return rc

const char* const kKernelNames[KID_COUNT] = {
    "rmsnorm", "gemm_qkv", "score_probs", "attention", "gemm_o", "rmsnorm_mlp",
    "gemm_gateup", "gemm_down", "salience", "budget", "select", "compact", "rope_table",
    "prune_fused", "smooth", "decompose", "feature_share", "candidate_masks", "mask_indices"};

}  // namespace

extern "C" {

int mvla_profile_enable(mvla_ctx* ctx, uint32_t kernel_mask, int max_records) {
    if (!ctx || max_records < 0) return MVLA_EINVAL;
    while ((int)ctx->prof_pool.size() < max_records) {
        ProfRecord r{};
        if (hipEventCreate(&r.start) != hipSuccess) return MVLA_EHIP;
        if (hipEventCreate(&r.stop) != hipSuccess) {
            (void)hipEventDestroy(r.start);
            return MVLA_EHIP;
        }
        ctx->prof_pool.push_back(r);
    }
    ctx->prof_mask = kernel_mask;
    ctx->prof_used = 0;
    return MVLA_OK;
}

int mvla_profile_read(mvla_ctx* ctx, int capacity, int32_t* ids, int32_t* tags, float* ms,
                      int32_t* n_out) {
    if (!ctx || !n_out || capacity < 0 || (capacity > 0 && (!ids || !tags || !ms)))
        return MVLA_EINVAL;
    const size_t n = ctx->prof_used < (size_t)capacity ? ctx->prof_used : (size_t)capacity;
    for (size_t i = 0; i < n; ++i) {
        ProfRecord& r = ctx->prof_pool[i];
        MVLA_HIP_CHECK(hipEventSynchronize(r.stop));
        float t = 0.f;
        MVLA_HIP_CHECK(hipEventElapsedTime(&t, r.start, r.stop));
        ids[i] = r.id;
        tags[i] = r.tag;
        ms[i] = t;
    }
    *n_out = (int32_t)n;
    ctx->prof_used = 0;
    return MVLA_OK;
}

const char* mvla_kernel_name(int id) {
    return (id >= 0 && id < KID_COUNT) ? kKernelNames[id] : "?";
}

const char* mvla_version(void) { return "0.1.0"; }

const char* mvla_strerror(int code) {
    switch (code) {
        case MVLA_OK: return "ok";
        case MVLA_EINVAL: return "invalid argument (null pointer, shape or alignment)";
        case MVLA_ENOMEM: return "workspace too small for this shape";
        case MVLA_EHIP: return "HIP runtime or launch failure";
        case MVLA_EUNSUPPORTED: return "shape not supported by the compiled kernels";
        case MVLA_ELIMIT: return "shape exceeds the fixed scratch of the allocation-free entry point";
        default: return "unknown status";
    }
}

size_t mvla_workspace_bytes(int B, int S, int D, int H, int F, int n_query_tail) {
    if (B <= 0 || S <= 0 || D <= 0 || H <= 0 || F <= 0 || n_query_tail < 0) return 0;
    const size_t sal = salience_scratch_bytes(B, H, n_query_tail > 0 ? n_query_tail : 1, S);
    const LayerBuffers lb = layer_buffers(nullptr, B, S, D, F);
    return kCounterBytes + gemm_partial_bytes() + (sal > lb.bytes ? sal : lb.bytes) + 256;
}

int mvla_create(mvla_ctx** out, int device, void* hip_stream, void* workspace,
                size_t workspace_bytes) {
    if (!out || !workspace || device < 0) return MVLA_EINVAL;
    const size_t fixed = kCounterBytes + gemm_partial_bytes();
    if (!aligned(workspace, 256) || workspace_bytes < fixed + 256) return MVLA_EINVAL;
    MVLA_HIP_CHECK(hipSetDevice(device));
    mvla_ctx* c = new (std::nothrow) mvla_ctx;
    if (!c) return MVLA_ENOMEM;
    c->device = device;
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->ws = static_cast<char*>(workspace);
    c->ws_bytes = workspace_bytes;
    c->counters = reinterpret_cast<uint32_t*>(c->ws);
    c->gemm_partial = reinterpret_cast<float*>(c->ws + kCounterBytes);
    c->gemm_partial_bytes = gemm_partial_bytes();
    c->scratch = c->ws + fixed;
    c->scratch_bytes = workspace_bytes - fixed;
    if (hipMemsetAsync(c->counters, 0, kCounterBytes, c->stream) != hipSuccess) {
        delete c;
        return MVLA_EHIP;
    }
    *out = c;
    return MVLA_OK;
}

int mvla_set_stream(mvla_ctx* ctx, void* hip_stream) {
    if (!ctx) return MVLA_EINVAL;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    return MVLA_OK;
}

void mvla_destroy(mvla_ctx* ctx) {
    if (!ctx) return;
    for (ProfRecord& r : ctx->prof_pool) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    delete ctx;
}

// ---------------------------------------------------------------------------
int mvla_salience(mvla_ctx* ctx, const float* attn, int B, int H, int Nq, int S, int n_vis,
                  float* sal) {
    if (!ctx || !attn || !sal) return MVLA_EINVAL;
    if (B <= 0 || H <= 0 || Nq <= 0 || S <= 0 || n_vis <= 0 || n_vis > S) return MVLA_EINVAL;
    if (!aligned(attn, 4) || !aligned(sal, 4)) return MVLA_EINVAL;
    if (salience_scratch_bytes(B, H, Nq, n_vis) > ctx->scratch_bytes) return MVLA_ENOMEM;
    int rc;
    TIMED(ctx, KID_SALIENCE, B, launch_salience(attn, B, H, Nq, S, n_vis, sal,
                                                reinterpret_cast<float*>(ctx->scratch),
                                                ctx->counters, 0, ctx->stream));
    return MVLA_OK;
}

int mvla_modality_budget(mvla_ctx* ctx, const float* sal, int B, int n2, int n3, int k_total,
                         int min2, int min3, int32_t* k2k3, float* mass) {
    if (!ctx || !sal || !k2k3) return MVLA_EINVAL;
    if (B <= 0 || n2 < 0 || n3 < 0 || n2 + n3 <= 0) return MVLA_EINVAL;
    if (k_total < 0 || k_total > n2 + n3) return MVLA_EINVAL;
    if (min2 < 0 || min3 < 0 || min2 > n2 || min3 > n3 || min2 + min3 > k_total)
        return MVLA_EINVAL;
    int rc;
    TIMED(ctx, KID_BUDGET, B, launch_budget(sal, B, n2, n3, k_total, min2, min3, k2k3, mass,
                                            ctx->stream));
    return MVLA_OK;
}

int mvla_select_topk(mvla_ctx* ctx, const float* sal, const int32_t* k2k3, int B, int n2, int n3,
                     int n_text, int k_total, int32_t* kept_idx) {
    if (!ctx || !sal || !k2k3 || !kept_idx) return MVLA_EINVAL;
    if (B <= 0 || n2 < 0 || n3 < 0 || n2 + n3 <= 0 || n_text < 0) return MVLA_EINVAL;
    if (k_total < 0 || k_total > n2 + n3) return MVLA_EINVAL;
    int rc;
    TIMED(ctx, KID_SELECT, B, launch_select(sal, k2k3, B, n2, n3, n_text, k_total, kept_idx,
                                            ctx->stream));
    return MVLA_OK;
}

int mvla_compact(mvla_ctx* ctx, const void* h, const int32_t* pos, const int32_t* kept_idx, int B,
                 int S, int S_out, int D, void* h_out, int32_t* pos_out) {
    if (!ctx || !h || !pos || !kept_idx || !h_out || !pos_out) return MVLA_EINVAL;
    if (B <= 0 || S <= 0 || S_out < 0 || S_out > S || D <= 0 || D % 8 != 0) return MVLA_EINVAL;
    if (!aligned(h, 16) || !aligned(h_out, 16)) return MVLA_EINVAL;
    {   // overlap check of the two hidden-state buffers
        const char* a = static_cast<const char*>(h);
        const char* b = static_cast<const char*>(h_out);
        const size_t na = (size_t)B * S * D * 2, nb = (size_t)B * S_out * D * 2;
        if (a < b + nb && b < a + na) return MVLA_EINVAL;
    }
    int rc;
    TIMED(ctx, KID_COMPACT, B * S_out,
          launch_compact(static_cast<const bf16_t*>(h), pos, kept_idx, B, S, S_out, D,
                         static_cast<bf16_t*>(h_out), pos_out, ctx->stream));
    return MVLA_OK;
}

int mvla_prune_step(mvla_ctx* ctx, const float* attn, int H, int Nq, const void* h,
                    const int32_t* pos, int B, int S, int D, int n2, int n3, int n_text,
                    int k_total, int min2, int min3, float* sal, int32_t* k2k3,
                    int32_t* kept_idx, void* h_out, int32_t* pos_out) {
    if (n2 < 0 || n3 < 0 || n_text < 0 || S != n2 + n3 + n_text) return MVLA_EINVAL;
    // validate everything before the first launch
    if (!ctx || !attn || !sal || !k2k3 || !kept_idx || !h || !pos || !h_out || !pos_out)
        return MVLA_EINVAL;
    if (B <= 0 || H <= 0 || Nq <= 0 || n2 + n3 <= 0 || D <= 0 || D % 8 != 0) return MVLA_EINVAL;
    if (k_total < 0 || k_total > n2 + n3) return MVLA_EINVAL;
    if (min2 < 0 || min3 < 0 || min2 > n2 || min3 > n3 || min2 + min3 > k_total)
        return MVLA_EINVAL;
    if (!aligned(h, 16) || !aligned(h_out, 16)) return MVLA_EINVAL;
    if (n2 > 16384 || n3 > 16384) return MVLA_EUNSUPPORTED;
    if (salience_scratch_bytes(B, H, Nq, n2 + n3) > ctx->scratch_bytes) return MVLA_ENOMEM;
    {   // overlap check of the two hidden-state buffers, before anything is launched
        const char* a = static_cast<const char*>(h);
        const char* bb = static_cast<const char*>(h_out);
        const size_t na = (size_t)B * S * D * 2, nb = (size_t)B * (k_total + n_text) * D * 2;
        if (a < bb + nb && bb < a + na) return MVLA_EINVAL;
    }
    int rc;
    TIMED(ctx, KID_PRUNE_FUSED, B,
          launch_prune_fused(attn, B, H, Nq, S, n2, n3, n_text, k_total, min2, min3, sal, k2k3,
                             kept_idx, reinterpret_cast<float*>(ctx->scratch), ctx->counters, 0,
                             ctx->stream));
    return mvla_compact(ctx, h, pos, kept_idx, B, S, k_total + n_text, D, h_out, pos_out);
}

int mvla_modality_decompose(mvla_ctx* ctx, const float* attn, int B, int H, int Nq, int S,
                            int n_patch, float* m2d, float* m3d) {
    if (!ctx || !attn || !m2d || !m3d) return MVLA_EINVAL;
    if (B <= 0 || H <= 0 || Nq <= 0 || S <= 0 || n_patch <= 0 || 2 * (long)n_patch > S)
        return MVLA_EINVAL;
    int rc;
    TIMED(ctx, KID_DECOMPOSE, B, launch_decompose(attn, B, H, Nq, S, n_patch, m2d, m3d, ctx->stream));
    return MVLA_OK;
}

int mvla_temporal_smooth(mvla_ctx* ctx, const float* x_t, float* x_hat, size_t n, int t, int k,
                         double beta) {
    if (!ctx || !x_t || !x_hat) return MVLA_EINVAL;
    if (t < 1 || k < 1 || !(beta > 0.0 && beta < 1.0)) return MVLA_EINVAL;
    int rc;
    TIMED(ctx, KID_SMOOTH, (int)(n > 0x7fffffff ? 0x7fffffff : n),
          launch_smooth(x_t, x_hat, n, t, k, beta, ctx->stream));
    return MVLA_OK;
}

int mvla_feature_share(mvla_ctx* ctx, const void* feat, int B, int S, int D, int n_patch,
                       float* m2d, float* m3d) {
    if (!ctx || !feat || !m2d || !m3d) return MVLA_EINVAL;
    if (B <= 0 || S <= 0 || D <= 0 || D % 8 != 0 || n_patch <= 0 || 2 * (long)n_patch > S)
        return MVLA_EINVAL;
    int rc;
    TIMED(ctx, KID_FEATURE_SHARE, B * n_patch,
          launch_feature_share(static_cast<const bf16_t*>(feat), B, S, D, n_patch, m2d, m3d,
                               ctx->stream));
    return MVLA_OK;
}

void mvla_mask_rules_default(mvla_mask_rules* r) {
    if (!r) return;
    r->tau_2d = 0.08f;
    r->tau_3d = 0.20f;
    r->bg_drop = 0.9f;
    r->obj_2d_min = 0.9f;
    r->obj_3d_max = 0.01f;
    r->kmeans_max_iter = 32;
}

int mvla_candidate_masks(mvla_ctx* ctx, const float* x_hat, const float* sal, const float* u, int B,
                         int n_patch, int n_text, const mvla_mask_rules* rules, uint8_t* mask2d,
                         uint8_t* mask3d, uint8_t* sem, int32_t* kept_len) {
    if (!ctx || !x_hat || !sal || !u || !rules || !mask2d || !mask3d || !kept_len)
        return MVLA_EINVAL;
    if (B <= 0 || n_patch <= 0 || n_text < 0 || rules->kmeans_max_iter < 1) return MVLA_EINVAL;
    if (!(rules->tau_2d <= rules->tau_3d) || !(rules->bg_drop >= 0.f && rules->bg_drop <= 1.f))
        return MVLA_EINVAL;
    if (n_patch > 16384) return MVLA_EUNSUPPORTED;   // scores and labels are staged in LDS
    int rc;
    TIMED(ctx, KID_CANDIDATE, B,
          launch_candidate_masks(x_hat, sal, u, B, n_patch, n_text, *rules, mask2d, mask3d, sem,
                                 kept_len, ctx->stream));
    return MVLA_OK;
}

int mvla_mask_indices(mvla_ctx* ctx, const uint8_t* mask2d, const uint8_t* mask3d, int B,
                      int n_patch, int n_text, int S_pad, int32_t* kept_idx) {
    if (!ctx || !mask2d || !mask3d || !kept_idx) return MVLA_EINVAL;
    if (B <= 0 || n_patch <= 0 || n_text < 0 || S_pad <= 0) return MVLA_EINVAL;
    int rc;
    TIMED(ctx, KID_MASK_INDEX, B,
          launch_mask_indices(mask2d, mask3d, B, n_patch, n_text, S_pad, kept_idx, ctx->stream));
    return MVLA_OK;
}

// ---------------------------------------------------------------------------
int mvla_rope_table(mvla_ctx* ctx, double base, int rope_len, int dh, float* cos_out,
                    float* sin_out) {
    if (!ctx || !cos_out || !sin_out) return MVLA_EINVAL;
    if (rope_len <= 0 || dh <= 0 || dh % 2 != 0 || !(base > 0.0)) return MVLA_EINVAL;
    int rc;
    TIMED(ctx, KID_ROPE_TABLE, rope_len,
          launch_rope_table(base, rope_len, dh, cos_out, sin_out, ctx->stream));
    return MVLA_OK;
}

// What the scoring rows of a layer are reduced to when the probabilities are not wanted:
// the salience alone, or salience + budget + selection (kept_idx != null).
struct ScoreReduce {
    int n2, n3, n_text, k_total, min2, min3;
    float* sal;
    int32_t* k2k3;
    int32_t* kept_idx;
};

static int run_layer(mvla_ctx* ctx, const mvla_layer_cfg* cfg, const mvla_layer_weights* w,
                     const void* x, const int32_t* pos, int B, int S, void* y, int n_query_tail,
                     const float* key_bias, float* probs_out, const ScoreReduce* red) {
    int rc = check_layer_args(ctx, cfg, w, x, pos, B, S, n_query_tail,
                              red ? red->sal : probs_out, true);
    if (rc) return rc;
    if (!y || !aligned(y, 16)) return MVLA_EINVAL;
    const int D = cfg->D, H = cfg->H, dh = cfg->dh, F = cfg->F;
    if ((size_t)B * S > (size_t)INT32_MAX / 4) return MVLA_EUNSUPPORTED;
    const LayerBuffers lb = layer_buffers(ctx->scratch, B, S, D, F);
    if (lb.bytes > ctx->scratch_bytes) return MVLA_ENOMEM;
    const int M = B * S;
    hipStream_t st = ctx->stream;
    const bf16_t* xin = static_cast<const bf16_t*>(x);
    const bf16_t* wqkv = static_cast<const bf16_t*>(w->wqkv);

    TIMED(ctx, KID_RMSNORM, M,
          launch_rmsnorm(xin, static_cast<const bf16_t*>(w->g_attn), M, D, cfg->rms_eps, lb.u, st));
    // q and k leave the projection rotated, v transposed (no separate pass over q/k/v)
    const RopeEpilogue rope = {pos, w->rope_cos, w->rope_sin, lb.vt, w->rope_len, S, lb.S_pad, D, dh};
    TIMED(ctx, KID_GEMM_QKV, M,
          launch_gemm(lb.u, D, wqkv, M, 3 * D, D, lb.qkv, 3 * D, nullptr, 0, EPI_QKV_ROPE,
                      GEMM_WS(ctx), GEMM_PICK(ctx, M, 3 * D, D, EPI_QKV_ROPE), &rope, st));
    if (n_query_tail > 0 && !red) {
        TIMED(ctx, KID_SCORE_PROBS, M,
              launch_score_probs(lb.qkv, 3 * D, false, lb.qkv + D, 3 * D, key_bias, B, S, H, dh,
                                 n_query_tail, probs_out, 0, st));
    } else if (n_query_tail > 0) {
        // Column sums per 32-query tile go to the (still unused) MLP activation buffer, the
        // row-split partials of their reduction to the attention output buffer.
        const int n_vis = red->n2 + red->n3, tiles = (n_query_tail + 31) / 32;
        float* colsum = reinterpret_cast<float*>(lb.act);
        if ((size_t)B * H * tiles * n_vis * 4 > (size_t)M * F * 2 ||
            salience_scratch_bytes(B, H, tiles, n_vis) > (size_t)M * D * 2)
            return MVLA_ENOMEM;
        TIMED(ctx, KID_SCORE_PROBS, M,
              launch_score_probs(lb.qkv, 3 * D, false, lb.qkv + D, 3 * D, key_bias, B, S, H, dh,
                                 n_query_tail, colsum, n_vis, st));
        if (red->kept_idx) {
            TIMED(ctx, KID_PRUNE_FUSED, B,
                  launch_prune_fused(colsum, B, H, tiles, n_vis, red->n2, red->n3, red->n_text,
                                     red->k_total, red->min2, red->min3, red->sal, red->k2k3,
                                     red->kept_idx, reinterpret_cast<float*>(lb.attn),
                                     ctx->counters, H * n_query_tail, st));
        } else {
            TIMED(ctx, KID_SALIENCE, B,
                  launch_salience(colsum, B, H, tiles, n_vis, n_vis, red->sal,
                                  reinterpret_cast<float*>(lb.attn), ctx->counters,
                                  H * n_query_tail, st));
        }
    }
    TIMED(ctx, KID_ATTENTION, M,
          launch_attention(lb.qkv, lb.qkv + D, 3 * D, lb.vt, lb.S_pad, B, S, H, dh, lb.attn, D, st));
    TIMED(ctx, KID_GEMM_O, M,
          launch_gemm(lb.attn, D, static_cast<const bf16_t*>(w->wo), M, D, D, lb.x1, D, xin, D,
                      EPI_RES_BF16_TO_F32, GEMM_WS(ctx), GEMM_PICK(ctx, M, D, D, EPI_RES_BF16_TO_F32),
                      nullptr, st));
    TIMED(ctx, KID_RMSNORM_MLP, M,
          launch_rmsnorm_f32(lb.x1, static_cast<const bf16_t*>(w->g_mlp), M, D, cfg->rms_eps, lb.u,
                             st));
    TIMED(ctx, KID_GEMM_GATEUP, M,
          launch_gemm(lb.u, D, static_cast<const bf16_t*>(w->w_gateup), M, 2 * F, D, lb.act, F,
                      nullptr, 0, EPI_SILU_MUL, GEMM_WS(ctx), GEMM_PICK(ctx, M, 2 * F, D, EPI_SILU_MUL),
                      nullptr, st));
    TIMED(ctx, KID_GEMM_DOWN, M,
          launch_gemm(lb.act, F, static_cast<const bf16_t*>(w->w_down), M, D, F, y, D, lb.x1, D,
                      EPI_RES_F32_TO_BF16, GEMM_WS(ctx), GEMM_PICK(ctx, M, D, F, EPI_RES_F32_TO_BF16),
                      nullptr, st));
    return MVLA_OK;
}

int mvla_prefill_layer(mvla_ctx* ctx, const mvla_layer_cfg* cfg, const mvla_layer_weights* w,
                       const void* x, const int32_t* pos, int B, int S, void* y, int n_query_tail,
                       const float* key_bias, float* probs_out) {
    return run_layer(ctx, cfg, w, x, pos, B, S, y, n_query_tail, key_bias, probs_out, nullptr);
}

int mvla_prefill_layer_salience(mvla_ctx* ctx, const mvla_layer_cfg* cfg,
                                const mvla_layer_weights* w, const void* x, const int32_t* pos,
                                int B, int S, void* y, int n_query_tail, const float* key_bias,
                                int n_vis, float* sal) {
    if (!sal || n_query_tail <= 0 || n_vis <= 0 || n_vis > S) return MVLA_EINVAL;
    const ScoreReduce red{n_vis, 0, 0, 0, 0, 0, sal, nullptr, nullptr};
    return run_layer(ctx, cfg, w, x, pos, B, S, y, n_query_tail, key_bias, nullptr, &red);
}

int mvla_prefill_layer_prune(mvla_ctx* ctx, const mvla_layer_cfg* cfg, const mvla_layer_weights* w,
                             const void* x, const int32_t* pos, int B, int S, void* y, int n2, int n3,
                             int n_text, int k_total, int min2, int min3, const float* key_bias,
                             float* sal, int32_t* k2k3, int32_t* kept_idx, void* h_out,
                             int32_t* pos_out) {
    if (!sal || !k2k3 || !kept_idx || !h_out || !pos_out || !y) return MVLA_EINVAL;
    if (n2 < 0 || n3 < 0 || n2 + n3 <= 0 || n_text <= 0 || (long)n2 + n3 + n_text != S)
        return MVLA_EINVAL;
    if (k_total < 0 || k_total > n2 + n3) return MVLA_EINVAL;
    if (min2 < 0 || min3 < 0 || min2 > n2 || min3 > n3 || min2 + min3 > k_total)
        return MVLA_EINVAL;
    if (n2 > 16384 || n3 > 16384) return MVLA_EUNSUPPORTED;
    if (!aligned(h_out, 16)) return MVLA_EINVAL;
    if (cfg && B > 0) {   // the gathered rows must not overlap the layer output they are read from
        const char* a = static_cast<const char*>(y);
        const char* bb = static_cast<const char*>(h_out);
        const size_t na = (size_t)B * S * cfg->D * 2, nb = (size_t)B * (k_total + n_text) * cfg->D * 2;
        if (a < bb + nb && bb < a + na) return MVLA_EINVAL;
    }
    const ScoreReduce red{n2, n3, n_text, k_total, min2, min3, sal, k2k3, kept_idx};
    int rc = run_layer(ctx, cfg, w, x, pos, B, S, y, n_text, key_bias, nullptr, &red);
    if (rc) return rc;
    return mvla_compact(ctx, y, pos, kept_idx, B, S, k_total + n_text, cfg->D, h_out, pos_out);
}

// The whole pruned prefill: sequencing only, every step is one of the calls above.
int mvla_prefill(mvla_ctx* ctx, const mvla_layer_cfg* cfg, const mvla_layer_weights* layers,
                 const mvla_prefill_desc* d, const void* x, const int32_t* pos,
                 const float* key_bias, const mvla_prefill_buffers* buf, void** y_out,
                 int* rows_out) {
    if (!ctx || !cfg || !layers || !d || !x || !pos || !buf || !y_out || !rows_out)
        return MVLA_EINVAL;
    const int B = d->B, n2 = d->n2, n3 = d->n3, nt = d->n_text, L = d->n_layers, p = d->p;
    if (B <= 0 || n2 < 0 || n3 < 0 || n2 + n3 <= 0 || nt <= 0 || L <= 0 || p < 0 || p > L)
        return MVLA_EINVAL;
    if ((long)n2 + n3 + nt > INT32_MAX / 4) return MVLA_EUNSUPPORTED;
    const int n_vis = n2 + n3, S = n_vis + nt, K = d->k_total, S_kept = K + nt;
    if (K < 0 || K > n_vis) return MVLA_EINVAL;
    if (d->min2 < 0 || d->min3 < 0 || d->min2 > n2 || d->min3 > n3 || d->min2 + d->min3 > K)
        return MVLA_EINVAL;
    if (n2 > 16384 || n3 > 16384) return MVLA_EUNSUPPORTED;
    const int t = d->smooth_step;
    if (t < 0 || (t > 0 && (d->smooth_k < 1 || !(d->smooth_beta > 0.0 && d->smooth_beta < 1.0))))
        return MVLA_EINVAL;
    const bool smoothing = t > 0, cold = t == 1;
    // the probability tensor exists only when asked for, or when there is no layer to carry
    // the scoring (pruning before any layer)
    const bool need_probs = d->materialise_probs != 0 || p == 0;
    const bool fused_layer = !need_probs && !smoothing && !d->separate_prune_calls;
    if (!buf->h_full[0] || !buf->h_full[1] || !buf->sal || !buf->k2k3 || !buf->kept_idx ||
        !buf->pos_kept || (!cold && L > p && (!buf->h_kept[0] || !buf->h_kept[1])) ||
        (!cold && L == p && !buf->h_kept[0]) || (need_probs && !buf->probs) ||
        (smoothing && !buf->sal_hat))
        return MVLA_EINVAL;
    // every layer's descriptor and the workspace are checked before the first launch
    for (int l = 0; l < L; ++l) {
        const int rc = check_layer_args(ctx, cfg, &layers[l], x, pos, B, S, 0, nullptr, true);
        if (rc) return rc;
    }
    if ((size_t)B * S > (size_t)INT32_MAX / 4) return MVLA_EUNSUPPORTED;
    if (layer_buffers(nullptr, B, S, cfg->D, cfg->F).bytes > ctx->scratch_bytes ||
        salience_scratch_bytes(B, cfg->H, nt, n_vis) > ctx->scratch_bytes)
        return MVLA_ENOMEM;

    int rc;
    const void* h = x;
    // ---- full-sequence layers 0 .. p-2, then the scoring layer (or pass) ------------------
    if (p == 0) {
        rc = mvla_score_only(ctx, cfg, &layers[0], x, pos, B, S, nt, key_bias, buf->probs);
        if (rc) return rc;
    }
    for (int l = 0; l < p; ++l) {
        void* y = buf->h_full[l & 1];
        if (l < p - 1) {
            rc = mvla_prefill_layer(ctx, cfg, &layers[l], h, pos, B, S, y, 0, nullptr, nullptr);
        } else if (need_probs) {
            rc = mvla_prefill_layer(ctx, cfg, &layers[l], h, pos, B, S, y, nt, key_bias, buf->probs);
        } else if (fused_layer && !cold) {
            rc = mvla_prefill_layer_prune(ctx, cfg, &layers[l], h, pos, B, S, y, n2, n3, nt, K,
                                          d->min2, d->min3, key_bias, buf->sal, buf->k2k3,
                                          buf->kept_idx, buf->h_kept[0], buf->pos_kept);
        } else {
            rc = mvla_prefill_layer_salience(ctx, cfg, &layers[l], h, pos, B, S, y, nt, key_bias,
                                             n_vis, buf->sal);
        }
        if (rc) return rc;
        h = y;
    }
    const bool pruned_already = p >= 1 && fused_layer && !cold;
    // ---- the pruning step (unless the scoring layer carried it) ------------------------------
    if (!pruned_already) {
        if (need_probs && !smoothing && !d->separate_prune_calls) {
            rc = mvla_prune_step(ctx, buf->probs, cfg->H, nt, h, pos, B, S, cfg->D, n2, n3, nt, K,
                                 d->min2, d->min3, buf->sal, buf->k2k3, buf->kept_idx,
                                 buf->h_kept[0], buf->pos_kept);
            if (rc) return rc;
        } else {
            if (need_probs) {
                rc = mvla_salience(ctx, buf->probs, B, cfg->H, nt, S, n_vis, buf->sal);
                if (rc) return rc;
            }
            const float* score = buf->sal;
            if (smoothing) {   // Eqs. 8-9: selection reads the smoothed state in place
                rc = mvla_temporal_smooth(ctx, buf->sal, buf->sal_hat, (size_t)B * n_vis, t,
                                          d->smooth_k, d->smooth_beta);
                if (rc) return rc;
                score = buf->sal_hat;
            }
            if (!cold) {
                rc = mvla_modality_budget(ctx, score, B, n2, n3, K, d->min2, d->min3, buf->k2k3,
                                          nullptr);
                if (rc) return rc;
                rc = mvla_select_topk(ctx, score, buf->k2k3, B, n2, n3, nt, K, buf->kept_idx);
                if (rc) return rc;
                rc = mvla_compact(ctx, h, pos, buf->kept_idx, B, S, S_kept, cfg->D, buf->h_kept[0],
                                  buf->pos_kept);
                if (rc) return rc;
            }
        }
    }
    // ---- remaining layers: on every token at the cold start, else on the kept tokens --------
    if (cold) {
        for (int l = p; l < L; ++l) {
            void* y = buf->h_full[l & 1];
            rc = mvla_prefill_layer(ctx, cfg, &layers[l], h, pos, B, S, y, 0, nullptr, nullptr);
            if (rc) return rc;
            h = y;
        }
        *y_out = const_cast<void*>(h);
        *rows_out = S;
        return MVLA_OK;
    }
    h = buf->h_kept[0];
    for (int l = p; l < L; ++l) {
        void* y = buf->h_kept[(l - p + 1) & 1];
        rc = mvla_prefill_layer(ctx, cfg, &layers[l], h, buf->pos_kept, B, S_kept, y, 0, nullptr,
                                nullptr);
        if (rc) return rc;
        h = y;
    }
    *y_out = const_cast<void*>(h);
    *rows_out = S_kept;
    return MVLA_OK;
}

// One action-iteration step with the masks of Algorithm 1: sequencing only.
int mvla_masked_prefill_step(mvla_ctx* ctx, const mvla_layer_cfg* cfg,
                             const mvla_layer_weights* layers, const mvla_masked_desc* d,
                             const void* x, const int32_t* pos, const float* key_bias,
                             const float* u, const mvla_masked_buffers* buf, void** y_out,
                             int* rows_out, int32_t* lengths_out) {
    if (!ctx || !cfg || !layers || !d || !x || !pos || !buf || !y_out || !rows_out || !lengths_out)
        return MVLA_EINVAL;
    const int B = d->B, P = d->n_patch, nt = d->n_text, L = d->n_layers, p = d->p, t = d->t;
    if (B <= 0 || P <= 0 || nt <= 0 || L <= 0 || p < 1 || p > L || t < 1) return MVLA_EINVAL;
    if (P > 16384) return MVLA_EUNSUPPORTED;
    if ((long)2 * P + nt > INT32_MAX / 4) return MVLA_EUNSUPPORTED;
    if (d->smooth_k < 1 || !(d->smooth_beta > 0.0 && d->smooth_beta < 1.0)) return MVLA_EINVAL;
    if (d->rules.kmeans_max_iter < 1 || !(d->rules.tau_2d <= d->rules.tau_3d) ||
        !(d->rules.bg_drop >= 0.f && d->rules.bg_drop <= 1.f))
        return MVLA_EINVAL;
    const int S = 2 * P + nt;
    if (!buf->h_full[0] || !buf->h_full[1] || !buf->probs || !buf->sal || !buf->x_t || !buf->x_hat)
        return MVLA_EINVAL;
    if (t > 1 && (!u || !buf->h_kept[0] || !buf->h_kept[1] || !buf->mask2d || !buf->mask3d ||
                  !buf->kept_len || !buf->kept_idx || !buf->pos_kept))
        return MVLA_EINVAL;
    for (int l = 0; l < L; ++l) {
        const int rc = check_layer_args(ctx, cfg, &layers[l], x, pos, B, S, 0, nullptr, true);
        if (rc) return rc;
    }
    if ((size_t)B * S > (size_t)INT32_MAX / 4) return MVLA_EUNSUPPORTED;
    if (layer_buffers(nullptr, B, S, cfg->D, cfg->F).bytes > ctx->scratch_bytes ||
        salience_scratch_bytes(B, cfg->H, nt, 2 * P) > ctx->scratch_bytes)
        return MVLA_ENOMEM;

    int rc;
    const void* h = x;
    for (int l = 0; l < p; ++l) {
        void* y = buf->h_full[l & 1];
        const bool score = l == p - 1;
        rc = mvla_prefill_layer(ctx, cfg, &layers[l], h, pos, B, S, y, score ? nt : 0,
                                score ? key_bias : nullptr, score ? buf->probs : nullptr);
        if (rc) return rc;
        h = y;
    }
    // the four per-patch indicators of this step (Eq. 1 on the output of layer p-1, Eqs. 5-6 on
    // its language-query attention) and their smoothing (Eqs. 8-9)
    const size_t BP = (size_t)B * P;
    rc = mvla_salience(ctx, buf->probs, B, cfg->H, nt, S, 2 * P, buf->sal);
    if (rc) return rc;
    rc = mvla_feature_share(ctx, h, B, S, cfg->D, P, buf->x_t, buf->x_t + BP);
    if (rc) return rc;
    rc = mvla_modality_decompose(ctx, buf->probs, B, cfg->H, nt, S, P, buf->x_t + 2 * BP,
                                 buf->x_t + 3 * BP);
    if (rc) return rc;
    rc = mvla_temporal_smooth(ctx, buf->x_t, buf->x_hat, 4 * BP, t, d->smooth_k, d->smooth_beta);
    if (rc) return rc;
    if (t == 1) {   // cold start: every token goes through every layer
        for (int l = p; l < L; ++l) {
            void* y = buf->h_full[l & 1];
            rc = mvla_prefill_layer(ctx, cfg, &layers[l], h, pos, B, S, y, 0, nullptr, nullptr);
            if (rc) return rc;
            h = y;
        }
        for (int b = 0; b < B; ++b) lengths_out[b] = S;
        *y_out = const_cast<void*>(h);
        *rows_out = S;
        return MVLA_OK;
    }
    rc = mvla_candidate_masks(ctx, buf->x_hat, buf->sal, u, B, P, nt, &d->rules, buf->mask2d,
                              buf->mask3d, buf->sem, buf->kept_len);
    if (rc) return rc;
    // the kept length differs per sample: the one read-back of the step sizes the later launches
    MVLA_HIP_CHECK(hipMemcpyAsync(lengths_out, buf->kept_len, (size_t)B * sizeof(int32_t),
                                  hipMemcpyDeviceToHost, ctx->stream));
    MVLA_HIP_CHECK(hipStreamSynchronize(ctx->stream));
    int S_pad = 0;
    for (int b = 0; b < B; ++b) S_pad = lengths_out[b] > S_pad ? lengths_out[b] : S_pad;
    if (S_pad <= 0 || S_pad > S) return MVLA_EHIP;   // (every sample keeps its language tokens)
    rc = mvla_mask_indices(ctx, buf->mask2d, buf->mask3d, B, P, nt, S_pad, buf->kept_idx);
    if (rc) return rc;
    rc = mvla_compact(ctx, h, pos, buf->kept_idx, B, S, S_pad, cfg->D, buf->h_kept[0], buf->pos_kept);
    if (rc) return rc;
    h = buf->h_kept[0];
    for (int l = p; l < L; ++l) {
        void* y = buf->h_kept[(l - p + 1) & 1];
        rc = mvla_prefill_layer(ctx, cfg, &layers[l], h, buf->pos_kept, B, S_pad, y, 0, nullptr, nullptr);
        if (rc) return rc;
        h = y;
    }
    *y_out = const_cast<void*>(h);
    *rows_out = S_pad;
    return MVLA_OK;
}

int mvla_tune_layers(mvla_ctx* ctx, const mvla_layer_cfg* cfg, const mvla_layer_weights* layers,
                     int n_layers, int B, int S) {
    if (!ctx || !cfg || !layers || n_layers <= 0 || B <= 0 || S <= 0) return MVLA_EINVAL;
    for (int l = 0; l < n_layers; ++l) {
        static const int32_t dummy_pos = 0;
        int rc = check_layer_args(ctx, cfg, &layers[l], layers[l].wqkv, &dummy_pos, B, S, 0, nullptr,
                                  true);
        if (rc) return rc;
    }
    if ((size_t)B * S > (size_t)INT32_MAX / 4) return MVLA_EUNSUPPORTED;
    const int D = cfg->D, F = cfg->F, M = B * S;
    const LayerBuffers lb = layer_buffers(ctx->scratch, B, S, D, F);
    if (lb.bytes > ctx->scratch_bytes) return MVLA_ENOMEM;
    hipStream_t st = ctx->stream;
    // operands of the timed launches: zeros (timing does not depend on the values)
    MVLA_HIP_CHECK(hipMemsetAsync(lb.u, 0, (size_t)M * D * 2, st));
    MVLA_HIP_CHECK(hipMemsetAsync(lb.attn, 0, (size_t)M * D * 2, st));
    MVLA_HIP_CHECK(hipMemsetAsync(lb.x1, 0, (size_t)M * D * 4, st));
    MVLA_HIP_CHECK(hipMemsetAsync(lb.act, 0, (size_t)M * F * 2, st));
    hipEvent_t e0, e1;
    MVLA_HIP_CHECK(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return MVLA_EHIP;
    }
    struct Job {
        const bf16_t* A;
        int lda, N, K;
        void* C;
        int ldc;
        const void* R;
        int ldr, epi, which;
    };
    // the down projection writes into the (unused) q/k/v buffer instead of a layer output
    const Job jobs[4] = {
        {lb.u, D, 3 * D, D, lb.qkv, 3 * D, nullptr, 0, EPI_QKV_ROPE, 0},
        {lb.attn, D, D, D, lb.x1, D, lb.u, D, EPI_RES_BF16_TO_F32, 1},
        {lb.u, D, 2 * F, D, lb.act, F, nullptr, 0, EPI_SILU_MUL, 2},
        {lb.act, F, D, F, lb.qkv, D, lb.x1, D, EPI_RES_F32_TO_BF16, 3},
    };
    const int reps = n_layers < 4 ? 4 : (n_layers > 8 ? 8 : n_layers);
    static const int kSplitChoices[3] = {0, 50, 101};
    int rc = MVLA_OK;
    mvla_ctx::Tuned found_best[4];   // recorded in the context only when all four jobs succeeded
    int n_found = 0;
    for (const Job& j : jobs) {
        float best_ms = 0.f;
        int best_cfg = -1, best_pct = 0;
        for (int c = 0; c < gemm_num_configs() && rc == MVLA_OK; ++c)
            for (int sp = 0; sp < 3 && rc == MVLA_OK; ++sp) {
                // position ids of the timed q/k/v launches: the zeros of the attention buffer
                const RopeEpilogue rope = {reinterpret_cast<const int32_t*>(lb.attn), layers[0].rope_cos,
                                           layers[0].rope_sin, lb.vt, layers[0].rope_len, S, lb.S_pad,
                                           D, cfg->dh};
                if (!gemm_config_runs(c, j.epi, &rope)) continue;
                float ms = 0.f;
                for (int pass = 0; pass < 2 && rc == MVLA_OK; ++pass) {   // the better of two timings
                    for (int r = (pass == 0 ? -1 : 0); r < reps; ++r) {   // r == -1: untimed first launch
                        if (r == 0 && hipEventRecord(e0, st) != hipSuccess) rc = MVLA_EHIP;
                        const mvla_layer_weights& w = layers[(r + n_layers) % n_layers];
                        const void* wt = j.which == 0 ? w.wqkv : j.which == 1 ? w.wo
                                         : j.which == 2 ? w.w_gateup : w.w_down;
                        const int lrc = launch_gemm(j.A, j.lda, static_cast<const bf16_t*>(wt), M, j.N,
                                                    j.K, j.C, j.ldc, j.R, j.ldr, j.epi, GEMM_WS(ctx), c,
                                                    kSplitChoices[sp],
                                                    j.epi == EPI_QKV_ROPE ? &rope : nullptr, st);
                        if (lrc) rc = lrc;   // (configurations that cannot run were skipped above)
                    }
                    float t = 0.f;
                    if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                        hipEventElapsedTime(&t, e0, e1) != hipSuccess)
                        rc = MVLA_EHIP;
                    if (pass == 0 || t < ms) ms = t;
                }
                if (rc == MVLA_OK && (best_cfg < 0 || ms < best_ms)) {
                    best_ms = ms;
                    best_cfg = c;
                    best_pct = kSplitChoices[sp];
                }
            }
        if (rc != MVLA_OK || best_cfg < 0) {
            if (rc == MVLA_OK) rc = MVLA_EUNSUPPORTED;   // no configuration runs this shape
            break;
        }
        found_best[n_found++] = {M, j.N, j.K, j.epi, best_cfg, best_pct};
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != MVLA_OK) return rc;
    for (int i = 0; i < n_found; ++i)
        (void)mvla_set_gemm_choice(ctx, found_best[i].M, found_best[i].N, found_best[i].K,
                                   found_best[i].epi, found_best[i].cfg, found_best[i].split_pct);
    return MVLA_OK;
}

int mvla_set_gemm_choice(mvla_ctx* ctx, int M, int N, int K, int epilogue, int cfg, int split_pct) {
    if (!ctx || M <= 0 || N <= 0 || K <= 0 || epilogue < 0 || epilogue > 3) return MVLA_EINVAL;
    if (cfg >= gemm_num_configs() || split_pct < 0 || split_pct > 101) return MVLA_EINVAL;
    for (size_t i = 0; i < ctx->tuned.size(); ++i) {
        auto& t = ctx->tuned[i];
        if (t.M == M && t.N == N && t.K == K && t.epi == epilogue) {
            if (cfg < 0) {
                ctx->tuned.erase(ctx->tuned.begin() + (long)i);
            } else {
                t.cfg = cfg;
                t.split_pct = split_pct;
            }
            return MVLA_OK;
        }
    }
    if (cfg >= 0) ctx->tuned.push_back({M, N, K, epilogue, cfg, split_pct});
    return MVLA_OK;
}

int mvla_tuned_choice(mvla_ctx* ctx, int M, int N, int K, int epilogue, int* cfg_out,
                      int* split_pct_out) {
    if (!ctx || !cfg_out || !split_pct_out) return MVLA_EINVAL;
    const GemmPick p = gemm_pick(ctx, M, N, K, epilogue);
    *cfg_out = p.cfg;
    *split_pct_out = p.split_pct;
    return MVLA_OK;
}

int mvla_peak_probe(mvla_ctx* ctx, int kind, void* buf, size_t bytes, int reps, double* result) {
    if (!ctx || !result || reps <= 0 || kind < 0 || kind > 3) return MVLA_EINVAL;
    if (kind != MVLA_PROBE_LAUNCH && (!buf || !aligned(buf, 16))) return MVLA_EINVAL;
    if ((kind == MVLA_PROBE_READ || kind == MVLA_PROBE_COPY) && bytes < (1u << 20)) return MVLA_EINVAL;
    if (kind == MVLA_PROBE_MFMA && bytes < 8192) return MVLA_EINVAL;
    hipStream_t st = ctx->stream;
    const int n_cu = device_cu_count();
    const int mfma_iters = 4096;
    const size_t half = (bytes / 2) & ~(size_t)255;
    auto launch = [&]() -> int {
        switch (kind) {
            case MVLA_PROBE_READ: return launch_probe_read(buf, bytes & ~(size_t)15, nullptr, st);
            case MVLA_PROBE_COPY: return launch_probe_copy(buf, static_cast<char*>(buf) + half, half, st);
            case MVLA_PROBE_MFMA: return launch_probe_mfma(buf, n_cu, mfma_iters, nullptr, st);
            default: return launch_probe_empty(st);
        }
    };
    int rc = launch();   // untimed first launch
    if (rc) return rc;
    hipEvent_t e0, e1;
    MVLA_HIP_CHECK(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return MVLA_EHIP;
    }
    float ms = 0.f;
    if (hipEventRecord(e0, st) != hipSuccess) rc = MVLA_EHIP;
    for (int r = 0; r < reps && rc == MVLA_OK; ++r) rc = launch();
    if (rc == MVLA_OK && (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                          hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
        rc = MVLA_EHIP;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc) return rc;
    const double sec = (double)ms * 1e-3 / reps;
    switch (kind) {
        case MVLA_PROBE_READ: *result = (double)(bytes & ~(size_t)15) / sec * 1e-9; break;
        case MVLA_PROBE_COPY: *result = 2.0 * (double)half / sec * 1e-9; break;
        case MVLA_PROBE_MFMA:
            // per wave and iteration: 16 products of 32 x 32 x 16, two flops per multiply-add
            *result = (double)n_cu * 4 * mfma_iters * 16 * (2.0 * 32 * 32 * 16) / sec * 1e-12;
            break;
        default: *result = sec * 1e6; break;
    }
    return MVLA_OK;
}

int mvla_score_only(mvla_ctx* ctx, const mvla_layer_cfg* cfg, const mvla_layer_weights* w,
                    const void* x, const int32_t* pos, int B, int S, int n_query_tail,
                    const float* key_bias, float* probs_out) {
    int rc = check_layer_args(ctx, cfg, w, x, pos, B, S, n_query_tail, probs_out, false);
    if (rc) return rc;
    if (n_query_tail <= 0) return MVLA_EINVAL;
    const int D = cfg->D, H = cfg->H, dh = cfg->dh;
    if ((size_t)B * S > (size_t)INT32_MAX / 4) return MVLA_EUNSUPPORTED;
    const LayerBuffers lb = layer_buffers(ctx->scratch, B, S, D, cfg->F);
    if (lb.bytes > ctx->scratch_bytes) return MVLA_ENOMEM;
    const int M = B * S;
    hipStream_t st = ctx->stream;
    // Keys of every row: the key rows of wqkv on the normalised input, rotated, into the k
    // buffer [M, D].  Queries of the scoring rows only: the norm kernel writes those rows a
    // second time into a compact [B*n_query_tail, D] matrix (with their position ids beside it),
    // which is projected with the query rows of wqkv and rotated; the scoring kernel reads that
    // compact q.
    const bf16_t* wqkv = static_cast<const bf16_t*>(w->wqkv);
    const int Mq = B * n_query_tail;
    bf16_t* k_buf = lb.qkv;                       // [M, D]
    bf16_t* q_buf = lb.qkv + (size_t)M * D;       // [Mq, D]
    bf16_t* u_tail = lb.attn;                     // [Mq, D]  (attention output buffer, unused here)
    int32_t* pos_tail = reinterpret_cast<int32_t*>(lb.x1);   // [Mq]
    TIMED(ctx, KID_RMSNORM, M,
          launch_rmsnorm_tail(static_cast<const bf16_t*>(x), pos, static_cast<const bf16_t*>(w->g_attn),
                              B, S, n_query_tail, D, cfg->rms_eps, lb.u, u_tail, pos_tail, st));
    const RopeEpilogue rope_k = {pos, w->rope_cos, w->rope_sin, nullptr, w->rope_len, S, lb.S_pad, D, dh};
    TIMED(ctx, KID_GEMM_QKV, M,
          launch_gemm(lb.u, D, wqkv + (size_t)D * D, M, D, D, k_buf, D, nullptr, 0, EPI_QKV_ROPE,
                      GEMM_WS(ctx), GEMM_PICK(ctx, M, D, D, EPI_QKV_ROPE), &rope_k, st));
    const int nq_pad = (n_query_tail + 7) / 8 * 8;
    const RopeEpilogue rope_q = {pos_tail, w->rope_cos, w->rope_sin, nullptr, w->rope_len,
                                 n_query_tail, nq_pad, D, dh};
    TIMED(ctx, KID_GEMM_QKV, Mq,
          launch_gemm(u_tail, D, wqkv, Mq, D, D, q_buf, D, nullptr, 0, EPI_QKV_ROPE, GEMM_WS(ctx),
                      GEMM_PICK(ctx, Mq, D, D, EPI_QKV_ROPE), &rope_q, st));
    TIMED(ctx, KID_SCORE_PROBS, M,
          launch_score_probs(q_buf, D, true, k_buf, D, key_bias, B, S, H, dh, n_query_tail,
                             probs_out, 0, st));
    return MVLA_OK;
}

}  // extern "C"
