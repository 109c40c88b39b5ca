// Shared host-side declarations of the gfx950 pruned-prefill library.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "mvla.h"

typedef uint16_t bf16_t;  // raw bf16 storage

#include <vector>

// per-kernel timing records (HIP events on the context's stream)
enum KernelId {
    KID_RMSNORM = 0, KID_GEMM_QKV, KID_SCORE_PROBS, KID_ATTENTION, KID_GEMM_O,
    KID_RMSNORM_MLP, KID_GEMM_GATEUP, KID_GEMM_DOWN, KID_SALIENCE, KID_BUDGET, KID_SELECT,
    KID_COMPACT, KID_ROPE_TABLE, KID_PRUNE_FUSED, KID_SMOOTH, KID_DECOMPOSE, KID_FEATURE_SHARE,
    KID_CANDIDATE, KID_MASK_INDEX, KID_COUNT
};

struct ProfRecord {
    int id, tag;
    hipEvent_t start, stop;
};

struct mvla_ctx {
    // timing (off unless mvla_profile_enable was called)
    uint32_t prof_mask = 0;
    std::vector<ProfRecord> prof_pool;  // pre-created events
    size_t prof_used = 0;
    int device;
    hipStream_t stream;
    char* ws;          // caller-owned device workspace
    size_t ws_bytes;
    // fixed areas at the head of the workspace
    uint32_t* counters;  // kCounterWords block-arrival counters (kept at zero between calls):
                         // the first half serves the salience kernel, the second the GEMMs
    float* gemm_partial; // fp32 partial tiles of K-split GEMM workgroups
    size_t gemm_partial_bytes;
    char* scratch;       // everything after the fixed areas
    size_t scratch_bytes;
    // tile configuration and K-split threshold measured fastest for a GEMM shape (mvla_tune_layers)
    struct Tuned {
        int M, N, K, epi, cfg, split_pct;
    };
    std::vector<Tuned> tuned;
};

constexpr int kMaxDevices = 64;   // per-device one-time set-up flags
constexpr int kCounterWords = 16384;
constexpr size_t kCounterBytes = size_t(kCounterWords) * 4;

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

#define MVLA_HIP_CHECK(expr)                       \
    do {                                           \
        hipError_t e_ = (expr);                    \
        if (e_ != hipSuccess) return MVLA_EHIP;    \
    } while (0)

// ---- launchers implemented in the .hip files (all enqueue on `st`) ----------
namespace mvla {

// prune_kernels.hip
size_t salience_scratch_bytes(int B, int H, int Nq, int n_vis);
int launch_salience(const float* attn, int B, int H, int Nq, int S, int n_vis, float* sal,
                    float* partial, uint32_t* counters, int mean_rows, hipStream_t st);
// salience + budget + selection in one launch (same results as the three separate launches)
int launch_prune_fused(const float* attn, int B, int H, int Nq, int S, int n2, int n3, int n_text,
                       int k_total, int min2, int min3, float* sal, int32_t* k2k3,
                       int32_t* kept_idx, float* partial, uint32_t* counters, int mean_rows,
                       hipStream_t st);
int launch_budget(const float* sal, int B, int n2, int n3, int k_total, int min2, int min3,
                  int32_t* k2k3, float* mass, hipStream_t st);
int launch_select(const float* sal, const int32_t* k2k3, int B, int n2, int n3, int n_text,
                  int k_total, int32_t* kept_idx, hipStream_t st);
int launch_compact(const bf16_t* h, const int32_t* pos, const int32_t* kept_idx, int B, int S,
                   int S_out, int D, bf16_t* h_out, int32_t* pos_out, hipStream_t st);

int launch_decompose(const float* attn, int B, int H, int Nq, int S, int n_patch, float* m2d,
                     float* m3d, hipStream_t st);
int launch_smooth(const float* x_t, float* x_hat, size_t n, int t, int k, double beta,
                  hipStream_t st);

// mask_kernels.hip
int launch_feature_share(const bf16_t* feat, int B, int S, int D, int n_patch, float* m2d,
                         float* m3d, hipStream_t st);
int launch_candidate_masks(const float* x_hat, const float* sal, const float* u, int B, int P,
                           int n_text, const mvla_mask_rules& rules, uint8_t* mask2d,
                           uint8_t* mask3d, uint8_t* sem, int32_t* kept_len, hipStream_t st);
int launch_mask_indices(const uint8_t* mask2d, const uint8_t* mask3d, int B, int P, int n_text,
                        int S_pad, int32_t* kept_idx, hipStream_t st);

// layer_kernels.hip
int launch_rmsnorm(const bf16_t* x, const bf16_t* gain, int M, int D, float eps, bf16_t* out,
                   hipStream_t st);
int launch_rmsnorm_f32(const float* x, const bf16_t* gain, int M, int D, float eps, bf16_t* out,
                       hipStream_t st);
// all B*S rows normalised into out; the last `tail` rows of each sample a second time, packed,
// into out_tail [B*tail, D], their position ids into pos_out [B*tail]
int launch_rmsnorm_tail(const bf16_t* x, const int32_t* pos, const bf16_t* gain, int B, int S,
                        int tail, int D, float eps, bf16_t* out, bf16_t* out_tail, int32_t* pos_out,
                        hipStream_t st);
int launch_rope_table(double base, int rope_len, int dh, float* c, float* s, hipStream_t st);
// scoring probabilities of the last nq rows: probs [B,H,nq,S] fp32.  q_tail_only: q holds just
// those rows, nq per sample ([B*nq, q_row_stride]); otherwise all S rows of every sample.
int launch_score_probs(const bf16_t* q, int q_row_stride, bool q_tail_only, const bf16_t* k,
                       int k_row_stride, const float* key_bias, int B, int S, int H, int dh, int nq,
                       float* out, int colsum_n, hipStream_t st);

// gemm.hip:  C[M,N] = A[M,K] * W[N,K]^T  (bf16 in, fp32 accumulate)
// EPI_QKV_ROPE: the q/k/v projection (N = 3D, or 2D for q and k alone).  Columns [0, 2D) are
// rotated by the position of their row (pairs (d, d + dh/2) of every head, cos/sin from the
// tables, in fp32 on the accumulators) and stored as bf16 into C [M, ldc]; columns [2D, 3D) are
// stored transposed into vt [B, H, dh, S_pad] (zeros in [S, S_pad)) and not into C.
// EPI_RES_BF16_TO_F32: C fp32 = acc + R(bf16).  EPI_RES_F32_TO_BF16: C bf16 = acc + R(fp32).
// EPI_SILU_MUL: C bf16 [M, N/2] = SiLU(gate) * up.
enum GemmEpilogue { EPI_QKV_ROPE = 0, EPI_RES_BF16_TO_F32 = 1, EPI_RES_F32_TO_BF16 = 2,
                    EPI_SILU_MUL = 3 };
// What EPI_QKV_ROPE needs beyond C: rows are tokens b*S + s.
struct RopeEpilogue {
    const int32_t* pos;   // [M] position ids (clamped to the table)
    const float* rc;      // [rope_len, dh/2] cos
    const float* rs;      // [rope_len, dh/2] sin
    bf16_t* vt;           // [B, H, dh, S_pad], null when N = 2D
    int rope_len, S, S_pad, D, dh;
};
// partial: fp32 scratch of gemm_partial_bytes() for K-split tiles; counters: n_counters zeroed
// arrival counters (left at zero again when the kernel ends).
size_t gemm_partial_bytes();
// compute units of the current device (256 when it cannot be asked, e.g. no device present)
int device_cu_count();
int launch_gemm(const bf16_t* A, int lda, const bf16_t* W, int M, int N, int K, void* C, int ldc,
                const void* R, int ldr, int epilogue, float* partial, size_t partial_bytes,
                uint32_t* counters, int n_counters, int force_cfg, int force_split_pct,
                const RopeEpilogue* rope, hipStream_t st);
int gemm_num_configs();
// whether tile configuration cfg can run this epilogue (the rotating one needs whole heads per tile)
bool gemm_config_runs(int cfg, int epilogue, const RopeEpilogue* rope);

// probe_kernels.hip: measurement kernels (streaming read / copy, matrix-core loop, empty launch)
int launch_probe_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t st);
int launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t st);
int launch_probe_mfma(const void* operands, int n_cu, int iters, float* sink, hipStream_t st);
int launch_probe_empty(hipStream_t st);

// attention.hip: causal flash attention; q,k rows inside qkv (row stride ldqkv), vt [B,H,dh,S_pad]
int launch_attention(const bf16_t* q, const bf16_t* k, int ldqkv, const bf16_t* vt, int S_pad,
                     int B, int S, int H, int dh, bf16_t* out, int ldo, hipStream_t st);

}  // namespace mvla
