"""Plain, slow, fp64 numpy oracle of the pruned-prefill hot path.

TEST INFRASTRUCTURE ONLY -- never imported by the product package.

What is modelled (paper: "2D or 3D: Who Governs Salience in VLA Models?"):

* The backbone is a LLaMA-2 7B decoder stack over the concatenation
  [2D tokens | 3D tokens | language tokens] (Sec. 5.1 Setup; App. C "MVLA
  Models").  The paper only names the backbone, so the layer below is the
  public LLaMA-2 decoder layer: RMSNorm, rotary embedding (rotate-half
  pairing), causal multi-head attention, SiLU-gated MLP, no biases.
* Attention-score salience: the attention matrix is partitioned by token
  modality and every visual token is scored by the L1 norm of its attention
  column (Sec. 3.2, Eq. 3; the same norms enter Eq. 5).  Probabilities are
  non-negative, so the L1 norm is a plain sum; "avg" is read as the mean over
  the (head, text-query) rows.
* Modality mass ratio M^{S2}_{2D} = |a_2D|_1 / (|a_2D|_1 + |a_3D|_1)  (Eq. 5),
  the same normalised form as Eq. 1, used to split one keep budget into
  per-modality budgets (Sec. 5.2: different pruning rates for 2D and 3D).
* Selection: per modality keep the K_m highest-salience tokens, lower index
  wins ties, kept indices ascending.  This replaces the mask generation of
  Algorithm 1 by an exact budget; the mask semantics stay those of Eq. 10 /
  Sec. 4.4: kept tokens go on to the later layers, the rest are discarded.
* Temporal smoothing of an indicator (Sec. 4.3/4.4, Eqs. 7-9, Algorithm 1
  "Action Iteration Stage").
* The mask generation of Algorithm 1 itself (dual threshold on the per-patch
  feature share of Eq. 1, 1-D k-means into background / robot / object,
  the semantic rules with their two baselines, intersection fusion with the
  conflict fallback, Eq. 10), for inputs with one 3D token per 2D token.
  The random draws of the background rule are an input.

Every reduction is carried in float64.  Inputs are whatever values the caller
hands over (for bf16 workloads: the bf16-rounded values widened to float64);
nothing is rounded in between.

Pins (tests/test_oracle_pins.py): brute-force subset enumeration and
torch.topk for selection; closed forms for salience, budget, RMSNorm, RoPE,
EMA; a loop-written O(n^2) attention and torch's scaled_dot_product_attention;
an independently written torch-CPU decoder layer; keep-100% == unpruned;
scikit-learn's Lloyd iteration from the same start, well-separated clusters
and the fixed-point property for the k-means; hand-derived rule tables for the
candidate sets and their fusion.
End-to-end selection *quality* against the paper's success rates and measured
per-modality pruning rates is parity unpinned (needs the simulator and the
model checkpoint).
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "rmsnorm", "rope_rotate_half", "attention_probs", "decoder_layer",
    "score_only", "salience", "modality_budget", "select_topk", "compact",
    "keep_count", "pruned_prefill", "ema_indicator", "modality_decompose",
    "feature_share", "kmeans_1d", "candidate_masks", "mask_indices", "patch_score",
    "masked_prefill", "SEM_BG", "SEM_ROB", "SEM_OBJ",
]

F64 = np.float64


# --------------------------------------------------------------------------
# Backbone layer (App. C: LLaMA-2 7B backbone; public LLaMA-2 layer maths)
# --------------------------------------------------------------------------
def rmsnorm(x, gain, eps):
    """u_i = x_i * gain_i / sqrt(mean_j(x_j^2) + eps), over the last axis."""
    x = np.asarray(x, F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gain, F64)


def rope_rotate_half(t, pos, base=10000.0):
    """Rotary embedding with rotate-half pairing.

    t: [S, H, dh]; pos: [S] integer position ids.  Element i of the first half
    is paired with element i + dh/2; the pair is rotated by the angle
    pos * base**(-2 i / dh).
    """
    t = np.asarray(t, F64)
    S, H, dh = t.shape
    half = dh // 2
    inv_freq = base ** (-2.0 * np.arange(half, dtype=F64) / dh)
    ang = np.asarray(pos, F64)[:, None] * inv_freq[None, :]      # [S, half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    a = t[..., :half]
    b = t[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def attention_probs(q, k, causal=True, key_bias=None, q_row0=0):
    """Row-softmax attention probabilities for one sample.

    q: [Sq, H, dh] (rows q_row0 .. q_row0+Sq-1 of the sequence), k: [S, H, dh].
    logits[h, i, j] = q_i . k_j / sqrt(dh) (+ key_bias[j]); with `causal`,
    query row r only sees keys j <= r.  Returns [H, Sq, S].
    """
    q = np.asarray(q, F64)
    k = np.asarray(k, F64)
    Sq, H, dh = q.shape
    S = k.shape[0]
    # logits[h] = q[:, h, :] @ k[:, h, :].T
    logits = np.matmul(q.transpose(1, 0, 2), k.transpose(1, 2, 0)) / np.sqrt(F64(dh))
    if key_bias is not None:
        logits = logits + np.asarray(key_bias, F64)[None, None, :]
    if causal:
        rows = q_row0 + np.arange(Sq)[:, None]
        cols = np.arange(S)[None, :]
        logits = np.where(cols <= rows, logits, -np.inf)
    m = np.max(logits, axis=-1, keepdims=True)
    e = np.exp(logits - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def _silu(z):
    return z / (1.0 + np.exp(-z))


def _qk(x, pos, w, H, eps, base, rows=None):
    """Normalised input -> rotated q (optionally only `rows`) and k, plus u."""
    u = rmsnorm(x, w["g_attn"], eps)
    S, D = u.shape
    dh = D // H
    uq = u if rows is None else u[rows]
    pq = pos if rows is None else np.asarray(pos)[rows]
    q = (uq @ np.asarray(w["wq"], F64).T).reshape(-1, H, dh)
    k = (u @ np.asarray(w["wk"], F64).T).reshape(S, H, dh)
    return rope_rotate_half(q, pq, base), rope_rotate_half(k, pos, base), u


def decoder_layer(x, pos, w, H, eps=1e-5, base=10000.0, n_query_tail=0,
                  key_bias=None):
    """One LLaMA-2 decoder layer on one sample.

    x: [S, D]; pos: [S]; w: dict of wq, wk, wv, wo [D, D], w_gate, w_up [F, D],
    w_down [D, F] -- all stored [out_features, in_features] so a projection is
    x @ W.T -- and RMSNorm gains g_attn, g_mlp [D].

    Returns (y, probs): y [S, D]; probs [H, n_query_tail, S] are the attention
    probabilities of the last n_query_tail rows (the language-token queries),
    with `key_bias` added to *those* logits only (the layer's own attention is
    never biased), or None when n_query_tail == 0.
    """
    x = np.asarray(x, F64)
    S, D = x.shape
    dh = D // H
    q, k, u = _qk(x, pos, w, H, eps, base)
    v = (u @ np.asarray(w["wv"], F64).T).reshape(S, H, dh)
    A = attention_probs(q, k, causal=True)                        # [H, S, S]
    o = np.matmul(A, v.transpose(1, 0, 2)).transpose(1, 0, 2).reshape(S, D)
    x1 = x + o @ np.asarray(w["wo"], F64).T
    t = rmsnorm(x1, w["g_mlp"], eps)
    gate = t @ np.asarray(w["w_gate"], F64).T
    up = t @ np.asarray(w["w_up"], F64).T
    y = x1 + (_silu(gate) * up) @ np.asarray(w["w_down"], F64).T
    probs = None
    if n_query_tail > 0:
        r0 = S - n_query_tail
        probs = attention_probs(q[r0:], k, causal=True, key_bias=key_bias,
                                q_row0=r0)
    return y, probs


def score_only(x, pos, w, H, n_query_tail, eps=1e-5, base=10000.0,
               key_bias=None):
    """Scoring pass when pruning happens before any layer has run: the first
    layer's norm, q (tail rows) and k projections, RoPE and causal softmax --
    nothing else.  Returns [H, n_query_tail, S]."""
    x = np.asarray(x, F64)
    S = x.shape[0]
    r0 = S - n_query_tail
    q, k, _ = _qk(x, pos, w, H, eps, base, rows=np.arange(r0, S))
    return attention_probs(q, k, causal=True, key_bias=key_bias, q_row0=r0)


# --------------------------------------------------------------------------
# Pruning step
# --------------------------------------------------------------------------
def salience(probs, n_vis):
    """Attention-score salience of every visual token (Sec. 3.2, Eq. 3).

    probs: [B, H, Nq, S] row-softmaxed attention of the language-token
    queries.  sal[b, j] = mean over (h, q) of probs[b, h, q, j], j < n_vis:
    the L1 norm of token j's attention column, averaged over the rows.
    """
    p = np.asarray(probs, F64)
    B, H, Nq, S = p.shape
    return np.sum(p[:, :, :, :n_vis], axis=(1, 2)) / F64(H * Nq)


def keep_count(keep_permille, n_vis):
    """K = round-half-up(keep * n_vis) in integers (keep given in 1/1000)."""
    return (int(keep_permille) * int(n_vis) + 500) // 1000


def modality_budget(sal, n2, n3, k_total, min2=0, min3=0):
    """Split k_total between the 2D and 3D segments by salience mass (Eq. 5).

    sal: [B, n2+n3].  m2 = sum(sal[:n2]) / sum(sal);  K2 = floor(K*m2 + 1/2),
    clamped to [max(min2, K-n3), min(n2, K-min3)];  K3 = K - K2.  A sample
    with zero total mass falls back to m2 = n2 / (n2+n3).
    Returns (k2k3 int32 [B,2], mass float64 [B,2]).
    """
    s = np.asarray(sal, F64)
    B = s.shape[0]
    assert s.shape[1] == n2 + n3 and 0 <= k_total <= n2 + n3
    assert min2 + min3 <= k_total or k_total == 0
    k2k3 = np.zeros((B, 2), np.int32)
    mass = np.zeros((B, 2), F64)
    for b in range(B):
        a2 = np.sum(s[b, :n2])
        a3 = np.sum(s[b, n2:])
        m2 = a2 / (a2 + a3) if (a2 + a3) > 0.0 else F64(n2) / F64(n2 + n3)
        k2 = int(np.floor(k_total * m2 + 0.5))
        lo = max(min2, k_total - n3)
        hi = min(n2, k_total - min3)
        k2 = min(max(k2, lo), hi)
        k2k3[b] = (k2, k_total - k2)
        mass[b] = (m2, 1.0 - m2)
    return k2k3, mass


def select_topk(sal, k2k3, n2, n3, n_text):
    """Per-modality top-k with lower-index-wins ties, output ascending.

    The definition is written out literally: in each modality segment order
    the tokens by (salience descending, index ascending) with a stable sort,
    take the first K_m, then list the taken indices in ascending order.  All
    n_text language tokens follow (never pruned; Eq. 10 defines masks for the
    two visual modalities only).  Returns int32 [B, K2+K3+n_text].
    """
    s = np.asarray(sal)
    B = s.shape[0]
    assert not np.any(np.isnan(s)) and not np.any(np.isinf(s))
    rows = []
    for b in range(B):
        k2, k3 = int(k2k3[b][0]), int(k2k3[b][1])
        keep = []
        for start, n, k in ((0, n2, k2), (n2, n3, k3)):
            seg = s[b, start:start + n]
            order = np.argsort(-seg, kind="stable")     # ties keep index order
            keep.append(np.sort(order[:k]) + start)
        keep.append(np.arange(n2 + n3, n2 + n3 + n_text))
        rows.append(np.concatenate(keep))
    return np.stack(rows).astype(np.int32)


def compact(h, pos, kept_idx):
    """h'[b,i,:] = h[b, kept_idx[b,i], :],  pos'[b,i] = pos[b, kept_idx[b,i]]
    (Sec. 4.4: tokens with mask 1 proceed, tokens with mask 0 are dropped)."""
    h = np.asarray(h)
    pos = np.asarray(pos)
    B = h.shape[0]
    ho = np.stack([h[b, kept_idx[b]] for b in range(B)])
    po = np.stack([pos[b, kept_idx[b]] for b in range(B)])
    return ho, po


def pruned_prefill(x, pos, layers, H, n2, n3, n_text, k_total, p,
                   eps=1e-5, base=10000.0, key_bias=None, min2=0, min3=0):
    """Whole path on a batch: p layers on all S tokens (the last of them, or a
    scoring pass when p == 0, yields the language-query probabilities), the
    pruning step, then the remaining layers on the kept tokens with their
    original position ids.

    x: [B, S, D]; pos: [B, S]; layers: list of weight dicts.
    Returns dict(y, pos, kept_idx, k2k3, sal, probs).
    """
    x = np.asarray(x, F64)
    B, S, D = x.shape
    n_vis = n2 + n3
    assert S == n_vis + n_text
    h = x.copy()
    probs = [None] * B
    for li in range(p):
        tail = n_text if li == p - 1 else 0
        for b in range(B):
            kb = None if key_bias is None else key_bias[b]
            h[b], pr = decoder_layer(h[b], pos[b], layers[li], H, eps, base,
                                     tail, kb)
            if tail:
                probs[b] = pr
    if p == 0:
        for b in range(B):
            kb = None if key_bias is None else key_bias[b]
            probs[b] = score_only(h[b], pos[b], layers[0], H, n_text, eps,
                                  base, kb)
    probs = np.stack(probs)
    sal = salience(probs, n_vis).astype(np.float32)
    k2k3, _ = modality_budget(sal, n2, n3, k_total, min2, min3)
    kept = select_topk(sal, k2k3, n2, n3, n_text)
    h, pos2 = compact(h, pos, kept)
    h = h.copy()
    for li in range(p, len(layers)):
        for b in range(B):
            h[b], _ = decoder_layer(h[b], pos2[b], layers[li], H, eps, base)
    return dict(y=h, pos=pos2, kept_idx=kept, k2k3=k2k3, sal=sal, probs=probs)


# --------------------------------------------------------------------------
# Semantic-stage modality indicators per patch (Sec. 3.2, Eqs. 4-6)
# --------------------------------------------------------------------------
def modality_decompose(probs, n_patch):
    """Per-patch 2D share and "unique 3D" share of the attention.

    probs: [B, H, Nq, S]; patch p owns 2D token p and 3D token n_patch + p.
    Its two attention vectors a2, a3 run over the H*Nq (head, query) rows.
    a3 is split into the part parallel to a2 and the part orthogonal to it
    (Eq. 4); with L1 norms,
        M2D[p] = |a2|_1 / (|a2|_1 + |a3|_1)                       (Eq. 5)
        M3D[p] = |a3 - (<a3,a2>/<a2,a2>) a2|_1 / (|a2|_1 + |a3|_1)  (Eq. 6)
    (a2 = 0 leaves a3 whole; a zero denominator gives 0 for both).
    Returns (m2d, m3d), float64 [B, n_patch] each.
    """
    p = np.asarray(probs, F64)
    B, H, Nq, S = p.shape
    a2 = p[:, :, :, :n_patch].reshape(B, H * Nq, n_patch)
    a3 = p[:, :, :, n_patch:2 * n_patch].reshape(B, H * Nq, n_patch)
    s22 = np.sum(a2 * a2, axis=1)
    s23 = np.sum(a2 * a3, axis=1)
    coef = np.divide(s23, s22, out=np.zeros_like(s23), where=s22 > 0)
    ortho = a3 - coef[:, None, :] * a2
    l2 = np.sum(np.abs(a2), axis=1)
    l3 = np.sum(np.abs(a3), axis=1)
    lo = np.sum(np.abs(ortho), axis=1)
    den = l2 + l3
    m2d = np.divide(l2, den, out=np.zeros_like(den), where=den > 0)
    m3d = np.divide(lo, den, out=np.zeros_like(den), where=den > 0)
    return m2d, m3d


# --------------------------------------------------------------------------
# Action-iteration smoothing (Sec. 4.3, Eq. 7; Sec. 4.4, Eqs. 8-9; Alg. 1)
# --------------------------------------------------------------------------
def ema_indicator(x_hat_prev, x_t, t, k=7, beta=0.85):
    """Smoothed indicator at step t (1-based).

    t == 1: the observation itself (cold start; no pruning happens there).
    1 < t < k: running mean  ((t-1)/t) * prev + x_t / t          (Eq. 8).
    t >= k:  beta * prev + (1 - beta) * x_t                      (Eq. 9).
    """
    x_t = np.asarray(x_t, F64)
    if t == 1:
        return x_t.copy()
    prev = np.asarray(x_hat_prev, F64)
    if t < k:
        return prev * (F64(t - 1) / F64(t)) + x_t / F64(t)
    return beta * prev + (1.0 - beta) * x_t


# --------------------------------------------------------------------------
# Mask generation of the tri-stage framework (Sec. 4.1-4.4, Algorithm 1)
# --------------------------------------------------------------------------
def feature_share(feat, n_patch):
    """Data-preprocessing indicators per patch (Sec. 3.1, Eq. 1).

    feat: [B, S, D] token features; patch p owns rows p (2D) and n_patch + p
    (3D).  With l2 = |f_2D|_1 and l3 = |f_3D|_1 of the patch,
        M2D[p] = l2 / (l2 + l3),   M3D[p] = l3 / (l2 + l3)
    (both 0 when l2 + l3 == 0).  Returns (m2d, m3d), float64 [B, n_patch].
    """
    f = np.asarray(feat, F64)
    l2 = np.sum(np.abs(f[:, :n_patch, :]), axis=-1)
    l3 = np.sum(np.abs(f[:, n_patch:2 * n_patch, :]), axis=-1)
    den = l2 + l3
    m2d = np.divide(l2, den, out=np.zeros_like(den), where=den > 0)
    m3d = np.divide(l3, den, out=np.zeros_like(den), where=den > 0)
    return m2d, m3d


def kmeans_1d(v, max_iter=32):
    """Lloyd's k-means with 3 centres on the scalars v (Sec. 4.2: 1-D K-Means,
    K = 3, on the patches' attention scores).

    The paper fixes neither the start nor the stopping rule; taken here:
    centres start at (min, (min+max)/2, max); a point goes to the nearest
    centre, the lower-numbered one on equal distance; a centre becomes the
    mean of its points (a centre without points stays); stop when an
    assignment repeats the previous one or after max_iter assignments.
    Returns (labels int [n] in {0,1,2}, centres float64 [3], margin) where
    margin is the smallest gap, over all assignments made, between a point's
    nearest and second-nearest distance relative to the data range (tests
    use it to set aside inputs that sit on a rounding knife-edge).
    """
    x = np.asarray(v, F64).ravel()
    lo, hi = x.min(), x.max()
    c = np.array([lo, 0.5 * (lo + hi), hi], F64)
    span = hi - lo if hi > lo else 1.0
    labels, margin = None, np.inf
    for _ in range(max_iter):
        d = np.abs(x[:, None] - c[None, :])            # [n, 3]
        new = np.argmin(d, axis=1)                     # first minimum: lower centre on ties
        for a in range(3):                             # knife-edge measure, distinct centres only
            for b2 in range(a + 1, 3):
                if c[a] != c[b2]:
                    near = np.minimum(d[:, a], d[:, b2]) <= d.min(axis=1)
                    if near.any():
                        gap = np.abs(d[near, a] - d[near, b2]).min()
                        margin = min(margin, gap / span)
        if labels is not None and np.array_equal(new, labels):
            break
        labels = new
        for j in range(3):
            members = x[labels == j]
            if members.size:
                c[j] = members.sum() / members.size
    return labels.astype(np.int64), c, margin


SEM_BG, SEM_ROB, SEM_OBJ = 0, 1, 2


def candidate_masks(x_hat, score, u, tau_2d=0.08, tau_3d=0.20, bg_drop=0.9,
                    obj_2d_min=0.9, obj_3d_max=0.01, max_iter=32):
    """Candidate sets and retention masks of Algorithm 1 for t > 1
    (Sec. 4.1 dual threshold, Sec. 4.2 semantic rules, Sec. 4.4 fusion, Eq. 10).

    x_hat: float32 [4, B, P], the smoothed per-patch indicators in the order
           (M2D^S1, M3D^S1, M2D^S2, M3D^S2).
    score: float32 [B, P], the patch's attention score that is clustered.
    u    : float32 [B, P], uniform draws in [0, 1) for the background drop.
    The indicators and the rule constants are float32 data (that is how they
    are handed over: Algorithm 1's tau = 0.08 / 0.20 and the other constants
    reach either side as the float32 nearest to the decimal), so a threshold
    decision compares the float32 indicator with that float32 constant; the
    two baselines are float64 means over the sample's patches.
    Readings where the text gives no number: clusters are named by the order
    of their centres (lowest = background, middle = robot, highest = object);
    "2D far above 0 and 3D near 0" for an object patch is
    M2D^S2 > obj_2d_min and M3D^S2 < obj_3d_max.
    Returns dict(mask2d, mask3d uint8 [B, P]; sem uint8 [B, P];
    mu float64 [B, 2]; kmeans_margin, mu_margin float64 [B]).
    """
    xh = np.asarray(x_hat)
    assert xh.dtype == np.float32 and xh.shape[0] == 4
    sc = np.asarray(score)
    uu = np.asarray(u)
    assert sc.dtype == np.float32 and uu.dtype == np.float32
    _, B, P = xh.shape
    f32 = np.float32
    mask2d = np.zeros((B, P), np.uint8)
    mask3d = np.zeros((B, P), np.uint8)
    sem = np.zeros((B, P), np.uint8)
    mu = np.zeros((B, 2), F64)
    km_margin = np.zeros(B, F64)
    mu_margin = np.zeros(B, F64)
    for b in range(B):
        labels, _, km_margin[b] = kmeans_1d(sc[b], max_iter)
        m2 = xh[2, b].astype(F64)
        m3 = xh[3, b].astype(F64)
        mu2 = m2.sum() / P
        mu3 = m3.sum() / P
        mu[b] = (mu2, mu3)
        mu_margin[b] = min(np.min(np.abs(m2 - mu2)), np.min(np.abs(m3 - mu3)))
        for p in range(P):
            # data-preprocessing stage: dual threshold on the smoothed 3D share
            m3_s1 = xh[1, b, p]
            if m3_s1 < f32(tau_2d):
                c1 = {"2D"}
            elif m3_s1 > f32(tau_3d):
                c1 = {"3D"}
            else:
                c1 = {"2D", "3D"}
            # semantic stage
            s = int(labels[p])
            sem[b, p] = s
            if s == SEM_BG:
                c2 = set() if uu[b, p] < f32(bg_drop) else {"2D", "3D"}
            elif s == SEM_ROB:
                if m3[p] > mu3:
                    c2 = {"2D", "3D"}
                elif m2[p] > mu2:
                    c2 = {"2D"}
                else:
                    c2 = set()
            else:
                if xh[2, b, p] > f32(obj_2d_min) and xh[3, b, p] < f32(obj_3d_max):
                    c2 = {"2D"}
                else:
                    c2 = {"2D", "3D"}
            # fusion: patches without a semantic candidate are dropped
            if c2:
                cf = c2 & c1
                if not cf:
                    cf = c2
                mask2d[b, p] = 1 if "2D" in cf else 0
                mask3d[b, p] = 1 if "3D" in cf else 0
    return dict(mask2d=mask2d, mask3d=mask3d, sem=sem, mu=mu,
                kmeans_margin=km_margin, mu_margin=mu_margin)


def mask_indices(mask2d, mask3d, n_text):
    """Kept token indices per sample from the two masks (Eq. 10): 2D tokens
    with mask 1, then 3D tokens with mask 1 (offset by the patch count), then
    every language token.  Returns a list of B int32 arrays (ragged)."""
    m2 = np.asarray(mask2d)
    m3 = np.asarray(mask3d)
    B, P = m2.shape
    out = []
    for b in range(B):
        keep2 = [p for p in range(P) if m2[b, p]]
        keep3 = [P + p for p in range(P) if m3[b, p]]
        text = list(range(2 * P, 2 * P + n_text))
        out.append(np.array(keep2 + keep3 + text, np.int32))
    return out


def patch_score(sal, n_patch):
    """Attention score of a patch: its 2D token's salience plus its 3D token's
    (the summand of Eq. 3).  Scores cross the library boundary as float32, so
    the sum of the two float32 inputs is formed exactly (float64 holds it) and
    rounded once to float32."""
    s = np.asarray(sal, np.float32).astype(F64)
    return (s[:, :n_patch] + s[:, n_patch:2 * n_patch]).astype(np.float32)


def masked_prefill(x, pos, layers, H, n_patch, n_text, p, t, x_hat_prev, u,
                   eps=1e-5, base=10000.0, key_bias=None, k=7, beta=0.85,
                   **rule_kw):
    """One action-iteration step of the whole path with Algorithm 1's masks.

    p >= 1 layers run on all tokens; the p-th yields the language-query
    probabilities, and its output rows serve as the token features of Eq. 1
    (the paper hooks the last layer, where pruned tokens no longer exist;
    taken here: the last layer that still sees every token).  The four
    indicators are smoothed over steps (Eqs. 8-9); at t == 1 nothing is
    pruned; later the masks select the tokens and the remaining layers run
    per sample on its own kept tokens (ragged).
    Returns dict(y: list of [S'_b, D], kept: list of int32, x_hat float64
    [4,B,P], x_t, masks: dict or None, probs, sal, feat).
    """
    x = np.asarray(x, F64)
    B, S, D = x.shape
    assert p >= 1 and S == 2 * n_patch + n_text
    h = x.copy()
    probs = [None] * B
    for li in range(p):
        tail = n_text if li == p - 1 else 0
        for b in range(B):
            kb = None if key_bias is None else key_bias[b]
            h[b], pr = decoder_layer(h[b], pos[b], layers[li], H, eps, base, tail, kb)
            if tail:
                probs[b] = pr
    probs = np.stack(probs)
    m2_s1, m3_s1 = feature_share(h, n_patch)
    m2_s2, m3_s2 = modality_decompose(probs, n_patch)
    x_t = np.stack([m2_s1, m3_s1, m2_s2, m3_s2])
    x_hat = ema_indicator(x_hat_prev, x_t, t, k, beta)
    sal = salience(probs, 2 * n_patch).astype(np.float32)
    if t == 1:
        masks = None
        kept = [np.arange(S, dtype=np.int32) for _ in range(B)]
    else:
        masks = candidate_masks(x_hat.astype(np.float32), patch_score(sal, n_patch),
                                np.asarray(u, np.float32), **rule_kw)
        kept = mask_indices(masks["mask2d"], masks["mask3d"], n_text)
    ys = []
    for b in range(B):
        hb = h[b][kept[b]].copy()
        pb = np.asarray(pos)[b][kept[b]]
        for li in range(p, len(layers)):
            hb, _ = decoder_layer(hb, pb, layers[li], H, eps, base)
        ys.append(hb)
    return dict(y=ys, kept=kept, x_hat=x_hat, x_t=x_t, masks=masks, probs=probs,
                sal=sal, feat=h)
