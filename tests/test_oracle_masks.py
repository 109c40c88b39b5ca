"""Pins for the oracle's Algorithm-1 mask generation (CPU only).

Each check ties a function to something outside it: a closed form, a value
worked out by hand from the rule in the paper, scikit-learn's Lloyd iteration,
or an invariant the method guarantees.
"""
import numpy as np
import pytest

import oracle as O

f32 = np.float32


# ---------------------------------------------------------------------------------------------
# Eq. 1: per-patch L1 feature share
# ---------------------------------------------------------------------------------------------
def test_feature_share_hand_values_and_layout():
    P, nt, D = 3, 2, 3
    feat = np.zeros((1, 2 * P + nt, D))
    feat[0, 0] = [1, -2, 3]            # patch 0, 2D row: L1 = 6
    feat[0, P + 0] = [0.5, 0.5, -1]    # patch 0, 3D row: L1 = 2
    feat[0, 1] = [4, 0, 0]             # patch 1: 4 vs 12
    feat[0, P + 1] = [-4, -4, -4]
    # patch 2 stays zero; language rows must not matter
    feat[0, 2 * P:] = 1e6
    m2, m3 = O.feature_share(feat, P)
    assert np.allclose(m2[0], [0.75, 0.25, 0.0], atol=0, rtol=1e-15)
    assert np.allclose(m3[0], [0.25, 0.75, 0.0], atol=0, rtol=1e-15)


def test_feature_share_scale_invariance_and_unit_sum():
    r = np.random.default_rng(3)
    feat = r.normal(size=(2, 2 * 16 + 4, 32))
    m2, m3 = O.feature_share(feat, 16)
    assert np.allclose(m2 + m3, 1.0, atol=1e-15)
    m2s, m3s = O.feature_share(-7.5 * feat, 16)            # |.| and a common scale cancel
    assert np.allclose(m2, m2s, rtol=1e-14) and np.allclose(m3, m3s, rtol=1e-14)
    feat3 = feat.copy()
    feat3[:, 16:32] *= 3.0                                  # 3D rows x3: odds x3
    _, m3b = O.feature_share(feat3, 16)
    assert np.allclose(m3b / (1 - m3b), 3.0 * m3 / (1 - m3), rtol=1e-13)


# ---------------------------------------------------------------------------------------------
# 1-D k-means, K = 3
# ---------------------------------------------------------------------------------------------
def _start(x):
    lo, hi = x.min(), x.max()
    return np.array([lo, 0.5 * (lo + hi), hi])


@pytest.mark.parametrize("seed", range(8))
def test_kmeans_matches_sklearn_lloyd_from_same_start(seed):
    from sklearn.cluster import KMeans
    r = np.random.default_rng(seed)
    kind = seed % 4
    n = [64, 256, 257, 1000][seed % 4]
    if kind == 0:
        x = np.exp(r.normal(size=n))
    elif kind == 1:
        x = r.uniform(size=n)
    elif kind == 2:
        x = np.concatenate([r.normal(0, 1, n // 2), r.normal(6, 0.5, n - n // 2)])
    else:
        x = np.exp(1.5 * r.normal(size=n)) * 1e-3
    x = x.astype(f32).astype(np.float64)
    labels, centres, margin = O.kmeans_1d(x, max_iter=300)
    km = KMeans(n_clusters=3, init=_start(x).reshape(3, 1), n_init=1, max_iter=300, tol=0.0,
                algorithm="lloyd").fit(x.reshape(-1, 1))
    assert margin > 1e-9
    assert np.array_equal(labels, km.labels_)
    got = np.array([x[labels == j].mean() if np.any(labels == j) else centres[j] for j in range(3)])
    assert np.allclose(got, km.cluster_centers_.ravel(), rtol=1e-9)


def test_kmeans_well_separated_groups_and_permutation():
    r = np.random.default_rng(0)
    groups = [r.uniform(0.0, 0.1, 40), r.uniform(4.9, 5.1, 7), r.uniform(9.9, 10.0, 3)]
    x = np.concatenate(groups)
    want = np.concatenate([np.full(len(g), j) for j, g in enumerate(groups)])
    labels, centres, _ = O.kmeans_1d(x)
    assert np.array_equal(labels, want)
    assert np.allclose(centres, [g.mean() for g in groups], rtol=1e-14)
    perm = r.permutation(len(x))
    labels_p, centres_p, _ = O.kmeans_1d(x[perm])
    assert np.array_equal(labels_p, want[perm]) and np.allclose(centres_p, centres, rtol=1e-13)


@pytest.mark.parametrize("seed", range(4))
def test_kmeans_is_a_lloyd_fixed_point_with_ordered_clusters(seed):
    r = np.random.default_rng(100 + seed)
    x = np.exp(r.normal(size=300))
    labels, centres, _ = O.kmeans_1d(x, max_iter=500)
    # every centre with members is their mean; every point sits with its nearest centre
    for j in range(3):
        if np.any(labels == j):
            assert np.isclose(centres[j], x[labels == j].mean(), rtol=1e-13)
    nearest = np.argmin(np.abs(x[:, None] - centres[None, :]), axis=1)
    assert np.array_equal(nearest, labels)
    # clusters are intervals in value order
    order = np.argsort(x, kind="stable")
    assert np.all(np.diff(labels[order]) >= 0)
    # Lloyd's objective cannot be beaten by moving one boundary point (local optimality in 1-D)
    cost = np.sum((x - centres[labels]) ** 2)
    xs, ls = x[order], labels[order]
    for i in np.nonzero(np.diff(ls))[0]:
        for donor, taker in ((i, ls[i + 1]), (i + 1, ls[i])):
            l2 = ls.copy()
            l2[donor] = taker
            c2 = np.array([xs[l2 == j].mean() if np.any(l2 == j) else centres[j] for j in range(3)])
            # a single reassignment with re-fitted means may lower the cost (Lloyd is not
            # Hartigan), but never with the centres held fixed
            assert np.sum((xs - centres[l2]) ** 2) >= cost - 1e-12
            assert np.all(np.isfinite(c2))


def test_kmeans_degenerate_inputs_and_tie_rule():
    labels, centres, _ = O.kmeans_1d(np.full(9, 0.25))
    assert np.array_equal(labels, np.zeros(9, int)) and np.all(centres == 0.25)
    labels, _, _ = O.kmeans_1d(np.array([1.0, 3.0, 1.0, 3.0]))
    assert np.array_equal(labels, [0, 2, 0, 2])            # middle centre (2.0) has no points
    # 0.5 is exactly midway between the starting centres 0 and 1: the lower one takes it
    labels, centres, _ = O.kmeans_1d(np.array([0.0, 1.0, 2.0, 0.5]))
    assert np.array_equal(labels, [0, 1, 2, 0]) and np.allclose(centres, [0.25, 1.0, 2.0])
    # one assignment only: labels of the starting centres
    labels, _, _ = O.kmeans_1d(np.array([0.0, 0.9, 4.0, 10.0]), max_iter=1)
    assert np.array_equal(labels, [0, 0, 1, 2])


# ---------------------------------------------------------------------------------------------
# Candidate sets, fusion, masks: a rule table worked out by hand from Algorithm 1
# ---------------------------------------------------------------------------------------------
# columns: score, M3D^S1, M2D^S2, M3D^S2, u, expected sem, expected (mask2d, mask3d)
# baselines from the table itself: mean M2D^S2 = 0.538 (between 0.2 and 0.8),
# mean M3D^S2 = 0.078 (between 0.05 and 0.3).
_RULES = [
    # background (score ~ 0): dropped when u < 0.9, otherwise both modalities proposed
    (0.00, 0.15, 0.10, 0.10, 0.50, 0, (0, 0)),
    (0.01, 0.05, 0.10, 0.10, 0.95, 0, (1, 0)),   # kept, feature share < tau_2D: 2D only
    (0.02, 0.15, 0.25, 0.10, 0.90, 0, (1, 1)),   # u == 0.9 is not "< 0.9"
    # robot (score ~ 5)
    (5.00, 0.50, 0.40, 0.30, 0.00, 1, (0, 1)),   # ortho-3D above baseline: both; share > tau_3D: 3D
    (5.05, 0.50, 0.80, 0.05, 0.00, 1, (1, 0)),   # 2D only proposed; Stage 1 says 3D: conflict -> 2D
    (4.95, 0.15, 0.20, 0.05, 0.00, 1, (0, 0)),   # below both baselines: dropped
    (5.02, 0.15, 0.80, 0.05, 0.99, 1, (1, 0)),   # 2D above its baseline only
    # object (score ~ 10)
    (10.0, 0.10, 0.95, 0.005, 0.0, 2, (1, 0)),   # extreme 2D reliance, 3D ~ 0: 2D only
    (10.1, 0.01, 0.95, 0.05, 0.00, 2, (1, 0)),   # both proposed; share < tau_2D: 2D
    (9.90, 0.90, 0.50, 0.005, 0.0, 2, (0, 1)),   # both proposed; share > tau_3D: 3D
    (9.95, 0.08, 0.50, 0.10, 0.00, 2, (1, 1)),   # share == tau_2D is inside the band
    (10.0, 0.20, 0.50, 0.10, 0.00, 2, (1, 1)),   # share == tau_3D is inside the band
    (10.2, 0.50, 0.95, 0.005, 0.0, 2, (1, 0)),   # 2D only vs Stage-1 3D only: conflict -> 2D
]


def _table_inputs():
    t = np.array([[r[0], r[1], r[2], r[3], r[4]] for r in _RULES], np.float64)
    P = len(_RULES)
    x_hat = np.zeros((4, 1, P), f32)
    x_hat[1, 0] = t[:, 1].astype(f32)
    x_hat[0, 0] = f32(1) - x_hat[1, 0]
    x_hat[2, 0] = t[:, 2].astype(f32)
    x_hat[3, 0] = t[:, 3].astype(f32)
    return x_hat, t[:, 0].astype(f32)[None], t[:, 4].astype(f32)[None]


def test_candidate_rule_table():
    x_hat, score, u = _table_inputs()
    out = O.candidate_masks(x_hat, score, u)
    assert np.array_equal(out["sem"][0], [r[5] for r in _RULES])
    assert abs(out["mu"][0, 0] - np.mean([r[2] for r in _RULES])) < 1e-7
    assert abs(out["mu"][0, 1] - np.mean([r[3] for r in _RULES])) < 1e-7
    got = list(zip(out["mask2d"][0].tolist(), out["mask3d"][0].tolist()))
    assert got == [r[6] for r in _RULES]


def test_candidate_masks_limits_of_the_rules():
    x_hat, score, u = _table_inputs()
    # Stage-1 band covering everything: the masks are the semantic proposal itself
    out = O.candidate_masks(x_hat, score, u, tau_2d=-1.0, tau_3d=2.0)
    want = [(0, 0), (1, 1), (1, 1), (1, 1), (1, 0), (0, 0), (1, 0), (1, 0), (1, 1), (1, 1),
            (1, 1), (1, 1), (1, 0)]
    assert list(zip(out["mask2d"][0].tolist(), out["mask3d"][0].tolist())) == want
    # no background drop at all / certain drop
    keep_all = O.candidate_masks(x_hat, score, u, bg_drop=0.0)
    assert np.all((keep_all["mask2d"][0, :3] | keep_all["mask3d"][0, :3]) == 1)
    drop_all = O.candidate_masks(x_hat, score, u, bg_drop=1.0)
    assert np.all(drop_all["mask2d"][0, :3] == 0) and np.all(drop_all["mask3d"][0, :3] == 0)
    # the object exception switched off: object patches propose both
    no_exc = O.candidate_masks(x_hat, score, u, obj_2d_min=2.0)
    assert (no_exc["mask2d"][0, 7], no_exc["mask3d"][0, 7]) == (1, 1)


@pytest.mark.parametrize("seed", range(4))
def test_candidate_mask_invariants(seed):
    r = np.random.default_rng(seed)
    B, P = 3, 256
    m3_s1 = r.beta(2, 12, size=(B, P))
    m2_s2 = r.beta(4, 3, size=(B, P))
    m3_s2 = (1 - m2_s2) * r.beta(1, 4, size=(B, P))
    x_hat = np.stack([1 - m3_s1, m3_s1, m2_s2, m3_s2]).astype(f32)
    score = np.exp(r.normal(size=(B, P))).astype(f32)
    u = r.uniform(size=(B, P)).astype(f32)
    out = O.candidate_masks(x_hat, score, u)
    m2, m3, sem = out["mask2d"], out["mask3d"], out["sem"]
    kept = (m2 | m3).astype(bool)
    assert np.all(kept[sem == O.SEM_OBJ])                       # object patches always survive
    assert not np.any(kept[(sem == O.SEM_BG) & (u < f32(0.9))])
    assert np.all(kept[(sem == O.SEM_BG) & (u >= f32(0.9))])
    rob = sem == O.SEM_ROB
    for b in range(B):
        mu2, mu3 = out["mu"][b]
        above3 = rob[b] & (x_hat[3, b] > mu3)
        only2 = rob[b] & ~(x_hat[3, b] > mu3) & (x_hat[2, b] > mu2)
        none = rob[b] & ~(x_hat[3, b] > mu3) & ~(x_hat[2, b] > mu2)
        assert np.all(kept[b][above3]) and not np.any(kept[b][none])
        assert np.all(m2[b][only2] == 1) and np.all(m3[b][only2] == 0)
        # a 3D token survives only where the semantic stage proposed it, and Stage 1 alone never
        # adds a modality: inside the band the proposal passes unchanged
        band = (x_hat[1, b] >= f32(0.08)) & (x_hat[1, b] <= f32(0.20))
        assert np.all((m2[b] & m3[b])[band & above3] == 1)
    # clusters are ordered by score
    for b in range(B):
        order = np.argsort(score[b], kind="stable")
        assert np.all(np.diff(sem[b][order].astype(int)) >= 0)


def test_mask_indices_hand_case_and_structure():
    m2 = np.array([[1, 0, 1, 0], [0, 0, 0, 0]], np.uint8)
    m3 = np.array([[0, 0, 1, 1], [0, 0, 0, 0]], np.uint8)
    idx = O.mask_indices(m2, m3, 2)
    assert idx[0].tolist() == [0, 2, 6, 7, 8, 9]
    assert idx[1].tolist() == [8, 9]                               # only the language tokens
    r = np.random.default_rng(5)
    m2 = (r.uniform(size=(4, 33)) < 0.4).astype(np.uint8)
    m3 = (r.uniform(size=(4, 33)) < 0.2).astype(np.uint8)
    for b, row in enumerate(O.mask_indices(m2, m3, 5)):
        assert len(row) == m2[b].sum() + m3[b].sum() + 5
        assert np.all(np.diff(row) > 0) and row[-5:].tolist() == list(range(66, 71))
        sel = np.zeros(71, bool)
        sel[row] = True
        assert np.array_equal(sel[:33], m2[b] == 1) and np.array_equal(sel[33:66], m3[b] == 1)


def test_patch_score_hand_values_layout_and_single_rounding():
    """Hand values (all exactly representable): patch p adds column p and column n_patch + p;
    language columns are ignored.  The second sample pins the rounding: 1 + 2^-24 is a tie
    between two float32 neighbours and goes to the even one (1.0), 1 + 3 * 2^-25 goes up."""
    sal = np.array([[0.5, 0.25, 0.125, 2.0, 9.0],
                    [1.0, 1.0, 2.0 ** -24, 3 * 2.0 ** -25, 7.0]], np.float32)
    got = O.patch_score(sal, 2)
    assert got.dtype == np.float32
    assert got.tolist() == [[0.625, 2.25], [1.0, 1.0 + 2.0 ** -23]]


# ---------------------------------------------------------------------------------------------
# Whole step
# ---------------------------------------------------------------------------------------------
def _tiny_problem(seed=0, B=2, P=12, nt=4, D=32, H=2, F=64, L=3):
    r = np.random.default_rng(seed)
    S = 2 * P + nt

    def layer():
        g = lambda *s: r.normal(0, 0.2, size=s)
        return dict(wq=g(D, D), wk=g(D, D), wv=g(D, D), wo=g(D, D), w_gate=g(F, D), w_up=g(F, D),
                    w_down=g(D, F), g_attn=1 + g(D) * 0.1, g_mlp=1 + g(D) * 0.1)
    layers = [layer() for _ in range(L)]
    x = r.normal(size=(B, S, D))
    x[:, P:2 * P] *= 0.15                                    # 3D features weaker, as in Table 1
    pos = np.tile(np.arange(S), (B, 1))
    return x, pos, layers, H, P, nt


def test_masked_step_cold_start_keeps_everything():
    x, pos, layers, H, P, nt = _tiny_problem()
    u = np.zeros((2, P), f32)
    out = O.masked_prefill(x, pos, layers, H, P, nt, p=1, t=1, x_hat_prev=None, u=u)
    full = O.pruned_prefill(x, pos, layers, H, P, P, nt, k_total=2 * P, p=1)   # keep 100 %
    assert out["masks"] is None
    for b in range(2):
        assert np.array_equal(out["kept"][b], np.arange(2 * P + nt))
        assert np.allclose(out["y"][b], full["y"][b], rtol=1e-12, atol=1e-12)
    assert np.array_equal(out["x_hat"], out["x_t"])                # no history at t = 1


def test_masked_step_structure_and_smoothing_recursion():
    x, pos, layers, H, P, nt = _tiny_problem(1)
    r = np.random.default_rng(9)
    u = r.uniform(size=(2, P)).astype(f32)
    s1 = O.masked_prefill(x, pos, layers, H, P, nt, p=1, t=1, x_hat_prev=None, u=u)
    x2 = x + r.normal(0, 0.05, size=x.shape)
    s2 = O.masked_prefill(x2, pos, layers, H, P, nt, p=1, t=2, x_hat_prev=s1["x_hat"], u=u)
    assert np.allclose(s2["x_hat"], 0.5 * (s1["x_t"] + s2["x_t"]), rtol=1e-13)   # Eq. 8 at t = 2
    m = s2["masks"]
    for b in range(2):
        kept = s2["kept"][b]
        assert len(kept) == m["mask2d"][b].sum() + m["mask3d"][b].sum() + nt
        assert s2["y"][b].shape == (len(kept), x.shape[2])
        # the kept tokens' later layers see only kept tokens: same as running the remaining
        # layers on the gathered rows with the gathered positions
        h = s2["feat"][b][kept]
        for li in range(1, len(layers)):
            h, _ = O.decoder_layer(h, pos[b][kept], layers[li], H)
        assert np.allclose(h, s2["y"][b], rtol=1e-12, atol=1e-12)
    # indicators are what the two indicator functions give on this step's tensors
    m2, m3 = O.feature_share(s2["feat"], P)
    d2, d3 = O.modality_decompose(s2["probs"], P)
    assert np.array_equal(s2["x_t"], np.stack([m2, m3, d2, d3]))
