"""GPU parity of the action-iteration smoothing (Eqs. 8-9) and its use inside the pruned
prefill of a drifting episode."""
import numpy as np
import pytest
import torch

import oracle as O
from paper_2604_09244_amd import binding as mv
from paper_2604_09244_amd import workloads as W
from helpers import layer_cfg, to64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = mv.Context(B=4, S=544, D=4096, H=32, F=11008, n_query_tail=32)
    yield c
    c.close()


@pytest.mark.parametrize("n", [1, 513, 4 * 512])
def test_smooth_matches_oracle_stepwise(ctx, n):
    r = np.random.default_rng(n)
    xs = r.random((12, n)).astype(np.float32)
    hat_gpu = torch.zeros(n, device="cuda")
    hat_ref = None
    for t in range(1, 13):
        # teacher-forced: the GPU state is reset to the oracle's (fp32-rounded) previous state
        if hat_ref is not None:
            hat_gpu.copy_(torch.from_numpy(hat_ref.astype(np.float32)))
        hat_ref = O.ema_indicator(None if hat_ref is None else hat_ref.astype(np.float32), xs[t - 1], t)
        ctx.temporal_smooth(torch.from_numpy(xs[t - 1]).cuda(), hat_gpu, t)
        torch.cuda.synchronize()
        got = to64(hat_gpu)
        assert np.max(np.abs(got - hat_ref) / np.maximum(np.abs(hat_ref), 1e-30)) <= 1e-6, t
    # free-running over all steps stays within a few ulps as well
    hat = torch.zeros(n, device="cuda")
    ref = None
    for t in range(1, 13):
        ctx.temporal_smooth(torch.from_numpy(xs[t - 1]).cuda(), hat, t)
        ref = O.ema_indicator(ref, xs[t - 1], t)
    torch.cuda.synchronize()
    assert np.max(np.abs(to64(hat) - ref) / ref) <= 5e-6


def test_smooth_argument_errors(ctx):
    x = torch.zeros(4, device="cuda")
    lib = mv.load()
    assert lib.mvla_temporal_smooth(ctx.handle, x.data_ptr(), x.data_ptr(), 4, 0, 7, 0.85) == -1
    assert lib.mvla_temporal_smooth(ctx.handle, x.data_ptr(), x.data_ptr(), 4, 2, 7, 1.0) == -1
    assert lib.mvla_temporal_smooth(ctx.handle, None, x.data_ptr(), 4, 2, 7, 0.85) == -1


def test_smoothed_selection_in_an_episode(ctx):
    """Episode of 8 drifting steps at the single-view shape (2 layers to keep it short): step 1
    is the cold start (no pruning), later steps select on the smoothed salience.  The smoothed
    state and the selection are checked against the oracle at every step (teacher-forced on the
    GPU's own per-step salience), and smoothing must make consecutive kept sets more alike."""
    wl = W.WORKLOADS["action_iter"]
    from dataclasses import replace
    wl = replace(wl, L=2, p=2, B=2)
    layers = [mv.pack_layer(W.layer_weights(wl, l, device="cuda")) for l in range(wl.L)]
    plan = mv.PrefillPlan(ctx, layer_cfg(wl), layers, wl.B, wl.n2, wl.n3, wl.nt, wl.k_total, wl.p)
    x, pos = W.hidden_states(wl, device="cuda")
    ref_hat = None
    kept_smooth, kept_raw = [], []
    for t in range(1, 9):
        if t > 1:
            x = W.next_timestep(wl, x, t)
        kb = W.scoring_bias(wl, device="cuda", step=t)
        y = plan.run(x, pos, kb, smooth_step=t)
        torch.cuda.synchronize()
        # the raw salience of this step stays in the plan's buffer (selection reads the smoothed
        # state in place); it is what mvla_salience gives for the written probabilities
        assert torch.equal(ctx.salience(plan.probs, wl.n_vis), plan.prune["sal"])
        sal_t = plan.prune["sal"].cpu().numpy()
        ref_hat = O.ema_indicator(ref_hat, sal_t, t)
        got = plan.sal_hat.cpu().numpy()
        assert np.max(np.abs(got - ref_hat) / ref_hat) <= 5e-6, t
        if t == 1:
            assert y.shape == (wl.B, wl.S, wl.D)            # cold start: nothing pruned
            continue
        assert y.shape == (wl.B, wl.S_kept, wl.D)
        k2k3, mass = O.modality_budget(got, wl.n2, wl.n3, wl.k_total)
        frac = wl.k_total * mass[:, 0] - np.floor(wl.k_total * mass[:, 0])
        if np.all(np.abs(frac - 0.5) > 1e-9):
            assert np.array_equal(plan.prune["k2k3"].cpu().numpy(), k2k3)
            assert np.array_equal(plan.prune["kept_idx"].cpu().numpy(),
                                  O.select_topk(got, k2k3, wl.n2, wl.n3, wl.nt))
        kept_smooth.append(plan.prune["kept_idx"].cpu().numpy().copy())
        rk, _ = O.modality_budget(sal_t, wl.n2, wl.n3, wl.k_total)
        kept_raw.append(O.select_topk(sal_t, rk, wl.n2, wl.n3, wl.nt))

    def churn(seq):
        return np.mean([len(set(a[b]) ^ set(c[b])) for a, c in zip(seq[:-1], seq[1:])
                        for b in range(wl.B)])
    assert churn(kept_smooth) < churn(kept_raw), (churn(kept_smooth), churn(kept_raw))
