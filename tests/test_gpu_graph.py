"""The pruned prefill under HIP graph capture: the whole step (full-sequence layers, the layer
that carries the pruning step, compaction, kept-token layers; K-split projections with their
arrival counters included) is captured once and replayed; every replay, with eager work and
synchronisations in between, must reproduce the eager result bit for bit."""
import pytest
import torch

from paper_2604_09244_amd import binding as mv
from paper_2604_09244_amd import workloads as W
from helpers import layer_cfg

pytestmark = pytest.mark.gpu


def test_captured_step_replays_to_the_eager_result():
    wl = W.WORKLOADS["single_view"]
    layers = [mv.pack_layer(W.layer_weights(wl, l, device="cuda")) for l in range(wl.L)]
    x, pos = W.hidden_states(wl, device="cuda")
    kb = W.scoring_bias(wl, device="cuda")
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        ctx = mv.Context(wl.B, wl.S, wl.D, wl.H, wl.F, wl.nt)     # launches on `st`
        plan = mv.PrefillPlan(ctx, layer_cfg(wl), layers, wl.B, wl.n2, wl.n3, wl.nt, wl.k_total,
                              wl.p, rope_base=wl.rope_base)
        # every projection K-split whenever its last round is not full: the path with partial
        # buffers and arrival counters, which a replay must find at zero again
        D, F = wl.D, wl.F
        for M in (wl.B * wl.S, wl.B * wl.S_kept):
            for N, K, epi in ((3 * D, D, 0), (D, D, 1), (D, F, 2), (2 * F, D, 3)):
                ctx.set_gemm_choice(M, N, K, epi, 3, 101)
        for _ in range(2):
            y = plan.run(x, pos, kb, on_the_fly=True)
        st.synchronize()
        y_ref, kept_ref = y.clone(), plan.prune["kept_idx"].clone()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            y_g = plan.run(x, pos, kb, on_the_fly=True)
        st.synchronize()
        for _ in range(4):
            y_g.zero_()
            plan.prune["kept_idx"].zero_()
            g.replay()
            st.synchronize()
            assert torch.equal(y_g, y_ref)
            assert torch.equal(plan.prune["kept_idx"], kept_ref)
            # eager work of the same context between the replays
            y_e = plan.run(x, pos, kb, on_the_fly=True)
            st.synchronize()
            assert torch.equal(y_e, y_ref)
        ctx.close()


def test_captured_action_iteration_step_with_smoothing():
    """A whole action-iteration step at its launch shape (B = 4 episodes, S = 544 -> S' = 237,
    4 layers) including the smoothing of the salience (Eqs. 8-9) under graph capture.  The
    smoothed state is read and updated by the step, so it is put back to its value before the
    step ahead of every replay; each replay must then reproduce the eager step bit for bit:
    hidden states, kept indices and the new state."""
    wl = W.WORKLOADS["action_iter"]
    layers = [mv.pack_layer(W.layer_weights(wl, l, device="cuda")) for l in range(wl.L)]
    x, pos = W.hidden_states(wl, device="cuda")
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        ctx = mv.Context(wl.B, wl.S, wl.D, wl.H, wl.F, wl.nt)
        plan = mv.PrefillPlan(ctx, layer_cfg(wl), layers, wl.B, wl.n2, wl.n3, wl.nt, wl.k_total,
                              wl.p, rope_base=wl.rope_base)
        xs = [x]
        for t in (1, 2, 3):
            xs.append(W.next_timestep(wl, xs[-1], t))
        kbs = [W.scoring_bias(wl, device="cuda", step=t) for t in range(4)]
        y1 = plan.run(xs[1], pos, kbs[1], smooth_step=1, on_the_fly=True)     # cold start
        assert y1.shape == (wl.B, wl.S, wl.D)
        plan.run(xs[2], pos, kbs[2], smooth_step=2, on_the_fly=True)
        st.synchronize()
        state = plan.sal_hat.clone()
        y = plan.run(xs[3], pos, kbs[3], smooth_step=3, on_the_fly=True)      # the step to capture
        st.synchronize()
        y_ref, kept_ref, hat_ref = y.clone(), plan.prune["kept_idx"].clone(), plan.sal_hat.clone()
        assert y_ref.shape == (wl.B, wl.S_kept, wl.D) and not torch.equal(hat_ref, state)
        plan.sal_hat.copy_(state)
        st.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            y_g = plan.run(xs[3], pos, kbs[3], smooth_step=3, on_the_fly=True)
        st.synchronize()
        for _ in range(3):
            plan.sal_hat.copy_(state)
            y_g.zero_()
            plan.prune["kept_idx"].zero_()
            g.replay()
            st.synchronize()
            assert torch.equal(y_g, y_ref)
            assert torch.equal(plan.prune["kept_idx"], kept_ref)
            assert torch.equal(plan.sal_hat, hat_ref)
            # eager work of the same context between the replays
            plan.sal_hat.copy_(state)
            y_e = plan.run(xs[3], pos, kbs[3], smooth_step=3, on_the_fly=True)
            st.synchronize()
            assert torch.equal(y_e, y_ref)
        ctx.close()
