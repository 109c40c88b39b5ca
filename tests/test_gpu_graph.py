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
