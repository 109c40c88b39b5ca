"""Argument errors of the composed entry points and of the device probes: every invalid call
returns its status before anything is launched, and a valid call afterwards gives the same
bits as before (nothing was left half-done)."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2604_09244_amd import binding as mv
from paper_2604_09244_amd import workloads as W

pytestmark = pytest.mark.gpu

EINVAL = -1


@pytest.fixture(scope="module")
def tiny_plan():
    wl = W.WORKLOADS["tiny"]
    ctx = mv.Context(2, wl.S, wl.D, wl.H, wl.F, wl.nt)
    cfg = mv.LayerCfg(wl.D, wl.H, wl.dh, wl.F, wl.rms_eps)
    layers = [mv.pack_layer(W.layer_weights(wl, l, device="cuda")) for l in range(2)]
    plan = mv.PrefillPlan(ctx, cfg, layers, 2, wl.n2, wl.n3, wl.nt, wl.k_total, 1, wl.rope_base)
    x, pos = W.hidden_states(wl, device="cuda", B=2)
    return wl, ctx, plan, x, pos


def _prefill(plan, desc, x, pos, buffers=None, layers=None, y=True, rows=True):
    y_ptr, n = C.c_void_p(), C.c_int()
    return mv.load().mvla_prefill(plan.ctx.handle, C.byref(plan.cfg),
                                  layers if layers is not None else plan._layer_array,
                                  C.byref(desc), x.data_ptr() if x is not None else None,
                                  pos.data_ptr() if pos is not None else None, None,
                                  C.byref(buffers if buffers is not None else plan._buffers),
                                  C.byref(y_ptr) if y else None, C.byref(n) if rows else None)


def _desc(plan, **kw):
    f = dict(B=plan.B, n2=plan.n2, n3=plan.n3, n_text=plan.nt, k_total=plan.k_total, min2=0,
             min3=0, n_layers=plan.L, p=plan.p, smooth_step=0, smooth_k=7, smooth_beta=0.85,
             materialise_probs=0, separate_prune_calls=0)
    f.update(kw)
    return mv.PrefillDesc(*[f[name] for name, _ in mv.PrefillDesc._fields_])


def test_prefill_rejects_bad_descriptions_and_leaves_nothing_behind(tiny_plan):
    wl, ctx, plan, x, pos = tiny_plan
    good = plan.run(x, pos, on_the_fly=True).clone()
    kept = plan.prune["kept_idx"].clone()
    for kw in (dict(B=0), dict(n_text=0), dict(n2=0, n3=0), dict(n_layers=0), dict(p=-1),
               dict(p=plan.L + 1), dict(k_total=-1), dict(k_total=plan.n2 + plan.n3 + 1),
               dict(min2=plan.n2 + 1), dict(min2=plan.k_total, min3=1), dict(smooth_step=-1),
               dict(smooth_step=2, smooth_k=0), dict(smooth_step=2, smooth_beta=1.0),
               dict(smooth_step=2, smooth_beta=0.0)):
        assert _prefill(plan, _desc(plan, **kw), x, pos) == EINVAL, kw
    # missing pointers
    assert _prefill(plan, _desc(plan), None, pos) == EINVAL
    assert _prefill(plan, _desc(plan), x, None) == EINVAL
    assert _prefill(plan, _desc(plan), x, pos, y=False) == EINVAL
    assert _prefill(plan, _desc(plan), x, pos, rows=False) == EINVAL
    for field in ("sal", "k2k3", "kept_idx", "pos_kept"):
        b = mv.PrefillBuffers.from_buffer_copy(plan._buffers)
        setattr(b, field, None)
        assert _prefill(plan, _desc(plan), x, pos, buffers=b) == EINVAL, field
    b = mv.PrefillBuffers.from_buffer_copy(plan._buffers)
    b.probs = None                      # needed only when the probabilities are materialised
    assert _prefill(plan, _desc(plan, materialise_probs=1), x, pos, buffers=b) == EINVAL
    b = mv.PrefillBuffers.from_buffer_copy(plan._buffers)
    b.sal_hat = None                    # needed only with smoothing
    assert _prefill(plan, _desc(plan, smooth_step=2), x, pos, buffers=b) == EINVAL
    # a layer descriptor with a missing matrix is found before the first launch
    bad_layers = (mv.LayerWeightsC * plan.L)(*plan.structs)
    bad_layers[plan.L - 1].w_down = None
    assert _prefill(plan, _desc(plan), x, pos, layers=bad_layers) == EINVAL
    torch.cuda.synchronize()
    again = plan.run(x, pos, on_the_fly=True)
    assert torch.equal(again, good) and torch.equal(plan.prune["kept_idx"], kept)


def test_probe_argument_errors(tiny_plan):
    wl, ctx, plan, x, pos = tiny_plan
    lib = mv.load()
    out = C.c_double()
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    h = ctx.handle
    assert lib.mvla_peak_probe(None, mv.PROBE_LAUNCH, None, 0, 1, C.byref(out)) == EINVAL
    assert lib.mvla_peak_probe(h, 4, buf.data_ptr(), buf.numel(), 1, C.byref(out)) == EINVAL
    assert lib.mvla_peak_probe(h, -1, buf.data_ptr(), buf.numel(), 1, C.byref(out)) == EINVAL
    assert lib.mvla_peak_probe(h, mv.PROBE_READ, buf.data_ptr(), buf.numel(), 0, C.byref(out)) == EINVAL
    assert lib.mvla_peak_probe(h, mv.PROBE_READ, buf.data_ptr(), buf.numel(), 1, None) == EINVAL
    assert lib.mvla_peak_probe(h, mv.PROBE_READ, None, buf.numel(), 1, C.byref(out)) == EINVAL
    assert lib.mvla_peak_probe(h, mv.PROBE_READ, buf.data_ptr() + 8, buf.numel() - 8, 1,
                               C.byref(out)) == EINVAL          # not 16-byte aligned
    assert lib.mvla_peak_probe(h, mv.PROBE_COPY, buf.data_ptr(), (1 << 20) - 16, 1,
                               C.byref(out)) == EINVAL          # under 1 MiB
    assert lib.mvla_peak_probe(h, mv.PROBE_MFMA, buf.data_ptr(), 4096, 1, C.byref(out)) == EINVAL
    # and the smallest valid calls of each kind give a positive figure
    for kind in (mv.PROBE_READ, mv.PROBE_COPY, mv.PROBE_MFMA, mv.PROBE_LAUNCH):
        assert lib.mvla_peak_probe(h, kind, buf.data_ptr(), buf.numel(), 2, C.byref(out)) == 0
        assert np.isfinite(out.value) and out.value > 0


def test_masked_step_rejects_bad_descriptions(tiny_plan):
    """mvla_masked_prefill_step: every invalid description or missing buffer returns before a
    launch; a valid first step (cold start, nothing pruned) still runs afterwards."""
    wl, ctx, plan, x, pos = tiny_plan
    ep = mv.MaskedPrefill(plan)
    lib = mv.load()
    u = W.uniform_draws(wl, device="cuda", B=plan.B, step=1)

    def call(desc, x_=x, u_=u, buffers=None, lengths=True):
        y_ptr, rows = C.c_void_p(), C.c_int()
        ln = (C.c_int32 * plan.B)()
        return lib.mvla_masked_prefill_step(
            ctx.handle, C.byref(plan.cfg), plan._layer_array, C.byref(desc),
            x_.data_ptr() if x_ is not None else None, pos.data_ptr(), None,
            u_.data_ptr() if u_ is not None else None,
            C.byref(buffers if buffers is not None else ep._buffers), C.byref(y_ptr), C.byref(rows),
            ln if lengths else None)

    def desc(**kw):
        f = dict(B=plan.B, n_patch=plan.n2, n_text=plan.nt, n_layers=plan.L, p=plan.p, t=2,
                 smooth_k=7, smooth_beta=0.85, rules=mv.MaskRules.default())
        f.update(kw)
        return mv.MaskedDesc(*[f[name] for name, _ in mv.MaskedDesc._fields_])

    for kw in (dict(B=0), dict(n_patch=0), dict(n_text=0), dict(n_layers=0), dict(p=0),
               dict(p=plan.L + 1), dict(t=0), dict(smooth_k=0), dict(smooth_beta=1.0),
               dict(rules=mv.MaskRules.default(kmeans_max_iter=0)),
               dict(rules=mv.MaskRules.default(tau_2d=0.5, tau_3d=0.1)),
               dict(rules=mv.MaskRules.default(bg_drop=1.5))):
        assert call(desc(**kw)) == EINVAL, kw
    assert call(desc(n_patch=16385)) == -4                       # more patches than the LDS stages
    assert call(desc(), x_=None) == EINVAL
    assert call(desc(), u_=None) == EINVAL                       # t > 1 needs the draws
    assert call(desc(), lengths=False) == EINVAL
    for field in ("probs", "sal", "x_t", "x_hat", "mask2d", "kept_len", "kept_idx", "pos_kept"):
        b = mv.MaskedBuffers.from_buffer_copy(ep._buffers)
        setattr(b, field, None)
        assert call(desc(), buffers=b) == EINVAL, field
    torch.cuda.synchronize()
    y, lengths = ep.step(1, x, pos, u)
    torch.cuda.synchronize()
    assert y.shape[1] == plan.S and lengths == [plan.S] * plan.B
