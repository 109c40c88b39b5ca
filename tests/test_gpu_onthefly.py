"""GPU parity of the scoring that is reduced on the fly (no probability tensor): the layer call
that writes the salience directly, and the layer call that carries the whole pruning step."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle as O
from paper_2604_09244_amd import binding as mv
from paper_2604_09244_amd import workloads as W
from helpers import layer_cfg, oracle_weights, to64

pytestmark = pytest.mark.gpu


def _setup(name, B, layer=0):
    wl = replace(W.WORKLOADS[name], B=B)
    ctx = mv.Context(B, wl.S, wl.D, wl.H, wl.F, wl.nt)
    w_cpu = W.layer_weights(wl, layer)
    packed = mv.pack_layer({k: v.cuda() for k, v in w_cpu.items()})
    struct = ctx.layer_struct(packed, ctx.rope_table(wl.rope_base, wl.S, wl.dh))
    x, pos = W.hidden_states(wl, device="cuda")
    kb = W.scoring_bias(wl, device="cuda")
    return wl, ctx, w_cpu, packed, struct, x, pos, kb


@pytest.mark.parametrize("name,B", [("tiny", 1), ("single_view", 1), ("action_iter", 4),
                                    ("multi_view", 8), ("ratio_sweep", 16)])    # full launch shapes
def test_layer_salience_equals_two_call_route(name, B):
    """Same layer output bit for bit; salience equal to mvla_salience of the written
    probabilities up to summation order (1e-5 relative)."""
    wl, ctx, _, packed, struct, x, pos, kb = _setup(name, B)
    cfg = layer_cfg(wl)
    y_ref, probs = ctx.prefill_layer(cfg, struct, x, pos, n_query_tail=wl.nt, key_bias=kb)
    sal_ref = ctx.salience(probs, wl.n_vis)
    y, sal = ctx.prefill_layer_salience(cfg, struct, x, pos, wl.nt, wl.n_vis, key_bias=kb)
    torch.cuda.synchronize()
    assert torch.equal(y, y_ref)
    a, b = to64(sal), to64(sal_ref)
    assert np.all(np.abs(a - b) <= 1e-5 * np.abs(b))
    # and both equal the oracle's reduction of the written probabilities
    ref = O.salience(probs.cpu().numpy(), wl.n_vis)
    assert np.all(np.abs(a - ref) <= 1e-5 * ref)
    # a narrower column range and fewer query rows (ragged tile)
    nq, nv = max(1, wl.nt - 5), wl.n_vis - 3
    _, probs2 = ctx.prefill_layer(cfg, struct, x, pos, n_query_tail=nq, key_bias=kb)
    _, sal2 = ctx.prefill_layer_salience(cfg, struct, x, pos, nq, nv, key_bias=kb)
    torch.cuda.synchronize()
    ref2 = O.salience(probs2.cpu().numpy(), nv)
    assert np.all(np.abs(to64(sal2) - ref2) <= 1e-5 * ref2)
    ctx.close()


def test_layer_salience_against_oracle_layer():
    """Against the fp64 oracle layer (bf16 q and k underneath: the probabilities move by a few
    percent, their mean over 1024 rows by less)."""
    wl, ctx, w_cpu, packed, struct, x, pos, kb = _setup("single_view", 1)
    _, sal = ctx.prefill_layer_salience(layer_cfg(wl), struct, x, pos, wl.nt, wl.n_vis, key_bias=kb)
    torch.cuda.synchronize()
    _, probs = O.decoder_layer(to64(x[0]), pos[0].cpu().numpy(), oracle_weights(w_cpu), wl.H,
                               wl.rms_eps, wl.rope_base, wl.nt, kb[0].cpu().numpy())
    ref = O.salience(probs[None], wl.n_vis)[0]
    err = np.abs(to64(sal[0]) - ref) / ref
    print(f"[on the fly] salience vs oracle layer: max rel {err.max():.3e}", flush=True)
    assert err.max() <= 3e-2
    ctx.close()


@pytest.mark.parametrize("name,B", [("single_view", 1), ("action_iter", 4), ("multi_view", 2),
                                    ("ratio_sweep", 1)])
def test_layer_prune_call(name, B):
    wl, ctx, _, packed, struct, x, pos, kb = _setup(name, B)
    cfg = layer_cfg(wl)
    y = torch.empty_like(x)
    out = ctx.prefill_layer_prune(cfg, struct, x, pos, y, wl.n2, wl.n3, wl.nt, wl.k_total, kb)
    y_ref, sal_ref = ctx.prefill_layer_salience(cfg, struct, x, pos, wl.nt, wl.n_vis, key_bias=kb)
    torch.cuda.synchronize()
    assert torch.equal(y, y_ref) and torch.equal(out["sal"], sal_ref)
    # budget and selection: bit-exact against the oracle on the call's own fp32 scores
    sal = out["sal"].cpu().numpy()
    k2k3, _ = O.modality_budget(sal, wl.n2, wl.n3, wl.k_total)
    kept = O.select_topk(sal, k2k3, wl.n2, wl.n3, wl.nt)
    assert np.array_equal(out["k2k3"].cpu().numpy(), k2k3)
    assert np.array_equal(out["kept_idx"].cpu().numpy(), kept)
    idx = torch.from_numpy(kept).long().cuda()
    for b in range(B):
        assert torch.equal(out["h"][b], y[b][idx[b]])
        assert torch.equal(out["pos"][b], pos[b][idx[b]])
    ctx.close()


def test_layer_prune_argument_errors():
    wl, ctx, _, packed, struct, x, pos, kb = _setup("tiny", 1)
    cfg = layer_cfg(wl)
    y = torch.empty_like(x)
    with pytest.raises(mv.MvlaError):          # token counts do not add up to S
        ctx.prefill_layer_prune(cfg, struct, x, pos, y, wl.n2, wl.n3 - 1, wl.nt, wl.k_total, kb)
    with pytest.raises(mv.MvlaError):          # budget larger than the visual tokens
        ctx.prefill_layer_prune(cfg, struct, x, pos, y, wl.n2, wl.n3, wl.nt, wl.n_vis + 1, kb)
    out = ctx.prefill_layer_prune(cfg, struct, x, pos, y, wl.n2, wl.n3, wl.nt, wl.k_total, kb)
    with pytest.raises(mv.MvlaError):          # gathered rows overlapping the layer output
        bad = dict(out)
        bad["h"] = y.view(-1)[: out["h"].numel()].view_as(out["h"])
        ctx.prefill_layer_prune(cfg, struct, x, pos, y, wl.n2, wl.n3, wl.nt, wl.k_total, kb, out=bad)
    with pytest.raises(mv.MvlaError):
        ctx.prefill_layer_salience(cfg, struct, x, pos, 0, wl.n_vis)
    torch.cuda.synchronize()
    ctx.close()


def test_plan_on_the_fly_equals_default_route():
    """Whole pruned prefill, single-view: when both routes keep the same tokens (they do unless
    two scores differ only in summation order) every later tensor is identical."""
    wl = W.WORKLOADS["single_view"]
    ctx = mv.Context(wl.B, wl.S, wl.D, wl.H, wl.F, wl.nt)
    layers = [mv.pack_layer(W.layer_weights(wl, l, device="cuda")) for l in range(wl.L)]
    plan = mv.PrefillPlan(ctx, layer_cfg(wl), layers, wl.B, wl.n2, wl.n3, wl.nt, wl.k_total, wl.p)
    x, pos = W.hidden_states(wl, device="cuda")
    kb = W.scoring_bias(wl, device="cuda")
    y0 = plan.run(x, pos, kb).clone()
    kept0 = plan.prune["kept_idx"].clone()
    y1 = plan.run(x, pos, kb, on_the_fly=True).clone()
    kept1 = plan.prune["kept_idx"].clone()
    torch.cuda.synchronize()
    same = torch.equal(kept0, kept1)
    overlap = len(set(kept0[0].tolist()) & set(kept1[0].tolist())) / kept0.shape[1]
    print(f"[on the fly] kept sets identical: {same}, overlap {overlap:.4f}", flush=True)
    assert overlap >= 0.99
    if same:
        assert torch.equal(y0, y1)
    ctx.close()


def test_measured_kernel_choices_keep_the_results():
    """mvla_tune_layers records a tile configuration per projection shape; layer outputs with
    the recorded choices differ from the model-chosen ones only by fp32 summation order."""
    wl = replace(W.WORKLOADS["action_iter"], B=2)
    ctx = mv.Context(wl.B, wl.S, wl.D, wl.H, wl.F, wl.nt)
    ws = [mv.pack_layer(W.layer_weights(wl, l, device="cuda")) for l in range(2)]
    rope = ctx.rope_table(wl.rope_base, wl.S, wl.dh)
    structs = [ctx.layer_struct(w, rope) for w in ws]
    cfg = layer_cfg(wl)
    x, pos = W.hidden_states(wl, device="cuda")
    M = wl.B * wl.S
    assert ctx.tuned_choice(M, 3 * wl.D, wl.D, 0) == (-1, 0)
    y0 = ctx.prefill_layer(cfg, structs[0], x, pos).clone()
    ctx.tune_layers(cfg, structs, wl.B, wl.S)
    shapes = [(3 * wl.D, wl.D, 0), (wl.D, wl.D, 1), (wl.D, wl.F, 2), (2 * wl.F, wl.D, 3)]
    for N, K, epi in shapes:
        c, pct = ctx.tuned_choice(M, N, K, epi)
        print(f"[tune] M={M} N={N} K={K} epilogue {epi}: config {c}, split below {pct} %", flush=True)
        assert 0 <= c < 8 and pct in (0, 50, 101)
    y1 = ctx.prefill_layer(cfg, structs[0], x, pos)
    torch.cuda.synchronize()
    a, b = to64(y0), to64(y1)
    scale = float(np.sqrt(np.mean(a * a)))
    # one bf16 rounding step at most (2^-7 relative), a little more next to zero
    assert np.all(np.abs(a - b) <= np.maximum(np.abs(a), np.abs(b)) * 2.0 ** -7 + 4e-3 * scale)
    assert np.mean(a != b) < 0.05
    ctx.close()
