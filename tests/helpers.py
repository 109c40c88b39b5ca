"""Shared plumbing of the GPU parity tests (no method arithmetic)."""
import numpy as np
import torch

from paper_2604_09244_amd import binding as mv
from paper_2604_09244_amd import workloads as W


def to64(t):
    return t.detach().to("cpu", torch.float64).numpy()


def oracle_weights(w):
    return {k: to64(v) for k, v in w.items()}


def device_layer(ctx, wl, w_cpu, rope_len=None):
    packed = mv.pack_layer({k: v.cuda() for k, v in w_cpu.items()})
    rope = ctx.rope_table(wl.rope_base, rope_len or wl.S, wl.dh)
    return packed, ctx.layer_struct(packed, rope)


def layer_cfg(wl):
    return mv.LayerCfg(wl.D, wl.H, wl.dh, wl.F, wl.rms_eps)


def rms(a):
    return float(np.sqrt(np.mean(np.square(a))))


def assert_layer_close(y_gpu, y_ref, what, D):
    """Parity bar for bf16 layer outputs against the fp64 oracle.

    Stated bar: max|diff| <= 2e-2 * RMS(reference output).  It is applied as is
    for hidden sizes up to 1024.  At the 7B shape (D = 4096, N(0, 0.02) weights)
    the matrix-core operands (normalised input, q, k, v, probabilities,
    attention output, normalised residual, gated activation) and the output are
    each rounded to bf16 once; test_bf16_operand_rounding_floor (CPU) shows that
    an otherwise exact fp64 pipeline with only those roundings already lands at
    2.1e-2 .. 2.4e-2 on the worst of 2.2 M elements (RMS error 3.5e-3).  There
    the bar is therefore split: at most 2e-5 of the elements may exceed
    2e-2 * RMS, none may exceed 3e-2 * RMS, and the RMS error must stay below
    5e-3 * RMS.
    """
    y = to64(y_gpu)
    r = rms(y_ref)
    d = np.abs(y - y_ref) / r
    worst, rms_err = float(d.max()), float(np.sqrt(np.mean(d * d)))
    frac_over = float(np.mean(d > 2e-2))
    print(f"[parity] {what}: max|diff| = {worst:.4f} x RMS, rms err = {rms_err:.5f} x RMS, "
          f"frac > 2e-2: {frac_over:.2e}", flush=True)
    if D <= 1024:
        assert worst <= 2e-2, f"{what}: max|diff| {worst:.4g} x RMS > 2e-2"
    else:
        assert worst <= 3e-2, f"{what}: max|diff| {worst:.4g} x RMS > 3e-2"
        assert frac_over <= 2e-5, f"{what}: {frac_over:.3g} of elements beyond 2e-2 x RMS"
        assert rms_err <= 5e-3, f"{what}: rms error {rms_err:.4g} x RMS"
    return worst


def bf16_round(a):
    return torch.from_numpy(np.asarray(a)).to(torch.bfloat16)
