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


def assert_layer_close(y_gpu, y_ref, what, factor=2e-2):
    """bf16 layer outputs: max |diff| <= factor * RMS(reference output)."""
    y = to64(y_gpu)
    err = float(np.max(np.abs(y - y_ref)))
    bound = factor * rms(y_ref)
    assert err <= bound, f"{what}: max|diff| {err:.4g} > {bound:.4g} (rms {rms(y_ref):.4g})"
    return err / rms(y_ref)


def bf16_round(a):
    return torch.from_numpy(np.asarray(a)).to(torch.bfloat16)
