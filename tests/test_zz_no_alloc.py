"""The allocation-free salience entry point (fixed scratch inside the library, no context)
against mvla_salience through the C ABI: identical results on two calls in a row, the second
on a smaller input; shapes beyond the fixed scratch are refused."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle as O
from paper_2604_09244_amd import binding as mv

pytestmark = pytest.mark.gpu


def _probs(B, H, Nq, S, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    e = torch.rand(B, H, Nq, S, generator=g, device="cuda", dtype=torch.float32) ** 4
    return (e / e.sum(-1, keepdim=True)).contiguous()


def test_noalloc_salience_equals_the_context_call_twice_in_a_row():
    lib = mv.load()
    ctx = mv.Context(8, 1840, 4096, 32, 11008, 48)
    stream = torch.cuda.current_stream().cuda_stream
    # first call: the multi-view shape (row-split partial sums, 8 x 28 column chunks);
    # second call: smaller in every dimension, ragged columns, on the scratch the first one used
    for B, H, Nq, S, n_vis, seed in ((8, 32, 48, 1840, 1792, 1), (3, 8, 20, 548, 509, 2)):
        attn = _probs(B, H, Nq, S, seed)
        want = torch.empty(B, n_vis, dtype=torch.float32, device="cuda")
        got = torch.full_like(want, -1.0)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        rc = lib.mvla_salience_noalloc(stream, attn.data_ptr(), B, H, Nq, S, n_vis, got.data_ptr())
        assert rc == 0, lib.mvla_strerror(rc)
        assert torch.cuda.memory_allocated() == before
        assert lib.mvla_salience(ctx.handle, attn.data_ptr(), B, H, Nq, S, n_vis, want.data_ptr()) == 0
        torch.cuda.synchronize()
        assert torch.equal(got, want)                                  # same kernel, same order
        ref = O.salience(attn.cpu().numpy(), n_vis)
        assert np.max(np.abs(got.cpu().numpy().astype(np.float64) - ref) / ref) <= 1e-5
    ctx.close()


def test_noalloc_salience_refuses_what_does_not_fit_and_bad_arguments():
    lib = mv.load()
    a = torch.zeros(16, device="cuda")
    s = torch.zeros(16, device="cuda")
    # partial sums of this shape need more than the 16 MiB the library holds
    assert lib.mvla_salience_noalloc(None, a.data_ptr(), 64, 32, 64, 8192, 8192, s.data_ptr()) == -5
    assert b"fixed scratch" in lib.mvla_strerror(-5)
    assert lib.mvla_salience_noalloc(None, None, 1, 1, 1, 4, 4, s.data_ptr()) == -1
    assert lib.mvla_salience_noalloc(None, a.data_ptr(), 1, 1, 1, 4, 5, s.data_ptr()) == -1
    torch.cuda.synchronize()
