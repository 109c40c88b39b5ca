"""The C-ABI library loads without a GPU and exports every symbol mvla.h declares."""
import ctypes
import os
import re

from paper_2604_09244_amd import binding as mv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "mvla.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mvla_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = mv.load()
    names = _declared()
    assert set(names) == set(mv.EXPORTS), (names, mv.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_host_only_calls():
    lib = mv.load()
    assert lib.mvla_version().decode().count(".") == 2
    assert b"workspace" in lib.mvla_strerror(-2)
    assert lib.mvla_workspace_bytes(0, 1, 1, 1, 1, 0) == 0
    small = lib.mvla_workspace_bytes(1, 144, 256, 4, 1024, 16)
    big = lib.mvla_workspace_bytes(8, 1840, 4096, 32, 11008, 48)
    assert 0 < small < big < 8 << 30
    # null context / null pointers are rejected on the host before anything touches a GPU
    assert lib.mvla_salience(None, None, 1, 1, 1, 1, 1, None) == -1
    assert lib.mvla_compact(None, None, None, None, 1, 1, 1, 8, None, None) == -1
    assert lib.mvla_create(None, 0, None, None, 0) == -1
    lib.mvla_destroy(None)


def test_pack_layer_layout():
    import torch
    F, D = 64, 8
    w = dict(wq=torch.zeros(D, D), wk=torch.ones(D, D), wv=torch.full((D, D), 2.0),
             wo=torch.zeros(D, D), w_gate=torch.arange(F).float()[:, None].repeat(1, D),
             w_up=-torch.arange(F).float()[:, None].repeat(1, D), w_down=torch.zeros(D, F),
             g_attn=torch.ones(D), g_mlp=torch.ones(D))
    p = mv.pack_layer(w)
    assert p["wqkv"][:, 0].tolist() == [0.0] * D + [1.0] * D + [2.0] * D
    col = p["w_gateup"][:, 0].tolist()
    assert col[:32] == list(range(32)) and col[32:64] == [-float(i) for i in range(32)]
    assert col[64:96] == list(range(32, 64))


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU; asking for more ends with a message, before any GPU work."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""
