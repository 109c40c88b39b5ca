"""ctypes binding of libmvla.so: argument marshalling only.

Every function here allocates outputs as torch tensors (device memory and
streams are PyTorch's job), passes raw pointers to the C ABI declared in
``include/mvla.h`` and raises on a non-zero status.  No step of the method is
computed in Python, and there is no fallback: if the library is missing,
``load()`` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmvla.so")
_lib = None

EXPORTS = [
    "mvla_version", "mvla_strerror", "mvla_workspace_bytes", "mvla_create", "mvla_set_stream",
    "mvla_destroy", "mvla_salience", "mvla_modality_budget", "mvla_select_topk", "mvla_compact",
    "mvla_prune_step", "mvla_rope_table", "mvla_prefill_layer", "mvla_score_only",
    "mvla_profile_enable", "mvla_profile_read", "mvla_kernel_name", "mvla_temporal_smooth",
    "mvla_modality_decompose", "mvla_feature_share", "mvla_mask_rules_default",
    "mvla_candidate_masks", "mvla_mask_indices", "mvla_prefill_layer_salience",
    "mvla_prefill_layer_prune", "mvla_tune_layers", "mvla_tuned_choice",
    "mvla_set_gemm_choice", "mvla_prefill", "mvla_peak_probe", "mvla_salience_noalloc", "mvla_masked_prefill_step",
]


class MvlaError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = load().mvla_strerror(code).decode()
        super().__init__(f"{where}: {msg} ({code})")


class LayerCfg(C.Structure):
    _fields_ = [("D", C.c_int), ("H", C.c_int), ("dh", C.c_int), ("F", C.c_int),
                ("rms_eps", C.c_float)]


class LayerWeightsC(C.Structure):
    _fields_ = [("wqkv", C.c_void_p), ("wo", C.c_void_p), ("w_gateup", C.c_void_p),
                ("w_down", C.c_void_p), ("g_attn", C.c_void_p), ("g_mlp", C.c_void_p),
                ("rope_cos", C.c_void_p), ("rope_sin", C.c_void_p), ("rope_len", C.c_int)]


class MaskRules(C.Structure):
    """Constants of Algorithm 1's mask rules (mvla_mask_rules)."""
    _fields_ = [("tau_2d", C.c_float), ("tau_3d", C.c_float), ("bg_drop", C.c_float),
                ("obj_2d_min", C.c_float), ("obj_3d_max", C.c_float),
                ("kmeans_max_iter", C.c_int32)]

    @classmethod
    def default(cls, **over) -> "MaskRules":
        r = cls()
        load().mvla_mask_rules_default(C.byref(r))
        for k, v in over.items():
            assert hasattr(r, k), k
            setattr(r, k, v)
        return r


class PrefillDesc(C.Structure):
    """mvla_prefill_desc."""
    _fields_ = [("B", C.c_int), ("n2", C.c_int), ("n3", C.c_int), ("n_text", C.c_int),
                ("k_total", C.c_int), ("min2", C.c_int), ("min3", C.c_int),
                ("n_layers", C.c_int), ("p", C.c_int), ("smooth_step", C.c_int),
                ("smooth_k", C.c_int), ("smooth_beta", C.c_double),
                ("materialise_probs", C.c_int), ("separate_prune_calls", C.c_int)]


class PrefillBuffers(C.Structure):
    """mvla_prefill_buffers."""
    _fields_ = [("h_full", C.c_void_p * 2), ("h_kept", C.c_void_p * 2), ("probs", C.c_void_p),
                ("sal", C.c_void_p), ("sal_hat", C.c_void_p), ("k2k3", C.c_void_p),
                ("kept_idx", C.c_void_p), ("pos_kept", C.c_void_p)]


class MaskedDesc(C.Structure):
    """mvla_masked_desc."""
    _fields_ = [("B", C.c_int), ("n_patch", C.c_int), ("n_text", C.c_int), ("n_layers", C.c_int),
                ("p", C.c_int), ("t", C.c_int), ("smooth_k", C.c_int), ("smooth_beta", C.c_double),
                ("rules", MaskRules)]


class MaskedBuffers(C.Structure):
    """mvla_masked_buffers."""
    _fields_ = [("h_full", C.c_void_p * 2), ("h_kept", C.c_void_p * 2), ("probs", C.c_void_p),
                ("sal", C.c_void_p), ("x_t", C.c_void_p), ("x_hat", C.c_void_p),
                ("mask2d", C.c_void_p), ("mask3d", C.c_void_p), ("sem", C.c_void_p),
                ("kept_len", C.c_void_p), ("kept_idx", C.c_void_p), ("pos_kept", C.c_void_p)]


PROBE_READ, PROBE_COPY, PROBE_MFMA, PROBE_LAUNCH = 0, 1, 2, 3


def load() -> C.CDLL:
    """Load the HIP library; raise if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} not found: build it first (python -m paper_2604_09244_amd.build)")
    lib = C.CDLL(LIB_PATH)
    vp, i, f, sz = C.c_void_p, C.c_int, C.c_float, C.c_size_t
    lib.mvla_version.restype = C.c_char_p
    lib.mvla_strerror.restype = C.c_char_p
    lib.mvla_strerror.argtypes = [i]
    lib.mvla_workspace_bytes.restype = sz
    lib.mvla_workspace_bytes.argtypes = [i] * 6
    lib.mvla_create.argtypes = [C.POINTER(vp), i, vp, vp, sz]
    lib.mvla_set_stream.argtypes = [vp, vp]
    lib.mvla_destroy.argtypes = [vp]
    lib.mvla_destroy.restype = None
    lib.mvla_salience.argtypes = [vp, vp, i, i, i, i, i, vp]
    lib.mvla_salience_noalloc.argtypes = [vp, vp, i, i, i, i, i, vp]
    lib.mvla_modality_budget.argtypes = [vp, vp, i, i, i, i, i, i, vp, vp]
    lib.mvla_select_topk.argtypes = [vp, vp, vp, i, i, i, i, i, vp]
    lib.mvla_compact.argtypes = [vp, vp, vp, vp, i, i, i, i, vp, vp]
    lib.mvla_prune_step.argtypes = [vp, vp, i, i, vp, vp, i, i, i, i, i, i, i, i, i, vp, vp, vp,
                                    vp, vp]
    lib.mvla_rope_table.argtypes = [vp, C.c_double, i, i, vp, vp]
    lib.mvla_prefill_layer.argtypes = [vp, C.POINTER(LayerCfg), C.POINTER(LayerWeightsC), vp, vp,
                                       i, i, vp, i, vp, vp]
    lib.mvla_prefill_layer_salience.argtypes = [vp, C.POINTER(LayerCfg), C.POINTER(LayerWeightsC),
                                                vp, vp, i, i, vp, i, vp, i, vp]
    lib.mvla_prefill_layer_prune.argtypes = [vp, C.POINTER(LayerCfg), C.POINTER(LayerWeightsC), vp,
                                             vp, i, i, vp, i, i, i, i, i, i, vp, vp, vp, vp, vp, vp]
    lib.mvla_tune_layers.argtypes = [vp, C.POINTER(LayerCfg), C.POINTER(LayerWeightsC), i, i, i]
    lib.mvla_set_gemm_choice.argtypes = [vp, i, i, i, i, i, i]
    lib.mvla_tuned_choice.argtypes = [vp, i, i, i, i, C.POINTER(C.c_int), C.POINTER(C.c_int)]
    lib.mvla_prefill.argtypes = [vp, C.POINTER(LayerCfg), C.POINTER(LayerWeightsC),
                                 C.POINTER(PrefillDesc), vp, vp, vp, C.POINTER(PrefillBuffers),
                                 C.POINTER(vp), C.POINTER(i)]
    lib.mvla_masked_prefill_step.argtypes = [vp, C.POINTER(LayerCfg), C.POINTER(LayerWeightsC),
                                             C.POINTER(MaskedDesc), vp, vp, vp, vp,
                                             C.POINTER(MaskedBuffers), C.POINTER(vp),
                                             C.POINTER(i), vp]
    lib.mvla_peak_probe.argtypes = [vp, i, vp, sz, i, C.POINTER(C.c_double)]
    lib.mvla_score_only.argtypes = [vp, C.POINTER(LayerCfg), C.POINTER(LayerWeightsC), vp, vp,
                                    i, i, i, vp, vp]
    lib.mvla_modality_decompose.argtypes = [vp, vp, i, i, i, i, i, vp, vp]
    lib.mvla_temporal_smooth.argtypes = [vp, vp, vp, sz, i, i, C.c_double]
    lib.mvla_feature_share.argtypes = [vp, vp, i, i, i, i, vp, vp]
    lib.mvla_mask_rules_default.argtypes = [C.POINTER(MaskRules)]
    lib.mvla_mask_rules_default.restype = None
    lib.mvla_candidate_masks.argtypes = [vp, vp, vp, vp, i, i, i, C.POINTER(MaskRules), vp, vp, vp,
                                         vp]
    lib.mvla_mask_indices.argtypes = [vp, vp, vp, i, i, i, i, vp]
    lib.mvla_profile_enable.argtypes = [vp, C.c_uint32, i]
    lib.mvla_profile_read.argtypes = [vp, i, vp, vp, vp, vp]
    lib.mvla_kernel_name.restype = C.c_char_p
    lib.mvla_kernel_name.argtypes = [i]
    _lib = lib
    return lib


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise MvlaError(rc, where)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _dev(t: torch.Tensor, dtype) -> torch.Tensor:
    assert t.is_cuda and t.dtype == dtype and t.is_contiguous(), (t.device, t.dtype)
    return t


def salience_noalloc(attn: torch.Tensor, n_vis: int, out: torch.Tensor) -> torch.Tensor:
    """mvla_salience_noalloc on the current stream: no context, no workspace; ``out`` [B, n_vis]
    must exist already (this wrapper allocates nothing either)."""
    B, H, Nq, S = _dev(attn, torch.float32).shape
    assert _dev(out, torch.float32).shape == (B, n_vis)
    stream = torch.cuda.current_stream(attn.device).cuda_stream
    _check(load().mvla_salience_noalloc(stream, attn.data_ptr(), B, H, Nq, S, n_vis,
                                        out.data_ptr()), "mvla_salience_noalloc")
    return out


def pack_layer(w: Dict[str, torch.Tensor]) -> Dict[str, torch.Tensor]:
    """Lay separate [out,in] bf16 matrices out the way the library reads them:
    q|k|v rows stacked; gate/up rows interleaved in blocks of 32."""
    F, D = w["w_gate"].shape
    assert F % 32 == 0
    gu = torch.stack([w["w_gate"].view(F // 32, 32, D), w["w_up"].view(F // 32, 32, D)], dim=1)
    return dict(wqkv=torch.cat([w["wq"], w["wk"], w["wv"]], dim=0).contiguous(),
                wo=w["wo"].contiguous(), w_gateup=gu.reshape(2 * F, D).contiguous(),
                w_down=w["w_down"].contiguous(), g_attn=w["g_attn"].contiguous(),
                g_mlp=w["g_mlp"].contiguous())


class Context:
    """Owns a device workspace and a library context bound to the current stream."""

    def __init__(self, B: int, S: int, D: int, H: int, F: int, n_query_tail: int = 0,
                 device: Optional[torch.device] = None):
        lib = load()
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the HIP path has no CPU fallback")
        self.device = torch.device("cuda", torch.cuda.current_device()) if device is None else device
        nbytes = lib.mvla_workspace_bytes(B, S, D, H, F, n_query_tail)
        if nbytes == 0:
            raise MvlaError(-1, "mvla_workspace_bytes")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self._h = C.c_void_p()
        stream = torch.cuda.current_stream(self.device).cuda_stream
        _check(lib.mvla_create(C.byref(self._h), self.device.index or 0, stream,
                               self.workspace.data_ptr(), nbytes), "mvla_create")
        self._rope = {}

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            load().mvla_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def handle(self):
        return self._h

    def set_stream(self, stream: torch.cuda.Stream):
        _check(load().mvla_set_stream(self._h, stream.cuda_stream), "mvla_set_stream")

    # ---- timing ----------------------------------------------------------
    def profile_enable(self, kernel_ids: Optional[Sequence[int]], max_records: int = 4096):
        """kernel_ids None = all kernels, [] = off."""
        mask = 0xFFFFFFFF if kernel_ids is None else sum(1 << k for k in kernel_ids)
        _check(load().mvla_profile_enable(self._h, mask, max_records), "mvla_profile_enable")
        self._prof_cap = max_records

    def profile_read(self):
        """-> list of (kernel name, tag, milliseconds) in launch order."""
        cap = getattr(self, "_prof_cap", 0)
        ids = (C.c_int32 * max(cap, 1))()
        tags = (C.c_int32 * max(cap, 1))()
        ms = (C.c_float * max(cap, 1))()
        n = C.c_int32(0)
        _check(load().mvla_profile_read(self._h, cap, ids, tags, ms, C.byref(n)),
               "mvla_profile_read")
        lib = load()
        return [(lib.mvla_kernel_name(ids[j]).decode(), tags[j], ms[j]) for j in range(n.value)]

    # ---- pruning step --------------------------------------------------
    def salience(self, attn: torch.Tensor, n_vis: int, out: Optional[torch.Tensor] = None):
        B, H, Nq, S = _dev(attn, torch.float32).shape
        sal = torch.empty(B, n_vis, dtype=torch.float32, device=attn.device) if out is None else out
        _check(load().mvla_salience(self._h, attn.data_ptr(), B, H, Nq, S, n_vis, sal.data_ptr()),
               "mvla_salience")
        return sal

    def modality_budget(self, sal: torch.Tensor, n2: int, n3: int, k_total: int, min2: int = 0,
                        min3: int = 0, want_mass: bool = False,
                        out: Optional[torch.Tensor] = None):
        B = _dev(sal, torch.float32).shape[0]
        k2k3 = torch.empty(B, 2, dtype=torch.int32, device=sal.device) if out is None else out
        mass = torch.empty(B, 2, dtype=torch.float32, device=sal.device) if want_mass else None
        _check(load().mvla_modality_budget(self._h, sal.data_ptr(), B, n2, n3, k_total, min2, min3,
                                           k2k3.data_ptr(), _ptr(mass)), "mvla_modality_budget")
        return (k2k3, mass) if want_mass else k2k3

    def select_topk(self, sal: torch.Tensor, k2k3: torch.Tensor, n2: int, n3: int, n_text: int,
                    k_total: int, out: Optional[torch.Tensor] = None):
        B = _dev(sal, torch.float32).shape[0]
        _dev(k2k3, torch.int32)
        kept = (torch.empty(B, k_total + n_text, dtype=torch.int32, device=sal.device)
                if out is None else out)
        _check(load().mvla_select_topk(self._h, sal.data_ptr(), k2k3.data_ptr(), B, n2, n3, n_text,
                                       k_total, kept.data_ptr()), "mvla_select_topk")
        return kept

    def compact(self, h: torch.Tensor, pos: torch.Tensor, kept: torch.Tensor,
                out: Optional[Sequence[torch.Tensor]] = None):
        B, S, D = _dev(h, torch.bfloat16).shape
        _dev(pos, torch.int32)
        S_out = _dev(kept, torch.int32).shape[1]
        if out is None:
            h_out = torch.empty(B, S_out, D, dtype=torch.bfloat16, device=h.device)
            pos_out = torch.empty(B, S_out, dtype=torch.int32, device=h.device)
        else:
            h_out, pos_out = out
        _check(load().mvla_compact(self._h, h.data_ptr(), pos.data_ptr(), kept.data_ptr(), B, S,
                                   S_out, D, h_out.data_ptr(), pos_out.data_ptr()), "mvla_compact")
        return h_out, pos_out

    def modality_decompose(self, attn: torch.Tensor, n_patch: int, out=None):
        """Per-patch (M2D, M3D) of Eqs. 5-6 from the language-query attention rows."""
        B, H, Nq, S = _dev(attn, torch.float32).shape
        if out is None:
            m2d = torch.empty(B, n_patch, dtype=torch.float32, device=attn.device)
            m3d = torch.empty_like(m2d)
        else:
            m2d, m3d = out
        _check(load().mvla_modality_decompose(self._h, attn.data_ptr(), B, H, Nq, S, n_patch,
                                              m2d.data_ptr(), m3d.data_ptr()),
               "mvla_modality_decompose")
        return m2d, m3d

    def temporal_smooth(self, x_t: torch.Tensor, x_hat: torch.Tensor, t: int, k: int = 7,
                        beta: float = 0.85):
        """In-place update of x_hat with the observation x_t at step t (1-based)."""
        _dev(x_t, torch.float32)
        _dev(x_hat, torch.float32)
        assert x_t.numel() == x_hat.numel()
        _check(load().mvla_temporal_smooth(self._h, x_t.data_ptr(), x_hat.data_ptr(), x_t.numel(),
                                           t, k, beta), "mvla_temporal_smooth")
        return x_hat

    def feature_share(self, feat: torch.Tensor, n_patch: int, out=None):
        """Per-patch (M2D, M3D) of Eq. 1 from token features [B, S, D]."""
        B, S, D = _dev(feat, torch.bfloat16).shape
        if out is None:
            m2d = torch.empty(B, n_patch, dtype=torch.float32, device=feat.device)
            m3d = torch.empty_like(m2d)
        else:
            m2d, m3d = out
        _check(load().mvla_feature_share(self._h, feat.data_ptr(), B, S, D, n_patch,
                                         m2d.data_ptr(), m3d.data_ptr()), "mvla_feature_share")
        return m2d, m3d

    def candidate_masks(self, x_hat: torch.Tensor, sal: torch.Tensor, u: torch.Tensor,
                        n_text: int, rules: Optional[MaskRules] = None, out=None):
        """Retention masks of Algorithm 1 from smoothed indicators [4, B, P], salience [B, 2P]
        and uniform draws [B, P].  Returns (mask2d, mask3d, sem, kept_len)."""
        four, B, P = _dev(x_hat, torch.float32).shape
        assert four == 4 and _dev(sal, torch.float32).shape == (B, 2 * P)
        assert _dev(u, torch.float32).shape == (B, P)
        rules = rules or MaskRules.default()
        if out is None:
            mask2d = torch.empty(B, P, dtype=torch.uint8, device=sal.device)
            mask3d = torch.empty_like(mask2d)
            sem = torch.empty_like(mask2d)
            kept_len = torch.empty(B, dtype=torch.int32, device=sal.device)
        else:
            mask2d, mask3d, sem, kept_len = out
        _check(load().mvla_candidate_masks(self._h, x_hat.data_ptr(), sal.data_ptr(), u.data_ptr(),
                                           B, P, n_text, C.byref(rules), mask2d.data_ptr(),
                                           mask3d.data_ptr(), _ptr(sem), kept_len.data_ptr()),
               "mvla_candidate_masks")
        return mask2d, mask3d, sem, kept_len

    def mask_indices(self, mask2d: torch.Tensor, mask3d: torch.Tensor, n_text: int, S_pad: int,
                     out: Optional[torch.Tensor] = None):
        B, P = _dev(mask2d, torch.uint8).shape
        assert _dev(mask3d, torch.uint8).shape == (B, P)
        if out is None:
            out = torch.empty(B, S_pad, dtype=torch.int32, device=mask2d.device)
        assert out.shape == (B, S_pad) and out.dtype == torch.int32 and out.is_contiguous()
        _check(load().mvla_mask_indices(self._h, mask2d.data_ptr(), mask3d.data_ptr(), B, P,
                                        n_text, S_pad, out.data_ptr()), "mvla_mask_indices")
        return out

    def prune_step(self, attn, h, pos, n2, n3, n_text, k_total, min2=0, min3=0, out=None):
        B, H, Nq, S = _dev(attn, torch.float32).shape
        D = _dev(h, torch.bfloat16).shape[2]
        dev = h.device
        if out is None:
            out = dict(sal=torch.empty(B, n2 + n3, dtype=torch.float32, device=dev),
                       k2k3=torch.empty(B, 2, dtype=torch.int32, device=dev),
                       kept_idx=torch.empty(B, k_total + n_text, dtype=torch.int32, device=dev),
                       h=torch.empty(B, k_total + n_text, D, dtype=torch.bfloat16, device=dev),
                       pos=torch.empty(B, k_total + n_text, dtype=torch.int32, device=dev))
        _check(load().mvla_prune_step(self._h, attn.data_ptr(), H, Nq, h.data_ptr(),
                                      _dev(pos, torch.int32).data_ptr(), B, S, D, n2, n3, n_text,
                                      k_total, min2, min3, out["sal"].data_ptr(),
                                      out["k2k3"].data_ptr(), out["kept_idx"].data_ptr(),
                                      out["h"].data_ptr(), out["pos"].data_ptr()), "mvla_prune_step")
        return out

    # ---- backbone layer --------------------------------------------------
    def rope_table(self, base: float, rope_len: int, dh: int):
        key = (float(base), int(rope_len), int(dh))
        if key not in self._rope:
            c = torch.empty(rope_len, dh // 2, dtype=torch.float32, device=self.device)
            s = torch.empty_like(c)
            _check(load().mvla_rope_table(self._h, base, rope_len, dh, c.data_ptr(), s.data_ptr()),
                   "mvla_rope_table")
            self._rope[key] = (c, s)
        return self._rope[key]

    def layer_struct(self, packed: Dict[str, torch.Tensor], rope) -> LayerWeightsC:
        for k in ("wqkv", "wo", "w_gateup", "w_down", "g_attn", "g_mlp"):
            _dev(packed[k], torch.bfloat16)
        c, s = rope
        w = LayerWeightsC(packed["wqkv"].data_ptr(), packed["wo"].data_ptr(),
                          packed["w_gateup"].data_ptr(), packed["w_down"].data_ptr(),
                          packed["g_attn"].data_ptr(), packed["g_mlp"].data_ptr(),
                          c.data_ptr(), s.data_ptr(), c.shape[0])
        # the descriptor holds bare device addresses: the tensors live as long as it does (a caller
        # that passes a temporary would otherwise leave it pointing at freed memory)
        w._keep_alive = (packed, rope)
        return w

    def prefill_layer(self, cfg: LayerCfg, w: LayerWeightsC, x: torch.Tensor, pos: torch.Tensor,
                      y: Optional[torch.Tensor] = None, n_query_tail: int = 0,
                      key_bias: Optional[torch.Tensor] = None,
                      probs_out: Optional[torch.Tensor] = None):
        B, S, D = _dev(x, torch.bfloat16).shape
        _dev(pos, torch.int32)
        y = torch.empty_like(x) if y is None else y
        if n_query_tail > 0 and probs_out is None:
            probs_out = torch.empty(B, cfg.H, n_query_tail, S, dtype=torch.float32, device=x.device)
        if key_bias is not None:
            _dev(key_bias, torch.float32)
        _check(load().mvla_prefill_layer(self._h, C.byref(cfg), C.byref(w), x.data_ptr(),
                                         pos.data_ptr(), B, S, y.data_ptr(), n_query_tail,
                                         _ptr(key_bias), _ptr(probs_out)), "mvla_prefill_layer")
        return (y, probs_out) if n_query_tail > 0 else y

    def prefill_layer_salience(self, cfg: LayerCfg, w: LayerWeightsC, x: torch.Tensor,
                               pos: torch.Tensor, n_query_tail: int, n_vis: int,
                               y: Optional[torch.Tensor] = None,
                               key_bias: Optional[torch.Tensor] = None,
                               sal: Optional[torch.Tensor] = None):
        """Layer + salience of its last n_query_tail rows, without materialising the
        probabilities.  Returns (y, sal [B, n_vis])."""
        B, S, D = _dev(x, torch.bfloat16).shape
        _dev(pos, torch.int32)
        y = torch.empty_like(x) if y is None else y
        if sal is None:
            sal = torch.empty(B, n_vis, dtype=torch.float32, device=x.device)
        if key_bias is not None:
            _dev(key_bias, torch.float32)
        _check(load().mvla_prefill_layer_salience(self._h, C.byref(cfg), C.byref(w), x.data_ptr(),
                                                  pos.data_ptr(), B, S, y.data_ptr(), n_query_tail,
                                                  _ptr(key_bias), n_vis, sal.data_ptr()),
               "mvla_prefill_layer_salience")
        return y, sal

    def prefill_layer_prune(self, cfg: LayerCfg, w: LayerWeightsC, x: torch.Tensor,
                            pos: torch.Tensor, y: torch.Tensor, n2: int, n3: int, n_text: int,
                            k_total: int, key_bias: Optional[torch.Tensor] = None, min2: int = 0,
                            min3: int = 0, out=None):
        """Last full-sequence layer + salience + budget + selection + gather in one call.
        ``out``: dict(sal, k2k3, kept_idx, h, pos) of pre-allocated tensors (as prune_step)."""
        B, S, D = _dev(x, torch.bfloat16).shape
        dev = x.device
        if out is None:
            out = dict(sal=torch.empty(B, n2 + n3, dtype=torch.float32, device=dev),
                       k2k3=torch.empty(B, 2, dtype=torch.int32, device=dev),
                       kept_idx=torch.empty(B, k_total + n_text, dtype=torch.int32, device=dev),
                       h=torch.empty(B, k_total + n_text, D, dtype=torch.bfloat16, device=dev),
                       pos=torch.empty(B, k_total + n_text, dtype=torch.int32, device=dev))
        _check(load().mvla_prefill_layer_prune(
            self._h, C.byref(cfg), C.byref(w), x.data_ptr(), pos.data_ptr(), B, S, y.data_ptr(), n2,
            n3, n_text, k_total, min2, min3, _ptr(key_bias), out["sal"].data_ptr(),
            out["k2k3"].data_ptr(), out["kept_idx"].data_ptr(), out["h"].data_ptr(),
            out["pos"].data_ptr()), "mvla_prefill_layer_prune")
        return out

    def tune_layers(self, cfg: LayerCfg, structs: Sequence[LayerWeightsC], B: int, S: int):
        """Measure the projection kernels' tile configurations at M = B*S rows and keep the
        fastest per shape in this context (synchronises the stream)."""
        arr = (LayerWeightsC * len(structs))(*structs)
        _check(load().mvla_tune_layers(self._h, C.byref(cfg), arr, len(structs), B, S),
               "mvla_tune_layers")

    def set_gemm_choice(self, M: int, N: int, K: int, epilogue: int, cfg: int, split_pct: int = 50):
        _check(load().mvla_set_gemm_choice(self._h, M, N, K, epilogue, cfg, split_pct),
               "mvla_set_gemm_choice")

    def tuned_choice(self, M: int, N: int, K: int, epilogue: int):
        c, p = C.c_int(), C.c_int()
        _check(load().mvla_tuned_choice(self._h, M, N, K, epilogue, C.byref(c), C.byref(p)),
               "mvla_tuned_choice")
        return c.value, p.value

    def peak_probe(self, kind: int, buf: Optional[torch.Tensor], reps: int = 10) -> float:
        """Measured rate of a probe kernel (synchronises): GB/s for PROBE_READ / PROBE_COPY,
        TFLOP/s for PROBE_MFMA (operands: the first 8 KiB of buf), microseconds per launch for
        PROBE_LAUNCH."""
        out = C.c_double(0.0)
        nbytes = 0 if buf is None else buf.numel() * buf.element_size()
        _check(load().mvla_peak_probe(self._h, kind, _ptr(buf), nbytes, reps, C.byref(out)),
               "mvla_peak_probe")
        return out.value

    def score_only(self, cfg: LayerCfg, w: LayerWeightsC, x, pos, n_query_tail, key_bias=None,
                   probs_out=None):
        B, S, D = _dev(x, torch.bfloat16).shape
        if probs_out is None:
            probs_out = torch.empty(B, cfg.H, n_query_tail, S, dtype=torch.float32, device=x.device)
        _check(load().mvla_score_only(self._h, C.byref(cfg), C.byref(w), x.data_ptr(),
                                      _dev(pos, torch.int32).data_ptr(), B, S, n_query_tail,
                                      _ptr(key_bias), probs_out.data_ptr()), "mvla_score_only")
        return probs_out


class PrefillPlan:
    """Pre-allocated buffers and packed weights for one workload; ``run`` hands them to
    mvla_prefill (no allocation, no host synchronisation, no torch operation)."""

    def __init__(self, ctx: Context, cfg: LayerCfg, layers: List[Dict[str, torch.Tensor]],
                 B: int, n2: int, n3: int, nt: int, k_total: int, p: int,
                 rope_base: float = 10000.0, rope_len: Optional[int] = None, tune: bool = False):
        self.ctx, self.cfg, self.B, self.n2, self.n3, self.nt = ctx, cfg, B, n2, n3, nt
        self.k_total, self.p, self.L = k_total, p, len(layers)
        self.S, self.S_kept = n2 + n3 + nt, k_total + nt
        dev = ctx.device
        self.rope = ctx.rope_table(rope_base, rope_len or self.S, cfg.dh)
        self.packed = layers
        self.structs = [ctx.layer_struct(l, self.rope) for l in layers]
        if tune:   # measured kernel choices for the two row counts this plan runs at
            ctx.tune_layers(cfg, self.structs, B, self.S)
            if self.S_kept != self.S and self.S_kept > 0:
                ctx.tune_layers(cfg, self.structs, B, self.S_kept)
        bf, i32, f32 = torch.bfloat16, torch.int32, torch.float32
        self.h_full = [torch.empty(B, self.S, cfg.D, dtype=bf, device=dev) for _ in range(2)]
        self.h_kept = [torch.empty(B, self.S_kept, cfg.D, dtype=bf, device=dev) for _ in range(2)]
        self.probs = torch.empty(B, cfg.H, nt, self.S, dtype=f32, device=dev)
        self.sal_hat = torch.zeros(B, n2 + n3, dtype=f32, device=dev)   # smoothed salience state
        self.prune = dict(sal=torch.empty(B, n2 + n3, dtype=f32, device=dev),
                          k2k3=torch.empty(B, 2, dtype=i32, device=dev),
                          kept_idx=torch.empty(B, self.S_kept, dtype=i32, device=dev),
                          h=self.h_kept[0],
                          pos=torch.empty(B, self.S_kept, dtype=i32, device=dev))
        self._layer_array = (LayerWeightsC * len(self.structs))(*self.structs)
        hf, hk = (C.c_void_p * 2), (C.c_void_p * 2)
        self._buffers = PrefillBuffers(hf(*[t.data_ptr() for t in self.h_full]),
                                       hk(*[t.data_ptr() for t in self.h_kept]),
                                       self.probs.data_ptr(), self.prune["sal"].data_ptr(),
                                       self.sal_hat.data_ptr(), self.prune["k2k3"].data_ptr(),
                                       self.prune["kept_idx"].data_ptr(),
                                       self.prune["pos"].data_ptr())

    def run(self, x: torch.Tensor, pos: torch.Tensor, key_bias: Optional[torch.Tensor] = None,
            fused_prune: bool = True, smooth_step: int = 0, smooth_k: int = 7,
            smooth_beta: float = 0.85, on_the_fly: bool = False):
        """Pruned prefill: p full layers, pruning step, L-p layers on kept tokens -- one call
        of mvla_prefill, which does the sequencing.

        smooth_step > 0 turns on the action-iteration smoothing of the salience: the call is
        timestep ``smooth_step`` (1-based) of an episode; step 1 is the cold start and returns
        the unpruned prefill, later steps select on the smoothed salience.  ``on_the_fly``
        reduces the scoring rows inside the scoring kernel (no probability tensor)."""
        _dev(x, torch.bfloat16)
        _dev(pos, torch.int32)
        if key_bias is not None:
            _dev(key_bias, torch.float32)
        d = PrefillDesc(self.B, self.n2, self.n3, self.nt, self.k_total, 0, 0, self.L, self.p,
                        smooth_step, smooth_k, smooth_beta, 0 if on_the_fly else 1,
                        0 if fused_prune else 1)
        y_ptr, rows = C.c_void_p(), C.c_int()
        _check(load().mvla_prefill(self.ctx.handle, C.byref(self.cfg), self._layer_array,
                                   C.byref(d), x.data_ptr(), pos.data_ptr(), _ptr(key_bias),
                                   C.byref(self._buffers), C.byref(y_ptr), C.byref(rows)),
               "mvla_prefill")
        for t in self.h_kept + self.h_full:          # which of the plan's tensors holds the result
            if t.data_ptr() == y_ptr.value:
                assert t.shape[1] == rows.value
                return t
        raise RuntimeError("mvla_prefill returned a pointer outside the plan's buffers")

    def run_unpruned(self, x: torch.Tensor, pos: torch.Tensor):
        h = x
        for li in range(self.L):
            y = self.h_full[li & 1]
            self.ctx.prefill_layer(self.cfg, self.structs[li], h, pos, y)
            h = y
        return h


class MaskedPrefill:
    """One episode of action iterations with the masks of Algorithm 1 (needs one 3D token per
    2D token and p >= 1): buffers for mvla_masked_prefill_step, which sequences the step (p
    layers on all tokens, the four per-patch indicators, their smoothing, and for t > 1 the
    masks, the index scan, the gather and the remaining layers).  The kept length differs per
    sample; rows are padded at the end up to the longest sample of the step, which takes one
    read-back of B integers inside the call."""

    def __init__(self, plan: PrefillPlan, rules: Optional[MaskRules] = None, k: int = 7,
                 beta: float = 0.85):
        assert plan.n2 == plan.n3 and plan.p >= 1
        self.plan, self.rules, self.k, self.beta = plan, rules or MaskRules.default(), k, beta
        B, P, S, D = plan.B, plan.n2, plan.S, plan.cfg.D
        dev = plan.ctx.device
        f32, u8, i32 = torch.float32, torch.uint8, torch.int32
        self.P = P
        self.x_t = torch.zeros(4, B, P, dtype=f32, device=dev)
        self.x_hat = torch.zeros(4, B, P, dtype=f32, device=dev)
        self.sal = torch.empty(B, 2 * P, dtype=f32, device=dev)
        self.mask2d = torch.empty(B, P, dtype=u8, device=dev)
        self.mask3d = torch.empty(B, P, dtype=u8, device=dev)
        self.sem = torch.empty(B, P, dtype=u8, device=dev)
        self.kept_len = torch.empty(B, dtype=i32, device=dev)
        self.kept_idx = torch.empty(B * S, dtype=i32, device=dev)
        self.pos_kept = torch.empty(B * S, dtype=i32, device=dev)
        self.h_kept = [torch.empty(B * S * D, dtype=torch.bfloat16, device=dev) for _ in range(2)]
        two = C.c_void_p * 2
        self._buffers = MaskedBuffers(two(*[t.data_ptr() for t in plan.h_full]),
                                      two(*[t.data_ptr() for t in self.h_kept]),
                                      plan.probs.data_ptr(), self.sal.data_ptr(),
                                      self.x_t.data_ptr(), self.x_hat.data_ptr(),
                                      self.mask2d.data_ptr(), self.mask3d.data_ptr(),
                                      self.sem.data_ptr(), self.kept_len.data_ptr(),
                                      self.kept_idx.data_ptr(), self.pos_kept.data_ptr())

    def step(self, t: int, x: torch.Tensor, pos: torch.Tensor, u: torch.Tensor,
             key_bias: Optional[torch.Tensor] = None):
        """Timestep t (1-based): one call of mvla_masked_prefill_step.  Returns
        (y [B, S_pad, D], lengths): row i of sample b is valid for i < lengths[b]; at t == 1
        nothing is pruned."""
        pl = self.plan
        B, S, D = pl.B, pl.S, pl.cfg.D
        _dev(x, torch.bfloat16)
        _dev(pos, torch.int32)
        _dev(u, torch.float32)
        if key_bias is not None:
            _dev(key_bias, torch.float32)
        d = MaskedDesc(B, self.P, pl.nt, pl.L, pl.p, t, self.k, self.beta, self.rules)
        y_ptr, rows = C.c_void_p(), C.c_int()
        lengths = (C.c_int32 * B)()
        _check(load().mvla_masked_prefill_step(pl.ctx.handle, C.byref(pl.cfg), pl._layer_array,
                                               C.byref(d), x.data_ptr(), pos.data_ptr(),
                                               _ptr(key_bias), u.data_ptr(),
                                               C.byref(self._buffers), C.byref(y_ptr),
                                               C.byref(rows), lengths), "mvla_masked_prefill_step")
        S_pad = rows.value
        for buf in pl.h_full + self.h_kept:            # which buffer holds the result
            if buf.data_ptr() == y_ptr.value:
                y = buf.view(-1)[:B * S_pad * D].view(B, S_pad, D)
                break
        else:
            raise RuntimeError("mvla_masked_prefill_step returned a pointer outside the buffers")
        if t > 1:
            self.kept = self.kept_idx[:B * S_pad].view(B, S_pad)
            self.pos_out = self.pos_kept[:B * S_pad].view(B, S_pad)
        return y, list(lengths)
