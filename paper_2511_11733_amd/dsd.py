"""ctypes binding of libdsd.so: argument marshalling only, every step runs in the HIP library.

The function names are those of include/dsd.h.  Device buffers are torch tensors (PyTorch is
used for device memory and streams, nothing else); the wrappers check dtype, device and
contiguity and hand raw pointers to the C ABI.  There is no fallback: if the shared library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdsd.so")

DSD_F32, DSD_BF16 = 0, 1
DSD_TREE_LONGEST, DSD_TREE_FIRST_ACCEPTED = 0, 1
DSD_MAX_K, DSD_MAX_TOP_M = 64, 16

EXPORTS = [
    "dsd_last_error", "dsd_create", "dsd_destroy", "dsd_set_stream", "dsd_weights_create", "dsd_weights_destroy",
    "dsd_kv_create", "dsd_kv_destroy", "dsd_kv_import", "dsd_kv_export", "dsd_kv_set_len", "dsd_kv_get_len",
    "dsd_stage_verify", "dsd_stage_status", "dsd_accept", "dsd_accept_noalloc", "dsd_kv_commit", "dsd_profile_enable", "dsd_profile_read", "dsd_stream_probe",
]
KERNEL_CLASSES = ["qkv", "attn", "attn_combine", "oproj", "gateup", "down", "head", "accept", "other"]


class DsdError(RuntimeError):
    pass


class ModelDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("dtype", C.c_int32), ("has_embed", C.c_int32), ("has_head", C.c_int32),
                ("rope_theta", C.c_float), ("rms_eps", C.c_float)]


class AcceptParams(C.Structure):
    _fields_ = [("lambda1", C.c_double), ("lambda2", C.c_double), ("lambda3", C.c_double), ("tau", C.c_double),
                ("temperature", C.c_double), ("top_m", C.c_int32), ("tree_mode", C.c_int32),
                ("tau_override", C.c_void_p), ("norm_match_kind", C.c_int32), ("entropy_kind", C.c_int32)]


class AcceptStats(C.Structure):
    _fields_ = [("key_flags", C.c_void_p), ("node_accept", C.c_void_p), ("ratio", C.c_void_p),
                ("norm_match", C.c_void_p)]


_lib = None


def load() -> C.CDLL:
    """Loads libdsd.so from the package directory (built by paper_2511_11733_amd/build.py)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise DsdError(f"{LIB_PATH} is missing: build it with `python -m paper_2511_11733_amd.build`")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int, C.c_int64
    lib.dsd_last_error.restype = C.c_char_p
    lib.dsd_last_error.argtypes = []
    sig = {
        "dsd_create": [i32, vp, C.POINTER(vp)],
        "dsd_destroy": [vp],
        "dsd_set_stream": [vp, vp],
        "dsd_weights_create": [vp, C.POINTER(ModelDesc), C.POINTER(vp), i32, C.POINTER(vp)],
        "dsd_weights_destroy": [vp, vp],
        "dsd_kv_create": [vp, C.POINTER(ModelDesc), i32, i32, C.POINTER(vp)],
        "dsd_kv_destroy": [vp, vp],
        "dsd_kv_import": [vp, vp, i32, vp, vp, i32, i32],
        "dsd_kv_export": [vp, vp, i32, i32, i32, i32, vp, vp],
        "dsd_kv_set_len": [vp, vp, C.POINTER(C.c_int32), i32],
        "dsd_kv_get_len": [vp, vp, C.POINTER(C.c_int32), i32],
        "dsd_stage_verify": [vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, i64],
        "dsd_stage_status": [vp, C.POINTER(C.c_int64)],
        "dsd_accept": [vp, vp, vp, vp, vp, vp, C.POINTER(AcceptParams), i32, i32, i32, vp, vp, vp,
                       C.POINTER(AcceptStats)],
        "dsd_accept_noalloc": [vp, vp, vp, vp, vp, vp, C.POINTER(AcceptParams), i32, i32, i32, vp, vp, vp,
                               C.POINTER(AcceptStats)],
        "dsd_kv_commit": [vp, vp, vp, vp, i32, i32],
        "dsd_profile_enable": [vp, i32],
        "dsd_profile_read": [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64)],
        "dsd_stream_probe": [vp, vp, C.c_size_t, i32, i32, C.POINTER(C.c_double)],
    }
    for name, args in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = C.c_int
    _lib = lib
    return lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise DsdError(f"{what} failed ({rc}): {load().dsd_last_error().decode()}")


def _ptr(t: Optional[torch.Tensor], dtype=None, name: str = "tensor") -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise DsdError(f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise DsdError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise DsdError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def model_desc(m) -> ModelDesc:
    """From a workloads.ModelCfg-like object."""
    return ModelDesc(m.L, m.d, m.Hq, m.Hkv, m.hd, m.F, m.V, DSD_BF16 if m.dtype == "bf16" else DSD_F32,
                     int(m.has_embed), int(m.has_head), float(m.rope_theta), float(m.eps))


def torch_dtype(desc: ModelDesc):
    return torch.bfloat16 if desc.dtype == DSD_BF16 else torch.float32


class Context:
    """dsd_ctx on the current torch device and stream."""

    def __init__(self, device: int = 0, stream: Optional[torch.cuda.Stream] = None):
        self.lib = load()
        self.device = device
        h = C.c_void_p()
        sp = None if stream is None else stream.cuda_stream
        _check(self.lib.dsd_create(device, sp, C.byref(h)), "dsd_create")
        self.h = h

    def set_stream(self, stream: Optional[torch.cuda.Stream]) -> None:
        _check(self.lib.dsd_set_stream(self.h, None if stream is None else stream.cuda_stream), "dsd_set_stream")

    def profile_enable(self, on: bool) -> None:
        _check(self.lib.dsd_profile_enable(self.h, int(on)), "dsd_profile_enable")

    def profile_read(self) -> dict:
        """{kernel class: (total ms, launches)} since the last read."""
        n = len(KERNEL_CLASSES)
        ms = (C.c_double * n)()
        cnt = (C.c_int64 * n)()
        _check(self.lib.dsd_profile_read(self.h, ms, cnt), "dsd_profile_read")
        return {KERNEL_CLASSES[i]: (ms[i], cnt[i]) for i in range(n)}

    def stage_status(self) -> int:
        """Synchronises; raises DsdError if activations left the fp16 range since the last check, else returns 0."""
        n = C.c_int64()
        rc = self.lib.dsd_stage_status(self.h, C.byref(n))
        _check(rc, "dsd_stage_status")
        return n.value

    def stream_probe(self, buf: torch.Tensor, mode: int, iters: int) -> float:
        """Average milliseconds of one launch of the bare read (mode 0; 3: non-temporal loads; 2: one stream per
        wave) / copy (mode 1) kernel over buf."""
        ms = C.c_double()
        _check(self.lib.dsd_stream_probe(self.h, _ptr(buf, None, "buf"), buf.numel() * buf.element_size(), mode, iters,
                                         C.byref(ms)), "dsd_stream_probe")
        return ms.value

    def close(self) -> None:
        if self.h:
            self.lib.dsd_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Weights:
    def __init__(self, ctx: Context, desc: ModelDesc, tensors: Sequence[torch.Tensor]):
        self.ctx, self.desc = ctx, desc
        dt = torch_dtype(desc)
        ptrs = (C.c_void_p * len(tensors))(*[_ptr(t, dt, f"weight {i}") for i, t in enumerate(tensors)])
        h = C.c_void_p()
        _check(ctx.lib.dsd_weights_create(ctx.h, C.byref(desc), ptrs, len(tensors), C.byref(h)), "dsd_weights_create")
        self.h = h

    def close(self) -> None:
        if self.h and self.ctx.h:
            self.ctx.lib.dsd_weights_destroy(self.ctx.h, self.h)
        self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class KVCache:
    def __init__(self, ctx: Context, desc: ModelDesc, max_batch: int, max_slots: int):
        self.ctx, self.desc = ctx, desc
        h = C.c_void_p()
        _check(ctx.lib.dsd_kv_create(ctx.h, C.byref(desc), max_batch, max_slots, C.byref(h)), "dsd_kv_create")
        self.h = h

    def import_layer(self, layer: int, k: torch.Tensor, v: torch.Tensor) -> None:
        """k, v: [B, Hkv, n_slots, hd] in the model dtype."""
        dt = torch_dtype(self.desc)
        B, _, n, _ = k.shape
        _check(self.ctx.lib.dsd_kv_import(self.ctx.h, self.h, layer, _ptr(k, dt, "k"), _ptr(v, dt, "v"), B, n),
               "dsd_kv_import")

    def export_layer(self, layer: int, first_slot: int, n_slots: int, B: int):
        dt = torch_dtype(self.desc)
        shape = (B, self.desc.n_kv_heads, n_slots, self.desc.head_dim)
        k = torch.empty(shape, dtype=dt, device=f"cuda:{self.ctx.device}")
        v = torch.empty_like(k)
        _check(self.ctx.lib.dsd_kv_export(self.ctx.h, self.h, layer, first_slot, n_slots, B, k.data_ptr(), v.data_ptr()),
               "dsd_kv_export")
        return k, v

    def set_len(self, lens: Sequence[int]) -> None:
        arr = (C.c_int32 * len(lens))(*[int(x) for x in lens])
        _check(self.ctx.lib.dsd_kv_set_len(self.ctx.h, self.h, arr, len(lens)), "dsd_kv_set_len")

    def get_len(self, B: int):
        arr = (C.c_int32 * B)()
        _check(self.ctx.lib.dsd_kv_get_len(self.ctx.h, self.h, arr, B), "dsd_kv_get_len")
        return list(arr)

    def close(self) -> None:
        if self.h and self.ctx.h:
            self.ctx.lib.dsd_kv_destroy(self.ctx.h, self.h)
        self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def dsd_stage_verify(ctx: Context, w: Weights, kv: KVCache, hidden_in: Optional[torch.Tensor],
                     draft_tokens: Optional[torch.Tensor], tree_mask: Optional[torch.Tensor],
                     depth: Optional[torch.Tensor], B: int, k: int, hidden_out: Optional[torch.Tensor],
                     logits: Optional[torch.Tensor], logits_seq_stride: int = 0, logits_offset: int = 0) -> None:
    """logits_offset (elements) lets the k rows land behind a root row kept in the same buffer."""
    dt = torch_dtype(w.desc)
    lp = _ptr(logits, torch.float32, "logits")
    if lp is not None:
        lp += 4 * logits_offset
    _check(ctx.lib.dsd_stage_verify(ctx.h, w.h, kv.h, _ptr(hidden_in, dt, "hidden_in"),
                                    _ptr(draft_tokens, torch.int32, "draft_tokens"),
                                    _ptr(tree_mask, torch.int64, "tree_mask"), _ptr(depth, torch.int32, "depth"),
                                    B, k, _ptr(hidden_out, dt, "hidden_out"), lp, logits_seq_stride),
           "dsd_stage_verify")


def dsd_accept(ctx: Context, logits: torch.Tensor, draft_probs: torch.Tensor, draft_tokens: torch.Tensor,
               parent: Optional[torch.Tensor], uniforms: torch.Tensor, params: AcceptParams, B: int, k: int, V: int,
               accepted_len: torch.Tensor, next_token: torch.Tensor, accepted_path: Optional[torch.Tensor] = None,
               stats: Optional[AcceptStats] = None) -> None:
    _check(ctx.lib.dsd_accept(ctx.h, _ptr(logits, torch.float32, "logits"),
                              _ptr(draft_probs, torch.float32, "draft_probs"),
                              _ptr(draft_tokens, torch.int32, "draft_tokens"), _ptr(parent, torch.int32, "parent"),
                              _ptr(uniforms, torch.float32, "uniforms"), C.byref(params), B, k, V,
                              _ptr(accepted_len, torch.int32, "accepted_len"),
                              _ptr(next_token, torch.int32, "next_token"),
                              _ptr(accepted_path, torch.int32, "accepted_path"),
                              None if stats is None else C.byref(stats)), "dsd_accept")


def dsd_accept_noalloc(ctx: Context, logits: torch.Tensor, draft_probs: torch.Tensor, draft_tokens: torch.Tensor,
                       parent: Optional[torch.Tensor], uniforms: torch.Tensor, params: AcceptParams, B: int, k: int, V: int,
                       accepted_len: torch.Tensor, next_token: torch.Tensor, accepted_path: Optional[torch.Tensor] = None,
                       stats: Optional[AcceptStats] = None) -> None:
    _check(ctx.lib.dsd_accept_noalloc(ctx.h, _ptr(logits, torch.float32, "logits"),
                                      _ptr(draft_probs, torch.float32, "draft_probs"),
                                      _ptr(draft_tokens, torch.int32, "draft_tokens"), _ptr(parent, torch.int32, "parent"),
                                      _ptr(uniforms, torch.float32, "uniforms"), C.byref(params), B, k, V,
                                      _ptr(accepted_len, torch.int32, "accepted_len"),
                                      _ptr(next_token, torch.int32, "next_token"),
                                      _ptr(accepted_path, torch.int32, "accepted_path"),
                                      None if stats is None else C.byref(stats)), "dsd_accept_noalloc")


def dsd_kv_commit(ctx: Context, kv: KVCache, accepted_len: torch.Tensor, accepted_path: Optional[torch.Tensor],
                  B: int, k: int) -> None:
    _check(ctx.lib.dsd_kv_commit(ctx.h, kv.h, _ptr(accepted_len, torch.int32, "accepted_len"),
                                 _ptr(accepted_path, torch.int32, "accepted_path"), B, k), "dsd_kv_commit")


def accept_params(lambda1=float("inf"), lambda2=float("inf"), lambda3=float("-inf"), tau=0.0, temperature=1.0,
                  top_m=8, tree_mode=DSD_TREE_LONGEST, tau_override: Optional[torch.Tensor] = None,
                  norm_match_kind=0, entropy_kind=0) -> AcceptParams:
    return AcceptParams(lambda1, lambda2, lambda3, tau, temperature, top_m, tree_mode,
                        _ptr(tau_override, torch.float32, "tau_override"), norm_match_kind, entropy_kind)
