"""Glue for the GPU parity tests: moves seeded numpy inputs to the device, calls the C ABI through
the binding, brings results back, and states the comparison rules."""
from __future__ import annotations

import numpy as np
import torch

from paper_2511_11733_amd import dsd as D
from paper_2511_11733_amd import workloads as W

# Stated tolerances (relative to max(|ref|, rms of the ref row)); see assert_close.
TOL = {"bf16": 2e-2, "f32": 1e-4}


def to_dev(a: np.ndarray, dtype: str, dev="cuda:0") -> torch.Tensor:
    """numpy (float32 / uint16 bf16 bits / ints) -> device tensor."""
    if a.dtype == np.uint16:
        assert dtype == "bf16"
        return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
    if a.dtype == np.uint64:
        return torch.from_numpy(a.view(np.int64)).to(dev)
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype == "bf16" and t.dtype in (torch.float32, torch.float64):
        raise AssertionError("bf16 inputs travel as bit patterns")
    return t.to(dev)


def to_np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def assert_close(got: np.ndarray, ref: np.ndarray, tol: float, what: str):
    """|got - ref| <= tol * max(|ref|, rms(ref row)) for every element; returns the normalised
    RMS error (rms(got-ref)/rms(ref)) and the worst ratio to the allowance."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    rms = np.sqrt(np.mean(ref * ref, axis=-1, keepdims=True))
    allow = tol * np.maximum(np.abs(ref), rms)
    err = np.abs(got - ref)
    worst = float((err / np.maximum(allow, 1e-300)).max())
    nrms = float(np.sqrt(np.mean(err ** 2)) / max(np.sqrt(np.mean(ref ** 2)), 1e-300))
    assert worst <= 1.0, f"{what}: worst error is {worst:.3f} x the allowance (tol {tol}), normalised rms {nrms:.2e}"
    return nrms, worst


class GpuStage:
    """One node's layer block + KV cache on the device."""

    def __init__(self, model: W.ModelCfg, weights: dict, max_batch: int, max_slots: int, ctx=None):
        self.m = model
        self.ctx = ctx or D.Context(0)
        self.desc = D.model_desc(model)
        tens = [to_dev(weights[name], model.dtype) for name, _, _ in W.weight_specs(model)]
        self.w = D.Weights(self.ctx, self.desc, tens)
        del tens
        self.kv = D.KVCache(self.ctx, self.desc, max_batch, max_slots)
        self.tdt = torch.bfloat16 if model.dtype == "bf16" else torch.float32

    def import_kv(self, K: np.ndarray, V: np.ndarray, lens):
        """K, V: [L, B, Hkv, C, hd] (model dtype; float64 oracle output is rounded to it)."""
        if K.shape[3] > 0:
            for l in range(self.m.L):
                self.kv.import_layer(l, self._cast(K[l]), self._cast(V[l]))
        self.kv.set_len(lens)

    def _cast(self, a: np.ndarray) -> torch.Tensor:
        if a.dtype == np.uint16:
            return to_dev(a, "bf16")
        return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0").to(self.tdt).contiguous()

    def verify(self, hidden=None, tokens=None, parent=None, logits_buf=None, logits_offset=0, logits_seq_stride=0,
               want_hidden=True):
        m = self.m
        if hidden is not None:
            h = self._cast(hidden)
            B, k = h.shape[:2]
            tok = None
        else:
            tok = torch.from_numpy(np.asarray(tokens, dtype=np.int32)).to("cuda:0")
            B, k = tok.shape
            h = None
        mask = depth = None
        if parent is not None:
            mask = to_dev(W.tree_mask_bits(np.asarray(parent)), "u64")
            depth = torch.from_numpy(W.tree_depths(np.asarray(parent))).to("cuda:0")
        out = torch.empty((B, k, m.d), dtype=self.tdt, device="cuda:0") if want_hidden else None
        lg = None
        if m.has_head:
            lg = logits_buf if logits_buf is not None else torch.empty((B, k, m.V), dtype=torch.float32, device="cuda:0")
        D.dsd_stage_verify(self.ctx, self.w, self.kv, h, tok, mask, depth, B, k, out, lg, logits_seq_stride,
                           logits_offset)
        torch.cuda.synchronize()
        return out, lg

    def new_rows(self, layer: int, first: int, n: int, B: int):
        k, v = self.kv.export_layer(layer, first, n, B)
        torch.cuda.synchronize()
        return to_np64(k), to_np64(v)


def gpu_accept(ctx, logits: torch.Tensor, probs: torch.Tensor, tokens: np.ndarray, parent, uniforms: np.ndarray,
               prm: dict, tau_override=None):
    B, R, V = logits.shape
    k = R - 1
    dev = logits.device
    tok = torch.from_numpy(np.asarray(tokens, dtype=np.int32)).to(dev)
    par = None if parent is None else torch.from_numpy(np.asarray(parent, dtype=np.int32)).to(dev)
    u = torch.from_numpy(np.asarray(uniforms, dtype=np.float32)).to(dev)
    to = None if tau_override is None else torch.from_numpy(np.asarray(tau_override, dtype=np.float32)).to(dev)
    alen = torch.full((B,), -7, dtype=torch.int32, device=dev)
    nxt = torch.full((B,), -7, dtype=torch.int32, device=dev)
    path = torch.full((B, k), -7, dtype=torch.int32, device=dev)
    key = torch.zeros((B, k), dtype=torch.int32, device=dev)
    nacc = torch.zeros((B, k), dtype=torch.int32, device=dev)
    ratio = torch.zeros((B, k), dtype=torch.float64, device=dev)
    nm = torch.zeros((B, k), dtype=torch.float64, device=dev)
    st = D.AcceptStats(key.data_ptr(), nacc.data_ptr(), ratio.data_ptr(), nm.data_ptr())
    p = D.accept_params(tau_override=to, **prm)
    D.dsd_accept(ctx, logits, probs, tok, par, u, p, B, k, V, alen, nxt, path, st)
    torch.cuda.synchronize()
    return dict(accepted_len=alen.cpu().numpy(), next_token=nxt.cpu().numpy(), accepted_path=path.cpu().numpy(),
                key=key.cpu().numpy().astype(bool), node_accept=nacc.cpu().numpy().astype(bool),
                ratio=ratio.cpu().numpy(), norm_match=nm.cpu().numpy(), dev=(alen, nxt, path))


def compare_accept(gpu: dict, ora, what: str):
    """Integer outputs must be identical, except for sequences the oracle flags as near ties
    (a decision within the stated distance of its threshold).  Returns (mismatching sequences that
    were near ties, number of near-tie sequences)."""
    B = len(ora.accepted_len)
    excused = 0
    for b in range(B):
        same = (gpu["accepted_len"][b] == ora.accepted_len[b] and gpu["next_token"][b] == ora.next_token[b]
                and (gpu["accepted_path"][b] == ora.accepted_path[b][:gpu["accepted_path"].shape[1]]).all()
                and (gpu["key"][b] == ora.key[b]).all() and (gpu["node_accept"][b] == ora.node_accept[b]).all())
        if not same:
            assert ora.near_tie[b] != 0, (
                f"{what}: sequence {b} differs with no near tie: gpu len {gpu['accepted_len'][b]} tok "
                f"{gpu['next_token'][b]} path {gpu['accepted_path'][b]} vs oracle len {ora.accepted_len[b]} tok "
                f"{ora.next_token[b]} path {ora.accepted_path[b]}")
            excused += 1
    return excused, int((ora.near_tie != 0).sum())


def oracle_prm(O, prm: dict):
    return O.AcceptParams(lambda1=prm.get("lambda1", np.inf), lambda2=prm.get("lambda2", np.inf),
                          lambda3=prm.get("lambda3", -np.inf), tau=prm.get("tau", 0.0), top_m=prm.get("top_m", 8),
                          temperature=prm.get("temperature", 1.0), tree_mode=prm.get("tree_mode", 0),
                          norm_match_kind=prm.get("norm_match_kind", 0), entropy_kind=prm.get("entropy_kind", 0))
