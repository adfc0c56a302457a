"""dsd_accept_noalloc (the entry point for callers that cannot allocate) against dsd_accept: the same kernels
on a fixed scratch array in the library's device image, so every output must be identical, bit for bit.  Two
calls in a row, the second with a smaller input (the array keeps the first call's contents), then the
size limit.  Collected last on purpose."""
import numpy as np
import pytest
import torch

from paper_2511_11733_amd import dsd as D
from paper_2511_11733_amd import workloads as W

pytestmark = pytest.mark.gpu


def rows(seed, B, k, V, parent=None):
    g = torch.Generator(device="cuda:0")
    g.manual_seed(seed)
    lg = (torch.randn((B, k + 1, V), device="cuda:0", generator=g) * 1.28).contiguous()
    q = torch.softmax(lg + 0.5 * torch.randn((B, k + 1, V), device="cuda:0", generator=g), -1).contiguous()
    par = list(range(k)) if parent is None else [int(p) for p in parent]
    toks = torch.zeros((B, k), dtype=torch.int64, device="cuda:0")
    ar = torch.arange(B, device="cuda:0")
    for i in range(k):                      # siblings without replacement
        pr = q[:, par[i]].clone()
        for j in range(i):
            if par[j] == par[i]:
                pr[ar, toks[:, j]] = 0.0
        toks[:, i] = torch.multinomial(pr, 1, generator=g)[:, 0]
    u = torch.rand((B, k + 1), device="cuda:0", generator=g)
    return lg, q, toks.to(torch.int32).contiguous(), u


def call(fn, ctx, lg, q, toks, parent, u, prm):
    B, R, V = lg.shape
    k = R - 1
    dev = lg.device
    par = None if parent is None else torch.from_numpy(np.asarray(parent, dtype=np.int32)).to(dev)
    out = dict(alen=torch.full((B,), -7, dtype=torch.int32, device=dev), nxt=torch.full((B,), -7, dtype=torch.int32, device=dev),
               path=torch.full((B, k), -7, dtype=torch.int32, device=dev), key=torch.full((B, k), -7, dtype=torch.int32, device=dev),
               nacc=torch.full((B, k), -7, dtype=torch.int32, device=dev),
               ratio=torch.full((B, k), -7.0, dtype=torch.float64, device=dev),
               nm=torch.full((B, k), -7.0, dtype=torch.float64, device=dev))
    st = D.AcceptStats(out["key"].data_ptr(), out["nacc"].data_ptr(), out["ratio"].data_ptr(), out["nm"].data_ptr())
    fn(ctx, lg, q, toks, par, u, D.accept_params(**prm), B, k, V, out["alen"], out["nxt"], out["path"], st)
    torch.cuda.synchronize()
    return {n: t.cpu().numpy() for n, t in out.items()}


def same(a, b, what):
    for n in a:
        np.testing.assert_array_equal(a[n], b[n], err_msg=f"{what}: {n}")


def test_noalloc_entry_point_matches_dsd_accept_on_two_calls_in_a_row():
    ctx = D.Context(0)
    prm = dict(tau=0.2, lambda1=1.02, lambda2=1.8e-5, lambda3=0.4375, top_m=8)
    # first call: the chain workload's shape at the full vocabulary (most of the fixed array in use)
    big = rows(1, 16, 8, 128256)
    ref_big = call(D.dsd_accept, ctx, *big[:3], None, big[3], prm)
    got_big = call(D.dsd_accept_noalloc, ctx, *big[:3], None, big[3], prm)
    same(got_big, ref_big, "B=16 k=8 V=128256")
    assert 0 < ref_big["alen"].mean() < 8
    # second call right behind it, smaller in every dimension and a tree: the array still holds the first call's partials
    parent = W.ranked_tree_parents((3, 2), 6)
    small = rows(2, 3, 6, 5001, parent)
    ref_small = call(D.dsd_accept, ctx, *small[:3], parent, small[3], dict(prm, tree_mode=1))
    got_small = call(D.dsd_accept_noalloc, ctx, *small[:3], parent, small[3], dict(prm, tree_mode=1))
    same(got_small, ref_small, "B=3 k=6 V=5001 tree")
    # and the first input once more: nothing of the small call may leak into it
    same(call(D.dsd_accept_noalloc, ctx, *big[:3], None, big[3], prm), ref_big, "B=16 k=8 V=128256 again")
    # the other rules run on the same array: greedy verification, the lossless walk
    for extra in (dict(temperature=0.0), dict(tree_mode=2)):
        p2 = dict(prm, **extra)
        same(call(D.dsd_accept_noalloc, ctx, *small[:3], parent, small[3], p2),
             call(D.dsd_accept, ctx, *small[:3], parent, small[3], p2), f"small {extra}")


def test_noalloc_entry_point_refuses_what_the_fixed_array_cannot_hold():
    ctx = D.Context(0)
    B, k, V = 40, 8, 128256                  # about 12 MiB of partials: beyond the 8 MiB array
    lg = torch.zeros((B, k + 1, V), dtype=torch.float32, device="cuda:0")
    toks = torch.zeros((B, k), dtype=torch.int32, device="cuda:0")
    u = torch.zeros((B, k + 1), dtype=torch.float32, device="cuda:0")
    alen = torch.zeros(B, dtype=torch.int32, device="cuda:0")
    with pytest.raises(D.DsdError, match="fixed array"):
        D.dsd_accept_noalloc(ctx, lg, lg, toks, None, u, D.accept_params(), B, k, V, alen, alen.clone(), None)
