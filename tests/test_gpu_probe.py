"""GPU: the bare-stream probe entry point (the yardstick the bench reports beside its roofline figures)."""
import pytest
import torch

from paper_2511_11733_amd import dsd as D

pytestmark = pytest.mark.gpu


def test_stream_probe_modes_and_argument_checks():
    stream = torch.cuda.Stream()
    ctx = D.Context(0, stream)
    buf = torch.empty(64 << 20, dtype=torch.uint8, device="cuda:0")
    stream.synchronize()
    rates = {}
    for mode in (0, 1, 2, 3):
        ms = ctx.stream_probe(buf, mode, 3)
        assert ms > 0.0
        rates[mode] = buf.numel() / ms / 1e6          # GB/s
    # 64 MiB sits in the memory-side cache, so the figures say nothing about HBM; they only have to be sane
    assert all(100.0 < r < 20000.0 for r in rates.values()), rates
    print("stream probe on 64 MiB, GB/s by mode:", {k: round(v) for k, v in rates.items()})
    with pytest.raises(D.DsdError):
        ctx.stream_probe(buf, 4, 3)                  # no such mode
    with pytest.raises(D.DsdError):
        ctx.stream_probe(buf, 0, 0)                  # no iterations
    with pytest.raises(D.DsdError):
        ctx.stream_probe(buf[: 1 << 10], 0, 1)       # below the minimum size
