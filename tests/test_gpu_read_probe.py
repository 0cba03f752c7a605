"""The plain streaming-read probe (a measurement aid beside the kernel's own rate)."""
import pytest

from paper_2605_06914_amd import Context, TaperError, TAPER_EHIP, TAPER_EINVAL


def test_host_only_context_refuses_the_probe():
    import ctypes

    from paper_2605_06914_amd import load_library

    ctx = Context(64, 8, 128, device=-1)
    us = (ctypes.c_double * 2)()
    rc = load_library().taper_stream_read_probe(ctx._h, ctypes.c_void_p(4096), 1 << 24, 1 << 24, 8, 0, 1, None, us)
    assert rc == TAPER_EHIP
    ctx.close()


@pytest.mark.gpu
def test_probe_reads_at_a_plausible_rate_and_checks_its_arguments():
    import torch

    ctx = Context(64, 8, 128, device=0)
    buf = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda:0")
    r = ctx.stream_read_probe(buf, 256 << 20, n_workgroups=512, warmup=2, iters=8)
    assert r["us_min"] <= r["us"] and 500.0 < r["gbps"] < 8000.0
    whole = ctx.stream_read_probe(buf, 1 << 30, n_workgroups=256, warmup=1, iters=3)
    assert 500.0 < whole["gbps"] < 8000.0
    for bad in (dict(pass_bytes=(256 << 20) + 4096), dict(pass_bytes=2 << 30), dict(pass_bytes=0), dict(n_workgroups=0)):
        kw = dict(pass_bytes=256 << 20, n_workgroups=512)
        kw.update(bad)
        with pytest.raises(TaperError) as e:
            ctx.stream_read_probe(buf, kw["pass_bytes"], n_workgroups=kw["n_workgroups"])
        assert e.value.status == TAPER_EINVAL
    ctx.close()
