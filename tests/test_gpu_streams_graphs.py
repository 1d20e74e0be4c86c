"""The library enqueues on the caller's stream, allocates nothing and never synchronises: the whole
path runs on a non-default stream and can be captured into a HIP graph and replayed."""
import numpy as np
import pytest
import torch

from paper_2407_09105_amd import binding, workloads as wl
from tests.gpu_util import DEV, to_dev

pytestmark = pytest.mark.gpu


def _buffers(w):
    dt = w.cfg.dtype
    q, k, v, do = (to_dev(a, dt) for a in (w.q, w.k, w.v, w.do))
    pos = torch.from_numpy(w.position_ids).to(DEV)
    seg = binding.Segments(w.cfg.rows, w.cfg.tokens_per_row, DEV)
    o = torch.empty_like(q)
    lse = torch.empty((q.shape[1], q.shape[0]), dtype=torch.float32, device=DEV)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ws = binding.bwd_workspace(q, k)
    return dict(q=q, k=k, v=v, do=do, pos=pos, seg=seg, o=o, lse=lse, dq=dq, dk=dk, dv=dv, ws=ws)


def _step(b):
    binding.pack_to_cu_seqlens(b["pos"], b["seg"])
    binding.varlen_attn_fwd(b["q"], b["k"], b["v"], b["seg"], out=b["o"], lse=b["lse"])
    binding.varlen_attn_bwd(b["do"], b["q"], b["k"], b["v"], b["o"], b["lse"], b["seg"], dq=b["dq"], dk=b["dk"],
                            dv=b["dv"], workspace=b["ws"])


def _outputs(b):
    return [b[k].clone() for k in ("o", "lse", "dq", "dk", "dv")] + [b["seg"].seg_start.clone(), b["seg"].q_tile_order.clone()]


def test_non_default_stream_matches_default_stream():
    w = wl.make_custom([[300, 45, 1, 1, 200, 93]], 4, 2, 128, "bf16", seed=41)
    b = _buffers(w)
    _step(b)
    torch.cuda.synchronize()
    ref = _outputs(b)
    for t in (b["o"], b["lse"], b["dq"], b["dk"], b["dv"]):
        t.zero_()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        _step(b)
    side.synchronize()
    for got, want in zip(_outputs(b), ref):
        assert torch.equal(got, want)


def test_graph_capture_and_replay():
    w = wl.make_custom([[513, 31, 480]], 5, 1, 128, "bf16", seed=42)
    b = _buffers(w)
    _step(b)                       # eager reference (also warms up before capture)
    torch.cuda.synchronize()
    ref = _outputs(b)
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            _step(b)
    for rep in range(3):
        # new inputs each time: replays must recompute everything from the current buffer contents
        if rep:
            b["q"].mul_(-1.0)
            b["do"].mul_(0.5)
        for t in (b["o"], b["dq"], b["dk"], b["dv"]):
            t.zero_()                                   # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = _outputs(b)
        if rep == 0:
            for a, e in zip(got, ref):                  # the first replay reproduces the eager run before capture
                assert torch.equal(a, e)
        _step(b)                                        # eager result on the same inputs
        torch.cuda.synchronize()
        for a, e in zip(got, _outputs(b)):
            assert torch.equal(a, e), rep


def test_measurement_probes_run_and_report():
    """The matrix-rate probes behind the benchmark's measured peaks: FLOP counts, clock read-out."""
    from paper_2407_09105_amd import probes
    sink = torch.zeros(64, dtype=torch.float32, device=DEV)
    assert probes.probe_mfma(sink, 10) == 2048 * 4 * 10 * 16 * 2.0 * 32 * 32 * 16
    ops = torch.randn(32768, device=DEV).to(torch.bfloat16)
    clocks = torch.zeros(2, dtype=torch.int64, device=DEV)
    for lds, valu in ((0, 0), (16, 24), (8, 16)):
        assert probes.probe_mix(ops, lds, valu, sink, clocks, 50) == 2048 * 4 * 50 * 16 * 2.0 * 32 * 32 * 16
        torch.cuda.synchronize()
        c = clocks.cpu().numpy()
        assert c[0] > 0 and c[1] > 0
        assert 200.0 < c[0] / c[1] * 100.0 < 4000.0   # shader clock in MHz against the 100 MHz wall clock
    assert float(sink.abs().sum()) == 0.0
    with pytest.raises(probes.ProbeError):
        probes.probe_mix(ops, 3, 3, sink, clocks, 10)
