"""The library allocates nothing and records no memset, so its calls can be captured in a HIP
graph: every replay, with eager work and synchronisations in between, must reproduce the eager
result bit for bit."""
import numpy as np
import pytest

import workloads
from gpu_util import host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dx():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_1907_12205_amd as dx
    dx.lib()
    return dx


@pytest.mark.parametrize("aggregator,B,kw", [("multikrum", 5, dict(f=1, m=3)), ("coord_median", 5, {}),
                                             ("geomedian", 5, {}), ("bulyan", 15, dict(f=1)),
                                             ("trimmed_mean", 5, {})])
def test_captured_step_replays_bit_for_bit(dx, aggregator, B, kw):
    import torch
    from paper_1907_12205_amd.binding import StepBuffers
    w = workloads.config(3, d=300_001)
    G = w.to_device("cuda:0")
    buf = StepBuffers(w.n, w.d, w.r, B, G.device, materialise=False)

    def step():
        dx.detox_step(G, w.r, w.q, B, aggregator, buffers=buf, **kw)

    step()
    torch.cuda.synchronize()
    want_out, want_w = buf.out.clone(), buf.winner.clone()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    for i in range(4):
        buf.out.zero_()
        buf.winner.fill_(-7)
        scratch = torch.randn(1 << 16, device=G.device).sum()      # eager work between replays
        graph.replay()
        torch.cuda.synchronize()
        assert scratch.isfinite()
        assert torch.equal(buf.out, want_out), f"replay {i}"
        assert torch.equal(buf.winner, want_w), f"replay {i}"


def test_captured_average_of_many_rows_replays_bit_for_bit(dx):
    """Vanilla Multi-Krum and the geometric median on 24 rows of 2.1M columns: their averaging
    kernel holds results back in LDS and registers and may take several launches; captured and
    replayed it must give the eager result."""
    import torch
    X = torch.from_numpy(workloads.distinct_rows(5, 24, 2_100_003, sigma=0.03)).cuda()
    out = torch.empty(X.shape[1], device=X.device)
    need = max(dx.workspace_bytes("multikrum", 24, X.shape[1]), dx.workspace_bytes("geomedian", 24, X.shape[1]))
    ws = torch.empty(need, dtype=torch.uint8, device=X.device)
    for call in (lambda: dx.robust_multikrum(X, 2, 20, out=out, ws=ws, with_scores=False),
                 lambda: dx.robust_geomedian(X, iters=3, eps=1e-8, out=out, ws=ws)):
        call()
        torch.cuda.synchronize()
        want = out.clone()
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                call()
        for i in range(3):
            out.zero_()
            scratch = torch.randn(1 << 16, device=X.device).sum()      # eager work between replays
            graph.replay()
            torch.cuda.synchronize()
            assert scratch.isfinite()
            assert torch.equal(out, want), f"replay {i}"


def test_captured_step_sees_new_inputs(dx):
    """A replay reads the buffers as they are at replay time: changing a Byzantine row so that a
    group loses its majority switches the replay onto the repair path (the conditional kernels)."""
    import torch
    import oracle
    from paper_1907_12205_amd.binding import StepBuffers
    w = workloads.config(2, d=70_001)
    Gh = w.matrix().copy()
    G = torch.from_numpy(Gh).cuda()
    buf = StepBuffers(w.n, w.d, w.r, 5, G.device, materialise=False)
    side = torch.cuda.Stream()
    dx.detox_step(G, w.r, w.q, 5, "multikrum", f=1, m=3, buffers=buf)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            dx.detox_step(G, w.r, w.q, 5, "multikrum", f=1, m=3, buffers=buf)
    for trial in range(3):
        if trial == 1:                                   # group 0: three different rows
            Gh[1, 5] += 1.0
            Gh[2, 9] -= 1.0
        if trial == 2:                                   # and back to two equal rows
            Gh[2] = Gh[0]
        G.copy_(torch.from_numpy(Gh))
        graph.replay()
        torch.cuda.synchronize()
        ref_out, ref_w, _ = oracle.detox_step(Gh, w.r, 5, "multikrum", f=1, m=3)
        assert host(buf.winner).tolist() == ref_w.tolist()
        assert np.linalg.norm(host(buf.out) - ref_out) <= 1e-5 * np.linalg.norm(ref_out)
    assert ref_w[0] == 0


@pytest.mark.parametrize("which,count", [("bulyan", 105), ("geomedian", 100), ("multikrum", 128)])
def test_captured_aggregators_on_many_rows(dx, which, count):
    """Row counts whose selection kernels need more than 64 KB of LDS (the limit is raised once per
    device, outside any launch sequence): captured after one eager call, replayed, compared."""
    import torch
    X = torch.from_numpy(workloads.distinct_rows(5, count, 20_011, sigma=0.03)).cuda()
    X[3] += 0.05
    out = torch.empty(X.shape[1], dtype=torch.float32, device=X.device)
    ws = torch.empty(dx.workspace_bytes(which, count, X.shape[1]), dtype=torch.uint8, device=X.device)
    f = 10

    def call():
        if which == "bulyan":
            return dx.robust_bulyan(X, f, out=out, ws=ws)[1]
        if which == "multikrum":
            return dx.robust_multikrum(X, f, count - f, out=out, ws=ws, with_scores=False)[1]
        dx.robust_geomedian(X, 30, 1e-8, out=out, ws=ws)
        return None

    sel = call()
    torch.cuda.synchronize()
    want_out = out.clone()
    want_sel = None if sel is None else sel.clone()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            sel_g = call()
    for i in range(3):
        out.zero_()
        scratch = torch.randn(1 << 16, device=X.device).sum()      # eager work between replays
        graph.replay()
        torch.cuda.synchronize()
        assert scratch.isfinite()
        assert torch.equal(out, want_out), f"replay {i}"
        if want_sel is not None:
            assert torch.equal(sel_g, want_sel), f"replay {i}"
