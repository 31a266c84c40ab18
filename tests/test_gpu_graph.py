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
