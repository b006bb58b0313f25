"""The entry points only enqueue kernels on the stream they are given (no allocation, no
synchronisation, no memset nodes), so a caller may capture them in a HIP graph.  Each graph
is replayed several times on new input contents, with eager work and synchronisations in
between, and every replay is compared with the eager result on the same contents."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2510_20271_amd import api, synth
from tests.gpu_util import dev

pytestmark = pytest.mark.gpu


def _capture(fn):
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        fn()  # warm-up on the capture stream
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        fn()
    return g


@pytest.mark.parametrize("shape", [(64, 100), (300, 700), (40, 70, 131)])
def test_hard_curve_in_a_graph(shape, flow):
    nd = len(shape)
    fields = [np.stack([synth.grf(shape, 2.0, 10 * k + i) for i in range(2)]) for k in range(3)]
    x = dev(fields[0]).clone()
    ws = torch.empty(api.ecc_workspace_bytes(shape, 2, 128), dtype=torch.uint8, device="cuda")
    out = torch.empty((2, 128), dtype=torch.int64, device="cuda")
    g = _capture(lambda: api.ecc_hard(x, nd, 128, curve=out, workspace=ws))
    for f in fields + fields[::-1]:
        x.copy_(dev(f))
        want = api.ecc_hard(x, nd, 128).clone()   # eager, own buffers
        torch.cuda.synchronize()
        out.fill_(-7)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want)


def test_soft_forward_backward_in_a_graph():
    shape, T = (120, 300), 40
    fields = [np.stack([synth.grf(shape, 2.0, 50 + 10 * k + i) for i in range(2)]) for k in range(3)]
    x = dev(fields[0]).clone()
    u = dev(np.array([0.6, 0.8], np.float32))
    tau = dev(np.linspace(-2, 4, T).astype(np.float32))
    gup = dev(np.random.default_rng(0).standard_normal((2, T)).astype(np.float32))
    ws = torch.empty(api.ecc_workspace_bytes(shape, 2, T), dtype=torch.uint8, device="cuda")
    chi = torch.empty((2, T), dtype=torch.float32, device="cuda")
    gx = torch.empty_like(x)
    dt = torch.empty((2, T), dtype=torch.float32, device="cuda")
    du = torch.empty((2, T, 2), dtype=torch.float32, device="cuda")

    def step():
        api.ecc_soft_fwd(x, 2, u, 0.01, tau, 15.0, chi=chi, workspace=ws)
        api.ecc_soft_bwd(x, 2, u, 0.01, tau, 15.0, grad_chi=gup, grad_X=gx, dchi_dtau=dt, dchi_du=du, workspace=ws)
    g = _capture(step)
    for f in fields + fields[::-1]:
        x.copy_(dev(f))
        want_chi = api.ecc_soft_fwd(x, 2, u, 0.01, tau, 15.0).clone()
        want = [t.clone() for t in api.ecc_soft_bwd(x, 2, u, 0.01, tau, 15.0, grad_chi=gup)]
        torch.cuda.synchronize()
        for t in (chi, gx, dt, du):
            t.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        # the same kernels in the same order on the same data: identical bits
        assert torch.equal(chi, want_chi)
        assert torch.equal(gx, want[0]) and torch.equal(dt, want[1]) and torch.equal(du, want[2])
