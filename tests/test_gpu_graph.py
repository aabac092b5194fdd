"""The library only enqueues kernels on the caller's stream (no allocation, no memset, no synchronisation), so a
forward + backward can be captured into a HIP graph and replayed.  Every replay is checked bit for bit against
the eager result, with eager work and synchronisations between the replays."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2511_17599_amd import binding as B             # noqa: E402
from paper_2511_17599_amd import inputs as I              # noqa: E402
from paper_2511_17599_amd.runner import session_for       # noqa: E402


@pytest.fixture(autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


@pytest.mark.parametrize("dtype,N,d,V", [("bf16", 1030, 256, 5000), ("f32", 300, 64, 700)])
def test_forward_backward_replays_from_a_graph(dtype, N, d, V):
    wl = I.Workload(f"graph_{dtype}", N, d, V, dtype, "uniform", ignore_frac=0.1, seed=401)
    x = I.make_inputs(wl)
    s = session_for(wl, x)
    assert s.forward() == B.FLCE_OK and s.backward() == B.FLCE_OK      # eager: also loads the kernels
    torch.cuda.synchronize()
    want = [t.clone() for t in (s.loss, s.lse, s.dH, s.dW)]

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            assert s.forward() == B.FLCE_OK                             # launches go to the capturing stream
            assert s.backward() == B.FLCE_OK
    torch.cuda.synchronize()

    for rep in range(3):
        for t in (s.loss, s.lse, s.dH, s.dW):
            t.fill_(7.0)                                                # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, ref, name in zip((s.loss, s.lse, s.dH, s.dW), want, ("loss", "lse", "dH", "dW")):
            assert torch.equal(got, ref), (rep, name)
    st, nv = s.device_status()
    assert st == B.FLCE_OK and nv == int((x["y"] != wl.ignore_index).sum())
