"""The step under HIP graph capture: it is kernel launches only (no allocation, no memset, no synchronisation), so
a caller may capture it once and replay it.  Every replay must reproduce the eager result, with eager work and
synchronisations between the replays."""
import pytest

from paper_1910_06591_amd import seedinf, workloads as wl
from tests.parity import to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,B", [("C3", 70), ("C2", 33), ("C1", 5), ("C3", 2300), ("C2", 2100)])
def test_graph_replays_equal_eager(name, B):
    import torch
    cfg = wl.CONFIGS[name]
    net = seedinf.SeedInfer(seedinf.make_arch(cfg, max_batch=B), wl.make_weights(cfg))
    batches = [to_device(wl.make_batch(cfg, B, seed_shift=s)) for s in range(3)]
    static = {k: (None if v is None else v.clone()) for k, v in batches[0].items()}
    out = net.step(**static)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        net.step(out=out, **static)
    for r in range(5):
        b = batches[r % 3]
        for k, v in b.items():
            if v is not None:
                static[k].copy_(v)                       # eager work between the replays
        eager = {k: v.clone() for k, v in net.step(**b).items()}
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in eager:
            assert torch.equal(out[k], eager[k]), (r, k)
    net.close()
