"""als_epoch under HIP graph capture: the call enqueues kernels only (no allocation once the workspace has its
size, no copy, no wait), so a caller may record an epoch once and replay it.  Every replay is checked against
the same epoch run eagerly, with eager library calls and synchronisations between the replays."""
import pytest
import torch

from gpu_util import f64, rel_fro, say, to_dev
from paper_2112_02194_amd import binding as als
from synth import make_problem

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,kw", [("c1", {}), ("c3", {"rows": 60000, "cols": 60000})])
def test_a_captured_epoch_replays_like_eager_epochs(gpu_device, name, kw):
    say(f"graph capture of als_epoch, {name} {kw}")
    p = make_problem(name, **kw)
    ctx = als.Context(0)
    Y, Yt = to_dev(p, gpu_device)
    W, H = p.W0.clone().to(gpu_device), p.H0.clone().to(gpu_device)
    prm = als.make_params(p.alpha, p.lam)
    for _ in range(2):  # the workspace takes its size and the launch-size hints arrive
        als.als_epoch(ctx, Y, Yt, W, H, prm)
    als.als_status_sync(ctx)
    W0, H0 = W.clone(), H.clone()
    eager = []
    for _ in range(3):
        als.als_epoch(ctx, Y, Yt, W, H, prm)
        eager.append((W.clone(), H.clone(), als.als_loss(ctx, Y, W, H, prm)))
    W.copy_(W0)
    H.copy_(H0)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        als.als_epoch(ctx, Y, Yt, W, H, prm)
    torch.cuda.synchronize()
    assert bool(torch.equal(W, W0)) and bool(torch.equal(H, H0))  # recording runs nothing
    for i in range(3):
        graph.replay()
        loss = als.als_loss(ctx, Y, W, H, prm)  # eager work and a synchronisation between the replays
        als.als_status_sync(ctx)
        We, He, le = eager[i]
        say(f"  replay {i}: errW {rel_fro(f64(W), f64(We)):.1e} errH {rel_fro(f64(H), f64(He)):.1e}")
        assert rel_fro(f64(W), f64(We)) <= 1e-6 and rel_fro(f64(H), f64(He)) <= 1e-6
        assert abs(loss - le) <= 1e-6 * abs(le)
    ctx.close()
