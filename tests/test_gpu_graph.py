"""The entry points can be recorded into a HIP graph once the library's workspace is warm: no allocation, no
synchronisation and no memset node on the way (buffers are cleared by fill kernels).  Every replay is compared
with the eager result, with eager work and synchronisations between the replays."""
import numpy as np
import pytest

from paper_2106_00003_amd import binding, inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    binding.lib()
    binding.set_kernel(binding.KERNEL_AUTO)
    binding.set_reduction(binding.REDUCTION_AUTO)
    yield
    binding.set_reduction(binding.REDUCTION_AUTO)
    binding.release()


@pytest.mark.parametrize("n,B,dist,reduction", [(1024, 256, "normal0.1", "two_stage"), (512, 200, "uniform", "two_stage"),
                                                (256, 2048, "uniform", "gram"), (64, 4096, "uniform", "gram"),
                                                (2560, 2056, "normal0.1", "two_stage")])
def test_forward_and_backward_replay_from_a_graph(n, B, dist, reduction):
    mode = {"two_stage": binding.REDUCTION_TWO_STAGE, "gram": binding.REDUCTION_GRAM}[reduction]
    binding.set_reduction(mode)
    data = inputs.make_custom(n, B, seed=500 + n, theta_dist=dist)
    theta = torch.from_numpy(data["theta"]).cuda()
    X = torch.from_numpy(data["X"]).cuda()
    G = torch.from_numpy(data["G"]).cuda()
    Y, dX, dth = torch.empty_like(X), torch.empty_like(X), torch.empty_like(theta)

    def run():
        binding.givens_forward(theta, X, Y=Y)
        binding.givens_backward(theta, Y, G, dX=dX, dtheta=dth)

    run()                                                       # warms the workspace
    run()
    torch.cuda.synchronize()
    want = [t.clone() for t in (Y, dX, dth)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        run()                                                   # once more on the capture stream, eagerly
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run()
    torch.cuda.synchronize()
    for replay in range(3):
        for t in (Y, dX, dth):
            t.fill_(float("nan"))
        filler = (X @ X.T).sum()                                # unrelated eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.isfinite(filler)
        for got, ref, name in zip((Y, dX, dth), want, ("Y", "dX", "dtheta")):
            assert torch.equal(got, ref), f"replay {replay}: {name} differs from the eager result"
