"""owq_linear under HIP graph capture: every replay must give the eager result bit for bit,
with eager work and synchronisations between the replays (both layouts, several tokens)."""
import numpy as np
import pytest

from oracle import owq_ref
from synth import LayerSpec, make_layer, make_x

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2306_02272_amd import binding
    binding.lib()
    torch.cuda.set_device(0)
    return torch, binding


@pytest.mark.parametrize("layout,batch", [(0, 1), (0, 3), (1, 64), (1, 70)])
def test_graph_replays_equal_eager(env, layout, batch):
    torch, B = env
    print(f"layout {layout} batch {batch}", flush=True)
    specs = [LayerSpec("g_fc1", 1024, 2048, 3, 128 if layout == 0 else 0, 16, 91),
             LayerSpec("g_fc2", 2048, 1024, 4, 0, 24, 92)]
    layers = [make_layer(s) for s in specs]
    lins = [B.OwqLinear(L, layout=layout) for L in layers]
    xs = [torch.from_numpy(make_x(L, batch)).cuda() for L in layers]
    ys = [torch.zeros((batch, L.d_out), dtype=torch.float16, device="cuda") for L in layers]
    stream = torch.cuda.Stream()

    def calls():
        for lin, x, y in zip(lins, xs, ys):
            B.owq_linear(lin.handle, x.data_ptr(), y.data_ptr(), batch, stream.cuda_stream)

    with torch.cuda.stream(stream):
        calls()
        stream.synchronize()
        eager = [y.clone() for y in ys]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            calls()
            calls()                                   # the same layers twice in one graph
        for rep in range(4):
            for y in ys:
                y.zero_()                             # eager work between the replays
            stream.synchronize()
            graph.replay()
            stream.synchronize()
            for y, e in zip(ys, eager):
                assert torch.equal(y.view(torch.int16), e.view(torch.int16)), (layout, batch, rep)
    for L, x, e in zip(layers, xs, eager):
        want = owq_ref.owq_linear_layer(L, x.cpu().numpy())
        rel, mx = owq_ref.parity_errors(e.cpu().numpy(), want)
        assert rel <= 1e-3 and mx <= 1e-2, (L.spec.name, rel, mx)
    for lin in lins:
        lin.close()
