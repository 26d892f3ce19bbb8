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


def test_backward_and_search_replay_equal_eager(env):
    # Neither entry point allocates or synchronises, so both can be captured; every replay must
    # reproduce the eager outputs bit for bit (all their sums run in a fixed order).
    torch, B = env
    from synth import make_weights
    L = make_layer(LayerSpec("g_bwd", 1024, 512, 3, 128, 16, 93))
    lin = B.OwqLinear(L, layout=1)
    batch = 140                                        # two passes
    rng = np.random.default_rng(8)
    x = torch.from_numpy(make_x(L, batch)).cuda()
    dy = torch.from_numpy(rng.normal(0, 0.05, size=(batch, L.d_out)).astype(np.float16)).cuda()
    dx = torch.zeros((batch, L.d_in), dtype=torch.float16, device="cuda")
    dww = torch.zeros((L.d_out, L.k), dtype=torch.float32, device="cuda")
    ws = torch.empty(B.owq_backward_workspace_bytes(lin.handle, batch), dtype=torch.uint8, device="cuda")
    w_host, idx_host = make_weights(96, 1024, 8, seed=94)
    w, idx = torch.from_numpy(w_host).cuda(), torch.from_numpy(idx_host).cuda()
    scale = torch.zeros((96, 8), dtype=torch.float16, device="cuda")
    zero, codes = torch.zeros_like(scale), torch.zeros((96, 1024), dtype=torch.uint8, device="cuda")
    err = torch.zeros((96, 8), dtype=torch.float32, device="cuda")
    sd = B.SearchDesc(96, 1024, 3, 128, 8, 8, 8, 0.3)
    outs = [dx, dww, scale, zero, codes, err]
    stream = torch.cuda.Stream()

    def calls():
        B.owq_linear_backward(lin.handle, dy.data_ptr(), x.data_ptr(), dx.data_ptr(), dww.data_ptr(), batch,
                              ws.data_ptr(), int(ws.numel()), stream.cuda_stream)
        B.owq_search_config(sd, w.data_ptr(), idx.data_ptr(), scale.data_ptr(), zero.data_ptr(), codes.data_ptr(),
                            err.data_ptr(), 0, stream.cuda_stream)

    with torch.cuda.stream(stream):
        calls()
        stream.synchronize()
        eager = [o.clone() for o in outs]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            calls()
        for rep in range(3):
            for o in outs:
                o.zero_()
            ws.zero_()
            stream.synchronize()
            graph.replay()
            stream.synchronize()
            for o, e in zip(outs, eager):
                assert torch.equal(o.view(torch.uint8), e.view(torch.uint8)), rep
    lin.close()
