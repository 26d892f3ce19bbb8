"""One tile-layout handle on two streams at once: owq_linear_ws keeps each call's intermediate
results in a workspace of its own, so the calls may overlap.  Both results are compared with the
fp64 oracle (the forward path's bar) and, bit for bit, with owq_linear's."""
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


@pytest.mark.parametrize("batch", [64, 9])
def test_one_handle_two_streams(env, batch):
    torch, B = env
    layer = make_layer(LayerSpec("reent", 4096, 2048, 3, 128, 32, seed=11))
    lin = B.OwqLinear(layer, layout=1)
    nws = B.owq_workspace_bytes(lin.handle)
    assert nws > 0
    xs_host = [make_x(layer, batch, seed=s) for s in (1, 2)]
    xs = [torch.from_numpy(x).cuda() for x in xs_host]
    ys = [torch.zeros((batch, layer.d_out), dtype=torch.float16, device="cuda") for _ in xs]
    wss = [torch.empty(nws, dtype=torch.uint8, device="cuda") for _ in xs]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]      # default priority
    torch.cuda.synchronize()
    for rep in range(8):                                      # several rounds so that the calls do overlap
        for x, y, ws, st in zip(xs, ys, wss, streams):
            B.owq_linear_ws(lin.handle, x.data_ptr(), y.data_ptr(), batch, ws.data_ptr(), nws, st.cuda_stream)
    torch.cuda.synchronize()
    for x_host, x, y in zip(xs_host, xs, ys):
        want = owq_ref.owq_linear_layer(layer, x_host)
        got = y.cpu().numpy()
        rel, mx = owq_ref.parity_errors(got, want)
        assert rel <= 1e-3 and mx <= 1e-2, (rel, mx)
        alone = lin(x)                                        # owq_linear, nothing else running
        torch.cuda.synchronize()
        assert np.array_equal(alone.cpu().numpy().view(np.uint16), got.view(np.uint16))
    lin.close()


def test_workspace_checks(env):
    torch, B = env
    layer = make_layer(LayerSpec("reent_small", 512, 64, 4, 0, 4, seed=12))
    lin = B.OwqLinear(layer, layout=1)
    nws = B.owq_workspace_bytes(lin.handle)
    x = torch.zeros((2, 512), dtype=torch.float16, device="cuda")
    y = torch.zeros((2, 64), dtype=torch.float16, device="cuda")
    ws = torch.empty(nws + 256, dtype=torch.uint8, device="cuda")
    for ptr, size in ((ws.data_ptr(), nws - 1), (ws.data_ptr() + 16, nws)):
        with pytest.raises(B.OwqError) as e:
            B.owq_linear_ws(lin.handle, x.data_ptr(), y.data_ptr(), 2, ptr, size, 0)
        assert e.value.status == B.OWQ_ERR_BUFFER
    gemv = B.OwqLinear(layer, layout=0)
    assert B.owq_workspace_bytes(gemv.handle) == 0
    B.owq_linear_ws(gemv.handle, x.data_ptr(), y.data_ptr(), 2, 0, 0, 0)     # needs none
    torch.cuda.synchronize()
    gemv.close()
    lin.close()
