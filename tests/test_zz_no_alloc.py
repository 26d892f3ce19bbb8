"""owq_linear_static (the entry point that allocates nothing: its scratch memory is a static
device array inside the library) against owq_linear, through the C ABI.

Two calls in a row on every case, the second with a smaller input, so that the second call finds
the first one's contents in the shared array.  Bar: the forward path's (relative L2 <= 1e-3,
max-abs <= 1e-2 rms, per token) against the fp64 oracle for both entry points, and the two entry
points against each other at the same bar (the work split, hence the order of the partial sums,
may differ when the array holds fewer partial results than the blob's own scratch area)."""
import numpy as np
import pytest

from oracle import owq_ref
from synth import CONFIGS, LayerSpec, make_layer, make_x

pytestmark = pytest.mark.gpu

REL_L2 = 1e-3
MAX_ABS = 1e-2


@pytest.fixture(scope="module")
def env():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2306_02272_amd import binding
    binding.lib()
    torch.cuda.set_device(0)
    return torch, binding


def close(a, b, what):
    rel, mx = owq_ref.parity_errors(a, b)
    assert rel <= REL_L2 and mx <= MAX_ABS, (what, rel, mx)
    for n in range(b.shape[0]):
        rel, mx = owq_ref.parity_errors(a[n], b[n])
        assert rel <= REL_L2 and mx <= MAX_ABS, (what, n, rel, mx)


def both(env, lin, x):
    torch, B = env
    xd = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    batch = x.shape[0]
    y0 = torch.zeros((batch, lin.d_out), dtype=torch.float16, device="cuda")
    y1 = torch.full((batch, lin.d_out), 7.0, dtype=torch.float16, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    B.owq_linear(lin.handle, xd.data_ptr(), y0.data_ptr(), batch, stream)
    B.owq_linear_static(lin.handle, xd.data_ptr(), y1.data_ptr(), batch, stream)
    torch.cuda.synchronize()
    return y0.cpu().numpy(), y1.cpu().numpy()


CASES = [
    # name, d_in, d_out, bits, group, k, layout, first batch, second (smaller) batch
    ("tile3_ch", 1024, 600, 3, 0, 24, 1, 64, 40),        # three launches, then three launches on fewer tokens
    ("tile4_g128", 2048, 130, 4, 128, 16, 1, 48, 5),     # three launches, then the one-launch kernel
    ("tile3_split", 5120, 96, 3, 128, 51, 1, 16, 3),     # one-launch kernel with its columns split: partial sums in the array
    ("tile3_b130", 512, 70, 3, 0, 5, 1, 130, 33),        # several passes
    ("gemv3", 1024, 96, 3, 128, 8, 0, 2, 1),             # a layout without scratch memory runs as owq_linear does
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_static_scratch_matches_owq_linear(env, case):
    torch, B = env
    name, d_in, d_out, bits, group, k, layout, b1, b2 = case
    layer = make_layer(LayerSpec(name, d_in, d_out, bits, group, k, seed=77))
    lin = B.OwqLinear(layer, layout=layout)
    if name == "tile3_split":
        B.owq_set_launch(lin.handle, 0, 0, 0, 4)           # four column ranges per row tile
    for batch in (b1, b2):
        x = make_x(layer, batch, seed=batch)
        want = owq_ref.owq_linear_layer(layer, x)
        y_lin, y_static = both(env, lin, x)
        close(y_lin, want, (name, batch, "owq_linear"))
        close(y_static, want, (name, batch, "owq_linear_static"))
        close(y_static, y_lin.astype(np.float64), (name, batch, "static vs owq_linear"))
    lin.close()


def test_two_layers_share_the_array(env):
    """A big layer, then a small one of another shape: the second call must not see the first one's leftovers."""
    torch, B = env
    big = make_layer(LayerSpec("big", 4096, 1024, 3, 128, 32, seed=5))
    small = make_layer(LayerSpec("small", 512, 40, 4, 0, 3, seed=6))
    lb, ls = B.OwqLinear(big, layout=1), B.OwqLinear(small, layout=1)
    for layer, lin, batch in ((big, lb, 64), (small, ls, 20), (big, lb, 7), (small, ls, 64)):
        x = make_x(layer, batch, seed=batch + 1)
        want = owq_ref.owq_linear_layer(layer, x)
        y_lin, y_static = both(env, lin, x)
        close(y_static, want, (layer.spec.name, batch))
        close(y_static, y_lin.astype(np.float64), (layer.spec.name, batch, "vs owq_linear"))
    lb.close()
    ls.close()


def test_full_size_layer_fits_or_is_rejected(env):
    """configs[4]'s fc2 (36864 -> 9216, batch 64): its partial results fit the array with fewer workgroups."""
    torch, B = env
    spec = CONFIGS[4][1]
    layer = make_layer(spec)
    lin = B.OwqLinear(layer, layout=1)
    x = make_x(layer, 64)
    y_lin, y_static = both(env, lin, x)
    rows = np.arange(0, spec.d_out, 97)                      # sampled rows: the fp64 oracle on all of them is slow
    want = owq_ref.owq_linear_ref(layer.codes[rows], layer.scale[rows], layer.zero[rows], layer.group_size,
                                  layer.weak_idx, layer.weak_w[rows], x)
    close(y_static[:, rows], want, "fc2 static")
    close(y_static, y_lin.astype(np.float64), "fc2 static vs owq_linear")
    lin.close()


def test_too_large_is_rejected(env):
    """A layer whose staged activations alone exceed the array: OWQ_ERR_SCRATCH, nothing launched."""
    torch, B = env
    d_in = 400000                                            # 64 tokens x 400k columns x 2 B = 51 MB of staged activations
    rng = np.random.default_rng(0)
    layer = make_layer(LayerSpec("wide", d_in, 8, 3, 0, 0, seed=9))
    lin = B.OwqLinear(layer, layout=1)
    x = torch.zeros((2, d_in), dtype=torch.float16, device="cuda")
    y = torch.zeros((2, 8), dtype=torch.float16, device="cuda")
    with pytest.raises(B.OwqError) as e:
        B.owq_linear_static(lin.handle, x.data_ptr(), y.data_ptr(), 2, torch.cuda.current_stream().cuda_stream)
    assert e.value.status == B.OWQ_ERR_SCRATCH
    torch.cuda.synchronize()
    lin.close()
