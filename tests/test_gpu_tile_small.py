"""GPU parity of the one-launch kernel of the tile layout (passes of 32 tokens or fewer)
against the fp64 CPU oracle, through the C ABI."""
import zlib

import numpy as np
import pytest

from oracle import owq_ref
from synth import CONFIGS, LayerSpec, make_layer, make_x

pytestmark = pytest.mark.gpu
TILE = 1
REL_L2, MAX_ABS = 1e-3, 1e-2      # relative L2; max abs in units of rms(y)


@pytest.fixture(scope="module")
def env():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2306_02272_amd import binding
    binding.lib()
    torch.cuda.set_device(0)
    return torch, binding


def run_gpu(env, layer, x, split=0):
    """split: S + 100 c.  S = column ranges per row tile (0 = the library's choice); c = 0: the library
    chooses the row tiles per workgroup, c = 1, 2, 3: 1, 2 or 4 of them.  -1 = the three-launch path."""
    torch, B = env
    lin = B.OwqLinear(layer, layout=TILE)
    if split:
        B.owq_set_launch(lin.handle, 0, 0, 0, split)
    y = lin(torch.from_numpy(np.ascontiguousarray(x)).cuda())
    torch.cuda.synchronize()
    out = y.cpu().numpy()
    lin.close()
    return out


def check(y_gpu, y_ref, what=""):
    assert y_gpu.shape == y_ref.shape
    rel, mx = owq_ref.parity_errors(y_gpu, y_ref)
    assert rel <= REL_L2 and mx <= MAX_ABS, (what, rel, mx)
    for n in range(y_ref.shape[0]):
        rel, mx = owq_ref.parity_errors(y_gpu[n], y_ref[n])
        assert rel <= REL_L2 and mx <= MAX_ABS, (what, n, rel, mx)


CASES = [
    # name, d_in, d_out, bits, group, k, batch, split
    ("s3_ch", 1024, 96, 3, 0, 8, 16, 0),
    ("s4_ch", 1024, 96, 4, 0, 8, 32, 2),
    ("s3_b1", 512, 64, 3, 0, 4, 1, 0),
    ("s4_b1_one_block", 128, 40, 4, 0, 3, 1, 1),         # one block: three of the four waves have nothing
    ("s3_rows", 768, 600, 3, 0, 24, 5, 0),               # 19 row tiles, the last one ragged
    ("s3_g128", 2048, 130, 3, 128, 16, 4, 0),
    ("s4_g128", 2048, 130, 4, 128, 16, 16, 0),
    ("s4_g256", 2048, 67, 4, 256, 5, 31, 4),
    ("s3_g512", 2560, 300, 3, 512, 9, 17, 5),            # groups of four blocks
    ("s3_g128_split3", 2560, 300, 3, 128, 9, 7, 3),      # 20 blocks in ranges of 6, 7, 7
    ("s4_g128_split5", 1280, 64, 4, 128, 40, 8, 5),      # two blocks per workgroup: half of the waves idle
    ("s3_ch_split2", 3072, 100, 3, 0, 33, 8, 2),
    ("s3_split_max", 512, 64, 3, 0, 4, 2, 4),            # one block per workgroup
    ("s4_k0", 1536, 64, 4, 0, 0, 7, 0),
    ("s3_k0_split2", 1536, 64, 3, 128, 0, 7, 2),
    ("s3_many_weak", 256, 40, 3, 0, 200, 12, 0),         # 13 k-steps per wave: most of them not fetched ahead
    ("s4_many_weak_split2", 1024, 70, 4, 128, 500, 9, 2),
    ("s3_k_odd_units", 1024, 64, 3, 0, 24, 3, 0),        # kp = 24: the last weak k-step is half empty
    ("s3_one_row", 512, 1, 3, 0, 2, 3, 0),
    ("s3_rows_rt1", 768, 600, 3, 0, 24, 5, 101),          # one row tile per workgroup, four slices of the columns
    ("s3_rows_rt2", 768, 600, 3, 0, 24, 9, 202),          # two row tiles x two slices, two ranges; 19 row tiles: ragged
    ("s3_rows_rt4", 768, 600, 3, 0, 24, 32, 303),         # four row tiles, no slices, three ranges
    ("s4_g128_rt1", 2048, 130, 4, 128, 16, 16, 102),
    ("s4_g128_rt2", 2048, 130, 4, 128, 16, 3, 201),
    ("s4_g128_rt4", 2048, 130, 4, 128, 16, 32, 304),
    ("s3_g256_rt4", 4096, 260, 3, 256, 41, 20, 300),
    ("s4_wide", 8192, 64, 4, 128, 82, 16, 0),            # 64 blocks x 16 tokens: the ranges must be cut to fit LDS
    ("s3_tail_pass", 1024, 96, 3, 0, 8, 64 + 6, 0),      # 64 tokens by the three-launch path, 6 by this kernel
    ("s4_tail_pass_g", 1024, 96, 4, 128, 8, 128 + 32, 2),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_layers_match_oracle(env, case):
    name, d_in, d_out, bits, group, k, batch, split = case
    layer = make_layer(LayerSpec(name, d_in, d_out, bits, group, k, seed=zlib.crc32(name.encode()) % 10000))
    x = make_x(layer, batch)
    print(f"case {name}: d_in={d_in} d_out={d_out} bits={bits} group={group} k={k} batch={batch} split={split}", flush=True)
    check(run_gpu(env, layer, x, split), owq_ref.owq_linear_layer(layer, x), name)


def test_split_limits(env):
    torch, B = env
    layer = make_layer(LayerSpec("lim", 512, 64, 3, 0, 4, 3))
    lin = B.OwqLinear(layer, layout=TILE)
    B.owq_set_launch(lin.handle, 0, 0, 0, 4)
    with pytest.raises(B.OwqError):
        B.owq_set_launch(lin.handle, 0, 0, 0, 5)           # more ranges than blocks
    with pytest.raises(B.OwqError):
        B.owq_set_launch(lin.handle, 0, 0, 0, -2)
    with pytest.raises(B.OwqError):
        B.owq_set_launch(lin.handle, 0, 0, 0, 401)
    B.owq_set_launch(lin.handle, 0, 0, 0, 304)
    lin.close()


def test_a_shape_that_does_not_fit_the_batch_is_an_error(env):
    # one range of 24 blocks for 32 tokens is more than a workgroup stages; the library's own choice works
    torch, B = env
    layer = make_layer(LayerSpec("nofit", 3072, 64, 3, 0, 4, 3))
    x = torch.from_numpy(make_x(layer, 32)).cuda()
    lin = B.OwqLinear(layer, layout=TILE)
    B.owq_set_launch(lin.handle, 0, 0, 0, 1)
    with pytest.raises(B.OwqError):
        lin(x)
    B.owq_set_launch(lin.handle, 0, 0, 0, 300)         # the library chooses the ranges
    y = lin(x)
    torch.cuda.synchronize()
    lin.close()
    check(y.cpu().numpy(), owq_ref.owq_linear_layer(layer, x.cpu().numpy()), "nofit")


def test_all_columns_weak_reproduces_fp16_matmul(env):
    rng = np.random.default_rng(3)
    d_out, d_in = 48, 384
    w16 = rng.normal(0, 0.02, size=(d_out, d_in)).astype(np.float16)
    layer = make_layer(LayerSpec("allweak", d_in, d_out, 3, 0, 0, 5))
    layer.spec = LayerSpec("allweak", d_in, d_out, 3, 0, d_in, 5)
    layer.weak_idx = np.arange(d_in, dtype=np.int32)
    layer.weak_w = w16
    x = rng.normal(0, 1, size=(12, d_in)).astype(np.float16)
    want = x.astype(np.float64) @ w16.astype(np.float64).T
    check(run_gpu(env, layer, x), want, "allweak")
    check(run_gpu(env, layer, x, 2), want, "allweak split 2")


@pytest.mark.parametrize("bits,group,split", [(3, 0, 102), (4, 0, 202), (3, 128, 302), (4, 128, 2)])
def test_one_hot_probing_is_bit_exact(env, bits, group, split):
    # x = e_j, 32 columns per call, reads the whole effective matrix back through the kernel:
    # fp16(s*(q-z)) at dense positions, Ww at weak ones.
    torch, B = env
    d_in, d_out, k = 640, 70, 9
    layer = make_layer(LayerSpec("onehot", d_in, d_out, bits, group, k, 17 + bits + group))
    eye = np.eye(d_in, dtype=np.float16)
    want = owq_ref.to_fp16(owq_ref.owq_linear_layer(layer, eye))
    lin = B.OwqLinear(layer, layout=TILE)
    B.owq_set_launch(lin.handle, 0, 0, 0, split)
    xd = torch.from_numpy(eye).cuda()
    y = torch.empty((d_in, d_out), dtype=torch.float16, device="cuda")
    for j0 in range(0, d_in, 32):
        lin(xd[j0:j0 + 32], out=y[j0:j0 + 32])
    torch.cuda.synchronize()
    lin.close()
    np.testing.assert_array_equal(y.cpu().numpy().view(np.uint16), want.view(np.uint16))


@pytest.mark.parametrize("bits,group,d_in,split", [(3, 0, 4096, 108), (4, 128, 2048, 204), (3, 256, 1024, 302), (4, 0, 2048, 4)])
def test_integer_inputs_are_bit_exact(env, bits, group, d_in, split):
    # s = 2^-m, integer z, x in {-1, 0, 1}: every partial sum is a small dyadic number,
    # fp32 accumulation is exact, so y must equal the rounded oracle result bit for bit.
    rng = np.random.default_rng(bits * 100 + group)
    d_out, k = 64, 6
    layer = make_layer(LayerSpec("exact", d_in, d_out, bits, group, k, 5))
    layer.scale = (2.0 ** -rng.integers(3, 7, size=layer.scale.shape)).astype(np.float16)
    layer.weak_w = (rng.integers(-8, 9, size=layer.weak_w.shape) / 16.0).astype(np.float16)
    x = rng.integers(-1, 2, size=(32, d_in)).astype(np.float16)
    y = run_gpu(env, layer, x, split)
    want = owq_ref.to_fp16(owq_ref.owq_linear_layer(layer, x))
    np.testing.assert_array_equal(y.view(np.uint16), want.view(np.uint16))


def test_weak_positions_do_not_leak_into_the_dense_term(env):
    # Inf and NaN at weak positions of x reach y only through the weak columns (zero weights here)
    layer = make_layer(LayerSpec("leak", 1024, 64, 3, 128, 8, 21))
    layer.weak_w[:] = 0
    x = make_x(layer, 6)
    ref = owq_ref.owq_linear_layer(layer, np.where(np.isin(np.arange(1024), layer.weak_idx), 0, x).astype(np.float16))
    x[:, layer.weak_idx[::2]] = np.float16(6e4)            # finite but huge: 0 * 6e4 = 0 in the weak product
    y = run_gpu(env, layer, x)
    assert np.isfinite(y).all()
    check(y, ref, "leak")


def test_runs_are_reproducible_and_agree_with_three_launches(env):
    layer = make_layer(LayerSpec("repro", 2048, 200, 4, 128, 20, 77))
    x = make_x(layer, 16)
    a = run_gpu(env, layer, x, 2)
    b = run_gpu(env, layer, x, 2)
    np.testing.assert_array_equal(a.view(np.uint16), b.view(np.uint16))
    c = run_gpu(env, layer, x, -1)
    check(a, owq_ref.owq_linear_layer(layer, x), "one launch")
    check(c, owq_ref.owq_linear_layer(layer, x), "three launches")


def test_unaligned_x_takes_the_other_path(env):
    torch, B = env
    layer = make_layer(LayerSpec("unal", 1024, 64, 3, 0, 8, 4))
    x = make_x(layer, 5)
    lin = B.OwqLinear(layer, layout=TILE)
    buf = torch.zeros(5 * 1024 + 8, dtype=torch.float16, device="cuda")
    xv = buf[1:1 + 5 * 1024].view(5, 1024)                 # 2-byte aligned only
    xv.copy_(torch.from_numpy(x))
    y = torch.empty((5, 64), dtype=torch.float16, device="cuda")
    B.owq_linear(lin.handle, xv.data_ptr(), y.data_ptr(), 5, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    lin.close()
    check(y.cpu().numpy(), owq_ref.owq_linear_layer(layer, x), "unaligned")


@pytest.mark.parametrize("li,batch", [(0, 4), (1, 16), (2, 4), (2, 16)])
def test_llama13b_layers_sampled_rows(env, li, batch):
    # full-size layers of the 4-bit group-128 workload in the default launch configuration;
    # the oracle computes a sample of the output rows
    spec = CONFIGS[3][li]
    print(f"full-size {spec.name} batch={batch}", flush=True)
    layer = make_layer(spec)
    x = make_x(layer, batch)
    y = run_gpu(env, layer, x)
    rng = np.random.default_rng(li)
    rows = np.unique(np.concatenate([rng.integers(0, spec.d_out, size=600), [0, 31, 32, spec.d_out - 1]]))
    want = owq_ref.owq_linear_ref(layer.codes[rows], layer.scale[rows], layer.zero[rows], layer.group_size,
                                  layer.weak_idx, layer.weak_w[rows], x)
    check(y[:, rows], want, spec.name)
    assert np.isfinite(y.astype(np.float32)).all()
