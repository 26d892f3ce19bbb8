"""GPU parity of the batched (tile layout, matrix core) path against the fp64 CPU oracle.

Same bar as the single-token path: relative L2 error <= 1e-3 and max-abs error <=
1e-2 * rms(y) over the whole output and per token; bit-exact where the arithmetic is exact.
"""
import zlib

import numpy as np
import pytest

from oracle import owq_ref, packfmt
from synth import CONFIGS, LayerSpec, make_layer, make_x

pytestmark = pytest.mark.gpu

REL_L2 = 1e-3
MAX_ABS = 1e-2
TILE = 1


@pytest.fixture(scope="module")
def env():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2306_02272_amd import binding
    binding.lib()          # fails loudly if the HIP library is missing
    torch.cuda.set_device(0)
    return torch, binding


def run_gpu(env, layer, x, grid=0, three_launches=False):
    torch, B = env
    lin = B.OwqLinear(layer, layout=TILE)
    if grid or three_launches:
        # prefetch_depth = -1: passes of 32 tokens or fewer take the three-launch path too
        B.owq_set_launch(lin.handle, grid, 0, 0, -1 if three_launches else 0)
    xd = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    y = lin(xd)
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


SMALL = [
    # name, d_in, d_out, bits, group, k, batch
    ("t3_ch", 1024, 96, 3, 0, 8, 64),
    ("t4_ch", 1024, 96, 4, 0, 8, 64),
    ("t3_rows", 768, 600, 3, 0, 24, 64),            # three row groups, the last one ragged
    ("t3_b1", 512, 64, 3, 0, 4, 1),
    ("t4_b33", 512, 70, 4, 0, 5, 33),
    ("t3_b65", 512, 40, 3, 0, 16, 65),              # two passes
    ("t3_b130", 256, 33, 3, 0, 3, 130),             # three passes, one column step
    ("t3_g128", 2048, 130, 3, 128, 16, 40),
    ("t4_g256", 2048, 67, 4, 256, 5, 64),
    ("t3_g512", 2560, 300, 3, 512, 9, 17),          # groups span column steps and workgroups
    ("t3_ragged_in", 1000, 33, 3, 0, 7, 20),        # d_in not a multiple of 256 nor of 8
    ("t4_ragged_g", 1100, 45, 4, 128, 3, 64),       # last group and last block incomplete
    ("t3_one_row", 512, 1, 3, 0, 2, 3),
    ("t4_one_col", 1, 9, 4, 0, 0, 2),
    ("t3_k0", 1536, 64, 3, 0, 0, 64),
    ("t3_many_weak", 256, 40, 3, 0, 100, 64),
    ("t3_k_odd_units", 1024, 64, 3, 0, 24, 64),     # kp = 24: the last weak K-step is half empty
]


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_small_layers_match_oracle(env, case):
    name, d_in, d_out, bits, group, k, batch = case
    layer = make_layer(LayerSpec(name, d_in, d_out, bits, group, k, seed=zlib.crc32(name.encode()) % 10000))
    x = make_x(layer, batch)
    print(f"case {name}: d_in={d_in} d_out={d_out} bits={bits} group={group} k={k} batch={batch}", flush=True)
    want = owq_ref.owq_linear_layer(layer, x)
    check(run_gpu(env, layer, x), want, name)
    if batch % 64 and batch % 64 <= 16:       # the last pass would take the one-launch kernel: three launches too
        print("  three launches", flush=True)
        check(run_gpu(env, layer, x, three_launches=True), want, name + " three launches")


@pytest.mark.parametrize("grid", [1, 2, 3, 7, 12])
def test_any_number_of_workgroups_gives_the_same_sums(env, grid):
    # 3 row groups x 4 column steps = 12 steps cut into `grid` ranges
    layer = make_layer(LayerSpec("grid", 1024, 700, 3, 0, 16, 31))
    x = make_x(layer, 48)
    print(f"grid {grid}", flush=True)
    check(run_gpu(env, layer, x, grid), owq_ref.owq_linear_layer(layer, x), f"grid {grid}")


@pytest.mark.parametrize("split,waves", [(1, 4), (2, 4), (3, 4), (4, 4), (2, 8), (3, 8)])
def test_column_ranges_aligned_to_row_groups(env, split, waves):
    # 4 column steps per row group cut into `split` ranges; 3 row groups of 256 rows or 2 of 512
    torch, B = env
    layer = make_layer(LayerSpec("split", 1024, 700, 4, 0, 16, 32))
    x = make_x(layer, 64)
    lin = B.OwqLinear(layer, layout=TILE)
    B.owq_set_launch(lin.handle, 0, split, waves, 0)
    info = lin.info()
    print(f"split {split} waves {waves}: {info.workgroups} workgroups", flush=True)
    assert info.row_splits == split and info.waves_per_wg == waves
    assert info.workgroups == split * (3 if waves == 4 else 2)
    y = lin(torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    check(y.cpu().numpy(), owq_ref.owq_linear_layer(layer, x), f"split {split} waves {waves}")
    with pytest.raises(B.OwqError):
        B.owq_set_launch(lin.handle, 0, 5, waves, 0)       # more ranges than column steps
    lin.close()


def test_grouped_layers_take_four_waves_only(env):
    torch, B = env
    layer = make_layer(LayerSpec("g8", 1024, 300, 4, 128, 16, 33))
    lin = B.OwqLinear(layer, layout=TILE)
    with pytest.raises(B.OwqError) as e:
        B.owq_set_launch(lin.handle, 0, 0, 8, 0)
    assert e.value.status == B.OWQ_ERR_SHAPE
    B.owq_set_launch(lin.handle, 0, 2, 4, 0)
    x = make_x(layer, 64)
    y = lin(torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    check(y.cpu().numpy(), owq_ref.owq_linear_layer(layer, x), "grouped, two ranges")
    lin.close()


def test_all_columns_weak_reproduces_fp16_matmul(env):
    rng = np.random.default_rng(3)
    d_out, d_in = 48, 384
    w16 = rng.normal(0, 0.02, size=(d_out, d_in)).astype(np.float16)
    layer = make_layer(LayerSpec("allweak", d_in, d_out, 3, 0, 0, 5))
    layer.spec = LayerSpec("allweak", d_in, d_out, 3, 0, d_in, 5)
    layer.weak_idx = np.arange(d_in, dtype=np.int32)
    layer.weak_w = w16
    x = rng.normal(0, 1, size=(40, d_in)).astype(np.float16)
    want = x.astype(np.float64) @ w16.astype(np.float64).T
    check(run_gpu(env, layer, x), want, "allweak")


@pytest.mark.parametrize("bits,group", [(3, 0), (4, 0), (3, 128), (4, 128)])
def test_one_hot_probing_is_bit_exact(env, bits, group):
    # x = e_j for every j reads the whole effective matrix back through the kernels:
    # fp16(s*(q-z)) at dense positions, Ww at weak ones; checks every (row, column) ->
    # (tile, lane, bit) mapping, the operand layouts of the matrix instruction and the gather.
    d_in, d_out, k = 640, 70, 9
    layer = make_layer(LayerSpec("onehot", d_in, d_out, bits, group, k, 17 + bits + group))
    eye = np.eye(d_in, dtype=np.float16)
    y = run_gpu(env, layer, eye)                                  # [d_in, d_out]
    want = owq_ref.to_fp16(owq_ref.owq_linear_layer(layer, eye))
    np.testing.assert_array_equal(y.view(np.uint16), want.view(np.uint16))


@pytest.mark.parametrize("bits,group,d_in", [(3, 0, 4096), (4, 128, 2048), (3, 256, 1024)])
def test_integer_inputs_are_bit_exact(env, bits, group, d_in):
    # s = 2^-m, integer z, x in {-1, 0, 1}: every partial sum is a small dyadic number,
    # fp32 accumulation is exact, so y must equal the rounded oracle result bit for bit.
    rng = np.random.default_rng(bits * 100 + group)
    d_out, k = 64, 6
    layer = make_layer(LayerSpec("exact", d_in, d_out, bits, group, k, 5))
    layer.scale = (2.0 ** -rng.integers(3, 7, size=layer.scale.shape)).astype(np.float16)
    layer.weak_w = (rng.integers(-8, 9, size=layer.weak_w.shape) / 16.0).astype(np.float16)
    x = rng.integers(-1, 2, size=(64, d_in)).astype(np.float16)
    y = run_gpu(env, layer, x)
    want = owq_ref.to_fp16(owq_ref.owq_linear_layer(layer, x))
    np.testing.assert_array_equal(y.view(np.uint16), want.view(np.uint16))


def test_uploaded_blob_equals_oracle_pack_and_runs_are_reproducible(env):
    torch, B = env
    layer = make_layer(LayerSpec("blob", 2048, 77, 3, 0, 12, 8))
    lin = B.OwqLinear(layer, layout=TILE)
    info = lin.info()
    blob = B.owq_export_packed(lin.handle)
    want, geo = packfmt.pack_layer(layer.codes, layer.scale, layer.zero, layer.group_size,
                                   layer.weak_idx, layer.weak_w, layer.bits, layout=TILE)
    assert info.total_bytes >= geo.total_bytes and info.off_scratch == geo.off_scratch == geo.total_bytes
    np.testing.assert_array_equal(blob[:geo.off_scratch], want[:geo.off_scratch])
    x = torch.from_numpy(make_x(layer, 64)).cuda()
    a = lin(x).cpu().numpy()
    b = lin(x).cpu().numpy()
    np.testing.assert_array_equal(a.view(np.uint16), b.view(np.uint16))
    # the two layouts hold the same layer
    gemv = B.OwqLinear(layer)
    c = gemv(x).cpu().numpy()
    want_y = owq_ref.owq_linear_layer(layer, x.cpu().numpy())
    check(a, want_y, "tile")
    check(c, want_y, "gemv")
    gemv.close()
    lin.close()


def test_weak_positions_do_not_leak_into_the_dense_term(env):
    layer = make_layer(LayerSpec("leak", 1024, 64, 3, 0, 8, 12))
    layer.weak_w[:] = 0
    x = make_x(layer, 64)
    x2 = x.copy()
    x2[:, layer.weak_idx] = np.float16(30000.0)
    x2[3, layer.weak_idx[0]] = np.float16(np.inf)
    a = run_gpu(env, layer, x)
    b = run_gpu(env, layer, x2)
    keep = np.ones(64, dtype=bool)
    keep[3] = False                       # 0 * inf in the weak product of that token is NaN by definition
    np.testing.assert_array_equal(a[keep].view(np.uint16), b[keep].view(np.uint16))
    check(a, owq_ref.owq_linear_layer(layer, x), "leak")


def test_positive_mean_activations_stay_in_tolerance(env):
    layer = make_layer(LayerSpec("relu", 8192, 96, 3, 0, 16, 13))
    layer.zero[:] = np.float16(3.5)
    x = np.abs(make_x(layer, 64))
    check(run_gpu(env, layer, x), owq_ref.owq_linear_layer(layer, x), "relu")


def test_batch_edge_cases(env):
    torch, B = env
    layer = make_layer(LayerSpec("edge", 512, 32, 4, 0, 4, 16))
    lin = B.OwqLinear(layer, layout=TILE)
    x = torch.from_numpy(make_x(layer, 1)).cuda()
    y = torch.full((1, 32), 7.0, dtype=torch.float16, device="cuda")
    B.owq_linear(lin.handle, x.data_ptr(), y.data_ptr(), 0)         # no-op
    torch.cuda.synchronize()
    assert (y == 7.0).all()
    with pytest.raises(B.OwqError) as e:
        B.owq_linear(lin.handle, x.data_ptr(), y.data_ptr(), -1)
    assert e.value.status == B.OWQ_ERR_BATCH
    with pytest.raises(B.OwqError):
        B.owq_set_launch(lin.handle, 100000)
    with pytest.raises(B.OwqError):
        B.owq_set_launch(lin.handle, 1, 2, 0, 0)
    lin.close()


def _sampled_rows_check(env, spec, batch, n_rows, seed):
    """Full-size layer, launch shape as benchmarked; the oracle on a sample of the output rows."""
    torch, B = env
    layer = make_layer(spec)
    x = make_x(layer, batch)
    y = run_gpu(env, layer, x)
    rng = np.random.default_rng(seed)
    rows = np.unique(np.concatenate([rng.integers(0, spec.d_out, size=n_rows),
                                     [0, 31, 32, 255, 256, spec.d_out - 1]]))
    want = owq_ref.owq_linear_ref(layer.codes[rows], layer.scale[rows], layer.zero[rows], layer.group_size,
                                  layer.weak_idx, layer.weak_w[rows], x)
    check(y[:, rows], want, spec.name)
    assert np.isfinite(y.astype(np.float32)).all()


@pytest.mark.parametrize("li", [0, 1])
def test_opt66b_ffn_batch64_sampled_rows(env, li):
    spec = CONFIGS[4][li]
    print(f"full-size {spec.name} batch=64 (sampled rows)", flush=True)
    _sampled_rows_check(env, spec, 64, 768, 40 + li)


def test_llama13b_down_batch16_tile_layout(env):
    spec = CONFIGS[3][2]
    print(f"full-size {spec.name} batch=16, tile layout", flush=True)
    _sampled_rows_check(env, spec, 16, 512, 50)
