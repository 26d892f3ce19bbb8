"""GPU parity: owq_linear through the C ABI against the fp64 CPU oracle.

Tolerances (the project's stated bar for y, fp32 accumulation and fp16 output):
relative L2 error <= 1e-3 and max-abs error <= 1e-2 * rms(y), over the whole output and
per batch row.  Packing and indexing are compared for equality.
"""
import zlib

import numpy as np
import pytest

from oracle import owq_ref, packfmt
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
    binding.lib()          # fails loudly if the HIP library is missing
    torch.cuda.set_device(0)
    return torch, binding


def run_gpu(env, layer, x):
    torch, B = env
    lin = B.OwqLinear(layer)
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
    # name, d_in, d_out, bits, group, k, batch      (several tiles, ragged tails, odd tile shapes)
    ("b3_ch", 1024, 96, 3, 0, 8, 1),
    ("b4_ch", 1024, 96, 4, 0, 8, 1),
    ("b3_g128", 2048, 130, 3, 128, 16, 2),
    ("b4_g256", 2048, 67, 4, 256, 5, 3),
    ("b3_cw20", 128 * 40, 50, 3, 128, 51, 1),       # tiles of 3 rows x 20 blocks, 60 lanes
    ("b4_cw12", 128 * 108, 23, 4, 128, 138, 1),     # tiles of 5 rows x 12 blocks
    ("b3_cw64", 128 * 128, 40, 3, 0, 128, 1),       # two slabs of 64 blocks
    ("b3_ragged_in", 1000, 33, 3, 0, 7, 2),         # d_in not a multiple of 128 nor of 8
    ("b4_ragged_in", 203, 5, 4, 0, 3, 3),
    ("b3_one_row", 512, 1, 3, 0, 2, 1),
    ("b4_one_col", 1, 9, 4, 0, 0, 2),
    ("b3_k0", 1536, 64, 3, 128, 0, 1),
    ("b3_many_weak", 256, 40, 3, 0, 100, 2),        # more weak chunks than blocks
    ("b4_batch16", 1024, 128, 4, 128, 10, 16),
    # one slab of 16, 32 or 64 blocks: a wave owns whole rows and stores them itself
    ("b4_own32", 4096, 77, 4, 128, 40, 2),
    ("b3_own32_k0", 4096, 64, 3, 0, 0, 1),
    ("b3_own64", 8192, 50, 3, 0, 64, 2),
    ("b4_own64_g", 8192, 33, 4, 1024, 82, 3),
    ("b3_own16_kmax", 2048, 41, 3, 0, 128, 2),      # as many weak chunks as blocks
    ("b3_16_kover", 2048, 41, 3, 0, 136, 2),        # one more: rows go through the shared reduction again
]


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_small_layers_match_oracle(env, case):
    name, d_in, d_out, bits, group, k, batch = case
    layer = make_layer(LayerSpec(name, d_in, d_out, bits, group, k, seed=zlib.crc32(name.encode()) % 10000))
    x = make_x(layer, batch)
    print(f"case {name}: d_in={d_in} d_out={d_out} bits={bits} group={group} k={k} batch={batch}", flush=True)
    check(run_gpu(env, layer, x), owq_ref.owq_linear_layer(layer, x), name)


def test_all_columns_weak_reproduces_fp16_matmul(env):
    rng = np.random.default_rng(3)
    d_out, d_in = 48, 384
    w16 = rng.normal(0, 0.02, size=(d_out, d_in)).astype(np.float16)
    layer = make_layer(LayerSpec("allweak", d_in, d_out, 3, 0, 0, 5))
    layer.spec = LayerSpec("allweak", d_in, d_out, 3, 0, d_in, 5)
    layer.weak_idx = np.arange(d_in, dtype=np.int32)
    layer.weak_w = w16
    x = rng.normal(0, 1, size=(2, d_in)).astype(np.float16)
    want = x.astype(np.float64) @ w16.astype(np.float64).T
    check(run_gpu(env, layer, x), want, "allweak")


@pytest.mark.parametrize("bits,group", [(3, 0), (4, 0), (3, 128), (4, 128)])
def test_one_hot_probing_is_bit_exact(env, bits, group):
    # x = e_j for every j reads the whole effective matrix back through the kernel:
    # fp16(s*(q-z)) at dense positions (integer z: exact in fp32), Ww at weak ones.
    d_in, d_out, k = 384, 70, 9
    layer = make_layer(LayerSpec("onehot", d_in, d_out, bits, group, k, 17 + bits + group))
    eye = np.eye(d_in, dtype=np.float16)
    y = run_gpu(env, layer, eye)                                  # [d_in, d_out]
    want = owq_ref.to_fp16(owq_ref.owq_linear_layer(layer, eye))
    np.testing.assert_array_equal(y.view(np.uint16), want.view(np.uint16))


@pytest.mark.parametrize("bits,d_in", [(3, 2048), (4, 4096), (3, 8192)])
def test_one_hot_probing_of_sampled_columns_when_a_wave_owns_rows(env, bits, d_in):
    # the same read-back as above on the row-owning variants (one slab of 16, 32, 64 blocks), 192 sampled columns
    d_out, k = 37, 24
    layer = make_layer(LayerSpec("onehot_own", d_in, d_out, bits, 128, k, 23 + bits))
    rng = np.random.default_rng(d_in)
    cols = np.unique(np.concatenate([rng.integers(0, d_in, size=160), layer.weak_idx[:16], [0, d_in - 1]]))
    x = np.zeros((cols.size, d_in), dtype=np.float16)
    x[np.arange(cols.size), cols] = 1
    y = run_gpu(env, layer, x)
    want = owq_ref.to_fp16(owq_ref.owq_linear_layer(layer, x))
    np.testing.assert_array_equal(y.view(np.uint16), want.view(np.uint16))


@pytest.mark.parametrize("bits,group,d_in", [(3, 0, 4096), (4, 128, 2048), (3, 128, 1024), (4, 0, 8192), (3, 128, 8192)])
def test_integer_inputs_are_bit_exact(env, bits, group, d_in):
    # s = 2^-m, integer z, x in {-1, 0, 1}: every partial sum is a small dyadic number,
    # fp32 accumulation is exact, so y must equal the rounded oracle result bit for bit.
    rng = np.random.default_rng(bits * 100 + group)
    d_out, k = 64, 6
    layer = make_layer(LayerSpec("exact", d_in, d_out, bits, group, k, 5))
    layer.scale = (2.0 ** -rng.integers(3, 7, size=layer.scale.shape)).astype(np.float16)
    layer.weak_w = (rng.integers(-8, 9, size=layer.weak_w.shape) / 16.0).astype(np.float16)
    x = rng.integers(-1, 2, size=(2, d_in)).astype(np.float16)
    y = run_gpu(env, layer, x)
    want = owq_ref.to_fp16(owq_ref.owq_linear_layer(layer, x))
    np.testing.assert_array_equal(y.view(np.uint16), want.view(np.uint16))


def test_uploaded_blob_equals_oracle_pack_and_runs_are_reproducible(env):
    torch, B = env
    layer = make_layer(LayerSpec("blob", 2048, 77, 3, 128, 12, 8))
    lin = B.OwqLinear(layer)
    blob = B.owq_export_packed(lin.handle)
    want, _ = packfmt.pack_layer(layer.codes, layer.scale, layer.zero, layer.group_size,
                                 layer.weak_idx, layer.weak_w, layer.bits)
    np.testing.assert_array_equal(blob, want)
    x = torch.from_numpy(make_x(layer, 4)).cuda()
    a = lin(x).cpu().numpy()
    b = lin(x).cpu().numpy()
    np.testing.assert_array_equal(a.view(np.uint16), b.view(np.uint16))
    lin.close()


def test_weak_positions_do_not_leak_into_the_dense_term(env):
    # huge activations at the weak columns with zero weak weights: y must not move
    layer = make_layer(LayerSpec("leak", 1024, 64, 3, 0, 8, 12))
    layer.weak_w[:] = 0
    x = make_x(layer, 1)
    x2 = x.copy()
    x2[:, layer.weak_idx] = np.float16(30000.0)
    a = run_gpu(env, layer, x)
    b = run_gpu(env, layer, x2)
    np.testing.assert_array_equal(a.view(np.uint16), b.view(np.uint16))
    check(a, owq_ref.owq_linear_layer(layer, x), "leak")


def test_positive_mean_activations_stay_in_tolerance(env):
    # post-ReLU-like inputs make the constant part of the unpack trick large
    layer = make_layer(LayerSpec("relu", 8192, 96, 3, 0, 16, 13))
    layer.zero[:] = np.float16(3.5)            # near the mean code: the result is a small difference
    x = np.abs(make_x(layer, 2))
    check(run_gpu(env, layer, x), owq_ref.owq_linear_layer(layer, x), "relu")


def test_tiny_activations_keep_their_precision(env):
    layer = make_layer(LayerSpec("tinyx", 1024, 64, 4, 0, 4, 14))
    x = (make_x(layer, 1).astype(np.float32) * 1e-3).astype(np.float16)
    check(run_gpu(env, layer, x), owq_ref.owq_linear_layer(layer, x), "tinyx")


def test_launch_shapes_do_not_change_the_result(env):
    torch, B = env
    layer = make_layer(LayerSpec("shapes", 128 * 128, 64, 3, 128, 32, 15))
    x = make_x(layer, 1)
    want = owq_ref.owq_linear_layer(layer, x)
    lin = B.OwqLinear(layer)
    xd = torch.from_numpy(x).cuda()
    for rtw, rsplit, waves, depth in [(1, 1, 1, 2), (1, 1, 2, 4), (8, 2, 4, 2), (16, 4, 8, 4), (64, 1, 2, 4), (5, 5, 2, 2), (16, 2, 4, 8), (7, 1, 1, 8), (9, 3, 2, 3)]:
        B.owq_set_launch(lin.handle, rtw, rsplit, waves, depth)
        info = lin.info()
        print("shape", rtw, rsplit, waves, depth, "->", info.workgroups, info.lds_bytes, flush=True)
        y = lin(xd)
        torch.cuda.synchronize()
        check(y.cpu().numpy(), want, f"shape {rtw},{rsplit},{waves},{depth}")
    with pytest.raises(B.OwqError):
        B.owq_set_launch(lin.handle, 4, 3, 2, 4)       # 3 does not divide 4
    lin.close()


@pytest.mark.parametrize("d_in,bits,group,k", [(4096, 3, 128, 64), (2048, 4, 256, 21), (8192, 3, 0, 40), (16384, 4, 1024, 130)])
def test_launch_shapes_of_the_row_owning_and_deep_variants(env, d_in, bits, group, k):
    # One slab of 16, 32, 64 blocks (a wave owns its rows) and two slabs (rows shared), a ragged number of rows,
    # 2 to 4 tiles in flight, and shapes with so many rows per workgroup and so few threads that the staging of
    # the scales and weak weights through LDS takes its loop beyond the units fetched ahead.
    torch, B = env
    layer = make_layer(LayerSpec("own_shapes", d_in, 203, bits, group, k, 31 + bits))
    x = make_x(layer, 2)
    want = owq_ref.owq_linear_layer(layer, x)
    lin = B.OwqLinear(layer)
    xd = torch.from_numpy(x).cuda()
    nslab = lin.info().nslab
    for rtw, rsplit, waves, depth in [(4, 2, 2, 3), (8, 4, 4, 4), (3, 1, 1, 3), (6, 2, 2, 4), (16, 1, 1, 3), (32, 1, 1, 2), (12, 4, 4, 3)]:
        if (nslab * rsplit) % waves:
            continue
        B.owq_set_launch(lin.handle, rtw, rsplit, waves, depth)
        info = lin.info()
        print("shape", rtw, rsplit, waves, depth, "->", info.workgroups, info.lds_bytes, flush=True)
        y = lin(xd)
        torch.cuda.synchronize()
        check(y.cpu().numpy(), want, f"{d_in}: shape {rtw},{rsplit},{waves},{depth}")
    lin.close()


def test_batch_edge_cases(env):
    torch, B = env
    layer = make_layer(LayerSpec("edge", 512, 32, 4, 0, 4, 16))
    lin = B.OwqLinear(layer)
    x = torch.from_numpy(make_x(layer, 1)).cuda()
    y = torch.full((1, 32), 7.0, dtype=torch.float16, device="cuda")
    B.owq_linear(lin.handle, x.data_ptr(), y.data_ptr(), 0)         # no-op
    torch.cuda.synchronize()
    assert (y == 7.0).all()
    with pytest.raises(B.OwqError) as e:
        B.owq_linear(lin.handle, x.data_ptr(), y.data_ptr(), -1)
    assert e.value.status == B.OWQ_ERR_BATCH
    with pytest.raises(B.OwqError) as e:
        B.owq_linear(lin.handle, 0, y.data_ptr(), 1)
    assert e.value.status == B.OWQ_ERR_NULL
    lin.close()


FULL = [(1, 0, 1), (2, 0, 1), (2, 1, 1), (5, 0, 1), (3, 0, 4), (3, 2, 16)]


@pytest.mark.parametrize("cfg,li,batch", FULL, ids=[f"cfg{c}_{l}_b{b}" for c, l, b in FULL])
def test_full_size_configs(env, cfg, li, batch):
    spec = CONFIGS[cfg][li]
    print(f"full-size {spec.name} batch={batch}", flush=True)
    layer = make_layer(spec)
    x = make_x(layer, batch)
    check(run_gpu(env, layer, x), owq_ref.owq_linear_layer(layer, x), spec.name)
