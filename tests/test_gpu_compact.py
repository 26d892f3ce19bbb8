"""GPU parity of the storage-favoured layout (weak columns taken out of the low-bit matrix;
appendix B.2 of the paper) against the fp64 CPU oracle, through the C ABI."""
import zlib

import numpy as np
import pytest

from oracle import owq_ref, packfmt
from synth import CONFIGS, LayerSpec, make_layer, make_x

pytestmark = pytest.mark.gpu
COMPACT = 2
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


def run_gpu(env, layer, x):
    torch, B = env
    lin = B.OwqLinear(layer, layout=COMPACT)
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
    # name, d_in, d_out, bits, k, batch
    ("c3", 1024, 96, 3, 8, 1),
    ("c4", 1024, 96, 4, 8, 3),
    ("c3_block_saved", 1024 + 128, 70, 3, 128, 1),       # exactly one block of columns fewer
    ("c3_k1", 512, 64, 3, 1, 1),
    ("c4_k0", 768, 40, 4, 0, 2),                           # nothing to take out: same bytes as the other layout
    ("c3_many", 2048, 33, 3, 700, 1),
    ("c3_ragged", 1000, 33, 3, 7, 2),                      # d_in not a multiple of 128
    ("c4_odd", 1003, 45, 4, 40, 1),                        # d_in not a multiple of 8: element-wise staging
    ("c3_wide", 128 * 72, 64, 3, 64, 1),                   # more staging units than a thread keeps in registers
    ("c3_one_row", 512, 1, 3, 2, 1),
    ("c4_tall", 256, 1500, 4, 16, 1),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_layers_match_oracle(env, case):
    name, d_in, d_out, bits, k, batch = case
    layer = make_layer(LayerSpec(name, d_in, d_out, bits, 0, k, seed=zlib.crc32(name.encode()) % 10000))
    x = make_x(layer, batch)
    print(f"case {name}: d_in={d_in} d_out={d_out} bits={bits} k={k} batch={batch}", flush=True)
    check(run_gpu(env, layer, x), owq_ref.owq_linear_layer(layer, x), name)


@pytest.mark.parametrize("where", ["first", "last", "run", "every_8th"])
def test_weak_columns_in_special_places(env, where):
    d_in, d_out = 1024, 64
    idx = {"first": np.arange(0, 24), "last": np.arange(d_in - 24, d_in), "run": np.arange(500, 540),
           "every_8th": np.arange(0, d_in, 8)}[where].astype(np.int32)
    rng = np.random.default_rng(11)
    layer = make_layer(LayerSpec("place", d_in, d_out, 3, 0, 0, 3))
    layer.spec = LayerSpec("place", d_in, d_out, 3, 0, int(idx.size), 3)
    layer.weak_idx = idx
    layer.weak_w = rng.normal(0, 0.02, size=(d_out, idx.size)).astype(np.float16)
    layer.codes[:, idx] = 0
    x = make_x(layer, 2)
    check(run_gpu(env, layer, x), owq_ref.owq_linear_layer(layer, x), where)


def test_all_columns_weak_reproduces_fp16_matmul(env):
    rng = np.random.default_rng(3)
    d_out, d_in = 48, 384
    w16 = rng.normal(0, 0.02, size=(d_out, d_in)).astype(np.float16)
    layer = make_layer(LayerSpec("allweak", d_in, d_out, 3, 0, 0, 5))
    layer.spec = LayerSpec("allweak", d_in, d_out, 3, 0, d_in, 5)
    layer.weak_idx = np.arange(d_in, dtype=np.int32)
    layer.weak_w = w16
    x = rng.normal(0, 1, size=(3, d_in)).astype(np.float16)
    check(run_gpu(env, layer, x), x.astype(np.float64) @ w16.astype(np.float64).T, "allweak")


@pytest.mark.parametrize("bits", [3, 4])
def test_one_hot_probing_is_bit_exact(env, bits):
    # x = e_j for every j reads the whole effective matrix back: fp16(s*(q-z)) at the stored columns,
    # Ww at the weak ones; checks the move of every activation to its stored column.
    d_in, d_out, k = 640, 70, 37
    layer = make_layer(LayerSpec("onehot", d_in, d_out, bits, 0, k, 17 + bits))
    eye = np.eye(d_in, dtype=np.float16)
    y = run_gpu(env, layer, eye)
    want = owq_ref.to_fp16(owq_ref.owq_linear_layer(layer, eye))
    np.testing.assert_array_equal(y.view(np.uint16), want.view(np.uint16))


def test_integer_inputs_are_bit_exact(env):
    rng = np.random.default_rng(300)
    d_in, d_out, k = 2048, 64, 50
    layer = make_layer(LayerSpec("exact", d_in, d_out, 3, 0, k, 5))
    layer.scale = (2.0 ** -rng.integers(3, 7, size=layer.scale.shape)).astype(np.float16)
    layer.weak_w = (rng.integers(-8, 9, size=layer.weak_w.shape) / 16.0).astype(np.float16)
    x = rng.integers(-1, 2, size=(4, d_in)).astype(np.float16)
    y = run_gpu(env, layer, x)
    want = owq_ref.to_fp16(owq_ref.owq_linear_layer(layer, x))
    np.testing.assert_array_equal(y.view(np.uint16), want.view(np.uint16))


def test_uploaded_blob_equals_oracle_pack_and_is_smaller(env):
    torch, B = env
    layer = make_layer(LayerSpec("blob", 2048 + 256, 77, 3, 0, 300, 8))
    lin = B.OwqLinear(layer, layout=COMPACT)
    blob = B.owq_export_packed(lin.handle)
    want, geo = packfmt.pack_layer(layer.codes, layer.scale, layer.zero, 0, layer.weak_idx, layer.weak_w, 3, layout=2)
    np.testing.assert_array_equal(blob, want)
    plain = packfmt.geometry(77, 2048 + 256, 3, 0, 300, 0)
    assert geo.off_sz < plain.off_sz                       # two blocks of columns fewer
    lin.close()


def test_weak_positions_do_not_reach_the_dense_term(env):
    layer = make_layer(LayerSpec("leak", 1024, 64, 3, 0, 8, 21))
    layer.weak_w[:] = 0
    x = make_x(layer, 2)
    ref = owq_ref.owq_linear_layer(layer, np.where(np.isin(np.arange(1024), layer.weak_idx), 0, x).astype(np.float16))
    x[:, layer.weak_idx] = np.float16(6e4)
    y = run_gpu(env, layer, x)
    assert np.isfinite(y).all()
    check(y, ref, "leak")


def test_unaligned_x(env):
    torch, B = env
    layer = make_layer(LayerSpec("unal", 1024, 64, 3, 0, 8, 4))
    x = make_x(layer, 2)
    lin = B.OwqLinear(layer, layout=COMPACT)
    buf = torch.zeros(2 * 1024 + 8, dtype=torch.float16, device="cuda")
    xv = buf[1:1 + 2 * 1024].view(2, 1024)                 # 2-byte aligned only
    xv.copy_(torch.from_numpy(x))
    y = torch.empty((2, 64), dtype=torch.float16, device="cuda")
    B.owq_linear(lin.handle, xv.data_ptr(), y.data_ptr(), 2, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    lin.close()
    check(y.cpu().numpy(), owq_ref.owq_linear_layer(layer, x), "unaligned")


def test_several_tasks_share_the_dense_matrix(env):
    torch, B = env
    layer = make_layer(LayerSpec("multi", 1024, 96, 3, 0, 16, 6))
    rng = np.random.default_rng(9)
    sets = [rng.normal(0, 0.02, size=layer.weak_w.shape).astype(np.float16) for _ in range(3)]
    task = np.array([0, 2, -1, 1, 2], dtype=np.int32)
    x = make_x(layer, task.size)
    lin = B.OwqLinear(layer, layout=COMPACT)
    table, keep = lin.add_weak_sets(sets)
    y = lin.multi(torch.from_numpy(x).cuda(), table, torch.from_numpy(task).cuda())
    torch.cuda.synchronize()
    ref_task = [t if 0 <= t < 3 else 3 for t in task]         # -1: the layer's own columns
    want = owq_ref.owq_linear_multi_ref(layer.codes, layer.scale, layer.zero, 0, layer.weak_idx,
                                        sets + [layer.weak_w], ref_task, x)
    check(y.cpu().numpy(), want, "multi")
    lin.close()


@pytest.mark.parametrize("cfg,li", [(1, 0), (4, 1)])
def test_full_size_layers_sampled_rows(env, cfg, li):
    spec = CONFIGS[cfg][li]
    print(f"full-size {spec.name}, storage-favoured layout", flush=True)
    layer = make_layer(spec)
    x = make_x(layer, 1)
    y = run_gpu(env, layer, x)
    rng = np.random.default_rng(li)
    rows = np.unique(np.concatenate([rng.integers(0, spec.d_out, size=600), [0, spec.d_out - 1]]))
    want = owq_ref.owq_linear_ref(layer.codes[rows], layer.scale[rows], layer.zero[rows], layer.group_size,
                                  layer.weak_idx, layer.weak_w[rows], x)
    check(y[:, rows], want, spec.name)
