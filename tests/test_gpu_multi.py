"""GPU parity of weak-column tuning support: several tasks sharing one dense matrix
(owq_linear_multi) and in-place replacement of the weak columns (owq_update_weak),
against the fp64 CPU oracle.  Same tolerances as the other parity tests."""
import numpy as np
import pytest

from oracle import owq_ref
from synth import LayerSpec, make_layer, make_x

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


def check(y_gpu, y_ref, what=""):
    for n in range(y_ref.shape[0]):
        rel, mx = owq_ref.parity_errors(y_gpu[n], y_ref[n])
        assert rel <= REL_L2 and mx <= MAX_ABS, (what, n, rel, mx)


def make_sets(layer, n_sets, seed):
    rng = np.random.default_rng(seed)
    return [rng.normal(0, 0.02, size=(layer.d_out, layer.k)).astype(np.float16) for _ in range(n_sets)]


CASES = [
    # name, layout, d_in, d_out, bits, group, k, batch, n_sets
    ("gemv3", 0, 1024, 96, 3, 0, 8, 5, 3),
    ("gemv4_g", 0, 2048, 130, 4, 128, 16, 9, 4),
    ("gemv_many_weak", 0, 256, 40, 3, 0, 100, 4, 2),       # weak chunks beyond one per block
    ("tile3", 1, 1024, 96, 3, 0, 8, 64, 3),
    ("tile4_g", 1, 2048, 300, 4, 128, 24, 40, 5),
    ("tile3_two_passes", 1, 512, 70, 3, 0, 16, 100, 4),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_tokens_of_different_tasks_share_the_dense_matrix(env, case):
    torch, B = env
    name, layout, d_in, d_out, bits, group, k, batch, n_sets = case
    print(f"case {name}", flush=True)
    layer = make_layer(LayerSpec(name, d_in, d_out, bits, group, k, 77))
    sets = make_sets(layer, n_sets, 5)
    rng = np.random.default_rng(9)
    task = rng.integers(-1, n_sets + 1, size=batch).astype(np.int32)      # -1 and n_sets: the layer's own columns
    x = make_x(layer, batch)
    lin = B.OwqLinear(layer, layout=layout)
    table, bufs = lin.add_weak_sets(sets)
    y = lin.multi(torch.from_numpy(x).cuda(), table, torch.from_numpy(task).cuda())
    torch.cuda.synchronize()
    all_sets = sets + [layer.weak_w]
    ref_task = [t if 0 <= t < n_sets else n_sets for t in task]
    want = owq_ref.owq_linear_multi_ref(layer.codes, layer.scale, layer.zero, layer.group_size, layer.weak_idx,
                                        all_sets, ref_task, x)
    check(y.cpu().numpy(), want, name)
    # the plain call still uses the layer's own columns
    y0 = lin(torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    check(y0.cpu().numpy(), owq_ref.owq_linear_layer(layer, x), name + " plain")
    lin.close()


@pytest.mark.parametrize("layout", [0, 1])
def test_large_table_sparsely_used(env, layout):
    # A serving table of 4096 tasks of which a batch uses five: only the entries some token selects are read
    # (the others are null pointers here), and the cost must not grow with the table.
    torch, B = env
    layer = make_layer(LayerSpec("table", 1024, 200, 3, 128, 16, 91))
    used = [3, 777, 778, 2048, 4095]
    sets = make_sets(layer, len(used), 6)
    lin = B.OwqLinear(layer, layout=layout)
    small, bufs = lin.add_weak_sets(sets)
    table = torch.zeros(4096, dtype=torch.int64, device="cuda")
    table[torch.tensor(used, device="cuda")] = small
    batch = 50
    rng = np.random.default_rng(10)
    pick = rng.integers(0, len(used) + 1, size=batch)                        # len(used): the layer's own columns
    task = np.array([used[p] if p < len(used) else -1 for p in pick], dtype=np.int32)
    x = make_x(layer, batch)
    y = lin.multi(torch.from_numpy(x).cuda(), table, torch.from_numpy(task).cuda())
    torch.cuda.synchronize()
    want = owq_ref.owq_linear_multi_ref(layer.codes, layer.scale, layer.zero, layer.group_size, layer.weak_idx,
                                        sets + [layer.weak_w], [int(p) for p in pick], x)
    check(y.cpu().numpy(), want, "table")
    lin.close()


@pytest.mark.parametrize("layout", [0, 1])
def test_one_task_for_all_tokens_equals_the_plain_call_bit_for_bit(env, layout):
    torch, B = env
    layer = make_layer(LayerSpec("same", 1024, 128, 3, 0, 16, 78))
    x = torch.from_numpy(make_x(layer, 48)).cuda()
    lin = B.OwqLinear(layer, layout=layout)
    table, bufs = lin.add_weak_sets([layer.weak_w])                       # a copy of the layer's own columns
    task = torch.zeros(48, dtype=torch.int32, device="cuda")
    a = lin.multi(x, table, task).cpu().numpy()
    b = lin(x).cpu().numpy()
    np.testing.assert_array_equal(a.view(np.uint16), b.view(np.uint16))
    lin.close()


@pytest.mark.parametrize("layout", [0, 1])
def test_update_weak_equals_packing_the_new_columns(env, layout):
    torch, B = env
    layer = make_layer(LayerSpec("upd", 1024, 100, 4, 0, 12, 79))
    new_w = make_sets(layer, 1, 11)[0]
    x = make_x(layer, 33)
    xd = torch.from_numpy(x).cuda()
    lin = B.OwqLinear(layer, layout=layout)
    B.owq_update_weak(lin.handle, new_w, torch.cuda.current_stream().cuda_stream)
    y = lin(xd).cpu().numpy()
    layer2 = make_layer(LayerSpec("upd", 1024, 100, 4, 0, 12, 79))
    layer2.weak_w = new_w
    fresh = B.OwqLinear(layer2, layout=layout)
    y2 = fresh(xd).cpu().numpy()
    np.testing.assert_array_equal(y.view(np.uint16), y2.view(np.uint16))
    check(y, owq_ref.owq_linear_layer(layer2, x), "update")
    # only the weak-column section of the blob changed
    a, b = B.owq_export_packed(lin.handle), B.owq_export_packed(fresh.handle)
    info = lin.info()
    end = info.off_scratch if layout == 1 else info.total_bytes
    np.testing.assert_array_equal(a[:end], b[:end])
    lin.close()
    fresh.close()


def test_multi_argument_checks(env):
    torch, B = env
    layer = make_layer(LayerSpec("args", 512, 32, 4, 0, 4, 80))
    lin = B.OwqLinear(layer)
    table, bufs = lin.add_weak_sets(make_sets(layer, 2, 3))
    x = torch.from_numpy(make_x(layer, 2)).cuda()
    y = torch.empty((2, 32), dtype=torch.float16, device="cuda")
    task = torch.zeros(2, dtype=torch.int32, device="cuda")
    with pytest.raises(B.OwqError) as e:
        B.owq_linear_multi(lin.handle, table.data_ptr(), 0, task.data_ptr(), x.data_ptr(), y.data_ptr(), 2)
    assert e.value.status == B.OWQ_ERR_INDEX
    with pytest.raises(B.OwqError) as e:
        B.owq_linear_multi(lin.handle, 0, 2, task.data_ptr(), x.data_ptr(), y.data_ptr(), 2)
    assert e.value.status == B.OWQ_ERR_NULL
    with pytest.raises(B.OwqError) as e:
        B.owq_pack_weak_set(lin.handle, layer.weak_w, bufs[0].data_ptr(), 8)
    assert e.value.status == B.OWQ_ERR_BUFFER
    lin.close()
