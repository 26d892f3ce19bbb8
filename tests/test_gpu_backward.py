"""GPU parity of owq_linear_backward (derivatives of the layer for weak-column tuning; paper, section
"PEFT with Weak Column Tuning") against the fp64 CPU oracle, through the C ABI.

Tolerances.  dx: the forward path's bar (relative L2 <= 1e-3, max abs <= 1e-2 rms, whole batch and token
by token): dy times the step size is rounded to fp16 once (2^-11 relative per term, independent signs),
the sum is fp32 and dx is rounded to fp16 once.  dww is an fp32 sum of exact fp16 products over the
batch: relative L2 <= 1e-5.
"""
import numpy as np
import pytest

from oracle import backward, owq_ref
from synth import CONFIGS, LayerSpec, make_layer, make_x

pytestmark = pytest.mark.gpu
TILE = 1
REL_L2, MAX_ABS, DWW_REL = 1e-3, 1e-2, 1e-5


@pytest.fixture(scope="module")
def env():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2306_02272_amd import binding
    binding.lib()
    torch.cuda.set_device(0)
    return torch, binding


def make_dy(layer, batch, seed=0):
    rng = np.random.default_rng([layer.spec.seed, 9, batch, seed])
    return rng.normal(0, 0.05, size=(batch, layer.d_out)).astype(np.float16)


def run_gpu(env, layer, x, dy, want_dx=True, want_dww=True):
    torch, B = env
    lin = B.OwqLinear(layer, layout=TILE)
    dx, dww = lin.backward(torch.from_numpy(dy).cuda(), torch.from_numpy(x).cuda(), want_dx, want_dww)
    torch.cuda.synchronize()
    out = (None if dx is None else dx.cpu().numpy(), None if dww is None else dww.cpu().numpy())
    lin.close()
    return out


def check_dx(dx, ref, what=""):
    assert dx.shape == ref.shape and np.isfinite(dx).all()
    rel, mx = owq_ref.parity_errors(dx, ref)
    assert rel <= REL_L2 and mx <= MAX_ABS, (what, rel, mx)
    for n in range(ref.shape[0]):
        rel, mx = owq_ref.parity_errors(dx[n], ref[n])
        assert rel <= REL_L2 and mx <= MAX_ABS, (what, n, rel, mx)


def check_dww(dww, ref, what=""):
    assert dww.shape == ref.shape
    if ref.size:
        rel, _ = owq_ref.parity_errors(dww, ref)
        assert rel <= DWW_REL, (what, rel)


CASES = [
    # name, d_in, d_out, bits, group, k, batch
    ("b3_row", 512, 96, 3, 0, 8, 5),
    ("b4_row", 512, 96, 4, 0, 8, 33),
    ("b3_g128", 1024, 160, 3, 128, 10, 17),
    ("b4_g128", 768, 64, 4, 128, 6, 128),          # d_in not a multiple of 256: a padded block
    ("b4_g256", 1024, 128, 4, 256, 16, 64),
    ("ragged_rows", 512, 70, 3, 128, 5, 9),         # d_out not a multiple of 32
    ("ragged_cols", 1000, 64, 4, 0, 7, 12),         # d_in not a multiple of 128
    ("no_weak", 512, 64, 3, 128, 0, 4),
    ("one_token", 1024, 256, 3, 128, 9, 1),
    ("two_passes", 512, 64, 4, 128, 8, 130),        # 128 + 2 tokens
    ("three_passes", 256, 96, 3, 0, 3, 300),
    ("more_weak_tiles_than_block_pairs", 256, 96, 4, 0, 40, 11),   # the plain kernel for the weak columns of dx
    ("three_weak_tiles", 1024, 128, 3, 128, 70, 35),
    ("six_weak_tiles", 2048, 64, 4, 128, 170, 20),       # dww in two groups of tiles
    ("two_groups_of_passes", 256, 64, 4, 128, 5, 600),   # more than the 512 tokens one set of launches takes
    ("many_rows", 256, 2048, 3, 128, 4, 40),        # several ranges of rows per block pair
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_backward_matches_oracle(env, case):
    name, d_in, d_out, bits, gs, k, batch = case
    L = make_layer(LayerSpec(name, d_in, d_out, bits, gs, k, 500 + len(name)))
    x, dy = make_x(L, batch), make_dy(L, batch)
    dx, dww = run_gpu(env, L, x, dy)
    rdx, rdww = backward.owq_backward_ref(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, L.weak_w, x, dy)
    check_dx(dx, rdx, name)
    check_dww(dww, rdww, name)
    # the weak columns on their own: they come from another kernel and would drown in the whole-row error
    if k:
        rel, _ = owq_ref.parity_errors(dx[:, L.weak_idx], rdx[:, L.weak_idx])
        assert rel <= REL_L2, (name, rel)


@pytest.mark.parametrize("sigma", [1.0, 1e-3, 1e-5])
def test_gradient_magnitude_does_not_matter(env, sigma):
    # Gradients of weak-column tuning are small: with dy ~ 1e-3 and step sizes of 1e-3..1e-2 the fp16 product
    # dy * s would be a subnormal number.  The library scales dy by a power of two first; the error against the
    # oracle must stay at the forward path's bar on top of what rounding the exact result to fp16 costs (at
    # sigma = 1e-5 dx itself is a subnormal fp16 number).
    L = make_layer(LayerSpec("small_dy", 512, 2048, 3, 128, 8, 612))
    batch = 24
    x = make_x(L, batch)
    rng = np.random.default_rng(17)
    dy = rng.normal(0, sigma, size=(batch, L.d_out)).astype(np.float16)
    dx, dww = run_gpu(env, L, x, dy)
    rdx, rdww = backward.owq_backward_ref(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, L.weak_w, x, dy)
    for n in range(batch):
        den = np.linalg.norm(rdx[n])
        rel_gpu = np.linalg.norm(dx[n].astype(np.float64) - rdx[n]) / den
        rel_ideal = np.linalg.norm(owq_ref.to_fp16(rdx[n]).astype(np.float64) - rdx[n]) / den
        assert rel_gpu <= 1.05 * rel_ideal + REL_L2, (sigma, n, rel_gpu, rel_ideal)
    check_dww(dww, rdww, f"sigma {sigma}")


def test_integer_case_is_exact(env):
    # Step size 1, zero point 0, dy in {-1, 0, 1}: every product and sum is a small integer, so dx must be
    # exact, whatever the order of the additions.
    L = make_layer(LayerSpec("int", 512, 64, 4, 128, 4, 77))
    L.scale[:] = 1.0
    L.zero[:] = 0.0
    L.weak_w[:] = np.round(L.weak_w.astype(np.float32) * 100).astype(np.float16)
    rng = np.random.default_rng(3)
    dy = rng.integers(-1, 2, size=(7, 64)).astype(np.float16)
    x = rng.integers(-2, 3, size=(7, 512)).astype(np.float16)
    dx, dww = run_gpu(env, L, x, dy)
    rdx, rdww = backward.owq_backward_ref(L.codes, L.scale, L.zero, 128, L.weak_idx, L.weak_w, x, dy)
    assert np.array_equal(dx.astype(np.float64), rdx)
    assert np.array_equal(dww.astype(np.float64), rdww)


def test_one_hot_dy_reads_single_rows(env):
    # dy = e_i for token n: dx[n] is row i of the dequantised matrix, rounded to fp16 once; catches any
    # mix-up of rows between the turned codes and the staged dy.
    L = make_layer(LayerSpec("hot", 512, 96, 3, 128, 6, 78))
    rows = [0, 1, 31, 32, 45, 63, 64, 95]
    dy = np.zeros((len(rows), 96), np.float16)
    for n, i in enumerate(rows):
        dy[n, i] = 1.0
    x = make_x(L, len(rows))
    dx, _ = run_gpu(env, L, x, dy, want_dww=False)
    rdx, _ = backward.owq_backward_ref(L.codes, L.scale, L.zero, 128, L.weak_idx, L.weak_w, x, dy)
    assert np.array_equal(dx, owq_ref.to_fp16(rdx))


def test_adjoint_of_the_gpu_forward(env):
    # <dy, F(x)> = <dx, x> with both sides from the library (fp16 outputs: a loose bar)
    torch, B = env
    L = make_layer(LayerSpec("adj", 1024, 256, 4, 128, 10, 79))
    x, dy = make_x(L, 16), make_dy(L, 16)
    lin = B.OwqLinear(L, layout=TILE)
    xd, dyd = torch.from_numpy(x).cuda(), torch.from_numpy(dy).cuda()
    y = lin(xd).cpu().numpy().astype(np.float64)
    dx, _ = lin.backward(dyd, xd, want_dww=False)
    dx = dx.cpu().numpy().astype(np.float64)
    lin.close()
    lhs, rhs = np.sum(dy.astype(np.float64) * y), np.sum(dx * x.astype(np.float64))
    assert lhs == pytest.approx(rhs, rel=5e-3)


def test_only_one_output_wanted(env):
    L = make_layer(LayerSpec("half", 512, 64, 3, 0, 8, 80))
    x, dy = make_x(L, 6), make_dy(L, 6)
    rdx, rdww = backward.owq_backward_ref(L.codes, L.scale, L.zero, 0, L.weak_idx, L.weak_w, x, dy)
    dx, dww = run_gpu(env, L, x, dy, want_dww=False)
    assert dww is None
    check_dx(dx, rdx)
    dx, dww = run_gpu(env, L, x, dy, want_dx=False)
    assert dx is None
    check_dww(dww, rdww)


def test_dww_of_a_layer_without_weak_columns(env):
    # k = 0 and only dww wanted: nothing to compute, nothing launched, no error
    torch, B = env
    L = make_layer(LayerSpec("k0", 512, 64, 3, 128, 0, 82))
    x, dy = make_x(L, 3), make_dy(L, 3)
    dx, dww = run_gpu(env, L, x, dy, want_dx=False)
    assert dx is None and dww.shape == (64, 0)


def test_errors(env):
    torch, B = env
    L = make_layer(LayerSpec("err", 512, 64, 3, 0, 8, 81))
    dy = torch.zeros((4, 64), dtype=torch.float16, device="cuda")
    x = torch.zeros((4, 512), dtype=torch.float16, device="cuda")
    dx = torch.zeros((4, 512), dtype=torch.float16, device="cuda")
    gemv = B.OwqLinear(L, layout=0)
    with pytest.raises(B.OwqError) as e:
        B.owq_backward_workspace_bytes(gemv.handle, 4)
    assert e.value.status == B.OWQ_ERR_LAYOUT
    with pytest.raises(B.OwqError) as e:
        B.owq_linear_backward(gemv.handle, dy.data_ptr(), x.data_ptr(), dx.data_ptr(), 0, 4, dx.data_ptr(), 1 << 20)
    assert e.value.status == B.OWQ_ERR_LAYOUT
    gemv.close()
    lin = B.OwqLinear(L, layout=TILE)
    need = B.owq_backward_workspace_bytes(lin.handle, 4)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")

    def status(*a):
        try:
            B.owq_linear_backward(lin.handle, *a)
        except B.OwqError as err:
            return err.status
        return B.OWQ_OK
    assert status(dy.data_ptr(), x.data_ptr(), dx.data_ptr(), 0, 4, ws.data_ptr(), need - 1) == B.OWQ_ERR_BUFFER
    assert status(dy.data_ptr() + 2, x.data_ptr(), dx.data_ptr(), 0, 4, ws.data_ptr(), need) == B.OWQ_ERR_BUFFER
    assert status(0, x.data_ptr(), dx.data_ptr(), 0, 4, ws.data_ptr(), need) == B.OWQ_ERR_NULL
    assert status(dy.data_ptr(), x.data_ptr(), dx.data_ptr(), 0, 4, 0, 0) == B.OWQ_ERR_NULL
    assert status(dy.data_ptr(), x.data_ptr(), dx.data_ptr(), 0, -1, ws.data_ptr(), need) == B.OWQ_ERR_BATCH
    assert status(dy.data_ptr(), x.data_ptr(), dx.data_ptr(), 0, 0, ws.data_ptr(), need) == B.OWQ_OK
    lin.close()
    with pytest.raises(B.OwqError) as e:
        B.owq_backward_workspace_bytes(0, 4)
    assert e.value.status == B.OWQ_ERR_HANDLE


def test_full_size_512_tokens_whole_output(env):
    # configs[2]'s fc1 (4096 -> 16384) at the 512 tokens the benchmark times, the whole of dx and dww
    torch, B = env
    L = make_layer(CONFIGS[2][0])
    batch = 512
    x, dy = make_x(L, batch), make_dy(L, batch)
    dx, dww = run_gpu(env, L, x, dy)
    rdx, rdww = backward.owq_backward_ref(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, L.weak_w, x, dy)
    check_dx(dx, rdx, "fc1 512 tokens")
    check_dww(dww, rdww, "fc1 512 tokens")


def test_full_size_sampled(env):
    # configs[2]'s fc2 (16384 -> 4096, 3-bit, groups of 128, k = 128), 128 tokens, the shape the bench times:
    # sampled tokens and sampled rows of dww against the oracle.
    torch, B = env
    L = make_layer(CONFIGS[2][1])
    batch = 128
    x, dy = make_x(L, batch), make_dy(L, batch)
    dx, dww = run_gpu(env, L, x, dy)
    toks = [0, 31, 77, 127]
    rdx, _ = backward.owq_backward_ref(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, L.weak_w, x[toks], dy[toks])
    check_dx(dx[toks], rdx, "fc2")
    rows = [0, 1000, 4095]
    rdww = dy.astype(np.float64).T[rows] @ x.astype(np.float64)[:, L.weak_idx]
    check_dww(dww[rows], rdww, "fc2")
