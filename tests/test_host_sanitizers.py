"""The library's host code (geometry, validation, packer, unpacker: csrc/owq_pack.cpp) built with
g++ -fsanitize=address,undefined and driven through the pack / unpack / reject matrix of
tests/test_library_cpu.py by a small C++ harness (tests/host_sanitize.cpp).  CPU only.

The expected blobs come from the CPU oracle's format code (oracle/packfmt.py), the expected status
codes from include/owq.h; every buffer the harness passes has exactly the stated size, so a read or a
write past it ends the run."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import packfmt
from synth import LayerSpec, make_layer

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, NULL, SHAPE, BITS, GROUP, CODE, INDEX, BUFFER = 0, 1, 2, 3, 4, 5, 6, 7
LAYOUT = 12

PACK = [  # (spec, layout): the layers of tests/test_library_cpu.py and a few more shapes
    (LayerSpec("a", 512, 21, 3, 0, 5, 1), 0), (LayerSpec("b", 1000, 33, 4, 128, 9, 2), 0),
    (LayerSpec("c", 128 * 40, 10, 3, 256, 0, 3), 0), (LayerSpec("d", 128 * 108, 7, 4, 128, 138, 4), 0),
    (LayerSpec("e", 1, 1, 3, 0, 1, 5), 0), (LayerSpec("f", 4096, 64, 3, 128, 32, 6), 0),
    (LayerSpec("ta", 700, 45, 3, 256, 11, 21), 1), (LayerSpec("tb", 256, 32, 4, 0, 0, 22), 1),
    (LayerSpec("tc", 1000, 70, 4, 128, 9, 23), 1), (LayerSpec("td", 130, 3, 3, 0, 130, 24), 1),
    (LayerSpec("ca", 700, 45, 3, 0, 11, 21), 2), (LayerSpec("cb", 256, 32, 4, 0, 0, 22), 2),
    (LayerSpec("cc", 1003, 70, 4, 0, 107, 23), 2), (LayerSpec("cd", 130, 3, 3, 0, 130, 24), 2),
    (LayerSpec("ce", 128 * 6 + 8, 9, 3, 0, 8, 25), 2), (LayerSpec("one", 1, 1, 4, 0, 0, 26), 1),
]


def write_case(d, man, name, L, layout, want, null_mask=0, **over):
    f = dict(d_out=L.d_out, d_in=L.d_in, bits=L.bits, group_size=L.group_size, k=L.k, codes=L.codes, scale=L.scale,
             zero=L.zero, weak_idx=L.weak_idx, weak_w=L.weak_w)
    f.update(over)
    np.asarray(f["codes"], dtype=np.uint8).tofile(os.path.join(d, name + ".codes"))
    np.asarray(f["scale"], dtype=np.float16).tofile(os.path.join(d, name + ".scale"))
    np.asarray(f["zero"], dtype=np.float16).tofile(os.path.join(d, name + ".zero"))
    np.asarray(f["weak_idx"], dtype=np.int32).tofile(os.path.join(d, name + ".idx"))
    np.asarray(f["weak_w"], dtype=np.float16).tofile(os.path.join(d, name + ".ww"))
    blob = np.zeros(0, dtype=np.uint8)
    if want == OK:
        blob, _ = packfmt.pack_layer(L.codes, L.scale, L.zero, L.group_size, L.weak_idx, L.weak_w, L.bits, layout=layout)
    blob.tofile(os.path.join(d, name + ".blob"))
    L.codes.tofile(os.path.join(d, name + ".canon"))            # the generator already stores 0 at weak columns
    man.append(f"{name} {f['d_out']} {f['d_in']} {f['bits']} {f['group_size']} {f['k']} {layout} {null_mask} {want}")


@pytest.fixture(scope="module")
def harness(tmp_path_factory):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    out = tmp_path_factory.mktemp("san")
    exe = str(out / "host_sanitize")
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-I" + os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "host_sanitize.cpp"),
           os.path.join(ROOT, "paper_2306_02272_amd", "csrc", "owq_pack.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    return exe, out


def test_pack_unpack_reject_matrix_under_sanitizers(harness):
    exe, out = harness
    d = str(out)
    man = []
    for spec, layout in PACK:
        L = make_layer(spec)
        dirty = L.codes.copy()
        dirty[:, L.weak_idx] = 255                   # ignored at weak columns, stored as 0
        write_case(d, man, f"pack_{spec.name}_{layout}", L, layout, OK, codes=dirty)
    L = make_layer(LayerSpec("t", 256, 8, 3, 0, 4, 9))
    free_col = [j for j in range(L.d_in) if j not in set(L.weak_idx.tolist())][0]
    bad = L.codes.copy()
    bad[3, free_col] = 8
    rejects = [("bits5", dict(bits=5), BITS, 0), ("bits2", dict(bits=2), BITS, 0), ("rows0", dict(d_out=0), SHAPE, 0),
               ("colsneg", dict(d_in=-4), SHAPE, 0), ("group64", dict(group_size=64), GROUP, 0),
               ("groupneg", dict(group_size=-128), GROUP, 0), ("kbig", dict(k=L.d_in + 1), INDEX, 0),
               ("kneg", dict(k=-1), INDEX, 0), ("nocodes", {}, NULL, 1), ("noscale", {}, NULL, 2), ("nozero", {}, NULL, 4),
               ("noidx", {}, NULL, 8), ("noww", {}, NULL, 16), ("code8", dict(codes=bad), CODE, 0)]
    for i, idx in enumerate(([5, 5, 6, 7], [9, 3, 20, 21], [0, 1, 2, 256], [-1, 1, 2, 3])):
        rejects.append((f"idx{i}", dict(weak_idx=np.array(idx, dtype=np.int32)), INDEX, 0))
    for name, over, want, mask in rejects:
        for layout in (0, 1, 2):
            write_case(d, man, f"rej_{name}_{layout}", L, layout, want, mask, **over)
    write_case(d, man, "rej_layout", L, 7, LAYOUT)
    Lg = make_layer(LayerSpec("cg", 512, 8, 3, 128, 4, 9))
    write_case(d, man, "rej_compact_group", Lg, 2, GROUP)
    open(os.path.join(d, "manifest.txt"), "w").write("\n".join(man) + "\n")
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)
    res = subprocess.run([exe, d], capture_output=True, text=True, env=env, timeout=600)
    assert res.returncode == 0, (res.stdout[-2000:], res.stderr[-4000:])
    assert res.stdout.strip() == f"ok {len(man)} cases", res.stdout
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-4000:]
