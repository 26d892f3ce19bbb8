"""Developer check on the compiled kernels: which of them touch scratch memory.

    python -m paper_2306_02272_amd.check_isa [file.hip ...]

Compiles every HIP source of the library to gfx950 assembly (device side only, the flags of build.py) and
prints, per kernel, the scratch bytes, the spilled registers and the number of scratch instructions.  A kernel
that is not out of registers should show none: scratch loads count in `vmcnt`, so a loop that reads a counter
from scratch waits for every global load in flight each time round.  (hipcc puts loop counters there when an
`if` increments one of two variables: it turns that into one increment through a selected address.)
Exit status 1 if a kernel outside ALLOWED touches scratch."""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile

from . import build

HERE = os.path.dirname(os.path.abspath(__file__))
# kernels that are known to run out of registers (name fragments): none is a default launch
ALLOWED = ()


def kernels_of(asm: str):
    cur, counts = None, {}
    for line in asm.splitlines():
        m = re.match(r"^(_Z\w+):", line)
        if m:
            cur = m.group(1)
            counts[cur] = 0
        elif cur and re.search(r"\bscratch_(load|store)", line):
            counts[cur] += 1
    meta = {}
    for m in re.finditer(r"\.name:\s+(\S+)\n(?:.*\n)*?\s+\.private_segment_fixed_size:\s+(\d+)\n(?:.*\n)*?\s+\.vgpr_count:\s+(\d+)\n"
                         r"\s+\.vgpr_spill_count:\s+(\d+)", asm):
        meta[m.group(1)] = (int(m.group(2)), int(m.group(3)), int(m.group(4)))
    return counts, meta


def main(argv) -> int:
    sources = argv or [s for s in build.SOURCES if s.endswith(".hip")]
    bad = 0
    with tempfile.TemporaryDirectory() as tmp:
        for src in sources:
            path = src if os.path.isabs(src) or os.path.exists(src) else os.path.join(HERE, "csrc", src)
            out = os.path.join(tmp, os.path.basename(src) + ".s")
            cmd = [build.hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-I" + os.path.join(build.ROOT, "include"),
                   "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
                   "-S", "--cuda-device-only", "-o", out, path]
            res = subprocess.run(cmd, capture_output=True, text=True)
            if res.returncode != 0:
                sys.stderr.write(res.stderr)
                return 2
            counts, meta = kernels_of(open(out).read())
            touched = {k: v for k, v in counts.items() if v}
            print(f"{os.path.basename(src)}: {len(meta)} kernels, {len(touched)} with scratch instructions", flush=True)
            for name, n in touched.items():
                scratch, vgprs, spills = meta.get(name, (0, 0, 0))
                ok = any(a in name for a in ALLOWED)
                bad += 0 if ok else 1
                print(f"  {name}: {n} scratch instructions, {scratch} bytes, {vgprs} registers, {spills} spilled"
                      + ("" if ok else "   <-- not expected"))
    return 1 if bad else 0


if __name__ == "__main__":
    raise SystemExit(main(sys.argv[1:]))
