"""The vector path's write-through stores are issued by an asm statement the compiler does not
know to be a store, so nothing may overwrite its data registers between such a store and the end
of the kernel (see st16_through in th_kernels.hip).  This compiles the kernels to assembly and checks
exactly that, for every kernel that contains such a store."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2604_09107_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC) and shutil.which("hipcc") is None, reason="needs hipcc")
def test_write_through_stores_end_their_kernels(tmp_path):
    asm = str(tmp_path / "k.s")
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                    "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-S", "--cuda-device-only",
                    "-x", "hip", os.path.join(CSRC, "th_kernels.hip"), "-o", asm],
                   check=True, stderr=subprocess.DEVNULL)
    text = open(asm).read()
    kernels = re.split(r"^(\S+):\s*; @\S+\n", text, flags=re.M)
    through = re.compile(r"^\s*global_store_dwordx[24] (v\[\d+:\d+\]), (v\[\d+:\d+\]), off sc1 nt")

    def regs(op):
        m = re.match(r"v\[(\d+):(\d+)\]$", op)
        if m:
            return set(range(int(m.group(1)), int(m.group(2)) + 1))
        m = re.match(r"v(\d+)$", op)
        return {int(m.group(1))} if m else set()

    checked = 0
    for name, body in zip(kernels[1::2], kernels[2::2]):
        lines = [l for l in body.split(".Lfunc_end")[0].splitlines() if l.strip() and not l.strip().startswith(";")]
        firsts = [i for i, l in enumerate(lines) if through.match(l)]
        if not firsts:
            continue
        checked += 1
        # From the first write-through store to the s_endpgm that follows it, nothing writes a register
        # that holds the data of a write-through store issued before it (address registers are read at
        # issue and may be reused), and nothing else touches memory.
        tail = lines[firsts[0]:]
        end = next(i for i, l in enumerate(tail) if l.strip().startswith("s_endpgm"))
        stored = set()
        for l in tail[:end]:
            s = l.strip()
            m = through.match(l)
            if m:
                stored |= regs(m.group(2))
                continue
            if s.startswith("s_") or s.endswith(":") or s.startswith("."):
                continue
            assert s.startswith("v_"), "%s: '%s' follows a write-through store" % (name, s)
            dest = s.split(None, 1)[1].split(",")[0].strip()
            assert not (regs(dest) & stored), "%s: '%s' overwrites stored data" % (name, s)
        # ... and no write-through store anywhere else in the kernel
        assert all(i < firsts[0] + end for i in firsts), name
    # pack / unpack / direct x one and two vectors per thread x (checksum, inline) variants, and the plain copy
    assert checked >= 2 * (4 + 4 + 1) + 1, checked
