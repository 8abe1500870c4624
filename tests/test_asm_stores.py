"""The write-through stores of the kernels are issued by an asm statement the compiler does not know
to be a store.  For a store of more than 8 bytes the hardware still reads the data registers in the
cycles after the instruction has issued; the compiler separates such a store of its own from a vector
instruction that overwrites the data by `s_nop 1`.  The asm statement has to carry that wait itself
(see st16_through in th_kernels.hip).  Checked here on the compiled code: every 16-byte write-through
store is followed at once by a wait that is at least as long as the one the compiler uses."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2604_09107_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-S", "--cuda-device-only", "-x", "hip"]

pytestmark = pytest.mark.skipif(not os.path.exists(HIPCC) and shutil.which("hipcc") is None, reason="needs hipcc")


def instructions(body):
    return [l.strip() for l in body.split(".Lfunc_end")[0].splitlines()
            if l.strip() and not l.strip().startswith((";", "."))]


def compiler_wait_states(tmp_path):
    """Wait states the compiler puts between a 16-byte store of its own and a vector instruction that
    overwrites the stored registers (s_nop N waits N + 1)."""
    src = tmp_path / "hazard.hip"
    src.write_text("""
#include <hip/hip_runtime.h>
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__global__ void k(u32x4* a, u32x4* b) {
    u32x4 v = a[threadIdx.x];
    a[threadIdx.x + 64] = v;
    v.x += 1; v.y += 2; v.z += 3; v.w += 4;
    b[threadIdx.x] = v;
}
""")
    out = tmp_path / "hazard.s"
    subprocess.run([HIPCC] + FLAGS + [str(src), "-o", str(out)], check=True, stderr=subprocess.DEVNULL)
    lines = instructions(out.read_text())
    first = next(i for i, l in enumerate(lines) if l.startswith("global_store_dwordx4"))
    nxt = lines[first + 1]
    if nxt.startswith("v_add"):
        return 0
    m = re.match(r"s_nop (\d+)$", nxt)
    assert m and lines[first + 2].startswith("v_add"), lines[first:first + 3]
    return int(m.group(1)) + 1


def test_wide_write_through_stores_carry_the_compilers_wait(tmp_path):
    need = compiler_wait_states(tmp_path)
    assert need >= 1  # the window exists on this target: this is why the asm statement carries a wait
    asm = str(tmp_path / "k.s")
    subprocess.run([HIPCC] + FLAGS[:7] + ["-I", os.path.join(ROOT, "include"), "-I", CSRC] + FLAGS[7:] +
                   [os.path.join(CSRC, "th_kernels.hip"), "-o", asm], check=True, stderr=subprocess.DEVNULL)
    text = open(asm).read()
    kernels = re.split(r"^(\S+):\s*; @\S+\n", text, flags=re.M)
    wide = re.compile(r"global_store_dwordx[34] \S+ \S+ off sc1 nt")
    narrow = re.compile(r"global_store_dwordx2 \S+ \S+ off sc1 nt")
    with_wide = with_narrow = 0
    for name, body in zip(kernels[1::2], kernels[2::2]):
        lines = instructions(body)
        hits = [i for i, l in enumerate(lines) if wide.match(l)]
        with_narrow += any(narrow.match(l) for l in lines)
        if not hits:
            continue
        with_wide += 1
        for i in hits:
            m = re.match(r"s_nop (\d+)$", lines[i + 1])
            assert m and int(m.group(1)) + 1 >= need, "%s: '%s' follows '%s'" % (name, lines[i + 1], lines[i])
    # 16 pack, 16 unpack and 4 direct instances of the tile kernel hold both kinds, the plain copy the wide one
    assert with_wide >= 16 + 16 + 4 + 1, with_wide
    assert with_narrow >= 16 + 16 + 4, with_narrow
