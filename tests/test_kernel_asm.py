"""Host-side check of the code the compiler makes of the window loop (no GPU): a register spilled on the window path is
reloaded from scratch with a vector memory operation, and such operations complete in order, so the reload waits for
every row prefetch in flight.  The assembly of the two headline instantiations must hold no scratch load in a basic
block that does the windows' multiply-adds."""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2312_07743_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _assembly(template_args):
    with tempfile.TemporaryDirectory() as tmp:
        src = os.path.join(tmp, "unit.hip")
        with open(src, "w") as f:
            f.write('#include "w2v_train_kernel.h"\nnamespace w2v { namespace {\n'
                    f"template __global__ void train_kernel<{template_args}>(KernelArgs);\n}} }}\n")
        out = os.path.join(tmp, "unit.s")
        cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off", "-Xclang", "-target-feature",
               "-Xclang", "-packed-fp32-ops", "-I", CSRC, "--cuda-device-only", "-S", src, "-o", out]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        return open(out).read()


def _blocks(asm):
    blocks, cur = {}, "entry"
    for line in asm.splitlines():
        s = line.strip()
        m = re.match(r"^(\.LBB\d+_\d+):", s)
        if m:
            cur = m.group(1)
            continue
        if s and not s.startswith((".", ";")):
            blocks.setdefault(cur, []).append(s.split(";")[0].strip())
    return blocks


@pytest.mark.skipif(not shutil.which(HIPCC), reason="hipcc not found")
@pytest.mark.parametrize("name, args", [("mid", "2, 1, 0, 5, true, 1, false, false"),
                                        ("graph", "2, 1, 0, 10, true, 1, false, false")])
def test_no_spill_reload_where_the_windows_multiply_adds_are(name, args):
    asm = _assembly(args)
    spills = re.search(r"\.vgpr_spill_count:\s+(\d+)", asm)
    assert spills is not None
    hot = {}
    for label, ins in _blocks(asm).items():
        fma = sum(i.startswith(("v_fmac_f32", "v_fma_f32", "v_mul_f32_dpp")) for i in ins)
        reloads = [i for i in ins if i.startswith("scratch_load")]
        if fma >= 20 and reloads:
            hot[label] = reloads
    assert not hot, (name, hot)
    assert int(spills.group(1)) <= (8 if name == "mid" else 32), spills.group(1)
