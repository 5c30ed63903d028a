"""Properties of the generated gfx950 code that performance depends on and that no parity test sees:
no kernel uses scratch memory or spills registers, and the register-resident kernels are not
compiled into compare-and-select chains (an array of registers indexed through control flow the
compiler could not resolve costs one compare and one select per register and access: one such
instantiation ran at 2.5-4 TB/s instead of 6).  Compiles the kernels to assembly (about a minute)."""
import collections
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.fixture(scope="module")
def assembly(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("isa") / "kernels.s")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-S", "--cuda-device-only", os.path.join(ROOT, "paper_2505_23819_amd", "csrc", "kernels.hip"), "-o", out]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    return open(out).read()


def test_no_kernel_uses_scratch_or_spills(assembly):
    priv = re.findall(r"\.private_segment_fixed_size:\s+(\d+)", assembly)
    spills = re.findall(r"\.[sv]gpr_spill_count:\s+(\d+)", assembly)
    assert len(priv) > 300                                           # every instantiation is there
    assert all(int(p) == 0 for p in priv)
    assert all(int(x) == 0 for x in spills)


def test_register_kernels_have_no_select_chains(assembly):
    lines = assembly.splitlines()
    starts = [(i, l.split(":")[0]) for i, l in enumerate(lines) if l.startswith("_ZN2ll") and "@" in l]
    assert len(starts) > 300
    worst = {}
    for i, sym in starts:
        end = next(j for j in range(i, len(lines)) if lines[j].startswith(".Lfunc_end"))
        ops = collections.Counter(l.split()[0] for l in lines[i:end]
                                  if l.startswith("\t") and not l.strip().startswith((".", ";")))
        compares = sum(v for k, v in ops.items() if k.startswith("v_cmp_eq"))
        if "k_vec" in sym or "k_lds_elem" in sym or "k_pull" in sym:
            # conversions index their registers statically: a handful of compares (lane tests), never one per register
            assert compares <= 16, (sym, compares)
        worst[sym] = sum(ops.values())
    # the largest kernels are the 64-register gathers (about 4800 instructions); nothing may be far beyond
    assert max(worst.values()) < 8000, max(worst.items(), key=lambda kv: kv[1])
