"""ll_options through the binding (no GPU): the ctypes mirror matches the C struct, explicit options
do not look at the environment, NULL options are the process defaults read once from it, and a struct
from a caller built against a shorter definition leaves the fields it does not have automatic."""
import ctypes
import os
import subprocess
import sys

import pytest

import paper_2505_23819_amd as ll
import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def config_layouts(cid):
    c = wl.config(cid)
    a = ll.distributed_layout(c.nreg, c.nlane, c.nwave, c.out_dim_bits, c.src_bases)
    b = ll.distributed_layout(c.nreg, c.nlane, c.nwave, c.out_dim_bits, c.dst_bases)
    return c, a, b


def test_mirror_has_the_size_the_library_reports_and_starts_automatic():
    o = ll.ll_options_init()
    assert o.size == ctypes.sizeof(ll.ll_options)
    for name, _ in ll.ll_options._fields_:
        if name != "size":
            assert getattr(o, name) == ll.LL_AUTO, name
    with pytest.raises(ll.LLError):
        ll.ll_options_init(no_such_field=1)
    with pytest.raises(ll.LLError):
        ll.ll_options_init(size=4)


def test_a_shorter_struct_leaves_later_fields_automatic():
    c, a, b = config_layouts(4)
    full = ll.ll_options_init(strategy=ll.LL_STRATEGY_LDS_ELEM, elem_threads_log2=10, block_bytes=16384)
    info = ll.ll_plan_convert(a, b, c.elem_bytes, full).info()
    assert (info["strategy_name"], info["threads"]) == ("lds_elem", 1024)
    short = ll.ll_options_init(strategy=ll.LL_STRATEGY_LDS_ELEM, elem_threads_log2=10, block_bytes=16384)
    short.size = ll.ll_options.strategy.offset + 4           # a caller that knows `size` and `strategy` only
    info = ll.ll_plan_convert(a, b, c.elem_bytes, short).info()
    want = ll.ll_plan_convert(a, b, c.elem_bytes, ll.ll_options_init(strategy=ll.LL_STRATEGY_LDS_ELEM)).info()
    assert info == want and info["threads"] != 1024
    empty = ll.ll_options_init(strategy=ll.LL_STRATEGY_LDS_ELEM)
    empty.size = 0                                            # not even `strategy`: everything automatic
    assert ll.ll_plan_convert(a, b, c.elem_bytes, empty).info() == ll.ll_plan_convert(a, b, c.elem_bytes).info()


CHILD = r"""
import sys
sys.path.insert(0, {root!r})
import paper_2505_23819_amd as ll, workloads as wl
c = wl.config(2)
a = ll.distributed_layout(c.nreg, c.nlane, c.nwave, c.out_dim_bits, c.src_bases)
b = ll.distributed_layout(c.nreg, c.nlane, c.nwave, c.out_dim_bits, c.dst_bases)
env = ll.ll_options_from_env()
print(env.strategy, env.block_bytes, env.gather_kernel)
print(ll.ll_plan_convert(a, b, c.elem_bytes).info()["strategy_name"])                        # NULL: process defaults
print(ll.ll_plan_convert(a, b, c.elem_bytes, ll.ll_options_init()).info()["strategy_name"])  # explicit: no environment
import os
os.environ["LL_STRATEGY"] = "4"                                                               # too late: read once
print(ll.ll_plan_convert(a, b, c.elem_bytes).info()["strategy_name"])
"""


def test_null_options_are_the_environment_read_once_and_explicit_options_ignore_it():
    env = dict(os.environ, LL_STRATEGY="3", LL_BLOCK_BYTES="4096", LL_GATHER_KERNEL="not a number")
    res = subprocess.run([sys.executable, "-c", CHILD.format(root=ROOT)], env=env, capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = res.stdout.strip().splitlines()
    assert lines[0].split() == ["3", "4096", str(ll.LL_AUTO)]
    assert lines[1] == "lds_elem"
    assert lines[2] == "reg_permute"
    assert lines[3] == "lds_elem"
