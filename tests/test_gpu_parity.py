"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

import paper_2505_23819_amd as ll  # noqa: E402  (a missing library must fail loudly, not skip)

DTYPES = {1: torch.uint8, 2: torch.int16, 4: torch.int32, 8: torch.int64}
NP_DTYPES = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}


def layouts_of(cfg):
    a = ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.src_bases)
    b = None
    if cfg.dst_bases is not None:
        b = ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.dst_bases)
    return a, b


def run_convert(plan, src_bits: np.ndarray, d: int) -> np.ndarray:
    """src_bits: host array of unsigned ints (raw bits).  Returns the converted image."""
    w = src_bits.itemsize
    ntiles = src_bits.size >> d
    src = torch.from_numpy(src_bits.view({1: np.uint8, 2: np.int16, 4: np.int32, 8: np.int64}[w])).cuda()
    dst = torch.full_like(src, 0x5A if w == 1 else 0x5A5A)      # poison: every slot must be written
    ll.ll_convert(plan, src, dst, ntiles)
    torch.cuda.synchronize()
    return dst.cpu().numpy().view(NP_DTYPES[w])


def random_invertible(rng, d):
    while True:
        cols = [int(rng.integers(0, 1 << d)) for _ in range(d)]
        seen = {0}
        for c in cols:
            seen |= {x ^ c for x in seen}
        if len(seen) == 1 << d:
            return cols


@pytest.mark.parametrize("cid,ntiles", [(1, 1), (2, 3), (3, 5), (4, 2), (2, 1), (3, 1), (4, 1)])
def test_convert_configs_small(cid, ntiles):
    cfg = wl.config(cid)
    a, b = layouts_of(cfg)
    plan = ll.ll_plan_convert(a, b, cfg.elem_bytes)
    src = wl.to_numpy_bits(cfg.gen_data(0, ntiles))
    got = run_convert(plan, src, cfg.d)
    want = oracle.convert(cfg.src_bases, cfg.dst_bases, src)
    assert np.array_equal(got, want), f"config {cid}: {np.count_nonzero(got != want)} mismatches"


@pytest.mark.parametrize("w", [1, 2, 4, 8])
@pytest.mark.parametrize("d,nreg,nlane", [(8, 2, 5), (10, 2, 6), (12, 4, 6), (13, 3, 6), (15, 5, 6)])
def test_convert_random_xor_layouts(w, d, nreg, nlane):
    rng = np.random.default_rng(1000 * w + d)
    nwave = d - nreg - nlane
    for trial in range(3):
        ca, cb = random_invertible(rng, d), random_invertible(rng, d)
        a = ll.distributed_layout(nreg, nlane, nwave, [d], ca)
        b = ll.distributed_layout(nreg, nlane, nwave, [d], cb)
        plan = ll.ll_plan_convert(a, b, w)
        ntiles = int(rng.integers(1, 40))            # ragged: not a multiple of the tile group
        src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=ntiles << d, dtype=NP_DTYPES[w])
        got = run_convert(plan, src, d)
        want = oracle.convert(ca, cb, src)
        assert np.array_equal(got, want)


@pytest.mark.parametrize("w", [1, 2, 4, 8])
def test_convert_random_permutation_layouts(w):
    rng = np.random.default_rng(77 + w)
    for d, nreg, nlane in [(9, 3, 6), (12, 4, 6), (14, 6, 6), (16, 6, 6)]:
        nwave = d - nreg - nlane
        ca = [1 << int(p) for p in rng.permutation(d)]
        cb = [1 << int(p) for p in rng.permutation(d)]
        a = ll.distributed_layout(nreg, nlane, nwave, [d], ca)
        b = ll.distributed_layout(nreg, nlane, nwave, [d], cb)
        plan = ll.ll_plan_convert(a, b, w)
        ntiles = int(rng.integers(1, 9))
        src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=ntiles << d, dtype=NP_DTYPES[w])
        assert np.array_equal(run_convert(plan, src, d), oracle.convert(ca, cb, src))


def test_convert_identity_is_copy_and_zero_tiles():
    cfg = wl.config(1)
    a, _ = layouts_of(cfg)
    plan = ll.ll_plan_convert(a, a, 4)
    assert plan.info()["kind_name"] == "noop"
    src = wl.to_numpy_bits(cfg.gen_data(0, 3))
    assert np.array_equal(run_convert(plan, src, cfg.d), src)
    ll.ll_convert(plan, 0, 0, 0)                       # ntiles == 0: nothing is touched


def run_gather(layout, axis, inp_bits: np.ndarray, idx: np.ndarray, d: int, opts=None) -> np.ndarray:
    w = inp_bits.itemsize
    ntiles = inp_bits.size >> d
    tin = torch.from_numpy(inp_bits.view({1: np.uint8, 2: np.int16, 4: np.int32, 8: np.int64}[w])).cuda()
    tidx = torch.from_numpy(idx).cuda()
    tout = torch.full_like(tin, 0x5A if w == 1 else 0x5A5A)
    ll.ll_gather(layout, axis, w, tin, tidx, tout, ntiles, opts=opts)
    torch.cuda.synchronize()
    return tout.cpu().numpy().view(NP_DTYPES[w])


@pytest.mark.parametrize("ntiles", [1, 3])
def test_gather_config5_small(ntiles):
    cfg = wl.config(5)
    layout, _ = layouts_of(cfg)
    inp = wl.to_numpy_bits(cfg.gen_data(0, ntiles))
    idx = cfg.gen_idx(0, ntiles).numpy()
    got = run_gather(layout, cfg.axis, inp, idx, cfg.d)
    want = oracle.gather(cfg.src_bases, cfg.out_dim_bits, cfg.axis, inp, idx)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("w", [1, 2, 4, 8])
@pytest.mark.parametrize("nreg,nwave,axis_bits", [(2, 0, 6), (3, 1, 4), (4, 2, 6), (5, 1, 3), (1, 3, 5)])
def test_gather_random_lane_axis(w, nreg, nwave, axis_bits):
    """Axis bits live on an arbitrary subset of the lane bits, mixed by XOR with other lane bits;
    the other logical bits are spread over registers, the remaining lanes and waves.  Run through the
    library's own choice, through the wave kernels (shuffle / wave-staged) on request where a lane
    holds the 4 bytes they need, and through the workgroup-staged kernel on request."""
    rng = np.random.default_rng(31 * w + nreg + 7 * nwave + axis_bits)
    d = nreg + 6 + nwave
    other_bits = d - axis_bits
    dims = [axis_bits, other_bits]                    # axis is dim 0 (upper logical bits)
    # lane part: a random invertible 6x6 map of lane bits onto [axis bits | 6 - axis_bits others]
    lane_mix = random_invertible(rng, 6)
    others = list(rng.permutation(other_bits))        # logical "other" bit taken by each non-axis hw bit
    bases = [0] * d
    lane_targets = [1 << (other_bits + k) for k in range(axis_bits)] + \
                   [1 << int(others[k]) for k in range(6 - axis_bits)]
    for b in range(6):
        v = 0
        for k in range(6):
            if (lane_mix[b] >> k) & 1:
                v ^= lane_targets[k]
        bases[nreg + b] = v
    rest = [1 << int(o) for o in others[6 - axis_bits:]]
    for k, hw_bit in enumerate(list(range(nreg)) + list(range(nreg + 6, d))):
        bases[hw_bit] = rest[k]
    layout = ll.distributed_layout(nreg, 6, nwave, dims, bases)
    ntiles = 3
    inp = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=ntiles << d, dtype=NP_DTYPES[w])
    idx = rng.integers(0, 1 << axis_bits, size=ntiles << d, dtype=np.int32)
    idx[::17] += 1 << axis_bits                        # out-of-range entries wrap
    want = oracle.gather(bases, dims, 0, inp, idx)
    wave_ok = (1 << nreg) * w >= 4
    for kernel, allowed in ((None, ("shuffle", "wave_staged", "shuffle_rows", "block_staged")),
                            (ll.LL_GATHER_SHUFFLE, ("shuffle",) if wave_ok else ("block_staged",)),
                            (ll.LL_GATHER_WAVE_STAGED, ("shuffle", "wave_staged") if wave_ok else ("block_staged",)),
                            (ll.LL_GATHER_SHUFFLE_ROWS, ("shuffle", "shuffle_rows") if wave_ok else ("block_staged",)),
                            (ll.LL_GATHER_BLOCK_STAGED, ("block_staged",))):
        opts = None if kernel is None else ll.ll_options_init(gather_kernel=kernel, gather_waves=int(rng.choice([-1, 1, 2, 4])))
        assert ll.ll_gather_info(layout, 0, w, opts)["kernel_name"] in allowed, kernel
        if kernel == ll.LL_GATHER_SHUFFLE_ROWS and wave_ok and 32 <= (1 << nreg) * w <= 256:
            assert ll.ll_gather_info(layout, 0, w, opts)["kernel_name"] == "shuffle_rows"
        got = run_gather(layout, 0, inp, idx, d, opts)
        assert np.array_equal(got, want), kernel


@pytest.mark.parametrize("cid", [1, 2, 3, 4])
def test_convert_configs_reverse_direction(cid):
    cfg = wl.config(cid)
    a, b = layouts_of(cfg)
    plan = ll.ll_plan_convert(b, a, cfg.elem_bytes)
    src = wl.to_numpy_bits(cfg.gen_data(0, 3))
    assert np.array_equal(run_convert(plan, src, cfg.d), oracle.convert(cfg.dst_bases, cfg.src_bases, src))


@pytest.mark.parametrize("force,threads_log2", [(3, -1), (3, 6), (3, 8), (4, -1)])
@pytest.mark.parametrize("cid", [1, 2, 3, 4])
def test_convert_configs_forced_lds_strategies(cid, force, threads_log2):
    """Every config through the element-wide LDS kernel (3: workgroup size chosen by the planner, one
    wave, four waves) and, where it applies, the 128-bit one (4)."""
    cfg = wl.config(cid)
    a, b = layouts_of(cfg)
    plan = ll.ll_plan_convert(a, b, cfg.elem_bytes, ll.ll_options_init(strategy=force, elem_threads_log2=threads_log2))
    name = plan.info()["strategy_name"]
    assert name in ("lds_elem", "lds_vec") and (force != 3 or name == "lds_elem")
    if force == 3 and threads_log2 > 0:
        info = plan.info()
        one_wave_block = (cfg.elem_bytes << info["block_bits"]) == 4096      # the one-wave kernel takes 4 KiB blocks only
        assert info["threads"] == (1 << threads_log2 if threads_log2 != 6 or one_wave_block else 256)
    src = wl.to_numpy_bits(cfg.gen_data(1, 3))
    assert np.array_equal(run_convert(plan, src, cfg.d), oracle.convert(cfg.src_bases, cfg.dst_bases, src))


@pytest.mark.parametrize("w", [2, 4, 8])
@pytest.mark.parametrize("nreg", [2, 3, 4, 5, 6])
def test_convert_intra_wave_bit_permutations(w, nreg):
    """Register and lane bits permuted among themselves (wave bits fixed): the shuffle / register
    kernels where their structure applies, LDS otherwise; all must match the oracle."""
    rng = np.random.default_rng(500 + 10 * w + nreg)
    nwave = 2
    d = nreg + 6 + nwave
    seen = set()
    for trial in range(12):
        low = nreg + 6
        if trial % 3 == 2:      # registers only
            pa = list(rng.permutation(nreg)) + list(range(nreg, d))
            pb = list(rng.permutation(nreg)) + list(range(nreg, d))
        else:
            pa = list(rng.permutation(low)) + list(range(low, d))
            pb = list(rng.permutation(low)) + list(range(low, d))
        ca, cb = [1 << int(x) for x in pa], [1 << int(x) for x in pb]
        a = ll.distributed_layout(nreg, 6, nwave, [d], ca)
        b = ll.distributed_layout(nreg, 6, nwave, [d], cb)
        plan = ll.ll_plan_convert(a, b, w)
        info = plan.info()
        assert info["kind_name"] in ("noop", "reg_only", "intra_wave")
        seen.add(info["strategy_name"])
        ntiles = int(rng.integers(1, 6))
        src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=ntiles << d, dtype=NP_DTYPES[w])
        assert np.array_equal(run_convert(plan, src, d), oracle.convert(ca, cb, src)), (trial, info["strategy_name"])
    print("strategies used:", sorted(seen))


def test_convert_structured_shuffle_cases():
    """Hand-built conversions that need lane <-> register stages with the transpose before, after,
    and not at all (4-byte elements, 6 register + 6 lane bits)."""
    d, nreg = 12, 6
    ident = list(range(d))

    def swap(perm, x, y):
        p = perm[:]
        p[x], p[y] = p[y], p[x]
        return p

    cases = {
        "no transpose, one stage": swap(ident, 3, 8),                 # register bit 3 <-> lane bit 2
        "vector bits to lanes": swap(swap(ident, 0, 6), 1, 7),        # position bits <-> lane bits 0, 1
        "vector bits to registers": swap(swap(ident, 0, 4), 1, 5),    # position bits <-> register bits 4, 5
        "three stages": swap(swap(swap(ident, 2, 9), 3, 10), 4, 11),
    }
    rng = np.random.default_rng(9)
    used = {}
    for name, perm in cases.items():
        ca = [1 << k for k in range(d)]
        cb = [1 << perm[k] for k in range(d)]
        for x, y, cx, cy in ((ca, cb, ca, cb), (cb, ca, cb, ca)):
            a = ll.distributed_layout(nreg, 6, 0, [d], x)
            b = ll.distributed_layout(nreg, 6, 0, [d], y)
            plan = ll.ll_plan_convert(a, b, 4)
            used[name] = plan.info()["strategy_name"]
            src = rng.integers(0, 1 << 32, size=5 << d, dtype=np.uint32)
            assert np.array_equal(run_convert(plan, src, d), oracle.convert(cx, cy, src)), name
    print(used)


# ---------------------------------------------------------------------------------------------
# layouts with broadcasting (Sec. 5.1 "Broadcasting", Sec. 5.4 rule 2)
# ---------------------------------------------------------------------------------------------

def run_convert_general(plan, src_bits: np.ndarray, d_src: int, d_dst: int) -> np.ndarray:
    w = src_bits.itemsize
    ntiles = src_bits.size >> d_src
    tdt = {1: np.uint8, 2: np.int16, 4: np.int32, 8: np.int64}[w]
    src = torch.from_numpy(src_bits.view(tdt)).cuda()
    dst = torch.full((ntiles << d_dst,), 0x5A if w == 1 else 0x5A5A, dtype=src.dtype, device="cuda")
    ll.ll_convert(plan, src, dst, ntiles)
    torch.cuda.synchronize()
    return dst.cpu().numpy().view(NP_DTYPES[w])


def surjective_bases(rng, d_in, d_out):
    while True:
        cols = [int(rng.integers(0, 1 << d_out)) for _ in range(d_in)]
        if d_in > d_out:
            cols[int(rng.integers(0, d_in))] = 0
        seen = {0}
        for c in cols:
            seen |= {x ^ c for x in seen}
        if len(seen) == 1 << d_out:
            return cols


@pytest.mark.parametrize("w", [1, 2, 4, 8])
def test_convert_paper_zero_column_example(w):
    """Layout A of Sec. 4.1 and its copy with a zero column after the register bits: expand,
    collapse and replica-to-replica.  Replicas in the source hold different values, so reading any
    slot but the one whose replica bit is zero fails."""
    base = wl.PAPER_LAYOUT_A
    wide = base[:2] + [0] + base[2:]
    a = ll.ll_layout_create([(ll.LL_IN_REG, 2), (ll.LL_IN_LANE, 5), (ll.LL_IN_WAVE, 1)], [4, 4], base)
    b = ll.ll_layout_create([(ll.LL_IN_REG, 3), (ll.LL_IN_LANE, 5), (ll.LL_IN_WAVE, 1)], [4, 4], wide)
    rng = np.random.default_rng(w)
    for x, y, cx, cy in ((a, b, base, wide), (b, a, wide, base), (b, b, wide, wide)):
        plan = ll.ll_plan_convert(x, y, w)
        for ntiles in (1, 7, 150):
            src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=ntiles << len(cx), dtype=NP_DTYPES[w])
            got = run_convert_general(plan, src, len(cx), len(cy))
            assert np.array_equal(got, oracle.convert_general(cx, cy, 8, src)), (len(cx), len(cy), ntiles)


# the broadcast kernel as planned by default, with one wave per block, and with one wave on 4 KiB blocks
PULL_OPTION_SETS = (None, lambda: ll.ll_options_init(pull_threads_log2=6),
                    lambda: ll.ll_options_init(pull_threads_log2=6, block_bytes=4096))


@pytest.mark.parametrize("w", [1, 2, 4, 8])
@pytest.mark.parametrize("da,db,dl", [(9, 8, 8), (8, 10, 8), (12, 12, 10), (14, 13, 12), (16, 14, 12),
                                      (7, 9, 6), (10, 12, 10), (13, 13, 13)])
def test_convert_random_broadcast_layouts(w, da, db, dl):
    rng = np.random.default_rng(7000 + 100 * w + da + 3 * db)
    for trial in range(3):
        ca, cb = surjective_bases(rng, da, dl), surjective_bases(rng, db, dl)
        a = ll.ll_layout_create([(ll.LL_IN_REG, 2), (ll.LL_IN_LANE, da - 2)], [dl], ca)
        b = ll.ll_layout_create([(ll.LL_IN_REG, 2), (ll.LL_IN_LANE, db - 2)], [dl], cb)
        ntiles = int(rng.integers(1, 40))
        src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=ntiles << da, dtype=NP_DTYPES[w])
        want = oracle.convert_general(ca, cb, dl, src)
        for opts in PULL_OPTION_SETS:
            plan = ll.ll_plan_convert(a, b, w, opts() if opts else None)
            got = run_convert_general(plan, src, da, db)
            assert np.array_equal(got, want), (trial, plan.info()["strategy_name"], plan.info()["threads"])


@pytest.mark.parametrize("case", wl.broadcast_cases(), ids=lambda c: c.name.split(" (")[0].replace(" ", "_"))
def test_convert_broadcast_workloads_small(case):
    a = ll.distributed_layout(*case.src_in, case.out_dim_bits, case.src_bases)
    b = ll.distributed_layout(*case.dst_in, case.out_dim_bits, case.dst_bases)
    for opts in PULL_OPTION_SETS:
        plan = ll.ll_plan_convert(a, b, case.elem_bytes, opts() if opts else None)
        assert plan.info()["kind_name"] == "broadcast"
        for ntiles in (1, 5):
            src = wl.to_numpy_bits(case.gen_data(0, ntiles))
            got = run_convert_general(plan, src, case.d_src, case.d_dst)
            assert np.array_equal(got, oracle.convert_general(case.src_bases, case.dst_bases, case.d_out, src)), plan.info()["threads"]


# ---------------------------------------------------------------------------------------------
# LDS staging read back with the transposing LDS loads (Sec. 5.3 "Using SIMD Hardware Primitives")
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("w", [1, 2])
def test_convert_transposing_lds_reads(w):
    """Transposes and other bit permutations of 1- and 2-byte elements through ds_read_b64_tr_b8 /
    _tr_b16 (requested, so that 2-byte cases do not take the register path)."""
    tr = ll.ll_options_init(strategy=ll.LL_STRATEGY_LDS_TR)
    rng = np.random.default_rng(600 + w)
    used = 0
    cases = []
    c2 = wl.config(2)
    cases.append((c2.nreg, c2.nlane, c2.nwave, c2.out_dim_bits, c2.src_bases, c2.dst_bases))
    cases.append((c2.nreg, c2.nlane, c2.nwave, c2.out_dim_bits, c2.dst_bases, c2.src_bases))
    c3 = wl.config(3)
    cases.append((c3.nreg, c3.nlane, c3.nwave, c3.out_dim_bits, c3.src_bases, c3.dst_bases))
    for d, nreg in [(12, 4), (13, 5), (14, 6), (16, 6), (11, 4)]:
        for _ in range(4):
            ca = [1 << int(p) for p in rng.permutation(d)]
            cb = [1 << int(p) for p in rng.permutation(d)]
            cases.append((nreg, 6, d - nreg - 6, [d], ca, cb))
    for nreg, nlane, nwave, dims, ca, cb in cases:
        d = nreg + nlane + nwave
        plan = ll.ll_plan_convert(ll.distributed_layout(nreg, nlane, nwave, dims, ca),
                                  ll.distributed_layout(nreg, nlane, nwave, dims, cb), w, tr)
        used += plan.info()["strategy_name"] == "lds_tr"
        ntiles = int(rng.integers(1, 12))
        src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=ntiles << d, dtype=NP_DTYPES[w])
        assert np.array_equal(run_convert(plan, src, d), oracle.convert(ca, cb, src)), plan.info()["strategy_name"]
    assert used >= 3, "the transposing-read planner applied to %d cases only" % used


def test_one_byte_transpose_through_both_lds_kernels():
    c2 = wl.config(2)
    a, b = layouts_of(c2)
    src = np.random.default_rng(5).integers(0, 255, size=9 << c2.d, dtype=np.uint8)
    want = oracle.convert(c2.src_bases, c2.dst_bases, src)
    plan = ll.ll_plan_convert(a, b, 1)
    assert plan.info()["strategy_name"] == "lds_elem"
    assert np.array_equal(run_convert(plan, src, c2.d), want)
    plan = ll.ll_plan_convert(a, b, 1, ll.ll_options_init(strategy=ll.LL_STRATEGY_LDS_TR))
    info = plan.info()
    assert info["strategy_name"] == "lds_tr" and info["lds_read_bytes"] == 8
    assert np.array_equal(run_convert(plan, src, c2.d), want)


# ---------------------------------------------------------------------------------------------
# general gather: axis on register and wave bits, arbitrary XOR layouts (Sec. 5.5 extended)
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("axis,ntiles", [(1, 1), (1, 3), (0, 2)])
def test_gather_config5_any_axis(axis, ntiles):
    """Config 5's layout gathered along its columns (registers and waves: the workgroup-staged
    kernel) and along its rows with that kernel forced."""
    cfg = wl.config(5)
    layout, _ = layouts_of(cfg)
    opts = ll.ll_options_init(gather_kernel=ll.LL_GATHER_BLOCK_STAGED) if axis == 0 else None
    assert ll.ll_gather_info(layout, axis, cfg.elem_bytes, opts)["kernel_name"] == "block_staged"
    rng = np.random.default_rng(axis + 10 * ntiles)
    inp = wl.to_numpy_bits(cfg.gen_data(0, ntiles))
    idx = rng.integers(0, 1 << cfg.out_dim_bits[axis], size=ntiles << cfg.d, dtype=np.int32)
    idx[::13] += 1 << cfg.out_dim_bits[axis]                      # wraps
    got = run_gather(layout, axis, inp, idx, cfg.d, opts)
    want = oracle.gather(cfg.src_bases, cfg.out_dim_bits, axis, inp, idx)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("w", [1, 2, 4, 8])
@pytest.mark.parametrize("d,dims", [(8, [3, 5]), (10, [4, 3, 3]), (12, [6, 6]), (13, [2, 11]), (7, [7]), (11, [5, 6])])
def test_gather_random_xor_layouts_any_axis(w, d, dims):
    """Random invertible layouts (columns are arbitrary XOR combinations): every axis, so that its
    hardware bits fall on registers, lanes and waves alike; tiles smaller and larger than a block;
    ragged tile counts."""
    rng = np.random.default_rng(4000 + 17 * w + d)
    nreg = int(rng.integers(0, min(4, d - 2) + 1))
    nlane = min(6, d - nreg)
    nwave = d - nreg - nlane
    for axis in range(len(dims)):
        cols = random_invertible(rng, d)
        layout = ll.distributed_layout(nreg, nlane, nwave, dims, cols)
        info = ll.ll_gather_info(layout, axis, w)
        ntiles = int(rng.integers(1, 70))
        inp = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=ntiles << d, dtype=NP_DTYPES[w])
        idx = rng.integers(0, 1 << dims[axis], size=ntiles << d, dtype=np.int32)
        idx[::7] -= 1 << dims[axis]                                # negative entries wrap too
        got = run_gather(layout, axis, inp, idx, d)
        want = oracle.gather(cols, dims, axis, inp, idx)
        assert np.array_equal(got, want), (axis, info)


def test_gather_register_axis_and_identity_property():
    """Axis entirely on register bits (the paper's n = 2^bits rounds): idx[i, j] = i gives the
    input back; a constant index broadcasts one row."""
    nreg, d = 3, 11
    dims = [3, 8]
    bases = [1 << (8 + k) for k in range(3)] + [1 << k for k in range(8)]      # registers walk the axis
    layout = ll.distributed_layout(nreg, 6, 2, dims, bases)
    assert ll.ll_gather_info(layout, 0, 4)["paper_rounds"] == 8
    rng = np.random.default_rng(8)
    ntiles = 9
    inp = rng.integers(0, 1 << 32, size=ntiles << d, dtype=np.uint32)
    h = np.arange(ntiles << d) & ((1 << d) - 1)
    own = (h & 7).astype(np.int32)                                  # register index = axis coordinate
    assert np.array_equal(run_gather(layout, 0, inp, own, d), inp)
    const = np.full(ntiles << d, 5, dtype=np.int32)
    got = run_gather(layout, 0, inp, const, d)
    assert np.array_equal(got, oracle.gather(bases, dims, 0, inp, const))
    assert np.array_equal(got.reshape(-1, 8), np.repeat(inp.reshape(-1, 8)[:, 5:6], 8, axis=1))


# ---------------------------------------------------------------------------------------------
# affine layouts y = A x xor b: flips, half rolls, arbitrary constants (Conclusions)
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("cid", [1, 2, 3, 4])
def test_convert_configs_with_flips(cid):
    """Each configuration with its destination flipped along the rows, along both dims, and with
    an arbitrary constant on both sides (element positions inside the 16-byte vectors move too)."""
    cfg = wl.config(cid)
    a, b = layouts_of(cfg)
    dims = cfg.out_dim_bits
    rows = ((1 << dims[0]) - 1) << (cfg.d - dims[0])
    rng = np.random.default_rng(70 + cid)
    src = wl.to_numpy_bits(cfg.gen_data(0, 3))
    for oa, ob in ((0, rows), (0, (1 << cfg.d) - 1), (int(rng.integers(1, 1 << cfg.d)), int(rng.integers(1, 1 << cfg.d)))):
        plan = ll.ll_plan_convert(ll.ll_layout_with_offset(a, oa), ll.ll_layout_with_offset(b, ob), cfg.elem_bytes)
        got = run_convert(plan, src, cfg.d)
        want = oracle.convert_affine(cfg.src_bases, oa, cfg.dst_bases, ob, src)
        assert np.array_equal(got, want), (cid, oa, ob, plan.info()["strategy_name"])


@pytest.mark.parametrize("w", [1, 2, 4, 8])
def test_convert_random_affine_layouts(w):
    rng = np.random.default_rng(900 + w)
    for d, nreg in [(9, 3), (12, 4), (14, 6)]:
        for trial in range(6):
            if trial % 3 == 0:       # same layout, offsets only: a pure XOR shuffle of the image
                ca = cb = [1 << int(p) for p in rng.permutation(d)]
            elif trial % 3 == 1:
                ca, cb = [1 << int(p) for p in rng.permutation(d)], [1 << int(p) for p in rng.permutation(d)]
            else:
                ca, cb = random_invertible(rng, d), random_invertible(rng, d)
            oa, ob = int(rng.integers(0, 1 << d)), int(rng.integers(0, 1 << d))
            a = ll.ll_layout_with_offset(ll.distributed_layout(nreg, 6, d - nreg - 6, [d], ca), oa)
            b = ll.ll_layout_with_offset(ll.distributed_layout(nreg, 6, d - nreg - 6, [d], cb), ob)
            plan = ll.ll_plan_convert(a, b, w, ll.ll_options_init(strategy=ll.LL_STRATEGY_LDS_ELEM) if trial == 5 else None)
            ntiles = int(rng.integers(1, 20))
            src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=ntiles << d, dtype=NP_DTYPES[w])
            got = run_convert(plan, src, d)
            assert np.array_equal(got, oracle.convert_affine(ca, oa, cb, ob, src)), (d, trial, plan.info()["strategy_name"])


def test_flip_of_the_identity_layout_is_numpy_flip():
    d, dims = 13, [6, 7]
    ident = ll.distributed_layout(3, 6, 4, dims, [1 << k for k in range(d)])
    flipped = ll.ll_layout_with_offset(ident, ((1 << 6) - 1) << 7)          # rows reversed
    plan = ll.ll_plan_convert(ident, flipped, 2)
    src = np.random.default_rng(1).integers(0, 1 << 16, size=4 << d, dtype=np.uint16)
    got = run_convert(plan, src, d)
    assert np.array_equal(got.reshape(4, 64, 128), np.flip(src.reshape(4, 64, 128), axis=1))


@pytest.mark.parametrize("axis", [0, 1])
def test_gather_under_affine_layouts(axis):
    cfg = wl.config(5)
    base, _ = layouts_of(cfg)
    rng = np.random.default_rng(40 + axis)
    ntiles = 3
    inp = wl.to_numpy_bits(cfg.gen_data(0, ntiles))
    idx = rng.integers(0, 1 << cfg.out_dim_bits[axis], size=ntiles << cfg.d, dtype=np.int32)
    for off in ((1 << cfg.d) - 1, int(rng.integers(1, 1 << cfg.d))):
        layout = ll.ll_layout_with_offset(base, off)
        for staged in (ll.LL_GATHER_SHUFFLE, ll.LL_GATHER_WAVE_STAGED, ll.LL_GATHER_SHUFFLE_ROWS):
            got = run_gather(layout, axis, inp, idx, cfg.d, ll.ll_options_init(gather_kernel=staged))
            assert np.array_equal(got, oracle.gather_affine(cfg.src_bases, off, cfg.out_dim_bits, axis, inp, idx)), (off, staged)


# ---------------------------------------------------------------------------------------------
# extreme sizes
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("w", [1, 2, 4, 8])
def test_convert_tiny_tiles_are_bundled(w):
    """Tiles of 2 .. 128 elements (down to 2 bytes): many tiles share one workgroup block; ragged
    tile counts leave the last block partly empty."""
    rng = np.random.default_rng(300 + w)
    for d in range(1, 8):
        nreg = min(2, d)
        dims = [(ll.LL_IN_REG, nreg)] + ([(ll.LL_IN_LANE, d - nreg)] if d > nreg else [])
        ca, cb = random_invertible(rng, d), random_invertible(rng, d)
        plan = ll.ll_plan_convert(ll.ll_layout_create(dims, [d], ca), ll.ll_layout_create(dims, [d], cb), w)
        per16 = max(1, 16 // (w << d))            # tiles per 16-byte vector: buffers hold whole vectors
        for ntiles in (per16, 5 * per16, (1000 + int(rng.integers(0, 2000))) * per16):
            src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=ntiles << d, dtype=NP_DTYPES[w])
            assert np.array_equal(run_convert(plan, src, d), oracle.convert(ca, cb, src)), (d, ntiles)


def test_convert_one_large_tile():
    """A single tile of 2^25 four-byte elements (128 MiB, 65536 blocks of one tile)."""
    d = 25
    rng = np.random.default_rng(26)
    ca = [1 << int(p) for p in rng.permutation(d)]
    cb = [1 << int(p) for p in rng.permutation(d)]
    a = ll.distributed_layout(6, 6, d - 12, [d], ca)
    b = ll.distributed_layout(6, 6, d - 12, [d], cb)
    plan = ll.ll_plan_convert(a, b, 4)
    src = torch.randint(-2**31, 2**31 - 1, (1 << d,), dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    ll.ll_convert(plan, src, dst, 1)
    torch.cuda.synchronize()
    # sampled elements: destination index of h is the bit permutation cb^-1(ca(h))
    pos_b = {c: k for k, c in enumerate(cb)}
    hs = rng.integers(0, 1 << d, size=4096)
    hs[:2] = (0, (1 << d) - 1)
    to = np.zeros_like(hs)
    for k in range(d):
        to |= ((hs >> k) & 1) << pos_b[ca[k]]
    got = dst[torch.from_numpy(to).cuda()].cpu().numpy()
    want = src[torch.from_numpy(hs).cuda()].cpu().numpy()
    assert np.array_equal(got, want)
    # and the whole tile against the oracle's tabulated variant
    full, _ = oracle.convert(ca, cb, src.cpu().numpy().view(np.uint32), table=True)
    assert np.array_equal(dst.cpu().numpy().view(np.uint32), full)


@pytest.mark.parametrize("w,d", [(4, 16), (4, 17), (4, 20), (2, 19), (8, 18), (1, 15)])
def test_convert_large_tiles_random_xor(w, d):
    """Large tiles under random XOR layouts, a ragged number of tiles; 4-byte elements also through 16 KiB blocks of
    four waves (what 1- and 2-byte elements get from 2^17 elements on)."""
    rng = np.random.default_rng(9700 + 10 * w + d)
    ca, cb = wl.random_invertible_bases(500 + d, d), wl.random_invertible_bases(600 + d, d)
    a, b = ll.distributed_layout(4, 6, d - 10, [d], ca), ll.distributed_layout(4, 6, d - 10, [d], cb)
    plan = ll.ll_plan_convert(a, b, w)
    plans = [plan]
    if w == 4:            # 4 KiB blocks for one wave at every tile size; 16 KiB blocks for four waves on request
        info = plan.info()
        assert (info["threads"], info["vectors_per_thread"], info["block_bits"]) == (64, 4, 10)
        plans.append(ll.ll_plan_convert(a, b, w, ll.ll_options_init(block_bytes=16384)))
        info = plans[-1].info()
        assert (info["threads"], info["vectors_per_thread"], info["block_bits"]) == (256, 4, 12)
    src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=3 << d, dtype=NP_DTYPES[w])
    want = oracle.convert(ca, cb, src)
    for p in plans:
        assert np.array_equal(run_convert(p, src, d), want), p.info()["block_bits"]


# ---------------------------------------------------------------------------------------------
# memory layouts on one side (Sec. 5.3 "Shared Memory Load and Store": A^-1 o B)
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("w", [1, 2, 4])
def test_convert_between_memory_and_register_images(w):
    """Row-major and mma-swizzled memory images <-> the 32x32 accumulator layout over a 64 x 64 tile,
    and memory image <-> memory image (un-swizzling)."""
    plain = ll.ll_layout_mma_swizzle(6, 6, 1, 1, 1)                       # offset = row-major position
    swz = ll.ll_layout_mma_swizzle(6, 6, 8 // w if w < 8 else 1, 1, 8)
    acc = ll.ll_layout_mfma_accumulator(5)
    for label, dim in ((ll.LL_IN_WAVE, 0), (ll.LL_IN_WAVE, 1)):
        acc = ll.ll_product_dimwise(acc, ll.ll_layout_identity(label, dim, 1, 2))
    assert plain.in_dims == [(ll.LL_IN_OFFSET, 12)] and acc.in_dims == [(ll.LL_IN_REG, 4), (ll.LL_IN_LANE, 6), (ll.LL_IN_WAVE, 2)]
    rng = np.random.default_rng(50 + w)
    for x, y in ((plain, acc), (acc, plain), (swz, acc), (acc, swz), (swz, plain), (plain, swz)):
        plan = ll.ll_plan_convert(x, y, w)
        info = plan.info()
        assert info["kind_name"] == "lds"
        src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=7 << 12, dtype=NP_DTYPES[w])
        got = run_convert(plan, src, 12)
        assert np.array_equal(got, oracle.convert(x.bases, y.bases, src)), info["strategy_name"]
    # a row-major image converted to the swizzled layout and read with the swizzle formula
    plan = ll.ll_plan_convert(plain, swz, w)
    src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=1 << 12, dtype=NP_DTYPES[w])
    got = run_convert(plan, src, 12)
    vec = 8 // w
    for i, j in rng.integers(0, 64, size=(50, 2)):
        off = oracle.mma_swizzle_offset(int(i), int(j), 6, vec, 1, 8)
        assert got[off] == src[(int(i) << 6) | int(j)]
    assert ll.ll_plan_convert(plain, plain, w).info()["kind_name"] == "noop"


# ---------------------------------------------------------------------------------------------
# HIP graph capture: the entry points allocate nothing and never synchronize
# ---------------------------------------------------------------------------------------------

def test_entry_points_can_be_captured_in_a_hip_graph():
    """A conversion (config 1, launch bound) and a gather recorded into one graph and replayed with
    new inputs between replays; every replay must equal the eager result and the oracle."""
    c1, c5 = wl.config(1), wl.config(5)
    a, b = layouts_of(c1)
    plan = ll.ll_plan_convert(a, b, c1.elem_bytes)
    lay5, _ = layouts_of(c5)
    nt1, nt5 = 4, 2
    src = torch.zeros(nt1 << c1.d, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    inp = torch.zeros(nt5 << c5.d, dtype=torch.float16, device="cuda")
    idx = torch.zeros(nt5 << c5.d, dtype=torch.int32, device="cuda")
    out = torch.zeros_like(inp)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up outside capture
        ll.ll_convert(plan, src, dst, nt1)
        ll.ll_gather(lay5, c5.axis, c5.elem_bytes, inp, idx, out, nt5)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ll.ll_convert(plan, src, dst, nt1)
        ll.ll_gather(lay5, c5.axis, c5.elem_bytes, inp, idx, out, nt5)
    for rep in range(4):
        new_src = c1.gen_data(rep, nt1)
        new_inp, new_idx = c5.gen_data(rep, nt5), c5.gen_idx(rep, nt5)
        src.copy_(new_src.cuda())
        inp.copy_(new_inp.cuda())
        idx.copy_(new_idx.cuda())
        dst.zero_()
        out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(wl.to_numpy_bits(dst), oracle.convert(c1.src_bases, c1.dst_bases, wl.to_numpy_bits(new_src))), rep
        assert np.array_equal(wl.to_numpy_bits(out), oracle.gather(c5.src_bases, c5.out_dim_bits, c5.axis,
                                                                   wl.to_numpy_bits(new_inp), new_idx.numpy())), rep


def test_large_lds_gathers_can_be_captured_in_a_hip_graph():
    """The gather kernels that ask for more than 64 KiB of LDS (a 64 KiB closed block plus tables; the
    128 KiB chunks of the chunk-walking kernel) set a function attribute before every launch: that
    must be harmless under stream capture.  Two tiles each, replayed with new inputs, against
    torch.gather on the logical view."""
    d = 18
    staged = ll.distributed_layout(4, 6, 8, [9, 9], [1 << k for k in range(d)])
    walked = ll.distributed_layout(4, 6, 8, [13, 5], [1 << k for k in range(d)])
    assert ll.ll_gather_info(staged, 0, 2)["kernel_name"] == "block_staged"
    assert ll.ll_gather_info(walked, 0, 2)["kernel_name"] == "lds_phased"
    nt = 2
    inp = torch.zeros(nt << d, dtype=torch.int16, device="cuda")
    idx_s = torch.zeros(nt << d, dtype=torch.int32, device="cuda")
    idx_w = torch.zeros(nt << d, dtype=torch.int32, device="cuda")
    out_s, out_w = torch.zeros_like(inp), torch.zeros_like(inp)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up outside capture
        ll.ll_gather(staged, 0, 2, inp, idx_s, out_s, nt)
        ll.ll_gather(walked, 0, 2, inp, idx_w, out_w, nt)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ll.ll_gather(staged, 0, 2, inp, idx_s, out_s, nt)
        ll.ll_gather(walked, 0, 2, inp, idx_w, out_w, nt)
    gen = torch.Generator(device="cpu").manual_seed(77)
    for rep in range(3):
        inp.copy_(torch.randint(-2**15, 2**15 - 1, (nt << d,), dtype=torch.int16, generator=gen).cuda())
        idx_s.copy_(torch.randint(0, 512, (nt << d,), dtype=torch.int32, generator=gen).cuda())
        idx_w.copy_(torch.randint(0, 8192, (nt << d,), dtype=torch.int32, generator=gen).cuda())
        out_s.zero_()
        out_w.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_s.view(nt, 512, 512), torch.gather(inp.view(nt, 512, 512), 1, idx_s.view(nt, 512, 512).long())), rep
        assert torch.equal(out_w.view(nt, 8192, 32), torch.gather(inp.view(nt, 8192, 32), 1, idx_w.view(nt, 8192, 32).long())), rep


def test_layouts_with_a_tile_label():
    """A `tile` input dim passes through conversions untouched (the tile index is the workgroup
    dimension) and may not lie on a gather axis; everything else behaves as without it."""
    rng = np.random.default_rng(123)
    d_in, nt_bits = 10, 2
    d = d_in + nt_bits
    ca = [1 << int(p) for p in rng.permutation(d_in)] + [1 << (d_in + k) for k in range(nt_bits)]
    cb = [1 << int(p) for p in rng.permutation(d_in)] + [1 << (d_in + k) for k in range(nt_bits)]
    dims = [(ll.LL_IN_REG, 2), (ll.LL_IN_LANE, 6), (ll.LL_IN_WAVE, 2), (ll.LL_IN_TILE, nt_bits)]
    a, b = ll.ll_layout_create(dims, [2, 5, 5], ca), ll.ll_layout_create(dims, [2, 5, 5], cb)
    for w in (2, 4):
        plan = ll.ll_plan_convert(a, b, w)
        src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=6 << d, dtype=NP_DTYPES[w])
        assert np.array_equal(run_convert(plan, src, d), oracle.convert(ca, cb, src))
    inp = rng.integers(0, 1 << 32, size=3 << d, dtype=np.uint32)
    for axis in (1, 2):
        idx = rng.integers(0, 32, size=3 << d, dtype=np.int32)
        got = run_gather(a, axis, inp, idx, d)
        assert np.array_equal(got, oracle.gather(ca, [2, 5, 5], axis, inp, idx))
    with pytest.raises(ll.LLError) as e:
        run_gather(a, 0, inp, np.zeros(3 << d, dtype=np.int32), d)          # dim 0 is the tile dim
    assert e.value.status == ll.LL_ERR_TILE_MIXED


@pytest.mark.parametrize("w", [1, 2, 4, 8])
def test_convert_tiny_broadcast_tiles(w):
    """Broadcasting conversions of tiles of 2 .. 64 slots (bundled into blocks), ragged tile counts."""
    rng = np.random.default_rng(800 + w)
    for dl in range(1, 6):
        for extra_a, extra_b in ((0, 2), (2, 0), (1, 3), (3, 1)):
            da, db = dl + extra_a, dl + extra_b
            ca, cb = surjective_bases(rng, da, dl), surjective_bases(rng, db, dl)
            plan = ll.ll_plan_convert(ll.ll_layout_create([(ll.LL_IN_REG, da)], [dl], ca),
                                      ll.ll_layout_create([(ll.LL_IN_REG, db)], [dl], cb), w)
            assert plan.info()["strategy_name"] == "lds_pull"
            per16 = max(1, 16 // (w << min(da, db)))
            for ntiles in (per16, 37 * per16):
                src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=ntiles << da, dtype=NP_DTYPES[w])
                got = run_convert_general(plan, src, da, db)
                assert np.array_equal(got, oracle.convert_general(ca, cb, dl, src)), (dl, da, db, ntiles)


@pytest.mark.parametrize("w", [1, 2, 4, 8])
def test_convert_broadcast_affine_layouts(w):
    """Broadcasting and affine at once: the pull map carries a constant, whose low bits move elements
    inside the staged source vectors."""
    rng = np.random.default_rng(950 + w)
    for da, db, dl in [(9, 8, 8), (8, 10, 8), (12, 12, 10), (13, 11, 11), (7, 9, 6)]:
        for trial in range(2):
            ca, cb = surjective_bases(rng, da, dl), surjective_bases(rng, db, dl)
            oa, ob = int(rng.integers(0, 1 << dl)), int(rng.integers(0, 1 << dl))
            a = ll.ll_layout_with_offset(ll.ll_layout_create([(ll.LL_IN_REG, 2), (ll.LL_IN_LANE, da - 2)], [dl], ca), oa)
            b = ll.ll_layout_with_offset(ll.ll_layout_create([(ll.LL_IN_REG, 2), (ll.LL_IN_LANE, db - 2)], [dl], cb), ob)
            ntiles = int(rng.integers(1, 30))
            src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=ntiles << da, dtype=NP_DTYPES[w])
            want = oracle.convert_general_affine(ca, oa, cb, ob, dl, src)
            for opts in PULL_OPTION_SETS:
                plan = ll.ll_plan_convert(a, b, w, opts() if opts else None)
                got = run_convert_general(plan, src, da, db)
                assert np.array_equal(got, want), (da, db, trial, plan.info()["threads"])


def test_gather_along_an_axis_of_one_element():
    """A logical dim of size 1 as the gather axis: every index wraps to 0 and the output equals the input,
    through the wave kernels and through the workgroup-staged one (narrow lanes)."""
    rng = np.random.default_rng(11)
    for nreg, w in ((2, 4), (0, 4), (1, 2)):
        d = nreg + 6 + 2
        bases = [1 << k for k in range(d)]
        layout = ll.distributed_layout(nreg, 6, 2, [0, d], bases)
        inp = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=5 << d, dtype=NP_DTYPES[w])
        idx = rng.integers(-5, 5, size=5 << d, dtype=np.int32)
        got = run_gather(layout, 0, inp, idx, d)
        assert np.array_equal(got, inp) and np.array_equal(got, oracle.gather(bases, [0, d], 0, inp, idx))


# ---------------------------------------------------------------------------------------------
# Sliced layouts (Sec. 4.3): the result of a reduction, converted to compact and to other slices
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("w", [1, 2, 4, 8])
def test_convert_sliced_layouts(w):
    """A 2-D and a 3-D blocked tensor reduced along each dim: the slice built by the library must
    equal the oracle's, and its data must convert into a compact blocked layout of what is left,
    and into the slice of a differently blocked parent."""
    parents = [
        ([1, 2], [3, 3], [1, 1], [1, 0]),             # 32 x 64, rows fastest within lanes
        ([2, 1], [2, 4], [0, 2], [0, 1]),             # 16 x 128
        ([1, 1, 1], [2, 2, 2], [1, 0, 1], [2, 0, 1]),  # 16 x 8 x 16
    ]
    others = [
        ([2, 1], [3, 3], [0, 2], [0, 1]),
        ([1, 2], [2, 4], [1, 1], [1, 0]),
        ([0, 2, 1], [3, 1, 2], [1, 0, 1], [1, 2, 0]),
    ]
    rng = np.random.default_rng(8800 + w)
    for (r, t, wv, order), (r2, t2, wv2, order2) in zip(parents, others):
        parent = ll.ll_layout_blocked(r, t, wv, order)
        oparent = oracle.blocked_layout(r, t, wv, order)
        other = ll.ll_layout_blocked(r2, t2, wv2, order2)
        oother = oracle.blocked_layout(r2, t2, wv2, order2)
        assert oparent.out_dims == oother.out_dims
        d_in = oparent.d_in
        for dim in range(len(order)):
            s, os_ = ll.ll_layout_slice(parent, dim), oracle.slice_layout(oparent, dim)
            assert s.bases == os_.bases and s.out_dims == os_.out_dims
            rest = os_.out_dims
            dl = sum(rest)
            # compact destination: every remaining element once, 2 registers, then lanes, then waves
            nl = min(6, dl - 1)
            compact = ll.ll_layout_create([(ll.LL_IN_REG, 1), (ll.LL_IN_LANE, nl), (ll.LL_IN_WAVE, dl - 1 - nl)],
                                          rest, [1 << k for k in range(dl)])
            ntiles = int(rng.integers(1, 9)) * 16
            src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=ntiles << d_in, dtype=NP_DTYPES[w])
            plan = ll.ll_plan_convert(s, compact, w)
            assert plan.info()["kind_name"] == "broadcast"
            got = run_convert_general(plan, src, d_in, dl)
            assert np.array_equal(got, oracle.convert_general(os_.bases, [1 << k for k in range(dl)], dl, src)), (order, dim)
            # slice of another blocking of the same tensor
            s2, os2 = ll.ll_layout_slice(other, dim), oracle.slice_layout(oother, dim)
            assert s2.bases == os2.bases
            plan = ll.ll_plan_convert(s, s2, w)
            got = run_convert_general(plan, src, d_in, oother.d_in)
            assert np.array_equal(got, oracle.convert_general(os_.bases, os2.bases, dl, src)), (order, dim, "slice")


@pytest.mark.parametrize("w", [1, 2, 4, 8])
def test_convert_between_different_register_lane_wave_splits(w):
    """Bijective layouts of one tile that split its 2^d slots differently over registers, lanes and
    waves: the images are flat per tile, so the conversion is B^-1 o A on flat indices."""
    rng = np.random.default_rng(9100 + w)
    for d, (ra, la, wa), (rb, lb, wb) in [(10, (2, 6, 2), (4, 6, 0)), (12, (3, 6, 3), (5, 5, 2)), (9, (0, 6, 3), (3, 6, 0))]:
        ca, cb = random_invertible(rng, d), random_invertible(rng, d)
        a = ll.distributed_layout(ra, la, wa, [d], ca)
        b = ll.distributed_layout(rb, lb, wb, [d], cb)
        plan = ll.ll_plan_convert(a, b, w)
        ntiles = int(rng.integers(1, 20))
        src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=ntiles << d, dtype=NP_DTYPES[w])
        assert np.array_equal(run_convert(plan, src, d), oracle.convert(ca, cb, src))
    # blocked layouts of a 64 x 64 tile with 4 and with 16 registers per lane
    a = ll.ll_layout_blocked([0, 2], [3, 3], [3, 1], [1, 0])
    b = ll.ll_layout_blocked([2, 2], [2, 4], [2, 0], [0, 1])
    oa, ob = oracle.blocked_layout([0, 2], [3, 3], [3, 1], [1, 0]), oracle.blocked_layout([2, 2], [2, 4], [2, 0], [0, 1])
    plan = ll.ll_plan_convert(a, b, w)
    src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=7 << 12, dtype=NP_DTYPES[w])
    assert np.array_equal(run_convert(plan, src, 12), oracle.convert(oa.bases, ob.bases, src))


@pytest.mark.parametrize("w", [1, 2, 4, 8])
def test_gather_along_axes_larger_than_lds(w):
    """Axes whose aligned block exceeds what LDS stages (128 KiB) are walked through LDS in chunks
    (up to 1 MiB) or gathered straight from memory; blocks of 64 and 128 KiB are staged by
    1024-thread workgroups.  Random XOR layouts on tiles of 64, 128, 256 KiB and 2 MiB and of 2^18
    elements (every axis then reaches the top bits), a ragged number of tiles, and a permutation
    layout whose axis 0 is exactly the wave bits of a 2^17-element tile."""
    rng = np.random.default_rng(9300 + w)
    d128 = 17 - {1: 0, 2: 1, 4: 2, 8: 3}[w]                          # a tile of 128 KiB
    cases = [(d128 - 1, [d128 - 1]), (d128, [d128 // 2, d128 - d128 // 2]), (d128 + 1, [d128 + 1]), (18, [6, 6, 6]),
             (d128 + 4, [d128 + 4])]
    seen = set()
    for d, dims in cases:
        nreg, nlane = 4, 6
        cols = random_invertible(rng, d)
        layout = ll.distributed_layout(nreg, nlane, d - 10, dims, cols)
        for axis in range(len(dims)):
            info = ll.ll_gather_info(layout, axis, w)
            seen.add(info["kernel_name"])
            ntiles = int(rng.integers(1, 4))
            inp = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=ntiles << d, dtype=NP_DTYPES[w])
            idx = rng.integers(0, 1 << dims[axis], size=ntiles << d, dtype=np.int32)
            idx[::5] -= 1 << dims[axis]
            got = run_gather(layout, axis, inp, idx, d)
            assert np.array_equal(got, oracle.gather(cols, dims, axis, inp, idx)), (d, dims, axis, info)
    assert {"global", "lds_phased", "block_staged"} <= seen
    d, dims = 17, [7, 10]
    cols = [1 << k for k in range(10)] + [1 << (10 + k) for k in range(7)]     # rows = the 7 wave bits
    layout = ll.distributed_layout(4, 6, 7, dims, cols)
    # closed under the 7 wave bits with 128-byte runs: 2^7 rows of runs, far smaller than the aligned range
    assert ll.ll_gather_info(layout, 0, w)["block_bytes"] == 128 * 128
    inp = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=3 << d, dtype=NP_DTYPES[w])
    idx = rng.integers(0, 1 << 7, size=3 << d, dtype=np.int32)
    assert np.array_equal(run_gather(layout, 0, inp, idx, d), oracle.gather(cols, dims, 0, inp, idx))


# ---------------------------------------------------------------------------------------------
# Gather under broadcasting layouts (Sec. 5.5 with Sec. 5.1): replicas receive and supply data
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("w", [1, 2, 4, 8])
def test_gather_under_broadcasting_layouts(w):
    """Random surjective layouts with zero and dependent columns, every axis; `in` is the image of a
    logical tensor (equal replicas: what the gather is defined on), replicas of `idx` deliberately
    unequal (every slot of out follows its own index); a sliced blocked layout; an affine constant
    on top."""
    rng = np.random.default_rng(9500 + w)
    seen = set()
    for d_in, dims, nreg in [(10, [4, 4], 2), (12, [3, 6], 4), (13, [5, 2, 3], 3), (9, [7], 2), (16, [6, 7], 4)]:
        d_out = sum(dims)
        cols = surjective_bases(rng, d_in, d_out)
        nlane = min(6, d_in - nreg)
        layout = ll.ll_layout_create([(ll.LL_IN_REG, nreg), (ll.LL_IN_LANE, nlane), (ll.LL_IN_WAVE, d_in - nreg - nlane)], dims, cols)
        off = int(rng.integers(0, 1 << d_out))
        for axis in range(len(dims)):
            for lay, o in ((layout, 0), (ll.ll_layout_with_offset(layout, off), off)):
                seen.add(ll.ll_gather_info(lay, axis, w)["kernel_name"])
                ntiles = int(rng.integers(1, 6)) * 16
                inp = oracle.consistent_image(cols, d_out, rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=ntiles << d_in, dtype=NP_DTYPES[w]))
                idx = rng.integers(-(1 << dims[axis]), 1 << dims[axis], size=ntiles << d_in, dtype=np.int32)
                got = run_gather(lay, axis, inp, idx, d_in)
                assert np.array_equal(got, oracle.gather_general(cols, dims, axis, inp, idx, o)), (d_in, dims, axis, o)
    # the result of a reduction: a 64 x 64 blocked tile sliced along its rows, gathered along what is left
    parent = ll.ll_layout_blocked([1, 2], [3, 3], [2, 1], [1, 0])
    s = ll.ll_layout_slice(parent, 0)
    os_ = oracle.slice_layout(oracle.blocked_layout([1, 2], [3, 3], [2, 1], [1, 0]), 0)
    assert s.bases == os_.bases
    for opts in (None, ll.ll_options_init(gather_kernel=ll.LL_GATHER_BLOCK_STAGED)):
        seen.add(ll.ll_gather_info(s, 0, w, opts)["kernel_name"])
        inp = oracle.consistent_image(os_.bases, 6, rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=32 << 12, dtype=NP_DTYPES[w]))
        idx = rng.integers(0, 64, size=32 << 12, dtype=np.int32)
        assert np.array_equal(run_gather(s, 0, inp, idx, 12, opts), oracle.gather_general(os_.bases, [6], 0, inp, idx))
    assert "block_staged" in seen


@pytest.mark.parametrize("w", [1, 2, 4, 8])
def test_gather_through_lds_chunks_broadcasting_and_affine(w):
    """The chunk-walking kernel (aligned range of 256 KiB to 1 MiB that no closed block with long runs
    covers) under random XOR layouts that broadcast (one slot bit more than logical bits; `in` the
    image of a logical tensor, replicas of `idx` unequal) and carry an affine constant, indices partly
    out of range (they wrap)."""
    rng = np.random.default_rng(9900 + w)
    wl2 = {1: 0, 2: 1, 4: 2, 8: 3}[w]
    seen = set()
    for range_bytes_log2 in (18, 19, 20):
        d_in = range_bytes_log2 - wl2                 # slots per tile: the tile is the aligned range
        d_out = d_in - 1
        dims = [d_out - 3, 3]
        cols = surjective_bases(rng, d_in, d_out)
        layout = ll.ll_layout_create([(ll.LL_IN_REG, 4), (ll.LL_IN_LANE, 6), (ll.LL_IN_WAVE, d_in - 10)], dims, cols)
        off = int(rng.integers(1, 1 << d_out))
        for lay, o in ((layout, 0), (ll.ll_layout_with_offset(layout, off), off)):
            info = ll.ll_gather_info(lay, 0, w)
            seen.add(info["kernel_name"])
            ntiles = 3
            inp = oracle.consistent_image(cols, d_out, rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=ntiles << d_in, dtype=NP_DTYPES[w]))
            idx = rng.integers(-(1 << dims[0]), 1 << dims[0], size=ntiles << d_in, dtype=np.int32)
            got = run_gather(lay, 0, inp, idx, d_in)
            assert np.array_equal(got, oracle.gather_general(cols, dims, 0, inp, idx, o)), (d_in, dims, o, info)
    assert "lds_phased" in seen


@pytest.mark.parametrize("w", [1, 2, 4, 8])
def test_gather_on_memory_layouts(w):
    """in, idx and out as buffers indexed by memory offset: a row-major tensor (the identity memory
    layout) against torch.gather on the logical view, and an mma-swizzled buffer against the oracle."""
    rng = np.random.default_rng(9800 + w)
    shape = (5, 64, 128)
    ident = ll.ll_layout_create([(ll.LL_IN_OFFSET, 13)], [6, 7], [1 << k for k in range(13)])
    tdt = {1: torch.uint8, 2: torch.int16, 4: torch.int32, 8: torch.int64}[w]
    for axis in (0, 1):
        assert ll.ll_gather_info(ident, axis, w)["paper_rounds"] == 0
        x = torch.from_numpy(rng.integers(0, 127, size=shape).astype(NP_DTYPES[w]).view({1: np.uint8, 2: np.int16, 4: np.int32, 8: np.int64}[w])).cuda()
        idx = torch.from_numpy(rng.integers(0, shape[1 + axis], size=shape).astype(np.int32)).cuda()
        out = torch.full_like(x, 0x5A)
        ll.ll_gather(ident, axis, w, x, idx, out, shape[0])
        torch.cuda.synchronize()
        assert torch.equal(out, torch.gather(x, 1 + axis, idx.to(torch.int64))), axis
    sw = ll.ll_layout_mma_swizzle(6, 6, 8 // w if w < 8 else 1, 1, 8)
    osw = oracle.mma_swizzle_layout(6, 6, 8 // w if w < 8 else 1, 1, 8)
    assert sw.bases == osw.bases
    inp = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=6 << 12, dtype=NP_DTYPES[w])
    for axis in (0, 1):
        idx = rng.integers(0, 64, size=6 << 12, dtype=np.int32)
        assert np.array_equal(run_gather(sw, axis, inp, idx, 12), oracle.gather(osw.bases, [6, 6], axis, inp, idx)), axis


def test_binding_rejects_short_and_strided_gpu_tensors():
    cfg = wl.config(2)
    a, b = layouts_of(cfg)
    plan = ll.ll_plan_convert(a, b, cfg.elem_bytes)
    src = cfg.gen_data(0, 2, "cuda")
    with pytest.raises(ll.LLError) as e:
        ll.ll_convert(plan, src, torch.empty(src.numel() - 8, dtype=src.dtype, device="cuda"), 2)
    assert e.value.status == ll.LL_ERR_INVALID_ARG and "dst holds" in e.value.message
    with pytest.raises(ll.LLError) as e:
        ll.ll_convert(plan, torch.empty(2 * src.numel(), dtype=src.dtype, device="cuda")[::2], torch.empty_like(src), 2)
    assert e.value.status == ll.LL_ERR_INVALID_ARG and "contiguous" in e.value.message
    with pytest.raises(ll.LLError) as e:
        ll.ll_gather(a, 0, 2, src, torch.zeros(src.numel(), dtype=torch.int64, device="cuda"), torch.empty_like(src), 2)
    assert e.value.status == ll.LL_ERR_INVALID_ARG and "32-bit" in e.value.message


def test_entry_points_from_several_threads_and_streams():
    """Plans and layouts are immutable and the library keeps no global launch state: four host threads,
    each with its own stream, convert and gather concurrently through the same plan and layout."""
    import threading
    cfg, g = wl.config(2), wl.config(5)
    a, b = layouts_of(cfg)
    plan = ll.ll_plan_convert(a, b, cfg.elem_bytes)
    lay5, _ = layouts_of(g)
    nt = 64
    src = cfg.gen_data(0, nt, "cuda")
    inp, idx = g.gen_data(0, nt, "cuda"), g.gen_idx(0, nt, "cuda")
    want_c = oracle.convert(cfg.src_bases, cfg.dst_bases, wl.to_numpy_bits(src))
    want_g = oracle.gather(g.src_bases, g.out_dim_bits, g.axis, wl.to_numpy_bits(inp), idx.cpu().numpy())
    torch.cuda.synchronize()
    errors = []

    def work(k):
        try:
            stream = torch.cuda.Stream()
            outs_c = [torch.empty_like(src) for _ in range(4)]
            outs_g = [torch.empty_like(inp) for _ in range(4)]
            for rep in range(25):
                ll.ll_convert(plan, src, outs_c[rep % 4], nt, stream=stream)
                ll.ll_gather(lay5, g.axis, g.elem_bytes, inp, idx, outs_g[rep % 4], nt, stream=stream)
            stream.synchronize()
            for o in outs_c:
                assert np.array_equal(wl.to_numpy_bits(o), want_c)
            for o in outs_g:
                assert np.array_equal(wl.to_numpy_bits(o), want_g)
        except Exception as e:  # noqa: BLE001  (reported to the main thread)
            errors.append((k, repr(e)))

    threads = [threading.Thread(target=work, args=(k,)) for k in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors


@pytest.mark.parametrize("w", [1, 2, 4, 8])
def test_degenerate_layouts(w):
    """The smallest cases the method has: a scalar replicated over the slots of a tile (no logical bits
    at all), a two-element tile, and tiles of a single element under gather."""
    rng = np.random.default_rng(9900 + w)
    n = 64
    # a scalar held 8 times -> held 4 times: every destination slot copies source slot 0 of its tile
    a = ll.ll_layout_create([(ll.LL_IN_REG, 2), (ll.LL_IN_WAVE, 1)], [0], [0, 0, 0])
    b = ll.ll_layout_create([(ll.LL_IN_REG, 2)], [0], [0, 0])
    src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=n << 3, dtype=NP_DTYPES[w])
    got = run_convert_general(ll.ll_plan_convert(a, b, w), src, 3, 2)
    assert np.array_equal(got, oracle.convert_general([0, 0, 0], [0, 0], 0, src))
    assert np.array_equal(got.reshape(n, 4), np.repeat(src.reshape(n, 8)[:, :1], 4, axis=1))
    # two elements per tile, swapped
    two, swp = ll.ll_layout_create([(ll.LL_IN_REG, 1)], [1], [1]), ll.ll_layout_with_offset(ll.ll_layout_create([(ll.LL_IN_REG, 1)], [1], [1]), 1)
    src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=n << 1, dtype=NP_DTYPES[w])
    got = run_convert(ll.ll_plan_convert(two, swp, w), src, 1)
    assert np.array_equal(got.reshape(n, 2), src.reshape(n, 2)[:, ::-1])
    # gather on two-element tiles and on single-element tiles (an axis of one element: identity)
    idx = rng.integers(0, 2, size=n << 1, dtype=np.int32)
    assert np.array_equal(run_gather(two, 0, src, idx, 1), oracle.gather([1], [1], 0, src, idx))
    one = ll.ll_layout_create([(ll.LL_IN_REG, 0)], [0], [])
    src = rng.integers(0, np.iinfo(NP_DTYPES[w]).max, size=n, dtype=NP_DTYPES[w])
    idx = rng.integers(-5, 5, size=n, dtype=np.int32)
    assert np.array_equal(run_gather(one, 0, src, idx, 0), src)
