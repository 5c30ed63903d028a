"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times: EVERY tile
of every image is compared with the oracle, bit for bit.  The oracle's table variants (the per-tile
map tabulated once, tiles on all host threads; pinned against the plain definitions in
tests/test_oracle_pins.py) make that a matter of seconds; images come back from the device in
chunks of whole tiles."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

import paper_2505_23819_amd as ll  # noqa: E402  (a missing library must fail loudly, not skip)


CHUNK_BYTES = 256 << 20


def chunks_of_tiles(ntiles, tile_bytes):
    step = max(1, CHUNK_BYTES // tile_bytes)
    for t0 in range(0, ntiles, step):
        yield t0, min(step, ntiles - t0)


def assert_convert_all_tiles(src, dst, ntiles, src_bases, dst_bases, what, d_out=None):
    """dst == oracle(src) for every tile.  d_out given: layouts that broadcast (images of different sizes)."""
    ts, td = 1 << len(src_bases), 1 << len(dst_bases)
    for t0, n in chunks_of_tiles(ntiles, max(ts, td) * src.element_size()):
        s = wl.to_numpy_bits(src[t0 * ts:(t0 + n) * ts])
        if d_out is None:
            want, _ = oracle.convert(src_bases, dst_bases, s, table=True)
        else:
            want = oracle.convert_general(src_bases, dst_bases, d_out, s, table=True)
        got = wl.to_numpy_bits(dst[t0 * td:(t0 + n) * td])
        if not np.array_equal(got, want):
            bad = np.flatnonzero(got != want)
            raise AssertionError(f"{what}: {bad.size} elements differ in tiles {t0}..{t0 + n - 1}, first at tile {t0 + int(bad[0]) // td} slot {int(bad[0]) % td}")


def assert_gather_all_tiles(inp, idx, out, ntiles, bases, dims, axis, what):
    te = 1 << len(bases)
    for t0, n in chunks_of_tiles(ntiles, te * 4):
        want = oracle.gather(bases, dims, axis, wl.to_numpy_bits(inp[t0 * te:(t0 + n) * te]), idx[t0 * te:(t0 + n) * te].cpu().numpy(), table=True)
        got = wl.to_numpy_bits(out[t0 * te:(t0 + n) * te])
        if not np.array_equal(got, want):
            bad = np.flatnonzero(got != want)
            raise AssertionError(f"{what}: {bad.size} elements differ in tiles {t0}..{t0 + n - 1}, first at tile {t0 + int(bad[0]) // te} slot {int(bad[0]) % te}")


def sample_tiles(ntiles, count, seed):
    rng = np.random.default_rng(seed)
    picks = {0, ntiles - 1, ntiles // 2}
    while len(picks) < min(count, ntiles):
        picks.add(int(rng.integers(0, ntiles)))
    return sorted(picks)


@pytest.mark.parametrize("cid", [1, 2, 3, 4])
def test_convert_full_size_every_tile(cid):
    cfg = wl.config(cid)
    a = ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.src_bases)
    b = ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.dst_bases)
    plan = ll.ll_plan_convert(a, b, cfg.elem_bytes)
    src = cfg.gen_data(0, cfg.ntiles, "cuda")
    dst = torch.empty_like(src)
    wl.bits_view(dst).fill_(0x5A5A)
    ll.ll_convert(plan, src, dst, cfg.ntiles)
    torch.cuda.synchronize()
    te = cfg.tile_elems
    # the input on the device is what the seeded generator produces on the host too
    if cfg.data_recipe != "normal":
        for t in sample_tiles(cfg.ntiles, 6, cid):
            assert np.array_equal(wl.to_numpy_bits(src[t * te:(t + 1) * te]), wl.to_numpy_bits(cfg.gen_data(t, 1)))
    assert_convert_all_tiles(src, dst, cfg.ntiles, cfg.src_bases, cfg.dst_bases, f"config {cid}")
    # the plain (bit by bit) definition on a few tiles as well
    for t in sample_tiles(cfg.ntiles, 3, 10 + cid):
        want = oracle.convert(cfg.src_bases, cfg.dst_bases, wl.to_numpy_bits(src[t * te:(t + 1) * te]))
        assert np.array_equal(wl.to_numpy_bits(dst[t * te:(t + 1) * te]), want), f"config {cid} tile {t}"


@pytest.mark.parametrize("kernel", [None, "shuffle", "shuffle_rows", "block_staged"])
def test_gather_full_size_every_tile(kernel):
    """Config 5 with the library's choice (wave-private LDS staging) and with each other applicable kernel."""
    cfg = wl.config(5)
    layout = ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.src_bases)
    opts = None if kernel is None else ll.ll_options_init(gather_kernel=ll.GATHER_KERNEL_NAMES.index(kernel))
    assert ll.ll_gather_info(layout, cfg.axis, cfg.elem_bytes, opts)["kernel_name"] == (kernel or "wave_staged")
    inp = cfg.gen_data(0, cfg.ntiles, "cuda")
    idx = cfg.gen_idx(0, cfg.ntiles, "cuda")
    out = torch.empty_like(inp)
    wl.bits_view(out).fill_(0x5A5A)
    ll.ll_gather(layout, cfg.axis, cfg.elem_bytes, inp, idx, out, cfg.ntiles, opts=opts)
    torch.cuda.synchronize()
    te = cfg.tile_elems
    for t in sample_tiles(cfg.ntiles, 6, 5):
        assert np.array_equal(wl.to_numpy_bits(inp[t * te:(t + 1) * te]), wl.to_numpy_bits(cfg.gen_data(t, 1)))
        assert np.array_equal(idx[t * te:(t + 1) * te].cpu().numpy(), cfg.gen_idx(t, 1).numpy())
    assert_gather_all_tiles(inp, idx, out, cfg.ntiles, cfg.src_bases, cfg.out_dim_bits, cfg.axis, f"config 5 ({kernel})")
    for t in sample_tiles(cfg.ntiles, 2, 15):             # the plain definition on a few tiles as well
        want = oracle.gather(cfg.src_bases, cfg.out_dim_bits, cfg.axis, wl.to_numpy_bits(inp[t * te:(t + 1) * te]), idx[t * te:(t + 1) * te].cpu().numpy())
        assert np.array_equal(wl.to_numpy_bits(out[t * te:(t + 1) * te]), want), f"tile {t}"


def test_gather_both_kernels_agree():
    """The shuffle kernels (one ds_bpermute_b32 per element; a lane's row as it lies in memory, or
    coalesced pieces and lane <-> register butterflies) and the staged kernel on config 5, with one,
    two and four waves per workgroup."""
    cfg = wl.config(5)
    layout = ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.src_bases)
    nt = 37
    inp, idx = cfg.gen_data(0, nt, "cuda"), cfg.gen_idx(0, nt, "cuda")
    want = oracle.gather(cfg.src_bases, cfg.out_dim_bits, cfg.axis, wl.to_numpy_bits(inp), idx.cpu().numpy())
    for staged in (ll.LL_GATHER_SHUFFLE, ll.LL_GATHER_WAVE_STAGED, ll.LL_GATHER_SHUFFLE_ROWS):
        for waves in (-1, 1, 2, 4):
            opts = ll.ll_options_init(gather_kernel=staged, gather_waves=waves)
            assert ll.ll_gather_info(layout, cfg.axis, cfg.elem_bytes, opts)["kernel"] == staged
            out = torch.zeros_like(inp)
            ll.ll_gather(layout, cfg.axis, cfg.elem_bytes, inp, idx, out, nt, opts=opts)
            torch.cuda.synchronize()
            assert np.array_equal(wl.to_numpy_bits(out), want), f"kernel={staged} waves={waves}"


@pytest.mark.parametrize("case", wl.broadcast_cases(), ids=lambda c: c.name.split(" (")[0].replace(" ", "_"))
def test_broadcast_convert_full_size_every_tile(case):
    """Conversions between replicating layouts at the sizes bench.py times (source replicas hold
    different values, so reading a replica other than the canonical one fails)."""
    a = ll.distributed_layout(*case.src_in, case.out_dim_bits, case.src_bases)
    b = ll.distributed_layout(*case.dst_in, case.out_dim_bits, case.dst_bases)
    plan = ll.ll_plan_convert(a, b, case.elem_bytes)
    nt, ds, dd = case.ntiles, case.d_src, case.d_dst
    src = case.gen_data(0, nt, "cuda")
    dst = torch.empty(nt << dd, dtype=src.dtype, device="cuda")
    wl.bits_view(dst).fill_(0x5A5A)
    ll.ll_convert(plan, src, dst, nt)
    torch.cuda.synchronize()
    for t in sample_tiles(nt, 4, case.data_seed):
        assert np.array_equal(wl.to_numpy_bits(src[t << ds:(t + 1) << ds]), wl.to_numpy_bits(case.gen_data(t, 1)))
    assert_convert_all_tiles(src, dst, nt, case.src_bases, case.dst_bases, case.name, d_out=case.d_out)
    for t in sample_tiles(nt, 2, case.data_seed + 1):     # the plain definition on a few tiles as well
        want = oracle.convert_general(case.src_bases, case.dst_bases, case.d_out, wl.to_numpy_bits(src[t << ds:(t + 1) << ds]))
        assert np.array_equal(wl.to_numpy_bits(dst[t << dd:(t + 1) << dd]), want), f"{case.name} tile {t}"


@pytest.mark.parametrize("w,force", [(1, 6), (2, 6)])
def test_narrow_transpose_full_size_every_tile(w, force):
    """The 128 x 128 transpose with 1- and 2-byte elements through the transposing LDS loads, at the
    size bench.py times (256 MiB per side)."""
    cfg = wl.config(2)
    a = ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.src_bases)
    b = ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.dst_bases)
    plan = ll.ll_plan_convert(a, b, w, ll.ll_options_init(strategy=force))
    assert plan.info()["strategy_name"] == "lds_tr"
    te = cfg.tile_elems
    nt = (256 << 20) // (te * w)
    src = wl.raw_bits(21, 0, nt * te * w // 8, "cuda").view({1: torch.uint8, 2: torch.int16}[w])
    dst = torch.empty_like(src)
    ll.ll_convert(plan, src, dst, nt)
    torch.cuda.synchronize()
    assert_convert_all_tiles(src, dst, nt, cfg.src_bases, cfg.dst_bases, f"transpose, {w}-byte elements")


def test_gather_beyond_lds_full_size_every_tile():
    """A gather whose aligned axis block exceeds LDS, in the configuration bench.py times: 512 row-major
    512 x 512 tiles of two-byte elements, gather along the rows (staged as 512 rows x 128-byte runs)."""
    d, ntiles = 18, 512
    bases = [1 << k for k in range(d)]
    layout = ll.distributed_layout(4, 6, 8, [9, 9], bases)
    assert ll.ll_gather_info(layout, 0, 2)["block_bytes"] == 65536
    inp = wl.raw_bits(23, 0, (ntiles << d) * 2 // 8, "cuda").view(torch.int16)
    idx = wl.gen_index(53, 0, ntiles << d, 1 << 9, "cuda")
    out = torch.empty_like(inp)
    out.fill_(0x5A5A)
    ll.ll_gather(layout, 0, 2, inp, idx, out, ntiles)
    torch.cuda.synchronize()
    assert_gather_all_tiles(inp, idx, out, ntiles, bases, [9, 9], 0, "512 x 512 rows")
    # the layout is the identity, so the definition is also torch.gather on the logical view
    ref = torch.gather(inp.view(ntiles, 512, 512), 1, idx.view(ntiles, 512, 512).to(torch.int64))
    assert torch.equal(out.view(ntiles, 512, 512), ref)


@pytest.mark.parametrize("rows_bits,kernel", [(13, "lds_phased"), (14, "lds_phased"), (15, "global")])
def test_gather_beyond_lds_without_long_runs_full_size(rows_bits, kernel):
    """256 MiB of 8192 x 32 (16384 x 32, 32768 x 32) two-byte tiles gathered along the rows: no block
    closed under the rows fits LDS with runs of 64 bytes.  Aligned ranges of 512 KiB and 1 MiB are
    walked through LDS in chunks; the 2 MiB range is read from memory element by element.  Every tile
    against the oracle, and against torch.gather on the logical view."""
    d = rows_bits + 5
    ntiles = (256 << 20) // (2 << d)
    rows = 1 << rows_bits
    bases = [1 << k for k in range(d)]
    layout = ll.distributed_layout(4, 6, d - 10, [rows_bits, 5], bases)
    assert ll.ll_gather_info(layout, 0, 2)["kernel_name"] == kernel
    inp = wl.raw_bits(24, 0, (ntiles << d) * 2 // 8, "cuda").view(torch.int16)
    idx = wl.gen_index(54, 0, ntiles << d, rows, "cuda")
    out = torch.empty_like(inp)
    out.fill_(0x5A5A)
    ll.ll_gather(layout, 0, 2, inp, idx, out, ntiles)
    torch.cuda.synchronize()
    ref = torch.gather(inp.view(ntiles, rows, 32), 1, idx.view(ntiles, rows, 32).to(torch.int64))
    assert torch.equal(out.view(ntiles, rows, 32), ref)
    assert_gather_all_tiles(inp, idx, out, ntiles, bases, [rows_bits, 5], 0, f"{rows} x 32 rows")


def test_gather_short_runs_beyond_l2():
    """Rows of 4096 x 1024 four-byte row-major tiles (16 MiB each: beyond an XCD's L2): staged in 128 KiB
    blocks of 4096 rows x 32-byte runs.  Every tile against the oracle and against torch.gather."""
    d, ntiles = 22, 3
    bases = [1 << k for k in range(d)]
    layout = ll.ll_layout_create([(ll.LL_IN_OFFSET, d)], [12, 10], bases)
    info = ll.ll_gather_info(layout, 0, 4)
    assert info["kernel_name"] == "block_staged" and info["block_bytes"] == 128 * 1024
    inp = wl.raw_bits(25, 0, (ntiles << d) * 4 // 8, "cuda").view(torch.int32)
    idx = wl.gen_index(55, 0, ntiles << d, 1 << 12, "cuda")
    out = torch.empty_like(inp)
    out.fill_(0x5A5A5A5A)
    ll.ll_gather(layout, 0, 4, inp, idx, out, ntiles)
    torch.cuda.synchronize()
    ref = torch.gather(inp.view(ntiles, 4096, 1024), 1, idx.view(ntiles, 4096, 1024).to(torch.int64))
    assert torch.equal(out.view(ntiles, 4096, 1024), ref)
    assert_gather_all_tiles(inp, idx, out, ntiles, bases, [12, 10], 0, "4096 x 1024 rows")


@pytest.mark.parametrize("cid,force", [(1, None), (3, None), (4, None), (5, None), (2, 4), (2, 6)])
def test_buffers_beyond_four_gib(cid, force):
    """Images larger than 4 GiB (64-bit offsets in every kernel family: lane-register butterflies,
    register path, element-wide LDS staging, gather, and config 2 forced through the 128-bit LDS
    kernel and the transposing LDS loads), with a ragged tile count; every tile is compared with the
    oracle's table variant, tiles from both ends and around the 4 GiB mark with the plain one too."""
    opts = ll.ll_options_init(strategy=force) if force else None
    cfg = wl.config(cid)
    te, w = cfg.tile_elems, cfg.elem_bytes
    ntiles = (4 << 30) // (te * w) + 257 + 3
    step = max(1, (256 << 20) // (te * w))
    src = torch.empty(ntiles * te, dtype=cfg.dtype, device="cuda")
    for t0 in range(0, ntiles, step):
        n = min(step, ntiles - t0)
        src[t0 * te:(t0 + n) * te] = cfg.gen_data(t0, n, "cuda")
    dst = torch.empty_like(src)
    past = (4 << 30) // (te * w)
    picks = [0, 1, past - 1, past, past + 1, ntiles - 2, ntiles - 1]
    if cfg.kind == "gather":
        idx = torch.empty(ntiles * te, dtype=torch.int32, device="cuda")
        for t0 in range(0, ntiles, step):
            n = min(step, ntiles - t0)
            idx[t0 * te:(t0 + n) * te] = cfg.gen_idx(t0, n, "cuda")
        layout = ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.src_bases)
        ll.ll_gather(layout, cfg.axis, w, src, idx, dst, ntiles)
        torch.cuda.synchronize()
        assert_gather_all_tiles(src, idx, dst, ntiles, cfg.src_bases, cfg.out_dim_bits, cfg.axis, "config 5 beyond 4 GiB")
        for t in picks:
            want = oracle.gather(cfg.src_bases, cfg.out_dim_bits, cfg.axis, wl.to_numpy_bits(src[t * te:(t + 1) * te]),
                                 idx[t * te:(t + 1) * te].cpu().numpy())
            assert np.array_equal(wl.to_numpy_bits(dst[t * te:(t + 1) * te]), want), f"tile {t}"
        return
    a = ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.src_bases)
    b = ll.distributed_layout(cfg.nreg, cfg.nlane, cfg.nwave, cfg.out_dim_bits, cfg.dst_bases)
    plan = ll.ll_plan_convert(a, b, w, opts)
    want_kernel = {(1, None): "wave_shuffle", (3, None): "reg_permute", (4, None): "lds_elem", (2, 4): "lds_vec", (2, 6): "lds_tr"}
    assert plan.info()["strategy_name"] == want_kernel[(cid, force)]
    ll.ll_convert(plan, src, dst, ntiles)
    torch.cuda.synchronize()
    assert_convert_all_tiles(src, dst, ntiles, cfg.src_bases, cfg.dst_bases, f"config {cid} beyond 4 GiB")
    for t in picks:       # the plain definition at both ends and around the 4 GiB mark
        want = oracle.convert(cfg.src_bases, cfg.dst_bases, wl.to_numpy_bits(src[t * te:(t + 1) * te]))
        assert np.array_equal(wl.to_numpy_bits(dst[t * te:(t + 1) * te]), want), f"config {cid} tile {t}"


@pytest.mark.parametrize("which", [1, 0], ids=["destination", "source"])
def test_broadcast_images_beyond_four_gib(which):
    """The broadcasting kernel with a destination image past 4 GiB (expand 16x, 64 KiB per destination
    tile) and with a source image past 4 GiB (collapse 16x, 64 KiB per source tile)."""
    case = wl.broadcast_cases()[which]
    a = ll.distributed_layout(*case.src_in, case.out_dim_bits, case.src_bases)
    b = ll.distributed_layout(*case.dst_in, case.out_dim_bits, case.dst_bases)
    plan = ll.ll_plan_convert(a, b, case.elem_bytes)
    ts, td = 1 << case.d_src, 1 << case.d_dst
    past = (4 << 30) // (max(ts, td) * case.elem_bytes)
    ntiles = past + 1029
    src = case.gen_data(0, ntiles, "cuda")
    dst = torch.empty(ntiles * td, dtype=src.dtype, device="cuda")
    ll.ll_convert(plan, src, dst, ntiles)
    torch.cuda.synchronize()
    assert_convert_all_tiles(src, dst, ntiles, case.src_bases, case.dst_bases, case.name + " beyond 4 GiB", d_out=case.d_out)
    for t in (0, past - 1, past, past + 1, ntiles - 1):
        want = oracle.convert_general(case.src_bases, case.dst_bases, case.d_out, wl.to_numpy_bits(src[t * ts:(t + 1) * ts]))
        assert np.array_equal(wl.to_numpy_bits(dst[t * td:(t + 1) * td]), want), f"tile {t}"


@pytest.mark.parametrize("kernel", ["block_staged", "global", "lds_phased", "shuffle"])
def test_gather_general_kernels_beyond_four_gib(kernel):
    """The workgroup-staged, the memory-direct, the chunk-walking and the lane-shuffle gather with images past 4 GiB (4-byte
    elements, a ragged tile count): every tile against the oracle."""
    if kernel == "shuffle":
        bases, dims, axis, split = [1 << k for k in range(8)], [6, 2], 0, (2, 6, 0)
    elif kernel == "lds_phased":
        bases, dims, axis, split = [1 << k for k in range(17)], [13, 4], 0, (4, 6, 7)
    elif kernel == "block_staged":
        cfg = wl.config(5)
        bases, dims, axis, split = cfg.src_bases, cfg.out_dim_bits, 1, (cfg.nreg, cfg.nlane, cfg.nwave)
    else:
        bases, dims, axis, split = [1 << k for k in range(19)], [14, 5], 0, (4, 6, 9)
    layout = ll.distributed_layout(*split, dims, bases)
    assert ll.ll_gather_info(layout, axis, 4)["kernel_name"] == kernel
    d = sum(dims)
    te = 1 << d
    past = (4 << 30) // (te * 4)
    ntiles = past + 5
    n = ntiles * te
    inp = torch.empty(n, dtype=torch.int32, device="cuda")
    idx = torch.empty(n, dtype=torch.int32, device="cuda")
    step = 1 << 26
    for e0 in range(0, n, step):
        m = min(step, n - e0)
        inp[e0:e0 + m] = wl.raw_bits(26, e0 // 2, m // 2, "cuda").view(torch.int32)
        idx[e0:e0 + m] = wl.gen_index(56, e0, m, 1 << dims[axis], "cuda")
    out = torch.empty_like(inp)
    out.fill_(0x5A5A5A5A)
    ll.ll_gather(layout, axis, 4, inp, idx, out, ntiles)
    torch.cuda.synchronize()
    assert_gather_all_tiles(inp, idx, out, ntiles, bases, dims, axis, kernel + " beyond 4 GiB")
    for t in (0, past, ntiles - 1):
        want = oracle.gather(bases, dims, axis, inp[t * te:(t + 1) * te].cpu().numpy().view(np.uint32), idx[t * te:(t + 1) * te].cpu().numpy())
        assert np.array_equal(out[t * te:(t + 1) * te].cpu().numpy().view(np.uint32), want), f"tile {t}"
