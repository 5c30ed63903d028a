"""Randomized GPU parity sweep: conversions (bijective, re-split, affine, with a tile label), conversions
between broadcasting layouts, and gathers (any axis, broadcasting, affine) on randomly drawn layouts,
sizes, element widths and tile counts, each compared bit for bit with the CPU oracle.  Seeds are
fixed; a failure prints the tuple that regenerates its case."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu

import paper_2505_23819_amd as ll  # noqa: E402  (a missing library must fail loudly, not skip)

NP = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}
TD = {1: np.uint8, 2: np.int16, 4: np.int32, 8: np.int64}


def spans(cols, d_out):
    """True when the columns span all of F2^d_out (greedy XOR basis)."""
    basis = []
    for c in cols:
        x = c
        for b in basis:
            x = min(x, x ^ b)
        if x:
            basis.append(x)
    return len(basis) == d_out


def rand_cols(rng, d_in, d_out, kind):
    """Surjective columns: 0 arbitrary XOR combinations, 1 unit vectors and zeros (a distributed
    layout), 2 a few XORs on top of that."""
    while True:
        if kind == 0:
            cols = [int(rng.integers(0, 1 << d_out)) for _ in range(d_in)]
            if d_in > d_out and rng.integers(0, 2):
                cols[int(rng.integers(0, d_in))] = 0
        else:
            units = [1 << int(p) for p in rng.permutation(d_out)] + [0] * (d_in - d_out)
            cols = [units[int(i)] for i in rng.permutation(d_in)]
            if kind == 2:
                for _ in range(int(rng.integers(1, 4))):
                    i, j = (int(x) for x in rng.integers(0, d_in, size=2))
                    if i != j:
                        cols[i] ^= cols[j]
        if spans(cols, d_out):
            return cols


def split(rng, d):
    """Random (register, lane, wave, tile) bit counts with d bits in all."""
    nreg = int(rng.integers(0, min(6, d) + 1))
    nlane = min(6, d - nreg)
    if rng.integers(0, 4) == 0:
        nlane = int(rng.integers(0, nlane + 1))
    rest = d - nreg - nlane
    nwave = min(rest, int(rng.integers(0, 5)))
    ntile = rest - nwave
    if ntile and rng.integers(0, 2):
        nwave, ntile = nwave + ntile, 0
    return nreg, nlane, nwave, ntile


def mk(dims_in, out_dims, cols):
    labels = [(label, n) for label, n in zip((ll.LL_IN_REG, ll.LL_IN_LANE, ll.LL_IN_WAVE, ll.LL_IN_TILE), dims_in) if n > 0]
    return ll.ll_layout_create(labels or [(ll.LL_IN_REG, 0)], out_dims, cols)


def out_dims_of(rng, d):
    nd = int(rng.integers(1, 4))
    cuts = sorted(int(x) for x in rng.integers(0, d + 1, size=nd - 1))
    return [b - a for a, b in zip([0] + cuts, cuts + [d])]


def ntiles_for(rng, d, w, cap_bits=20):
    """A tile count whose image is a whole number of 16-byte vectors and at most 2^cap_bits elements."""
    lo = max(1, 16 // max(1, (w << d)))
    m = lo * int(rng.integers(1, 12))
    while (m << d) > (1 << cap_bits) and m > lo:
        m -= lo
    return m


def rand_options(seed, kind):
    """Options drawn from their documented domains (their own generator, so that the case drawn for a seed
    is the same with and without them): other kernels, block sizes, workgroup shapes and block orders."""
    rng = np.random.default_rng(seed ^ 0x5EED0)
    pick = lambda values: int(values[int(rng.integers(0, len(values)))])
    f = {}
    if kind == 0:
        if rng.integers(0, 2):
            f["strategy"] = pick([ll.LL_STRATEGY_LDS_ELEM, ll.LL_STRATEGY_LDS_VEC, ll.LL_STRATEGY_LDS_TR])
        if rng.integers(0, 2):
            f["elem_threads_log2"] = pick([6, 7, 8, 9, 10])
        if rng.integers(0, 3) == 0:
            f["block_bytes"] = pick([4096, 8192, 16384, 32768])
        if rng.integers(0, 3) == 0:
            f["vec_threads"] = pick([64, 128, 256])
        if rng.integers(0, 3) == 0:
            f["shuffle_block_bytes"] = pick([4096, 8192])
        if rng.integers(0, 3) == 0:
            f["xcd_chunk"] = pick([0, 1, 2, 16, 256])
        if rng.integers(0, 3) == 0:
            f["inflight_bytes"] = pick([16384, 32768, 65536, 131072])
        if rng.integers(0, 4) == 0:
            f["pref_bytes"] = pick([4096, 16384])
    elif kind == 1:
        if rng.integers(0, 2):
            f["pull_threads_log2"] = 6
        if rng.integers(0, 2):
            f["block_bytes"] = pick([1024, 4096, 8192, 16384])
        if rng.integers(0, 3) == 0:
            f["pull_mode"] = pick([0, 1, 2])
        if rng.integers(0, 3) == 0:
            f["pull_vec_bits"] = pick([0, 1, 2])
        if rng.integers(0, 3) == 0:
            f["pull_xcd_chunk"] = pick([0, 1, 4, 64])
        if rng.integers(0, 3) == 0:
            f["pull_inflight_bytes"] = pick([16384, 65536])
    else:
        if rng.integers(0, 3):
            f["gather_kernel"] = pick([ll.LL_GATHER_SHUFFLE, ll.LL_GATHER_WAVE_STAGED, ll.LL_GATHER_BLOCK_STAGED,
                                       ll.LL_GATHER_SHUFFLE_ROWS])
        if rng.integers(0, 2):
            f["gather_waves"] = pick([1, 2, 4])
        if rng.integers(0, 3) == 0:
            f["gather_threads_log2"] = pick([8, 9, 10])
        if rng.integers(0, 3) == 0:
            f["gather_block_bytes"] = pick([4096, 16384, 65536])
        if rng.integers(0, 3) == 0:
            f["gather_lds_max_bytes"] = pick([16384, 65536, 131072])
        if rng.integers(0, 3) == 0:
            f["gather_xcd_chunk"] = pick([0, 1, 4, 64])
        if rng.integers(0, 4) == 0:
            f["gather_phased_max_bytes"] = pick([262144, 1048576])
        if rng.integers(0, 4) == 0:
            f["gather_swizzle_always"] = 1
    return ll.ll_options_init(**f), tuple(sorted(f.items()))


def run_case(seed, with_options=False):
    rng = np.random.default_rng(seed)
    kind = int(rng.integers(0, 3))
    w = int(rng.choice([1, 2, 4, 8]))
    opts, chosen = rand_options(seed, kind) if with_options else (None, ())
    if kind == 0:
        d = int(rng.integers(2, 19))
        sa = split(rng, d)
        sb = sa if rng.integers(0, 3) else split(rng, d)
        if sb[3] != sa[3]:
            sb = sa
        dd = d - sa[3]
        if dd < 1:
            return None
        ka, kb = int(rng.integers(0, 3)), int(rng.integers(0, 3))
        ca = rand_cols(rng, dd, dd, ka) + [1 << k for k in range(dd, d)]
        cb = rand_cols(rng, dd, dd, kb) + [1 << k for k in range(dd, d)]
        offa = int(rng.integers(0, 1 << dd)) if rng.integers(0, 3) == 0 else 0
        offb = int(rng.integers(0, 1 << dd)) if rng.integers(0, 3) == 0 else 0
        od = out_dims_of(rng, d)
        desc = ("conv", seed, w, d, sa, sb, ka, kb, offa, offb, chosen)
        a = ll.ll_layout_with_offset(mk(sa, od, ca), offa)
        b = ll.ll_layout_with_offset(mk(sb, od, cb), offb)
        plan = ll.ll_plan_convert(a, b, w, opts)
        nt = ntiles_for(rng, d, w)
        src = rng.integers(0, np.iinfo(NP[w]).max, size=nt << d, dtype=NP[w])
        ts = torch.from_numpy(src.view(TD[w])).cuda()
        td = torch.full_like(ts, 0x5A)
        ll.ll_convert(plan, ts, td, nt)
        torch.cuda.synchronize()
        return desc, td.cpu().numpy().view(NP[w]), oracle.convert_affine(ca, offa, cb, offb, src)
    if kind == 1:
        dl = int(rng.integers(2, 15))
        da, db = dl + int(rng.integers(0, 5)), dl + int(rng.integers(0, 5))
        if da == dl and db == dl:
            da += 1
        sa, sb = split(rng, da), split(rng, db)
        sa, sb = (sa[0], sa[1], sa[2] + sa[3], 0), (sb[0], sb[1], sb[2] + sb[3], 0)
        ka, kb = int(rng.integers(0, 3)), int(rng.integers(0, 3))
        ca, cb = rand_cols(rng, da, dl, ka), rand_cols(rng, db, dl, kb)
        offa = int(rng.integers(0, 1 << dl)) if rng.integers(0, 3) == 0 else 0
        offb = int(rng.integers(0, 1 << dl)) if rng.integers(0, 3) == 0 else 0
        od = out_dims_of(rng, dl)
        desc = ("bcast", seed, w, dl, da, db, sa, sb, ka, kb, offa, offb, chosen)
        a = ll.ll_layout_with_offset(mk(sa, od, ca), offa)
        b = ll.ll_layout_with_offset(mk(sb, od, cb), offb)
        plan = ll.ll_plan_convert(a, b, w, opts)
        unit = max(1, 16 // w)
        nt = int(rng.integers(1, 12))
        while ((nt << da) % unit) or ((nt << db) % unit):
            nt += 1
        src = rng.integers(0, np.iinfo(NP[w]).max, size=nt << da, dtype=NP[w])
        ts = torch.from_numpy(src.view(TD[w])).cuda()
        td = torch.full((nt << db,), 0x5A, dtype=ts.dtype, device="cuda")
        ll.ll_convert(plan, ts, td, nt)
        torch.cuda.synchronize()
        return desc, td.cpu().numpy().view(NP[w]), oracle.convert_general_affine(ca, offa, cb, offb, dl, src)
    dl = int(rng.integers(2, 17))
    d = min(18, dl + (int(rng.integers(0, 4)) if rng.integers(0, 3) == 0 else 0))
    s = split(rng, d)
    s = (s[0], s[1], s[2] + s[3], 0)
    k = int(rng.integers(0, 3))
    cols = rand_cols(rng, d, dl, k)
    off = int(rng.integers(0, 1 << dl)) if rng.integers(0, 3) == 0 else 0
    od = out_dims_of(rng, dl)
    axis = int(rng.integers(0, len(od)))
    desc = ("gather", seed, w, dl, d, s, k, off, od, axis, chosen)
    lay = ll.ll_layout_with_offset(mk(s, od, cols), off)
    nt = ntiles_for(rng, d, w)
    inp = rng.integers(0, np.iinfo(NP[w]).max, size=nt << d, dtype=NP[w])
    if d > dl:                    # a broadcasting layout: the gather is defined on images of a logical tensor
        inp = oracle.consistent_image(cols, dl, inp)
    idx = rng.integers(-(1 << od[axis]) - 3, (1 << od[axis]) + 3, size=nt << d, dtype=np.int32)
    ti, tx = torch.from_numpy(inp.view(TD[w])).cuda(), torch.from_numpy(idx).cuda()
    to = torch.full_like(ti, 0x5A)
    ll.ll_gather(lay, axis, w, ti, tx, to, nt, opts=opts)
    torch.cuda.synchronize()
    return desc, to.cpu().numpy().view(NP[w]), oracle.gather_general(cols, od, axis, inp, idx, off)


@pytest.mark.parametrize("chunk", range(4))
def test_random_layouts_sizes_and_widths(chunk):
    counts = {"conv": 0, "bcast": 0, "gather": 0}
    for case in range(400):
        res = run_case(77000000 + 1000 * chunk + case)
        if res is None:
            continue
        desc, got, want = res
        assert np.array_equal(got, want), desc
        counts[desc[0]] += 1
    assert min(counts.values()) > 80


@pytest.mark.parametrize("chunk", range(4))
def test_random_layouts_under_random_options(chunk):
    """The same kinds of cases with options drawn at random: kernels the planner would not pick by itself,
    other block sizes, workgroup shapes and block orders must give the same bits."""
    counts = {"conv": 0, "bcast": 0, "gather": 0}
    for case in range(400):
        res = run_case(78000000 + 1000 * chunk + case, with_options=True)
        if res is None:
            continue
        desc, got, want = res
        assert np.array_equal(got, want), desc
        counts[desc[0]] += 1
    assert min(counts.values()) > 80
