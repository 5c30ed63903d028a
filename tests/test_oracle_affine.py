"""Pins of the oracle's affine conversion and gather (Conclusions: flips and slices as
y = A x xor b) to numpy's flip / roll / take_along_axis and to brute force."""
import numpy as np
import pytest

import oracle
import workloads as wl


def unit(d):
    return [1 << k for k in range(d)]


def dim_mask(dims, j, bits=None):
    """Flattened mask of logical dim j (all of its bits, or the given ones)."""
    shift = sum(dims[j + 1:])
    m = (1 << dims[j]) - 1 if bits is None else bits
    return m << shift


def test_zero_offsets_reduce_to_the_linear_oracle():
    rng = np.random.default_rng(0)
    d = 9
    a, b = wl.random_invertible_bases(11, d), wl.random_invertible_bases(12, d)
    src = rng.integers(0, 1 << 32, size=3 << d, dtype=np.uint32)
    assert np.array_equal(oracle.convert_affine(a, 0, b, 0, src), oracle.convert(a, b, src))
    dims = [4, 5]
    idx = rng.integers(0, 16, size=3 << d, dtype=np.int32)
    assert np.array_equal(oracle.gather_affine(a, 0, dims, 0, src, idx), oracle.gather(a, dims, 0, src, idx))


@pytest.mark.parametrize("w", [1, 2, 4, 8])
def test_flip_and_half_roll_on_the_identity_layout(w):
    """With the identity layout an image is the flattened tensor itself.  Converting to the same
    layout with offset = all ones of a dim stores the tensor flipped along that dim; offset = the
    top bit of a dim stores it rolled by half that dim."""
    rng = np.random.default_rng(w)
    dims = [3, 4, 2]
    d = sum(dims)
    shape = [1 << b for b in dims]
    dt = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}[w]
    src = rng.integers(0, np.iinfo(dt).max, size=5 << d, dtype=dt)
    t = src.reshape([5] + shape)
    for j in range(3):
        got = oracle.convert_affine(unit(d), 0, unit(d), dim_mask(dims, j), src)
        assert np.array_equal(got.reshape(t.shape), np.flip(t, axis=1 + j))
        got = oracle.convert_affine(unit(d), 0, unit(d), dim_mask(dims, j, 1 << (dims[j] - 1)), src)
        assert np.array_equal(got.reshape(t.shape), np.roll(t, shape[j] // 2, axis=1 + j))
    # all dims flipped: the flattened tile reversed
    got = oracle.convert_affine(unit(d), 0, unit(d), (1 << d) - 1, src)
    assert np.array_equal(got.reshape(5, -1), src.reshape(5, -1)[:, ::-1])
    # the offset on the source side undoes it
    assert np.array_equal(oracle.convert_affine(unit(d), (1 << d) - 1, unit(d), 0, got), src)


def test_flip_under_a_distributed_layout_is_a_flip_of_the_logical_tensor():
    """Layout A of Sec. 4.1 (16 x 16): image under A -> image under (A, rows flipped); read back
    through plain A, the logical tensor is flipped along the rows."""
    a = wl.PAPER_LAYOUT_A
    rng = np.random.default_rng(3)
    logical = rng.integers(0, 1 << 16, size=256, dtype=np.uint16)
    img = oracle.convert(unit(8), a, logical)                     # logical tensor -> image under A
    flipped_img = oracle.convert_affine(a, 0, a, dim_mask([4, 4], 0), img)
    back = oracle.convert(a, unit(8), flipped_img)                 # image under A -> logical tensor
    assert np.array_equal(back.reshape(16, 16), np.flip(logical.reshape(16, 16), axis=0))


def test_affine_conversion_brute_force_and_round_trip():
    rng = np.random.default_rng(4)
    for d in (3, 6, 8):
        a, b = wl.random_invertible_bases(20 + d, d), wl.random_invertible_bases(30 + d, d)
        oa, ob = int(rng.integers(0, 1 << d)), int(rng.integers(0, 1 << d))
        src = rng.integers(0, 1 << 32, size=2 << d, dtype=np.uint32)
        got = oracle.convert_affine(a, oa, b, ob, src)
        want = np.empty_like(src)
        for t in range(2):
            for h in range(1 << d):
                x = oracle.apply(a, h) ^ oa
                hb = next(k for k in range(1 << d) if oracle.apply(b, k) ^ ob == x)
                want[(t << d) + hb] = src[(t << d) + h]
        assert np.array_equal(got, want)
        assert np.array_equal(oracle.convert_affine(b, ob, a, oa, got), src)
    with pytest.raises(oracle.OracleError):
        oracle.convert_affine([1, 2, 3], 0, [1, 2, 4], 0, np.zeros(8, dtype=np.uint8))   # A singular


def test_gather_under_a_flipped_layout_is_take_along_axis_on_the_logical_tensor():
    """Identity layout with both dims flipped: image index h holds logical element ~h, so the
    logical tensors are the reversed images; the gather itself is numpy's take_along_axis."""
    rng = np.random.default_rng(5)
    dims = [5, 4]
    d = 9
    off = (1 << d) - 1
    nt = 3
    inp = rng.integers(0, 1 << 32, size=nt << d, dtype=np.uint32)
    for axis in (0, 1):
        idx = rng.integers(0, 1 << dims[axis], size=nt << d, dtype=np.int32)
        out = oracle.gather_affine(unit(d), off, dims, axis, inp, idx)
        rev = lambda a: a.reshape(nt, -1)[:, ::-1].reshape(nt, 32, 16)
        want_logical = np.take_along_axis(rev(inp), rev(idx).astype(np.int64), axis=1 + axis)
        assert np.array_equal(rev(out), want_logical)
    # flipping only the axis: idx[h] = own coordinate still returns the input
    off_rows = dim_mask(dims, 0)
    h = np.arange(nt << d) & ((1 << d) - 1)
    own = (((h ^ off_rows) >> 4) & 31).astype(np.int32)
    assert np.array_equal(oracle.gather_affine(unit(d), off_rows, dims, 0, inp, own), inp)


def test_broadcasting_affine_conversion_pins():
    rng = np.random.default_rng(6)
    # zero offsets: the linear broadcasting conversion; bijective layouts: the affine conversion
    base = wl.PAPER_LAYOUT_A
    wide = base[:2] + [0] + base[2:]
    src = rng.integers(0, 1 << 32, size=3 << 9, dtype=np.uint32)
    assert np.array_equal(oracle.convert_general_affine(wide, 0, base, 0, 8, src), oracle.convert_general(wide, base, 8, src))
    a, b = wl.random_invertible_bases(51, 8), wl.random_invertible_bases(52, 8)
    s8 = rng.integers(0, 1 << 32, size=2 << 8, dtype=np.uint32)
    assert np.array_equal(oracle.convert_general_affine(a, 0x35, b, 0xC1, 8, s8), oracle.convert_affine(a, 0x35, b, 0xC1, s8))
    # identity layout expanded by one replica bit (a zero column on top) and flipped: every logical
    # element appears twice, in reversed order
    d = 6
    ident = unit(d)
    flipped_wide = ident + [0]
    t = rng.integers(0, 1 << 16, size=4 << d, dtype=np.uint16)
    got = oracle.convert_general_affine(ident, 0, flipped_wide, (1 << d) - 1, d, t)
    rev = t.reshape(4, 1 << d)[:, ::-1]
    assert np.array_equal(got.reshape(4, 2, 1 << d), np.stack([rev, rev], axis=1))
    # collapsing a replicated, flipped source reads the replica whose free bit is zero
    src_wide = rng.integers(0, 1 << 16, size=4 << (d + 1), dtype=np.uint16)
    got = oracle.convert_general_affine(flipped_wide, (1 << d) - 1, ident, 0, d, src_wide)
    assert np.array_equal(got.reshape(4, 1 << d), src_wide.reshape(4, 2, 1 << d)[:, 0, ::-1])


def test_affine_product_division_and_contiguity():
    """Def. "Product" / "Left Division" with constants: the product of two affine layouts applied to
    (h1, h2) is, per logical dim, the pair of coordinates the factors give, the first factor's bits
    below the second's; division undoes it and refuses a tile with another constant.  Contiguity
    under a constant: the run of ascending consecutive elements in registers 0, 1, .. of thread 0,
    read off the elements directly."""
    from oracle.algebra import OLayout
    rng = np.random.default_rng(71)

    def coords(x, dims):
        out = []
        for n in reversed(dims):
            out.append(x & ((1 << n) - 1))
            x >>= n
        return out[::-1]

    for _ in range(30):
        nd = int(rng.integers(1, 4))
        fa = [[int(x) for x in rng.integers(0, 3, size=nd)] for _ in range(3)]
        fb = [[int(x) for x in rng.integers(0, 3, size=nd)] for _ in range(3)]
        order = [int(x) for x in rng.permutation(nd)]
        a, b = oracle.blocked_layout(*fa, order), oracle.blocked_layout(*fb, order)
        a.offset, b.offset = int(rng.integers(0, 1 << a.d_out)), int(rng.integers(0, 1 << b.d_out))
        p = oracle.product(a, b)
        # walk all (h1, h2): input bits are merged label by label, a's bits first
        for h1 in range(1 << a.d_in):
            for h2 in range(0, 1 << b.d_in, max(1, (1 << b.d_in) // 8)):
                h, pos, p1, p2 = 0, 0, 0, 0
                for (_, na), (_, nb) in zip(a.in_dims, b.in_dims):
                    h |= ((h1 >> p1) & ((1 << na) - 1)) << pos
                    h |= ((h2 >> p2) & ((1 << nb) - 1)) << (pos + na)
                    pos, p1, p2 = pos + na + nb, p1 + na, p2 + nb
                ca = coords(oracle.apply(a.bases, h1) ^ a.offset, a.out_dims)
                cb = coords(oracle.apply(b.bases, h2) ^ b.offset, b.out_dims)
                got = coords(oracle.apply(p.bases, h) ^ p.offset, p.out_dims)
                assert got == [x | (y << n) for x, y, n in zip(ca, cb, a.out_dims)]
        q = oracle.divide_left(p, a)
        assert q is not None and q.bases == b.bases and q.offset == b.offset
        if a.d_out:
            assert oracle.divide_left(p, OLayout(a.in_dims, a.out_dims, a.bases, a.offset ^ (1 << int(rng.integers(0, a.d_out))))) is None
    for off, want in ((0, 8), (4, 4), (6, 2), (2, 2), (1, 1), (0b1000, 8), (0b1100, 4)):
        lay = OLayout([(0, 3), (1, 2)], [5], [1, 2, 4, 8, 16], off)
        held = np.array([oracle.apply(lay.bases, r) ^ off for r in range(8)])
        run = 1
        while run < 8 and held[run] == held[0] + run:
            run += 1
        assert oracle.contiguity(lay) == run == want
