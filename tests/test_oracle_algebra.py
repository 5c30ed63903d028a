"""Pins of the oracle's layout algebra (product, left division, contiguity) to things other than
itself: scipy's block_diag, the paper's Layout A and its description as a tiling, hand cases,
single-entry perturbations, brute force."""
import itertools

import numpy as np
import pytest
import scipy.linalg

import oracle
import workloads as wl
from oracle import OLayout
from oracle.algebra import from_matrix, to_matrix

REG, LANE, WAVE = 0, 1, 2


def random_matrix(rng, rows, cols):
    return rng.integers(0, 2, size=(rows, cols), dtype=np.uint8)


def test_product_single_label_is_scipy_block_diag():
    rng = np.random.default_rng(0)
    for _ in range(20):
        r1, c1, r2, c2 = (int(x) for x in rng.integers(1, 5, size=4))
        m1, m2 = random_matrix(rng, r1, c1), random_matrix(rng, r2, c2)
        p = oracle.product(from_matrix(m1, [(REG, c1)], [r1]), from_matrix(m2, [(REG, c2)], [r2]))
        assert np.array_equal(to_matrix(p), scipy.linalg.block_diag(m1, m2))
        assert p.in_dims == [(REG, c1 + c2)] and p.out_dims == [r1 + r2]


def test_layout_a_is_the_product_of_its_tiles():
    """Sec. 4.1: Layout A tiles a 16x16 tensor by 2x2 registers, 4x8 threads and 2x1 warps
    (column index j fastest).  The product of the three identity-like tiles must be the paper's
    printed matrix."""
    regs = OLayout([(REG, 2)], [1, 1], [1, 2])                 # reg0 -> j0, reg1 -> i0
    thrs = OLayout([(LANE, 5)], [2, 3], [1, 2, 4, 8, 16])      # thr0..2 -> j, thr3..4 -> i
    warps = OLayout([(WAVE, 1)], [1, 0], [1])                  # warp0 -> i
    a = oracle.product(oracle.product(regs, thrs), warps)
    assert a.in_dims == [(REG, 2), (LANE, 5), (WAVE, 1)] and a.out_dims == [4, 4]
    assert a.bases == wl.PAPER_LAYOUT_A
    golden = np.loadtxt("tests/golden/paper_layout_a_matrix.txt", dtype=np.uint8, comments="#")
    assert np.array_equal(to_matrix(a), golden)


def test_division_undoes_product_and_layout_a_divides_by_its_register_tile():
    regs = OLayout([(REG, 2)], [1, 1], [1, 2])
    thrs = OLayout([(LANE, 5)], [2, 3], [1, 2, 4, 8, 16])
    warps = OLayout([(WAVE, 1)], [1, 0], [1])
    a = OLayout([(REG, 2), (LANE, 5), (WAVE, 1)], [4, 4], wl.PAPER_LAYOUT_A)
    q = oracle.divide_left(a, regs)
    rest = oracle.product(thrs, warps)
    assert q is not None and q.bases == rest.bases and q.out_dims == [3, 3]
    assert [d for d in q.in_dims if d[1]] == rest.in_dims
    # a tile that is not a factor: registers swapped
    assert oracle.divide_left(a, OLayout([(REG, 2)], [1, 1], [2, 1])) is None
    # a 4-wide row tile does not divide Layout A (its second register walks down a column)
    assert oracle.divide_left(a, OLayout([(REG, 2)], [0, 2], [1, 2])) is None


def test_division_random_products_and_single_entry_perturbations():
    rng = np.random.default_rng(1)
    for _ in range(30):
        t_in = [(REG, int(rng.integers(0, 3))), (LANE, int(rng.integers(0, 3)))]
        m_in = [(REG, int(rng.integers(0, 3))), (LANE, int(rng.integers(0, 3))), (WAVE, int(rng.integers(0, 2)))]
        t_out = [int(rng.integers(0, 3)), int(rng.integers(0, 3))]
        m_out = [int(rng.integers(0, 3)), int(rng.integers(0, 3))]
        if sum(n for _, n in t_in) == 0 or sum(t_out) == 0 or sum(n for _, n in m_in) == 0 or sum(m_out) == 0:
            continue
        t = from_matrix(random_matrix(rng, sum(t_out), sum(n for _, n in t_in)), t_in, t_out)
        m2 = from_matrix(random_matrix(rng, sum(m_out), sum(n for _, n in m_in)), m_in, m_out)
        p = oracle.product(t, m2)
        q = oracle.divide_left(p, t)
        assert q is not None and q.bases == m2.bases and q.out_dims == m2.out_dims
        # flipping any entry outside the two diagonal blocks destroys divisibility; flipping one
        # inside the M2 block keeps it and changes the quotient; inside the tile block destroys it
        mp = to_matrix(p)
        for r, c in itertools.product(range(mp.shape[0]), range(mp.shape[1])):
            bad = mp.copy()
            bad[r, c] ^= 1
            qq = oracle.divide_left(from_matrix(bad, p.in_dims, p.out_dims), t)
            if qq is not None:
                assert qq.bases != m2.bases                 # the flip fell inside the M2 block
                back = oracle.product(t, qq)
                assert np.array_equal(to_matrix(back), bad)


def test_vector_tile_division_equals_contiguity_for_distributed_layouts():
    """Sec. 5.3: the tile of a 2^n-element vector access is the n x n identity on registers.
    For layouts whose columns are distinct unit vectors, divisibility by it (on the flattened
    tensor) is the same as 2^n contiguous elements per thread (Sec. 5.1)."""
    rng = np.random.default_rng(2)
    for _ in range(40):
        d, nreg = 8, int(rng.integers(1, 5))
        cols = [1 << int(p) for p in rng.permutation(d)]
        if rng.integers(0, 2):                              # often make a few low registers contiguous
            k = int(rng.integers(1, nreg + 1))
            rest = [c for c in cols if c >= (1 << k)]
            cols = [1 << i for i in range(k)] + rest
        lay = OLayout([(REG, nreg), (LANE, d - nreg)], [d], cols)
        c = oracle.contiguity(lay)
        for n in range(0, nreg + 1):
            divisible = oracle.divide_left(lay, oracle.identity_tile(REG, n)) is not None
            assert divisible == (c >= (1 << n)), (cols, n, c)


def test_contiguity_hand_cases_and_forward_brute_force():
    # the paper's example: a [128, 1] tensor still vectorizes (the last dim has a single element)
    col_vec = OLayout([(REG, 2), (LANE, 5)], [7, 0], [1, 2, 4, 8, 16, 32, 64])
    assert oracle.contiguity(col_vec) == 4
    # Layout A: two contiguous elements per thread (its 2x2 register tile is 2 wide)
    assert oracle.contiguity(OLayout([(REG, 2), (LANE, 5), (WAVE, 1)], [4, 4], wl.PAPER_LAYOUT_A)) == 2
    # registers walk down a column of a row-major tensor: nothing contiguous
    assert oracle.contiguity(OLayout([(REG, 2), (LANE, 4)], [3, 3], [8, 16, 1, 2, 4, 32])) == 1
    # bijective layouts: the inverse sends element i to register i exactly when L sends register i to i
    rng = np.random.default_rng(3)
    for _ in range(30):
        d, nreg = 7, 3
        cols = wl.random_invertible_bases(int(rng.integers(1000)), d)
        if rng.integers(0, 2):
            cols[0] = 1
        if rng.integers(0, 2):
            cols[1] = 2
        if len({oracle.apply(cols, h) for h in range(1 << d)}) != 1 << d:
            continue
        forward = 0
        while forward < (1 << nreg) and oracle.apply(cols, forward) == forward:
            forward += 1
        assert oracle.contiguity(OLayout([(REG, nreg), (LANE, d - nreg)], [d], cols)) == max(forward, 1)


def test_generalized_vectorization_permutes_registers():
    """Sec. 5.3 "Generalized Vectorization": a column-major register order does not divide by the
    vector tile; after swapping the two register bits it does."""
    lay = OLayout([(REG, 2), (LANE, 2)], [2, 2], [4, 1, 2, 8])           # reg0 -> i0, reg1 -> j0
    tile = oracle.identity_tile(REG, 1, n_out_dims=2)
    assert oracle.divide_left(lay, tile) is None
    perm, q = oracle.divide_left_permuting(lay, tile, REG)
    assert perm == [1, 0]
    assert q.bases == [2, 1, 4] and q.out_dims == [2, 1]                 # i0 ; j1, i1 with j0 removed
    # no register maps to j0 at all: no permutation helps
    assert oracle.divide_left_permuting(OLayout([(REG, 1), (LANE, 1)], [1, 1], [2, 1]), tile, REG) is None
