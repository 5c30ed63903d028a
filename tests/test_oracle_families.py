"""Pins of the oracle's layout families: the paper's Layout A and swizzle matrix, the classical
index arithmetic of blocked layouts and of the CDNA matrix-instruction tiles, the benchmark
configurations' explicit bases, textbook XOR swizzling."""
import numpy as np
import pytest

import oracle
import workloads as wl
from oracle import OLayout
from oracle.algebra import to_matrix

REG, LANE, WAVE, OFFSET = 0, 1, 2, 4


def flat(coords, dims):
    x = 0
    for c, b in zip(coords, dims):
        x = (x << b) | c
    return x


def test_blocked_layout_reproduces_layout_a():
    a = oracle.blocked_layout([1, 1], [2, 3], [1, 0], order=[1, 0])
    assert a.in_dims == [(REG, 2), (LANE, 5), (WAVE, 1)] and a.out_dims == [4, 4]
    assert a.bases == wl.PAPER_LAYOUT_A


def delinearize(idx, bits, order):
    """Peel the per-dim coordinates off a linear id, fastest dim first."""
    out = [0] * len(bits)
    for dim in order:
        out[dim] = idx & ((1 << bits[dim]) - 1)
        idx >>= bits[dim]
    return out


def test_blocked_layout_matches_the_classical_index_arithmetic():
    """A blocked layout by its usual description: registers, lanes and waves each form a small
    grid over the dims, enumerated fastest dim first; coordinate = reg + R * (lane + T * wave)."""
    rng = np.random.default_rng(0)
    for _ in range(25):
        nd = int(rng.integers(1, 4))
        r = [int(x) for x in rng.integers(0, 3, size=nd)]
        t = [int(x) for x in rng.integers(0, 3, size=nd)]
        w = [int(x) for x in rng.integers(0, 2, size=nd)]
        order = [int(x) for x in rng.permutation(nd)]
        if sum(r) + sum(t) + sum(w) == 0:
            continue
        lay = oracle.blocked_layout(r, t, w, order)
        dims = [r[k] + t[k] + w[k] for k in range(nd)]
        assert lay.out_dims == dims
        nr, nt = sum(r), sum(t)
        for h in range(1 << (nr + nt + sum(w))):
            rc = delinearize(h & ((1 << nr) - 1), r, order)
            tc = delinearize((h >> nr) & ((1 << nt) - 1), t, order)
            wc = delinearize(h >> (nr + nt), w, order)
            coords = [rc[k] + (1 << r[k]) * (tc[k] + (1 << t[k]) * wc[k]) for k in range(nd)]
            assert oracle.apply(lay.bases, h) == flat(coords, dims), (r, t, w, order, h)
        assert oracle.is_distributed_layout(lay)


def test_mfma_accumulator_tiles_match_their_index_formulas_and_the_configs():
    t32 = oracle.mfma_accumulator_tile(5)
    assert t32.in_dims == [(REG, 4), (LANE, 6)] and t32.out_dims == [5, 5]
    for r in range(16):
        for l in range(64):
            row, col = (r % 4) + 4 * (l // 32) + 8 * (r // 4), l % 32
            assert oracle.apply(t32.bases, r | (l << 4)) == (row << 5) | col
    t16 = oracle.mfma_accumulator_tile(4)
    assert t16.in_dims[:2] == [(REG, 2), (LANE, 6)] and t16.out_dims == [4, 4]
    for r in range(4):
        for l in range(64):
            assert oracle.apply(t16.bases, r | (l << 2)) == ((r + 4 * (l // 16)) << 4) | (l % 16)
    # config 1's destination: the 32x32 tile, two waves along the rows, then two along the columns
    c1 = wl.config(1)
    full = oracle.product_of([t32, oracle.identity_map(WAVE, 0, 1, 2), oracle.identity_map(WAVE, 1, 1, 2)])
    assert full.bases == c1.dst_bases and full.out_dims == c1.out_dim_bits
    # config 3's source: the 16x16 tile repeated by registers over 4 row blocks and 4 column blocks
    c3 = wl.config(3)
    full = oracle.product_of([t16, oracle.identity_map(REG, 0, 2, 2), oracle.identity_map(REG, 1, 2, 2)])
    assert [d for d in full.in_dims if d[1]] == [(REG, 6), (LANE, 6)]
    assert full.bases == c3.src_bases


def test_mfma_operand_tile_matches_its_index_formula():
    for m_bits, kr in [(5, 2), (4, 2), (5, 3), (4, 3)]:
        t = oracle.mfma_operand_tile(m_bits, kr)
        k_bits = kr + 6 - m_bits
        assert t.out_dims == [m_bits, k_bits]
        for r in range(1 << kr):
            for l in range(64):
                i, k = l % (1 << m_bits), r + (1 << kr) * (l >> m_bits)
                assert oracle.apply(t.bases, r | (l << kr)) == (i << k_bits) | k


@pytest.mark.parametrize("m,n,vec,per_phase,max_phase", [(3, 3, 1, 1, 8), (4, 6, 8, 1, 8), (5, 5, 4, 2, 4),
                                                         (6, 4, 2, 4, 8), (3, 6, 8, 2, 2), (4, 4, 4, 1, 1)])
def test_mma_swizzle_has_the_closed_form_matrix(m, n, vec, per_phase, max_phase):
    """Sec. 4.3: the matrix of the swizzled layout is [[I_n, C], [0, I_m]] with the entries of C
    given by c_i = (vec * ((2^i / per_phase) mod max_phase)) mod 2^n for bit i of the row index."""
    lay = oracle.mma_swizzle_layout(m, n, vec, per_phase, max_phase)
    mat = to_matrix(lay)                              # rows: j bits (n) then i bits (m); same for columns
    want = np.zeros((m + n, m + n), dtype=np.uint8)
    want[:n, :n] = np.eye(n, dtype=np.uint8)
    want[n:, n:] = np.eye(m, dtype=np.uint8)
    for i in range(m):
        c = (vec * (((1 << i) // per_phase) % max_phase)) % (1 << n)
        for b in range(n):
            want[b, n + i] = (c >> b) & 1
    assert np.array_equal(mat, want)
    assert oracle.is_memory_layout(lay)
    # the definition itself, on every location: offset -> location is the inverse of the formula
    for i in range(1 << m):
        for j in range(1 << n):
            off = oracle.mma_swizzle_offset(i, j, n, vec, per_phase, max_phase)
            assert oracle.apply(lay.bases, off) == (i << n) | j


def test_mma_swizzle_special_case_is_the_textbook_xor_swizzle():
    # vec = 1, per_phase = 1, max_phase = row length: element (i, j) sits at column i xor j
    n = 5
    lay = oracle.mma_swizzle_layout(n, n, 1, 1, 1 << n)
    for i in range(1 << n):
        for j in range(1 << n):
            assert oracle.mma_swizzle_offset(i, j, n, 1, 1, 1 << n) == (i << n) | (i ^ j)
    # 32 lanes reading a row and 32 lanes reading a column of fp32 are both conflict free
    cols_bits, rows_bits = [1 << k for k in range(n)], [1 << (n + k) for k in range(n)]
    row_read = rows_bits + cols_bits                  # registers walk the rows, lanes the columns
    col_read = cols_bits + rows_bits                  # registers walk the columns, lanes the rows
    one_phase = [0] * 32
    for access in (row_read, col_read):
        assert oracle.wavefronts(lay.bases, access, 5, 5, 4, 0, 32, one_phase)[0] == 1
    plain = oracle.mma_swizzle_layout(n, n, 1, 1, 1)  # no swizzle: a column read hits one bank 32 times
    assert oracle.wavefronts(plain.bases, col_read, 5, 5, 4, 0, 32, one_phase)[0] == 32
    assert oracle.wavefronts(plain.bases, row_read, 5, 5, 4, 0, 32, one_phase)[0] == 1


def test_family_definitions():
    a = OLayout([(REG, 2), (LANE, 5), (WAVE, 1)], [4, 4], wl.PAPER_LAYOUT_A)
    assert oracle.is_distributed_layout(a)
    wide = OLayout([(REG, 3), (LANE, 5), (WAVE, 1)], [4, 4], a.bases[:2] + [0] + a.bases[2:])
    assert oracle.is_distributed_layout(wide)                       # zero columns are allowed
    dup = OLayout([(REG, 3), (LANE, 5), (WAVE, 1)], [4, 4], a.bases[:2] + [a.bases[0]] + a.bases[2:])
    assert not oracle.is_distributed_layout(dup)                    # a repeated non-zero column
    assert not oracle.is_distributed_layout(OLayout([(REG, 2)], [3], [1, 2]))          # not surjective
    c4 = wl.config(4)
    assert not oracle.is_distributed_layout(OLayout([(REG, 6), (LANE, 6), (WAVE, 4)], [16], c4.src_bases))
    ident = OLayout([(OFFSET, 4)], [2, 2], [1, 2, 4, 8])            # the unswizzled layout
    assert oracle.is_memory_layout(ident)
    assert not oracle.is_memory_layout(OLayout([(OFFSET, 4)], [2, 2], [1, 2, 4, 7]))   # three bits
    assert not oracle.is_memory_layout(OLayout([(OFFSET, 4)], [2, 2], [1, 2, 3, 3]))   # singular
    assert oracle.is_memory_layout(OLayout([(OFFSET, 8)], [4, 4], a.bases))             # a permutation matrix qualifies
    assert not oracle.is_memory_layout(wide)                        # not square


def coords_of(x, dims):
    out = []
    for b in reversed(dims):
        out.append(x & ((1 << b) - 1))
        x >>= b
    return out[::-1]


def test_slice_drops_the_coordinate_of_the_reduced_dim():
    """Sec. 4.3 "Sliced Layouts" by its meaning: wherever the layout put element (c_0, .., c_n), the
    slice along dim j puts (c_0, .., c_n) without c_j; checked for every hardware index of random
    blocked layouts.  The Remark's two facts: still surjective, and exactly the input bits that ran
    along the reduced dim turn into zero columns."""
    rng = np.random.default_rng(77)
    for _ in range(30):
        nd = int(rng.integers(2, 4))
        r = [int(x) for x in rng.integers(0, 3, size=nd)]
        t = [int(x) for x in rng.integers(0, 3, size=nd)]
        w = [int(x) for x in rng.integers(0, 2, size=nd)]
        order = [int(x) for x in rng.permutation(nd)]
        lay = oracle.blocked_layout(r, t, w, order)
        for dim in range(nd):
            s = oracle.slice_layout(lay, dim)
            rest = [b for j, b in enumerate(lay.out_dims) if j != dim]
            assert s.out_dims == rest and s.in_dims == lay.in_dims
            images = set()
            for h in range(1 << lay.d_in):
                c = coords_of(oracle.apply(lay.bases, h), lay.out_dims)
                del c[dim]
                assert oracle.apply(s.bases, h) == flat(c, rest)
                images.add(flat(c, rest))
            assert len(images) == 1 << sum(rest)                      # surjective
            assert sum(1 for b in s.bases if b == 0) == lay.out_dims[dim]
            assert oracle.is_distributed_layout(s)


def test_slice_of_layout_a_along_each_dim():
    """Layout A (Sec. 4.1, 16 x 16): along dim 1 (j) the slice keeps the i bits, along dim 0 the j bits."""
    a = OLayout([(REG, 2), (LANE, 5), (WAVE, 1)], [4, 4], wl.PAPER_LAYOUT_A)
    assert oracle.slice_layout(a, 1).bases == [b >> 4 for b in wl.PAPER_LAYOUT_A]
    assert oracle.slice_layout(a, 0).bases == [b & 15 for b in wl.PAPER_LAYOUT_A]
    with pytest.raises(ValueError):
        oracle.slice_layout(oracle.slice_layout(a, 0), 0)
