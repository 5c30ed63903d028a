"""Pins for the CPU oracle: values the paper prints, closed forms, textbook routines, brute force.

Nothing here calls the HIP library.  Helper arithmetic in this file is written
independently of oracle/ (numpy bit matrices, Python sets) so that a mistake in
the oracle cannot hide behind the same mistake in its test.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
import workloads as wl


# ----------------------------------------------------------------------------
# independent helpers (numpy / python only)
# ----------------------------------------------------------------------------

def cols_to_matrix(cols, d_out):
    """uint8 matrix M[i, k] = bit i of column k."""
    return np.array([[(c >> i) & 1 for c in cols] for i in range(d_out)], dtype=np.uint8)


def matrix_to_cols(m):
    return [int(sum(int(m[i, k]) << i for i in range(m.shape[0]))) for k in range(m.shape[1])]


def np_apply(cols, d_out, h):
    m = cols_to_matrix(cols, d_out)
    v = np.array([(h >> k) & 1 for k in range(len(cols))], dtype=np.uint8)
    w = (m.astype(np.int64) @ v.astype(np.int64)) % 2
    return int(sum(int(w[i]) << i for i in range(d_out)))


def np_images(cols, d):
    """L(h) for every h in [0, 2^d), vectorised XOR of the selected columns."""
    h = np.arange(1 << d, dtype=np.int64)
    img = np.zeros(1 << d, dtype=np.int64)
    for k, c in enumerate(cols):
        img ^= ((h >> k) & 1) * int(c)
    return img


def span(vectors):
    s = {0}
    for v in vectors:
        s |= {x ^ v for x in s}
    return s


def random_invertible(rng, d):
    while True:
        cols = [int(rng.integers(0, 1 << d)) for _ in range(d)]
        if len(span(cols)) == 1 << d:
            return cols


def random_bit_permutation(rng, d):
    return [1 << int(p) for p in rng.permutation(d)]


# ----------------------------------------------------------------------------
# the paper's Layout A (Sec. 4.1)
# ----------------------------------------------------------------------------

def load_layout_a(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "paper_layout_a_matrix.txt"))
            if l.strip() and not l.startswith("#")]
    m = np.array(rows, dtype=np.uint8)
    assert m.shape == (8, 8)
    return matrix_to_cols(m)


def load_table(golden_dir):
    return [tuple(int(x) for x in l.split())
            for l in open(os.path.join(golden_dir, "paper_layout_a_table.txt"))
            if l.strip() and not l.startswith("#")]


def test_layout_a_columns_match_printed_matrix(golden_dir):
    assert load_layout_a(golden_dir) == wl.PAPER_LAYOUT_A


def test_layout_a_worked_example(golden_dir):
    # Sec. 4.1: register r1 of thread t9 in warp w0 -> (i, j) = (2, 3)
    a = load_layout_a(golden_dir)
    h = 1 | (9 << 2) | (0 << 7)
    x = oracle.apply(a, h)
    assert (x >> 4, x & 15) == (2, 3)
    # the same location is loc_w ^ loc_t ^ loc_r = (0,0) ^ (2,2) ^ (0,1)
    loc_r = oracle.apply(a, 1)
    loc_t = oracle.apply(a, 9 << 2)
    loc_w = oracle.apply(a, 0 << 7)
    assert (loc_r >> 4, loc_r & 15) == (0, 1)
    assert (loc_t >> 4, loc_t & 15) == (2, 2)
    assert (loc_w >> 4, loc_w & 15) == (0, 0)
    assert loc_r ^ loc_t ^ loc_w == x


def test_layout_a_table_forward_and_inverse(golden_dir):
    a = load_layout_a(golden_dir)
    inv = oracle.inverse_table(a)
    for i, j, reg, thr, warp in load_table(golden_dir):
        h = reg | (thr << 2) | (warp << 7)
        assert oracle.apply(a, h) == (j | (i << 4))
        assert int(inv[j | (i << 4)]) == h


def test_register_zero_has_even_coordinates(golden_dir):
    # Sec. 4.1: r0 of every thread sits where the last bits of i and j are 0;
    # r1 where the last bit of i is 0 and the last bit of j is 1.
    a = load_layout_a(golden_dir)
    for thr in range(32):
        for warp in range(2):
            x0 = oracle.apply(a, 0 | (thr << 2) | (warp << 7))
            x1 = oracle.apply(a, 1 | (thr << 2) | (warp << 7))
            assert (x0 & 1, (x0 >> 4) & 1) == (0, 0)
            assert (x1 & 1, (x1 >> 4) & 1) == (1, 0)


def test_zero_column_aliases_registers(golden_dir):
    # Sec. 5.1 "Broadcasting": a zero column added to A_reg makes registers 4-7
    # hold the same tensor elements as registers 0-3.
    a = load_layout_a(golden_dir)
    widened = a[:2] + [0] + a[2:]          # a third register bit with a zero column
    for thr in range(32):
        for r in range(4):
            lo = oracle.apply(widened, r | (thr << 3))
            hi = oracle.apply(widened, (r + 4) | (thr << 3))
            assert lo == hi == oracle.apply(a, r | (thr << 2))


# ----------------------------------------------------------------------------
# apply / compose / inverse against numpy bit-matrix arithmetic and brute force
# ----------------------------------------------------------------------------

def test_apply_matches_numpy_matvec():
    rng = np.random.default_rng(11)
    for d_in, d_out in [(3, 5), (8, 8), (12, 12), (16, 16), (5, 3)]:
        cols = [int(rng.integers(0, 1 << d_out)) for _ in range(d_in)]
        for h in rng.integers(0, 1 << d_in, size=40):
            assert oracle.apply(cols, int(h)) == np_apply(cols, d_out, int(h))


def test_compose_matches_numpy_matmul():
    rng = np.random.default_rng(12)
    for d_in, d_mid, d_out in [(4, 4, 4), (6, 3, 5), (12, 12, 12), (3, 7, 2)]:
        inner = [int(rng.integers(0, 1 << d_mid)) for _ in range(d_in)]
        outer = [int(rng.integers(0, 1 << d_out)) for _ in range(d_mid)]
        want = (cols_to_matrix(outer, d_out).astype(np.int64)
                @ cols_to_matrix(inner, d_mid).astype(np.int64)) % 2
        assert oracle.compose(outer, d_out, inner) == matrix_to_cols(want)
        # and composition means outer(inner(u)) for every u
        for u in range(1 << d_in):
            assert oracle.apply(oracle.compose(outer, d_out, inner), u) == \
                oracle.apply(outer, oracle.apply(inner, u))


def test_compose_is_not_commutative_and_order_is_outer_after_inner():
    # a shear and a swap on 2 bits: outer o inner != inner o outer
    shear = [0b11, 0b10]      # e0 -> e0^e1, e1 -> e1
    swap = [0b10, 0b01]
    assert oracle.compose(shear, 2, swap) == [0b10, 0b11]
    assert oracle.compose(swap, 2, shear) == [0b11, 0b01]


def test_inverse_table_brute_force():
    rng = np.random.default_rng(13)
    for d in range(1, 9):
        for _ in range(5):
            cols = random_invertible(rng, d)
            inv = oracle.inverse_table(cols)
            for x in range(1 << d):
                # the unique h with L(h) = x, by linear search with numpy arithmetic
                hits = [h for h in range(1 << d) if np_apply(cols, d, h) == x]
                assert hits == [int(inv[x])]


def test_inverse_table_rejects_singular():
    with pytest.raises(oracle.OracleError) as e:
        oracle.inverse_table([1, 2, 3])          # third column = sum of the first two
    assert e.value.code == oracle.ERR_NOT_BIJECTIVE
    with pytest.raises(oracle.OracleError):
        oracle.inverse_table([1, 2, 0])          # broadcast (zero column)
    with pytest.raises(oracle.OracleError):
        oracle.inverse_table([1, 2, 8])          # image leaves the 3-bit space


# ----------------------------------------------------------------------------
# conversion
# ----------------------------------------------------------------------------

def brute_convert(a, b, src, d):
    """dst[hB] = src[hA] where B(hB) == A(hA), found by linear search with numpy arithmetic."""
    n = 1 << d
    dst = np.empty_like(src)
    img_b = [np_apply(b, d, h) for h in range(n)]
    for t in range(src.size // n):
        for ha in range(n):
            x = np_apply(a, d, ha)
            hb = img_b.index(x)
            dst[t * n + hb] = src[t * n + ha]
    return dst


@pytest.mark.parametrize("dtype", [np.uint8, np.uint16, np.uint32, np.uint64])
def test_convert_brute_force_small(dtype):
    rng = np.random.default_rng(14)
    for d in [1, 2, 3, 5, 7, 8]:
        a, b = random_invertible(rng, d), random_invertible(rng, d)
        src = rng.integers(0, np.iinfo(dtype).max, size=3 << d, dtype=dtype)
        want = brute_convert(a, b, src, d)
        assert np.array_equal(oracle.convert(a, b, src), want)
        got_t, threads = oracle.convert(a, b, src, table=True)
        assert np.array_equal(got_t, want) and threads >= 1


def test_convert_is_bijective_and_round_trips():
    rng = np.random.default_rng(15)
    for d in [4, 9, 12, 14]:
        a, b = random_invertible(rng, d), random_invertible(rng, d)
        src = np.arange(2 << d, dtype=np.uint32)        # distinct values
        dst = oracle.convert(a, b, src)
        for t in range(2):                               # every slot written exactly once, tiles do not mix
            assert sorted(dst[t << d:(t + 1) << d]) == list(range(t << d, (t + 1) << d))
        assert np.array_equal(oracle.convert(b, a, dst), src)          # A->B->A = identity
        assert np.array_equal(oracle.convert(a, a, src), src)          # A = B is a copy


def test_convert_identity_on_shared_labels():
    # Sec. 5.4 rule 1: where A and B agree on a label, the conversion leaves that label alone.
    # A, B: same lane and wave columns, different register columns.
    rng = np.random.default_rng(16)
    nreg, nlane, nwave = 3, 4, 2
    d = nreg + nlane + nwave
    perm = random_bit_permutation(rng, d)
    a = perm
    regs = perm[:nreg]
    b = [regs[2], regs[0], regs[1]] + perm[nreg:]
    src = np.arange(1 << d, dtype=np.uint32)
    dst = oracle.convert(a, b, src)
    for hb in range(1 << d):
        ha = int(dst[hb])
        assert ha >> nreg == hb >> nreg          # lane and wave unchanged


def test_convert_config2_is_textbook_transpose():
    # Config 2: B is A with row and col bits swapped, so reading dst through A gives the
    # transposed logical tile.
    cfg = wl.config(2)
    a, b, d = cfg.src_bases, cfg.dst_bases, cfg.d
    rng = np.random.default_rng(17)
    src = rng.integers(0, 1 << 16, size=2 << d, dtype=np.uint16)
    dst = oracle.convert(a, b, src)
    inv_a = np.empty(1 << d, dtype=np.int64)
    inv_a[np_images(a, d)] = np.arange(1 << d)
    for t in range(2):
        logical_in = src[t << d:(t + 1) << d][inv_a].reshape(128, 128)     # in[r][c] = src[A^-1(r, c)]
        logical_out = dst[t << d:(t + 1) << d][inv_a].reshape(128, 128)    # dst read through A
        assert np.array_equal(logical_out, logical_in.T)


def test_convert_config1_hand_derived_values():
    # Hand derivation for config 1 (64x64, flat = col | row << 6), source index 0x123:
    #   reg = 3 -> col0, col1; lane = 0x12 -> lane bit 1 = col3, lane bit 4 = row0; wave 0
    #   logical = col0|col1|col3|row0 = 0b1001011 = 0x4B
    #   destination: col0, col1, col3 are lane bits 0, 1, 3; row0 is reg bit 0
    #   hB = reg 1 | lane 0b001011 << 4 = 0xB1
    cfg = wl.config(1)
    src = np.arange(1 << cfg.d, dtype=np.uint32)
    dst = oracle.convert(cfg.src_bases, cfg.dst_bases, src)
    assert int(dst[0xB1]) == 0x123
    assert int(dst[0]) == 0 and int(dst[0xFFF]) == 0xFFF
    # source bit 0 (col0) is destination lane bit 0 = index bit 4
    assert int(dst[0x010]) == 0x001


def test_convert_rejects_non_bijective():
    src = np.zeros(8, dtype=np.uint32)
    with pytest.raises(oracle.OracleError):
        oracle.convert([1, 2, 4], [1, 2, 3], src)
    with pytest.raises(oracle.OracleError):
        oracle.convert([1, 2, 0], [1, 2, 4], src)
    with pytest.raises(oracle.OracleError):
        oracle.convert([1, 2, 0], [1, 2, 4], src, table=True)


def test_convert_zero_tiles():
    out = oracle.convert([1, 2], [2, 1], np.zeros(0, dtype=np.uint32))
    assert out.size == 0


# ----------------------------------------------------------------------------
# gather
# ----------------------------------------------------------------------------

def logical_views(bases, d, img):
    """logical[x] = img[L^-1(x)] with L^-1 by linear search (numpy arithmetic)."""
    inv = np.empty(1 << d, dtype=np.int64)
    for h in range(1 << d):
        inv[np_apply(bases, d, h)] = h
    return img[inv], inv


@pytest.mark.parametrize("axis", [0, 1])
def test_gather_matches_take_along_axis(axis):
    rng = np.random.default_rng(18)
    dims = [3, 4]                                   # 8 x 16 logical tile
    d = sum(dims)
    for _ in range(4):
        bases = random_invertible(rng, d)
        inp = rng.integers(0, 1 << 16, size=1 << d, dtype=np.uint16)
        idx = rng.integers(0, 1 << dims[axis], size=1 << d, dtype=np.int32)
        out = oracle.gather(bases, dims, axis, inp, idx)
        in_log, inv = logical_views(bases, d, inp)
        idx_log, _ = logical_views(bases, d, idx)
        out_log, _ = logical_views(bases, d, out)
        shape = (1 << dims[0], 1 << dims[1])
        want = np.take_along_axis(in_log.reshape(shape), idx_log.reshape(shape).astype(np.int64), axis=axis)
        assert np.array_equal(out_log.reshape(shape), want)


def test_gather_identity_index_and_row_permutation():
    cfg = wl.config(5)
    d = cfg.d
    rng = np.random.default_rng(19)
    inp = rng.integers(0, 1 << 16, size=1 << d, dtype=np.uint16)
    inv = oracle.inverse_table(cfg.src_bases).astype(np.int64)
    rows = np.arange(1 << d) >> 8                   # logical flat = col | row << 8
    # idx[i, j] = i  =>  out == in
    idx_img = np.empty(1 << d, dtype=np.int32)
    idx_img[inv] = rows.astype(np.int32)
    assert np.array_equal(oracle.gather(cfg.src_bases, cfg.out_dim_bits, 0, inp, idx_img), inp)
    # idx[i, j] = perm[i]  =>  logical out = logical in with rows permuted
    perm = rng.permutation(64).astype(np.int32)
    idx_img[inv] = perm[rows]
    out = oracle.gather(cfg.src_bases, cfg.out_dim_bits, 0, inp, idx_img)
    assert np.array_equal(out[inv].reshape(64, 256), inp[inv].reshape(64, 256)[perm, :])


def test_gather_brute_force_4x4_loops():
    rng = np.random.default_rng(20)
    dims, d = [2, 2], 4
    bases = random_invertible(rng, d)
    inp = rng.integers(0, 255, size=2 << d, dtype=np.uint8)
    idx = rng.integers(0, 4, size=2 << d, dtype=np.int32)
    out = oracle.gather(bases, dims, 0, inp, idx)
    for t in range(2):
        where = {np_apply(bases, d, h): h for h in range(16)}     # logical flat -> hardware index
        for i in range(4):
            for j in range(4):
                s = int(idx[t * 16 + where[j | (i << 2)]])
                assert out[t * 16 + where[j | (i << 2)]] == inp[t * 16 + where[j | (s << 2)]]


def test_gather_out_of_range_index_wraps():
    dims, d = [2, 2], 4
    bases = [1, 2, 4, 8]
    inp = np.arange(16, dtype=np.uint32)
    idx = np.full(16, 5, dtype=np.int32)            # 5 & 3 == 1
    idx_ok = np.full(16, 1, dtype=np.int32)
    assert np.array_equal(oracle.gather(bases, dims, 0, inp, idx),
                          oracle.gather(bases, dims, 0, inp, idx_ok))


# ----------------------------------------------------------------------------
# wavefront (bank conflict) enumerator
# ----------------------------------------------------------------------------

def one_phase(nlanes):
    return [0] * nlanes


def test_wavefronts_row_major_textbook():
    # 32 x 32 fp32 tile stored row-major in 32 four-byte banks (the textbook case):
    # a wave reading one row touches 32 banks once; a wave reading one column hits one
    # bank 32 times.
    d = 10
    mem = [1 << k for k in range(d)]                       # offset = col | row << 5
    row_access = [1 << k for k in range(5, 10)] + [1 << k for k in range(0, 5)]   # regs->rows, lanes->cols
    col_access = [1 << k for k in range(0, 5)] + [1 << k for k in range(5, 10)]   # regs->cols, lanes->rows
    assert oracle.wavefronts(mem, row_access, 5, 5, 4, 0, 32, one_phase(32))[0] == 1
    mx, tot, nph = oracle.wavefronts(mem, col_access, 5, 5, 4, 0, 32, one_phase(32))
    assert (mx, tot, nph) == (32, 32 * 32, 32)


def test_wavefronts_padding_and_xor_swizzle_textbook():
    # offset = row * 32 + (col ^ row): both the row and the column access are conflict free.
    d = 10
    swz_inv_cols = [(1 << k) for k in range(5)] + [(1 << (5 + k)) | (1 << k) for k in range(5)]
    # swz_inv_cols is the map logical (col,row) -> offset; it is an involution, so it is also
    # the memory layout offset -> logical.
    row_access = [1 << k for k in range(5, 10)] + [1 << k for k in range(0, 5)]
    col_access = [1 << k for k in range(0, 5)] + [1 << k for k in range(5, 10)]
    assert oracle.wavefronts(swz_inv_cols, row_access, 5, 5, 4, 0, 32, one_phase(32))[0] == 1
    assert oracle.wavefronts(swz_inv_cols, col_access, 5, 5, 4, 0, 32, one_phase(32))[0] == 1


def test_wavefronts_same_word_is_a_broadcast():
    # two-byte elements: lanes l and l^1 share a 4-byte word -> still one wavefront
    d = 6
    mem = [1 << k for k in range(d)]
    access = [1 << 5] + [1 << k for k in range(5)]         # 1 reg bit (high), 5 lane bits (low)
    assert oracle.wavefronts(mem, access, 1, 5, 2, 0, 32, one_phase(32))[0] == 1


@pytest.mark.parametrize("vec_bits,elem_bytes", [(0, 4), (1, 4), (2, 4), (1, 2), (2, 2), (0, 8)])
def test_wavefronts_match_lemma_closed_form(vec_bits, elem_bytes):
    # Appendix lemma: with S = [vec | bank | idx] and a distributed layout L,
    #   c = |span(S_vec u S_idx) n span(L_thr)|, and the access takes n*c wavefronts when
    #   each vectorized element covers n = 2^v w / 4 >= 1 banks, with the hardware serving
    #   128-byte transactions (32 banks): a vectorized instruction is split so that each
    #   transaction holds 32/n lanes.
    rng = np.random.default_rng(21 + vec_bits * 7 + elem_bytes)
    nbanks = 32
    n_cover = (1 << vec_bits) * elem_bytes // 4
    if n_cover < 1:
        pytest.skip("lemma covers only 2^v w >= 4")
    nlane = 5
    for trial in range(12):
        nreg = vec_bits + int(rng.integers(0, 3))
        d = nreg + nlane + int(rng.integers(0, 2))
        b = 5 - (n_cover.bit_length() - 1)                # log2(128 / (2^v w))
        if vec_bits + b > d:
            continue
        mem = random_invertible(rng, d)                   # columns: vec | bank | idx
        s_vec, s_idx = mem[:vec_bits], mem[vec_bits + b:]
        # L: registers r0..r_{v-1} must be the memory vector (S_vec subset of L_reg, in order)
        rest = [x for x in random_invertible(rng, d)]
        basis, have = list(s_vec), span(s_vec)
        for x in rest:                                     # complete s_vec to a basis
            if x not in have:
                basis.append(x)
                have = span(basis)
        L = basis[:vec_bits] + list(rng.permutation(np.array(basis[vec_bits:], dtype=object)))
        L = [int(x) for x in L]
        l_thr = L[nreg:nreg + nlane]
        # transactions: lanes are served 32/n at a time, in order
        per = 32 // n_cover
        phases = [l // per for l in range(32)]
        # the lemma counts per instruction: c from the lanes of the whole wave; per phase the
        # count is the intersection with the span of the lane bits that vary inside a phase
        lanes_in_phase = l_thr[:per.bit_length() - 1]
        c_phase = len(span(s_vec + s_idx) & span(lanes_in_phase))
        mx, tot, nph = oracle.wavefronts(mem, L, nreg, nlane, elem_bytes, vec_bits, nbanks, phases)
        assert mx == c_phase and tot == c_phase * nph
        # whole-instruction form of the lemma: n * c wavefronts when nothing else collides
        c = len(span(s_vec + s_idx) & span(l_thr))
        if c == 1:
            assert tot == nph                               # conflict free: one wavefront per transaction


# ----------------------------------------------------------------------------
# broadcasting: right inverse with free variables zero, conversion between non-injective layouts
# ----------------------------------------------------------------------------

def random_surjective(rng, d_in, d_out):
    while True:
        cols = [int(rng.integers(0, 1 << d_out)) for _ in range(d_in)]
        cols[int(rng.integers(0, d_in))] = 0 if d_in > d_out else cols[0]      # make a zero column likely
        if len(span(cols)) == 1 << d_out:
            return cols


def test_right_inverse_small_hand_cases():
    # duplicated column: the leftmost copy is the pivot, the second stays zero
    assert list(oracle.right_inverse_table([1, 1, 2], 2)) == [0, 1, 4, 5]
    # zero column in the middle (Sec. 5.1: a zero register column = broadcast): never used
    assert list(oracle.right_inverse_table([1, 0, 2], 2)) == [0, 1, 4, 5]
    # third column = sum of the first two: free variable
    assert list(oracle.right_inverse_table([1, 2, 3, 4], 3)) == [0, 1, 2, 3, 8, 9, 10, 11]
    with pytest.raises(oracle.OracleError):
        oracle.right_inverse_table([1, 1, 1], 2)          # not surjective


def test_right_inverse_is_a_right_inverse_with_zero_free_variables():
    rng = np.random.default_rng(23)
    for d_in, d_out in [(4, 3), (6, 4), (9, 8), (12, 8), (5, 5)]:
        for _ in range(4):
            cols = random_surjective(rng, d_in, d_out)
            table = oracle.right_inverse_table(cols, d_out)
            # pivots = columns not in the span of the earlier ones (python sets, independent of the oracle)
            pivots, have = [], {0}
            for k, c in enumerate(cols):
                if c not in have:
                    pivots.append(k)
                    have |= {x ^ c for x in have}
            pivot_mask = sum(1 << k for k in pivots)
            for x in range(1 << d_out):
                h = int(table[x])
                assert np_apply(cols, d_out, h) == x           # M X = I
                assert h & ~pivot_mask == 0                    # free variables are zero
    # bijective case: coincides with the plain inverse
    cols = random_invertible(np.random.default_rng(24), 7)
    assert np.array_equal(oracle.right_inverse_table(cols, 7), oracle.inverse_table(cols))


def test_convert_general_delivers_the_logical_element():
    # "every destination unit receives the element at logical B(hB)": build a consistent source
    # image from a logical tensor X (src[hA] = X[A hA]); then dst[hB] must be X[B hB], whatever
    # representative the right inverse picks.
    rng = np.random.default_rng(25)
    for da, db, d_out in [(5, 4, 4), (4, 6, 4), (7, 7, 5), (10, 9, 8), (8, 8, 8)]:
        for _ in range(3):
            a, b = random_surjective(rng, da, d_out), random_surjective(rng, db, d_out)
            x_log = rng.integers(0, 1 << 32, size=2 << d_out, dtype=np.uint32).reshape(2, -1)
            src = np.stack([x_log[t][np_images(a, da) if da == d_out else
                                     np.array([np_apply(a, d_out, h) for h in range(1 << da)])] for t in range(2)]).reshape(-1)
            dst = oracle.convert_general(a, b, d_out, src)
            img_b = np.array([np_apply(b, d_out, h) for h in range(1 << db)])
            want = np.stack([x_log[t][img_b] for t in range(2)]).reshape(-1)
            assert np.array_equal(dst, want)


def test_convert_general_reads_the_canonical_source_unit():
    # inconsistent source (replicas differ): the value must come from the unit with free variables zero
    a = [1, 1, 2]          # bits 0 and 1 of the source index are replicas of logical bit 0
    b = [1, 2]
    src = np.arange(8, dtype=np.uint32) + 100
    dst = oracle.convert_general(a, b, 2, src)
    assert list(dst) == [100 + 0, 100 + 1, 100 + 4, 100 + 5]
    # bijective layouts: same as the plain conversion
    rng = np.random.default_rng(26)
    a, b = random_invertible(rng, 6), random_invertible(rng, 6)
    src = rng.integers(0, 1 << 16, size=3 << 6, dtype=np.uint16)
    assert np.array_equal(oracle.convert_general(a, b, 6, src), oracle.convert(a, b, src))


def test_convert_general_paper_broadcast_example(golden_dir):
    # Sec. 5.1: a zero column added to A_reg makes registers 4-7 hold the same elements as 0-3.
    a = load_layout_a(golden_dir)
    widened = a[:2] + [0] + a[2:]
    rng = np.random.default_rng(27)
    src = rng.integers(0, 1 << 32, size=256, dtype=np.uint32)             # image under Layout A
    wide = oracle.convert_general(a, widened, 8, src)                    # 512 elements
    for h in range(512):
        reg, rest = h & 7, h >> 3
        assert wide[h] == src[(reg & 3) | (rest << 2)]                    # registers 4-7 alias 0-3
    back = oracle.convert_general(widened, a, 8, wide)
    assert np.array_equal(back, src)


def test_convert_spot_values_of_the_configurations(golden_dir):
    """tests/golden/config_spot_values.txt: hand-derived (source index, destination index) pairs of
    configs 1-3 and the image of every source bit of config 1."""
    rows = [l.split() for l in open(os.path.join(golden_dir, "config_spot_values.txt")) if l.strip() and not l.startswith("#")]
    images = {}
    for cid in (1, 2, 3):
        cfg = wl.config(cid)
        images[cid] = oracle.convert(cfg.src_bases, cfg.dst_bases, np.arange(1 << cfg.d, dtype=np.uint32))
        assert int(images[cid][0]) == 0 and int(images[cid][-1]) == (1 << cfg.d) - 1
    seen = 0
    for r in rows:
        if r[0] == "P":
            for k, col in enumerate(r[1:]):
                assert int(images[1][int(col, 16)]) == 1 << k
            assert len(r) == 13
        else:
            assert int(images[int(r[0])][int(r[2], 16)]) == int(r[1], 16), r
            seen += 1
    assert seen == 12


# ----------------------------------------------------------------------------
# table variants used to check whole full-size images: the same results as the plain functions
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("axis", [0, 1])
def test_gather_table_matches_take_along_axis_and_the_plain_function(axis):
    rng = np.random.default_rng(180 + axis)
    for dims, dtype, ntiles in (([3, 4], np.uint16, 1), ([5, 2], np.uint8, 37), ([4, 6], np.uint32, 5), ([6, 8], np.uint64, 3)):
        d = sum(dims)
        bases = random_invertible(rng, d)
        inp = rng.integers(0, np.iinfo(dtype).max, size=ntiles << d, dtype=dtype)
        idx = rng.integers(-(1 << dims[axis]), 2 << dims[axis], size=ntiles << d, dtype=np.int32)     # out of range: wraps
        out = oracle.gather(bases, dims, axis, inp, idx, table=True)
        assert np.array_equal(out, oracle.gather(bases, dims, axis, inp, idx))
        shape = (1 << dims[0], 1 << dims[1])
        for t in range(ntiles):                       # and against numpy on the logical views, tile by tile
            sl = slice(t << d, (t + 1) << d)
            in_log, _ = logical_views(bases, d, inp[sl])
            idx_log, _ = logical_views(bases, d, idx[sl])
            out_log, _ = logical_views(bases, d, out[sl])
            want = np.take_along_axis(in_log.reshape(shape), (idx_log.reshape(shape) & ((1 << dims[axis]) - 1)).astype(np.int64), axis=axis)
            assert np.array_equal(out_log.reshape(shape), want)


def test_gather_table_rejects_what_the_plain_function_rejects():
    singular = [1, 2, 3, 8]
    img = np.zeros(16, dtype=np.uint16)
    idx = np.zeros(16, dtype=np.int32)
    for table in (False, True):
        with pytest.raises(oracle.OracleError):
            oracle.gather(singular, [2, 2], 0, img, idx, table=table)
        with pytest.raises(oracle.OracleError):
            oracle.gather([1, 2, 4, 8], [2, 2], 2, img, idx, table=table)


def test_convert_general_table_matches_the_plain_function_and_the_logical_element():
    rng = np.random.default_rng(250)
    for da, db, d_out, ntiles in [(5, 4, 4, 1), (4, 6, 4, 19), (7, 7, 5, 3), (10, 9, 8, 6), (8, 8, 8, 2)]:
        for dtype in (np.uint8, np.uint32, np.uint64):
            a, b = random_surjective(rng, da, d_out), random_surjective(rng, db, d_out)
            src = rng.integers(0, np.iinfo(dtype).max, size=ntiles << da, dtype=dtype)      # replicas differ
            got = oracle.convert_general(a, b, d_out, src, table=True)
            assert np.array_equal(got, oracle.convert_general(a, b, d_out, src))
            # independent of the plain function: from a consistent source, slot hB receives X[B hB]
            x_log = rng.integers(0, np.iinfo(dtype).max, size=ntiles << d_out, dtype=dtype).reshape(ntiles, -1)
            img_a = np.array([np_apply(a, d_out, h) for h in range(1 << da)])
            img_b = np.array([np_apply(b, d_out, h) for h in range(1 << db)])
            src2 = np.stack([x_log[t][img_a] for t in range(ntiles)]).reshape(-1)
            want = np.stack([x_log[t][img_b] for t in range(ntiles)]).reshape(-1)
            assert np.array_equal(oracle.convert_general(a, b, d_out, src2, table=True), want)
    with pytest.raises(oracle.OracleError):
        oracle.convert_general([1, 1], [1, 2], 2, np.zeros(4, dtype=np.uint8), table=True)      # A misses part of the tensor
