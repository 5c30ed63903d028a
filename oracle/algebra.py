"""Layout algebra of the CPU oracle: label-wise product and left division, contiguity.

TEST INFRASTRUCTURE ONLY (see the package docstring).  Everything here works on explicit
0/1 numpy matrices, entry by entry, exactly as the definitions are stated:

* a layout is a matrix over F2 whose columns are the images of the input bits (Sec. 4.1);
  inputs carry labels (register, lane, wave, ...), outputs are the logical dims, last fastest;
* Def. "Product": L1 x L2 is the block-diagonal matrix [[L1, 0], [0, L2]], taken label-wise:
  inside every input label and inside every output dim the bits of L1 sit below those of L2;
* Def. "Left Division": M is divisible on the left by M1 if, with rows and columns grouped
  label-wise, M = [[M1, 0], [0, M2]]; the quotient is M2;
* Sec. 5.1 "Contiguous elements": the largest run of consecutive logical elements that
  consecutive registers of one thread hold.
"""
from __future__ import annotations

from dataclasses import dataclass
from itertools import permutations
from typing import List, Optional, Sequence, Tuple

import numpy as np


@dataclass
class OLayout:
    in_dims: List[Tuple[int, int]]      # (label, bits), in input-bit order
    out_dims: List[int]                 # bits per logical dim, slowest first
    bases: List[int]                    # image of every input bit, flattened (last dim fastest)
    offset: int = 0                     # affine layouts (Conclusions): index h holds element (bases h) xor offset

    @property
    def d_in(self) -> int:
        return sum(n for _, n in self.in_dims)

    @property
    def d_out(self) -> int:
        return sum(self.out_dims)


def out_shift(out_dims: Sequence[int], j: int) -> int:
    """Position of bit 0 of logical dim j in the flattened index (last dim fastest)."""
    return sum(out_dims[j + 1:])


def to_matrix(lay: OLayout) -> np.ndarray:
    """Rows = flattened output bits, columns = input bits, entries 0/1."""
    m = np.zeros((lay.d_out, lay.d_in), dtype=np.uint8)
    for c, b in enumerate(lay.bases):
        for r in range(lay.d_out):
            m[r, c] = (b >> r) & 1
    return m


def split_dims(x: int, out_dims: Sequence[int]) -> List[int]:
    """Per-dim coordinates of a flattened index (slowest dim first)."""
    return [(x >> out_shift(out_dims, j)) & ((1 << n) - 1) for j, n in enumerate(out_dims)]


def join_dims(coords: Sequence[int], out_dims: Sequence[int]) -> int:
    return sum(c << out_shift(out_dims, j) for j, c in enumerate(coords))


def from_matrix(m: np.ndarray, in_dims, out_dims) -> OLayout:
    bases = [int(sum(int(m[r, c]) << r for r in range(m.shape[0]))) for c in range(m.shape[1])]
    return OLayout(list(in_dims), list(out_dims), bases)


def _input_positions(lay: OLayout, label: int) -> List[int]:
    pos, out = 0, []
    for l, n in lay.in_dims:
        if l == label:
            out.extend(range(pos, pos + n))
        pos += n
    return out


def product(a: OLayout, b: OLayout) -> OLayout:
    """Def. "Product", label-wise on inputs and dim-wise on outputs (same number of dims)."""
    if len(a.out_dims) != len(b.out_dims):
        raise ValueError("product needs the same number of logical dims")
    labels = []
    for l, _ in a.in_dims + b.in_dims:
        if l not in labels:
            labels.append(l)
    labels.sort()
    out_dims = [x + y for x, y in zip(a.out_dims, b.out_dims)]
    ma, mb = to_matrix(a), to_matrix(b)
    # row of the result that holds bit i of dim j of a (or of b)
    def row_of(which, j, i):
        return out_shift(out_dims, j) + (i if which == 0 else a.out_dims[j] + i)
    in_dims, cols = [], []
    for l in labels:
        pa, pb = _input_positions(a, l), _input_positions(b, l)
        in_dims.append((l, len(pa) + len(pb)))
        for which, lay, mat, plist in ((0, a, ma, pa), (1, b, mb, pb)):
            for c in plist:
                col = np.zeros(sum(out_dims), dtype=np.uint8)
                for j, nb in enumerate(lay.out_dims):
                    for i in range(nb):
                        col[row_of(which, j, i)] = mat[out_shift(lay.out_dims, j) + i, c]
                cols.append(col)
    full = np.stack(cols, axis=1) if cols else np.zeros((sum(out_dims), 0), dtype=np.uint8)
    res = from_matrix(full, in_dims, out_dims)
    # affine factors: element (x1 ^ b1, x2 ^ b2) per dim, a's bits below b's
    res.offset = join_dims([ca | (cb << a.out_dims[j]) for j, (ca, cb) in
                            enumerate(zip(split_dims(a.offset, a.out_dims), split_dims(b.offset, b.out_dims)))], out_dims)
    return res


def divide_left(lay: OLayout, tile: OLayout) -> Optional[OLayout]:
    """Def. "Left Division": the M2 with lay = tile x M2 (label-wise), or None if lay does not have
    that structure.  The tile's input labels must occur in `lay` and it must have as many logical
    dims; the tile owns the low bits of each of its labels and of every logical dim."""
    if len(tile.out_dims) != len(lay.out_dims):
        return None
    if any(t > l for t, l in zip(tile.out_dims, lay.out_dims)):
        return None
    m, mt = to_matrix(lay), to_matrix(tile)
    tile_cols, rest_cols, q_in = [], [], []
    for l, n in lay.in_dims:
        pos = _input_positions(lay, l)
        nt = len(_input_positions(tile, l))
        if nt > n:
            return None
        tile_cols.extend(pos[:nt])
        rest_cols.extend(pos[nt:])
        q_in.append((l, n - nt))
    if any(l not in [x for x, _ in lay.in_dims] for l, n in tile.in_dims if n > 0):
        return None
    # the tile's own column order, label by label, as it sits inside `lay`
    tile_own = []
    for l, _ in lay.in_dims:
        tile_own.extend(_input_positions(tile, l))
    tile_rows, rest_rows, tile_own_rows = [], [], []
    for j, nb in enumerate(lay.out_dims):
        for i in range(nb):
            r = out_shift(lay.out_dims, j) + i
            (tile_rows if i < tile.out_dims[j] else rest_rows).append(r)
    # rows of the tile matrix in the same (dim, bit) order as tile_rows: fastest dim first
    tile_rows_sorted = sorted(tile_rows)
    for r in tile_rows_sorted:
        # which (dim, bit) is row r of lay?
        for j, nb in enumerate(lay.out_dims):
            s = out_shift(lay.out_dims, j)
            if s <= r < s + nb:
                tile_own_rows.append(out_shift(tile.out_dims, j) + (r - s))
    top_left = m[np.ix_(tile_rows_sorted, tile_cols)]
    top_right = m[np.ix_(tile_rows_sorted, rest_cols)]
    bottom_left = m[np.ix_(sorted(rest_rows), tile_cols)]
    bottom_right = m[np.ix_(sorted(rest_rows), rest_cols)]
    if not np.array_equal(top_left, mt[np.ix_(tile_own_rows, tile_own)]):
        return None
    if top_right.any() or bottom_left.any():
        return None
    q_out = [l - t for l, t in zip(lay.out_dims, tile.out_dims)]
    q = from_matrix(bottom_right, q_in, q_out)
    # affine layouts: lay = tile x q also for the constants, dim by dim
    lo, to = split_dims(lay.offset, lay.out_dims), split_dims(tile.offset, tile.out_dims)
    if any((l & ((1 << tb) - 1)) != t for l, t, tb in zip(lo, to, tile.out_dims)):
        return None
    q.offset = join_dims([l >> tb for l, tb in zip(lo, tile.out_dims)], q_out)
    return q


def divide_left_permuting(lay: OLayout, tile: OLayout, label: int):
    """Sec. 5.3 "Generalized Vectorization": a permutation of the input bits of `label` after
    which the layout is divisible by the tile.  Returns (permutation, quotient) with
    new_bit[k] = old bit permutation[k], or None.  Brute force over permutations (tiny inputs)."""
    pos = _input_positions(lay, label)
    for perm in permutations(range(len(pos))):
        bases = list(lay.bases)
        for k, src in enumerate(perm):
            bases[pos[k]] = lay.bases[pos[src]]
        q = divide_left(OLayout(lay.in_dims, lay.out_dims, bases, lay.offset), tile)
        if q is not None:
            return list(perm), q
    return None


def contiguity(lay: OLayout, reg_label: int = 0) -> int:
    """Sec. 5.1 "Contiguous elements": the number c of leading logical elements x0..x0+c-1 that the
    inverse of the layout sends, by the identity map, onto registers 0..c-1 (of thread 0, wave 0):
    the largest block that one thread can move with a single vector access.  Taken literally on
    the tabulated inverse; the register bits must be the first input bits.  x0 is the element of
    register 0: 0 for a linear layout, the constant for an affine one (slot h holds L h ^ offset, so
    element x sits at the inverse of x ^ offset)."""
    from . import right_inverse_table
    if not lay.in_dims or lay.in_dims[0][0] != reg_label:
        return 1
    nreg = lay.in_dims[0][1]
    table = right_inverse_table(lay.bases, lay.d_out)
    c = 0
    x0 = lay.offset
    while c < min(1 << nreg, 1 << lay.d_out) and x0 + c < (1 << lay.d_out) and int(table[(x0 + c) ^ lay.offset]) == c:
        c += 1
    return max(c, 1)


def identity_tile(label: int, bits: int, n_out_dims: int = 1) -> OLayout:
    """The tile of a vectorized access (Sec. 5.3): identity from `bits` input bits of `label` to the
    low `bits` bits of the fastest logical dim."""
    out = [0] * (n_out_dims - 1) + [bits]
    return OLayout([(label, bits)], out, [1 << k for k in range(bits)])
