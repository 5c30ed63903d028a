"""Layout families of the CPU oracle: identity maps between labelled dims, blocked layouts, matrix-
instruction tiles as products of identities, the legacy `mma` swizzle, and the two family
definitions (distributed / memory layout).

TEST INFRASTRUCTURE ONLY (see the package docstring).  Each function follows the passage it cites,
step by step, on the explicit objects of `oracle.algebra`.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np

from .algebra import OLayout, product, to_matrix


def identity_map(label: int, dim: int, k: int, n_dims: int) -> OLayout:
    """Appendix "Notation": id_k^{label, dim}, the k x k identity from the first k bits of input
    label `label` to the first k bits of logical dim `dim` (dims numbered slowest first)."""
    out = [0] * n_dims
    out[dim] = k
    shift = 0                                        # the other dims have no bits: dim's bit 0 is flat bit 0
    return OLayout([(label, k)], out, [1 << (shift + i) for i in range(k)])


def product_of(factors: Sequence[OLayout]) -> OLayout:
    """Left-to-right label-wise product: later factors take the next bits of their label and dim."""
    acc = factors[0]
    for f in factors[1:]:
        acc = product(acc, f)
    return acc


def blocked_layout(reg_bits: Sequence[int], lane_bits: Sequence[int], wave_bits: Sequence[int],
                   order: Sequence[int], labels=(0, 1, 2)) -> OLayout:
    """Proposition "Blocked layouts are linear layouts" (appendix): with R, T, W the log2 numbers
    of registers, threads and warps per dim and `order[i]` the i-th fastest dim,
    id_R^o x id_T^o x id_W^o where id_X^o = id_{x_{o_1}}^{label, o_1} x ... x id_{x_{o_l}}^{label, o_l}.
    Output dims keep their names, so the permutation sigma_o^{-1} of the statement is already
    applied."""
    n = len(order)
    factors: List[OLayout] = []
    for label, bits in zip(labels, (reg_bits, lane_bits, wave_bits)):
        for dim in order:
            factors.append(identity_map(label, dim, bits[dim], n))
    return product_of(factors)


def mfma_accumulator_tile(m_bits: int, reg=0, lane=1) -> OLayout:
    """Output tile of a CDNA matrix instruction with a 2^m x 2^m fp32 result on 64 lanes (m = 4 or 5),
    written as a product of identities in the manner of the appendix's proof for `mma`:
    a lane holds 4 consecutive rows of one column; the lane index runs along the column index
    first and then along the row blocks; further registers step over the remaining row blocks.
        id_2^{reg,0} x id_m^{lane,1} x id_{6-m}^{lane,0} x id_{2m-8}^{reg,0}"""
    return product_of([identity_map(reg, 0, 2, 2), identity_map(lane, 1, m_bits, 2),
                       identity_map(lane, 0, 6 - m_bits, 2), identity_map(reg, 0, 2 * m_bits - 8, 2)])


def mfma_operand_tile(m_bits: int, k_reg_bits: int, reg=0, lane=1) -> OLayout:
    """Left-hand operand tile (2^m rows x K) of the same instructions: a lane holds 2^k_reg_bits
    consecutive elements along K for one row; lanes run along the rows first, then along K.
        id_{kr}^{reg,1} x id_m^{lane,0} x id_{6-m}^{lane,1}"""
    return product_of([identity_map(reg, 1, k_reg_bits, 2), identity_map(lane, 0, m_bits, 2),
                       identity_map(lane, 1, 6 - m_bits, 2)])


def mma_swizzle_offset(i: int, j: int, n_bits: int, vec: int, per_phase: int, max_phase: int) -> int:
    """Def. "mma swizzling": the offset (in elements) of location (i, j) of a row-major
    2^m x 2^n tensor: the row keeps its place, inside the row
    ((i / per_phase mod max_phase) xor j / vec) * vec xor (j mod vec)."""
    inside = ((((i // per_phase) % max_phase) ^ (j // vec)) * vec) ^ (j % vec)
    return (i << n_bits) | inside


def mma_swizzle_layout(m_bits: int, n_bits: int, vec: int, per_phase: int, max_phase: int) -> OLayout:
    """The memory layout (offset -> logical (i, j)) of the swizzle: tabulate the definition for all
    locations, invert the table, read the images of the offset bits off it."""
    size = 1 << (m_bits + n_bits)
    where = np.full(size, -1, dtype=np.int64)        # offset -> flattened location
    for i in range(1 << m_bits):
        for j in range(1 << n_bits):
            off = mma_swizzle_offset(i, j, n_bits, vec, per_phase, max_phase)
            if off >= size or where[off] >= 0:
                raise ValueError("the swizzle parameters do not give a bijection")
            where[off] = (i << n_bits) | j
    bases = [int(where[1 << k]) for k in range(m_bits + n_bits)]
    # linearity of the tabulated map (Proposition "MMA swizzled layouts are linear layouts")
    for off in range(size):
        acc = 0
        for k in range(m_bits + n_bits):
            if (off >> k) & 1:
                acc ^= bases[k]
        if acc != int(where[off]):
            raise ValueError("the tabulated swizzle is not linear")
    return OLayout([(4, m_bits + n_bits)], [m_bits, n_bits], bases)


def slice_layout(lay: OLayout, dim: int) -> OLayout:
    """Sec. 4.3 "Sliced Layouts" (the layout of the result of a reduction along `dim`): removing a
    logical dim is the linear map that deletes that dim's rows of the matrix.  Inputs keep their
    labels and sizes; columns that ran along the removed dim become zero (the result is broadcast
    over them), and a surjective layout stays surjective."""
    if not 0 <= dim < len(lay.out_dims) or len(lay.out_dims) < 2:
        raise ValueError("slice needs a layout of at least two dims and a dim inside it")
    m = to_matrix(lay)
    lo = sum(lay.out_dims[dim + 1:])                 # flat position of bit 0 of `dim`
    keep = [r for r in range(lay.d_out) if not lo <= r < lo + lay.out_dims[dim]]
    out_dims = [n for j, n in enumerate(lay.out_dims) if j != dim]
    bases = [int(sum(int(m[r, c]) << i for i, r in enumerate(keep))) for c in range(lay.d_in)]
    offset = sum(((lay.offset >> r) & 1) << i for i, r in enumerate(keep))      # the constant loses the same rows
    return OLayout(list(lay.in_dims), out_dims, bases, offset)


def is_distributed_layout(lay: OLayout) -> bool:
    """Def. "Distributed Layout": surjective, every column has at most one non-zero bit, and no
    non-zero column is repeated (a permutation matrix with zero columns interleaved)."""
    m = to_matrix(lay)
    nonzero = []
    for c in range(m.shape[1]):
        ones = int(m[:, c].sum())
        if ones > 1:
            return False
        if ones == 1:
            nonzero.append(int(np.argmax(m[:, c])))
    if len(set(nonzero)) != len(nonzero):
        return False
    return len(set(nonzero)) == lay.d_out            # surjective: every output bit is hit


def is_memory_layout(lay: OLayout) -> bool:
    """Def. "Memory Layout": invertible, every column has one or two non-zero bits."""
    m = to_matrix(lay)
    if m.shape[0] != m.shape[1]:
        return False
    if any(int(m[:, c].sum()) not in (1, 2) for c in range(m.shape[1])):
        return False
    images = set()
    for h in range(1 << lay.d_in):                   # invertible: all images distinct
        v = 0
        for k in range(lay.d_in):
            if (h >> k) & 1:
                v ^= lay.bases[k]
        images.add(v)
    return len(images) == (1 << lay.d_in)
