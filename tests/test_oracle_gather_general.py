"""Pins of the oracle's gather under broadcasting layouts (Sec. 5.5 with Sec. 5.1 "Broadcasting").

The function is pinned through the logical view (numpy take_along_axis), through its reduction to
the plain gather, by its definition evaluated slot by slot, and by a hand-worked example."""
import numpy as np
import pytest

import oracle


def apply(bases, h):
    x = 0
    for k, c in enumerate(bases):
        if (h >> k) & 1:
            x ^= c
    return x


def surjective_with_replicas(rng, d_in, d_out):
    """Random surjective layout on d_in > d_out bits with at least one zero column."""
    while True:
        cols = [int(rng.integers(0, 1 << d_out)) for _ in range(d_in)]
        cols[int(rng.integers(0, d_in))] = 0
        span = {0}
        for c in cols:
            span |= {x ^ c for x in span}
        if len(span) == 1 << d_out:
            return cols


def image_of(logical, bases, d_in, off=0):
    """Image of a logical tensor under the layout: slot h holds logical[L h ^ off] (all replicas equal)."""
    flat = logical.reshape(-1)
    return np.array([flat[apply(bases, h) ^ off] for h in range(1 << d_in)], dtype=flat.dtype)


@pytest.mark.parametrize("dims", [[3, 3], [2, 2, 2], [5], [1, 4]])
def test_consistent_replicas_give_the_image_of_take_along_axis(dims):
    rng = np.random.default_rng(100 + len(dims) + dims[0])
    d_out = sum(dims)
    shape = [1 << b for b in dims]
    for d_in in (d_out + 1, d_out + 3):
        for trial in range(4):
            bases = surjective_with_replicas(rng, d_in, d_out)
            off = int(rng.integers(0, 1 << d_out)) if trial % 2 else 0
            for axis in range(len(dims)):
                ntiles = 3
                imgs_in, imgs_idx, want = [], [], []
                for t in range(ntiles):
                    lin = rng.integers(0, 1 << 30, size=shape, dtype=np.int64).astype(np.uint32)
                    lidx = rng.integers(0, shape[axis], size=shape).astype(np.int32)
                    imgs_in.append(image_of(lin, bases, d_in, off))
                    imgs_idx.append(image_of(lidx, bases, d_in, off))
                    want.append(image_of(np.take_along_axis(lin, lidx.astype(np.int64), axis=axis), bases, d_in, off))
                got = oracle.gather_general(bases, dims, axis, np.concatenate(imgs_in), np.concatenate(imgs_idx), off)
                assert np.array_equal(got, np.concatenate(want)), (bases, axis, off)


def test_bijective_layouts_reduce_to_the_plain_gather():
    rng = np.random.default_rng(5)
    for dims in ([4, 4], [3, 2, 3], [8]):
        d = sum(dims)
        while True:
            bases = [int(rng.integers(1, 1 << d)) for _ in range(d)]
            span = {0}
            for c in bases:
                span |= {x ^ c for x in span}
            if len(span) == 1 << d:
                break
        inp = rng.integers(0, 1 << 16, size=5 << d).astype(np.uint16)
        for axis in range(len(dims)):
            idx = rng.integers(-50, 50, size=5 << d).astype(np.int32)
            assert np.array_equal(oracle.gather_general(bases, dims, axis, inp, idx), oracle.gather(bases, dims, axis, inp, idx))
            off = int(rng.integers(0, 1 << d))
            assert np.array_equal(oracle.gather_general(bases, dims, axis, inp, idx, off),
                                  oracle.gather_affine(bases, off, dims, axis, inp, idx))


def test_every_slot_uses_its_own_index_and_unequal_replicas_of_in_are_refused():
    """Replicas of idx may differ: every slot of out is filled from its own slot of idx.  Replicas of
    `in` may not: the result would depend on a choice the paper does not make."""
    rng = np.random.default_rng(9)
    dims, d_in = [3, 2], 8
    d_out = sum(dims)
    for trial in range(6):
        bases = surjective_with_replicas(rng, d_in, d_out)
        for axis in range(2):
            shift = sum(dims[axis + 1:])
            mask = (1 << dims[axis]) - 1
            logical = rng.integers(0, 1 << 30, size=1 << d_out).astype(np.uint32)
            inp = image_of(logical, bases, d_in)
            idx = rng.integers(-9, 9 + (1 << dims[axis]), size=1 << d_in).astype(np.int32)    # replicas of idx differ on purpose
            got = oracle.gather_general(bases, dims, axis, inp, idx)
            for h in range(1 << d_in):
                x = apply(bases, h)
                wanted = (x & ~(mask << shift)) | ((int(idx[h]) & mask) << shift)
                assert got[h] == logical[wanted]
            assert np.array_equal(oracle.consistent_image(bases, d_out, inp), inp)
            broken = inp.copy()
            lplus = oracle.right_inverse_table(bases, d_out)
            replica = next(h for h in range(1 << d_in) if int(lplus[apply(bases, h)]) != h)      # a non-canonical slot
            broken[replica] ^= 1
            with pytest.raises(ValueError):
                oracle.gather_general(bases, dims, axis, broken, idx)
            assert np.array_equal(oracle.consistent_image(bases, d_out, broken), inp)            # the canonical slots decide


def test_worked_example_one_zero_column():
    """4 logical elements (one dim), registers [e0, 0, e1]: slot h = r0 + 2 r1 + 4 r2 holds element
    r0 + 2 r2; r1 enumerates two replicas.  X = (10, 11, 12, 13) lies at slots (0, 1, 4, 5) and again at
    (2, 3, 6, 7).  Slot 6 (element 2, second replica) asks for element 1 and gets 11; all others ask for
    element 0 and get 10."""
    bases = [1, 0, 2]
    inp = np.array([10, 11, 10, 11, 12, 13, 12, 13], dtype=np.uint8)
    idx = np.zeros(8, dtype=np.int32)
    idx[6] = 1
    out = oracle.gather_general(bases, [2], 0, inp, idx)
    assert list(out) == [10, 10, 10, 10, 10, 10, 11, 10]
