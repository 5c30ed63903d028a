"""CPU oracle for the Linear-Layouts conversion / gather hot path.

TEST INFRASTRUCTURE ONLY: imported by tests/, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  The product package never
imports this module, and this module never imports the product package.

The arithmetic lives in ``ll_oracle.c`` (plain C, written from the paper's
definitions); this file only builds that C file with gcc and marshals numpy
arrays into it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ll_oracle.c")
_LIB = os.path.join(_HERE, "libll_oracle.so")

OK, ERR_ARG, ERR_NOT_BIJECTIVE, ERR_AXIS, ERR_ALLOC = 0, 1, 2, 3, 4


class OracleError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"oracle {what} failed with status {code}")
        self.code = code


def build(force: bool = False) -> str:
    """Compile ll_oracle.c into libll_oracle.so (gcc, OpenMP for the table variant)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u64p = ctypes.POINTER(ctypes.c_uint64)
        i32p = ctypes.POINTER(ctypes.c_int32)
        i64p = ctypes.POINTER(ctypes.c_int64)
        lib.oracle_apply.restype = ctypes.c_uint64
        lib.oracle_apply.argtypes = [u64p, ctypes.c_int, ctypes.c_uint64]
        lib.oracle_compose.restype = ctypes.c_int
        lib.oracle_compose.argtypes = [u64p, ctypes.c_int, ctypes.c_int, u64p, ctypes.c_int, u64p]
        lib.oracle_inverse_table.restype = ctypes.c_int
        lib.oracle_inverse_table.argtypes = [u64p, ctypes.c_int, ctypes.POINTER(ctypes.c_uint32)]
        lib.oracle_right_inverse_table.restype = ctypes.c_int
        lib.oracle_right_inverse_table.argtypes = [u64p, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_uint32)]
        lib.oracle_convert_general.restype = ctypes.c_int
        lib.oracle_convert_general.argtypes = [u64p, ctypes.c_int, u64p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                               ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64]
        lib.oracle_convert_general_affine.restype = ctypes.c_int
        lib.oracle_convert_general_affine.argtypes = [u64p, ctypes.c_uint64, ctypes.c_int, u64p, ctypes.c_uint64, ctypes.c_int,
                                                      ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64]
        lib.oracle_convert.restype = ctypes.c_int
        lib.oracle_convert.argtypes = [u64p, u64p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                       ctypes.c_void_p, ctypes.c_int64]
        lib.oracle_convert_table.restype = ctypes.c_int
        lib.oracle_convert_table.argtypes = [u64p, u64p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                             ctypes.c_void_p, ctypes.c_int64,
                                             ctypes.POINTER(ctypes.c_int)]
        lib.oracle_convert_affine.restype = ctypes.c_int
        lib.oracle_convert_affine.argtypes = [u64p, ctypes.c_uint64, u64p, ctypes.c_uint64, ctypes.c_int, ctypes.c_int,
                                              ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64]
        lib.oracle_gather_affine.restype = ctypes.c_int
        lib.oracle_gather_affine.argtypes = [u64p, ctypes.c_uint64, ctypes.c_int, i32p, ctypes.c_int, ctypes.c_int,
                                             ctypes.c_int, ctypes.c_void_p, i32p, ctypes.c_void_p, ctypes.c_int64]
        lib.oracle_gather.restype = ctypes.c_int
        lib.oracle_gather.argtypes = [u64p, ctypes.c_int, i32p, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_int, ctypes.c_void_p, i32p, ctypes.c_void_p,
                                      ctypes.c_int64]
        lib.oracle_gather_table.restype = ctypes.c_int
        lib.oracle_gather_table.argtypes = lib.oracle_gather.argtypes
        lib.oracle_convert_general_table.restype = ctypes.c_int
        lib.oracle_convert_general_table.argtypes = lib.oracle_convert_general.argtypes
        lib.oracle_wavefronts.restype = ctypes.c_int
        lib.oracle_wavefronts.argtypes = [u64p, u64p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                          ctypes.c_int, ctypes.c_int, ctypes.c_int, i32p,
                                          i64p, i64p, i64p]
        _lib = lib
    return _lib


def _u64(bases: Sequence[int]):
    arr = (ctypes.c_uint64 * len(bases))(*[int(b) for b in bases])
    return arr


def apply(bases: Sequence[int], h: int) -> int:
    """L(h): XOR of the columns selected by the set bits of h."""
    return int(_load().oracle_apply(_u64(bases), len(bases), int(h)))


def compose(outer: Sequence[int], d_out: int, inner: Sequence[int]) -> list:
    """Columns of outer o inner (matrix product over F2)."""
    res = (ctypes.c_uint64 * len(inner))()
    rc = _load().oracle_compose(_u64(outer), len(outer), d_out, _u64(inner), len(inner), res)
    if rc != OK:
        raise OracleError(rc, "compose")
    return [int(x) for x in res]


def inverse_table(bases: Sequence[int]) -> np.ndarray:
    """table[L(h)] = h for a bijective layout on len(bases) bits."""
    d = len(bases)
    table = np.empty(1 << d, dtype=np.uint32)
    rc = _load().oracle_inverse_table(_u64(bases), d,
                                      table.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)))
    if rc != OK:
        raise OracleError(rc, "inverse_table")
    return table


def right_inverse_table(bases: Sequence[int], d_out: int) -> np.ndarray:
    """table[x] = the h with L(h) = x whose free variables are zero (surjective L, broadcasting allowed)."""
    table = np.empty(1 << d_out, dtype=np.uint32)
    rc = _load().oracle_right_inverse_table(_u64(bases), len(bases), d_out,
                                            table.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)))
    if rc != OK:
        raise OracleError(rc, "right_inverse_table")
    return table


def convert_general(bases_a: Sequence[int], bases_b: Sequence[int], d_out: int, src: np.ndarray,
                    table: bool = False) -> np.ndarray:
    """Conversion with broadcasting: dst[hB] = src[A^+(B hB)]; src holds ntiles * 2^len(A) elements.
    table=True: the same with the pull map tabulated once and tiles on all host threads."""
    da, db = len(bases_a), len(bases_b)
    _check_img(src, da, "src")
    ntiles = src.size >> da
    dst = np.empty(ntiles << db, dtype=src.dtype)
    fn = _load().oracle_convert_general_table if table else _load().oracle_convert_general
    rc = fn(_u64(bases_a), da, _u64(bases_b), db, d_out, src.itemsize, src.ctypes.data, dst.ctypes.data, ntiles)
    if rc != OK:
        raise OracleError(rc, "convert_general")
    return dst


def convert_general_affine(bases_a: Sequence[int], off_a: int, bases_b: Sequence[int], off_b: int, d_out: int,
                           src: np.ndarray) -> np.ndarray:
    """Broadcasting conversion between affine layouts: dst[hB] = src[A^+(B hB ^ off_b ^ off_a)]."""
    da, db = len(bases_a), len(bases_b)
    _check_img(src, da, "src")
    ntiles = src.size >> da
    dst = np.empty(ntiles << db, dtype=src.dtype)
    rc = _load().oracle_convert_general_affine(_u64(bases_a), int(off_a), da, _u64(bases_b), int(off_b), db, d_out,
                                               src.itemsize, src.ctypes.data, dst.ctypes.data, ntiles)
    if rc != OK:
        raise OracleError(rc, "convert_general_affine")
    return dst


def _check_img(a: np.ndarray, d: int, what: str):
    if not a.flags["C_CONTIGUOUS"]:
        raise ValueError(f"{what} must be C-contiguous")
    if a.size % (1 << d) != 0:
        raise ValueError(f"{what} size {a.size} is not a multiple of 2^{d}")


def convert(bases_a: Sequence[int], bases_b: Sequence[int], src: np.ndarray,
            table: bool = False):
    """Image under A -> image under B.  Returns dst (and threads used if table=True)."""
    d = len(bases_a)
    if len(bases_b) != d:
        raise ValueError("A and B must have the same number of input bits")
    _check_img(src, d, "src")
    ntiles = src.size >> d
    dst = np.empty_like(src)
    lib = _load()
    if table:
        used = ctypes.c_int(0)
        rc = lib.oracle_convert_table(_u64(bases_a), _u64(bases_b), d, src.itemsize,
                                      src.ctypes.data, dst.ctypes.data, ntiles,
                                      ctypes.byref(used))
        if rc != OK:
            raise OracleError(rc, "convert_table")
        return dst, used.value
    rc = lib.oracle_convert(_u64(bases_a), _u64(bases_b), d, src.itemsize,
                            src.ctypes.data, dst.ctypes.data, ntiles)
    if rc != OK:
        raise OracleError(rc, "convert")
    return dst


def gather(bases_l: Sequence[int], out_dim_bits: Sequence[int], axis: int,
           inp: np.ndarray, idx: np.ndarray, table: bool = False) -> np.ndarray:
    """out[.., i, ..] = in[.., idx[.., i, ..], ..] along `axis`, all images under L.
    table=True: the same with L and its inverse tabulated once and tiles on all host threads."""
    d = len(bases_l)
    _check_img(inp, d, "in")
    _check_img(idx, d, "idx")
    if idx.dtype != np.int32 or idx.size != inp.size:
        raise ValueError("idx must be int32 with as many elements as in")
    ntiles = inp.size >> d
    out = np.empty_like(inp)
    dims = (ctypes.c_int32 * len(out_dim_bits))(*[int(b) for b in out_dim_bits])
    fn = _load().oracle_gather_table if table else _load().oracle_gather
    rc = fn(_u64(bases_l), d, dims, len(out_dim_bits), int(axis), inp.itemsize, inp.ctypes.data,
            idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), out.ctypes.data, ntiles)
    if rc != OK:
        raise OracleError(rc, "gather")
    return out


def convert_affine(bases_a: Sequence[int], off_a: int, bases_b: Sequence[int], off_b: int,
                   src: np.ndarray) -> np.ndarray:
    """Image under h -> A h ^ off_a to image under h -> B h ^ off_b (both bijective on the same bits)."""
    d = len(bases_a)
    if len(bases_b) != d:
        raise ValueError("A and B must have the same number of input bits")
    _check_img(src, d, "src")
    dst = np.empty_like(src)
    rc = _load().oracle_convert_affine(_u64(bases_a), int(off_a), _u64(bases_b), int(off_b), d, src.itemsize,
                                       src.ctypes.data, dst.ctypes.data, src.size >> d)
    if rc != OK:
        raise OracleError(rc, "convert_affine")
    return dst


def gather_affine(bases_l: Sequence[int], off: int, out_dim_bits: Sequence[int], axis: int,
                  inp: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """Gather along `axis` with in, idx and out under the affine layout h -> L h ^ off."""
    d = len(bases_l)
    _check_img(inp, d, "in")
    _check_img(idx, d, "idx")
    if idx.dtype != np.int32 or idx.size != inp.size:
        raise ValueError("idx must be int32 with as many elements as in")
    out = np.empty_like(inp)
    dims = (ctypes.c_int32 * len(out_dim_bits))(*[int(b) for b in out_dim_bits])
    rc = _load().oracle_gather_affine(_u64(bases_l), int(off), d, dims, len(out_dim_bits), int(axis), inp.itemsize,
                                      inp.ctypes.data, idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                      out.ctypes.data, inp.size >> d)
    if rc != OK:
        raise OracleError(rc, "gather_affine")
    return out


def gather_general(bases_l: Sequence[int], out_dim_bits: Sequence[int], axis: int,
                   inp: np.ndarray, idx: np.ndarray, off: int = 0) -> np.ndarray:
    """Gather (Sec. 5.5) under a surjective layout that may broadcast (Sec. 5.1), optionally affine.
    Slot h of a tile holds the logical element x = L h ^ off; `in` must be the image of a logical
    tensor X, i.e. all replicas of an element hold the same value (ValueError otherwise: the paper
    does not say which replica a gather would read, and the library leaves it unspecified).  Every
    slot of `out` is written, from its own slot of `idx` (replicas of idx may differ):
        out[h] = X[x with the axis coordinate replaced by idx[h] mod the axis length].
    X is read off the canonical slots, X[x] = in[L^+(x ^ off)] with L^+ the right inverse with free
    variables zero (Def. "Right Inverse"; Sec. 5.4 rule 2).  For a bijective layout this is the
    plain gather."""
    d, d_out = len(bases_l), int(sum(out_dim_bits))
    _check_img(inp, d, "in")
    _check_img(idx, d, "idx")
    if idx.dtype != np.int32 or idx.size != inp.size:
        raise ValueError("idx must be int32 with as many elements as in")
    if not 0 <= axis < len(out_dim_bits):
        raise ValueError("axis")
    shift = int(sum(out_dim_bits[axis + 1:]))
    mask = (1 << int(out_dim_bits[axis])) - 1
    lplus = right_inverse_table(bases_l, d_out).astype(np.int64)     # logical index -> canonical slot
    h = np.arange(1 << d, dtype=np.int64)
    lh = np.zeros(1 << d, dtype=np.int64)
    for k, col in enumerate(bases_l):
        lh ^= ((h >> k) & 1) * int(col)
    x = lh ^ int(off)                                                 # logical element of every slot
    canon = lplus[np.arange(1 << d_out, dtype=np.int64) ^ int(off)]   # X[x] sits at slot canon[x]
    out = np.empty_like(inp)
    src_img, idx_img, out_img = inp.reshape(-1, 1 << d), idx.reshape(-1, 1 << d), out.reshape(-1, 1 << d)
    for t in range(src_img.shape[0]):
        logical = src_img[t][canon]                                   # the logical tensor X of this tile
        if not np.array_equal(src_img[t], logical[x]):
            raise ValueError("replicas of `in` differ in tile %d: the gather is defined for images of a logical tensor" % t)
        want = idx_img[t].astype(np.int64) & mask
        out_img[t] = logical[(x & ~(mask << shift)) | (want << shift)]
    return out


def consistent_image(bases_l: Sequence[int], d_out: int, img: np.ndarray, off: int = 0) -> np.ndarray:
    """Copy of `img` (tiles of 2^len(bases) slots) in which every replica holds the value of the
    canonical slot of its logical element: the image of a logical tensor."""
    d = len(bases_l)
    _check_img(img, d, "img")
    lplus = right_inverse_table(bases_l, d_out).astype(np.int64)
    h = np.arange(1 << d, dtype=np.int64)
    lh = np.zeros(1 << d, dtype=np.int64)
    for k, col in enumerate(bases_l):
        lh ^= ((h >> k) & 1) * int(col)
    return np.ascontiguousarray(img.reshape(-1, 1 << d)[:, lplus[lh]]).reshape(-1)


def wavefronts(mem_bases: Sequence[int], dist_bases: Sequence[int], nreg: int, nlane: int,
               elem_bytes: int, vec_bits: int, nbanks: int, phase_of_lane: Sequence[int]):
    """Exhaustive wavefront count: returns (max per phase, total, conflict-free total)."""
    d = len(mem_bases)
    if len(dist_bases) != d:
        raise ValueError("memory and distributed layouts must act on the same number of bits")
    if len(phase_of_lane) != (1 << nlane):
        raise ValueError("phase_of_lane needs one entry per lane")
    ph = (ctypes.c_int32 * len(phase_of_lane))(*[int(p) for p in phase_of_lane])
    mx, tot, nph = ctypes.c_int64(0), ctypes.c_int64(0), ctypes.c_int64(0)
    rc = _load().oracle_wavefronts(_u64(mem_bases), _u64(dist_bases), d, nreg, nlane,
                                   elem_bytes, vec_bits, nbanks, ph,
                                   ctypes.byref(mx), ctypes.byref(tot), ctypes.byref(nph))
    if rc != OK:
        raise OracleError(rc, "wavefronts")
    return mx.value, tot.value, nph.value


from .algebra import OLayout, contiguity, divide_left, divide_left_permuting, identity_tile, product  # noqa: E402
from .families import (blocked_layout, identity_map, is_distributed_layout, is_memory_layout,  # noqa: E402
                       mfma_accumulator_tile, mfma_operand_tile, mma_swizzle_layout, mma_swizzle_offset,
                       product_of, slice_layout)
