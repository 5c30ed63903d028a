"""Seeded synthetic inputs and the five benchmark configurations.

This module serves BOTH the CPU oracle's tests and the HIP path's tests and
benchmark.  It holds input plumbing only: layout bases written out as lists,
a counter-based random generator, and dtype conversion.  None of the method's
arithmetic (composition, inversion, planning, conversion, gather) lives here.

Layout bases are the matrix columns of a linear layout (paper Sec. 4.1):
``bases[k]`` is the image of input bit k as a flattened logical index, input
bits ordered register, lane, wave (least-significant first); the last logical
dimension is the fastest, so for a rows x cols tile ``row k`` is the value
``1 << (log2(cols) + k)`` and ``col k`` is ``1 << k``.

Random values: element i of stream `seed` is splitmix64(seed * 2**40 + i), a
counter-based generator, so any slice of any tensor can be produced on its own,
on the CPU or on the GPU, with identical bits for the integer and uniform
recipes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np
import torch

_M64 = (1 << 64) - 1


def _s64(x: int) -> int:
    """Python int (mod 2**64) -> the same bit pattern as a signed 64-bit value."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


_GAMMA = _s64(0x9E3779B97F4A7C15)
_MUL1 = _s64(0xBF58476D1CE4E5B9)
_MUL2 = _s64(0x94D049BB133111EB)


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of int64 lanes."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def splitmix64(counter: torch.Tensor) -> torch.Tensor:
    """The splitmix64 output function applied to int64 counters (wrapping arithmetic)."""
    z = counter + _GAMMA
    z = (z ^ _lsr(z, 30)) * _MUL1
    z = (z ^ _lsr(z, 27)) * _MUL2
    return z ^ _lsr(z, 31)


def splitmix64_py(counter: int) -> int:
    """Scalar reference of the same function on Python integers (used by tests)."""
    z = (counter + 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def raw_bits(seed: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """int64 tensor: splitmix64(seed * 2**40 + i) for i in [start, start + count)."""
    i = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return splitmix64(i + _s64(seed << 40))


def _chunks(count: int, chunk: int):
    pos = 0
    while pos < count:
        n = min(chunk, count - pos)
        yield pos, n
        pos += n


def gen_int32(seed: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """Uniform over the full int32 range (low 32 bits of the stream)."""
    out = torch.empty(count, dtype=torch.int32, device=device)
    for pos, n in _chunks(count, 1 << 24):
        z = raw_bits(seed, start + pos, n, device)
        out[pos:pos + n] = (z & 0xFFFFFFFF).to(torch.int64).add_(-(1 << 31)).to(torch.int32)
    return out


def _uniform_pm1_f32(seed: int, start: int, count: int, device) -> torch.Tensor:
    """fp32 uniform in [-1, 1): 2 * (top 24 bits / 2**24) - 1, exact in fp32."""
    z = raw_bits(seed, start, count, device)
    top = _lsr(z, 40).to(torch.float32)          # 24 bits, exactly representable
    return top * (2.0 / (1 << 24)) - 1.0


def gen_uniform_pm1(seed: int, start: int, count: int, dtype: torch.dtype, device="cpu") -> torch.Tensor:
    """Uniform [-1, 1) drawn in fp32 and rounded to nearest-even into `dtype` (bf16 / fp16 / fp32)."""
    out = torch.empty(count, dtype=dtype, device=device)
    for pos, n in _chunks(count, 1 << 24):
        out[pos:pos + n] = _uniform_pm1_f32(seed, start + pos, n, device).to(dtype)
    return out


def gen_normal_f32(seed: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """normal(0, 1) by Box-Muller in fp64 from two uniforms per element, rounded to fp32."""
    out = torch.empty(count, dtype=torch.float32, device=device)
    for pos, n in _chunks(count, 1 << 23):
        z = raw_bits(seed, 2 * (start + pos), 2 * n, device)
        u = (_lsr(z, 11).to(torch.float64) + 0.5) * (1.0 / (1 << 53))   # (0, 1)
        u1, u2 = u[0::2], u[1::2]
        r = torch.sqrt(-2.0 * torch.log(u1))
        out[pos:pos + n] = (r * torch.cos(2.0 * np.pi * u2)).to(torch.float32)
    return out


def gen_index(seed: int, start: int, count: int, upper: int, device="cpu") -> torch.Tensor:
    """int32 uniform in [0, upper), upper a power of two (top bits of the stream)."""
    bits = upper.bit_length() - 1
    assert upper == 1 << bits and bits >= 1
    out = torch.empty(count, dtype=torch.int32, device=device)
    for pos, n in _chunks(count, 1 << 24):
        out[pos:pos + n] = _lsr(raw_bits(seed, start + pos, n, device), 64 - bits).to(torch.int32)
    return out


def bits_view(t: torch.Tensor) -> torch.Tensor:
    """Reinterpret a tensor as the signed integer type of the same width (raw bits)."""
    return t.view({1: torch.int8, 2: torch.int16, 4: torch.int32, 8: torch.int64}[t.element_size()])


def to_numpy_bits(t: torch.Tensor) -> np.ndarray:
    """Host numpy array holding the raw bits of `t` (uint of the same width)."""
    a = bits_view(t).cpu().numpy()
    return a.view({1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}[a.itemsize])


# ---------------------------------------------------------------------------
# Layout bases of the five configurations
# ---------------------------------------------------------------------------

def _rc(spec: Sequence[str], col_bits: int) -> List[int]:
    """['col0', 'row4', ...] -> flattened basis values for a rows x 2**col_bits tile."""
    out = []
    for s in spec:
        kind, k = s[:3], int(s[3:])
        out.append(1 << k if kind == "col" else 1 << (col_bits + k))
    return out


def _swap_rc(spec: Sequence[str]) -> List[str]:
    return [("row" if s.startswith("col") else "col") + s[3:] for s in spec]


def _rank_gf2(cols: Sequence[int]) -> int:
    """Rank over GF(2) of integers read as bit vectors (plain XOR elimination on the leading bit).
    An acceptance test for the sampler below: no layout is applied, composed or inverted here."""
    pivots = {}                                  # leading bit -> reduced vector
    for c in cols:
        while c:
            top = c.bit_length() - 1
            if top not in pivots:
                pivots[top] = c
                break
            c ^= pivots[top]
    return len(pivots)


def random_invertible_bases(seed: int, d: int) -> List[int]:
    """d columns drawn uniformly from d-bit values; the whole matrix is redrawn until it has
    rank d (rejection sampling of an invertible matrix)."""
    attempt = 0
    while True:
        raw = raw_bits(seed, attempt * d, d).numpy().view(np.uint64)
        cols = [int(x) & ((1 << d) - 1) for x in raw]
        if _rank_gf2(cols) == d:
            return cols
        attempt += 1


@dataclass
class Config:
    """One benchmark configuration: layouts, shapes and the recipe of its data."""
    cid: int
    name: str
    kind: str                       # "convert" or "gather"
    nreg: int
    nlane: int
    nwave: int
    out_dim_bits: List[int]         # logical dims, slowest first
    dtype: torch.dtype
    ntiles: int
    src_bases: List[int]
    dst_bases: Optional[List[int]]  # None for gather
    data_seed: int
    data_recipe: str                # "int32" | "uniform_pm1" | "normal"
    idx_seed: Optional[int] = None
    axis: Optional[int] = None
    note: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def d(self) -> int:
        return self.nreg + self.nlane + self.nwave

    @property
    def elem_bytes(self) -> int:
        return torch.empty((), dtype=self.dtype).element_size()

    @property
    def tile_elems(self) -> int:
        return 1 << self.d

    def algorithmic_bytes(self, ntiles: Optional[int] = None) -> int:
        """Read + write bytes the operation must move (gather also reads the int32 index)."""
        n = (self.ntiles if ntiles is None else ntiles) * self.tile_elems
        if self.kind == "gather":
            return n * (2 * self.elem_bytes + 4)
        return n * 2 * self.elem_bytes

    def gen_data(self, tile_start: int, ntiles: int, device="cpu") -> torch.Tensor:
        start, count = tile_start * self.tile_elems, ntiles * self.tile_elems
        if self.data_recipe == "int32":
            return gen_int32(self.data_seed, start, count, device)
        if self.data_recipe == "uniform_pm1":
            return gen_uniform_pm1(self.data_seed, start, count, self.dtype, device)
        if self.data_recipe == "normal":
            return gen_normal_f32(self.data_seed, start, count, device)
        raise ValueError(self.data_recipe)

    def gen_idx(self, tile_start: int, ntiles: int, device="cpu") -> torch.Tensor:
        assert self.kind == "gather"
        start, count = tile_start * self.tile_elems, ntiles * self.tile_elems
        return gen_index(self.idx_seed, start, count, 1 << self.out_dim_bits[self.axis], device)


def make_configs() -> List[Config]:
    c1_src = ["col0", "col1", "row4", "row5", "col2", "col3", "col4", "col5", "row0", "row1", "row2", "row3"]
    c1_dst = ["row0", "row1", "row3", "row4", "col0", "col1", "col2", "col3", "col4", "row2", "row5", "col5"]
    c2_src = ["col0", "col1", "col2", "row4", "row5", "row6",
              "col3", "col4", "col5", "col6", "row0", "row1", "row2", "row3"]
    c3_src = ["row0", "row1", "row4", "row5", "col4", "col5", "col0", "col1", "col2", "col3", "row2", "row3"]
    c3_dst = ["col0", "col1", "row2", "row3", "row4", "row5", "col2", "col3", "col4", "col5", "row0", "row1"]
    c5 = ["col0", "col1", "col2", "col3", "row0", "row1", "row2", "row3", "row4", "row5",
          "col4", "col5", "col6", "col7"]
    return [
        Config(1, "blocked->mfma32-acc 64x64 int32", "convert", 4, 6, 2, [6, 6], torch.int32, 1,
               _rc(c1_src, 6), _rc(c1_dst, 6), 1, "int32"),
        Config(2, "transpose 128x128 bf16", "convert", 6, 6, 2, [7, 7], torch.bfloat16, 8192,
               _rc(c2_src, 7), _rc(_swap_rc(c2_src), 7), 2, "uniform_pm1"),
        Config(3, "mfma16-acc->blocked 64x64 fp32, one wave", "convert", 6, 6, 0, [6, 6],
               torch.float32, 32768, _rc(c3_src, 6), _rc(c3_dst, 6), 3, "normal"),
        Config(4, "random invertible 16-bit XOR layouts int32", "convert", 6, 6, 4, [16],
               torch.int32, 4096, random_invertible_bases(40, 16), random_invertible_bases(41, 16),
               4, "int32"),
        Config(5, "wave-local gather 64x256 fp16", "gather", 4, 6, 4, [6, 8], torch.float16, 16384,
               _rc(c5, 8), None, 5, "uniform_pm1", idx_seed=50, axis=0),
    ]


_CONFIGS: Optional[List[Config]] = None


def configs() -> List[Config]:
    global _CONFIGS
    if _CONFIGS is None:
        _CONFIGS = make_configs()
    return _CONFIGS


def config(cid: int) -> Config:
    return configs()[cid - 1]


# The worked example of the paper (Sec. 4.1, "Layout A"): a 16x16 tensor tiled by
# 2x2 registers, 4x8 threads and 2x1 warps.  Columns in input order
# reg0, reg1, thr0..thr4, warp0 -> j0, i0, j1, j2, j3, i1, i2, i3 with
# flat = j | i << 4.
PAPER_LAYOUT_A = [1 << 0, 1 << 4, 1 << 1, 1 << 2, 1 << 3, 1 << 5, 1 << 6, 1 << 7]


# ---------------------------------------------------------------------------
# Layouts with broadcasting (paper Sec. 5.1 "Broadcasting"): zero columns mean that several
# hardware slots hold the same logical element, as the result of a reduction along lanes does.
# ---------------------------------------------------------------------------

@dataclass
class BroadcastCase:
    """Conversion between layouts of one logical tensor that replicate it differently."""
    name: str
    out_dim_bits: List[int]
    src_in: List[int]               # [register bits, lane bits, wave bits]
    dst_in: List[int]
    src_bases: List[int]
    dst_bases: List[int]
    dtype: torch.dtype
    ntiles: int
    data_seed: int

    @property
    def d_out(self) -> int:
        return sum(self.out_dim_bits)

    @property
    def d_src(self) -> int:
        return sum(self.src_in)

    @property
    def d_dst(self) -> int:
        return sum(self.dst_in)

    @property
    def elem_bytes(self) -> int:
        return torch.empty((), dtype=self.dtype).element_size()

    def algorithmic_bytes(self, ntiles: Optional[int] = None) -> int:
        """One copy of every logical element read, every destination slot written."""
        n = self.ntiles if ntiles is None else ntiles
        return n * ((1 << self.d_out) + (1 << self.d_dst)) * self.elem_bytes

    def gen_data(self, tile_start: int, ntiles: int, device="cpu") -> torch.Tensor:
        """Source image.  Replicas of one logical element are NOT made equal: which replica a
        conversion reads is part of its definition, and unequal replicas expose a wrong choice."""
        start, count = tile_start << self.d_src, ntiles << self.d_src
        if self.dtype == torch.int32:
            return gen_int32(self.data_seed, start, count, device)
        return gen_uniform_pm1(self.data_seed, start, count, self.dtype, device)


def _bits(spec: Sequence[Optional[int]]) -> List[int]:
    return [0 if s is None else 1 << s for s in spec]


def broadcast_cases() -> List[BroadcastCase]:
    Z = None
    # a 1024-vector left by a row reduction: 16 lanes of every wave hold the same values
    sliced = _bits([0, 1, 6, 7] + [Z, Z, Z, Z, 2, 3] + [4, 5, 8, 9])
    blocked = _bits([0, 1] + [2, 3, 4, 5, 6, 7] + [8, 9])
    # a 64 x 64 tile whose rows are replicated over 4 lanes and 2 waves, against a plain blocked one
    rep2d = _bits([0, 1, 10, 11] + [2, 3, Z, Z, 4, 5] + [6, 7, Z, 8, 9])
    blk2d = _bits([0, 1, 2, 3] + [4, 5, 6, 7, 8, 9] + [10, 11])
    return [
        BroadcastCase("reduction result -> blocked vector (collapse 16x)", [10], [4, 6, 4], [2, 6, 2],
                      sliced, blocked, torch.float32, 1 << 16, 61),
        BroadcastCase("blocked vector -> replicated over 16 lanes (expand 16x)", [10], [2, 6, 2], [4, 6, 4],
                      blocked, sliced, torch.float32, 1 << 16, 62),
        BroadcastCase("64x64 replicated 8x -> blocked bf16", [6, 6], [4, 6, 5], [4, 6, 2],
                      rep2d, blk2d, torch.bfloat16, 1 << 14, 63),
        BroadcastCase("64x64 blocked -> replicated 8x bf16", [6, 6], [4, 6, 2], [4, 6, 5],
                      blk2d, rep2d, torch.bfloat16, 1 << 14, 64),
        BroadcastCase("replicated 16x -> differently replicated 8x int32", [10], [4, 6, 4], [3, 6, 4],
                      sliced, _bits([0, 1, 2] + [3, Z, 4, Z, 5, 6] + [7, 8, Z, 9]), torch.int32, 1 << 15, 65),
    ]
