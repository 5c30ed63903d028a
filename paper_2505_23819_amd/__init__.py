"""MI355X-native Linear-Layouts library: Python binding of the C ABI in include/ll.h.

Argument marshalling only: every step of the hot path runs in the HIP kernels of
``libll355.so``.  PyTorch is used by callers for device memory and streams; this
module only needs ``tensor.data_ptr()`` and a stream handle.  There is no CPU
fallback: if the library cannot be loaded the import fails, and device calls
without a GPU return an error status (raised as ``LLError``).
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

# PyTorch-ROCm ships its own copy of the HIP runtime.  A process must end up with ONE runtime: if this
# library were loaded first it would bring in the system copy, PyTorch would then load its own next to
# it, and launches into the second runtime fail with "no ROCm-capable device is detected".  Importing
# torch first makes the dynamic linker satisfy this library's dependency with the copy torch loaded.
import torch  # noqa: F401

from . import build as _build

# ---- status codes and enums of ll.h ------------------------------------------------------------
LL_OK, LL_ERR_INVALID_ARG, LL_ERR_DIM_MISMATCH, LL_ERR_NOT_SURJECTIVE, LL_ERR_NOT_INJECTIVE, \
    LL_ERR_TILE_MIXED, LL_ERR_AXIS_NOT_IN_WAVE, LL_ERR_UNSUPPORTED, LL_ERR_DEVICE, LL_ERR_NOT_DIVISIBLE = range(10)
LL_IN_REG, LL_IN_LANE, LL_IN_WAVE, LL_IN_TILE, LL_IN_OFFSET = range(5)
LL_KIND_NOOP, LL_KIND_REG_ONLY, LL_KIND_INTRA_WAVE, LL_KIND_LDS, LL_KIND_BROADCAST = range(5)
LL_STRATEGY_COPY, LL_STRATEGY_REG_PERMUTE, LL_STRATEGY_WAVE_SHUFFLE, LL_STRATEGY_LDS_ELEM, \
    LL_STRATEGY_LDS_VEC, LL_STRATEGY_LDS_PULL, LL_STRATEGY_LDS_TR = range(7)
LL_MAX_IN_DIMS, LL_MAX_OUT_DIMS, LL_MAX_BITS, LL_PLAN_MAX_BLOCK_BITS = 5, 8, 30, 20

KIND_NAMES = ["noop", "reg_only", "intra_wave", "lds", "broadcast"]
STRATEGY_NAMES = ["copy", "reg_permute", "wave_shuffle", "lds_elem", "lds_vec", "lds_pull", "lds_tr"]

EXPORTED_SYMBOLS = [
    "ll_layout_create", "ll_layout_destroy", "ll_layout_get", "ll_layout_apply", "ll_compose",
    "ll_product", "ll_invert", "ll_plan_convert", "ll_plan_info", "ll_plan_destroy", "ll_convert",
    "ll_gather", "ll_copy", "ll_last_error", "ll_product_dimwise", "ll_divide_left",
    "ll_divide_left_permuted", "ll_contiguity", "ll_layout_identity", "ll_layout_blocked",
    "ll_layout_mfma_accumulator", "ll_layout_mfma_operand", "ll_layout_mma_swizzle", "ll_layout_classify",
    "ll_gather_info", "ll_layout_with_offset", "ll_layout_get_offset", "ll_layout_slice",
    "ll_options_init", "ll_options_from_env", "ll_plan_convert_opts", "ll_gather_opts", "ll_gather_info_opts",
]
LL_AUTO = -1
LL_GATHER_SHUFFLE, LL_GATHER_WAVE_STAGED, LL_GATHER_BLOCK_STAGED, LL_GATHER_GLOBAL, LL_GATHER_PHASED, \
    LL_GATHER_SHUFFLE_ROWS = range(6)
GATHER_KERNEL_NAMES = ["shuffle", "wave_staged", "block_staged", "global", "lds_phased", "shuffle_rows"]


class ll_gather_desc(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_int32), ("axis_reg_bits", ctypes.c_int32), ("axis_lane_bits", ctypes.c_int32),
                ("axis_wave_bits", ctypes.c_int32), ("paper_rounds", ctypes.c_int32), ("block_bytes", ctypes.c_int32)]
LL_LAYOUT_SURJECTIVE, LL_LAYOUT_INJECTIVE, LL_LAYOUT_DISTRIBUTED, LL_LAYOUT_MEMORY = 1, 2, 4, 8


class ll_options(ctypes.Structure):
    """Mirror of the C struct: every field an int32, LL_AUTO = the library's choice."""
    _fields_ = [(name, ctypes.c_int32) for name in (
        "size", "strategy", "gather_kernel", "block_bytes", "pref_bytes", "elem_threads_log2", "vec_block_bytes",
        "vec_threads", "shuffle_block_bytes", "inflight_bytes", "lds_pad_bytes", "xcd_chunk", "pull_mode",
        "pull_vec_bits", "pull_inflight_bytes", "pull_xcd_chunk", "gather_block_bytes", "gather_lds_max_bytes",
        "gather_min_run_bytes", "gather_phased_max_bytes", "gather_threads_log2", "gather_inflight_bytes",
        "gather_xcd_chunk", "gather_swizzle_always", "copy_xcd_chunk", "debug", "gather_waves", "pull_threads_log2")]


class ll_in_dim(ctypes.Structure):
    _fields_ = [("label", ctypes.c_int32), ("nbits", ctypes.c_int32)]


class ll_out_dim(ctypes.Structure):
    _fields_ = [("nbits", ctypes.c_int32)]


class ll_plan_desc(ctypes.Structure):
    _fields_ = [
        ("kind", ctypes.c_int32), ("strategy", ctypes.c_int32), ("d", ctypes.c_int32), ("d_dst", ctypes.c_int32),
        ("elem_bytes", ctypes.c_int32),
        ("conv", ctypes.c_uint64 * LL_MAX_BITS), ("conv_offset", ctypes.c_uint64),
        ("pull", ctypes.c_uint64 * LL_MAX_BITS),
        ("global_vec_bytes", ctypes.c_int32), ("src_lines_per_access", ctypes.c_int32),
        ("dst_lines_per_access", ctypes.c_int32), ("lds_write_bytes", ctypes.c_int32),
        ("lds_read_bytes", ctypes.c_int32), ("lds_bytes", ctypes.c_int32),
        ("threads", ctypes.c_int32), ("vectors_per_thread", ctypes.c_int32),
        ("block_bits", ctypes.c_int32), ("group_bits", ctypes.c_int32),
        ("segment_bits", ctypes.c_int32), ("shuffle_rounds", ctypes.c_int32),
        ("register_transpose", ctypes.c_int32),
        ("lds_mem", ctypes.c_uint64 * LL_PLAN_MAX_BLOCK_BITS),
        ("lds_write", ctypes.c_uint64 * LL_PLAN_MAX_BLOCK_BITS),
        ("lds_read", ctypes.c_uint64 * LL_PLAN_MAX_BLOCK_BITS),
        ("lds_write_reg_bits", ctypes.c_int32), ("lds_read_reg_bits", ctypes.c_int32),
        ("lds_vec_bits", ctypes.c_int32), ("lds_banks", ctypes.c_int32), ("lds_banks_write", ctypes.c_int32),
        ("lds_phase_lanes_write", ctypes.c_int32), ("lds_phase_lanes_read", ctypes.c_int32),
        ("predicted_wavefronts_write", ctypes.c_int32), ("predicted_wavefronts_read", ctypes.c_int32),
        ("sched_valid", ctypes.c_int32), ("sched_nv", ctypes.c_int32), ("sched_ni", ctypes.c_int32),
        ("sched_ng", ctypes.c_int32), ("sched_nr", ctypes.c_int32),
        ("sched_v", ctypes.c_uint64 * 2), ("sched_i", ctypes.c_uint64 * 8), ("sched_g", ctypes.c_uint64 * 8),
        ("sched_r", ctypes.c_uint64 * LL_MAX_BITS),
    ]


class LLError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"ll status {status}: {message}")
        self.status = status
        self.message = message


def _load() -> ctypes.CDLL:
    path = _build.LIB
    if not os.path.exists(path):
        _build.build(force=True)      # nothing built yet: build once, loudly on failure
    lib = ctypes.CDLL(path)
    vp, i32, i64, u64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_uint64
    P = ctypes.POINTER
    lib.ll_layout_create.argtypes = [P(ll_in_dim), i32, P(ll_out_dim), i32, P(u64), P(vp)]
    lib.ll_layout_destroy.argtypes = [vp]
    lib.ll_layout_get.argtypes = [vp, P(i32), P(ll_in_dim), P(i32), P(ll_out_dim), P(u64)]
    lib.ll_layout_apply.argtypes = [vp, u64, P(u64)]
    lib.ll_compose.argtypes = [vp, vp, P(vp)]
    lib.ll_product.argtypes = [vp, vp, P(vp)]
    lib.ll_invert.argtypes = [vp, P(vp)]
    lib.ll_plan_convert.argtypes = [vp, vp, i32, P(vp)]
    lib.ll_plan_info.argtypes = [vp, P(ll_plan_desc)]
    lib.ll_plan_destroy.argtypes = [vp]
    lib.ll_convert.argtypes = [vp, vp, vp, i64, vp]
    lib.ll_gather.argtypes = [vp, i32, i32, vp, vp, vp, i64, vp]
    lib.ll_copy.argtypes = [vp, vp, i64, vp]
    lib.ll_options_init.argtypes = [P(ll_options)]
    lib.ll_options_from_env.argtypes = [P(ll_options)]
    lib.ll_plan_convert_opts.argtypes = [vp, vp, i32, P(ll_options), P(vp)]
    lib.ll_gather_opts.argtypes = [vp, i32, i32, P(ll_options), vp, vp, vp, i64, vp]
    lib.ll_gather_info_opts.argtypes = [vp, i32, i32, P(ll_options), P(ll_gather_desc)]
    lib.ll_last_error.restype = ctypes.c_char_p
    lib.ll_last_error.argtypes = []
    for name in EXPORTED_SYMBOLS:
        if name != "ll_last_error":
            getattr(lib, name).restype = ctypes.c_int
    return lib


_lib = _load()
LIBRARY_PATH = _build.LIB


def _check(status: int):
    if status != LL_OK:
        raise LLError(status, (_lib.ll_last_error() or b"").decode())


def ll_last_error() -> str:
    return (_lib.ll_last_error() or b"").decode()


# ---- handles ------------------------------------------------------------------------------------

class Layout:
    """Owning wrapper of an ``ll_layout*``."""

    def __init__(self, handle: int):
        self._h = ctypes.c_void_p(handle)

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:
            _lib.ll_layout_destroy(h)

    def get(self) -> Tuple[List[Tuple[int, int]], List[int], List[int]]:
        n_in, n_out = ctypes.c_int(0), ctypes.c_int(0)
        ind = (ll_in_dim * LL_MAX_IN_DIMS)()
        outd = (ll_out_dim * LL_MAX_OUT_DIMS)()
        bases = (ctypes.c_uint64 * LL_MAX_BITS)()
        _check(_lib.ll_layout_get(self._h, ctypes.byref(n_in), ind, ctypes.byref(n_out), outd, bases))
        in_dims = [(ind[i].label, ind[i].nbits) for i in range(n_in.value)]
        out_dims = [outd[i].nbits for i in range(n_out.value)]
        d_in = sum(b for _, b in in_dims)
        return in_dims, out_dims, [int(bases[k]) for k in range(d_in)]

    @property
    def bases(self) -> List[int]:
        return self.get()[2]

    @property
    def in_dims(self):
        return self.get()[0]

    @property
    def out_dims(self):
        return self.get()[1]

    @property
    def d_in(self) -> int:
        """Input bits (index bits of one tile image), read once: layouts are immutable."""
        if getattr(self, "_d_in", None) is None:
            self._d_in = sum(b for _, b in self.get()[0])
        return self._d_in

    def apply(self, index: int) -> int:
        return ll_layout_apply(self, index)


class Plan:
    """Owning wrapper of an ``ll_plan*``."""

    def __init__(self, handle: int):
        self._h = ctypes.c_void_p(handle)

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:
            _lib.ll_plan_destroy(h)

    def info(self) -> dict:
        return ll_plan_info(self)

    def sizes(self) -> Tuple[int, int, int]:
        """(index bits of a source tile, of a destination tile, element bytes), read once."""
        if getattr(self, "_sizes", None) is None:
            i = ll_plan_info(self)
            self._sizes = (i["d"], i["d_dst"], i["elem_bytes"])
        return self._sizes


# ---- the calls of ll.h, same names --------------------------------------------------------------

def ll_layout_create(in_dims: Sequence[Tuple[int, int]], out_dims: Sequence[int], bases: Sequence[int]) -> Layout:
    """in_dims: [(label, nbits)] in canonical order; out_dims: [nbits] slowest first; bases: columns."""
    ind = (ll_in_dim * max(1, len(in_dims)))(*[ll_in_dim(int(l), int(n)) for l, n in in_dims])
    outd = (ll_out_dim * max(1, len(out_dims)))(*[ll_out_dim(int(n)) for n in out_dims])
    arr = (ctypes.c_uint64 * max(1, len(bases)))(*[int(b) for b in bases])
    h = ctypes.c_void_p()
    _check(_lib.ll_layout_create(ind, len(in_dims), outd, len(out_dims), arr, ctypes.byref(h)))
    return Layout(h.value)


def ll_layout_apply(layout: Layout, index: int) -> int:
    out = ctypes.c_uint64(0)
    _check(_lib.ll_layout_apply(layout._h, int(index), ctypes.byref(out)))
    return int(out.value)


def _binary(fn, a: Layout, b: Layout) -> Layout:
    h = ctypes.c_void_p()
    _check(fn(a._h, b._h, ctypes.byref(h)))
    return Layout(h.value)


def ll_compose(outer: Layout, inner: Layout) -> Layout:
    return _binary(_lib.ll_compose, outer, inner)


def ll_product(a: Layout, b: Layout) -> Layout:
    return _binary(_lib.ll_product, a, b)


def ll_product_dimwise(a: Layout, b: Layout) -> Layout:
    return _binary(_lib.ll_product_dimwise, a, b)


def ll_divide_left(layout: Layout, tile: Layout) -> Layout:
    return _binary(_lib.ll_divide_left, layout, tile)


def ll_divide_left_permuted(layout: Layout, tile: Layout, label: int):
    """Returns (perm, quotient): new input bit k of `label` = old bit perm[k]."""
    n = dict(layout.in_dims).get(label, 0)
    perm = (ctypes.c_int32 * max(n, 1))()
    h = ctypes.c_void_p()
    _check(_lib.ll_divide_left_permuted(layout._h, tile._h, int(label), perm, ctypes.byref(h)))
    return list(perm)[:n], Layout(h.value)


def ll_contiguity(layout: Layout) -> int:
    out = ctypes.c_int32()
    _check(_lib.ll_contiguity(layout._h, ctypes.byref(out)))
    return out.value


def _made(status, h) -> Layout:
    _check(status)
    return Layout(h.value)


def ll_layout_identity(label: int, dim: int, k: int, n_dims: int) -> Layout:
    h = ctypes.c_void_p()
    return _made(_lib.ll_layout_identity(int(label), int(dim), int(k), int(n_dims), ctypes.byref(h)), h)


def ll_layout_blocked(reg_bits: Sequence[int], lane_bits: Sequence[int], wave_bits: Sequence[int],
                      order: Sequence[int]) -> Layout:
    n = len(order)
    arr = lambda xs: (ctypes.c_int32 * n)(*[int(x) for x in xs])
    h = ctypes.c_void_p()
    return _made(_lib.ll_layout_blocked(n, arr(reg_bits), arr(lane_bits), arr(wave_bits), arr(order), ctypes.byref(h)), h)


def ll_layout_mfma_accumulator(m_bits: int) -> Layout:
    h = ctypes.c_void_p()
    return _made(_lib.ll_layout_mfma_accumulator(int(m_bits), ctypes.byref(h)), h)


def ll_layout_mfma_operand(m_bits: int, k_reg_bits: int) -> Layout:
    h = ctypes.c_void_p()
    return _made(_lib.ll_layout_mfma_operand(int(m_bits), int(k_reg_bits), ctypes.byref(h)), h)


def ll_layout_mma_swizzle(m_bits: int, n_bits: int, vec: int, per_phase: int, max_phase: int) -> Layout:
    h = ctypes.c_void_p()
    return _made(_lib.ll_layout_mma_swizzle(int(m_bits), int(n_bits), int(vec), int(per_phase), int(max_phase),
                                            ctypes.byref(h)), h)


def ll_options_init(**fields) -> ll_options:
    """A new ll_options with every field LL_AUTO, then the given fields set."""
    o = ll_options()
    _check(_lib.ll_options_init(ctypes.byref(o)))
    for k, v in fields.items():
        if k == "size" or k not in dict(ll_options._fields_):
            raise LLError(LL_ERR_INVALID_ARG, f"ll_options has no settable field {k!r}")
        setattr(o, k, int(v))
    return o


def ll_options_from_env() -> ll_options:
    o = ll_options()
    _check(_lib.ll_options_from_env(ctypes.byref(o)))
    return o


def _opts(opts):
    return None if opts is None else ctypes.byref(opts)


def ll_gather_info(layout: Layout, axis: int, elem_bytes: int, opts: Optional[ll_options] = None) -> dict:
    d = ll_gather_desc()
    _check(_lib.ll_gather_info_opts(layout._h, int(axis), int(elem_bytes), _opts(opts), ctypes.byref(d)))
    out = {name: getattr(d, name) for name, _ in ll_gather_desc._fields_}
    out["kernel_name"] = GATHER_KERNEL_NAMES[d.kernel]
    return out


def ll_layout_with_offset(layout: Layout, offset: int) -> Layout:
    h = ctypes.c_void_p()
    return _made(_lib.ll_layout_with_offset(layout._h, ctypes.c_uint64(int(offset)), ctypes.byref(h)), h)


def ll_layout_slice(layout: Layout, dim: int) -> Layout:
    h = ctypes.c_void_p()
    return _made(_lib.ll_layout_slice(layout._h, ctypes.c_int(int(dim)), ctypes.byref(h)), h)


def ll_layout_get_offset(layout: Layout) -> int:
    off = ctypes.c_uint64()
    _check(_lib.ll_layout_get_offset(layout._h, ctypes.byref(off)))
    return off.value


def ll_layout_classify(layout: Layout) -> int:
    flags = ctypes.c_uint32()
    _check(_lib.ll_layout_classify(layout._h, ctypes.byref(flags)))
    return flags.value


def ll_invert(layout: Layout) -> Layout:
    h = ctypes.c_void_p()
    _check(_lib.ll_invert(layout._h, ctypes.byref(h)))
    return Layout(h.value)


def ll_plan_convert(src: Layout, dst: Layout, elem_bytes: int, opts: Optional[ll_options] = None) -> Plan:
    h = ctypes.c_void_p()
    if opts is None:
        _check(_lib.ll_plan_convert(src._h, dst._h, int(elem_bytes), ctypes.byref(h)))
    else:
        _check(_lib.ll_plan_convert_opts(src._h, dst._h, int(elem_bytes), ctypes.byref(opts), ctypes.byref(h)))
    return Plan(h.value)


ll_plan_convert_opts = ll_plan_convert


def ll_plan_info(plan: Plan) -> dict:
    d = ll_plan_desc()
    _check(_lib.ll_plan_info(plan._h, ctypes.byref(d)))
    out = {}
    for name, _ in ll_plan_desc._fields_:
        v = getattr(d, name)
        out[name] = [int(x) for x in v] if hasattr(v, "__len__") else int(v)
    out["conv"] = out["conv"][:d.d]
    out["pull"] = out["pull"][:d.d_dst]
    for key in ("lds_mem", "lds_write", "lds_read"):
        out[key] = out[key][:d.block_bits]
    for key, cnt in (("sched_v", d.sched_nv), ("sched_i", d.sched_ni), ("sched_g", d.sched_ng), ("sched_r", d.sched_nr)):
        out[key] = out[key][:cnt]
    out["kind_name"] = KIND_NAMES[d.kind]
    out["strategy_name"] = STRATEGY_NAMES[d.strategy]
    return out


def _ptr(x, need_bytes: int = 0, what: str = "buffer") -> int:
    """Device pointer of a torch tensor (or a raw integer address, taken on trust).  A tensor must
    live on the GPU, be contiguous and hold at least `need_bytes`: a host pointer or a short buffer
    handed to a kernel would be a memory fault on the device, not an exception."""
    if not hasattr(x, "data_ptr"):
        return int(x)
    if not getattr(x, "is_cuda", False):
        raise LLError(LL_ERR_INVALID_ARG, f"{what} is not a GPU tensor")
    if not x.is_contiguous():
        raise LLError(LL_ERR_INVALID_ARG, f"{what} is not contiguous")
    have = x.numel() * x.element_size()
    if have < need_bytes:
        raise LLError(LL_ERR_INVALID_ARG, f"{what} holds {have} bytes, the call needs {need_bytes}")
    return int(x.data_ptr())


def _current_stream_fn():
    """torch's current raw stream handle.  The public path (building a Stream object) costs about
    3 us per call, as much as the launch itself; torch's own kernels use the raw-handle query."""
    import torch
    raw = getattr(torch._C, "_cuda_getCurrentRawStream", None)
    if raw is None:
        return lambda: int(torch.cuda.current_stream().cuda_stream)
    return lambda: int(raw(torch.cuda.current_device()))


_current_stream = None


def _stream(stream) -> int:
    global _current_stream
    if stream is None:
        if _current_stream is None:
            _current_stream = _current_stream_fn()
        return _current_stream()
    return int(getattr(stream, "cuda_stream", stream))


def ll_convert(plan: Plan, src, dst, ntiles: int, stream=None) -> None:
    """Enqueue the conversion on `stream` (default: torch's current stream)."""
    d, d_dst, w = plan.sizes()
    n = max(0, int(ntiles))
    _check(_lib.ll_convert(plan._h, _ptr(src, (n << d) * w, "src"), _ptr(dst, (n << d_dst) * w, "dst"), int(ntiles),
                           _stream(stream)))


def ll_gather(layout: Layout, axis: int, elem_bytes: int, inp, idx, out, ntiles: int, stream=None,
              opts: Optional[ll_options] = None) -> None:
    n = max(0, int(ntiles)) << layout.d_in
    if hasattr(idx, "element_size") and idx.element_size() != 4:
        raise LLError(LL_ERR_INVALID_ARG, "idx must hold 32-bit integers")
    if opts is None:
        _check(_lib.ll_gather(layout._h, int(axis), int(elem_bytes), _ptr(inp, n * int(elem_bytes), "in"), _ptr(idx, n * 4, "idx"),
                              _ptr(out, n * int(elem_bytes), "out"), int(ntiles), _stream(stream)))
    else:
        _check(_lib.ll_gather_opts(layout._h, int(axis), int(elem_bytes), ctypes.byref(opts), _ptr(inp, n * int(elem_bytes), "in"),
                                   _ptr(idx, n * 4, "idx"), _ptr(out, n * int(elem_bytes), "out"), int(ntiles), _stream(stream)))


ll_gather_opts = ll_gather
ll_gather_info_opts = ll_gather_info


def ll_copy(src, dst, nbytes: int, stream=None) -> None:
    _check(_lib.ll_copy(_ptr(src, int(nbytes), "src"), _ptr(dst, int(nbytes), "dst"), int(nbytes), _stream(stream)))


# ---- small conveniences --------------------------------------------------------------------------

def distributed_layout(nreg: int, nlane: int, nwave: int, out_dims: Sequence[int], bases: Sequence[int]) -> Layout:
    """Layout with register / lane / wave inputs (labels with zero bits are dropped)."""
    dims = [(l, n) for l, n in ((LL_IN_REG, nreg), (LL_IN_LANE, nlane), (LL_IN_WAVE, nwave)) if n > 0]
    return ll_layout_create(dims, out_dims, bases)
