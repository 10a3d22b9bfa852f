"""ctypes binding of libpipeoptim (argument marshalling only).

Function names mirror the C ABI of ``include/pipeoptim.h``.  Every step of the
path runs in the HIP library; there is no Python or CPU fallback: if the
library has not been built, loading raises.
"""
import ctypes
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpipeoptim.so")

PO_OK, PO_EINVAL, PO_EALIGN, PO_EHIP, PO_ENOMEM = 0, -1, -2, -3, -4
PO_SGDM, PO_ADAM, PO_ADAMW, PO_NESTEROV, PO_RMSPROP, PO_ADAGRAD = 0, 1, 2, 3, 4, 5
PO_WHAT_F32, PO_WHAT_BF16 = 0, 1
PO_GRAD_F32, PO_GRAD_BF16 = 0, 1
PO_LDS_AUTO = -1
PO_KERNEL_KIND_FUSED, PO_KERNEL_KIND_PREDICT = 0, 1
OPTIMIZERS = {"sgdm": PO_SGDM, "adam": PO_ADAM, "adamw": PO_ADAMW, "nesterov": PO_NESTEROV, "rmsprop": PO_RMSPROP,
              "adagrad": PO_ADAGRAD}
WHAT_DTYPES = {"f32": PO_WHAT_F32, "bf16": PO_WHAT_BF16}
GRAD_DTYPES = {"f32": PO_GRAD_F32, "bf16": PO_GRAD_BF16}


class PipeOptimError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("pipeoptim status %d: %s" % (status, message))
        self.status = status


class po_hyper(ctypes.Structure):
    _fields_ = [("opt", ctypes.c_int32), ("decay_in_prediction", ctypes.c_int32),
                ("lr", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("eps", ctypes.c_double), ("weight_decay", ctypes.c_double)]


class po_coeffs(ctypes.Structure):
    _fields_ = [(n, ctypes.c_float) for n in
                ("beta1", "grad_scale", "beta2", "one_m_beta2", "inv_bc1", "inv_sqrt_bc2", "eps", "lr", "s_lr",
                 "wd_coupled", "wd_step", "wd_pred")] + [("s_is_zero", ctypes.c_int32)]


class po_chunk(ctypes.Structure):
    _fields_ = [("tensor", ctypes.c_uint32), ("chunk", ctypes.c_uint32)]


class po_launch(ctypes.Structure):
    _fields_ = [("block", ctypes.c_int32), ("lds_bytes", ctypes.c_int32), ("chunk_elems", ctypes.c_int64)]


EXPORTS = (
    "pipeoptim_plan_create", "pipeoptim_plan_create_mixed", "pipeoptim_plan_destroy", "pipeoptim_plan_set_pointers",
    "pipeoptim_plan_get_launch", "pipeoptim_plan_set_launch", "pipeoptim_plan_info",
    "pipeoptim_step_predict", "pipeoptim_predict", "pipeoptim_plan_get_predict_launch",
    "pipeoptim_plan_set_predict_launch", "pipeoptim_version_difference", "pipeoptim_coefficients",
    "pipeoptim_chunk_table_build", "pipeoptim_probe_copy", "pipeoptim_probe_copy_near", "pipeoptim_auto_lds_bytes",
    "pipeoptim_last_error",
    "pipeoptim_arena_create", "pipeoptim_arena_alloc", "pipeoptim_arena_set_skew", "pipeoptim_arena_near_half",
    "pipeoptim_arena_info", "pipeoptim_arena_check", "pipeoptim_arena_destroy", "pipeoptim_plan_localize", "pipeoptim_plan_effective_launch",
    "pipeoptim_local_tile", "pipeoptim_local_slot", "pipeoptim_plan_local_params", "pipeoptim_plan_launch_phase",
    "pipeoptim_device_sync_count", "pipeoptim_step_predict_static", "pipeoptim_plan_learn_layout", "pipeoptim_plan_chunk_marks",
    "pipeoptim_plan_near_share", "pipeoptim_chunk_vote", "pipeoptim_whole_pieces",
)
PO_STATIC_MAX_TENSORS, PO_STATIC_MAX_CHUNKS = 1024, 65536

_lib = None


def lib():
    """The loaded library.  Raises if it was not built (``python -m paper_2312_00839_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libpipeoptim.so is not built: run `python -m paper_2312_00839_amd.build` "
                              "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        P = ctypes.POINTER
        L.pipeoptim_plan_create.argtypes = [P(vp), i64, P(i64), P(vp), P(vp), P(vp), P(vp), P(vp), i32, vp]
        L.pipeoptim_plan_create_mixed.argtypes = [P(vp), i64, P(i64), P(vp), P(vp), i32, P(vp), P(vp), P(vp), i32, vp]
        L.pipeoptim_plan_destroy.argtypes = [vp]
        L.pipeoptim_plan_set_pointers.argtypes = [vp, i32, P(vp), vp]
        L.pipeoptim_device_sync_count.argtypes = [P(i64)]
        L.pipeoptim_step_predict_static.argtypes = [i64, P(i64), P(vp), P(vp), P(vp), P(vp), P(vp), i32, P(po_hyper), i64, i32, vp]
        L.pipeoptim_plan_get_launch.argtypes = [vp, P(po_launch)]
        L.pipeoptim_plan_set_launch.argtypes = [vp, P(po_launch)]
        L.pipeoptim_plan_info.argtypes = [vp, P(i64), P(i64), P(i64)]
        L.pipeoptim_step_predict.argtypes = [vp, P(po_hyper), i64, i32, vp]
        L.pipeoptim_predict.argtypes = [vp, P(po_hyper), i64, i32, vp]
        L.pipeoptim_plan_get_predict_launch.argtypes = [vp, P(po_launch)]
        L.pipeoptim_plan_set_predict_launch.argtypes = [vp, P(po_launch)]
        L.pipeoptim_version_difference.argtypes = [i32, i32, P(i32)]
        L.pipeoptim_coefficients.argtypes = [P(po_hyper), i64, i32, P(po_coeffs)]
        L.pipeoptim_chunk_table_build.argtypes = [i64, P(i64), i64, P(po_chunk), i64, P(i64)]
        L.pipeoptim_probe_copy.argtypes = [vp, vp, i64, vp]
        L.pipeoptim_probe_copy_near.argtypes = [vp, vp, vp, i64, i32, vp]
        L.pipeoptim_auto_lds_bytes.argtypes = [i32, i32, i64, P(i32)]
        L.pipeoptim_arena_create.argtypes = [P(vp), i64]
        L.pipeoptim_arena_alloc.argtypes = [vp, i64, P(i64), P(vp)]
        L.pipeoptim_arena_set_skew.argtypes = [vp, i64]
        L.pipeoptim_arena_near_half.argtypes = [vp, vp, P(i32)]
        L.pipeoptim_arena_info.argtypes = [vp, P(i64), P(i64), P(i64), P(i32), P(i32)]
        L.pipeoptim_arena_check.argtypes = [vp, P(i64), P(i64)]
        L.pipeoptim_arena_destroy.argtypes = [vp]
        L.pipeoptim_plan_localize.argtypes = [vp, vp, vp, P(i64)]
        L.pipeoptim_plan_local_params.argtypes = [vp, P(i64)]
        L.pipeoptim_plan_learn_layout.argtypes = [vp, vp, P(i64)]
        L.pipeoptim_plan_chunk_marks.argtypes = [vp, P(ctypes.c_int8), i64, P(i64)]
        L.pipeoptim_plan_near_share.argtypes = [vp, P(ctypes.c_double)]
        L.pipeoptim_whole_pieces.argtypes = [i64, P(ctypes.c_uint64), P(ctypes.c_uint64), P(ctypes.c_uint64), P(ctypes.c_uint64),
                                             i64, P(i64)]
        L.pipeoptim_chunk_vote.argtypes = [i32, P(ctypes.c_uint64), P(i32), i64, i64, P(ctypes.c_uint64), P(ctypes.c_int8),
                                           P(ctypes.c_double)]
        L.pipeoptim_plan_launch_phase.argtypes = [vp, P(i32)]
        L.pipeoptim_plan_effective_launch.argtypes = [vp, i32, i32, P(po_launch)]
        L.pipeoptim_local_tile.argtypes = [ctypes.c_uint32, i32, P(ctypes.c_uint32)]
        L.pipeoptim_local_slot.argtypes = [ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32, P(ctypes.c_uint32)]
        for name in EXPORTS:
            getattr(L, name).restype = ctypes.c_int
        L.pipeoptim_last_error.restype = ctypes.c_char_p
        L.pipeoptim_last_error.argtypes = []
        _lib = L
    return _lib


def pipeoptim_last_error() -> str:
    return lib().pipeoptim_last_error().decode()


def _check(rc):
    if rc != PO_OK:
        raise PipeOptimError(rc, pipeoptim_last_error())


def make_hyper(opt, lr, beta1, beta2, eps=0.0, weight_decay=0.0, decay_in_prediction=True) -> po_hyper:
    if isinstance(opt, str):
        opt = OPTIMIZERS[opt]
    return po_hyper(int(opt), int(bool(decay_in_prediction)), float(lr), float(beta1), float(beta2),
                    float(eps), float(weight_decay))


def pipeoptim_version_difference(D: int, rank: int) -> int:
    s = ctypes.c_int32(-1)
    _check(lib().pipeoptim_version_difference(int(D), int(rank), ctypes.byref(s)))
    return s.value


def pipeoptim_coefficients(hyper: po_hyper, t: int, s: int) -> po_coeffs:
    c = po_coeffs()
    _check(lib().pipeoptim_coefficients(ctypes.byref(hyper), int(t), int(s), ctypes.byref(c)))
    return c


def pipeoptim_auto_lds_bytes(kernel: int, opt, n_params: int) -> int:
    """The lds_bytes a call resolves PO_LDS_AUTO to."""
    if isinstance(opt, str):
        opt = OPTIMIZERS[opt]
    out = ctypes.c_int32(0)
    _check(lib().pipeoptim_auto_lds_bytes(int(kernel), int(opt), int(n_params), ctypes.byref(out)))
    return out.value


def pipeoptim_chunk_table_build(numel: Sequence[int], chunk_elems: int):
    """Host-only: list of (tensor, chunk) pairs for a ragged list."""
    n = len(numel)
    arr = (ctypes.c_int64 * max(n, 1))(*numel)
    count = ctypes.c_int64(0)
    _check(lib().pipeoptim_chunk_table_build(n, arr, int(chunk_elems), None, 0, ctypes.byref(count)))
    buf = (po_chunk * max(count.value, 1))()
    _check(lib().pipeoptim_chunk_table_build(n, arr, int(chunk_elems), buf, count.value, ctypes.byref(count)))
    return [(buf[i].tensor, buf[i].chunk) for i in range(count.value)]


def pipeoptim_local_tile(tile_in_chunk: int, first_block_half: int) -> int:
    """Host-only: the tile a workgroup at this position of its chunk takes in the near-memory order."""
    out = ctypes.c_uint32(0)
    _check(lib().pipeoptim_local_tile(int(tile_in_chunk), int(first_block_half), ctypes.byref(out)))
    return out.value


def pipeoptim_whole_pieces(ranges):
    """Host-only: the runs [lo, hi) of whole 2 MiB pieces inside the union of the byte ranges [(lo, hi), ...]."""
    n = len(ranges)
    lo = (ctypes.c_uint64 * max(n, 1))(*[r[0] for r in ranges])
    hi = (ctypes.c_uint64 * max(n, 1))(*[r[1] for r in ranges])
    out_lo, out_hi = (ctypes.c_uint64 * max(n, 1))(), (ctypes.c_uint64 * max(n, 1))()
    k = ctypes.c_int64(0)
    _check(lib().pipeoptim_whole_pieces(n, lo, hi, out_lo, out_hi, n, ctypes.byref(k)))
    return [(out_lo[j], out_hi[j]) for j in range(k.value)]


def pipeoptim_chunk_vote(first_byte, weight, elems: int, piece_addr, even_blocks_near):
    """Host-only: (near[0], near[1]) = bytes of traffic each tile-order mark would make near for one chunk."""
    ns, npieces = len(first_byte), len(piece_addr)
    near = (ctypes.c_double * 2)()
    _check(lib().pipeoptim_chunk_vote(ns, (ctypes.c_uint64 * max(ns, 1))(*first_byte), (ctypes.c_int32 * max(ns, 1))(*weight),
                                      int(elems), npieces, (ctypes.c_uint64 * max(npieces, 1))(*piece_addr),
                                      (ctypes.c_int8 * max(npieces, 1))(*even_blocks_near), near))
    return near[0], near[1]


def pipeoptim_local_slot(workgroup: int, phase: int, n_slots: int) -> int:
    """Host-only: the position workgroup id `workgroup` takes when launches start on XCC `phase`."""
    out = ctypes.c_uint32(0)
    _check(lib().pipeoptim_local_slot(int(workgroup), int(phase), int(n_slots), ctypes.byref(out)))
    return out.value


class Arena:
    """Owner of a ``po_arena*``: device memory with a known block-to-die layout (MI355X)."""

    def __init__(self, capacity_bytes: int):
        self._h = ctypes.c_void_p()
        _check(lib().pipeoptim_arena_create(ctypes.byref(self._h), int(capacity_bytes)))

    def alloc(self, sizes_bytes: Sequence[int]):
        """Device addresses of len(sizes_bytes) buffers with one layout (the streams of one tensor)."""
        n = len(sizes_bytes)
        sizes = (ctypes.c_int64 * max(n, 1))(*[int(b) for b in sizes_bytes])
        ptrs = (ctypes.c_void_p * max(n, 1))()
        _check(lib().pipeoptim_arena_alloc(self._h, n, sizes, ptrs))
        return [int(ptrs[k] or 0) for k in range(n)]

    def set_skew(self, skew_bytes: int) -> None:
        _check(lib().pipeoptim_arena_set_skew(self._h, int(skew_bytes)))

    def near_half(self, ptr: int) -> int:
        half = ctypes.c_int32(-2)
        _check(lib().pipeoptim_arena_near_half(self._h, ctypes.c_void_p(ptr), ctypes.byref(half)))
        return half.value

    def info(self):
        a, b, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
        n, f = ctypes.c_int32(), ctypes.c_int32()
        _check(lib().pipeoptim_arena_info(self._h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.byref(n),
                                          ctypes.byref(f)))
        return {"backed_bytes": a.value, "used_bytes": b.value, "released_pieces": c.value,
                "near_cycles": n.value, "far_cycles": f.value}

    def probe_copy(self, dst: int, src: int, nbytes: int, lds_bytes: int = 0, stream: int = 0) -> None:
        """dst[0..nbytes) = src[0..nbytes) in the near-memory tile order (both from one alloc call of this arena)."""
        _check(lib().pipeoptim_probe_copy_near(self._h, ctypes.c_void_p(dst), ctypes.c_void_p(src), int(nbytes),
                                               int(lds_bytes), ctypes.c_void_p(stream)))

    def check(self):
        """Times every backed piece again: (pieces that could be told apart, pieces that contradict the layout)."""
        a, b = ctypes.c_int64(), ctypes.c_int64()
        _check(lib().pipeoptim_arena_check(self._h, ctypes.byref(a), ctypes.byref(b)))
        return a.value, b.value

    def destroy(self) -> None:
        if self._h:
            h, self._h = self._h, ctypes.c_void_p()
            _check(lib().pipeoptim_arena_destroy(h))

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _ptr_array(ptrs: Sequence[int]):
    return (ctypes.c_void_p * max(len(ptrs), 1))(*[ctypes.c_void_p(p) for p in ptrs])


class Plan:
    """Owner of a ``po_plan*``.  Pointers are raw device addresses (ints), e.g. ``tensor.data_ptr()``."""

    def __init__(self, numel: Sequence[int], W: Sequence[int], g: Sequence[int], m: Optional[Sequence[int]],
                 v: Optional[Sequence[int]], What: Sequence[int], what_dtype, stream: int = 0, grad_dtype="f32"):
        if isinstance(what_dtype, str):
            what_dtype = WHAT_DTYPES[what_dtype]
        if isinstance(grad_dtype, str):
            grad_dtype = GRAD_DTYPES[grad_dtype]
        n = len(numel)
        self._h = ctypes.c_void_p()
        self.n_tensors = n
        self.what_dtype = what_dtype
        self.grad_dtype = grad_dtype
        numel_arr = (ctypes.c_int64 * max(n, 1))(*numel)
        v_arr = _ptr_array(v) if v is not None else None
        m_arr = _ptr_array(m) if m is not None else None
        if grad_dtype == PO_GRAD_F32:
            _check(lib().pipeoptim_plan_create(
                ctypes.byref(self._h), n, numel_arr, _ptr_array(W), _ptr_array(g), m_arr, v_arr,
                _ptr_array(What), int(what_dtype), ctypes.c_void_p(stream)))
        else:
            _check(lib().pipeoptim_plan_create_mixed(
                ctypes.byref(self._h), n, numel_arr, _ptr_array(W), _ptr_array(g), int(grad_dtype), m_arr,
                v_arr, _ptr_array(What), int(what_dtype), ctypes.c_void_p(stream)))

    def step_predict(self, hyper: po_hyper, t: int, s: int, stream: int = 0) -> None:
        _check(lib().pipeoptim_step_predict(self._h, ctypes.byref(hyper), int(t), int(s), ctypes.c_void_p(stream)))

    def predict(self, hyper: po_hyper, t: int, s: int, stream: int = 0) -> None:
        _check(lib().pipeoptim_predict(self._h, ctypes.byref(hyper), int(t), int(s), ctypes.c_void_p(stream)))

    def get_predict_launch(self) -> po_launch:
        L = po_launch()
        _check(lib().pipeoptim_plan_get_predict_launch(self._h, ctypes.byref(L)))
        return L

    def set_predict_launch(self, **kw) -> po_launch:
        L = self.get_predict_launch()
        for k, val in kw.items():
            if not hasattr(L, k):
                raise TypeError("po_launch has no field %r" % k)
            setattr(L, k, int(val))
        _check(lib().pipeoptim_plan_set_predict_launch(self._h, ctypes.byref(L)))
        return L

    def set_pointers(self, which: int, ptrs: Sequence[int], stream: int = 0) -> None:
        _check(lib().pipeoptim_plan_set_pointers(self._h, int(which), _ptr_array(ptrs), ctypes.c_void_p(stream)))

    def get_launch(self) -> po_launch:
        L = po_launch()
        _check(lib().pipeoptim_plan_get_launch(self._h, ctypes.byref(L)))
        return L

    def set_launch(self, **kw) -> po_launch:
        L = self.get_launch()
        for k, val in kw.items():
            if not hasattr(L, k):
                raise TypeError("po_launch has no field %r" % k)
            setattr(L, k, int(val))
        _check(lib().pipeoptim_plan_set_launch(self._h, ctypes.byref(L)))
        return L

    def localize(self, arena: Optional["Arena"], stream: int = 0) -> int:
        """Marks the tensors whose fp32 streams lie in `arena` for the near-memory tile order; returns the
        number of parameters marked (None clears the marks).  `stream`: the stream the plan will run on."""
        n = ctypes.c_int64(0)
        _check(lib().pipeoptim_plan_localize(self._h, arena._h if arena is not None else None,
                                             ctypes.c_void_p(stream), ctypes.byref(n)))
        return n.value

    def learn_layout(self, stream: int = 0) -> int:
        """Finds the die layout of the plan's (caller-placed) buffers by timing loads and gives every chunk the
        near-memory tile order that suits it; returns the number of parameters in such chunks.  Blocking."""
        n = ctypes.c_int64(0)
        _check(lib().pipeoptim_plan_learn_layout(self._h, ctypes.c_void_p(stream), ctypes.byref(n)))
        return n.value

    def chunk_marks(self):
        """Per chunk-table entry: -1 plain order, 0 / 1 the XCC half that takes the first block of each group."""
        n = ctypes.c_int64(0)
        _check(lib().pipeoptim_plan_chunk_marks(self._h, None, 0, ctypes.byref(n)))
        buf = (ctypes.c_int8 * max(n.value, 1))()
        _check(lib().pipeoptim_plan_chunk_marks(self._h, buf, n.value, ctypes.byref(n)))
        return [buf[k] for k in range(n.value)]

    def near_share(self) -> float:
        """Estimated share of the fused call's HBM bytes served by the near die (0.5: plain order)."""
        x = ctypes.c_double(0.0)
        _check(lib().pipeoptim_plan_near_share(self._h, ctypes.byref(x)))
        return x.value

    def launch_phase(self) -> int:
        """XCC on which the plan's last reported launch started its round (-1: never localized)."""
        k = ctypes.c_int32(-2)
        _check(lib().pipeoptim_plan_launch_phase(self._h, ctypes.byref(k)))
        return k.value

    def local_params(self) -> int:
        n = ctypes.c_int64(-1)
        _check(lib().pipeoptim_plan_local_params(self._h, ctypes.byref(n)))
        return n.value

    def effective_launch(self, kernel: int, opt) -> po_launch:
        if isinstance(opt, str):
            opt = OPTIMIZERS[opt]
        L = po_launch()
        _check(lib().pipeoptim_plan_effective_launch(self._h, int(kernel), int(opt), ctypes.byref(L)))
        return L

    def info(self):
        a, b, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
        _check(lib().pipeoptim_plan_info(self._h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
        return {"n_params": a.value, "n_chunks": b.value, "n_unaligned": c.value}

    def destroy(self) -> None:
        if self._h:
            h, self._h = self._h, ctypes.c_void_p()
            _check(lib().pipeoptim_plan_destroy(h))

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def pipeoptim_device_sync_count() -> int:
    """How often the library has waited for the whole device so far (diagnostic)."""
    n = ctypes.c_int64(-1)
    _check(lib().pipeoptim_device_sync_count(ctypes.byref(n)))
    return n.value


def pipeoptim_step_predict_static(numel: Sequence[int], W: Sequence[int], g: Sequence[int], m: Optional[Sequence[int]],
                                  v: Optional[Sequence[int]], What: Sequence[int], what_dtype, hyper: po_hyper,
                                  t: int, s: int, stream: int = 0) -> None:
    """The fused call without a plan and without any allocation (tables in the library's fixed device array)."""
    if isinstance(what_dtype, str):
        what_dtype = WHAT_DTYPES[what_dtype]
    n = len(numel)
    numel_arr = (ctypes.c_int64 * max(n, 1))(*numel)
    _check(lib().pipeoptim_step_predict_static(
        n, numel_arr, _ptr_array(W), _ptr_array(g), _ptr_array(m) if m is not None else None,
        _ptr_array(v) if v is not None else None, _ptr_array(What), int(what_dtype), ctypes.byref(hyper),
        int(t), int(s), ctypes.c_void_p(stream)))


def pipeoptim_probe_copy(dst: int, src: int, nbytes: int, stream: int = 0) -> None:
    _check(lib().pipeoptim_probe_copy(ctypes.c_void_p(dst), ctypes.c_void_p(src), int(nbytes),
                                      ctypes.c_void_p(stream)))
