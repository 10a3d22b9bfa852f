"""ctypes front end of ``po_oracle.c`` (argument marshalling only).

Test infrastructure: see the header of ``po_oracle.c``.  ``build()`` compiles
the C file with gcc into ``libpo_oracle.so`` next to it; ``OracleLib`` wraps one
built library (the tests also load deliberately broken builds through it, to
check that the pins notice); the module-level functions use the real one.
"""
import ctypes
import os
import subprocess

import numpy as np

SGDM, ADAM, ADAMW, NESTEROV, RMSPROP, ADAGRAD = 0, 1, 2, 3, 4, 5

_HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(_HERE, "po_oracle.c")
_LIB = os.path.join(_HERE, "libpo_oracle.so")

# No fast-math, no FMA contraction: the arithmetic is exactly the fp64 operations the source spells out.
CFLAGS = ["-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra"]


def compile_source(src, out):
    tmp = out + ".tmp.%d" % os.getpid()
    subprocess.run(["gcc"] + CFLAGS + ["-o", tmp, src, "-lm"], check=True)
    os.replace(tmp, out)
    return out


def build(force=False):
    """Compile po_oracle.c (if it is newer than the library, or if forced)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(SOURCE):
        return _LIB
    return compile_source(SOURCE, _LIB)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


class OracleLib:
    """One loaded build of the oracle."""

    SGDM, ADAM, ADAMW, NESTEROV, RMSPROP, ADAGRAD = SGDM, ADAM, ADAMW, NESTEROV, RMSPROP, ADAGRAD

    def __init__(self, path):
        lib = ctypes.CDLL(path)
        f32p = ctypes.POINTER(ctypes.c_float)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        scal = [ctypes.c_int, ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_double,
                ctypes.c_double, ctypes.c_int, ctypes.c_longlong, ctypes.c_int, ctypes.c_longlong]
        lib.po_oracle_step_predict.restype = ctypes.c_int
        lib.po_oracle_step_predict.argtypes = scal + [f32p, f32p, f32p, f32p, f32p, f32p, f32p, f32p, u16p, ctypes.c_int]
        lib.po_oracle_predict.restype = ctypes.c_int
        lib.po_oracle_predict.argtypes = scal + [f32p, f32p, f32p, f32p, u16p, ctypes.c_int]
        lib.po_oracle_bf16_from_f32_array.restype = None
        lib.po_oracle_bf16_from_f32_array.argtypes = [f32p, u16p, ctypes.c_longlong]
        lib.po_oracle_version_difference.restype = ctypes.c_int
        lib.po_oracle_version_difference.argtypes = [ctypes.c_int, ctypes.c_int]
        self._lib = lib

    def step_predict(self, opt, W, g, m, v=None, *, lr, beta1, beta2, eps=0.0, weight_decay=0.0,
                     decay_in_prediction=True, t=1, s=0, nthreads=1):
        """One fused step + prediction on flat fp32 arrays.

        Returns a dict with ``W``, ``m``, ``v`` (None where the optimizer has no such state),
        ``What`` (fp32) and ``What_bf16`` (uint16 bit patterns).  SGDM: ``beta1`` is the momentum
        factor and ``beta2`` the dampening; Nesterov: ``beta1`` is the momentum factor; RMSprop:
        ``beta2`` is the smoothing constant; Adagrad uses neither.
        """
        W, pW = _f32(W)
        g, pg = _f32(g)
        n = W.size
        null_f = ctypes.POINTER(ctypes.c_float)()
        if g.size != n or (m is not None and np.asarray(m).size != n) or (v is not None and np.asarray(v).size != n):
            raise ValueError("oracle: operand sizes differ")
        if m is not None:
            m, pm = _f32(m)
        else:
            pm = null_f
        if v is not None:
            v, pv = _f32(v)
            v_out = np.empty(n, np.float32)
            pvo = v_out.ctypes.data_as(ctypes.POINTER(ctypes.c_float))
        else:
            pv, v_out, pvo = null_f, None, null_f
        W_out = np.empty(n, np.float32)
        m_out = np.empty(n, np.float32) if m is not None else None
        pmo = m_out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)) if m is not None else null_f
        What = np.empty(n, np.float32)
        What16 = np.empty(n, np.uint16)
        rc = self._lib.po_oracle_step_predict(
            int(opt), float(lr), float(beta1), float(beta2), float(eps), float(weight_decay),
            int(bool(decay_in_prediction)), int(t), int(s), n, pW, pg, pm, pv,
            W_out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), pmo, pvo,
            What.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
            What16.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), int(nthreads))
        if rc != 0:
            raise ValueError("oracle: invalid argument (opt=%r t=%r s=%r)" % (opt, t, s))
        return {"W": W_out, "m": m_out, "v": v_out, "What": What, "What_bf16": What16}

    def predict(self, opt, W, m, v=None, *, lr, beta1, beta2, eps=0.0, weight_decay=0.0,
                decay_in_prediction=True, t=1, s=0, nthreads=1):
        """Prediction from the cached state alone.  Returns ``What`` (fp32) and ``What_bf16`` (uint16 patterns)."""
        W, pW = _f32(W)
        m, pm = _f32(m)
        n = W.size
        if m.size != n or (v is not None and np.asarray(v).size != n):
            raise ValueError("oracle: operand sizes differ")
        if v is not None:
            v, pv = _f32(v)
        else:
            pv = ctypes.POINTER(ctypes.c_float)()
        What = np.empty(n, np.float32)
        What16 = np.empty(n, np.uint16)
        rc = self._lib.po_oracle_predict(
            int(opt), float(lr), float(beta1), float(beta2), float(eps), float(weight_decay),
            int(bool(decay_in_prediction)), int(t), int(s), n, pW, pm, pv,
            What.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
            What16.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), int(nthreads))
        if rc != 0:
            raise ValueError("oracle: invalid argument (opt=%r t=%r s=%r)" % (opt, t, s))
        return {"What": What, "What_bf16": What16}

    def bf16_from_f32(self, x):
        """Round fp32 values to bf16 bit patterns (nearest, ties to even)."""
        x, px = _f32(np.asarray(x).reshape(-1))
        out = np.empty(x.size, np.uint16)
        self._lib.po_oracle_bf16_from_f32_array(px, out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), x.size)
        return out

    @staticmethod
    def f32_from_bf16(bits):
        """Widen bf16 bit patterns to fp32 (exact: a bf16 is the upper half of an fp32)."""
        return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)

    def version_difference(self, D, rank):
        """Paper Eq. 4."""
        return self._lib.po_oracle_version_difference(int(D), int(rank))


_default = None


def _get():
    global _default
    if _default is None:
        _default = OracleLib(build())
    return _default


def step_predict(*a, **k):
    return _get().step_predict(*a, **k)


def predict(*a, **k):
    return _get().predict(*a, **k)


def bf16_from_f32(x):
    return _get().bf16_from_f32(x)


def f32_from_bf16(bits):
    return OracleLib.f32_from_bf16(bits)


def version_difference(D, rank):
    return _get().version_difference(D, rank)


step_predict.__doc__ = OracleLib.step_predict.__doc__
predict.__doc__ = OracleLib.predict.__doc__
