"""ctypes front end of the C loop-nest oracle (einsum_ref.c).  TEST INFRASTRUCTURE ONLY.

`einsum_ref(spec, X, Y, ...)` evaluates one extended-einsum vertex exactly as the
general form of Section 3 of the paper states it: every output index gets the
(+)-aggregate, over all bindings of the labels missing from the output, of the
scalar function (x) applied to the joined input entries.  Inputs are numpy
arrays in their stored dtype (float64, float32, or uint16 holding bf16 bits).
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

from . import build as _build

_lib = None

OTIMES = {"mul": 0, "add": 1, "sub": 2, "div": 3, "sqdiff": 4, "absdiff": 5, "exp_sub": 6,
          "relu_grad": 7, "silu_mul": 8,
          "ident": 32, "scale": 33, "relu": 34, "exp": 35, "log": 36}
OPLUS = {"none": 0, "sum": 1, "max": 2}
_DT = {"f64": 0, "f32": 1, "bf16": 2}


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(os.environ.get("EINSUM_REF_LIB") or _build.build())   # override: another build of the same source (sanitizers)
        _lib.einsum_ref.restype = ctypes.c_int
        _lib.er_round_bf16.restype = ctypes.c_double
        _lib.er_round_bf16.argtypes = [ctypes.c_double]
    return _lib


def round_bf16(x: float) -> float:
    return float(_load().er_round_bf16(float(x)))


def _dt_of(a: np.ndarray, dtype: Optional[str]) -> str:
    if dtype is not None:
        return dtype
    if a.dtype == np.float64:
        return "f64"
    if a.dtype == np.float32:
        return "f32"
    if a.dtype == np.uint16:
        return "bf16"
    raise TypeError(f"unsupported array dtype {a.dtype}")


def split_spec(spec: str):
    lhs, rhs = spec.split("->")
    ops = lhs.split(",")
    if len(ops) not in (1, 2):
        raise ValueError("an EinSum is unary or binary")
    return list(ops[0]), (list(ops[1]) if len(ops) == 2 else None), list(rhs)


def einsum_ref(spec: str, X: np.ndarray, Y: Optional[np.ndarray] = None, *,
               otimes: str = "mul", oplus: str = "sum", alpha: float = 1.0,
               out_dtype: str = "f64", x_dtype: Optional[str] = None, y_dtype: Optional[str] = None,
               sel: Optional[Sequence[int]] = None) -> np.ndarray:
    """Evaluate one vertex; returns float64 values already rounded to out_dtype.

    With sel (flat row-major indices into Z) only those outputs are computed and a
    1-D array is returned; otherwise a dense array with Z's bound.
    """
    lib = _load()
    lX, lY, lZ = split_spec(spec)
    if (lY is None) != (Y is None):
        raise ValueError("operand count does not match the spec")
    labels = []
    for l in lX + (lY or []):
        if l not in labels:
            labels.append(l)
    if X.ndim != len(lX) or (Y is not None and Y.ndim != len(lY)):
        raise ValueError("operand rank does not match its label list")
    bound = {}
    for l, n in zip(lX, X.shape):
        bound[l] = int(n)
    if Y is not None:
        for l, n in zip(lY, Y.shape):
            if l in bound and bound[l] != int(n):
                raise ValueError(f"label {l}: bounds {bound[l]} and {n} differ")
            bound[l] = int(n)
    for l in lZ:
        if l not in bound:
            raise ValueError(f"output label {l} is in neither input (broadcast)")
    lid = {l: i for i, l in enumerate(labels)}
    b = (ctypes.c_int64 * max(1, len(labels)))(*[bound[l] for l in labels])

    def prep(a, labs, dt):
        isz = a.dtype.itemsize
        lab = (ctypes.c_int * max(1, len(labs)))(*[lid[l] for l in labs])
        st = (ctypes.c_int64 * max(1, len(labs)))(*[s // isz for s in a.strides])
        return lab, st, a.ctypes.data_as(ctypes.c_void_p), _DT[dt]

    X = np.asarray(X)
    labXc, stX, pX, dX = prep(X, lX, _dt_of(X, x_dtype))
    if Y is not None:
        Y = np.asarray(Y)
        labYc, stY, pY, dY = prep(Y, lY, _dt_of(Y, y_dtype))
        rankY = len(lY)
    else:
        labYc, stY, pY, dY, rankY = None, None, None, 0, 0
    labZc = (ctypes.c_int * max(1, len(lZ)))(*[lid[l] for l in lZ])
    zshape = tuple(bound[l] for l in lZ)
    if sel is not None:
        selarr = np.ascontiguousarray(sel, dtype=np.int64)
        out = np.empty(selarr.size, dtype=np.float64)
        psel, nsel = selarr.ctypes.data_as(ctypes.c_void_p), selarr.size
    else:
        out = np.empty(zshape, dtype=np.float64)
        psel, nsel = None, 0
    rc = lib.einsum_ref(ctypes.c_int(len(labels)), b,
                        ctypes.c_int(len(lX)), labXc, stX, pX, ctypes.c_int(dX),
                        ctypes.c_int(rankY), labYc, stY, pY, ctypes.c_int(dY),
                        ctypes.c_int(len(lZ)), labZc,
                        ctypes.c_int(OTIMES[otimes]), ctypes.c_int(OPLUS[oplus]), ctypes.c_double(alpha),
                        ctypes.c_int(_DT[out_dtype]),
                        out.ctypes.data_as(ctypes.c_void_p), ctypes.c_int64(nsel), psel)
    if rc != 0:
        raise ValueError(f"einsum_ref rejected the request (code {rc}) for spec {spec!r}")
    return out
