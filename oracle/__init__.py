"""Float64 CPU oracle for DeepPoly bound propagation -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline``
leg may import this package.  It shares no code with the GPU library and never
imports it.  ``deeppoly_oracle.c`` holds the arithmetic (plain loops following
the DeepPoly specification of the paper's Appendix C under the map / traverse
semantics of Sections 2.2 and 3.2); this file only marshals numpy arrays.

``neuron_level.py`` is a second, independent pure-Python implementation (a table of
neurons, sparse expressions, one substitution loop) used as a brute-force
cross-check on tiny networks.

Networks are duck-typed: an object with ``n_in`` and ``layers``; each layer has
``kind`` in {"affine", "conv", "relu", "add"}, ``W``, ``b`` and, for conv, ``stride``,
``pad``, ``in_shape`` = (Ci, H, W).  Neurons of a conv layer are flattened
(channel, row, column).  An "add" layer (residual networks) outputs the layer below plus
the output of layer index ``skip`` (0 = the input, i = the i-th layer).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "deeppoly_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Layer(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int), ("n_in", ctypes.c_int), ("n_out", ctypes.c_int),
                ("W", ctypes.c_void_p), ("b", ctypes.c_void_p),
                ("Ci", ctypes.c_int), ("H", ctypes.c_int), ("Wd", ctypes.c_int), ("Co", ctypes.c_int),
                ("kh", ctypes.c_int), ("kw", ctypes.c_int), ("stride", ctypes.c_int), ("pad", ctypes.c_int),
                ("Ho", ctypes.c_int), ("Wo", ctypes.c_int), ("skip", ctypes.c_int)]


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.dpo_run.restype = ctypes.c_int
        _lib.dpo_run_reuse.restype = ctypes.c_int
        assert _lib.dpo_layer_struct_size() == ctypes.sizeof(_Layer)
    return _lib


@dataclass
class OracleResult:
    l: List[np.ndarray]                    # index 0 = input layer; [B, n_i] float64
    u: List[np.ndarray]
    lam: Dict[int, np.ndarray] = field(default_factory=dict)   # ReLU layer index -> [B, n]
    mu: Dict[int, np.ndarray] = field(default_factory=dict)
    nu: Dict[int, np.ndarray] = field(default_factory=dict)
    margin: Optional[np.ndarray] = None    # [B, nK-1]
    verdict: Optional[np.ndarray] = None   # [B] int32, 1 = verified
    sym: Optional[dict] = None             # {"cl","kl","cu","ku"} input-level expressions


def run(net, lo, hi, label=None, sym_layer: int = -1, max_depth: int = -1,
        threads: Optional[int] = None, certifier: str = "deeppoly", max_depth_last: Optional[int] = None) -> OracleResult:
    """certifier: "deeppoly" (Appendix C, DeepPoly; max_depth >= 0 gives DeepPoly_p; max_depth_last, if given, is the
    limit of the last layer and the property rows: max_depth = 0, max_depth_last = -1 is CROWN-IBP) or "reusecert" (Appendix C,
    ReuseCert: l, u of affine layers are the concretised stored bounds, ReLU-layer l, u stay 0, sym_layer may
    name any affine layer)."""
    lib = _load()
    assert certifier in ("deeppoly", "reusecert")
    assert certifier == "deeppoly" or (max_depth < 0 and max_depth_last is None)
    if threads is not None:
        os.environ["OMP_NUM_THREADS"] = str(threads)
    lo = np.ascontiguousarray(lo, dtype=np.float32)
    hi = np.ascontiguousarray(hi, dtype=np.float32)
    B, n0 = lo.shape
    assert n0 == net.n_in and hi.shape == lo.shape
    nl = len(net.layers)
    arr = (_Layer * nl)()
    keep = []
    n_prev = n0
    sizes = [n0]
    for i, L in enumerate(net.layers):
        a = arr[i]
        a.n_in = n_prev
        if L.kind == "affine":
            W = np.ascontiguousarray(L.W, dtype=np.float32)
            b = np.ascontiguousarray(L.b, dtype=np.float32)
            assert W.shape[1] == n_prev and b.shape == (W.shape[0],)
            keep += [W, b]
            a.kind, a.n_out = 0, W.shape[0]
            a.W, a.b = W.ctypes.data, b.ctypes.data
        elif L.kind == "conv":
            W = np.ascontiguousarray(L.W, dtype=np.float32)
            b = np.ascontiguousarray(L.b, dtype=np.float32)
            keep += [W, b]
            Ci, H, Wd = L.in_shape
            Co, Ci2, kh, kw = W.shape
            assert Ci2 == Ci and Ci * H * Wd == n_prev and b.shape == (Co,)
            Ho = (H + 2 * L.pad - kh) // L.stride + 1
            Wo = (Wd + 2 * L.pad - kw) // L.stride + 1
            a.kind, a.n_out = 1, Co * Ho * Wo
            a.W, a.b = W.ctypes.data, b.ctypes.data
            a.Ci, a.H, a.Wd, a.Co, a.kh, a.kw = Ci, H, Wd, Co, kh, kw
            a.stride, a.pad, a.Ho, a.Wo = L.stride, L.pad, Ho, Wo
        elif L.kind == "relu":
            a.kind, a.n_out = 2, n_prev
        elif L.kind == "add":
            assert certifier == "deeppoly", "ReuseCert is specified for chain networks only"
            assert 0 <= L.skip <= i and sizes[L.skip] == n_prev
            a.kind, a.n_out, a.skip = 3, n_prev, L.skip
        else:
            raise ValueError(L.kind)
        n_prev = a.n_out
        sizes.append(n_prev)

    PD = ctypes.POINTER(ctypes.c_double)
    l = [np.zeros((B, n), dtype=np.float64) for n in sizes]
    u = [np.zeros((B, n), dtype=np.float64) for n in sizes]
    res = OracleResult(l=l, u=u)

    def ptrs(arrs):
        out = (ctypes.c_void_p * (nl + 1))()
        for i, a in enumerate(arrs):
            out[i] = a.ctypes.data if a is not None else None
        return out

    lam = [None] * (nl + 1)
    mu = [None] * (nl + 1)
    nu = [None] * (nl + 1)
    for i, L in enumerate(net.layers):
        if L.kind == "relu":
            for d, store in ((lam, res.lam), (mu, res.mu), (nu, res.nu)):
                d[i + 1] = np.zeros((B, sizes[i + 1]), dtype=np.float64)
                store[i + 1] = d[i + 1]

    lab_p = None
    mar_p = None
    ver_p = None
    if label is not None:
        label = np.ascontiguousarray(label, dtype=np.int32)
        assert label.shape == (B,)
        res.margin = np.zeros((B, sizes[-1] - 1), dtype=np.float64)
        res.verdict = np.zeros((B,), dtype=np.int32)
        lab_p, mar_p, ver_p = label.ctypes.data, res.margin.ctypes.data, res.verdict.ctypes.data

    sp = [None] * 4
    if sym_layer >= 0:
        # nl + 1 names the property's rows (lower expressions of logit[label] - logit[o]; "cu", "ku" stay zero)
        ns = sizes[sym_layer] if sym_layer <= nl else sizes[-1] - 1
        res.sym = dict(cl=np.zeros((B, ns, n0)), kl=np.zeros((B, ns)),
                       cu=np.zeros((B, ns, n0)), ku=np.zeros((B, ns)))
        sp = [res.sym[k].ctypes.data for k in ("cl", "kl", "cu", "ku")]

    vp = ctypes.c_void_p
    if certifier == "reusecert":
        rc = lib.dpo_run_reuse(ctypes.c_int(nl), arr, ctypes.c_int(B), vp(lo.ctypes.data), vp(hi.ctypes.data), vp(lab_p),
                               ptrs(l), ptrs(u), ptrs(lam), ptrs(mu), ptrs(nu), vp(mar_p), vp(ver_p),
                               ctypes.c_int(sym_layer), vp(sp[0]), vp(sp[1]), vp(sp[2]), vp(sp[3]))
    else:
        rc = lib.dpo_run(ctypes.c_int(nl), arr, ctypes.c_int(B), vp(lo.ctypes.data), vp(hi.ctypes.data), vp(lab_p),
                         ptrs(l), ptrs(u), ptrs(lam), ptrs(mu), ptrs(nu), vp(mar_p), vp(ver_p),
                         ctypes.c_int(sym_layer), vp(sp[0]), vp(sp[1]), vp(sp[2]), vp(sp[3]),
                         ctypes.c_int(max_depth), ctypes.c_int(-2 if max_depth_last is None else max_depth_last))
    if rc != 0:
        raise ValueError(f"the oracle rejected its input (code {rc})")
    del keep
    return res
