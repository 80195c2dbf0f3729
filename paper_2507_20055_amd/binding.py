"""ctypes binding of libdpcert.so: argument marshalling only, same names as the C ABI
(include/dpcert.h).  Every step of the path runs in the library's HIP kernels; there is no
fallback: if the library has not been built, importing this module raises."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np
import torch  # noqa: F401  -- imported BEFORE the library is loaded, on purpose: PyTorch ships its own
#               libamdhip64.so.7; loading it first makes the dynamic loader resolve this library's
#               dependency on the HIP runtime to that same copy, so the process holds ONE runtime and
#               device pointers / streams of torch tensors are valid inside the library.

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdpcert.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it first (python -m paper_2507_20055_amd.build "
                      "or __graft_entry__.build()); there is no CPU fallback")

_lib = ctypes.CDLL(LIB_PATH)

c_i32, c_i64, c_vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p


class dpc_options(ctypes.Structure):
    _fields_ = [("struct_size", c_i32), ("max_backsub_depth", c_i32), ("keep_symbolic", c_i32),
                ("fuse", c_i32), ("profile", c_i32), ("use_graph", c_i32), ("certifier", c_i32), ("final_backsub_depth", c_i32), ("stream", c_vp)]


CERTIFIERS = {"deeppoly": 0, "reusecert": 1, "skippoly": 2}


class dpc_profile(ctypes.Structure):
    _fields_ = [("struct_size", c_i32), ("contract_launches", c_i32), ("relax_launches", c_i32),
                ("concretise_launches", c_i32), ("other_launches", c_i32),
                ("contract_ms", ctypes.c_double), ("relax_ms", ctypes.c_double),
                ("concretise_ms", ctypes.c_double), ("other_ms", ctypes.c_double), ("total_ms", ctypes.c_double),
                ("contract_flop", ctypes.c_double), ("relax_bytes", ctypes.c_double),
                ("concretise_bytes", ctypes.c_double),
                ("chain_ms", ctypes.c_double), ("chain_flop", ctypes.c_double),
                ("chain_launches", c_i32), ("reserved", c_i32)]


EXPORTS = {
    "dpc_network_create": [ctypes.POINTER(c_vp)],
    "dpc_network_add_affine": [c_vp, c_i32, c_i32, c_vp, c_vp],
    "dpc_network_add_conv2d": [c_vp, c_i32, c_i32, c_i32, c_i32, c_i32, c_i32, c_i32, c_i32, c_vp, c_vp],
    "dpc_network_add_relu": [c_vp],
    "dpc_network_add_skip": [c_vp, c_i32],
    "dpc_network_finalize": [c_vp, c_i32],
    "dpc_network_destroy": [c_vp],
    "dpc_options_default": [ctypes.POINTER(dpc_options)],
    "dpc_certify": [c_vp, c_i32, c_vp, c_vp, c_vp, ctypes.POINTER(dpc_options), ctypes.POINTER(c_vp)],
    "dpc_certify_static": [c_vp, c_i32, c_vp, c_vp, c_vp, ctypes.POINTER(dpc_options), c_vp, c_vp, c_vp, c_vp],
    "dpc_result_concrete": [c_vp, c_i32, c_vp, c_vp],
    "dpc_result_relaxation": [c_vp, c_i32, c_vp, c_vp, c_vp],
    "dpc_result_symbolic": [c_vp, c_i32, c_i32, c_vp, c_vp],
    "dpc_result_margin_symbolic": [c_vp, c_vp, c_vp],
    "dpc_result_relu_symbolic": [c_vp, c_i32, c_i32, c_vp, c_vp],
    "dpc_result_verdict": [c_vp, c_vp, c_vp],
    "dpc_result_profile": [c_vp, ctypes.POINTER(dpc_profile)],
    "dpc_result_destroy": [c_vp],
    "dpc_op_contract": [c_vp, c_i64, c_i32, c_i32, c_vp, c_i32, c_i32, c_vp, c_i32, c_vp],
    "dpc_op_relax_step": [c_vp, c_i32, c_vp, c_i32, c_i32, c_i32, c_i32, c_vp, c_vp, c_vp, c_vp, c_vp, c_i32, c_vp],
    "dpc_op_concretise": [c_vp, c_i32, c_vp, c_i32, c_i32, c_i32, c_i32, c_vp, c_vp, c_vp, c_vp, c_vp],
    "dpc_op_conv_transpose": [c_vp, c_i64, c_i32, c_i32, c_i32, c_i32, c_i32, c_i32, c_i32, c_i32, c_i32, c_vp,
                              c_vp, c_i32, c_i32, c_i32, c_vp],
    "dpc_tuning_set": [ctypes.c_char_p, c_i32],
    "dpc_network_tuning_set": [c_vp, ctypes.c_char_p, c_i32],
}
for _name, _args in EXPORTS.items():
    _f = getattr(_lib, _name)
    _f.argtypes = _args
    _f.restype = c_i32
_lib.dpc_last_error.restype = ctypes.c_char_p
_lib.dpc_last_error.argtypes = []
_lib.dpc_version.restype = ctypes.c_char_p
_lib.dpc_version.argtypes = []

STATUS = {0: "DPC_OK", 1: "DPC_EINVAL", 2: "DPC_EUNSUPPORTED", 3: "DPC_ENOMEM", 4: "DPC_EHIP", 5: "DPC_ESTATE"}


class DpcError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{STATUS.get(code, code)}: {msg}")
        self.code = code


def _check(code: int):
    if code != 0:
        raise DpcError(code, _lib.dpc_last_error().decode())


def dpc_version() -> str:
    return _lib.dpc_version().decode()


def dpc_tuning_set(key: str, value: int):
    _check(_lib.dpc_tuning_set(key.encode(), value))


TUNING_DEFAULT = -2 ** 31          # DPC_TUNING_DEFAULT: removes a network's override


def _ptr(a):
    """Address of a numpy array or torch tensor (host or device); None -> NULL."""
    if a is None:
        return None
    if isinstance(a, np.ndarray):
        assert a.flags["C_CONTIGUOUS"]
        return a.ctypes.data
    assert a.is_contiguous()
    return a.data_ptr()


def _f32(a):
    if isinstance(a, np.ndarray):
        return np.ascontiguousarray(a, dtype=np.float32)
    import torch
    assert a.dtype == torch.float32
    return a.contiguous()


class Network:
    """dpc_network handle.  `net` is duck-typed like workloads.Network."""

    def __init__(self, net, device: int = 0):
        self._h = c_vp()
        _check(_lib.dpc_network_create(ctypes.byref(self._h)))
        self.sizes = [net.n_in]
        self.kinds = []
        try:
            for L in net.layers:
                if L.kind == "affine":
                    W, b = _f32(np.asarray(L.W)), _f32(np.asarray(L.b))
                    _check(_lib.dpc_network_add_affine(self._h, W.shape[0], W.shape[1], _ptr(W), _ptr(b)))
                    self.sizes.append(W.shape[0])
                elif L.kind == "conv":
                    K, b = _f32(np.asarray(L.W)), _f32(np.asarray(L.b))
                    Ci, H, Wd = L.in_shape
                    Co, _, kh, kw = K.shape
                    _check(_lib.dpc_network_add_conv2d(self._h, Ci, H, Wd, Co, kh, kw, L.stride, L.pad, _ptr(K), _ptr(b)))
                    Ho = (H + 2 * L.pad - kh) // L.stride + 1
                    Wo = (Wd + 2 * L.pad - kw) // L.stride + 1
                    self.sizes.append(Co * Ho * Wo)
                elif L.kind == "relu":
                    _check(_lib.dpc_network_add_relu(self._h))
                    self.sizes.append(self.sizes[-1])
                elif L.kind == "add":
                    _check(_lib.dpc_network_add_skip(self._h, int(L.skip)))
                    self.sizes.append(self.sizes[-1])
                else:
                    raise ValueError(L.kind)
                self.kinds.append(L.kind)
            _check(_lib.dpc_network_finalize(self._h, device))
        except Exception:
            _lib.dpc_network_destroy(self._h)
            self._h = None
            raise
        self._results = []

    def tuning_set(self, key: str, value: int = TUNING_DEFAULT):
        """dpc_network_tuning_set: this network's value of a tuning knob (TUNING_DEFAULT: back to the process-wide one)."""
        _check(_lib.dpc_network_tuning_set(self._h, key.encode(), value))

    def certify(self, lo, hi, label=None, *, max_backsub_depth: int = -1, keep_symbolic: int = 0,
                fuse: int = 1, profile: int = 0, use_graph: int = 1, stream: int = 0,
                reuse: Optional["Result"] = None, certifier: str = "deeppoly",
                final_backsub_depth: int = -2) -> "Result":
        lo, hi = _f32(lo), _f32(hi)
        batch = int(lo.shape[0])
        assert tuple(lo.shape) == (batch, self.sizes[0]) and tuple(hi.shape) == tuple(lo.shape)
        if label is not None and isinstance(label, np.ndarray):
            label = np.ascontiguousarray(label, dtype=np.int32)
        opt = dpc_options()
        _check(_lib.dpc_options_default(ctypes.byref(opt)))
        opt.max_backsub_depth, opt.keep_symbolic, opt.fuse, opt.profile = max_backsub_depth, keep_symbolic, fuse, profile
        opt.use_graph = use_graph
        opt.certifier = CERTIFIERS[certifier]
        opt.final_backsub_depth = final_backsub_depth
        opt.stream = stream or None
        h = c_vp(reuse._h.value) if reuse is not None else c_vp()
        _check(_lib.dpc_certify(self._h, batch, _ptr(lo), _ptr(hi), _ptr(label), ctypes.byref(opt), ctypes.byref(h)))
        if reuse is not None:
            return reuse
        r = Result(self, h, batch)
        self._results.append(r)
        return r

    def certify_static(self, lo, hi, label, out_l, out_u, margin_lb=None, verdict=None, *, max_backsub_depth: int = -1,
                       fuse: int = 1, stream: int = 0, final_backsub_depth: int = -2):
        """dpc_certify_static: device tensors in, device tensors out, no device allocation inside the call."""
        batch = int(lo.shape[0])
        assert tuple(lo.shape) == (batch, self.sizes[0]) and tuple(hi.shape) == tuple(lo.shape)
        opt = dpc_options()
        _check(_lib.dpc_options_default(ctypes.byref(opt)))
        opt.max_backsub_depth, opt.fuse, opt.final_backsub_depth = max_backsub_depth, fuse, final_backsub_depth
        opt.stream = stream or None
        _check(_lib.dpc_certify_static(self._h, batch, _ptr(lo), _ptr(hi), _ptr(label), ctypes.byref(opt),
                                       _ptr(out_l), _ptr(out_u), _ptr(margin_lb), _ptr(verdict)))

    def close(self):
        for r in self._results:
            r.close()
        self._results = []
        if self._h:
            _check(_lib.dpc_network_destroy(self._h))
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Result:
    def __init__(self, net: Network, handle, batch: int):
        self.net, self._h, self.batch = net, handle, batch

    def concrete(self, layer: int):
        n = self.net.sizes[layer]
        l = np.empty((self.batch, n), np.float32)
        u = np.empty((self.batch, n), np.float32)
        _check(_lib.dpc_result_concrete(self._h, layer, _ptr(l), _ptr(u)))
        return l, u

    def relaxation(self, layer: int):
        n = self.net.sizes[layer]
        out = [np.empty((self.batch, n), np.float32) for _ in range(3)]
        _check(_lib.dpc_result_relaxation(self._h, layer, *[_ptr(a) for a in out]))
        return tuple(out)

    def symbolic(self, layer: int, side: int):
        n, n0 = self.net.sizes[layer], self.net.sizes[0]
        coeff = np.empty((self.batch, n, n0), np.float32)
        cst = np.empty((self.batch, n), np.float32)
        _check(_lib.dpc_result_symbolic(self._h, layer, side, _ptr(coeff), _ptr(cst)))
        return coeff, cst

    def relu_symbolic(self, layer: int, side: int):
        n, nb = self.net.sizes[layer], self.net.sizes[layer - 2]
        coeff = np.empty((self.batch, n, nb), np.float32)
        cst = np.empty((self.batch, n), np.float32)
        _check(_lib.dpc_result_relu_symbolic(self._h, layer, side, _ptr(coeff), _ptr(cst)))
        return coeff, cst

    def margin_symbolic(self):
        nq, n0 = self.net.sizes[-1] - 1, self.net.sizes[0]
        coeff = np.empty((self.batch, nq, n0), np.float32)
        cst = np.empty((self.batch, nq), np.float32)
        _check(_lib.dpc_result_margin_symbolic(self._h, _ptr(coeff), _ptr(cst)))
        return coeff, cst

    def verdict(self):
        nq = self.net.sizes[-1] - 1
        v = np.empty((self.batch,), np.int32)
        m = np.empty((self.batch, nq), np.float32)
        _check(_lib.dpc_result_verdict(self._h, _ptr(v), _ptr(m)))
        return v, m

    def profile(self) -> dict:
        p = dpc_profile()
        p.struct_size = ctypes.sizeof(dpc_profile)
        _check(_lib.dpc_result_profile(self._h, ctypes.byref(p)))
        return {k: getattr(p, k) for k, _ in dpc_profile._fields_ if k != "struct_size"}

    def close(self):
        if self._h:
            _check(_lib.dpc_result_destroy(self._h))
            self._h = None


# ---- the three hot kernels on device tensors (torch is used for device memory only) ----------

def dpc_op_contract(A, K: int, W, N: int, Cout, stream: int = 0):
    M = A.shape[0]
    _check(_lib.dpc_op_contract(A.data_ptr(), M, K, A.stride(0), W.data_ptr(), N, W.stride(0),
                                Cout.data_ptr(), Cout.stride(0), stream or None))


def dpc_op_relax_step(C, cst, nsides: int, batch: int, R: int, n: int, lam, mu, nu, bias,
                      shared_src=None, stream: int = 0):
    _check(_lib.dpc_op_relax_step(C.data_ptr(), C.stride(0), cst.data_ptr(), nsides, batch, R, n,
                                  _ptr(lam), _ptr(mu), _ptr(nu), _ptr(bias), _ptr(shared_src),
                                  shared_src.stride(0) if shared_src is not None else 0, stream or None))


def dpc_op_concretise(C, cst, nsides: int, batch: int, R: int, n: int, lo, hi, out_l, out_u, stream: int = 0):
    _check(_lib.dpc_op_concretise(C.data_ptr(), C.stride(0), cst.data_ptr(), nsides, batch, R, n,
                                  lo.data_ptr(), hi.data_ptr(), out_l.data_ptr(), _ptr(out_u), stream or None))


def dpc_op_conv_transpose(inp, ih: int, iw: int, Co: int, K_host, stride: int, off: int, out, oh: int, ow: int, stream: int = 0):
    K_host = np.ascontiguousarray(K_host, dtype=np.float32)
    Co2, Ci, kh, kw = K_host.shape
    assert Co2 == Co
    _check(_lib.dpc_op_conv_transpose(inp.data_ptr(), inp.shape[0], inp.stride(0), ih, iw, Co, Ci, kh, kw, stride, off,
                                      K_host.ctypes.data, out.data_ptr(), out.stride(0), oh, ow, stream or None))
