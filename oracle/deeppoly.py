"""ctypes wrapper of the C oracle (oracle/deeppoly_oracle.c).  TEST INFRASTRUCTURE ONLY.

The wrapper only marshals arguments; all arithmetic is in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "deeppoly_oracle.c")
_LIB = os.path.join(_HERE, "libdeeppoly_oracle.so")
# The mutation checks of the test suite (tests/test_oracle_mutations.py) point this at a copy of the C file with
# one mistake planted, and run single pins against it in a process of their own; nothing else sets it.
if os.environ.get("DEEPPOLY_ORACLE_SRC"):
    _SRC = os.path.abspath(os.environ["DEEPPOLY_ORACLE_SRC"])
    _LIB = os.path.splitext(_SRC)[0] + ".so"
_lib = None

# -frounding-math: the code switches the rounding mode; -ffp-contract=off: no fused multiply-add
_CFLAGS = ["-O2", "-std=c11", "-frounding-math", "-fno-fast-math", "-ffp-contract=off", "-fopenmp",
           "-shared", "-fPIC", "-Wall", "-Wno-unknown-pragmas"]


def build_oracle(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *_CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build_oracle()
    L = C.CDLL(_LIB)
    P = C.c_void_p
    fp = C.POINTER(C.c_float)
    dp = C.POINTER(C.c_double)
    ip = C.POINTER(C.c_int)
    bp = C.POINTER(C.c_byte)
    L.dp_create.restype = P
    L.dp_create.argtypes = [C.c_int] * 3
    L.dp_destroy.argtypes = [P]
    L.dp_add_dense.argtypes = [P, C.c_int, C.c_int, fp, fp]
    L.dp_add_conv2d.argtypes = [P] + [C.c_int] * 8 + [fp, fp]
    L.dp_add_avgpool2d.argtypes = [P] + [C.c_int] * 7
    L.dp_add_relu.argtypes = [P, C.c_int]
    L.dp_add_residual.argtypes = [P, C.c_int, C.c_int]
    L.dp_num_layers.argtypes = [P]
    L.dp_layer_size.argtypes = [P, C.c_int]
    L.dp_set_options.argtypes = [P, C.c_int, C.c_int]
    L.dp_request_bounds.argtypes = [P, C.c_int]
    L.dp_set_collapse.argtypes = [P, C.c_int]
    L.dp_set_early_termination.argtypes = [P, C.c_int]
    L.dp_set_float_inference.argtypes = [P, C.c_int]
    L.dp_get_inference_error.argtypes = [P, C.c_int, dp]
    L.dp_set_term_override.argtypes = [P, C.c_int, ip]
    L.dp_get_term_layer.argtypes = [P, C.c_int, ip]
    L.dp_get_interval_image.argtypes = [P, C.c_int, dp, dp]
    L.dp_set_lambda_override.argtypes = [P, C.c_int, bp]
    L.dp_set_gamma_override.argtypes = [P, C.c_int, dp]
    L.dp_set_box.argtypes = [P, dp, dp]
    L.dp_set_ball.argtypes = [P, fp, C.c_float, C.c_float, C.c_float]
    L.dp_set_bounds.argtypes = [P, C.c_int, dp, dp]
    L.dp_get_bounds.argtypes = [P, C.c_int, dp, dp]
    L.dp_get_relaxation.argtypes = [P, C.c_int, dp, dp, bp]
    L.dp_bound_rows.argtypes = [P, C.c_int, ip, C.c_int, dp, dp]
    L.dp_analyze_layer.argtypes = [P, C.c_int]
    L.dp_analyze.argtypes = [P]
    L.dp_certify.argtypes = [P, C.c_int, ip, dp]
    L.dp_bound_forms.argtypes = [P, C.c_int, dp, dp, dp]
    L.dp_selftest_rounding.argtypes = [C.c_double] * 3
    L.dp_num_threads.restype = C.c_int
    bad = L.dp_selftest_rounding(1.0, 1e-30, 1.0 / 3.0)
    if bad:
        raise RuntimeError(f"oracle: directed rounding idioms broken by the compiler (mask {bad})")
    _lib = L
    return L


def oracle_threads() -> int:
    return int(_load().dp_num_threads())


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(C.POINTER(C.c_float))


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(C.POINTER(C.c_double))


class OracleError(RuntimeError):
    pass


class OracleNet:
    """Same method names as the HIP binding so that one topology replay serves both."""

    LAMBDA_HEURISTIC, LAMBDA_ZERO, LAMBDA_ONE = 0, 1, 2
    CAND_ALL, CAND_INPUT_ONLY = 0, 1

    def __init__(self, c: int, h: int = 1, w: int = 1):
        self._L = _load()
        self._h = self._L.dp_create(c, h, w)
        if not self._h:
            raise OracleError("dp_create failed")

    def __del__(self):
        if getattr(self, "_h", None):
            self._L.dp_destroy(self._h)
            self._h = None

    def _chk(self, rc, what):
        if rc != 0:
            raise OracleError(f"{what}: status {rc}")

    # -- topology ---------------------------------------------------------------------------
    def add_dense(self, src, W, b=None) -> int:
        W, pW = _f32(W)
        if b is not None:
            b, pb = _f32(b)
        else:
            pb = None
        lid = self._L.dp_add_dense(self._h, src, W.shape[0], pW, pb)
        if lid < 0:
            raise OracleError("add_dense")
        return lid

    def add_conv2d(self, src, W, b=None, stride=1, pad=0) -> int:
        W, pW = _f32(W)
        if b is not None:
            b, pb = _f32(b)
        else:
            pb = None
        sh, sw = (stride, stride) if np.isscalar(stride) else stride
        ph, pw = (pad, pad) if np.isscalar(pad) else pad
        lid = self._L.dp_add_conv2d(self._h, src, W.shape[0], W.shape[2], W.shape[3], sh, sw, ph, pw, pW, pb)
        if lid < 0:
            raise OracleError("add_conv2d")
        return lid

    def add_avgpool2d(self, src, kernel, stride=None, pad=0) -> int:
        kh, kw = (kernel, kernel) if np.isscalar(kernel) else kernel
        if stride is None:
            stride = (kh, kw)
        sh, sw = (stride, stride) if np.isscalar(stride) else stride
        ph, pw = (pad, pad) if np.isscalar(pad) else pad
        lid = self._L.dp_add_avgpool2d(self._h, src, kh, kw, sh, sw, ph, pw)
        if lid < 0:
            raise OracleError("add_avgpool2d")
        return lid

    def add_relu(self, src) -> int:
        lid = self._L.dp_add_relu(self._h, src)
        if lid < 0:
            raise OracleError("add_relu")
        return lid

    def add_residual(self, a, b) -> int:
        lid = self._L.dp_add_residual(self._h, a, b)
        if lid < 0:
            raise OracleError("add_residual")
        return lid

    @property
    def num_layers(self) -> int:
        return self._L.dp_num_layers(self._h)

    def layer_size(self, lid) -> int:
        return self._L.dp_layer_size(self._h, lid)

    def set_options(self, lambda_policy=0, candidates=0):
        self._chk(self._L.dp_set_options(self._h, lambda_policy, candidates), "set_options")

    def set_collapse(self, on: bool):
        """False: keep interval coefficients for the whole back-substitution (the literal scheme of Section 4.1)."""
        self._chk(self._L.dp_set_collapse(self._h, 1 if on else 0), "set_collapse")

    def set_early_termination(self, on: bool):
        """Forward interval pass + termination criterion (Sections 3.2 and 4.2)."""
        self._chk(self._L.dp_set_early_termination(self._h, 1 if on else 0), "set_early_termination")

    def set_float_inference(self, on: bool):
        """Bounds that also hold for every float32 evaluation order of the network (Section 4.1, last paragraph)."""
        self._chk(self._L.dp_set_float_inference(self._h, 1 if on else 0), "set_float_inference")

    def get_inference_error(self, lid) -> np.ndarray:
        """Per neuron of an affine or sum layer: the bound on |float32 evaluation - exact value| the last analysis used."""
        eta = np.empty(self.layer_size(lid), np.float64)
        self._chk(self._L.dp_get_inference_error(self._h, lid, eta.ctypes.data_as(C.POINTER(C.c_double))),
                  "get_inference_error")
        return eta

    def set_term_override(self, lid, term: Optional[np.ndarray]):
        """Per neuron of layer lid: where its back-substitution stops (-1: the criterion decides)."""
        if term is None:
            self._chk(self._L.dp_set_term_override(self._h, lid, None), "set_term_override")
            return
        t = np.ascontiguousarray(term, dtype=np.int32)
        assert t.size == self.layer_size(lid)
        self._chk(self._L.dp_set_term_override(self._h, lid, t.ctypes.data_as(C.POINTER(C.c_int))),
                  "set_term_override")

    def get_term_layer(self, lid) -> np.ndarray:
        t = np.empty(self.layer_size(lid), np.int32)
        self._chk(self._L.dp_get_term_layer(self._h, lid, t.ctypes.data_as(C.POINTER(C.c_int))), "get_term_layer")
        return t

    def get_interval_image(self, lid) -> Tuple[np.ndarray, np.ndarray]:
        n = self.layer_size(lid)
        lo = np.empty(n, np.float64)
        hi = np.empty(n, np.float64)
        self._chk(self._L.dp_get_interval_image(self._h, lid, lo.ctypes.data_as(C.POINTER(C.c_double)),
                                                hi.ctypes.data_as(C.POINTER(C.c_double))), "get_interval_image")
        return lo, hi

    def request_bounds(self, lid):
        self._chk(self._L.dp_request_bounds(self._h, lid), "request_bounds")

    def set_lambda_override(self, lid, force: Optional[np.ndarray]):
        if force is None:
            self._chk(self._L.dp_set_lambda_override(self._h, lid, None), "set_lambda_override")
            return
        f = np.ascontiguousarray(force, dtype=np.int8)
        assert f.size == self.layer_size(lid)
        self._chk(self._L.dp_set_lambda_override(self._h, lid, f.ctypes.data_as(C.POINTER(C.c_byte))),
                  "set_lambda_override")

    def set_gamma_override(self, lid, gam: Optional[np.ndarray]):
        if gam is None:
            self._chk(self._L.dp_set_gamma_override(self._h, lid, None), "set_gamma_override")
            return
        g, pg = _f64(gam)
        assert g.size == self.layer_size(lid)
        self._chk(self._L.dp_set_gamma_override(self._h, lid, pg), "set_gamma_override")

    # -- analysis ---------------------------------------------------------------------------
    def set_box(self, lo, hi):
        lo, plo = _f64(lo)
        hi, phi = _f64(hi)
        assert lo.size == hi.size == self.layer_size(0)
        self._chk(self._L.dp_set_box(self._h, plo, phi), "set_box")

    def set_ball(self, center, eps, clip_lo=0.0, clip_hi=1.0):
        c, pc = _f32(center)
        assert c.size == self.layer_size(0)
        self._chk(self._L.dp_set_ball(self._h, pc, eps, clip_lo, clip_hi), "set_ball")

    def analyze(self, center=None, eps=None, clip_lo=0.0, clip_hi=1.0):
        if center is not None:
            self.set_ball(center, eps, clip_lo, clip_hi)
        self._chk(self._L.dp_analyze(self._h), "analyze")

    def analyze_box(self, lo, hi):
        self.set_box(lo, hi)
        self._chk(self._L.dp_analyze(self._h), "analyze")

    def analyze_layer(self, lid):
        self._chk(self._L.dp_analyze_layer(self._h, lid), "analyze_layer")

    def set_bounds(self, lid, lo, hi):
        lo, plo = _f64(lo)
        hi, phi = _f64(hi)
        assert lo.size == hi.size == self.layer_size(lid)
        self._chk(self._L.dp_set_bounds(self._h, lid, plo, phi), "set_bounds")

    def get_bounds(self, lid) -> Tuple[np.ndarray, np.ndarray]:
        n = self.layer_size(lid)
        lo = np.empty(n, np.float64)
        hi = np.empty(n, np.float64)
        self._chk(self._L.dp_get_bounds(self._h, lid, lo.ctypes.data_as(C.POINTER(C.c_double)),
                                        hi.ctypes.data_as(C.POINTER(C.c_double))), "get_bounds")
        return lo, hi

    def get_relaxation(self, lid):
        n = self.layer_size(lid)
        g = np.empty(n, np.float64)
        d = np.empty(n, np.float64)
        lam = np.empty(n, np.int8)
        self._chk(self._L.dp_get_relaxation(self._h, lid, g.ctypes.data_as(C.POINTER(C.c_double)),
                                            d.ctypes.data_as(C.POINTER(C.c_double)),
                                            lam.ctypes.data_as(C.POINTER(C.c_byte))), "get_relaxation")
        return g, d, lam

    def bound_rows(self, lid, rows) -> Tuple[np.ndarray, np.ndarray]:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        lo = np.empty(rows.size, np.float64)
        hi = np.empty(rows.size, np.float64)
        self._chk(self._L.dp_bound_rows(self._h, lid, rows.ctypes.data_as(C.POINTER(C.c_int)), rows.size,
                                        lo.ctypes.data_as(C.POINTER(C.c_double)),
                                        hi.ctypes.data_as(C.POINTER(C.c_double))), "bound_rows")
        return lo, hi

    def certify(self, label) -> Tuple[bool, np.ndarray]:
        n = self.layer_size(self.num_layers - 1)
        m = np.empty(n - 1, np.float64)
        v = C.c_int(0)
        self._chk(self._L.dp_certify(self._h, int(label), C.byref(v), m.ctypes.data_as(C.POINTER(C.c_double))),
                  "certify")
        return bool(v.value), m

    def bound_outputs(self, coef, offset=None) -> np.ndarray:
        """Lower bounds of the linear forms coef @ y + offset of the last layer (rows of coef)."""
        n = self.layer_size(self.num_layers - 1)
        cf, pc = _f64(np.atleast_2d(coef))
        assert cf.shape[1] == n
        if offset is not None:
            off, po = _f64(offset)
            assert off.size == cf.shape[0]
        else:
            po = None
        out = np.empty(cf.shape[0], np.float64)
        self._chk(self._L.dp_bound_forms(self._h, cf.shape[0], pc, po, out.ctypes.data_as(C.POINTER(C.c_double))),
                  "bound_forms")
        return out
