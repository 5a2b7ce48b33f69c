"""Python binding of libgpupoly_hip.so: argument marshalling only; every step of the analysis runs
in the library's HIP kernels.  Raises if the library is missing: there is no CPU fallback."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libgpupoly_hip.so")
_lib = None

STATUS = {0: "GP_OK", 1: "GP_ERR_ARG", 2: "GP_ERR_SHAPE", 3: "GP_ERR_STATE", 4: "GP_ERR_NOMEM", 5: "GP_ERR_DEVICE",
          6: "GP_ERR_NONFINITE", 7: "GP_ERR_WORKSPACE", 8: "GP_ERR_UNSUPPORTED"}

# every symbol include/gpupoly.h declares
EXPORTS = ["gp_net_create", "gp_net_destroy", "gp_add_dense", "gp_add_conv2d", "gp_add_avgpool2d", "gp_add_relu", "gp_add_residual",
           "gp_request_bounds", "gp_set_early_termination", "gp_set_float_inference", "gp_set_coefficient_storage", "gp_set_chain_fusion", "gp_set_interval_coefficients", "gp_set_graph_replay", "gp_get_term_layer", "gp_get_early_termination_stats",
           "gp_set_stream", "gp_workspace_size", "gp_set_workspace", "gp_analyze",
           "gp_analyze_box", "gp_analyze_batch", "gp_analyze_batch_dev", "gp_analyze_batch_dev_static", "gp_get_bounds", "gp_get_bounds_batch",
           "gp_get_bounds_f64", "gp_get_relu_lambda", "gp_get_relu_slopes", "gp_certify", "gp_certify_batch", "gp_bound_outputs", "gp_debug_plan", "gp_debug_set_accumulation_roundoff",
           "gp_profile_enable", "gp_profile_read", "gp_profile_dump", "gp_debug_mfma_f64", "gp_debug_mfma_f64_4col", "gp_num_layers", "gp_layer_size", "gp_last_error", "gp_version"]


class GpuPolyError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{STATUS.get(status, status)}: {msg}")
        self.status = status


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2007_10868_amd.build` "
                          "(there is no CPU fallback)")
    L = C.CDLL(_LIB_PATH)
    P, i32, f32 = C.c_void_p, C.c_int32, C.c_float
    fp, dp, ip = C.POINTER(C.c_float), C.POINTER(C.c_double), C.POINTER(C.c_int32)
    L.gp_net_create.argtypes = [i32, i32, i32, C.POINTER(P)]
    L.gp_net_destroy.argtypes = [P]
    L.gp_net_destroy.restype = None
    L.gp_add_dense.argtypes = [P, i32, i32, fp, fp, ip]
    L.gp_add_conv2d.argtypes = [P] + [i32] * 8 + [fp, fp, ip]
    L.gp_add_avgpool2d.argtypes = [P] + [i32] * 7 + [ip]
    L.gp_add_relu.argtypes = [P, i32, ip]
    L.gp_add_residual.argtypes = [P, i32, i32, ip]
    L.gp_request_bounds.argtypes = [P, i32]
    L.gp_set_stream.argtypes = [P, P]
    L.gp_set_early_termination.argtypes = [P, i32]
    L.gp_set_float_inference.argtypes = [P, i32]
    L.gp_set_coefficient_storage.argtypes = [P, i32]
    L.gp_set_chain_fusion.argtypes = [P, i32]
    L.gp_debug_set_accumulation_roundoff.argtypes = [P, C.c_double]
    L.gp_set_interval_coefficients.argtypes = [P, i32]
    L.gp_set_graph_replay.argtypes = [P, i32]
    L.gp_get_term_layer.argtypes = [P, i32, i32, ip]
    L.gp_get_early_termination_stats.argtypes = [P, dp, dp]
    L.gp_workspace_size.argtypes = [P, i32, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    L.gp_set_workspace.argtypes = [P, P, C.c_int64]
    L.gp_analyze.argtypes = [P, fp, f32, f32, f32]
    L.gp_analyze_box.argtypes = [P, fp, fp]
    L.gp_analyze_batch.argtypes = [P, i32, fp, f32, f32, f32]
    L.gp_analyze_batch_dev.argtypes = [P, i32, P, f32, f32, f32]
    L.gp_analyze_batch_dev_static.argtypes = [P, i32, P, f32, f32, f32, P, P]
    L.gp_get_bounds.argtypes = [P, i32, fp, fp]
    L.gp_get_bounds_batch.argtypes = [P, i32, i32, fp, fp]
    L.gp_get_bounds_f64.argtypes = [P, i32, i32, dp, dp]
    L.gp_get_relu_lambda.argtypes = [P, i32, i32, C.POINTER(C.c_int8)]
    L.gp_get_relu_slopes.argtypes = [P, i32, i32, fp]
    L.gp_certify.argtypes = [P, i32, ip, fp]
    L.gp_certify_batch.argtypes = [P, ip, ip, fp]
    L.gp_bound_outputs.argtypes = [P, i32, fp, fp, fp]
    L.gp_debug_plan.argtypes = [P, i32, ip, i32, ip]
    L.gp_num_layers.argtypes = [P]
    L.gp_layer_size.argtypes = [P, i32]
    L.gp_last_error.argtypes = [P]
    L.gp_last_error.restype = C.c_char_p
    L.gp_version.restype = C.c_char_p
    L.gp_profile_enable.argtypes = [P, i32]
    L.gp_profile_read.argtypes = [P, C.POINTER(C.c_int64), dp, dp, dp]
    L.gp_profile_dump.argtypes = [P, C.c_char_p]
    L.gp_debug_mfma_f64.argtypes = [P, P, P, i32, P]
    L.gp_debug_mfma_f64_4col.argtypes = [P, P, P, i32, P]
    _lib = L
    return L


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(C.POINTER(C.c_float))


class Net:
    """One network + its device state.  Method names mirror the C ABI (gp_ prefix dropped)."""

    def __init__(self, c: int, h: int = 1, w: int = 1):
        self._L = load_library()
        self._h = C.c_void_p()
        st = self._L.gp_net_create(c, h, w, C.byref(self._h))
        if st != 0:
            raise GpuPolyError(st, "gp_net_create")
        self._ws = None

    def __del__(self):
        if getattr(self, "_h", None):
            self._L.gp_net_destroy(self._h)
            self._h = None

    def _chk(self, st):
        if st != 0:
            raise GpuPolyError(st, self._L.gp_last_error(self._h).decode())

    # ---- topology
    def add_dense(self, src, W, b=None) -> int:
        W, pW = _f32(W)
        pb = None
        if b is not None:
            b, pb = _f32(b)
        lid = C.c_int32(-1)
        self._chk(self._L.gp_add_dense(self._h, src, W.shape[0], pW, pb, C.byref(lid)))
        return lid.value

    def add_conv2d(self, src, W, b=None, stride=1, pad=0) -> int:
        W, pW = _f32(W)
        pb = None
        if b is not None:
            b, pb = _f32(b)
        sh, sw = (stride, stride) if np.isscalar(stride) else stride
        ph, pw = (pad, pad) if np.isscalar(pad) else pad
        lid = C.c_int32(-1)
        self._chk(self._L.gp_add_conv2d(self._h, src, W.shape[0], W.shape[2], W.shape[3], sh, sw, ph, pw, pW, pb,
                                        C.byref(lid)))
        return lid.value

    def add_avgpool2d(self, src, kernel, stride=None, pad=0) -> int:
        kh, kw = (kernel, kernel) if np.isscalar(kernel) else kernel
        if stride is None:
            stride = (kh, kw)
        sh, sw = (stride, stride) if np.isscalar(stride) else stride
        ph, pw = (pad, pad) if np.isscalar(pad) else pad
        lid = C.c_int32(-1)
        self._chk(self._L.gp_add_avgpool2d(self._h, src, kh, kw, sh, sw, ph, pw, C.byref(lid)))
        return lid.value

    def add_relu(self, src) -> int:
        lid = C.c_int32(-1)
        self._chk(self._L.gp_add_relu(self._h, src, C.byref(lid)))
        return lid.value

    def add_residual(self, a, b) -> int:
        lid = C.c_int32(-1)
        self._chk(self._L.gp_add_residual(self._h, a, b, C.byref(lid)))
        return lid.value

    def request_bounds(self, lid):
        self._chk(self._L.gp_request_bounds(self._h, lid))

    @property
    def num_layers(self) -> int:
        return self._L.gp_num_layers(self._h)

    def layer_size(self, lid) -> int:
        return self._L.gp_layer_size(self._h, lid)

    # ---- device plumbing (torch is used for memory and streams only)
    def set_float_inference(self, on=True):
        """Bounds that also hold for every float32 evaluation order of the network (Section 4.1, inference rounding)."""
        self._chk(self._L.gp_set_float_inference(self._h, 1 if on else 0))

    def set_coefficient_storage(self, bits=32):
        """32 (default): coefficients stored in float32; 64: in float64 (the paper's double precision build, Section 5)."""
        self._chk(self._L.gp_set_coefficient_storage(self._h, bits))

    def set_interval_coefficients(self, on=True):
        """The literal scheme of Section 4.1: interval coefficients with directed rounding, kept to the end."""
        self._chk(self._L.gp_set_interval_coefficients(self._h, 1 if on else 0))

    def debug_set_accumulation_roundoff(self, unit: float):
        """Price the accumulation-error term of every crossing at this unit roundoff (default 2^-50); a study hook."""
        self._chk(self._L.gp_debug_set_accumulation_roundoff(self._h, float(unit)))

    def set_chain_fusion(self, on=True):
        """Chains of narrow dense layers in one fused launch per start layer (default) or through the general kernels."""
        self._chk(self._L.gp_set_chain_fusion(self._h, 1 if on else 0))

    def set_graph_replay(self, on=True):
        """Capture the launches of an analysis into a HIP graph once and replay it on later calls."""
        self._chk(self._L.gp_set_graph_replay(self._h, 1 if on else 0))

    def set_early_termination(self, on=True):
        self._chk(self._L.gp_set_early_termination(self._h, 1 if on else 0))

    def get_term_layer(self, lid, batch_index=0):
        t = np.empty(self.layer_size(lid), np.int32)
        self._chk(self._L.gp_get_term_layer(self._h, lid, batch_index, t.ctypes.data_as(C.POINTER(C.c_int32))))
        return t

    def early_termination_stats(self):
        """(flop carried out by the crossings, flop of the same analysis with no row removed)"""
        a, b = C.c_double(0), C.c_double(0)
        self._chk(self._L.gp_get_early_termination_stats(self._h, C.byref(a), C.byref(b)))
        return a.value, b.value

    def set_stream(self, stream=None):
        """stream: a torch.cuda.Stream (or None for the default stream)."""
        self._chk(self._L.gp_set_stream(self._h, C.c_void_p(stream.cuda_stream if stream is not None else 0)))

    def workspace_size(self, batch=1) -> Tuple[int, int]:
        mn, full = C.c_int64(0), C.c_int64(0)
        self._chk(self._L.gp_workspace_size(self._h, batch, C.byref(mn), C.byref(full)))
        return mn.value, full.value

    def set_workspace(self, tensor):
        """tensor: a torch uint8 CUDA tensor the caller keeps alive (None: library-owned workspace)."""
        if tensor is None:
            self._chk(self._L.gp_set_workspace(self._h, None, 0))
            self._ws = None
            return
        self._ws = tensor
        self._chk(self._L.gp_set_workspace(self._h, C.c_void_p(tensor.data_ptr()), tensor.numel() * tensor.element_size()))

    # ---- analysis
    def analyze(self, center, eps, clip_lo=0.0, clip_hi=1.0):
        c, pc = _f32(center)
        assert c.size == self.layer_size(0)
        self._chk(self._L.gp_analyze(self._h, pc, eps, clip_lo, clip_hi))

    def analyze_box(self, lo, hi):
        lo, plo = _f32(lo)
        hi, phi = _f32(hi)
        assert lo.size == hi.size == self.layer_size(0)
        self._chk(self._L.gp_analyze_box(self._h, plo, phi))

    def analyze_batch(self, centers, eps, clip_lo=0.0, clip_hi=1.0):
        c, pc = _f32(centers)
        assert c.ndim == 2 and c.shape[1] == self.layer_size(0)
        self._chk(self._L.gp_analyze_batch(self._h, c.shape[0], pc, eps, clip_lo, clip_hi))

    def analyze_batch_dev(self, centers_tensor, eps, clip_lo=0.0, clip_hi=1.0):
        """centers_tensor: contiguous float32 CUDA tensor [batch, n_in]."""
        t = centers_tensor
        assert t.is_cuda and t.is_contiguous() and t.dim() == 2 and t.shape[1] == self.layer_size(0)
        self._chk(self._L.gp_analyze_batch_dev(self._h, t.shape[0], C.c_void_p(t.data_ptr()), eps, clip_lo, clip_hi))

    def analyze_batch_dev_static(self, centers_tensor, eps, lower_tensor, upper_tensor, clip_lo=0.0, clip_hi=1.0):
        """The allocation-free variant: centers [batch, n_in] float32, lower/upper [batch, n_out] float64, all
        contiguous CUDA tensors of the caller."""
        t = centers_tensor
        assert t.is_cuda and t.is_contiguous() and t.dim() == 2 and t.shape[1] == self.layer_size(0)
        n_out = self.layer_size(self.num_layers - 1)
        for o in (lower_tensor, upper_tensor):
            assert o.is_cuda and o.is_contiguous() and o.dtype.itemsize == 8 and o.numel() == t.shape[0] * n_out
        self._chk(self._L.gp_analyze_batch_dev_static(self._h, t.shape[0], C.c_void_p(t.data_ptr()), eps, clip_lo, clip_hi,
                                                      C.c_void_p(lower_tensor.data_ptr()), C.c_void_p(upper_tensor.data_ptr())))

    def get_bounds(self, lid, batch_index=0):
        n = self.layer_size(lid)
        lo = np.empty(n, np.float32)
        hi = np.empty(n, np.float32)
        self._chk(self._L.gp_get_bounds_batch(self._h, lid, batch_index, lo.ctypes.data_as(C.POINTER(C.c_float)),
                                              hi.ctypes.data_as(C.POINTER(C.c_float))))
        return lo, hi

    def get_bounds_f64(self, lid, batch_index=0):
        n = self.layer_size(lid)
        lo = np.empty(n, np.float64)
        hi = np.empty(n, np.float64)
        self._chk(self._L.gp_get_bounds_f64(self._h, lid, batch_index, lo.ctypes.data_as(C.POINTER(C.c_double)),
                                            hi.ctypes.data_as(C.POINTER(C.c_double))))
        return lo, hi

    def get_relu_lambda(self, lid, batch_index=0):
        n = self.layer_size(lid)
        lam = np.empty(n, np.int8)
        self._chk(self._L.gp_get_relu_lambda(self._h, lid, batch_index, lam.ctypes.data_as(C.POINTER(C.c_int8))))
        return lam

    def get_relu_slopes(self, lid, batch_index=0):
        n = self.layer_size(lid)
        g = np.empty(n, np.float32)
        self._chk(self._L.gp_get_relu_slopes(self._h, lid, batch_index, g.ctypes.data_as(C.POINTER(C.c_float))))
        return g

    def certify(self, label):
        n = self.layer_size(self.num_layers - 1)
        m = np.empty(n - 1, np.float32)
        v = C.c_int32(0)
        self._chk(self._L.gp_certify(self._h, int(label), C.byref(v), m.ctypes.data_as(C.POINTER(C.c_float))))
        return bool(v.value), m

    def certify_batch(self, labels):
        labels = np.ascontiguousarray(labels, dtype=np.int32)
        n = self.layer_size(self.num_layers - 1)
        m = np.empty((labels.size, n - 1), np.float32)
        v = np.zeros(labels.size, np.int32)
        self._chk(self._L.gp_certify_batch(self._h, labels.ctypes.data_as(C.POINTER(C.c_int32)),
                                           v.ctypes.data_as(C.POINTER(C.c_int32)),
                                           m.ctypes.data_as(C.POINTER(C.c_float))))
        return v.astype(bool), m

    def bound_outputs(self, coef, offset=None, batch=1):
        """Lower bounds of coef @ y + offset over each analysed box; returns [batch, n_forms] float32."""
        cf = np.ascontiguousarray(np.atleast_2d(coef), dtype=np.float32)
        assert cf.shape[1] == self.layer_size(self.num_layers - 1)
        po = None
        if offset is not None:
            off = np.ascontiguousarray(offset, dtype=np.float32)
            assert off.size == cf.shape[0]
            po = off.ctypes.data_as(C.POINTER(C.c_float))
        out = np.empty((batch, cf.shape[0]), np.float32)
        self._chk(self._L.gp_bound_outputs(self._h, cf.shape[0], cf.ctypes.data_as(C.POINTER(C.c_float)), po,
                                           out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    def profile_enable(self, on=True):
        self._chk(self._L.gp_profile_enable(self._h, 1 if on else 0))

    def profile_dump(self, path):
        self._chk(self._L.gp_profile_dump(self._h, str(path).encode()))

    def profile_read(self):
        """{kernel: dict(launches, ms, flop, bytes)} for the crossing and the scan kernel; resets."""
        n = (C.c_int64 * 2)()
        ms, fl, by = (C.c_double * 2)(), (C.c_double * 2)(), (C.c_double * 2)()
        self._chk(self._L.gp_profile_read(self._h, n, ms, fl, by))
        return {k: dict(launches=int(n[i]), ms=float(ms[i]), flop=float(fl[i]), bytes=float(by[i]))
                for i, k in enumerate(("cross", "scan"))}

    def debug_plan(self, lid):
        n = C.c_int32(0)
        self._chk(self._L.gp_debug_plan(self._h, lid, None, 0, C.byref(n)))
        buf = np.zeros((n.value, 8), np.int32)
        self._chk(self._L.gp_debug_plan(self._h, lid, buf.ctypes.data_as(C.POINTER(C.c_int32)), n.value, C.byref(n)))
        keys = ["kind", "layer", "window_h", "window_w", "channels", "acc_stride_h", "acc_pad_h", "merged"]
        return [dict(zip(keys, map(int, row))) for row in buf]
