"""ctypes binding of libfastforward.so: argument marshalling only.

Every function here has the name of the C entry point it calls (without the
``ff_`` prefix) and does nothing but turn torch tensors into device pointers.
Torch is used for device memory and streams; all arithmetic of the path runs in
the library's HIP kernels.  If the library is missing this module raises: there
is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libfastforward.so")

ACT = {"silu": 0, "relu": 1, "identity": 2}
OUT_BF16, OUT_F32 = 0, 1


class Shape(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("d_ffn", C.c_int32), ("n_tokens", C.c_int32),
                ("block", C.c_int32), ("r_pred", C.c_int32), ("r_comp", C.c_int32)]


class Predictor(C.Structure):
    _fields_ = [("q_pred", C.c_void_p), ("w1", C.c_void_p), ("w2", C.c_void_p)]


class FfnWeights(C.Structure):
    _fields_ = [("w_gate", C.c_void_p), ("w_up", C.c_void_p), ("w_down", C.c_void_p)]


class Compensator(C.Structure):
    _fields_ = [("wc1", C.c_void_p), ("wc2", C.c_void_p), ("act", C.c_int32)]


class FFError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"fastforward status {status}: {what}")
        self.status = status


_lib = None


def load_library(build_if_missing: bool = True):
    """Loads the in-tree library; builds it first only if it has never been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise FileNotFoundError(LIB_PATH)
        from . import _build
        _build.build()
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    P = C.POINTER
    sig = {
        "ff_create": ([P(vp), C.c_int, vp], C.c_int),
        "ff_destroy": ([vp], C.c_int),
        "ff_set_stream": ([vp, vp], C.c_int),
        "ff_status_str": ([C.c_int], C.c_char_p),
        "ff_last_error": ([vp], C.c_char_p),
        "ff_workspace_bytes": ([P(Shape), i32, P(sz)], C.c_int),
        "ff_set_workspace": ([vp, vp, sz], C.c_int),
        "ff_set_option": ([vp, C.c_char_p, i32], C.c_int),
        "ff_k_from_sparsity": ([i32, C.c_double, P(i32)], C.c_int),
        "ff_layer_budgets": ([P(C.c_double), i32, C.c_double, P(C.c_double)], C.c_int),
        "ff_predict": ([vp, P(Shape), vp, P(Predictor), P(i32), i32, vp, vp], C.c_int),
        "ff_predict_static": ([vp, P(Shape), vp, P(Predictor), P(i32), i32, vp, vp], C.c_int),
        "ff_sparse_ffn": ([vp, P(Shape), vp, P(FfnWeights), P(Compensator), vp, P(i32), i32, vp, i32], C.c_int),
        "ff_dense_ffn": ([vp, P(Shape), vp, P(FfnWeights), vp, i32], C.c_int),
        "ff_ffn_stack": ([vp, P(Shape), i32, vp, P(Predictor), P(FfnWeights), P(Compensator), P(i32), i32,
                          C.c_float, vp, vp], C.c_int),
        "ff_profile_enable": ([vp, i32, C.c_uint32], C.c_int),
        "ff_profile_read": ([vp, P(C.c_double), P(i32)], C.c_int),
        "ff_rmsnorm": ([vp, i32, i32, vp, C.c_float, vp], C.c_int),
        "ff_residual_add": ([vp, i32, i32, vp, vp], C.c_int),
        "ff_copy": ([vp, vp, vp, sz], C.c_int),
        "ff_mfma_peak": ([vp, i32, i32, P(C.c_double)], C.c_int),
    }
    for name, (argt, rest) in sig.items():
        fn = getattr(lib, name)
        fn.argtypes, fn.restype = argt, rest
    _lib = lib
    return lib


EXPORTS = ["ff_create", "ff_destroy", "ff_set_stream", "ff_status_str", "ff_last_error", "ff_workspace_bytes",
           "ff_set_workspace", "ff_set_option", "ff_k_from_sparsity", "ff_layer_budgets", "ff_predict", "ff_predict_static",
           "ff_sparse_ffn", "ff_dense_ffn", "ff_ffn_stack", "ff_rmsnorm", "ff_residual_add",
           "ff_profile_enable", "ff_profile_read", "ff_copy", "ff_mfma_peak"]

STAGES = ("pool", "mlp", "topk", "gemm1", "gemm2", "glue")


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA tensors"
    return C.c_void_p(t.data_ptr())


def _i32_array(values: Sequence[int]):
    a = np.ascontiguousarray(np.asarray(values, dtype=np.int32))
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


def k_from_sparsity(d_ffn: int, sparsity: float) -> int:
    out = C.c_int32()
    st = load_library().ff_k_from_sparsity(d_ffn, float(sparsity), C.byref(out))
    if st:
        raise FFError(st, "ff_k_from_sparsity")
    return out.value


def layer_budgets(importance: Sequence[float], budget: float) -> np.ndarray:
    imp = np.ascontiguousarray(np.asarray(importance, dtype=np.float64))
    out = np.empty_like(imp)
    dp = C.POINTER(C.c_double)
    st = load_library().ff_layer_budgets(imp.ctypes.data_as(dp), len(imp), float(budget), out.ctypes.data_as(dp))
    if st:
        raise FFError(st, "ff_layer_budgets")
    return out


def workspace_bytes(shape: Shape, k_max: int) -> int:
    out = C.c_size_t()
    st = load_library().ff_workspace_bytes(C.byref(shape), int(k_max), C.byref(out))
    if st:
        raise FFError(st, "ff_workspace_bytes")
    return out.value


class Context:
    """One ff_ctx bound to a torch device and stream; owns its workspace tensor."""

    def __init__(self, device: int = 0, stream: Optional[torch.cuda.Stream] = None):
        self.lib = load_library()
        self.device = device
        self._h = C.c_void_p()
        s = stream.cuda_stream if stream is not None else torch.cuda.current_stream(device).cuda_stream
        st = self.lib.ff_create(C.byref(self._h), device, C.c_void_p(s))
        if st:
            raise FFError(st, "ff_create: " + self.lib.ff_status_str(st).decode())
        self._ws = None

    def close(self):
        if self._h:
            self.lib.ff_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st:
            raise FFError(st, self.lib.ff_last_error(self._h).decode())

    def set_stream(self, stream: torch.cuda.Stream):
        self._check(self.lib.ff_set_stream(self._h, C.c_void_p(stream.cuda_stream)))

    def set_option(self, name: str, value: int):
        self._check(self.lib.ff_set_option(self._h, name.encode(), int(value)))

    def ensure_workspace(self, shape: Shape, k_max: int):
        need = workspace_bytes(shape, k_max)
        if self._ws is None or self._ws.numel() < need:
            self._ws = None
            self._ws = torch.empty(need, dtype=torch.uint8, device=f"cuda:{self.device}")
            self._check(self.lib.ff_set_workspace(self._h, _ptr(self._ws), self._ws.numel()))

    def set_workspace(self, ws: Optional[torch.Tensor]):
        self._ws = ws
        self._check(self.lib.ff_set_workspace(self._h, _ptr(ws), 0 if ws is None else ws.numel()))

    def profile_enable(self, max_records: int, stages: Sequence[str] = STAGES):
        mask = 0
        for n in stages:
            mask |= 1 << STAGES.index(n)
        self._check(self.lib.ff_profile_enable(self._h, int(max_records), mask))

    def profile_read(self):
        """-> {stage: (total ms, launches)} since the last read; synchronises the stream."""
        ms = (C.c_double * len(STAGES))()
        cnt = (C.c_int32 * len(STAGES))()
        self._check(self.lib.ff_profile_read(self._h, ms, cnt))
        return {n: (ms[i], cnt[i]) for i, n in enumerate(STAGES)}

    # ---- compute calls (same names as the C entry points) -----------------
    def predict(self, shape: Shape, x, pred: Predictor, k_per_block, k_stride: int, indices, scores=None):
        _, kp = _i32_array(k_per_block)
        self._check(self.lib.ff_predict(self._h, C.byref(shape), _ptr(x), C.byref(pred), kp, k_stride,
                                        _ptr(indices), _ptr(scores)))

    def predict_static(self, shape: Shape, x, pred: Predictor, k_per_block, k_stride: int, indices, scores=None):
        _, kp = _i32_array(k_per_block)
        self._check(self.lib.ff_predict_static(self._h, C.byref(shape), _ptr(x), C.byref(pred), kp, k_stride,
                                               _ptr(indices), _ptr(scores)))

    def sparse_ffn(self, shape: Shape, x, w: FfnWeights, comp: Optional[Compensator], indices, k_per_block,
                   k_stride: int, y, out_dtype: int = OUT_BF16):
        _, kp = _i32_array(k_per_block)
        self._check(self.lib.ff_sparse_ffn(self._h, C.byref(shape), _ptr(x), C.byref(w),
                                           C.byref(comp) if comp is not None else None, _ptr(indices), kp,
                                           k_stride, _ptr(y), out_dtype))

    def dense_ffn(self, shape: Shape, x, w: FfnWeights, y, out_dtype: int = OUT_BF16):
        self._check(self.lib.ff_dense_ffn(self._h, C.byref(shape), _ptr(x), C.byref(w), _ptr(y), out_dtype))

    def ffn_stack(self, shape: Shape, h, preds, weights, comps, k_per_layer_block, k_stride: int, rms_eps: float,
                  indices=None, x_dump=None):
        n_layers = len(weights)
        pa = (Predictor * n_layers)(*preds)
        wa = (FfnWeights * n_layers)(*weights)
        ca = (Compensator * n_layers)(*comps) if comps is not None else None
        _, kp = _i32_array(np.asarray(k_per_layer_block).reshape(-1))
        self._check(self.lib.ff_ffn_stack(self._h, C.byref(shape), n_layers, _ptr(h), pa, wa, ca, kp, k_stride,
                                          float(rms_eps), _ptr(indices), _ptr(x_dump)))

    def rmsnorm(self, h, eps: float, x):
        self._check(self.lib.ff_rmsnorm(self._h, h.shape[0], h.shape[1], _ptr(h), float(eps), _ptr(x)))

    def copy(self, dst, src):
        n = src.numel() * src.element_size()
        assert dst.numel() * dst.element_size() >= n
        self._check(self.lib.ff_copy(self._h, _ptr(dst), _ptr(src), n))

    def mfma_peak(self, iters: int, zero_operands: bool = False) -> float:
        """Enqueues the matrix-pipe calibration loop; returns the FLOPs one launch performs."""
        fl = C.c_double()
        self._check(self.lib.ff_mfma_peak(self._h, int(iters), int(bool(zero_operands)), C.byref(fl)))
        return fl.value

    def residual_add(self, h, y):
        self._check(self.lib.ff_residual_add(self._h, h.shape[0], h.shape[1], _ptr(h), _ptr(y)))


# ---- helpers to move generator output onto the device ----------------------

def to_device_bf16(bits: np.ndarray, device: str = "cuda:0") -> torch.Tensor:
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on the GPU (no value change)."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def make_structs(layer, device: str = "cuda:0"):
    """Uploads one LayerTensors; returns (dict of device tensors, Predictor, FfnWeights, Compensator)."""
    d = {n: to_device_bf16(getattr(layer, n), device)
         for n in ("w_gate", "w_up", "w_down", "w1", "w2", "wc1", "wc2")}
    q = to_device_bf16(layer.q_pred, device) if layer.q_pred is not None else None
    d["q_pred"] = q
    pred = Predictor(q.data_ptr() if q is not None else None, d["w1"].data_ptr(), d["w2"].data_ptr())
    w = FfnWeights(d["w_gate"].data_ptr(), d["w_up"].data_ptr(), d["w_down"].data_ptr())
    comp = Compensator(d["wc1"].data_ptr(), d["wc2"].data_ptr(), ACT["silu"])
    return d, pred, w, comp
