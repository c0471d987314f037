"""ctypes binding of libl4q.so.  Argument marshalling only: every step of the layer runs in
the HIP kernels.  PyTorch supplies device memory and the current stream, nothing else.

Function names and argument order follow include/l4q.h.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Tuple

from .inputs import DTYPE_BF16, DTYPE_F32, LayerSpec

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libl4q.so")

FLAG_UNFUSED_BACKWARD = 1
FLAG_ACCUMULATE_GRADS = 2
INIT_ASYMM, INIT_SYMM, INIT_L4Q, INIT_LSQPLUS = 0, 1, 2, 3

EXPORTED = ["l4q_version", "l4q_status_string", "l4q_workspace_bytes", "l4q_forward", "l4q_backward",
            "l4q_export_codes", "l4q_init_qparams", "l4q_profile_gemm", "l4q_profile_gemm_read", "l4q_mfma_probe", "l4q_quant_errors", "l4q_export_packed", "l4q_quantized_forward", "l4q_quantized_forward_workspace_bytes", "l4q_adamw_step", "l4q_cosine_lr",
            "l4q_qatlora_workspace_bytes", "l4q_qatlora_forward", "l4q_qatlora_backward", "l4q_quant_errors_static", "l4q_profile_read", "l4q_check_fast_divide"]


class L4QDesc(ctypes.Structure):
    _fields_ = [("tokens", ctypes.c_int64), ("in_features", ctypes.c_int64), ("out_features", ctypes.c_int64),
                ("rank", ctypes.c_int32), ("bits", ctypes.c_int32), ("group_size", ctypes.c_int32),
                ("alpha", ctypes.c_float), ("dtype", ctypes.c_int32), ("flags", ctypes.c_int32)]


class L4QAdamW(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float), ("step", ctypes.c_int32)]


class L4QError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libl4q.so; fail loudly when it is missing (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(LIB_PATH)
    vp, fp = ctypes.c_void_p, ctypes.c_void_p
    dp = ctypes.POINTER(L4QDesc)
    lib.l4q_version.restype = ctypes.c_int
    lib.l4q_status_string.restype = ctypes.c_char_p
    lib.l4q_status_string.argtypes = [ctypes.c_int]
    lib.l4q_workspace_bytes.restype = ctypes.c_int
    lib.l4q_workspace_bytes.argtypes = [dp, ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(ctypes.c_size_t)]
    lib.l4q_forward.restype = ctypes.c_int
    lib.l4q_forward.argtypes = [dp, vp, vp, vp, vp, fp, fp, vp, vp, ctypes.c_size_t, vp]
    lib.l4q_backward.restype = ctypes.c_int
    lib.l4q_backward.argtypes = [dp, vp, vp, vp, vp, vp, fp, fp, vp, fp, fp, fp, fp, vp, ctypes.c_size_t, vp]
    lib.l4q_qatlora_workspace_bytes.restype = ctypes.c_int
    lib.l4q_qatlora_workspace_bytes.argtypes = [dp, ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(ctypes.c_size_t)]
    lib.l4q_qatlora_forward.restype = ctypes.c_int
    lib.l4q_qatlora_forward.argtypes = [dp, vp, vp, vp, vp, fp, fp, vp, vp, ctypes.c_size_t, vp]
    lib.l4q_qatlora_backward.restype = ctypes.c_int
    lib.l4q_qatlora_backward.argtypes = [dp, vp, vp, vp, vp, vp, fp, fp, vp, fp, fp, fp, fp, vp, ctypes.c_size_t, vp]
    lib.l4q_export_codes.restype = ctypes.c_int
    lib.l4q_export_codes.argtypes = [dp, vp, vp, vp, fp, fp, vp, vp, vp, vp]
    lib.l4q_init_qparams.restype = ctypes.c_int
    lib.l4q_init_qparams.argtypes = [dp, vp, vp, vp, ctypes.c_int, fp, fp, vp]
    lib.l4q_profile_gemm.restype = ctypes.c_int
    lib.l4q_profile_gemm.argtypes = [ctypes.c_int]
    lib.l4q_profile_gemm_read.restype = ctypes.c_int
    lib.l4q_profile_gemm_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64),
                                          ctypes.POINTER(ctypes.c_double)]
    lib.l4q_profile_read.restype = ctypes.c_int
    lib.l4q_profile_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64),
                                     ctypes.POINTER(ctypes.c_double)]
    lib.l4q_check_fast_divide.restype = ctypes.c_int
    lib.l4q_check_fast_divide.argtypes = [ctypes.c_uint32, ctypes.c_uint32, vp, vp]
    lib.l4q_quant_errors.restype = ctypes.c_int
    lib.l4q_quant_errors.argtypes = [dp, vp, vp, vp, fp, fp, fp, vp, ctypes.c_size_t, vp]
    lib.l4q_quant_errors_static.restype = ctypes.c_int
    lib.l4q_quant_errors_static.argtypes = [dp, vp, vp, vp, fp, fp, fp, vp]
    lib.l4q_export_packed.restype = ctypes.c_int
    lib.l4q_export_packed.argtypes = [dp, vp, vp, vp, fp, fp, vp, vp, ctypes.c_size_t, vp]
    lib.l4q_quantized_forward.restype = ctypes.c_int
    lib.l4q_quantized_forward.argtypes = [dp, vp, vp, fp, fp, vp, vp, ctypes.c_size_t, vp]
    lib.l4q_quantized_forward_workspace_bytes.restype = ctypes.c_int
    lib.l4q_quantized_forward_workspace_bytes.argtypes = [dp, ctypes.POINTER(ctypes.c_size_t)]
    lib.l4q_adamw_step.restype = ctypes.c_int
    lib.l4q_adamw_step.argtypes = [dp, ctypes.POINTER(L4QAdamW)] + [fp] * 10 + [vp, vp, vp]
    lib.l4q_cosine_lr.restype = ctypes.c_float
    lib.l4q_cosine_lr.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_double, ctypes.c_double]
    lib.l4q_mfma_probe.restype = ctypes.c_int
    lib.l4q_mfma_probe.argtypes = [vp, ctypes.c_int, ctypes.c_int, fp, ctypes.POINTER(ctypes.c_double), vp]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().l4q_status_string(int(status)).decode()


def make_desc(spec: LayerSpec, flags: int = 0) -> L4QDesc:
    return L4QDesc(spec.tokens, spec.in_features, spec.out_features, spec.rank, spec.bits, spec.group_size,
                   float(spec.alpha), spec.dtype, flags)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _check(status: int, where: str) -> None:
    if status != 0:
        raise L4QError(status, where)


def l4q_workspace_bytes(desc: L4QDesc) -> Tuple[int, int]:
    f, b = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(load_library().l4q_workspace_bytes(ctypes.byref(desc), ctypes.byref(f), ctypes.byref(b)),
           "l4q_workspace_bytes")
    return f.value, b.value


def l4q_forward(desc: L4QDesc, X, W0, A, B, scale, zero, Y, workspace) -> None:
    _check(load_library().l4q_forward(ctypes.byref(desc), _ptr(X), _ptr(W0), _ptr(A), _ptr(B), _ptr(scale),
                                      _ptr(zero), _ptr(Y), _ptr(workspace),
                                      0 if workspace is None else workspace.numel() * workspace.element_size(),
                                      _stream()), "l4q_forward")


def l4q_backward(desc: L4QDesc, X, dY, W0, A, B, scale, zero, dX, dA, dB, dscale, dzero, workspace) -> None:
    _check(load_library().l4q_backward(ctypes.byref(desc), _ptr(X), _ptr(dY), _ptr(W0), _ptr(A), _ptr(B),
                                       _ptr(scale), _ptr(zero), _ptr(dX), _ptr(dA), _ptr(dB), _ptr(dscale),
                                       _ptr(dzero), _ptr(workspace),
                                       0 if workspace is None else workspace.numel() * workspace.element_size(),
                                       _stream()), "l4q_backward")


def l4q_qatlora_workspace_bytes(desc: L4QDesc) -> Tuple[int, int]:
    f, b = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(load_library().l4q_qatlora_workspace_bytes(ctypes.byref(desc), ctypes.byref(f), ctypes.byref(b)),
           "l4q_qatlora_workspace_bytes")
    return f.value, b.value


def l4q_qatlora_forward(desc: L4QDesc, X, W0, A, B, scale, zero, Y, workspace) -> None:
    _check(load_library().l4q_qatlora_forward(ctypes.byref(desc), _ptr(X), _ptr(W0), _ptr(A), _ptr(B), _ptr(scale),
                                              _ptr(zero), _ptr(Y), _ptr(workspace),
                                              0 if workspace is None else workspace.numel() * workspace.element_size(),
                                              _stream()), "l4q_qatlora_forward")


def l4q_qatlora_backward(desc: L4QDesc, X, dY, W0, A, B, scale, zero, dX, dA, dB, dscale, dzero, workspace) -> None:
    _check(load_library().l4q_qatlora_backward(ctypes.byref(desc), _ptr(X), _ptr(dY), _ptr(W0), _ptr(A), _ptr(B),
                                               _ptr(scale), _ptr(zero), _ptr(dX), _ptr(dA), _ptr(dB), _ptr(dscale),
                                               _ptr(dzero), _ptr(workspace),
                                               0 if workspace is None else workspace.numel() * workspace.element_size(),
                                               _stream()), "l4q_qatlora_backward")


def l4q_export_codes(desc: L4QDesc, W0, A, B, scale, zero, codes=None, wcomb=None, mask=None) -> None:
    _check(load_library().l4q_export_codes(ctypes.byref(desc), _ptr(W0), _ptr(A), _ptr(B), _ptr(scale), _ptr(zero),
                                           _ptr(codes), _ptr(wcomb), _ptr(mask), _stream()), "l4q_export_codes")


def l4q_init_qparams(desc: L4QDesc, W0, A, B, method: int, scale, zero) -> None:
    _check(load_library().l4q_init_qparams(ctypes.byref(desc), _ptr(W0), _ptr(A), _ptr(B), int(method), _ptr(scale),
                                           _ptr(zero), _stream()), "l4q_init_qparams")


def l4q_quant_errors(desc: L4QDesc, W0, A, B, scale, zero, errors, workspace) -> None:
    _check(load_library().l4q_quant_errors(ctypes.byref(desc), _ptr(W0), _ptr(A), _ptr(B), _ptr(scale), _ptr(zero),
                                           _ptr(errors), _ptr(workspace),
                                           workspace.numel() * workspace.element_size(), _stream()),
           "l4q_quant_errors")


STATIC_SCRATCH_BYTES = 8 << 20


def l4q_quant_errors_static(desc: L4QDesc, W0, A, B, scale, zero, errors) -> None:
    _check(load_library().l4q_quant_errors_static(ctypes.byref(desc), _ptr(W0), _ptr(A), _ptr(B), _ptr(scale),
                                                  _ptr(zero), _ptr(errors), _stream()), "l4q_quant_errors_static")


def l4q_export_packed(desc: L4QDesc, W0, A, B, scale, zero, packed, workspace) -> None:
    _check(load_library().l4q_export_packed(ctypes.byref(desc), _ptr(W0), _ptr(A), _ptr(B), _ptr(scale), _ptr(zero),
                                            _ptr(packed), _ptr(workspace),
                                            workspace.numel() * workspace.element_size(), _stream()),
           "l4q_export_packed")


def l4q_quantized_forward(desc: L4QDesc, X, packed, scale, zero, Y, workspace=None) -> None:
    _check(load_library().l4q_quantized_forward(ctypes.byref(desc), _ptr(X), _ptr(packed), _ptr(scale), _ptr(zero),
                                                _ptr(Y), _ptr(workspace),
                                                0 if workspace is None else workspace.numel() * workspace.element_size(),
                                                _stream()), "l4q_quantized_forward")


def l4q_quantized_forward_workspace_bytes(desc: L4QDesc) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().l4q_quantized_forward_workspace_bytes(ctypes.byref(desc), ctypes.byref(n)),
           "l4q_quantized_forward_workspace_bytes")
    return int(n.value)


def l4q_adamw_step(desc: L4QDesc, hp: L4QAdamW, A32, B32, scale, zero, dA, dB, dscale, dzero, m, v,
                   A_copy=None, B_copy=None) -> None:
    _check(load_library().l4q_adamw_step(ctypes.byref(desc), ctypes.byref(hp), _ptr(A32), _ptr(B32), _ptr(scale),
                                         _ptr(zero), _ptr(dA), _ptr(dB), _ptr(dscale), _ptr(dzero), _ptr(m), _ptr(v),
                                         _ptr(A_copy), _ptr(B_copy), _stream()), "l4q_adamw_step")


def l4q_cosine_lr(step: int, total_steps: int, lr_max: float, warmup_fraction: float = 0.1) -> float:
    return float(load_library().l4q_cosine_lr(step, total_steps, lr_max, warmup_fraction))


def l4q_profile_gemm(enable: bool) -> None:
    _check(load_library().l4q_profile_gemm(1 if enable else 0), "l4q_profile_gemm")


def l4q_profile_gemm_read() -> Tuple[float, int, float]:
    """(summed GEMM kernel milliseconds, launches, algorithmic FLOPs) since profiling was enabled."""
    ms, n, fl = ctypes.c_double(0), ctypes.c_int64(0), ctypes.c_double(0)
    _check(load_library().l4q_profile_gemm_read(ctypes.byref(ms), ctypes.byref(n), ctypes.byref(fl)),
           "l4q_profile_gemm_read")
    return ms.value, n.value, fl.value


PROFILE_GEMM, PROFILE_MERGE_FORWARD, PROFILE_MERGE_BACKWARD = 0, 1, 2


def l4q_profile_read(kind: int) -> Tuple[float, int, float]:
    """(summed kernel milliseconds, launches, algorithmic work) of one kind of launch since profiling was enabled."""
    ms, n, wk = ctypes.c_double(0), ctypes.c_int64(0), ctypes.c_double(0)
    _check(load_library().l4q_profile_read(int(kind), ctypes.byref(ms), ctypes.byref(n), ctypes.byref(wk)),
           "l4q_profile_read")
    return ms.value, n.value, wk.value


def l4q_check_fast_divide(first_significand: int, count: int, counts) -> None:
    """counts: int64 device tensor of 3 elements, zeroed by the caller."""
    _check(load_library().l4q_check_fast_divide(int(first_significand), int(count), _ptr(counts), _stream()),
           "l4q_check_fast_divide")


def l4q_mfma_probe(data, iterations: int, workgroups: int, sink) -> float:
    """Enqueue the matrix-core-only probe; returns the FLOPs of the launch."""
    fl = ctypes.c_double(0)
    _check(load_library().l4q_mfma_probe(_ptr(data), int(iterations), int(workgroups), _ptr(sink), ctypes.byref(fl),
                                         _stream()), "l4q_mfma_probe")
    return fl.value


# ---------------------------------------------------------------------------
# device-side plumbing used by tests, the smoke check and the benchmark
# ---------------------------------------------------------------------------

@dataclass
class DeviceLayer:
    """Device buffers of one layer call pair.  Only X has to live from forward to backward."""
    spec: LayerSpec
    desc: L4QDesc
    X: object
    W0: object
    A: object
    B: object
    dY: object
    scale: object
    zero: object
    Y: object
    dX: object
    dA: object
    dB: object
    dscale: object
    dzero: object
    ws: object
    fwd_bytes: int
    bwd_bytes: int

    def forward(self):
        l4q_forward(self.desc, self.X, self.W0, self.A, self.B, self.scale, self.zero, self.Y, self.ws)

    def backward(self):
        l4q_backward(self.desc, self.X, self.dY, self.W0, self.A, self.B, self.scale, self.zero, self.dX, self.dA,
                     self.dB, self.dscale, self.dzero, self.ws)


def upload(spec: LayerSpec, arrays, scale=None, zero=None, flags: int = 0, device="cuda:0") -> DeviceLayer:
    """Copy host arrays (float32 numpy, already bf16-representable in bf16 mode) to the GPU and
    allocate outputs and workspace.  scale/zero may be None: they are then left uninitialised
    for l4q_init_qparams to fill."""
    import torch
    tdt = torch.bfloat16 if spec.dtype == DTYPE_BF16 else torch.float32
    dev = torch.device(device)

    def up(a):
        return torch.from_numpy(a).to(dev).to(tdt).contiguous()

    T, i, o, r, G = spec.tokens, spec.in_features, spec.out_features, spec.rank, spec.groups
    desc = make_desc(spec, flags)
    fb, bb = l4q_workspace_bytes(desc)
    f32 = dict(dtype=torch.float32, device=dev)
    mk = lambda a: torch.empty((o, G), **f32) if a is None else torch.from_numpy(a).to(dev).float().contiguous()
    return DeviceLayer(
        spec=spec, desc=desc, X=up(arrays["X"]), W0=up(arrays["W0"]), A=up(arrays["A"]), B=up(arrays["B"]),
        dY=up(arrays["dY"]), scale=mk(scale), zero=mk(zero),
        Y=torch.empty((T, o), dtype=tdt, device=dev), dX=torch.empty((T, i), dtype=tdt, device=dev),
        dA=torch.empty((r, i), **f32), dB=torch.empty((o, r), **f32),
        dscale=torch.empty((o, G), **f32), dzero=torch.empty((o, G), **f32),
        ws=torch.empty(max(fb, bb), dtype=torch.uint8, device=dev), fwd_bytes=fb, bwd_bytes=bb)
