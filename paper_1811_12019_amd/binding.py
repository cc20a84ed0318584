"""ctypes binding of the K-FAC C ABI (include/kfac.h).  Argument marshalling only.

Every function here has the name and argument order of the C entry point it calls; tensors are
torch device tensors used purely as owned device memory (``data_ptr()``), and the stream is torch's
current HIP stream unless one is given.  Nothing is computed in Python, and there is no fallback:
if the compiled library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

from . import synth

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG_DIR, "libkfac_hip.so")

KFAC_OK = 0
KFAC_ERR_INVALID_ARG, KFAC_ERR_UNSUPPORTED, KFAC_ERR_WORKSPACE, KFAC_ERR_HIP, KFAC_ERR_TOO_LARGE = -1, -2, -3, -4, -5
KFAC_F32, KFAC_BF16, KFAC_F16 = 0, 1, 2
KFAC_NCHW, KFAC_NHWC = 0, 1
KFAC_ORDER_C_KH_KW, KFAC_ORDER_KH_KW_C = 0, 1
KFAC_OP_FACTOR_A, KFAC_OP_FACTOR_G = 0, 1

EXPORTED_SYMBOLS = (
    "kfac_status_string", "kfac_factor_workspace_bytes", "kfac_factor_A", "kfac_factor_G", "kfac_factor_batched",
    "kfac_ema", "kfac_ema_batched", "kfac_pack_upper_batched", "kfac_ema_packed_batched",
    "kfac_factor_diff_workspace_bytes", "kfac_factor_diff_batched", "kfac_factor_diff_batched_noalloc",
    "kfac_factor_diff_noalloc_max_elements",
    "kfac_weight_update_workspace_bytes", "kfac_weight_update_batched",
    "kfac_bn_sample_grads_workspace_bytes", "kfac_bn_sample_grads", "kfac_bn_diag_precondition",
    "kfac_bn_sample_grads_batched_workspace_bytes", "kfac_bn_sample_grads_batched",
    "kfac_inverse_workspace_bytes", "kfac_inverse_planes_bytes", "kfac_damped_inverse", "kfac_damped_inverse_batched",
    "kfac_pi_damping_batched", "kfac_warmup_damping_alpha", "kfac_warmup_damping_next", "kfac_bn_damping",
    "kfac_refresh_interval",
    "kfac_precondition_workspace_bytes", "kfac_precondition", "kfac_precondition_batched",
    "kfac_kernel_timing_enable", "kfac_kernel_timing_report", "kfac_probe_mfma", "kfac_probe_copy", "kfac_probe_read",
)


class kfac_layer_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "C_in", "H", "W", "C_out", "kh", "kw", "stride", "pad", "has_bias", "layout", "dtype", "order")]


class kfac_factor_item(ctypes.Structure):
    _fields_ = [("desc", kfac_layer_desc), ("x", ctypes.c_void_p), ("out", ctypes.c_void_p), ("ws", ctypes.c_void_p),
                ("ws_bytes", ctypes.c_size_t), ("scale", ctypes.c_float), ("op", ctypes.c_int32),
                ("running", ctypes.c_void_p), ("decay", ctypes.c_float), ("packed", ctypes.c_int32)]


class kfac_ema_item(ctypes.Structure):
    _fields_ = [("running", ctypes.c_void_p), ("fresh", ctypes.c_void_p), ("dim", ctypes.c_int32)]


class kfac_pack_item(ctypes.Structure):
    _fields_ = [("full", ctypes.c_void_p), ("packed", ctypes.c_void_p), ("dim", ctypes.c_int32)]


class kfac_ema_packed_item(ctypes.Structure):
    _fields_ = [("running", ctypes.c_void_p), ("packed_fresh", ctypes.c_void_p), ("dim", ctypes.c_int32)]


class kfac_diff_item(ctypes.Structure):
    _fields_ = [("x", ctypes.c_void_p), ("x_prev", ctypes.c_void_p), ("dim", ctypes.c_int32)]


class kfac_bn_item(ctypes.Structure):
    _fields_ = [("xhat", ctypes.c_void_p), ("gout", ctypes.c_void_p), ("g", ctypes.c_void_p), ("N", ctypes.c_int32),
                ("C", ctypes.c_int32), ("HW", ctypes.c_int32), ("dtype", ctypes.c_int32)]


class kfac_update_item(ctypes.Structure):
    _fields_ = [("w", ctypes.c_void_p), ("w_prev", ctypes.c_void_p), ("precond", ctypes.c_void_p),
                ("n", ctypes.c_int32), ("d_out", ctypes.c_int32)]


class kfac_inverse_item(ctypes.Structure):
    _fields_ = [("S", ctypes.c_void_p), ("Minv", ctypes.c_void_p), ("ws", ctypes.c_void_p), ("info", ctypes.c_void_p),
                ("dim", ctypes.c_int32), ("damping", ctypes.c_float), ("damping_dev", ctypes.c_void_p),
                ("planes", ctypes.c_void_p)]


class kfac_pi_item(ctypes.Structure):
    _fields_ = [("A", ctypes.c_void_p), ("G", ctypes.c_void_p), ("dA", ctypes.c_int32), ("dG", ctypes.c_int32)]


class kfac_precond_item(ctypes.Structure):
    _fields_ = [("Ginv", ctypes.c_void_p), ("Ainv", ctypes.c_void_p), ("gradW", ctypes.c_void_p),
                ("out", ctypes.c_void_p), ("ws", ctypes.c_void_p), ("dG", ctypes.c_int32), ("dA", ctypes.c_int32),
                ("Ginv_planes", ctypes.c_void_p), ("Ainv_planes", ctypes.c_void_p)]


class KfacError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libkfac_hip.so (built by paper_1811_12019_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it first (python -m paper_1811_12019_amd.build). "
            "There is no CPU fallback.")
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, i32, f32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_float
    descp = ctypes.POINTER(kfac_layer_desc)
    itemp = ctypes.POINTER(kfac_inverse_item)
    lib.kfac_status_string.restype = ctypes.c_char_p
    lib.kfac_status_string.argtypes = [ctypes.c_int]
    lib.kfac_factor_workspace_bytes.restype = sz
    lib.kfac_factor_workspace_bytes.argtypes = [ctypes.c_int, descp]
    for name in ("kfac_factor_A", "kfac_factor_G"):
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int
        fn.argtypes = [descp, vp, f32, vp, vp, sz, vp]
    lib.kfac_factor_batched.restype = ctypes.c_int
    lib.kfac_factor_batched.argtypes = [ctypes.POINTER(kfac_factor_item), vp, i32, vp]
    lib.kfac_ema.restype = ctypes.c_int
    lib.kfac_ema.argtypes = [vp, vp, i32, f32, vp]
    lib.kfac_ema_batched.restype = ctypes.c_int
    lib.kfac_ema_batched.argtypes = [ctypes.POINTER(kfac_ema_item), i32, f32, vp]
    lib.kfac_pack_upper_batched.restype = ctypes.c_int
    lib.kfac_pack_upper_batched.argtypes = [ctypes.POINTER(kfac_pack_item), i32, vp]
    lib.kfac_ema_packed_batched.restype = ctypes.c_int
    lib.kfac_ema_packed_batched.argtypes = [ctypes.POINTER(kfac_ema_packed_item), i32, f32, vp]
    lib.kfac_factor_diff_workspace_bytes.restype = sz
    lib.kfac_factor_diff_workspace_bytes.argtypes = [ctypes.POINTER(kfac_diff_item), i32]
    lib.kfac_factor_diff_batched.restype = ctypes.c_int
    lib.kfac_factor_diff_batched.argtypes = [ctypes.POINTER(kfac_diff_item), i32, vp, vp, sz, vp]
    lib.kfac_factor_diff_batched_noalloc.restype = ctypes.c_int
    lib.kfac_factor_diff_batched_noalloc.argtypes = [ctypes.POINTER(kfac_diff_item), i32, vp, vp]
    lib.kfac_factor_diff_noalloc_max_elements.restype = sz
    lib.kfac_factor_diff_noalloc_max_elements.argtypes = []
    lib.kfac_weight_update_workspace_bytes.restype = sz
    lib.kfac_weight_update_workspace_bytes.argtypes = [ctypes.POINTER(kfac_update_item), i32]
    lib.kfac_weight_update_batched.restype = ctypes.c_int
    lib.kfac_weight_update_batched.argtypes = [ctypes.POINTER(kfac_update_item), i32, f32, f32, f32, vp, sz, vp]
    lib.kfac_bn_sample_grads_workspace_bytes.restype = sz
    lib.kfac_bn_sample_grads_workspace_bytes.argtypes = [i32, i32, i32]
    lib.kfac_bn_sample_grads.restype = ctypes.c_int
    lib.kfac_bn_sample_grads.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, sz, vp]
    lib.kfac_bn_sample_grads_batched_workspace_bytes.restype = sz
    lib.kfac_bn_sample_grads_batched_workspace_bytes.argtypes = [ctypes.POINTER(kfac_bn_item), i32]
    lib.kfac_bn_sample_grads_batched.restype = ctypes.c_int
    lib.kfac_bn_sample_grads_batched.argtypes = [ctypes.POINTER(kfac_bn_item), i32, vp, sz, vp]
    lib.kfac_bn_diag_precondition.restype = ctypes.c_int
    lib.kfac_bn_diag_precondition.argtypes = [vp, i32, i32, vp, f32, vp, vp, vp]
    lib.kfac_inverse_workspace_bytes.restype = sz
    lib.kfac_inverse_workspace_bytes.argtypes = [i32]
    lib.kfac_inverse_planes_bytes.restype = sz
    lib.kfac_inverse_planes_bytes.argtypes = [i32]
    lib.kfac_damped_inverse.restype = ctypes.c_int
    lib.kfac_damped_inverse.argtypes = [vp, i32, f32, vp, vp, vp, sz, vp]
    lib.kfac_damped_inverse_batched.restype = ctypes.c_int
    lib.kfac_damped_inverse_batched.argtypes = [itemp, i32, vp]
    lib.kfac_pi_damping_batched.restype = ctypes.c_int
    lib.kfac_pi_damping_batched.argtypes = [ctypes.POINTER(kfac_pi_item), i32, f32, vp, vp]
    f64 = ctypes.c_double
    lib.kfac_warmup_damping_alpha.restype = f64
    lib.kfac_warmup_damping_alpha.argtypes = [f64, f64, f64]
    lib.kfac_warmup_damping_next.restype = f64
    lib.kfac_warmup_damping_next.argtypes = [f64, f64, f64]
    lib.kfac_bn_damping.restype = f64
    lib.kfac_bn_damping.argtypes = [f64, f64]
    lib.kfac_refresh_interval.restype = i32
    lib.kfac_refresh_interval.argtypes = [i32, i32]
    lib.kfac_precondition_workspace_bytes.restype = sz
    lib.kfac_precondition_workspace_bytes.argtypes = [i32, i32]
    lib.kfac_precondition.restype = ctypes.c_int
    lib.kfac_precondition.argtypes = [vp, vp, vp, i32, i32, vp, vp, sz, vp]
    lib.kfac_precondition_batched.restype = ctypes.c_int
    lib.kfac_precondition_batched.argtypes = [ctypes.POINTER(kfac_precond_item), vp, i32, vp]
    lib.kfac_kernel_timing_enable.restype = ctypes.c_int
    lib.kfac_kernel_timing_enable.argtypes = [ctypes.c_int]
    lib.kfac_kernel_timing_report.restype = ctypes.c_int
    lib.kfac_kernel_timing_report.argtypes = [ctypes.c_char_p, sz]
    lib.kfac_probe_mfma.restype = ctypes.c_int
    lib.kfac_probe_mfma.argtypes = [i32, i32, i32, vp, vp]
    lib.kfac_probe_copy.restype = ctypes.c_int
    lib.kfac_probe_copy.argtypes = [vp, vp, sz, i32, vp]
    lib.kfac_probe_read.restype = ctypes.c_int
    lib.kfac_probe_read.argtypes = [vp, vp, sz, i32, vp]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().kfac_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != KFAC_OK:
        raise KfacError(status, where)


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


_TORCH_DTYPE = {KFAC_F32: torch.float32, KFAC_BF16: torch.bfloat16, KFAC_F16: torch.float16}


def make_desc(shape: "synth.LayerShape", layout: int, dtype: int, order: int) -> kfac_layer_desc:
    return kfac_layer_desc(shape.N, shape.C_in, shape.H, shape.W, shape.C_out, shape.kh, shape.kw, shape.stride,
                           shape.pad, int(shape.has_bias), layout, dtype, order)


def to_device_tensor(x_nchw, layout: int, dtype: int, device="cuda") -> torch.Tensor:
    """Place a logical (n, c, y, x) array in device memory in the given layout and dtype (contiguous)."""
    t = torch.as_tensor(x_nchw)
    if layout == KFAC_NHWC:
        t = t.permute(0, 2, 3, 1)
    return t.contiguous().to(device=device, dtype=_TORCH_DTYPE[dtype]).contiguous()


def alloc_workspace(nbytes: int, device="cuda") -> Optional[torch.Tensor]:
    """Device scratch of at least nbytes (torch's allocator hands out 512-byte aligned blocks)."""
    if nbytes <= 0:
        return None
    return torch.empty(int(nbytes), dtype=torch.uint8, device=device)


# ------------------------------------------------------------------------------------------------
# entry points, same names as the C ABI
# ------------------------------------------------------------------------------------------------
def kfac_factor_workspace_bytes(op: int, desc: kfac_layer_desc) -> int:
    return int(load_library().kfac_factor_workspace_bytes(op, ctypes.byref(desc)))


def _factor(name: str, op: int, desc, x, scale, out, ws, stream):
    lib = load_library()
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    rc = getattr(lib, name)(ctypes.byref(desc), _ptr(x), float(scale), _ptr(out), _ptr(ws), ws_bytes, _stream(stream))
    _check(rc, name)
    return out


def kfac_factor_A(desc: kfac_layer_desc, act: torch.Tensor, scale: float, A: torch.Tensor,
                  ws: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    return _factor("kfac_factor_A", KFAC_OP_FACTOR_A, desc, act, scale, A, ws, stream)


def kfac_factor_G(desc: kfac_layer_desc, gout: torch.Tensor, scale: float, G: torch.Tensor,
                  ws: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    return _factor("kfac_factor_G", KFAC_OP_FACTOR_G, desc, gout, scale, G, ws, stream)


class FactorBatch:
    """Host + device copies of a kfac_factor_item table (built once, reused every step).

    builds: sequence of (op, desc, x tensor, out tensor, scale).
    running: None, or one tensor per build: the build's result is folded into it (running average with `decay`) and the
    out tensor of that build is not written.  packed: the out tensors receive packed upper triangles.
    ws: None (scratch is allocated here), or one scratch tensor (or None where none is needed) per build, at least
    kfac_factor_workspace_bytes(op, desc) bytes each, which tables that never run at the same time may share."""

    def __init__(self, builds, device="cuda", running=None, decay: float = 0.0, packed: bool = False, ws=None):
        n = len(builds)
        self.count = n
        self.ws = (list(ws) if ws is not None else
                   [alloc_workspace(kfac_factor_workspace_bytes(op, desc), device) for op, desc, _, _, _ in builds])
        self.keep = (list(builds), running)
        arr = (kfac_factor_item * n)()
        for i, (op, desc, x, out, scale) in enumerate(builds):
            ws = self.ws[i]
            run = None if running is None else running[i]
            arr[i] = kfac_factor_item(desc, x.data_ptr(), None if run is not None else out.data_ptr(), _ptr(ws),
                                      0 if ws is None else ws.numel(), float(scale), int(op),
                                      _ptr(run), float(decay) if run is not None else 0.0, int(bool(packed)))
        self.host = arr
        self.dev = torch.frombuffer(bytearray(bytes(arr)), dtype=torch.uint8).to(device)


def kfac_factor_batched(batch: FactorBatch, stream=None) -> None:
    rc = load_library().kfac_factor_batched(batch.host, batch.dev.data_ptr(), batch.count, _stream(stream))
    _check(rc, "kfac_factor_batched")


def kfac_ema(running: torch.Tensor, fresh: torch.Tensor, dim: int, decay: float, stream=None) -> torch.Tensor:
    _check(load_library().kfac_ema(_ptr(running), _ptr(fresh), int(dim), float(decay), _stream(stream)), "kfac_ema")
    return running


class EmaBatch:
    """A kfac_ema_item table (host memory; built once, reused every step)."""

    def __init__(self, running: Sequence[torch.Tensor], fresh: Sequence[torch.Tensor]):
        n = len(running)
        self.count = n
        self.keep = (list(running), list(fresh))
        arr = (kfac_ema_item * max(n, 1))()
        for i in range(n):
            arr[i] = kfac_ema_item(running[i].data_ptr(), fresh[i].data_ptr(), int(running[i].shape[0]))
        self.host = arr


def kfac_ema_batched(batch: EmaBatch, decay: float, stream=None) -> None:
    rc = load_library().kfac_ema_batched(batch.host, batch.count, float(decay), _stream(stream))
    _check(rc, "kfac_ema_batched")


def packed_elems(dim: int) -> int:
    return dim * (dim + 1) // 2


class PackBatch:
    """kfac_pack_item / kfac_ema_packed_item tables (host memory) over the same (full, packed) tensor pairs."""

    def __init__(self, full: Sequence[torch.Tensor], packed: Sequence[torch.Tensor]):
        n = len(full)
        self.count = n
        self.keep = (list(full), list(packed))
        self.pack_items = (kfac_pack_item * max(n, 1))()
        self.ema_items = (kfac_ema_packed_item * max(n, 1))()
        for i in range(n):
            d = int(full[i].shape[0])
            assert packed[i].numel() == packed_elems(d)
            self.pack_items[i] = kfac_pack_item(full[i].data_ptr(), packed[i].data_ptr(), d)
            self.ema_items[i] = kfac_ema_packed_item(full[i].data_ptr(), packed[i].data_ptr(), d)


def kfac_pack_upper_batched(batch: PackBatch, stream=None) -> None:
    """packed[i] <- upper triangle of full[i]."""
    _check(load_library().kfac_pack_upper_batched(batch.pack_items, batch.count, _stream(stream)), "kfac_pack_upper_batched")


def kfac_ema_packed_batched(batch: PackBatch, decay: float, stream=None) -> None:
    """full[i] (a running average) <- decay * full[i] + (1 - decay) * unpack(packed[i])."""
    _check(load_library().kfac_ema_packed_batched(batch.ema_items, batch.count, float(decay), _stream(stream)),
           "kfac_ema_packed_batched")


class DiffBatch:
    """A kfac_diff_item table (host memory), its scratch and its device output (one float per matrix)."""

    def __init__(self, x: Sequence[torch.Tensor], x_prev: Sequence[torch.Tensor], device="cuda"):
        n = len(x)
        self.count = n
        self.keep = (list(x), list(x_prev))
        self.host = (kfac_diff_item * max(n, 1))()
        for i in range(n):
            self.host[i] = kfac_diff_item(x[i].data_ptr(), x_prev[i].data_ptr(), int(x[i].shape[0]))
        nbytes = int(load_library().kfac_factor_diff_workspace_bytes(self.host, n)) if n else 0
        self.ws = alloc_workspace(nbytes, device) if nbytes else None
        self.out = torch.zeros(max(n, 1), dtype=torch.float32, device=device)


def kfac_factor_diff_batched(batch: DiffBatch, stream=None) -> torch.Tensor:
    """out[i] = ||x[i] - x_prev[i]||_F / ||x_prev[i]||_F; returns the device tensor of results."""
    ws_bytes = 0 if batch.ws is None else batch.ws.numel() * batch.ws.element_size()
    rc = load_library().kfac_factor_diff_batched(batch.host, batch.count, _ptr(batch.out), _ptr(batch.ws), ws_bytes,
                                                 _stream(stream))
    _check(rc, "kfac_factor_diff_batched")
    return batch.out[:batch.count]


def kfac_factor_diff_batched_noalloc(items_host, count: int, out: torch.Tensor, stream=None) -> torch.Tensor:
    """The same computation with the library's fixed scratch: nothing is allocated (items_host: a kfac_diff_item array)."""
    rc = load_library().kfac_factor_diff_batched_noalloc(items_host, int(count), _ptr(out), _stream(stream))
    _check(rc, "kfac_factor_diff_batched_noalloc")
    return out


def kfac_factor_diff_noalloc_max_elements() -> int:
    return int(load_library().kfac_factor_diff_noalloc_max_elements())


class UpdateBatch:
    """A kfac_update_item table (host memory) and its scratch; d_out of a layer = rows of its weight matrix."""

    def __init__(self, w: Sequence[torch.Tensor], w_prev: Sequence[torch.Tensor], precond: Sequence[torch.Tensor],
                 device="cuda"):
        n = len(w)
        self.count = n
        self.keep = (list(w), list(w_prev), list(precond))
        self.host = (kfac_update_item * max(n, 1))()
        for i in range(n):
            self.host[i] = kfac_update_item(w[i].data_ptr(), w_prev[i].data_ptr(), precond[i].data_ptr(),
                                            int(w[i].numel()), int(w[i].shape[0]))
        nbytes = int(load_library().kfac_weight_update_workspace_bytes(self.host, n)) if n else 0
        self.ws = alloc_workspace(nbytes, device) if nbytes else None


def kfac_weight_update_batched(batch: UpdateBatch, eta: float, momentum: float, eps: float = 1e-9, stream=None) -> None:
    ws_bytes = 0 if batch.ws is None else batch.ws.numel() * batch.ws.element_size()
    rc = load_library().kfac_weight_update_batched(batch.host, batch.count, float(eta), float(momentum), float(eps),
                                                   _ptr(batch.ws), ws_bytes, _stream(stream))
    _check(rc, "kfac_weight_update_batched")


def kfac_bn_sample_grads_workspace_bytes(N: int, C: int, HW: int) -> int:
    return int(load_library().kfac_bn_sample_grads_workspace_bytes(int(N), int(C), int(HW)))


def kfac_bn_sample_grads(xhat: torch.Tensor, gout: torch.Tensor, dtype: int, g: Optional[torch.Tensor] = None,
                         ws: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """xhat, gout: (N, H, W, C) or (N, HW, C) channels-last tensors of the given kfac dtype; returns g (N, 2C) fp32."""
    N, C = int(xhat.shape[0]), int(xhat.shape[-1])
    HW = int(xhat.numel() // (N * C))
    if g is None:
        g = torch.empty((N, 2 * C), dtype=torch.float32, device=xhat.device)
    if ws is None:
        ws = alloc_workspace(int(load_library().kfac_bn_sample_grads_workspace_bytes(N, C, HW)), xhat.device)
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    rc = load_library().kfac_bn_sample_grads(_ptr(xhat), _ptr(gout), N, C, HW, int(dtype), _ptr(g), _ptr(ws), ws_bytes,
                                             _stream(stream))
    _check(rc, "kfac_bn_sample_grads")
    return g


class BnBatch:
    """A kfac_bn_item table (host memory), the per-sample gradient tensors (N, 2C) and the scratch, for many BN layers.
    xhat[i], gout[i]: channels-last (N, H, W, C) or (N, HW, C) tensors of kfac dtype dtype[i] (one value: all layers)."""

    def __init__(self, xhat: Sequence[torch.Tensor], gout: Sequence[torch.Tensor], dtype, device="cuda"):
        n = len(xhat)
        dtypes = list(dtype) if isinstance(dtype, (list, tuple)) else [int(dtype)] * n
        self.count = n
        self.g = []
        self.host = (kfac_bn_item * max(n, 1))()
        for i in range(n):
            N, C = int(xhat[i].shape[0]), int(xhat[i].shape[-1])
            HW = int(xhat[i].numel() // (N * C))
            self.g.append(torch.empty((N, 2 * C), dtype=torch.float32, device=device))
            self.host[i] = kfac_bn_item(xhat[i].data_ptr(), gout[i].data_ptr(), self.g[i].data_ptr(), N, C, HW, dtypes[i])
        self.keep = (list(xhat), list(gout))
        nbytes = int(load_library().kfac_bn_sample_grads_batched_workspace_bytes(self.host, n)) if n else 0
        self.ws = alloc_workspace(nbytes, device) if nbytes else None


def kfac_bn_sample_grads_batched(batch: BnBatch, stream=None):
    ws_bytes = 0 if batch.ws is None else batch.ws.numel() * batch.ws.element_size()
    rc = load_library().kfac_bn_sample_grads_batched(batch.host, batch.count, _ptr(batch.ws), ws_bytes, _stream(stream))
    _check(rc, "kfac_bn_sample_grads_batched")
    return batch.g


def kfac_bn_diag_precondition(g: torch.Tensor, grad: Optional[torch.Tensor], damping: float,
                              fisher_diag: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                              stream=None) -> None:
    N, C2 = int(g.shape[0]), int(g.shape[1])
    rc = load_library().kfac_bn_diag_precondition(_ptr(g), N, C2, _ptr(grad), float(damping), _ptr(fisher_diag), _ptr(out),
                                                  _stream(stream))
    _check(rc, "kfac_bn_diag_precondition")


def kfac_inverse_workspace_bytes(dim: int) -> int:
    return int(load_library().kfac_inverse_workspace_bytes(int(dim)))


def kfac_damped_inverse(S: torch.Tensor, dim: int, damping: float, Minv: torch.Tensor,
                        info: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None,
                        stream=None) -> torch.Tensor:
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    rc = load_library().kfac_damped_inverse(_ptr(S), int(dim), float(damping), _ptr(Minv), _ptr(info), _ptr(ws),
                                            ws_bytes, _stream(stream))
    _check(rc, "kfac_damped_inverse")
    return Minv


class InverseBatch:
    """A kfac_inverse_item table (host memory; built once, reused every step) and the scratch it points to."""

    def __init__(self, S: Sequence[torch.Tensor], Minv: Sequence[torch.Tensor], dampings: Sequence[float],
                 info: Optional[torch.Tensor] = None, device="cuda",
                 dampings_dev: Optional[Sequence[Optional[int]]] = None, ws=None, planes=None):
        """dampings_dev[i]: None, or the device address of a float that replaces dampings[i] when the work runs.
        planes: None, or per matrix None / a byte tensor of kfac_inverse_planes_bytes(dim) that receives the inverse as
        fp16 piece planes (what PrecondBatch takes as Ginv_planes / Ainv_planes).
        ws: None (scratch is allocated here), or one scratch tensor per matrix of kfac_inverse_workspace_bytes(dim)
        bytes, which tables that never run at the same time may share."""
        n = len(S)
        dims = [int(s.shape[0]) for s in S]
        self.order = sorted(range(n), key=lambda i: -dims[i])        # the ABI wants largest first
        self.count = n
        self.ws = list(ws) if ws is not None else [alloc_workspace(kfac_inverse_workspace_bytes(d), device) for d in dims]
        self.info = info if info is not None else torch.zeros(n, dtype=torch.int32, device=device)
        self.keep = (list(S), list(Minv), None if planes is None else list(planes))
        arr = (kfac_inverse_item * n)()
        for slot, i in enumerate(self.order):
            arr[slot] = kfac_inverse_item(S[i].data_ptr(), Minv[i].data_ptr(), _ptr(self.ws[i]),
                                          self.info.data_ptr() + 4 * i, dims[i], float(dampings[i]),
                                          None if dampings_dev is None else dampings_dev[i],
                                          None if planes is None else _ptr(planes[i]))
        self.host = arr


def kfac_inverse_planes_bytes(dim: int) -> int:
    return int(load_library().kfac_inverse_planes_bytes(int(dim)))


def kfac_damped_inverse_batched(batch: InverseBatch, stream=None) -> None:
    rc = load_library().kfac_damped_inverse_batched(batch.host, batch.count, _stream(stream))
    _check(rc, "kfac_damped_inverse_batched")


KFAC_REFRESH_GROWING, KFAC_REFRESH_LATE = 0, 1


class PiBatch:
    """A kfac_pi_item table (host memory) and the device array of per-factor dampings it fills: lam[2 i] for A_i,
    lam[2 i + 1] for G_i."""

    def __init__(self, A: Sequence[torch.Tensor], G: Sequence[torch.Tensor], device="cuda"):
        n = len(A)
        self.count = n
        self.keep = (list(A), list(G))
        self.host = (kfac_pi_item * max(n, 1))()
        for i in range(n):
            self.host[i] = kfac_pi_item(A[i].data_ptr(), G[i].data_ptr(), int(A[i].shape[0]), int(G[i].shape[0]))
        self.lam = torch.zeros(2 * max(n, 1), dtype=torch.float32, device=device)

    def address(self, layer: int, which: int) -> int:
        """Device address of lambda_A (which = 0) or lambda_G (which = 1) of a layer."""
        return self.lam.data_ptr() + 4 * (2 * layer + which)


def kfac_pi_damping_batched(batch: PiBatch, gamma: float, stream=None) -> torch.Tensor:
    rc = load_library().kfac_pi_damping_batched(batch.host, batch.count, float(gamma), _ptr(batch.lam), _stream(stream))
    _check(rc, "kfac_pi_damping_batched")
    return batch.lam[:2 * batch.count]


def kfac_warmup_damping_alpha(gamma0: float, gamma_target: float, t_warmup: float) -> float:
    return float(load_library().kfac_warmup_damping_alpha(float(gamma0), float(gamma_target), float(t_warmup)))


def kfac_warmup_damping_next(gamma: float, gamma_target: float, alpha: float) -> float:
    return float(load_library().kfac_warmup_damping_next(float(gamma), float(gamma_target), float(alpha)))


def kfac_bn_damping(gamma: float, rho_bn: float) -> float:
    return float(load_library().kfac_bn_damping(float(gamma), float(rho_bn)))


def kfac_refresh_interval(epoch: int, heuristic: int = KFAC_REFRESH_GROWING) -> int:
    return int(load_library().kfac_refresh_interval(int(epoch), int(heuristic)))


def kfac_precondition_workspace_bytes(dG: int, dA: int) -> int:
    return int(load_library().kfac_precondition_workspace_bytes(int(dG), int(dA)))


def kfac_precondition(Ginv: torch.Tensor, Ainv: torch.Tensor, gradW: torch.Tensor, dG: int, dA: int,
                      out: torch.Tensor, ws: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    rc = load_library().kfac_precondition(_ptr(Ginv), _ptr(Ainv), _ptr(gradW), int(dG), int(dA), _ptr(out), _ptr(ws),
                                          ws_bytes, _stream(stream))
    _check(rc, "kfac_precondition")
    return out


class PrecondBatch:
    """Host + device copies of a kfac_precond_item table (built once, reused every step).  ws: None (scratch is
    allocated here), or one scratch tensor per layer of kfac_precondition_workspace_bytes(d_G, d_A) bytes."""

    def __init__(self, Ginv: Sequence[torch.Tensor], Ainv: Sequence[torch.Tensor], gradW: Sequence[torch.Tensor],
                 out: Sequence[torch.Tensor], device="cuda", ws=None, Ginv_planes=None, Ainv_planes=None):
        """Ginv_planes / Ainv_planes: None, or per layer None / the planes tensor an InverseBatch filled for that inverse."""
        n = len(out)
        shapes = [tuple(g.shape) for g in gradW]
        self.order = sorted(range(n), key=lambda i: -shapes[i][1])       # large d_A first: best load balance
        self.count = n
        self.ws = (list(ws) if ws is not None else
                   [alloc_workspace(kfac_precondition_workspace_bytes(dG, dA), device) for dG, dA in shapes])
        self.keep = (list(Ginv), list(Ainv), list(gradW), list(out), Ginv_planes, Ainv_planes)
        arr = (kfac_precond_item * n)()
        for slot, i in enumerate(self.order):
            arr[slot] = kfac_precond_item(Ginv[i].data_ptr(), Ainv[i].data_ptr(), gradW[i].data_ptr(),
                                          out[i].data_ptr(), self.ws[i].data_ptr(), shapes[i][0], shapes[i][1],
                                          None if Ginv_planes is None else _ptr(Ginv_planes[i]),
                                          None if Ainv_planes is None else _ptr(Ainv_planes[i]))
        self.host = arr
        self.dev = torch.frombuffer(bytearray(bytes(arr)), dtype=torch.uint8).to(device)


def kfac_precondition_batched(batch: PrecondBatch, stream=None) -> None:
    rc = load_library().kfac_precondition_batched(batch.host, batch.dev.data_ptr(), batch.count, _stream(stream))
    _check(rc, "kfac_precondition_batched")


def kfac_kernel_timing_enable(enable: bool) -> None:
    _check(load_library().kfac_kernel_timing_enable(int(bool(enable))), "kfac_kernel_timing_enable")


def kfac_probe_mfma(dtype: int, workgroups: int, iters: int, out: torch.Tensor, stream=None) -> None:
    _check(load_library().kfac_probe_mfma(int(dtype), int(workgroups), int(iters), _ptr(out), _stream(stream)), "kfac_probe_mfma")


def kfac_probe_copy(src: torch.Tensor, dst: torch.Tensor, workgroups: int, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    _check(load_library().kfac_probe_copy(_ptr(src), _ptr(dst), nbytes, int(workgroups), _stream(stream)), "kfac_probe_copy")


def kfac_probe_read(src: torch.Tensor, sink: torch.Tensor, workgroups: int, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    _check(load_library().kfac_probe_read(_ptr(src), _ptr(sink), nbytes, int(workgroups), _stream(stream)), "kfac_probe_read")


def kfac_kernel_timing_report() -> dict:
    """{kernel name: (total milliseconds, launches)} since timing was enabled or last reported."""
    buf = ctypes.create_string_buffer(1 << 16)
    _check(load_library().kfac_kernel_timing_report(buf, len(buf)), "kfac_kernel_timing_report")
    out = {}
    for line in buf.value.decode().splitlines():
        name, ms, n = line.rsplit(" ", 2)
        out[name] = (float(ms), int(n))
    return out
