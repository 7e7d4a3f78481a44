"""Thin ctypes binding over libmpcnn.so (the C ABI declared in include/mpcnn.h).

Argument marshalling only: every step of the whole-image forward / backward
runs in the library's HIP kernels.  PyTorch supplies device memory (tensors'
`data_ptr()`) and the stream.  There is no fallback: if the library has not
been built, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmpcnn.so")

KIND_C, KIND_MP, KIND_FC = 0, 1, 2
STATIC_WORKSPACE_BYTES = 64 * 1024 * 1024   # MPCNN_STATIC_WORKSPACE_BYTES
F32, BF16 = 0, 1

STATUS = {0: "MPCNN_OK", 1: "MPCNN_EINVAL", 2: "MPCNN_ESHAPE", 3: "MPCNN_EWORKSPACE",
          4: "MPCNN_EUNSUPPORTED", 5: "MPCNN_EHIP", 6: "MPCNN_ENOMEM"}

# every symbol include/mpcnn.h declares
SYMBOLS = [
    "mpcnn_net_create", "mpcnn_net_destroy", "mpcnn_net_patch", "mpcnn_net_classes",
    "mpcnn_param_count", "mpcnn_layer_shape", "mpcnn_set_params", "mpcnn_get_params",
    "mpcnn_get_grads", "mpcnn_workspace_bytes", "mpcnn_seg_forward", "mpcnn_seg_backward",
    "mpcnn_sgd_step", "mpcnn_get_activation", "mpcnn_get_argmax", "mpcnn_last_error",
    "mpcnn_profile_enable", "mpcnn_profile_read", "mpcnn_workspace_bytes_same", "mpcnn_seg_forward_same",
    "mpcnn_set_loss", "mpcnn_class_balance_weights", "mpcnn_seg_loss", "mpcnn_armijo_step",
    "mpcnn_lbfgs_step", "mpcnn_lbfgs_reset", "mpcnn_set_activation", "mpcnn_set_conv_tiling",
    "mpcnn_workspace_bytes_banded", "mpcnn_seg_backward_banded", "mpcnn_seg_forward_static",
    "mpcnn_plan_describe",
]


class MpcnnError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("%s: %s" % (STATUS.get(status, status), message))
        self.status = status


class _LayerDesc(C.Structure):
    _fields_ = [("kind", C.c_int), ("maps", C.c_int), ("k", C.c_int), ("k2", C.c_int)]


class KernelStat(C.Structure):
    """mpcnn_kernel_stat: one launch site (kernel x layer) of the profiled calls."""
    _fields_ = [("name", C.c_char * 48), ("layer", C.c_int), ("step", C.c_int),
                ("launches", C.c_int), ("ms_total", C.c_double), ("flops", C.c_double),
                ("bytes", C.c_double)]


_lib = None


def lib():
    """Load libmpcnn.so (built by `python -m paper_1302_1690_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libmpcnn.so is not built: run `python -m paper_1302_1690_amd.build` "
                              "(there is no fallback path)")
        # torch ships its own copy of the HIP runtime (same soname as the system one):
        # it must be loaded first so that the library binds to it and both share one
        # runtime, hence one set of device allocations and streams.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp, sz, i = C.c_void_p, C.c_size_t, C.c_int
        L.mpcnn_net_create.argtypes = [C.POINTER(_LayerDesc), i, i, i, i, C.POINTER(vp)]
        L.mpcnn_net_destroy.argtypes = [vp]
        L.mpcnn_net_destroy.restype = None
        L.mpcnn_net_patch.argtypes = [vp]
        L.mpcnn_net_classes.argtypes = [vp]
        L.mpcnn_param_count.argtypes = [vp]
        L.mpcnn_param_count.restype = sz
        L.mpcnn_layer_shape.argtypes = [vp, i, i, i] + [C.POINTER(i)] * 4
        L.mpcnn_plan_describe.argtypes = [vp, i, i, i, i, C.c_char_p, sz]
        L.mpcnn_set_params.argtypes = [vp, vp, sz]
        L.mpcnn_get_params.argtypes = [vp, vp, sz]
        L.mpcnn_get_grads.argtypes = [vp, vp, sz]
        L.mpcnn_workspace_bytes.argtypes = [vp, i, i, i, i]
        L.mpcnn_workspace_bytes.restype = sz
        L.mpcnn_seg_forward.argtypes = [vp, vp, i, i, i, vp, vp, sz, vp]
        L.mpcnn_seg_forward_static.argtypes = [vp, vp, i, i, i, vp, vp]
        L.mpcnn_workspace_bytes_same.argtypes = [vp, i, i, i]
        L.mpcnn_workspace_bytes_same.restype = sz
        L.mpcnn_seg_forward_same.argtypes = [vp, vp, i, i, i, vp, vp, sz, vp]
        L.mpcnn_seg_loss.argtypes = [vp, vp, vp, vp, i, i, i, vp, vp, sz, vp]
        L.mpcnn_armijo_step.argtypes = [vp, vp, vp, vp, i, i, i, C.c_double, C.c_float, C.c_float, C.c_float,
                                        C.c_float, i, vp, sz, vp, C.POINTER(C.c_float), C.POINTER(C.c_double),
                                        C.POINTER(i)]
        L.mpcnn_lbfgs_step.argtypes = [vp, vp, vp, vp, i, i, i, C.c_double, i, C.c_float, C.c_float, C.c_float,
                                       i, vp, sz, vp, C.POINTER(C.c_float), C.POINTER(C.c_double),
                                       C.POINTER(i), C.POINTER(i)]
        L.mpcnn_lbfgs_reset.argtypes = [vp]
        L.mpcnn_set_loss.argtypes = [vp, i]
        L.mpcnn_workspace_bytes_banded.argtypes = [vp, i, i, i]
        L.mpcnn_workspace_bytes_banded.restype = sz
        L.mpcnn_seg_backward_banded.argtypes = [vp, vp, vp, vp, i, i, i, i, vp, vp, vp, sz, vp]
        L.mpcnn_set_activation.argtypes = [vp, i]
        L.mpcnn_set_conv_tiling.argtypes = [vp, i, i]
        L.mpcnn_class_balance_weights.argtypes = [vp, vp, i, i, i, vp, vp, vp]
        L.mpcnn_seg_backward.argtypes = [vp, vp, vp, vp, i, i, i, vp, vp, vp, sz, vp]
        L.mpcnn_sgd_step.argtypes = [vp, C.c_float, C.c_float, vp]
        L.mpcnn_get_activation.argtypes = [vp, i, vp, sz]
        L.mpcnn_get_argmax.argtypes = [vp, i, vp, sz]
        L.mpcnn_last_error.restype = C.c_char_p
        L.mpcnn_profile_enable.argtypes = [vp, i]
        L.mpcnn_profile_read.argtypes = [vp, C.POINTER(KernelStat), i, C.POINTER(i)]
        _lib = L
    return _lib


def _check(st: int):
    if st != 0:
        raise MpcnnError(st, lib().mpcnn_last_error().decode())


def _stream_handle(stream) -> int:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return int(getattr(stream, "cuda_stream", stream))


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


class Net:
    """mpcnn_net handle.  `layers`: (kind, maps, k) triples; see include/mpcnn.h."""

    def __init__(self, layers: Sequence[Tuple[int, int, int]], in_channels: int, patch: int,
                 dtype: int = F32):
        arr = (_LayerDesc * len(layers))(*[_LayerDesc(int(l[0]), int(l[1]), int(l[2]), int(l[3]) if len(l) > 3 else 0)
                                           for l in layers])
        h = C.c_void_p()
        _check(lib().mpcnn_net_create(arr, len(layers), in_channels, patch, dtype, C.byref(h)))
        self._h = h
        self.layers = [tuple(int(v) for v in l) for l in layers]
        self.in_channels = in_channels
        self._ws = None

    def close(self):
        if getattr(self, "_h", None):
            lib().mpcnn_net_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except TypeError:     # interpreter shutdown: the module's globals are already gone
            pass

    # ---- host-only queries
    @property
    def patch(self) -> int:
        return lib().mpcnn_net_patch(self._h)

    @property
    def n_classes(self) -> int:
        return lib().mpcnn_net_classes(self._h)

    @property
    def param_count(self) -> int:
        return lib().mpcnn_param_count(self._h)

    def layer_shape(self, H: int, W: int, layer: int):
        r, c, ch, sp = C.c_int(), C.c_int(), C.c_int(), C.c_int()
        _check(lib().mpcnn_layer_shape(self._h, H, W, layer, C.byref(r), C.byref(c), C.byref(ch),
                                       C.byref(sp)))
        return r.value, c.value, ch.value, sp.value

    def workspace_bytes(self, B: int, H: int, W: int, training: bool) -> int:
        return lib().mpcnn_workspace_bytes(self._h, B, H, W, 1 if training else 0)

    def plan_describe(self, B: int, H: int, W: int, training: bool) -> str:
        """Text: the kernel, tiling and launch shape of every layer for a call of these sizes."""
        buf = C.create_string_buffer(1 << 16)
        _check(lib().mpcnn_plan_describe(self._h, B, H, W, 1 if training else 0, buf, len(buf)))
        return buf.value.decode()

    # ---- parameters
    def set_params(self, params: np.ndarray):
        p = np.ascontiguousarray(params, dtype=np.float32)
        _check(lib().mpcnn_set_params(self._h, p.ctypes.data, p.size))

    def get_params(self) -> np.ndarray:
        out = np.empty(self.param_count, dtype=np.float32)
        _check(lib().mpcnn_get_params(self._h, out.ctypes.data, out.size))
        return out

    def get_grads(self) -> np.ndarray:
        out = np.empty(self.param_count, dtype=np.float32)
        _check(lib().mpcnn_get_grads(self._h, out.ctypes.data, out.size))
        return out

    # ---- device calls (torch tensors carry the memory)
    def alloc_workspace(self, B: int, H: int, W: int, training: bool):
        import torch
        need = self.workspace_bytes(B, H, W, training)
        if need == 0:
            raise MpcnnError(2, "image %dx%d does not fit the net" % (H, W))
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        return self._ws

    def seg_forward(self, image, probs=None, ws=None, stream=None):
        """image [B,C0,H,W] fp32 cuda tensor -> probs [B,n_cls,H-P+1,W-P+1]."""
        import torch
        B, _, H, W = image.shape
        assert image.is_cuda and image.dtype == torch.float32 and image.is_contiguous()
        if ws is None:
            ws = self.alloc_workspace(B, H, W, False)
        if probs is None:
            probs = torch.empty((B, self.n_classes, H - self.patch + 1, W - self.patch + 1),
                                dtype=torch.float32, device=image.device)
        _check(lib().mpcnn_seg_forward(self._h, _ptr(image), B, H, W, _ptr(probs), _ptr(ws),
                                       ws.numel(), _stream_handle(stream)))
        return probs

    def seg_forward_static(self, image, probs, stream=None):
        """seg_forward on the library's fixed device workspace: no allocation anywhere in the
        call (the caller supplies `probs`)."""
        B, _, H, W = image.shape
        _check(lib().mpcnn_seg_forward_static(self._h, _ptr(image), B, H, W, _ptr(probs), _stream_handle(stream)))
        return probs

    def seg_loss(self, image, labels, pixw=None, ws=None, stream=None) -> float:
        """Summed loss at the current parameters (forward only, nothing kept)."""
        import torch
        B, _, H, W = image.shape
        if ws is None:
            ws = self.alloc_workspace(B, H, W, False)
        loss = torch.zeros(1, dtype=torch.float64, device=image.device)
        _check(lib().mpcnn_seg_loss(self._h, _ptr(image), _ptr(labels), _ptr(pixw), B, H, W, _ptr(loss),
                                    _ptr(ws), ws.numel(), _stream_handle(stream)))
        return float(loss.item())

    def armijo_step(self, image, labels, f0, alpha0, pixw=None, grad_scale=1.0, c=1e-4, beta=0.5,
                    max_trials=20, ws=None, stream=None):
        """Safeguarded gradient step after seg_backward on the same inputs -> (alpha, loss, trials)."""
        B, _, H, W = image.shape
        if ws is None:
            ws = self.alloc_workspace(B, H, W, False)
        a, f, t = C.c_float(0), C.c_double(0), C.c_int(0)
        _check(lib().mpcnn_armijo_step(self._h, _ptr(image), _ptr(labels), _ptr(pixw), B, H, W, f0, alpha0,
                                       grad_scale, c, beta, max_trials, _ptr(ws), ws.numel(),
                                       _stream_handle(stream), C.byref(a), C.byref(f), C.byref(t)))
        return a.value, f.value, t.value

    def lbfgs_step(self, image, labels, f0, history=8, alpha0=1.0, pixw=None, c=1e-4, beta=0.5,
                   max_trials=20, ws=None, stream=None):
        """Limited-memory BFGS iteration after seg_backward on the same inputs
        -> (alpha, loss, trials, pairs used)."""
        B, _, H, W = image.shape
        if ws is None:
            ws = self.alloc_workspace(B, H, W, False)
        a, f, t, m = C.c_float(0), C.c_double(0), C.c_int(0), C.c_int(0)
        _check(lib().mpcnn_lbfgs_step(self._h, _ptr(image), _ptr(labels), _ptr(pixw), B, H, W, f0, history,
                                      alpha0, c, beta, max_trials, _ptr(ws), ws.numel(),
                                      _stream_handle(stream), C.byref(a), C.byref(f), C.byref(t), C.byref(m)))
        return a.value, f.value, t.value, m.value

    def lbfgs_reset(self):
        _check(lib().mpcnn_lbfgs_reset(self._h))

    def set_loss(self, kind: str):
        """"mcce": softmax + cross-entropy (default); "mse": linear outputs, half the squared error."""
        _check(lib().mpcnn_set_loss(self._h, {"mcce": 0, "mse": 1}.get(kind, -1)))

    def seg_backward_banded(self, image, labels, band_rows, pixw=None, probs=None, loss=None, stream=None):
        """Forward + backward with the image taken in bands of `band_rows` output rows; the
        workspace (allocated here) is one band's.  Gradients stay in the net."""
        import torch
        B, _, H, W = image.shape
        assert image.is_cuda and image.dtype == torch.float32 and image.is_contiguous()
        assert labels.dtype == torch.int32 and labels.is_contiguous() and tuple(labels.shape) == (B, H, W)
        n = lib().mpcnn_workspace_bytes_banded(self._h, B, W, band_rows)
        if n == 0:
            raise MpcnnError(2, "no plan for bands of %d rows" % band_rows)
        ws = torch.empty(n, dtype=torch.uint8, device=image.device)
        _check(lib().mpcnn_seg_backward_banded(self._h, _ptr(image), _ptr(labels), _ptr(pixw), B, H, W, band_rows,
                                               _ptr(probs), _ptr(loss), _ptr(ws), ws.numel(),
                                               _stream_handle(stream)))
        return probs, loss

    def set_activation(self, kind: str):
        """"tanh" (default) or "logistic": the squashing function of C and hidden FC layers."""
        _check(lib().mpcnn_set_activation(self._h, {"tanh": 0, "logistic": 1}.get(kind, -1)))

    def set_conv_tiling(self, position_tiles: int = 0, tiles_per_wave: int = 0):
        """Restrict the matrix-core convolution kernel's tiling (0 = the planner's choice)."""
        _check(lib().mpcnn_set_conv_tiling(self._h, position_tiles, tiles_per_wave))

    def class_balance_weights(self, labels, stream=None):
        """labels [B,H,W] int32 cuda -> pixw [B,H,W] fp32 cuda, 1/N_k at output pixels of class k."""
        import torch
        B, H, W = labels.shape
        assert labels.is_cuda and labels.dtype == torch.int32 and labels.is_contiguous()
        pixw = torch.empty((B, H, W), dtype=torch.float32, device=labels.device)
        counts = torch.empty(16, dtype=torch.int32, device=labels.device)
        _check(lib().mpcnn_class_balance_weights(self._h, _ptr(labels), B, H, W, _ptr(pixw), _ptr(counts),
                                                 _stream_handle(stream)))
        return pixw, counts

    def seg_forward_same(self, image, probs=None, ws=None, stream=None):
        """Deployment forward with mirrored borders: image [B,C0,H,W] -> probs [B,n_cls,H,W]."""
        import torch
        B, _, H, W = image.shape
        assert image.is_cuda and image.dtype == torch.float32 and image.is_contiguous()
        if ws is None:
            need = lib().mpcnn_workspace_bytes_same(self._h, B, H, W)
            if need == 0:
                raise MpcnnError(2, "image %dx%d does not fit the net" % (H, W))
            if self._ws is None or self._ws.numel() < need:
                self._ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            ws = self._ws
        if probs is None:
            probs = torch.empty((B, self.n_classes, H, W), dtype=torch.float32, device=image.device)
        _check(lib().mpcnn_seg_forward_same(self._h, _ptr(image), B, H, W, _ptr(probs), _ptr(ws),
                                            ws.numel(), _stream_handle(stream)))
        return probs

    def seg_backward(self, image, labels, pixw=None, probs=None, loss=None, ws=None, stream=None):
        """Forward + backward; gradients stay in the net.  Returns (probs, loss) as given."""
        import torch
        B, _, H, W = image.shape
        assert image.is_cuda and image.dtype == torch.float32 and image.is_contiguous()
        assert labels.dtype == torch.int32 and labels.is_contiguous() and tuple(labels.shape) == (B, H, W)
        if pixw is not None:
            assert pixw.dtype == torch.float32 and pixw.is_contiguous() and tuple(pixw.shape) == (B, H, W)
        if loss is not None:
            assert loss.dtype == torch.float64 and loss.numel() == 1
        if ws is None:
            ws = self.alloc_workspace(B, H, W, True)
        _check(lib().mpcnn_seg_backward(self._h, _ptr(image), _ptr(labels), _ptr(pixw), B, H, W,
                                        _ptr(probs), _ptr(loss), _ptr(ws), ws.numel(),
                                        _stream_handle(stream)))
        return probs, loss

    def sgd_step(self, lr: float, grad_scale: float = 1.0, stream=None):
        _check(lib().mpcnn_sgd_step(self._h, lr, grad_scale, _stream_handle(stream)))

    # ---- per-kernel timing
    def profile_enable(self, on: bool):
        _check(lib().mpcnn_profile_enable(self._h, 1 if on else 0))

    def profile_read(self):
        """List of dicts (name, layer, step, launches, ms_total, flops, bytes), waits for the GPU."""
        cap = 256
        arr = (KernelStat * cap)()
        n = C.c_int(0)
        _check(lib().mpcnn_profile_read(self._h, arr, cap, C.byref(n)))
        return [dict(name=arr[k].name.decode(), layer=arr[k].layer, step=arr[k].step,
                     launches=arr[k].launches, ms_total=arr[k].ms_total, flops=arr[k].flops,
                     bytes=arr[k].bytes) for k in range(min(n.value, cap))]

    # ---- test hooks
    def get_activation(self, B: int, H: int, W: int, layer: int) -> np.ndarray:
        r, c, ch, _ = self.layer_shape(H, W, layer)
        out = np.empty((B, r, c, ch), dtype=np.float32)
        _check(lib().mpcnn_get_activation(self._h, layer, out.ctypes.data, out.size))
        return out

    def get_argmax(self, B: int, H: int, W: int, layer: int) -> np.ndarray:
        r, c, ch, _ = self.layer_shape(H, W, layer)
        out = np.empty((B, r, c, ch), dtype=np.uint8)
        _check(lib().mpcnn_get_argmax(self._h, layer, out.ctypes.data, out.size))
        return out
