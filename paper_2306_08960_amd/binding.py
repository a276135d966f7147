"""Thin Python binding over libapb.so (argument marshalling only).

Every step of the APB layer forward pass runs in the HIP kernels of the library; PyTorch is
used for device memory and streams, nothing else.  There is no CPU fallback: if the library
is missing or cannot be loaded, importing this module's functions raises.

Function names and argument order follow include/apb.h.
"""
from __future__ import annotations

import ctypes
import math
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libapb.so")

EXPORTS = (
    "apb_compress", "apb_layer_info", "apb_layer_export", "apb_layer_free", "apb_acts_bytes",
    "apb_quantize_acts", "apb_forward", "apb_forward_kernel_name", "apb_quantize_forward", "apb_quantize_forward_static", "apb_quantize_forward_is_one_kernel", "apb_forward_requant", "apb_forward_conv3x3", "apb_forward_conv3x3_requant",
    "apb_forward_int", "apb_forward_int_popcount", "apb_forward_popcount",
    "apb_w2_pack", "apb_w2_export", "apb_w2_free", "apb_gemm_2_2_int", "apb_gemm_2_2",
    "apb_train_workspace_bytes", "apb_train_forward", "apb_train_backward",
    "apb_probe_out_bytes", "apb_probe_rate",
    "apb_strerror", "apb_last_hip_error",
)

APB_OK = 0
APB_ERR_NULL, APB_ERR_SHAPE, APB_ERR_BITS, APB_ERR_VALUE, APB_ERR_NOMEM, APB_ERR_HIP = -1, -2, -3, -4, -5, -6
APB_ERR_SCRATCH = -7
APB_STATIC_SCRATCH_BYTES = 32 << 20

_lib: Optional[ctypes.CDLL] = None


class ApbError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {strerror(code)} (status {code})")
        self.code = code


def load() -> ctypes.CDLL:
    """Load libapb.so; raises if it has not been built (python paper_2306_08960_amd/build.py)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python {os.path.join(_HERE, 'build.py')}` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    lib.apb_compress.argtypes = [vp, ci, ci, cf, cf, vp, ctypes.POINTER(vp)]
    lib.apb_compress.restype = ci
    lib.apb_layer_info.argtypes = [vp, ctypes.POINTER(ci), ctypes.POINTER(ci), ctypes.POINTER(cf),
                                   ctypes.POINTER(ctypes.c_longlong), ctypes.POINTER(ctypes.c_longlong)]
    lib.apb_layer_info.restype = ci
    lib.apb_layer_export.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    lib.apb_layer_export.restype = ci
    lib.apb_layer_free.argtypes = [vp]
    lib.apb_layer_free.restype = None
    lib.apb_acts_bytes.argtypes = [ci, ci, ci]
    lib.apb_acts_bytes.restype = ctypes.c_size_t
    lib.apb_quantize_acts.argtypes = [vp, ci, ci, ci, cf, vp, vp]
    lib.apb_quantize_acts.restype = ci
    lib.apb_forward.argtypes = [vp, vp, ci, ci, cf, vp, vp]
    lib.apb_forward.restype = ci
    lib.apb_quantize_forward.argtypes = [vp, vp, ci, ci, cf, vp, vp, vp]
    lib.apb_quantize_forward.restype = ci
    lib.apb_forward_kernel_name.argtypes = [vp, ci, ci]
    lib.apb_forward_kernel_name.restype = ctypes.c_char_p
    lib.apb_quantize_forward_static.argtypes = [vp, vp, ci, ci, cf, vp, vp]
    lib.apb_quantize_forward_static.restype = ci
    lib.apb_quantize_forward_is_one_kernel.argtypes = [vp, ci, ci]
    lib.apb_quantize_forward_is_one_kernel.restype = ci
    lib.apb_forward_requant.argtypes = [vp, vp, ci, ci, cf, vp, vp, ci, cf, vp, vp]
    lib.apb_forward_requant.restype = ci
    lib.apb_forward_conv3x3.argtypes = [vp, vp, ci, ci, ci, ci, ci, cf, vp, ctypes.c_size_t, vp, vp]
    lib.apb_forward_conv3x3.restype = ci
    lib.apb_forward_conv3x3_requant.argtypes = [vp, vp, ci, ci, ci, ci, ci, cf, vp, vp, ci, cf, vp, ctypes.c_size_t, vp, vp]
    lib.apb_forward_conv3x3_requant.restype = ci
    lib.apb_forward_int.argtypes = [vp, vp, ci, ci, vp, vp]
    lib.apb_forward_int.restype = ci
    lib.apb_forward_int_popcount.argtypes = [vp, vp, ci, ci, vp, vp]
    lib.apb_forward_int_popcount.restype = ci
    lib.apb_forward_popcount.argtypes = [vp, vp, ci, ci, cf, vp, vp]
    lib.apb_forward_popcount.restype = ci
    lib.apb_w2_pack.argtypes = [vp, ci, ci, cf, vp, ctypes.POINTER(vp)]
    lib.apb_w2_pack.restype = ci
    lib.apb_w2_export.argtypes = [vp, vp, vp]
    lib.apb_w2_export.restype = ci
    lib.apb_w2_free.argtypes = [vp]
    lib.apb_w2_free.restype = None
    lib.apb_gemm_2_2_int.argtypes = [vp, vp, ci, vp, vp]
    lib.apb_gemm_2_2_int.restype = ci
    lib.apb_gemm_2_2.argtypes = [vp, vp, ci, cf, vp, vp]
    lib.apb_gemm_2_2.restype = ci
    lib.apb_train_workspace_bytes.argtypes = []
    lib.apb_train_workspace_bytes.restype = ctypes.c_size_t
    lib.apb_train_forward.argtypes = [vp, ctypes.c_longlong, cf, cf, vp, vp]
    lib.apb_train_forward.restype = ci
    lib.apb_train_backward.argtypes = [vp, vp, ctypes.c_longlong, cf, cf, vp, vp, vp, vp, vp]
    lib.apb_train_backward.restype = ci
    lib.apb_probe_out_bytes.argtypes = []
    lib.apb_probe_out_bytes.restype = ctypes.c_size_t
    lib.apb_probe_rate.argtypes = [ci, ci, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.apb_probe_rate.restype = ci
    lib.apb_strerror.argtypes = [ci]
    lib.apb_strerror.restype = ctypes.c_char_p
    lib.apb_last_hip_error.argtypes = []
    lib.apb_last_hip_error.restype = ci
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load().apb_strerror(int(code)).decode()


def _check(code: int, what: str) -> None:
    if code != APB_OK:
        extra = f" [hipError {load().apb_last_hip_error()}]" if code == APB_ERR_HIP else ""
        raise ApbError(code, what + extra)


def _stream(stream: Optional[torch.cuda.Stream]) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _dev_ptr(t: torch.Tensor, dtype: torch.dtype, name: str) -> int:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous {dtype} tensor on the GPU")
    return t.data_ptr()


class ApbLayer:
    """Owner of one opaque apb_layer handle."""

    def __init__(self, handle: int):
        self._h = ctypes.c_void_p(handle)

    @property
    def handle(self) -> ctypes.c_void_p:
        if not self._h:
            raise RuntimeError("layer already freed")
        return self._h

    def info(self) -> dict:
        return apb_layer_info(self)

    def free(self) -> None:
        if self._h:
            load().apb_layer_free(self._h)
            self._h = ctypes.c_void_p(None)

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def apb_compress(W: torch.Tensor, delta: float, alpha: Optional[float] = None,
                 stream: Optional[torch.cuda.Stream] = None) -> ApbLayer:
    """W: [N,K] float32 on the GPU.  alpha=None asks the library for its default scale."""
    if W.dim() != 2:
        raise TypeError("W must be 2-D [N, K]")
    ptr = _dev_ptr(W, torch.float32, "W")
    N, K = W.shape
    out = ctypes.c_void_p(None)
    a = math.nan if alpha is None else float(alpha)
    _check(load().apb_compress(ptr, N, K, float(delta), a, _stream(stream), ctypes.byref(out)), "apb_compress")
    return ApbLayer(out.value)


def apb_layer_info(layer: ApbLayer) -> dict:
    N, K, a = ctypes.c_int(), ctypes.c_int(), ctypes.c_float()
    nnz, bits = ctypes.c_longlong(), ctypes.c_longlong()
    _check(load().apb_layer_info(layer.handle, ctypes.byref(N), ctypes.byref(K), ctypes.byref(a),
                                 ctypes.byref(nnz), ctypes.byref(bits)), "apb_layer_info")
    return {"N": N.value, "K": K.value, "alpha": a.value, "nnz": nnz.value, "mem_bits": bits.value}


def apb_layer_export(layer: ApbLayer, stream: Optional[torch.cuda.Stream] = None) -> dict:
    """Canonical representation as GPU tensors: sign_words uint32-as-int32 [N,Kw], CSR, rowsum."""
    i = apb_layer_info(layer)
    N, K, nnz = i["N"], i["K"], i["nnz"]
    Kw = (K + 31) // 32
    dev = torch.device("cuda", torch.cuda.current_device())
    sign = torch.empty((N, Kw), dtype=torch.int32, device=dev)
    row_ptr = torch.empty(N + 1, dtype=torch.int32, device=dev)
    col = torch.empty(max(nnz, 1), dtype=torch.int32, device=dev)
    val = torch.empty(max(nnz, 1), dtype=torch.float32, device=dev)
    rowsum = torch.empty(N, dtype=torch.int32, device=dev)
    _check(load().apb_layer_export(layer.handle, sign.data_ptr(), row_ptr.data_ptr(), col.data_ptr(),
                                   val.data_ptr(), rowsum.data_ptr(), _stream(stream)), "apb_layer_export")
    return {"sign_words": sign, "row_ptr": row_ptr, "col_idx": col[:nnz], "val": val[:nnz], "rowsum": rowsum,
            **i}


def apb_acts_bytes(K: int, M: int, bits: int) -> int:
    return int(load().apb_acts_bytes(int(K), int(M), int(bits)))


def alloc_packed(K: int, M: int, bits: int, device=None) -> torch.Tensor:
    nbytes = apb_acts_bytes(K, M, bits)
    if nbytes == 0:
        raise ApbError(APB_ERR_SHAPE if bits in (1, 2) else APB_ERR_BITS, "apb_acts_bytes")
    dev = device if device is not None else torch.device("cuda", torch.cuda.current_device())
    return torch.empty(nbytes // 4, dtype=torch.int32, device=dev)


def apb_quantize_acts(X: torch.Tensor, bits: int, step: float, packed: Optional[torch.Tensor] = None,
                      stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """X: [K,M] float32 on the GPU -> packed int32 buffer (planes + column sums)."""
    if X.dim() != 2:
        raise TypeError("X must be 2-D [K, M]")
    ptr = _dev_ptr(X, torch.float32, "X")
    K, M = X.shape
    if packed is None:
        packed = alloc_packed(K, M, bits, X.device)
    elif packed.numel() * packed.element_size() < apb_acts_bytes(K, M, bits):
        raise ValueError("packed buffer too small")
    _check(load().apb_quantize_acts(ptr, K, M, int(bits), float(step), _dev_ptr(packed, torch.int32, "packed"),
                                    _stream(stream)), "apb_quantize_acts")
    return packed


def _check_packed(layer: ApbLayer, packed: torch.Tensor, M: int, bits: int) -> Tuple[int, int]:
    i = apb_layer_info(layer)
    need = apb_acts_bytes(i["K"], M, bits)
    if need and packed.numel() * packed.element_size() < need:
        raise ValueError("packed buffer smaller than apb_acts_bytes(K, M, bits)")
    return i["N"], i["K"]


def apb_forward(layer: ApbLayer, packed: torch.Tensor, M: int, bits: int, step: float,
                Y: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    N, _ = _check_packed(layer, packed, M, bits)
    if Y is None:
        Y = torch.empty((N, M), dtype=torch.float32, device=packed.device)
    elif tuple(Y.shape) != (N, M):
        raise ValueError("Y must be [N, M]")
    _check(load().apb_forward(layer.handle, _dev_ptr(packed, torch.int32, "packed"), int(M), int(bits),
                              float(step), _dev_ptr(Y, torch.float32, "Y"), _stream(stream)), "apb_forward")
    return Y


def apb_quantize_forward(layer: ApbLayer, X: torch.Tensor, bits: int, step: float, packed: Optional[torch.Tensor] = None,
                         Y: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """apb_quantize_acts + apb_forward in one call; `packed` is scratch."""
    if X.dim() != 2:
        raise TypeError("X must be 2-D [K, M]")
    K, M = X.shape
    if packed is None:
        packed = alloc_packed(K, M, bits, X.device)
    N, _ = _check_packed(layer, packed, M, bits)
    if apb_layer_info(layer)["K"] != K:
        raise ValueError("X must have the layer's K rows")
    if Y is None:
        Y = torch.empty((N, M), dtype=torch.float32, device=X.device)
    elif tuple(Y.shape) != (N, M):
        raise ValueError("Y must be [N, M]")
    _check(load().apb_quantize_forward(layer.handle, _dev_ptr(X, torch.float32, "X"), int(M), int(bits), float(step),
                                       _dev_ptr(packed, torch.int32, "packed"), _dev_ptr(Y, torch.float32, "Y"),
                                       _stream(stream)), "apb_quantize_forward")
    return Y


def apb_forward_kernel_name(layer: ApbLayer, M: int, bits: int) -> str:
    return load().apb_forward_kernel_name(layer.handle, int(M), int(bits)).decode()


def apb_quantize_forward_static(layer: ApbLayer, X: torch.Tensor, bits: int, step: float, Y: torch.Tensor,
                                stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """apb_quantize_forward through the library's static scratch array; allocates nothing (Y is the caller's)."""
    if X.dim() != 2:
        raise TypeError("X must be 2-D [K, M]")
    K, M = X.shape
    i = apb_layer_info(layer)
    if i["K"] != K:
        raise ValueError("X must have the layer's K rows")
    if tuple(Y.shape) != (i["N"], M):
        raise ValueError("Y must be [N, M]")
    _check(load().apb_quantize_forward_static(layer.handle, _dev_ptr(X, torch.float32, "X"), int(M), int(bits),
                                              float(step), _dev_ptr(Y, torch.float32, "Y"), _stream(stream)),
           "apb_quantize_forward_static")
    return Y


def apb_quantize_forward_is_one_kernel(layer: ApbLayer, M: int, bits: int) -> bool:
    return bool(load().apb_quantize_forward_is_one_kernel(layer.handle, int(M), int(bits)))


def apb_forward_requant(layer: ApbLayer, packed: torch.Tensor, M: int, bits: int, step: float, bits_out: int,
                        step_out: float, scale: Optional[torch.Tensor] = None, shift: Optional[torch.Tensor] = None,
                        packed_out: Optional[torch.Tensor] = None,
                        stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """The layer's output, quantized for the next layer and packed (its K = this layer's N)."""
    N, _ = _check_packed(layer, packed, M, bits)
    if (scale is None) != (shift is None):
        raise ValueError("scale and shift go together")
    for name, t in (("scale", scale), ("shift", shift)):
        if t is not None and t.numel() != N:
            raise ValueError(f"{name} must hold N floats")
    if packed_out is None:
        packed_out = alloc_packed(N, M, bits_out, packed.device)
    elif packed_out.numel() * packed_out.element_size() < apb_acts_bytes(N, M, bits_out):
        raise ValueError("packed_out smaller than apb_acts_bytes(N, M, bits_out)")
    _check(load().apb_forward_requant(layer.handle, _dev_ptr(packed, torch.int32, "packed"), int(M), int(bits),
                                      float(step), None if scale is None else _dev_ptr(scale, torch.float32, "scale"),
                                      None if shift is None else _dev_ptr(shift, torch.float32, "shift"),
                                      int(bits_out), float(step_out), _dev_ptr(packed_out, torch.int32, "packed_out"),
                                      _stream(stream)), "apb_forward_requant")
    return packed_out


def _workspace(t: Optional[torch.Tensor]):
    """(pointer, bytes) of an optional scratch tensor."""
    if t is None:
        return None, 0
    return _dev_ptr(t, torch.int32, "workspace"), t.numel() * t.element_size()


def _check_fmap(layer: ApbLayer, fmap: torch.Tensor, B: int, H: int, W: int, bits: int, stride: int) -> Tuple[int, int]:
    """(N, output pixels B*Ho*Wo) after checking the size of the input map's buffer."""
    i = apb_layer_info(layer)
    if i["K"] % 9:
        raise ValueError("the layer's K is not 9 * C")
    if stride not in (1, 2):
        raise ValueError("stride must be 1 or 2")
    P = int(B) * int(H) * int(W)
    need = apb_acts_bytes(i["K"] // 9, P, bits)
    if need and fmap.numel() * fmap.element_size() < need:
        raise ValueError("fmap smaller than apb_acts_bytes(C, B*H*W, bits)")
    return i["N"], int(B) * ((int(H) - 1) // stride + 1) * ((int(W) - 1) // stride + 1)


def apb_forward_conv3x3(layer: ApbLayer, fmap: torch.Tensor, B: int, H: int, W: int, bits: int, step: float,
                        Y: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None,
                        stride: int = 1, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """3x3 convolution (padding 1) over a packed feature map [C, B*H*W]; Y is [N, B*Ho*Wo].  `workspace`: an
    optional int32 scratch tensor (see the header)."""
    N, P = _check_fmap(layer, fmap, B, H, W, bits, stride)
    if Y is None:
        Y = torch.empty((N, P), dtype=torch.float32, device=fmap.device)
    elif tuple(Y.shape) != (N, P):
        raise ValueError("Y must be [N, B*Ho*Wo]")
    _check(load().apb_forward_conv3x3(layer.handle, _dev_ptr(fmap, torch.int32, "fmap"), int(B), int(H), int(W), int(stride),
                                      int(bits), float(step), *_workspace(workspace), _dev_ptr(Y, torch.float32, "Y"),
                                      _stream(stream)),
           "apb_forward_conv3x3")
    return Y


def apb_forward_conv3x3_requant(layer: ApbLayer, fmap: torch.Tensor, B: int, H: int, W: int, bits: int, step: float,
                                bits_out: int, step_out: float, scale: Optional[torch.Tensor] = None,
                                shift: Optional[torch.Tensor] = None, fmap_out: Optional[torch.Tensor] = None,
                                stream: Optional[torch.cuda.Stream] = None, stride: int = 1,
                                workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    N, P = _check_fmap(layer, fmap, B, H, W, bits, stride)
    if (scale is None) != (shift is None):
        raise ValueError("scale and shift go together")
    for name, t in (("scale", scale), ("shift", shift)):
        if t is not None and t.numel() != N:
            raise ValueError(f"{name} must hold N floats")
    if fmap_out is None:
        fmap_out = alloc_packed(N, P, bits_out, fmap.device)
    elif fmap_out.numel() * fmap_out.element_size() < apb_acts_bytes(N, P, bits_out):
        raise ValueError("fmap_out smaller than apb_acts_bytes(N, B*Ho*Wo, bits_out)")
    _check(load().apb_forward_conv3x3_requant(
        layer.handle, _dev_ptr(fmap, torch.int32, "fmap"), int(B), int(H), int(W), int(stride), int(bits), float(step),
        None if scale is None else _dev_ptr(scale, torch.float32, "scale"),
        None if shift is None else _dev_ptr(shift, torch.float32, "shift"), int(bits_out), float(step_out),
        *_workspace(workspace), _dev_ptr(fmap_out, torch.int32, "fmap_out"), _stream(stream)), "apb_forward_conv3x3_requant")
    return fmap_out


def apb_forward_int(layer: ApbLayer, packed: torch.Tensor, M: int, bits: int,
                    D: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    N, _ = _check_packed(layer, packed, M, bits)
    if D is None:
        D = torch.empty((N, M), dtype=torch.int32, device=packed.device)
    elif tuple(D.shape) != (N, M):
        raise ValueError("D must be [N, M]")
    _check(load().apb_forward_int(layer.handle, _dev_ptr(packed, torch.int32, "packed"), int(M), int(bits),
                                  _dev_ptr(D, torch.int32, "D"), _stream(stream)), "apb_forward_int")
    return D


def apb_forward_int_popcount(layer: ApbLayer, packed: torch.Tensor, M: int, bits: int,
                             D: Optional[torch.Tensor] = None,
                             stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    N, _ = _check_packed(layer, packed, M, bits)
    if D is None:
        D = torch.empty((N, M), dtype=torch.int32, device=packed.device)
    elif tuple(D.shape) != (N, M):
        raise ValueError("D must be [N, M]")
    _check(load().apb_forward_int_popcount(layer.handle, _dev_ptr(packed, torch.int32, "packed"), int(M), int(bits),
                                           _dev_ptr(D, torch.int32, "D"), _stream(stream)),
           "apb_forward_int_popcount")
    return D


def apb_forward_popcount(layer: ApbLayer, packed: torch.Tensor, M: int, bits: int, step: float,
                         Y: Optional[torch.Tensor] = None,
                         stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    N, _ = _check_packed(layer, packed, M, bits)
    if Y is None:
        Y = torch.empty((N, M), dtype=torch.float32, device=packed.device)
    elif tuple(Y.shape) != (N, M):
        raise ValueError("Y must be [N, M]")
    _check(load().apb_forward_popcount(layer.handle, _dev_ptr(packed, torch.int32, "packed"), int(M), int(bits),
                                       float(step), _dev_ptr(Y, torch.float32, "Y"), _stream(stream)),
           "apb_forward_popcount")
    return Y


# ----------------------------------------------------------------------------- 2/2 routine

class ApbW2:
    """Owner of an apb_w2 handle (packed 2-bit weights)."""

    def __init__(self, handle: int, N: int, K: int):
        self._h = ctypes.c_void_p(handle)
        self.N, self.K = N, K

    @property
    def handle(self) -> ctypes.c_void_p:
        if not self._h:
            raise RuntimeError("weights already freed")
        return self._h

    def free(self) -> None:
        if self._h:
            load().apb_w2_free(self._h)
            self._h = ctypes.c_void_p(None)

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def apb_w2_pack(W: torch.Tensor, step_w: float, stream: Optional[torch.cuda.Stream] = None) -> ApbW2:
    if W.dim() != 2:
        raise ValueError("W must be [N, K]")
    ptr = _dev_ptr(W, torch.float32, "W")
    N, K = int(W.shape[0]), int(W.shape[1])
    out = ctypes.c_void_p(None)
    _check(load().apb_w2_pack(ptr, N, K, float(step_w), _stream(stream), ctypes.byref(out)), "apb_w2_pack")
    return ApbW2(out.value, N, K)


def apb_w2_export(w2: ApbW2, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """int32 view of the canonical planes, shape [2, N, ceil(K/32)]."""
    Kw = (w2.K + 31) // 32
    planes = torch.empty((2, w2.N, Kw), dtype=torch.int32, device="cuda")
    _check(load().apb_w2_export(w2.handle, planes.data_ptr(), _stream(stream)), "apb_w2_export")
    return planes


def _check_packed_w2(w2: ApbW2, packed: torch.Tensor, M: int) -> None:
    need = apb_acts_bytes(w2.K, M, 2)
    if need == 0:
        raise ValueError("bad K, M")
    if packed.numel() * packed.element_size() < need:
        raise ValueError("packed buffer smaller than apb_acts_bytes(K, M, 2)")


def apb_gemm_2_2_int(w2: ApbW2, packed: torch.Tensor, M: int, D: Optional[torch.Tensor] = None,
                     stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    _check_packed_w2(w2, packed, M)
    if D is None:
        D = torch.empty((w2.N, M), dtype=torch.int32, device=packed.device)
    elif tuple(D.shape) != (w2.N, M):
        raise ValueError("D must be [N, M]")
    _check(load().apb_gemm_2_2_int(w2.handle, _dev_ptr(packed, torch.int32, "packed"), int(M),
                                   _dev_ptr(D, torch.int32, "D"), _stream(stream)), "apb_gemm_2_2_int")
    return D


def apb_gemm_2_2(w2: ApbW2, packed: torch.Tensor, M: int, step_a: float, Y: Optional[torch.Tensor] = None,
                 stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    _check_packed_w2(w2, packed, M)
    if Y is None:
        Y = torch.empty((w2.N, M), dtype=torch.float32, device=packed.device)
    elif tuple(Y.shape) != (w2.N, M):
        raise ValueError("Y must be [N, M]")
    _check(load().apb_gemm_2_2(w2.handle, _dev_ptr(packed, torch.int32, "packed"), int(M), float(step_a),
                               _dev_ptr(Y, torch.float32, "Y"), _stream(stream)), "apb_gemm_2_2")
    return Y


# ----------------------------------------------------------------------------- instruction-rate probes

PROBES = {"mfma_fp4": 0, "mfma_i8": 1, "and_bcnt": 2, "fma_f64": 3, "lds_u8": 4, "lds_b128": 5, "mfma_fp4_lds": 6,
          "mfma_fp4_lds_barrier": 7, "mfma_fp4_lds_barrier_valu": 8}


def apb_probe_out_bytes() -> int:
    return int(load().apb_probe_out_bytes())


def apb_probe_rate(kind: int, iters: int, out: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> float:
    """Launch one probe; returns the work of the launch (flops or lane operations)."""
    if out.numel() * out.element_size() < apb_probe_out_bytes():
        raise ValueError("out smaller than apb_probe_out_bytes()")
    work = ctypes.c_double()
    _check(load().apb_probe_rate(int(kind), int(iters), out.data_ptr(), ctypes.byref(work), _stream(stream)),
           "apb_probe_rate")
    return work.value


# ----------------------------------------------------------------------------- training-side operators

def apb_train_workspace_bytes() -> int:
    return int(load().apb_train_workspace_bytes())


def apb_train_forward(W: torch.Tensor, alpha: float, delta: float, out: Optional[torch.Tensor] = None,
                      stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """APB(w) element-wise on the latent weights (any shape, contiguous float32)."""
    ptr = _dev_ptr(W, torch.float32, "W")
    if out is None:
        out = torch.empty_like(W)
    elif out.shape != W.shape:
        raise ValueError("out must have W's shape")
    _check(load().apb_train_forward(ptr, W.numel(), float(alpha), float(delta), _dev_ptr(out, torch.float32, "out"),
                                    _stream(stream)), "apb_train_forward")
    return out


def apb_train_backward(W: torch.Tensor, G: torch.Tensor, alpha: float, delta: float, want_grad_w: bool = True,
                       grad_w: Optional[torch.Tensor] = None, sums: Optional[torch.Tensor] = None,
                       count: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                       stream: Optional[torch.cuda.Stream] = None):
    """Returns (grad_w or None, sums [grad_alpha, grad_delta] float64 on the GPU, count int64 on the GPU)."""
    if W.shape != G.shape:
        raise ValueError("G must have W's shape")
    if want_grad_w and grad_w is None:
        grad_w = torch.empty_like(G)
    if sums is None:
        sums = torch.empty(2, dtype=torch.float64, device=W.device)
    if count is None:
        count = torch.empty(1, dtype=torch.int64, device=W.device)
    if workspace is None:
        workspace = torch.empty(apb_train_workspace_bytes() // 8, dtype=torch.float64, device=W.device)
    elif workspace.numel() * workspace.element_size() < apb_train_workspace_bytes():
        raise ValueError("workspace smaller than apb_train_workspace_bytes()")
    _check(load().apb_train_backward(_dev_ptr(W, torch.float32, "W"), _dev_ptr(G, torch.float32, "G"), W.numel(),
                                     float(alpha), float(delta),
                                     None if grad_w is None else _dev_ptr(grad_w, torch.float32, "grad_w"),
                                     sums.data_ptr(), count.data_ptr(), workspace.data_ptr(), _stream(stream)),
           "apb_train_backward")
    return grad_w, sums, count
