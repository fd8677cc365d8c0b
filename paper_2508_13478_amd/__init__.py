"""Python binding of libdhq (include/dhq.h): argument marshalling only.

Every function below has the name of the C entry point it forwards to; all
computation happens in the HIP library.  PyTorch supplies device memory and the
stream.  There is no CPU fallback: if libdhq.so is missing or does not load,
`lib()` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdhq.so")

DHQ_OK, DHQ_EINVAL, DHQ_EUNSUPPORTED, DHQ_ENOMEM, DHQ_EHIP, DHQ_ENOSCALE, DHQ_ETOOBIG = 0, -1, -2, -3, -4, -5, -6
DHQ_AUTO, DHQ_LAYERWISE, DHQ_FUSED = 0, 1, 2
DHQ_DYNAMIC = 4
DHQ_ROTATE_IN, DHQ_ROTATE_BOTH = 0, 1
DHQ_W8A8, DHQ_W8A32, DHQ_W32A32 = 0x00, 0x10, 0x20

# every symbol include/dhq.h declares
EXPORTS = ("dhq_quantize_weights", "dhq_quantize_weights_mode", "dhq_quantize_weights_wavelet", "dhq_quantize_weights_complex", "dhq_get_dynamic_scales", "dhq_set_act_scales", "dhq_calibrate", "dhq_get_scales",
           "dhq_get_weight_codes", "dhq_forward", "dhq_reserve_dynamic", "dhq_forward_noalloc", "dhq_noalloc_max_rows",
           "dhq_forward_debug", "dhq_forward_debug_fused", "dhq_gemm_i8", "dhq_has_fused", "dhq_select_wide_kernel",
           "dhq_free", "dhq_strerror", "dhq_version")


class dhq_net_desc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("dims", C.POINTER(C.c_int32)), ("omega0", C.c_float),
                ("bits_w", C.c_int32), ("bits_a", C.c_int32)]


class DhqError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {dhq_strerror(status)} ({status})")


_lib: Optional[C.CDLL] = None
_fpp = C.POINTER(C.POINTER(C.c_float))


def lib() -> C.CDLL:
    """Loads libdhq.so (building it first only if it has never been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _b
            _b.build(force=True)
        # PyTorch ships its own HIP runtime; load it first so that this library binds to the
        # same runtime instance as the tensors and streams it is handed
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(LIB_PATH)
        L.dhq_quantize_weights.argtypes = [C.POINTER(dhq_net_desc), _fpp, _fpp, C.POINTER(C.c_void_p)]
        L.dhq_quantize_weights_mode.argtypes = [C.POINTER(dhq_net_desc), C.c_uint32, _fpp, _fpp, C.POINTER(C.c_void_p)]
        L.dhq_quantize_weights_wavelet.argtypes = [C.POINTER(dhq_net_desc), C.c_uint32, C.c_float, _fpp, _fpp,
                                                   C.POINTER(C.c_void_p)]
        L.dhq_quantize_weights_complex.argtypes = [C.POINTER(dhq_net_desc), C.c_float, _fpp, _fpp, _fpp, _fpp, C.POINTER(C.c_void_p)]
        L.dhq_get_dynamic_scales.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.c_void_p]
        L.dhq_set_act_scales.argtypes = [C.c_void_p, C.POINTER(C.c_float)]
        L.dhq_calibrate.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.dhq_get_scales.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_float)]
        L.dhq_get_weight_codes.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int8)]
        L.dhq_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_uint32]
        L.dhq_reserve_dynamic.argtypes = [C.c_void_p, C.c_int64]
        L.dhq_forward_noalloc.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_uint32]
        L.dhq_noalloc_max_rows.argtypes = [C.c_void_p]
        L.dhq_noalloc_max_rows.restype = C.c_int64
        L.dhq_forward_debug.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_void_p]
        L.dhq_forward_debug_fused.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p]
        L.dhq_gemm_i8.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        L.dhq_has_fused.argtypes = [C.c_void_p]
        L.dhq_select_wide_kernel.argtypes = [C.c_void_p, C.c_int32]
        L.dhq_free.argtypes = [C.c_void_p]
        L.dhq_free.restype = None
        L.dhq_strerror.argtypes = [C.c_int]
        L.dhq_strerror.restype = C.c_char_p
        L.dhq_version.argtypes = []
        _lib = L
    return _lib


def _ok(rc: int, what: str) -> None:
    if rc != DHQ_OK:
        raise DhqError(rc, what)


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _dptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


# ------------------------------------------------------------------ C entry points, same names
def dhq_strerror(status: int) -> str:
    return lib().dhq_strerror(int(status)).decode()


def dhq_version() -> int:
    return lib().dhq_version()


def dhq_quantize_weights(dims: Sequence[int], omega0: float, bits_w: int, bits_a: int,
                         W: Sequence[np.ndarray], b: Sequence[np.ndarray]) -> int:
    """Returns the model handle (an integer address). W[l]: (dims[l+1], dims[l]) fp32 host arrays."""
    return dhq_quantize_weights_mode(dims, omega0, bits_w, bits_a, DHQ_ROTATE_IN, W, b)


def dhq_quantize_weights_mode(dims: Sequence[int], omega0: float, bits_w: int, bits_a: int, mode: int,
                              W: Sequence[np.ndarray], b: Sequence[np.ndarray]) -> int:
    return _quantize(dims, omega0, bits_w, bits_a, mode, None, W, b)


def dhq_quantize_weights_wavelet(dims: Sequence[int], omega0: float, bits_w: int, bits_a: int, mode: int, s0: float,
                                 W: Sequence[np.ndarray], b: Sequence[np.ndarray]) -> int:
    """A network whose hidden layers end in the wavelet cos(omega0 y) exp(-(s0 y)^2)."""
    return _quantize(dims, omega0, bits_w, bits_a, mode, float(s0), W, b)


def _quantize(dims, omega0, bits_w, bits_a, mode, s0, W, b) -> int:
    L = len(dims) - 1
    dims_a = (C.c_int32 * (L + 1))(*[int(d) for d in dims])
    desc = dhq_net_desc(L, dims_a, float(omega0), int(bits_w), int(bits_a))
    Wc = [np.ascontiguousarray(w, dtype=np.float32) for w in W]
    bc = [np.ascontiguousarray(x, dtype=np.float32) for x in b]
    for l in range(L):
        if Wc[l].shape != (dims[l + 1], dims[l]) or bc[l].shape != (dims[l + 1],):
            raise DhqError(DHQ_EINVAL, f"dhq_quantize_weights_mode: layer {l} has the wrong shape")
    Wp = (C.POINTER(C.c_float) * L)(*[w.ctypes.data_as(C.POINTER(C.c_float)) for w in Wc])
    bp = (C.POINTER(C.c_float) * L)(*[x.ctypes.data_as(C.POINTER(C.c_float)) for x in bc])
    h = C.c_void_p()
    if s0 is None:
        _ok(lib().dhq_quantize_weights_mode(C.byref(desc), int(mode), Wp, bp, C.byref(h)), "dhq_quantize_weights_mode")
    else:
        _ok(lib().dhq_quantize_weights_wavelet(C.byref(desc), int(mode), C.c_float(s0), Wp, bp, C.byref(h)),
            "dhq_quantize_weights_wavelet")
    return h.value


def dhq_quantize_weights_complex(dims_c: Sequence[int], omega0: float, bits_w: int, bits_a: int, s0: float,
                                 Wc: Sequence[np.ndarray], bc: Sequence[np.ndarray]) -> int:
    """A network with complex-valued hidden layers: Wc[l] complex, dims_c[l+1] x dims_c[l] (dims_c holds the
    complex widths of the hidden layers); the library runs it as a real network of interleaved (Re, Im) features."""
    L = len(dims_c) - 1
    dims_a = (C.c_int32 * (L + 1))(*[int(d) for d in dims_c])
    desc = dhq_net_desc(L, dims_a, float(omega0), int(bits_w), int(bits_a))
    parts = []
    for arrs, shape_of in ((Wc, lambda l: (dims_c[l + 1], dims_c[l])), (bc, lambda l: (dims_c[l + 1],))):
        for part in (np.real, np.imag):
            a = [np.ascontiguousarray(part(x), dtype=np.float32) for x in arrs]
            for l in range(L):
                if a[l].shape != tuple(shape_of(l)):
                    raise DhqError(DHQ_EINVAL, f"dhq_quantize_weights_complex: layer {l} has the wrong shape")
            parts.append(a)
    ptrs = [(C.POINTER(C.c_float) * L)(*[x.ctypes.data_as(C.POINTER(C.c_float)) for x in a]) for a in parts]
    h = C.c_void_p()
    _ok(lib().dhq_quantize_weights_complex(C.byref(desc), C.c_float(s0), ptrs[0], ptrs[1], ptrs[2], ptrs[3], C.byref(h)),
        "dhq_quantize_weights_complex")
    return h.value


def dhq_set_act_scales(model: int, s_a: Sequence[float]) -> None:
    a = np.ascontiguousarray(s_a, dtype=np.float32)
    _ok(lib().dhq_set_act_scales(model, a.ctypes.data_as(C.POINTER(C.c_float))), "dhq_set_act_scales")


def dhq_calibrate(model: int, coords, stream=None) -> None:
    _ok(lib().dhq_calibrate(model, _dptr(coords), coords.shape[0], _stream_ptr(stream)), "dhq_calibrate")


def dhq_get_scales(model: int, n_layers: int) -> Tuple[np.ndarray, np.ndarray]:
    sw = np.zeros(n_layers, dtype=np.float32)
    sa = np.zeros(n_layers, dtype=np.float32)
    _ok(lib().dhq_get_scales(model, sw.ctypes.data_as(C.POINTER(C.c_float)),
                             sa.ctypes.data_as(C.POINTER(C.c_float))), "dhq_get_scales")
    return sw, sa


def dhq_get_dynamic_scales(model: int, n_layers: int, stream=None) -> np.ndarray:
    sa = np.zeros(n_layers, dtype=np.float32)
    _ok(lib().dhq_get_dynamic_scales(model, sa.ctypes.data_as(C.POINTER(C.c_float)), _stream_ptr(stream)),
        "dhq_get_dynamic_scales")
    return sa


def dhq_get_weight_codes(model: int, layer: int, shape: Tuple[int, int]) -> np.ndarray:
    q = np.zeros(shape, dtype=np.int8)
    _ok(lib().dhq_get_weight_codes(model, layer, q.ctypes.data_as(C.POINTER(C.c_int8))), "dhq_get_weight_codes")
    return q


def dhq_forward(model: int, coords, out, stream=None, flags: int = DHQ_AUTO) -> None:
    """coords: (n, dims[0]) fp32 device tensor; out: (n, dims[-1]) fp32 device tensor."""
    _ok(lib().dhq_forward(model, _dptr(coords), coords.shape[0], _dptr(out), _stream_ptr(stream), flags),
        "dhq_forward")


def dhq_reserve_dynamic(model: int, n: int) -> None:
    _ok(lib().dhq_reserve_dynamic(model, int(n)), "dhq_reserve_dynamic")


def dhq_forward_noalloc(model: int, coords, out, stream=None, flags: int = DHQ_AUTO) -> None:
    """dhq_forward(..., flags | DHQ_DYNAMIC) on the library's fixed scratch buffer; allocates nothing."""
    _ok(lib().dhq_forward_noalloc(model, _dptr(coords), coords.shape[0], _dptr(out), _stream_ptr(stream), flags),
        "dhq_forward_noalloc")


def dhq_noalloc_max_rows(model: int) -> int:
    return int(lib().dhq_noalloc_max_rows(model))


def dhq_forward_debug(model: int, x, layer: int, codes=None, acc=None, act=None, stream=None) -> None:
    _ok(lib().dhq_forward_debug(model, _dptr(x), x.shape[0], layer, _dptr(codes), _dptr(acc), _dptr(act),
                                _stream_ptr(stream)), "dhq_forward_debug")


def dhq_forward_debug_fused(model: int, codes_in, layer: int, xhat=None, codes_out=None, acc=None, stream=None) -> None:
    _ok(lib().dhq_forward_debug_fused(model, _dptr(codes_in), codes_in.shape[0], layer, _dptr(xhat), _dptr(codes_out),
                                      _dptr(acc), _stream_ptr(stream)), "dhq_forward_debug_fused")


def dhq_gemm_i8(model: int, layer: int, codes, acc, stream=None) -> None:
    _ok(lib().dhq_gemm_i8(model, layer, _dptr(codes), codes.shape[0], _dptr(acc), _stream_ptr(stream)),
        "dhq_gemm_i8")


def dhq_has_fused(model: int) -> bool:
    rc = lib().dhq_has_fused(model)
    if rc < 0:
        raise DhqError(rc, "dhq_has_fused")
    return bool(rc)


def dhq_select_wide_kernel(model: int, which: int) -> None:
    _ok(lib().dhq_select_wide_kernel(model, int(which)), "dhq_select_wide_kernel")


def dhq_free(model: int) -> None:
    lib().dhq_free(model)


# ---------------------------------------------------------------------------- convenience
class Model:
    """Owns a dhq_model handle; methods forward to the functions above."""

    def __init__(self, dims: Sequence[int], omega0: float, W, b, bits_w: int = 8, bits_a: int = 8,
                 mode: int = DHQ_ROTATE_IN, wavelet_s0: Optional[float] = None):
        self.dims: List[int] = [int(d) for d in dims]
        self.n_layers = len(self.dims) - 1
        self.mode = int(mode)
        self.handle = _quantize(self.dims, omega0, bits_w, bits_a, mode, wavelet_s0, W, b)

    @classmethod
    def complex_wavelet(cls, dims_c: Sequence[int], omega0: float, Wc, bc, s0: float, bits_w: int = 8, bits_a: int = 8):
        """A network with complex-valued hidden layers (dims_c: their complex widths); the model has the real
        dims [fan-in, 2 x width, ..., fan-out]."""
        self = cls.__new__(cls)
        self.dims = [int(dims_c[0])] + [2 * int(d) for d in dims_c[1:-1]] + [int(dims_c[-1])]
        self.n_layers = len(self.dims) - 1
        self.mode = DHQ_ROTATE_IN
        self.handle = dhq_quantize_weights_complex(dims_c, omega0, bits_w, bits_a, s0, Wc, bc)
        return self

    def close(self) -> None:
        if getattr(self, "handle", None):
            dhq_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def kp(self, layer: int) -> int:
        k = self.dims[layer]
        return 1 << (k - 1).bit_length() if k > 1 else 1

    def mg(self, layer: int) -> int:
        """Rows of layer's code matrix = columns of its accumulators."""
        m = self.dims[layer + 1]
        if (self.mode & 0xF) == DHQ_ROTATE_BOTH:
            return 1 << (m - 1).bit_length() if m > 1 else 1
        return m

    def dynamic_scales(self, stream=None) -> np.ndarray:
        return dhq_get_dynamic_scales(self.handle, self.n_layers, stream)

    def set_act_scales(self, s_a) -> None:
        dhq_set_act_scales(self.handle, s_a)

    def calibrate(self, coords, stream=None) -> None:
        dhq_calibrate(self.handle, coords, stream)

    def scales(self):
        return dhq_get_scales(self.handle, self.n_layers)

    def weight_codes(self, layer: int) -> np.ndarray:
        return dhq_get_weight_codes(self.handle, layer, (self.mg(layer), self.kp(layer)))

    def has_fused(self) -> bool:
        return dhq_has_fused(self.handle)

    def select_wide_kernel(self, which: int) -> None:
        dhq_select_wide_kernel(self.handle, which)

    def forward(self, coords, out=None, flags: int = DHQ_AUTO, stream=None):
        import torch
        if out is None:
            out = torch.empty((coords.shape[0], self.dims[-1]), dtype=torch.float32, device=coords.device)
        dhq_forward(self.handle, coords, out, stream, flags)
        return out

    def forward_debug(self, x, layer: int, stream=None):
        import torch
        n = x.shape[0]
        codes = torch.empty((n, self.kp(layer)), dtype=torch.int8, device=x.device)
        acc = torch.empty((n, self.mg(layer)), dtype=torch.int32, device=x.device)
        act = torch.empty((n, self.dims[layer + 1]), dtype=torch.float32, device=x.device)
        dhq_forward_debug(self.handle, x, layer, codes, acc, act, stream)
        return codes, acc, act

    def forward_debug_fused(self, codes_in, layer: int, stream=None):
        import torch
        n, w = codes_in.shape[0], self.kp(layer + 1)
        xhat = torch.empty((n, w), dtype=torch.float32, device=codes_in.device)
        codes = torch.empty((n, w), dtype=torch.int8, device=codes_in.device)
        acc = torch.empty((n, self.mg(layer)), dtype=torch.int32, device=codes_in.device)
        dhq_forward_debug_fused(self.handle, codes_in, layer, xhat, codes, acc, stream)
        return xhat, codes, acc

    def gemm_i8(self, layer: int, codes, stream=None):
        import torch
        acc = torch.empty((codes.shape[0], self.mg(layer)), dtype=torch.int32, device=codes.device)
        dhq_gemm_i8(self.handle, layer, codes, acc, stream)
        return acc
