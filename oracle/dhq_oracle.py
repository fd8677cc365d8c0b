"""ctypes binding of the CPU oracle (oracle/dhq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU library never imports or calls this.
All arithmetic lives in the C file; this module only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dhq_oracle.c")
_LIB = os.path.join(_HERE, "libdhq_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (+OpenMP). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        _lib = C.CDLL(_LIB)
        _declare(_lib)
    return _lib


_dp = C.POINTER(C.c_double)
_fp = C.POINTER(C.c_float)
_i8p = C.POINTER(C.c_int8)
_i32p = C.POINTER(C.c_int32)


def _declare(L: C.CDLL) -> None:
    L.dhqo_next_pow2.argtypes = [C.c_int]
    L.dhqo_next_pow2.restype = C.c_int
    L.dhqo_qmax.argtypes = [C.c_int]
    L.dhqo_qmax.restype = C.c_int
    L.dhqo_hadamard.argtypes = [C.c_int, _dp]
    L.dhqo_rotate_rows.argtypes = [_dp, C.c_int64, C.c_int, _dp]
    L.dhqo_rotate_two_sided.argtypes = [_dp, C.c_int, C.c_int, _dp]
    L.dhqo_absmax_scale.argtypes = [_dp, C.c_int64, C.c_int]
    L.dhqo_absmax_scale.restype = C.c_float
    L.dhqo_quantize.argtypes = [_dp, C.c_int64, C.c_float, C.c_int, _i8p]
    L.dhqo_dequantize.argtypes = [_i8p, C.c_int64, C.c_float, _dp]
    L.dhqo_dequantize.restype = None
    L.dhqo_igemm.argtypes = [_i8p, _i8p, C.c_int64, C.c_int, C.c_int, _i32p]
    L.dhqo_activation.argtypes = [C.c_double, C.c_int, C.c_double, C.c_double]
    L.dhqo_activation.restype = C.c_double
    L.dhqo_activation_complex.argtypes = [C.c_double, C.c_double, C.c_double, C.c_double, _dp, _dp]
    L.dhqo_activation_complex.restype = None
    L.dhqo_complex_layer_to_real.argtypes = [_fp, _fp, _fp, _fp, C.c_int, C.c_int, C.c_int, C.c_int, _fp, _fp]
    L.dhqo_epilogue.argtypes = [_i32p, C.c_int64, C.c_int, C.c_float, C.c_float, _fp, C.c_int,
                                C.c_float, C.c_float, _fp]
    L.dhqo_quantize_weights.argtypes = [_fp, C.c_int, C.c_int, C.c_int, _i8p, _fp, _dp]
    L.dhqo_layer.argtypes = [_fp, C.c_int64, C.c_int, C.c_int, _i8p, C.c_float, _fp, _fp, C.c_int,
                             C.c_int, C.c_int, C.c_float, C.c_float, _fp, _dp, _i8p, _i32p]
    L.dhqo_forward.argtypes = [C.c_int, _i32p, C.c_int, C.c_float, C.c_float, C.c_int, C.POINTER(_i8p), _fp,
                               C.POINTER(_fp), _fp, C.c_int, _fp, C.c_int64, _fp,
                               C.POINTER(_dp), C.POINTER(_i8p), C.POINTER(_i32p), C.POINTER(_fp)]
    L.dhqo_quantize_weights_two_sided.argtypes = [_fp, C.c_int, C.c_int, C.c_int, _i8p, _fp, _dp]
    L.dhqo_unrotate_acc.argtypes = [_i32p, C.c_int64, C.c_int, _i32p]
    L.dhqo_layer_two_sided.argtypes = [_fp, C.c_int64, C.c_int, C.c_int, _i8p, C.c_float, _fp, _fp, C.c_int,
                                       C.c_int, C.c_int, C.c_float, C.c_float, _fp, _dp, _i8p, _i32p, _i32p]
    L.dhqo_forward_two_sided.argtypes = L.dhqo_forward.argtypes
    L.dhqo_dequantize_weights.argtypes = [_i8p, C.c_float, C.c_int, C.c_int, _fp]
    L.dhqo_mlp_float.argtypes = [C.c_int, _i32p, C.c_int, C.c_float, C.c_float, C.POINTER(_fp), C.POINTER(_fp), _fp,
                                 C.c_int64, _dp, _fp]
    L.dhqo_mlp_rotated_f64.argtypes = [C.c_int, _i32p, C.c_float, C.POINTER(_fp), C.POINTER(_fp),
                                       _fp, C.c_int64, _dp]


class OracleError(RuntimeError):
    pass


def _check(rc: int, what: str) -> None:
    if rc != 0:
        names = {-1: "invalid argument", -2: "out of memory", -3: "int32 accumulator overflow"}
        raise OracleError(f"{what}: {names.get(rc, rc)}")


def _c(a: np.ndarray, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _ptr(a: Optional[np.ndarray], ptype):
    return a.ctypes.data_as(ptype) if a is not None else ptype()


def next_pow2(k: int) -> int:
    return lib().dhqo_next_pow2(int(k))


def qmax(bits: int) -> int:
    return lib().dhqo_qmax(int(bits))


def hadamard(n: int) -> np.ndarray:
    H = np.empty((n, n), dtype=np.float64)
    _check(lib().dhqo_hadamard(n, _ptr(H, _dp)), "hadamard")
    return H


def rotate_rows(x: np.ndarray) -> np.ndarray:
    x = _c(np.atleast_2d(x), np.float64)
    rows, K = x.shape
    out = np.empty((rows, next_pow2(K)), dtype=np.float64)
    _check(lib().dhqo_rotate_rows(_ptr(x, _dp), rows, K, _ptr(out, _dp)), "rotate_rows")
    return out


def rotate_two_sided(W: np.ndarray) -> np.ndarray:
    W = _c(W, np.float64)
    m, n = W.shape
    out = np.empty_like(W)
    _check(lib().dhqo_rotate_two_sided(_ptr(W, _dp), m, n, _ptr(out, _dp)), "rotate_two_sided")
    return out


def absmax_scale(x: np.ndarray, bits: int) -> np.float32:
    x = _c(x, np.float64)
    return np.float32(lib().dhqo_absmax_scale(_ptr(x, _dp), x.size, bits))


def quantize(x: np.ndarray, s: float, bits: int) -> np.ndarray:
    x = _c(x, np.float64)
    q = np.empty(x.shape, dtype=np.int8)
    _check(lib().dhqo_quantize(_ptr(x, _dp), x.size, C.c_float(s), bits, _ptr(q, _i8p)), "quantize")
    return q


def dequantize(q: np.ndarray, s: float) -> np.ndarray:
    q = _c(q, np.int8)
    x = np.empty(q.shape, dtype=np.float64)
    lib().dhqo_dequantize(_ptr(q, _i8p), q.size, C.c_float(s), _ptr(x, _dp))
    return x


def igemm(q: np.ndarray, w: np.ndarray) -> np.ndarray:
    q = _c(q, np.int8)
    w = _c(w, np.int8)
    N, Kp = q.shape
    M, Kp2 = w.shape
    assert Kp == Kp2
    acc = np.empty((N, M), dtype=np.int32)
    _check(lib().dhqo_igemm(_ptr(q, _i8p), _ptr(w, _i8p), N, M, Kp, _ptr(acc, _i32p)), "igemm")
    return acc


ACT_NONE, ACT_SINE, ACT_GABOR, ACT_GABOR_COMPLEX = 0, 1, 2, 3


class ComplexSpread(float):
    """A wavelet spread s0 that also says: the layers are complex-valued (features interleaved
    as Re, Im; the activation is the complex Gabor wavelet on pairs).  Passed wherever a real
    wavelet's spread is passed as `gabor_s0`."""


def _act(apply_act: bool, gabor_s0: Optional[float]):
    """(activation code, spread) of a layer: none for the output layer, else the sine, or the
    wavelet cos(omega0 y) exp(-(s0 y)^2) when a spread s0 is given, or the complex wavelet on
    (Re, Im) pairs when the spread is a ComplexSpread."""
    if not apply_act:
        return ACT_NONE, 0.0
    if isinstance(gabor_s0, ComplexSpread):
        return ACT_GABOR_COMPLEX, float(gabor_s0)
    return (ACT_SINE, 0.0) if gabor_s0 is None else (ACT_GABOR, float(gabor_s0))


def activation_complex(y: np.ndarray, omega0: float, s0: float) -> np.ndarray:
    """The complex Gabor wavelet exp(j omega0 y - |s0 y|^2) of a complex array, in fp64."""
    y = np.asarray(y, dtype=np.complex128)
    out = np.empty(y.shape, dtype=np.complex128)
    f = lib().dhqo_activation_complex
    ar, ai = C.c_double(0), C.c_double(0)
    for idx, v in np.ndenumerate(y):
        f(float(v.real), float(v.imag), float(omega0), float(s0), C.byref(ar), C.byref(ai))
        out[idx] = complex(ar.value, ai.value)
    return out


def complex_net_to_real(dims_c: Sequence[int], Wc: Sequence[np.ndarray], bc: Sequence[np.ndarray]):
    """A network with complex weights (Wc[l] complex, dims_c[l+1] x dims_c[l]; real inputs, the real
    part of the last layer as output) as the real network of interleaved (Re, Im) features that
    computes the same thing.  Returns (dims, W, b) of that real network."""
    L = len(dims_c) - 1
    dims = [int(dims_c[0])] + [2 * int(d) for d in dims_c[1:-1]] + [int(dims_c[-1])]
    W, b = [], []
    for l in range(L):
        M, K = int(dims_c[l + 1]), int(dims_c[l])
        wre, wim = _c(np.real(Wc[l]), np.float32), _c(np.imag(Wc[l]), np.float32)
        bre, bim = _c(np.real(bc[l]), np.float32), _c(np.imag(bc[l]), np.float32)
        assert wre.shape == (M, K)
        in_c, out_c = int(l > 0), int(l < L - 1)
        Wl = np.empty((dims[l + 1], dims[l]), dtype=np.float32)
        bl = np.empty(dims[l + 1], dtype=np.float32)
        _check(lib().dhqo_complex_layer_to_real(_ptr(wre, _fp), _ptr(wim, _fp), _ptr(bre, _fp), _ptr(bim, _fp), M, K,
                                                in_c, out_c, _ptr(Wl, _fp), _ptr(bl, _fp)), "complex_layer_to_real")
        W.append(Wl)
        b.append(bl)
    return dims, W, b


def activation(y: np.ndarray, omega0: float, gabor_s0: Optional[float] = None) -> np.ndarray:
    """Elementwise activation in fp64: sin(omega0 y), or the wavelet if gabor_s0 is given."""
    act, s0 = _act(True, gabor_s0)
    y = np.asarray(y, dtype=np.float64)
    f = lib().dhqo_activation
    return np.array([f(float(v), act, float(omega0), s0) for v in y.ravel()]).reshape(y.shape)


def epilogue(acc: np.ndarray, s_a: float, s_w: float, b: np.ndarray, apply_sine: bool,
             omega0: float, gabor_s0: Optional[float] = None) -> np.ndarray:
    acc = _c(acc, np.int32)
    b = _c(b, np.float32)
    N, M = acc.shape
    out = np.empty((N, M), dtype=np.float32)
    _check(lib().dhqo_epilogue(_ptr(acc, _i32p), N, M, C.c_float(s_a), C.c_float(s_w),
                               _ptr(b, _fp), _act(apply_sine, gabor_s0)[0], C.c_float(omega0),
                               C.c_float(_act(apply_sine, gabor_s0)[1]), _ptr(out, _fp)),
           "epilogue")
    return out


def quantize_weights(W: np.ndarray, bits: int, want_rot: bool = False):
    """Rotate over the input dim, per-tensor scale, quantize. Returns (Wq, s_w[, rot])."""
    W = _c(W, np.float32)
    M, K = W.shape
    Kp = next_pow2(K)
    Wq = np.empty((M, Kp), dtype=np.int8)
    s = C.c_float(0)
    rot = np.empty((M, Kp), dtype=np.float64) if want_rot else None
    _check(lib().dhqo_quantize_weights(_ptr(W, _fp), M, K, bits, _ptr(Wq, _i8p), C.byref(s),
                                       _ptr(rot, _dp)), "quantize_weights")
    if want_rot:
        return Wq, np.float32(s.value), rot
    return Wq, np.float32(s.value)


def quantize_weights_two_sided(W: np.ndarray, bits: int, want_rot: bool = False):
    """Eq. 4-5 as printed: rotate over both sides (fan-out zero-padded to a power of two),
    per-tensor scale, quantize. Returns (Wq [Mp x Kp], s_w[, rot])."""
    W = _c(W, np.float32)
    M, K = W.shape
    Kp, Mp = next_pow2(K), next_pow2(M)
    Wq = np.empty((Mp, Kp), dtype=np.int8)
    s = C.c_float(0)
    rot = np.empty((Mp, Kp), dtype=np.float64) if want_rot else None
    _check(lib().dhqo_quantize_weights_two_sided(_ptr(W, _fp), M, K, bits, _ptr(Wq, _i8p), C.byref(s),
                                                 _ptr(rot, _dp)), "quantize_weights_two_sided")
    if want_rot:
        return Wq, np.float32(s.value), rot
    return Wq, np.float32(s.value)


def unrotate_acc(acc: np.ndarray) -> np.ndarray:
    """z = acc H_Mp on int32 rows (exact; raises on int32 overflow)."""
    acc = _c(acc, np.int32)
    N, Mp = acc.shape
    z = np.empty_like(acc)
    _check(lib().dhqo_unrotate_acc(_ptr(acc, _i32p), N, Mp, _ptr(z, _i32p)), "unrotate_acc")
    return z


@dataclass
class QuantizedNet:
    dims: List[int]
    omega0: float
    bits_w: int
    bits_a: int
    Wq: List[np.ndarray]
    s_w: np.ndarray
    bias: List[np.ndarray]
    s_a: Optional[np.ndarray] = None
    two_sided: bool = False
    gabor_s0: Optional[float] = None  # None: sine layers; a number: wavelet layers with that spread


@dataclass
class ForwardDump:
    rot: List[np.ndarray] = field(default_factory=list)
    codes: List[np.ndarray] = field(default_factory=list)
    acc: List[np.ndarray] = field(default_factory=list)
    act: List[np.ndarray] = field(default_factory=list)


def quantize_net(dims: Sequence[int], omega0: float, bits_w: int, bits_a: int,
                 W: Sequence[np.ndarray], bias: Sequence[np.ndarray], two_sided: bool = False,
                 gabor_s0: Optional[float] = None) -> QuantizedNet:
    Wq, s_w = [], []
    for Wl in W:
        q, s = (quantize_weights_two_sided if two_sided else quantize_weights)(Wl, bits_w)
        Wq.append(q)
        s_w.append(s)
    return QuantizedNet(list(dims), float(omega0), bits_w, bits_a, Wq,
                        np.asarray(s_w, dtype=np.float32),
                        [_c(b, np.float32) for b in bias], None, two_sided, gabor_s0)


def forward(net: QuantizedNet, coords: np.ndarray, calibrate: bool = False, dump: bool = False):
    """Quantized forward. With calibrate=True the per-layer activation scales are
    measured (sequentially, per tensor) and stored in net.s_a. Returns out or (out, dump)."""
    L = len(net.dims) - 1
    coords = _c(coords, np.float32)
    N = coords.shape[0]
    assert coords.shape[1] == net.dims[0]
    dimsa = np.asarray(net.dims, dtype=np.int32)
    if calibrate:
        s_a = np.zeros(L, dtype=np.float32)
    else:
        if net.s_a is None:
            raise OracleError("forward: activation scales not set")
        s_a = _c(net.s_a, np.float32).copy()
    out = np.empty((N, net.dims[-1]), dtype=np.float32)
    Wq_p = (_i8p * L)(*[_ptr(w, _i8p) for w in net.Wq])
    b_p = (_fp * L)(*[_ptr(b, _fp) for b in net.bias])
    d = ForwardDump()
    rot_p = cod_p = acc_p = act_p = None
    if dump:
        for l in range(L):
            Kp = next_pow2(net.dims[l])
            d.rot.append(np.empty((N, Kp), dtype=np.float64))
            d.codes.append(np.empty((N, Kp), dtype=np.int8))
            Mo = next_pow2(net.dims[l + 1]) if net.two_sided else net.dims[l + 1]
            d.acc.append(np.empty((N, Mo), dtype=np.int32))
            d.act.append(np.empty((N, net.dims[l + 1]), dtype=np.float32))
        rot_p = (_dp * L)(*[_ptr(a, _dp) for a in d.rot])
        cod_p = (_i8p * L)(*[_ptr(a, _i8p) for a in d.codes])
        acc_p = (_i32p * L)(*[_ptr(a, _i32p) for a in d.acc])
        act_p = (_fp * L)(*[_ptr(a, _fp) for a in d.act])
    fwd = lib().dhqo_forward_two_sided if net.two_sided else lib().dhqo_forward
    act, s0 = _act(True, net.gabor_s0)
    rc = fwd(L, _ptr(dimsa, _i32p), act, C.c_float(net.omega0), C.c_float(s0), net.bits_a, Wq_p,
            _ptr(net.s_w, _fp), b_p, _ptr(s_a, _fp), int(calibrate),
            _ptr(coords, _fp), N, _ptr(out, _fp), rot_p, cod_p, acc_p, act_p)
    _check(rc, "forward")
    if calibrate:
        net.s_a = s_a
    return (out, d) if dump else out


def layer(a_in: np.ndarray, Wq: np.ndarray, s_w: float, bias: np.ndarray, s_a: Optional[float],
          bits_a: int, apply_sine: bool, omega0: float, gabor_s0: Optional[float] = None):
    """One quantized layer. s_a=None measures the scale on this input.
    Returns dict(rot, codes, acc, act, s_a)."""
    a_in = _c(a_in, np.float32)
    N, K = a_in.shape
    M, Kp = Wq.shape
    assert Kp == next_pow2(K)
    Wq = _c(Wq, np.int8)
    bias = _c(bias, np.float32)
    rot = np.empty((N, Kp), dtype=np.float64)
    codes = np.empty((N, Kp), dtype=np.int8)
    acc = np.empty((N, M), dtype=np.int32)
    out = np.empty((N, M), dtype=np.float32)
    s = C.c_float(0.0 if s_a is None else s_a)
    rc = lib().dhqo_layer(_ptr(a_in, _fp), N, K, M, _ptr(Wq, _i8p), C.c_float(s_w), _ptr(bias, _fp),
                          C.byref(s), int(s_a is None), bits_a, _act(apply_sine, gabor_s0)[0], C.c_float(omega0),
                          C.c_float(_act(apply_sine, gabor_s0)[1]),
                          _ptr(out, _fp), _ptr(rot, _dp), _ptr(codes, _i8p), _ptr(acc, _i32p))
    _check(rc, "layer")
    return dict(rot=rot, codes=codes, acc=acc, act=out, s_a=np.float32(s.value))


def layer_two_sided(a_in: np.ndarray, M: int, Wq: np.ndarray, s_w: float, bias: np.ndarray,
                    s_a: Optional[float], bits_a: int, apply_sine: bool, omega0: float,
                    gabor_s0: Optional[float] = None):
    """One two-sided layer (Wq is Mp x Kp, M outputs kept). s_a=None measures the scale.
    Returns dict(rot, codes, acc [N x Mp, rotated], unrot [N x Mp], act [N x M], s_a)."""
    a_in = _c(a_in, np.float32)
    N, K = a_in.shape
    Mp, Kp = Wq.shape
    assert Kp == next_pow2(K) and Mp == next_pow2(M)
    Wq = _c(Wq, np.int8)
    bias = _c(bias, np.float32)
    rot = np.empty((N, Kp), dtype=np.float64)
    codes = np.empty((N, Kp), dtype=np.int8)
    acc = np.empty((N, Mp), dtype=np.int32)
    unrot = np.empty((N, Mp), dtype=np.int32)
    out = np.empty((N, M), dtype=np.float32)
    s = C.c_float(0.0 if s_a is None else s_a)
    rc = lib().dhqo_layer_two_sided(_ptr(a_in, _fp), N, K, M, _ptr(Wq, _i8p), C.c_float(s_w), _ptr(bias, _fp),
                                    C.byref(s), int(s_a is None), bits_a, _act(apply_sine, gabor_s0)[0],
                                    C.c_float(omega0), C.c_float(_act(apply_sine, gabor_s0)[1]), _ptr(out, _fp), _ptr(rot, _dp), _ptr(codes, _i8p), _ptr(acc, _i32p),
                                    _ptr(unrot, _i32p))
    _check(rc, "layer_two_sided")
    return dict(rot=rot, codes=codes, acc=acc, unrot=unrot, act=out, s_a=np.float32(s.value))


def dequantize_weights(Wq: np.ndarray, s_w: float, K: int) -> np.ndarray:
    """W~ = (s_w Wq) Hn, first K columns, fp32: the weights a weight-only-quantized network uses."""
    Wq = _c(Wq, np.int8)
    M = Wq.shape[0]
    assert Wq.shape[1] == next_pow2(K)
    Wt = np.empty((M, K), dtype=np.float32)
    _check(lib().dhqo_dequantize_weights(_ptr(Wq, _i8p), C.c_float(s_w), M, K, _ptr(Wt, _fp)), "dequantize_weights")
    return Wt


def mlp_w8a32(dims: Sequence[int], omega0: float, bits_w: int, W: Sequence[np.ndarray],
              bias: Sequence[np.ndarray], coords: np.ndarray, gabor_s0: Optional[float] = None):
    """Weight-only quantization: the plain MLP on the de-quantized weights. Returns (out_fp64, out_fp32, W~)."""
    Wt = []
    for l, Wl in enumerate(W):
        q, s = quantize_weights(Wl, bits_w)
        Wt.append(dequantize_weights(q, s, dims[l]))
    o64, o32 = mlp_float(dims, omega0, Wt, bias, coords, gabor_s0=gabor_s0)
    return o64, o32, Wt


def mlp_float(dims: Sequence[int], omega0: float, W: Sequence[np.ndarray],
              bias: Sequence[np.ndarray], coords: np.ndarray, want_f32: bool = True,
              gabor_s0: Optional[float] = None):
    """Plain un-rotated, un-quantized MLP: returns (out_fp64, out_fp32 or None)."""
    L = len(dims) - 1
    Wc = [_c(w, np.float32) for w in W]
    bc = [_c(b, np.float32) for b in bias]
    coords = _c(coords, np.float32)
    N = coords.shape[0]
    dimsa = np.asarray(dims, dtype=np.int32)
    o64 = np.empty((N, dims[-1]), dtype=np.float64)
    o32 = np.empty((N, dims[-1]), dtype=np.float32) if want_f32 else None
    W_p = (_fp * L)(*[_ptr(w, _fp) for w in Wc])
    b_p = (_fp * L)(*[_ptr(b, _fp) for b in bc])
    act, s0 = _act(True, gabor_s0)
    _check(lib().dhqo_mlp_float(L, _ptr(dimsa, _i32p), act, C.c_float(omega0), C.c_float(s0), W_p, b_p,
                                _ptr(coords, _fp), N, _ptr(o64, _dp), _ptr(o32, _fp)), "mlp_float")
    return o64, o32


def mlp_rotated_f64(dims: Sequence[int], omega0: float, W: Sequence[np.ndarray],
                    bias: Sequence[np.ndarray], coords: np.ndarray) -> np.ndarray:
    """Rotation on, quantizer off (fp64)."""
    L = len(dims) - 1
    Wc = [_c(w, np.float32) for w in W]
    bc = [_c(b, np.float32) for b in bias]
    coords = _c(coords, np.float32)
    N = coords.shape[0]
    dimsa = np.asarray(dims, dtype=np.int32)
    o64 = np.empty((N, dims[-1]), dtype=np.float64)
    W_p = (_fp * L)(*[_ptr(w, _fp) for w in Wc])
    b_p = (_fp * L)(*[_ptr(b, _fp) for b in bc])
    _check(lib().dhqo_mlp_rotated_f64(L, _ptr(dimsa, _i32p), C.c_float(omega0), W_p, b_p,
                                      _ptr(coords, _fp), N, _ptr(o64, _dp)), "mlp_rotated_f64")
    return o64
