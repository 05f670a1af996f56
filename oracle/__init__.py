"""CPU oracle for the binarized convolution / GEMM path.  TEST INFRASTRUCTURE.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package; the product path never does, and this
package imports nothing from the product.

The arithmetic lives in ``oracle.c`` (plain loops on -1/+1 float values: the
Gemm-Accumulation of section 3.2 and the direct convolution of section 2.1).
What is written here in numpy is only the *encoding* of section 3.1 (value -1 <->
bit 0, value +1 <-> bit 1) laid out in the library's packed format, so that the
outputs of the encode / im2col entry points can be compared word for word:
element k of a row sits in bit (k mod 64), least-significant bit first, of 64-bit
word (k div 64); padding bits are 0.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

from . import build as _build

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if os.environ.get("ORACLE_SANITIZE") == "1":
            # the ASan / UBSan build of the same source (the process must preload libasan)
            path = _build.build_sanitized()
        else:
            path = _build.LIB
            if not os.path.exists(path):
                _build.build()
        L = ctypes.CDLL(path)
        i64, p, i32 = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        L.oracle_sign.restype = ctypes.c_float
        L.oracle_sign.argtypes = [ctypes.c_float]
        L.oracle_sign_array.argtypes = [p, i64, p]
        L.oracle_gemm_pm1.argtypes = [p, p, i64, i64, i64, p]
        L.oracle_conv2d_pm1.argtypes = [p, p] + [i64] * 11 + [p]
        L.oracle_conv2d_pm1_at.argtypes = [p, p] + [i64] * 11 + [p, i64, p]
        L.oracle_scale_bias.argtypes = [p, i64, i64, p, p, i32, i64, p]
        L.oracle_maxpool2x2_i32.argtypes = [p, i64, i64, i64, p]
        L.oracle_conv2d_f32_seq.argtypes = [p, p] + [i64] * 11 + [p, p, p]
        L.oracle_fc_f32_seq.argtypes = [p, p, p, i64, i64, i64, i32, p]
        L.oracle_num_threads.restype = i32
        for name in ("oracle_sign_array", "oracle_gemm_pm1", "oracle_conv2d_pm1", "oracle_conv2d_pm1_at",
                     "oracle_scale_bias", "oracle_maxpool2x2_i32", "oracle_conv2d_f32_seq",
                     "oracle_fc_f32_seq"):
            getattr(L, name).restype = None
        _lib = L
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


# ----------------------------------------------------------------------------
# Definitions on binary values (C).
# ----------------------------------------------------------------------------
def sign(x) -> np.ndarray:
    """Sign(x) of section 4.2 with predicate x >= 0 -> +1.0, else -1.0 (NaN -> -1)."""
    x = _f32(x)
    s = np.empty_like(x)
    lib().oracle_sign_array(_ptr(x), x.size, _ptr(s))
    return s


def gemm_pm1(A, B) -> np.ndarray:
    """C[m,n] = sum_k s(A[m,k]) s(B[n,k]); A [M,K], B [N,K] fp32 -> int32 [M,N]
    (section 3.2, Gemm-Accumulation on binary values)."""
    A, B = _f32(A), _f32(B)
    assert A.ndim == 2 and B.ndim == 2 and A.shape[1] == B.shape[1]
    # the sum of K terms +-1 is accumulated in fp32, which holds every integer only below 2^24
    if A.shape[1] >= 1 << 24:
        raise ValueError("gemm_pm1: K >= 2^24 is outside the range in which the fp32 sum is exact")
    C = np.empty((A.shape[0], B.shape[0]), dtype=np.int32)
    lib().oracle_gemm_pm1(_ptr(A), _ptr(B), A.shape[0], B.shape[0], A.shape[1], _ptr(C))
    return C


def conv_out_hw(H, W, kH, kW, sH, sW, pH, pW):
    return (H + 2 * pH - kH) // sH + 1, (W + 2 * pW - kW) // sW + 1


def conv2d_pm1(x, w, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    """Direct convolution of section 2.1 on binary values; x NCHW fp32, w [D,C,kH,kW]
    fp32, zero padding applied before the sign (pad taps are +1) -> int32 NCHW."""
    x, w = _f32(x), _f32(w)
    if w[0].size >= 1 << 24:
        raise ValueError("conv2d_pm1: C*kH*kW >= 2^24 is outside the range in which the fp32 sum is exact")
    N, C, H, W = x.shape
    D, C2, kH, kW = w.shape
    assert C == C2
    OH, OW = conv_out_hw(H, W, kH, kW, *stride, *pad)
    out = np.empty((N, D, OH, OW), dtype=np.int32)
    lib().oracle_conv2d_pm1(_ptr(x), _ptr(w), N, C, H, W, D, kH, kW, stride[0], stride[1], pad[0], pad[1],
                            _ptr(out))
    return out


def conv2d_pm1_at(x, w, flat_idx, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    """conv2d_pm1 evaluated only at the given flat indices of the NCHW output."""
    x, w = _f32(x), _f32(w)
    if w[0].size >= 1 << 24:
        raise ValueError("conv2d_pm1: C*kH*kW >= 2^24 is outside the range in which the fp32 sum is exact")
    N, C, H, W = x.shape
    D, C2, kH, kW = w.shape
    assert C == C2
    idx = np.ascontiguousarray(flat_idx, dtype=np.int64)
    out = np.empty(idx.shape, dtype=np.int32)
    lib().oracle_conv2d_pm1_at(_ptr(x), _ptr(w), N, C, H, W, D, kH, kW, stride[0], stride[1], pad[0], pad[1],
                               _ptr(idx), idx.size, _ptr(out))
    return out


def scale_bias(acc, scale, bias, axis: str) -> np.ndarray:
    """y = fma(scale[ch], float(acc), bias[ch]), one rounding.
    axis 'row' / 'col' for a 2-D acc; 'nchw' for a 4-D acc with ch = dim 1."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    scale, bias = _f32(scale), _f32(bias)
    y = np.empty(acc.shape, dtype=np.float32)
    if axis == "nchw":
        N, D, OH, OW = acc.shape
        assert scale.size == D and bias.size == D
        lib().oracle_scale_bias(_ptr(acc), N * D, OH * OW, _ptr(scale), _ptr(bias), 1, D, _ptr(y))
    elif axis == "row":
        assert scale.size == acc.shape[0]
        lib().oracle_scale_bias(_ptr(acc), acc.shape[0], acc.shape[1], _ptr(scale), _ptr(bias), 1, 0, _ptr(y))
    elif axis == "col":
        assert scale.size == acc.shape[1]
        lib().oracle_scale_bias(_ptr(acc), acc.shape[0], acc.shape[1], _ptr(scale), _ptr(bias), 2, 0, _ptr(y))
    else:
        raise ValueError(axis)
    return y


def maxpool2x2_i32(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.int32)
    N, C, H, W = a.shape
    out = np.empty((N, C, H // 2, W // 2), dtype=np.int32)
    lib().oracle_maxpool2x2_i32(_ptr(a), N * C, H, W, _ptr(out))
    return out


def conv2d_f32_seq(x, w, stride=(1, 1), pad=(0, 0), scale=None, bias=None) -> np.ndarray:
    """fp32 convolution, sequential fma order (c, kh, kw), optional fma(scale, acc, bias)."""
    x, w = _f32(x), _f32(w)
    N, C, H, W = x.shape
    D, C2, kH, kW = w.shape
    assert C == C2 and (scale is None) == (bias is None)
    if scale is not None:
        scale, bias = _f32(scale), _f32(bias)
    OH, OW = conv_out_hw(H, W, kH, kW, *stride, *pad)
    out = np.empty((N, D, OH, OW), dtype=np.float32)
    lib().oracle_conv2d_f32_seq(_ptr(x), _ptr(w), N, C, H, W, D, kH, kW, stride[0], stride[1], pad[0], pad[1],
                                _ptr(scale), _ptr(bias), _ptr(out))
    return out


def fc_f32_seq(x, w, bias=None, sign_input: bool = False) -> np.ndarray:
    """out[m,n] = (sequential fma over k of x[m,k]*w[n,k]) + bias[n]."""
    x, w = _f32(x), _f32(w)
    if bias is not None:
        bias = _f32(bias)
    M, K = x.shape
    N, K2 = w.shape
    assert K == K2
    out = np.empty((M, N), dtype=np.float32)
    lib().oracle_fc_f32_seq(_ptr(x), _ptr(w), _ptr(bias), M, K, N, int(sign_input), _ptr(out))
    return out


# ----------------------------------------------------------------------------
# Encoding of section 3.1 in the packed layout (numpy; no arithmetic of the method).
# ----------------------------------------------------------------------------
def packed_words(K: int) -> int:
    return (K + 63) // 64


def encode_rows(x) -> np.ndarray:
    """fp32 [rows, K] -> uint64 [rows, ceil(K/64)]; bit = 1 iff value is +1."""
    s = sign(x)
    rows, K = s.shape
    Kw = packed_words(K)
    bits = np.zeros((rows, Kw * 64), dtype=np.uint8)
    bits[:, :K] = s > 0
    return np.packbits(bits, axis=1, bitorder="little").view("<u8").reshape(rows, Kw)


def decode_rows(words, K: int) -> np.ndarray:
    """uint64 [rows, Kw] -> float +-1 [rows, K] (inverse of encode_rows on the first K bits)."""
    w = np.ascontiguousarray(words, dtype="<u8")
    bits = np.unpackbits(w.view(np.uint8).reshape(w.shape[0], -1), axis=1, bitorder="little")[:, :K]
    return bits.astype(np.float32) * 2.0 - 1.0


def conv_kwords(C: int, kH: int, kW: int) -> int:
    """Words per packed patch: each of the kH*kW taps holds its C channels in
    ceil(C/64) words of its own (pad bits 0)."""
    return kH * kW * packed_words(C)


def pack_conv_weight(w) -> np.ndarray:
    """[D,C,kH,kW] fp32 -> uint64 [D, kH*kW*ceil(C/64)], reduction axis ordered
    (kh, kw, c) with c innermost, each tap padded to whole words."""
    w = _f32(w)
    D, C, kH, kW = w.shape
    taps = np.transpose(w, (0, 2, 3, 1)).reshape(D * kH * kW, C)  # rows = (d, kh, kw)
    return encode_rows(taps).reshape(D, kH * kW * packed_words(C))


def im2col_packed(x, kH, kW, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    """NCHW fp32 -> uint64 [N*OH*OW, kH*kW*ceil(C/64)]: zero-pad the fp32 image,
    take signs (pads become +1), gather each output pixel's patch in (kh, kw, c)
    order, encode each tap's channel run into whole words."""
    x = _f32(x)
    N, C, H, W = x.shape
    sH, sW = stride
    pH, pW = pad
    OH, OW = conv_out_hw(H, W, kH, kW, sH, sW, pH, pW)
    xp = np.zeros((N, C, H + 2 * pH, W + 2 * pW), dtype=np.float32)
    xp[:, :, pH:pH + H, pW:pW + W] = x
    Cw = packed_words(C)
    cols = np.empty((N, OH, OW, kH * kW, Cw), dtype="<u8")
    for kh in range(kH):
        for kw in range(kW):
            tap = xp[:, :, kh:kh + sH * (OH - 1) + 1:sH, kw:kw + sW * (OW - 1) + 1:sW]  # [N,C,OH,OW]
            rows = np.transpose(tap, (0, 2, 3, 1)).reshape(N * OH * OW, C)
            cols[:, :, :, kh * kW + kw, :] = encode_rows(rows).reshape(N, OH, OW, Cw)
    return cols.reshape(N * OH * OW, kH * kW * Cw)


def pack_nhwc(y) -> np.ndarray:
    """fp32 NCHW map -> packed NHWC image uint64 [N, H, W, ceil(C/64)]: bit c of a pixel is
    1 iff y[n, c, h, w] >= 0 (the encoding of section 3.1 applied along the channel axis)."""
    y = _f32(y)
    N, C, H, W = y.shape
    rows = np.transpose(y, (0, 2, 3, 1)).reshape(N * H * W, C)
    return encode_rows(rows).reshape(N, H, W, packed_words(C))


def pack_fc_weight_nhwc(w, C: int, H: int, W: int) -> np.ndarray:
    """[Nout, C*H*W] fp32 (NCHW flatten order) -> uint64 [Nout, H*W*ceil(C/64)] with the
    reduction axis re-ordered to (h, w, c) and every pixel padded to whole words."""
    w = _f32(w)
    n_out = w.shape[0]
    assert w.shape[1] == C * H * W
    rows = np.transpose(w.reshape(n_out, C, H * W), (0, 2, 1)).reshape(n_out * H * W, C)
    return encode_rows(rows).reshape(n_out, H * W * packed_words(C))


# ----------------------------------------------------------------------------
# The VGG-small stack as a composition of the definitions above.
# Block order: conv -> int32 -> (2x2 max-pool on int32 if pooled) -> fma(scale, acc,
# bias) -> sign taken by the next binarized layer.  Flatten order is NCHW.
# Pinned (tests/test_oracle_pins.py) on a five-layer table with small-integer data
# against a float64 composition of torch CPU routines (conv2d on +-1 tensors padded
# with +1, max_pool2d, affine, NCHW reshape, x >= 0), which is exact there; the case
# fails for affine-before-pool (negative scales), an NHWC flatten or a missing sign
# before the classifier.
# ----------------------------------------------------------------------------
def vgg_stack(x, layers: Sequence, params: Sequence[Dict[str, np.ndarray]]) -> Dict[str, object]:
    acts: List[np.ndarray] = []
    h = _f32(x)
    for L, p in zip(layers, params):
        if L.kind == "conv_f32":
            h = conv2d_f32_seq(h, p["w"], (1, 1), (1, 1), p["scale"], p["bias"])
        elif L.kind == "bconv":
            acc = conv2d_pm1(h, p["w"], (1, 1), (1, 1))
            if L.pool:
                acc = maxpool2x2_i32(acc)
            h = scale_bias(acc, p["scale"], p["bias"], "nchw")
        elif L.kind == "bfc":
            acc = gemm_pm1(h.reshape(h.shape[0], -1), p["w"])
            h = scale_bias(acc, p["scale"], p["bias"], "col")
        elif L.kind == "fc_f32":
            h = fc_f32_seq(h.reshape(h.shape[0], -1), p["w"], p["bias"], sign_input=True)
        else:
            raise ValueError(L.kind)
        acts.append(h)
    return {"out": h, "acts": acts}
