"""Thin ctypes binding of libbnn.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their
data pointers, sizes and the current HIP stream to the C entry point of the same
name, and raises ``BnnError`` on a non-zero status.  No arithmetic of the method
happens in Python, and there is no CPU fallback: if the HIP library has not been
built, loading fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Tuple

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
# BNN_SANITIZE=1 (host-only checks, see build.py): the build whose host code carries ASan / UBSan
LIB_PATH = os.path.join(HERE, "libbnn_san.so" if os.environ.get("BNN_SANITIZE") == "1" else "libbnn.so")

_i64, _i32, _p, _sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t

# name -> (restype, argtypes); the list mirrors include/bnn.h one to one.
SIGNATURES = {
    "bnn_status_str": (ctypes.c_char_p, [_i32]),
    "bnn_packed_words": (_i64, [_i64]),
    "bnn_conv_kwords": (_i64, [_i32, _i32, _i32]),
    "bnn_conv_out_dim": (_i64, [_i64, _i64, _i64, _i64]),
    "bnn_encode": (_i32, [_p, _i64, _i64, _i64, _p, _i64, _p]),
    "bnn_pack_conv_weight": (_i32, [_p, _i32, _i32, _i32, _i32, _p, _p]),
    "bnn_im2col_packed": (_i32, [_p] + [_i32] * 10 + [_p, _p, _sz, _p]),
    "bnn_im2col_workspace_bytes": (_sz, [_i32] * 10),
    "bnn_xnor_gemm": (_i32, [_p, _i64, _p, _i64, _p, _i64, _i64, _i64, _i64, _p]),
    "bnn_xnor_gemm_mfma_i8": (_i32, [_p, _i64, _p, _i64, _p, _i64, _i64, _i64, _i64, _p]),
    "bnn_xnor_gemm_mfma_fp4": (_i32, [_p, _i64, _p, _i64, _p, _i64, _i64, _i64, _i64, _p]),
    "bnn_fp4_row_bytes": (_i64, [_i64]),
    "bnn_expand_fp4": (_i32, [_p, _i64, _i64, _i64, _p, _i64, _p]),
    "bnn_xnor_gemm_mfma_fp4_expanded": (_i32, [_p, _i64, _p, _i64, _p, _i64, _i64, _i64, _i64, _p]),
    "bnn_conv2d_mfma_fp4_expanded": (_i32, [_p, _p] + [_i32] * 11 + [_p, _p]),
    "bnn_control_conv2d_f32": (_i32, [_p, _p] + [_i32] * 11 + [_p, _p]),
    "bnn_xnor_gemm_epilogue": (_i32, [_p, _i64, _p, _i64, _i64, _i64, _i64, _p, _i64, _p, _i64, _p, _p, _i32, _p]),
    "bnn_conv2d": (_i32, [_p, _p] + [_i32] * 11 + [_p, _p, _p, _p, _p, _sz, _p]),
    "bnn_conv2d_workspace_bytes": (_sz, [_i32] * 10),
    "bnn_conv2d_noalloc": (_i32, [_p, _p] + [_i32] * 11 + [_p, _p, _p, _p, _p]),
    "bnn_conv2d_noalloc_max_bytes": (_sz, []),
    "bnn_conv2d_packed": (_i32, [_p, _p] + [_i32] * 12 + [_p, _p, _p, _p, _p, _p]),
    "bnn_conv2d_f32_sign": (_i32, [_p, _p] + [_i32] * 11 + [_p, _p, _p, _p]),
    "bnn_pack_fc_weight_nhwc": (_i32, [_p, _i64, _i32, _i32, _i32, _p, _p]),
    "bnn_maxpool2x2": (_i32, [_p, _i32, _i32, _i32, _i32, _p, _p, _p, _p, _p]),
    "bnn_conv2d_f32": (_i32, [_p, _p] + [_i32] * 11 + [_p, _p, _p, _p]),
    "bnn_fc_f32": (_i32, [_p, _p, _p, _i64, _i64, _i64, _i32, _p, _p]),
}

# include/bnn_testing.h: the same calls with the kernel variant chosen by the caller, the
# kernel-timing hook and the two yardstick kernels.  Tests and bench.py only.
TESTING_SIGNATURES = {
    "bnn_testing_xnor_gemm_epilogue": (_i32, [_p, _i64, _p, _i64, _i64, _i64, _i64, _p, _i64, _p, _i64, _p, _p, _i32,
                                              _i32, _p]),
    "bnn_testing_conv2d": (_i32, [_p, _p] + [_i32] * 11 + [_p, _p, _p, _p, _p, _sz, _i32, _i32, _p]),
    "bnn_testing_conv2d_packed": (_i32, [_p, _p] + [_i32] * 12 + [_p, _p, _p, _p, _p, _i32, _i32, _p]),
    "bnn_testing_xnor_gemm_mfma_fp4_expanded": (_i32, [_p, _i64, _p, _i64, _p, _i64, _i64, _i64, _i64, _i32, _p]),
    "bnn_prof_enable": (_i32, [_i32]),
    "bnn_prof_reset": (_i32, []),
    "bnn_prof_count": (_i64, []),
    "bnn_prof_get": (_i32, [_i64, ctypes.POINTER(_i32), ctypes.POINTER(ctypes.c_float)]),
    "bnn_kernel_name": (ctypes.c_char_p, [_i32]),
    "bnn_valu_peak_probe": (_i32, [_p, _i32, _i32, _i32, _p]),
    "bnn_copy_probe": (_i32, [_p, _p, _sz, _p]),
}

BNN_OK = 0
CH_NONE, CH_ROW, CH_COL = 0, 1, 2

_lib: Optional[ctypes.CDLL] = None


class BnnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        name = lib().bnn_status_str(self.status).decode()
        super().__init__(f"{where} failed: {name} ({self.status})")


def lib() -> ctypes.CDLL:
    """Load libbnn.so (built by paper_1911_04477_amd/build.py).  No fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python paper_1911_04477_amd/build.py` "
                "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in list(SIGNATURES.items()) + list(TESTING_SIGNATURES.items()):
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _check(st: int, where: str) -> None:
    if st != BNN_OK:
        raise BnnError(st, where)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _dev(t: torch.Tensor, dtype: torch.dtype, name: str) -> None:
    if not t.is_cuda or t.dtype != dtype:
        raise TypeError(f"{name} must be a GPU tensor of dtype {dtype}")


def packed_words(K: int) -> int:
    return int(lib().bnn_packed_words(K))


def conv_kwords(C: int, kH: int, kW: int) -> int:
    return int(lib().bnn_conv_kwords(C, kH, kW))


def conv_out_dim(n: int, k: int, s: int, p: int) -> int:
    return int(lib().bnn_conv_out_dim(n, k, s, p))


def bnn_encode(src: torch.Tensor, dst: Optional[torch.Tensor] = None) -> torch.Tensor:
    """src fp32 [rows, K] (row stride = src.stride(0)) -> int64-typed packed words [rows, Kw]."""
    _dev(src, torch.float32, "src")
    assert src.dim() == 2 and src.stride(1) == 1
    rows, K = src.shape
    Kw = packed_words(K)
    if dst is None:
        dst = torch.empty((rows, Kw), dtype=torch.int64, device=src.device)
    _dev(dst, torch.int64, "dst")
    assert dst.stride(1) == 1
    _check(lib().bnn_encode(_ptr(src), rows, K, src.stride(0) if rows > 1 else max(K, src.stride(0)), _ptr(dst),
                            dst.stride(0) if rows > 1 else max(Kw, dst.stride(0)), _stream()), "bnn_encode")
    return dst


def bnn_pack_conv_weight(w: torch.Tensor) -> torch.Tensor:
    _dev(w, torch.float32, "w")
    assert w.dim() == 4 and w.is_contiguous()
    D, C, kH, kW = w.shape
    out = torch.empty((D, conv_kwords(C, kH, kW)), dtype=torch.int64, device=w.device)
    _check(lib().bnn_pack_conv_weight(_ptr(w), D, C, kH, kW, _ptr(out), _stream()), "bnn_pack_conv_weight")
    return out


def im2col_workspace_bytes(x_shape, kH, kW, stride, pad) -> int:
    N, C, H, W = x_shape
    return int(lib().bnn_im2col_workspace_bytes(N, C, H, W, kH, kW, stride[0], stride[1], pad[0], pad[1]))


def bnn_im2col_packed(x: torch.Tensor, kH: int, kW: int, stride=(1, 1), pad=(0, 0),
                      cols: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev(x, torch.float32, "x")
    assert x.dim() == 4 and x.is_contiguous()
    N, C, H, W = x.shape
    geo = (N, C, H, W, kH, kW, stride[0], stride[1], pad[0], pad[1])
    OH, OW = conv_out_dim(H, kH, stride[0], pad[0]), conv_out_dim(W, kW, stride[1], pad[1])
    if cols is None:
        cols = torch.empty((N * OH * OW, conv_kwords(C, kH, kW)), dtype=torch.int64, device=x.device)
    _dev(cols, torch.int64, "cols")
    assert cols.is_contiguous() and cols.numel() == N * OH * OW * conv_kwords(C, kH, kW)
    nbytes = int(lib().bnn_im2col_workspace_bytes(*geo))
    if workspace is None:
        workspace = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=x.device)
    _check(lib().bnn_im2col_packed(_ptr(x), *geo, _ptr(cols), _ptr(workspace), workspace.numel(), _stream()),
           "bnn_im2col_packed")
    return cols


def bnn_xnor_gemm(A: torch.Tensor, B: torch.Tensor, K: int, C: Optional[torch.Tensor] = None,
                  cfg: Optional[int] = None) -> torch.Tensor:
    """A [M, >=Kw], B [N, >=Kw] packed (int64-typed) -> int32 [M, N].
    cfg (tests only): the same call through bnn_testing_xnor_gemm_epilogue on that tile configuration."""
    _dev(A, torch.int64, "A")
    _dev(B, torch.int64, "B")
    M, N = A.shape[0], B.shape[0]
    if C is None:
        C = torch.empty((M, N), dtype=torch.int32, device=A.device)
    _dev(C, torch.int32, "C")
    lda = A.stride(0) if M > 1 else max(A.shape[1], 1)
    ldb = B.stride(0) if N > 1 else max(B.shape[1], 1)
    ldc = C.stride(0) if M > 1 else max(N, 1)
    if cfg is None:
        _check(lib().bnn_xnor_gemm(_ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, M, N, K, _stream()), "bnn_xnor_gemm")
    else:
        _check(lib().bnn_testing_xnor_gemm_epilogue(_ptr(A), lda, _ptr(B), ldb, M, N, K, _ptr(C), ldc, None, 0, None,
                                                    None, CH_NONE, cfg, _stream()), "bnn_testing_xnor_gemm_epilogue")
    return C


def bnn_xnor_gemm_mfma_i8(A: torch.Tensor, B: torch.Tensor, K: int, C: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Ablation: same contract as bnn_xnor_gemm, computed with int8 MFMA."""
    _dev(A, torch.int64, "A")
    _dev(B, torch.int64, "B")
    M, N = A.shape[0], B.shape[0]
    if C is None:
        C = torch.empty((M, N), dtype=torch.int32, device=A.device)
    lda = A.stride(0) if M > 1 else max(A.shape[1], 1)
    ldb = B.stride(0) if N > 1 else max(B.shape[1], 1)
    _check(lib().bnn_xnor_gemm_mfma_i8(_ptr(A), lda, _ptr(B), ldb, _ptr(C), C.stride(0) if M > 1 else max(N, 1), M, N,
                                       K, _stream()), "bnn_xnor_gemm_mfma_i8")
    return C


def bnn_xnor_gemm_mfma_fp4(A: torch.Tensor, B: torch.Tensor, K: int, C: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Ablation: same contract as bnn_xnor_gemm, computed with the 4-bit floating-point MFMA."""
    _dev(A, torch.int64, "A")
    _dev(B, torch.int64, "B")
    M, N = A.shape[0], B.shape[0]
    if C is None:
        C = torch.empty((M, N), dtype=torch.int32, device=A.device)
    lda = A.stride(0) if M > 1 else max(A.shape[1], 1)
    ldb = B.stride(0) if N > 1 else max(B.shape[1], 1)
    _check(lib().bnn_xnor_gemm_mfma_fp4(_ptr(A), lda, _ptr(B), ldb, _ptr(C), C.stride(0) if M > 1 else max(N, 1), M, N,
                                        K, _stream()), "bnn_xnor_gemm_mfma_fp4")
    return C


def bnn_expand_fp4(packed: torch.Tensor, K: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Ablation: packed sign rows [rows, >= ceil(K/64)] int64 -> E2M1 rows [rows, 32 * ceil(K/64)] uint8."""
    _dev(packed, torch.int64, "packed")
    rows = packed.shape[0]
    rb = int(lib().bnn_fp4_row_bytes(K))
    if out is None:
        out = torch.empty((rows, rb), dtype=torch.uint8, device=packed.device)
    src_ld = packed.stride(0) if rows > 1 else max(packed.shape[1], 1)
    dst_ld = out.stride(0) if rows > 1 else max(out.shape[1], 16)
    _check(lib().bnn_expand_fp4(_ptr(packed), rows, K, src_ld, _ptr(out), dst_ld, _stream()), "bnn_expand_fp4")
    return out


def bnn_xnor_gemm_mfma_fp4_expanded(A4: torch.Tensor, B4: torch.Tensor, K: int, C: Optional[torch.Tensor] = None,
                                    tile: Optional[int] = None) -> torch.Tensor:
    """Ablation: the binarized GEMM on operands kept in memory as E2M1 +-1 rows (bnn_expand_fp4)."""
    _dev(A4, torch.uint8, "A4")
    _dev(B4, torch.uint8, "B4")
    M, N = A4.shape[0], B4.shape[0]
    if C is None:
        C = torch.empty((M, N), dtype=torch.int32, device=A4.device)
    lda = A4.stride(0) if M > 1 else max(A4.shape[1], 16)
    ldb = B4.stride(0) if N > 1 else max(B4.shape[1], 16)
    ldc = C.stride(0) if M > 1 else max(N, 1)
    if tile is None:
        _check(lib().bnn_xnor_gemm_mfma_fp4_expanded(_ptr(A4), lda, _ptr(B4), ldb, _ptr(C), ldc, M, N, K, _stream()),
               "bnn_xnor_gemm_mfma_fp4_expanded")
    else:
        _check(lib().bnn_testing_xnor_gemm_mfma_fp4_expanded(_ptr(A4), lda, _ptr(B4), ldb, _ptr(C), ldc, M, N, K, tile,
                                                             _stream()), "bnn_testing_xnor_gemm_mfma_fp4_expanded")
    return C


def bnn_conv2d_mfma_fp4_expanded(x4: torch.Tensor, w4: torch.Tensor, C: int, D: int, kH: int, kW: int, stride=(1, 1),
                                 pad=(0, 0), out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Ablation: x4 [N, H, W, C/2] uint8 (E2M1 codes), w4 [D, kH*kW*C/2] uint8 -> int32 NCHW."""
    _dev(x4, torch.uint8, "x4")
    _dev(w4, torch.uint8, "w4")
    assert x4.dim() == 4 and x4.is_contiguous() and w4.is_contiguous()
    N, H, W, _ = x4.shape
    OH, OW = conv_out_dim(H, kH, stride[0], pad[0]), conv_out_dim(W, kW, stride[1], pad[1])
    if out is None:
        out = torch.empty((N, D, OH, OW), dtype=torch.int32, device=x4.device)
    _check(lib().bnn_conv2d_mfma_fp4_expanded(_ptr(x4), _ptr(w4), N, C, H, W, D, kH, kW, stride[0], stride[1], pad[0],
                                              pad[1], _ptr(out), _stream()), "bnn_conv2d_mfma_fp4_expanded")
    return out


def bnn_control_conv2d_f32(x: torch.Tensor, w: torch.Tensor, stride=(1, 1), pad=(0, 0),
                           out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Control group: the binarized convolution as an fp32 GEMM on sign(x), sign(w)."""
    _dev(x, torch.float32, "x")
    _dev(w, torch.float32, "w")
    N, C, H, W = x.shape
    D, _, kH, kW = w.shape
    OH, OW = conv_out_dim(H, kH, stride[0], pad[0]), conv_out_dim(W, kW, stride[1], pad[1])
    if out is None:
        out = torch.empty((N, D, OH, OW), dtype=torch.float32, device=x.device)
    _check(lib().bnn_control_conv2d_f32(_ptr(x), _ptr(w), N, C, H, W, D, kH, kW, stride[0], stride[1], pad[0], pad[1],
                                        _ptr(out), _stream()), "bnn_control_conv2d_f32")
    return out


def bnn_xnor_gemm_epilogue(A: torch.Tensor, B: torch.Tensor, K: int, scale: torch.Tensor, bias: torch.Tensor,
                           axis: int, want_int: bool = False, out_y: Optional[torch.Tensor] = None,
                           cfg: Optional[int] = None) -> Tuple[Optional[torch.Tensor], torch.Tensor]:
    _dev(A, torch.int64, "A")
    _dev(B, torch.int64, "B")
    M, N = A.shape[0], B.shape[0]
    if out_y is not None:
        _dev(out_y, torch.float32, "out_y")
        assert out_y.shape == (M, N) and out_y.is_contiguous()
    Y = out_y if out_y is not None else torch.empty((M, N), dtype=torch.float32, device=A.device)
    C = torch.empty((M, N), dtype=torch.int32, device=A.device) if want_int else None
    lda = A.stride(0) if M > 1 else max(A.shape[1], 1)
    ldb = B.stride(0) if N > 1 else max(B.shape[1], 1)
    if cfg is None:
        _check(lib().bnn_xnor_gemm_epilogue(_ptr(A), lda, _ptr(B), ldb, M, N, K, _ptr(C), max(N, 1), _ptr(Y), max(N, 1),
                                            _ptr(scale), _ptr(bias), axis, _stream()), "bnn_xnor_gemm_epilogue")
    else:
        _check(lib().bnn_testing_xnor_gemm_epilogue(_ptr(A), lda, _ptr(B), ldb, M, N, K, _ptr(C), max(N, 1), _ptr(Y),
                                                    max(N, 1), _ptr(scale), _ptr(bias), axis, cfg, _stream()),
               "bnn_testing_xnor_gemm_epilogue")
    return C, Y


def conv2d_workspace_bytes(x_shape, kH, kW, stride, pad) -> int:
    N, C, H, W = x_shape
    return int(lib().bnn_conv2d_workspace_bytes(N, C, H, W, kH, kW, stride[0], stride[1], pad[0], pad[1]))


def bnn_conv2d(x: torch.Tensor, w_packed: torch.Tensor, D: int, kH: int, kW: int, stride=(1, 1), pad=(0, 0),
               scale: Optional[torch.Tensor] = None, bias: Optional[torch.Tensor] = None, want_int: bool = True,
               workspace: Optional[torch.Tensor] = None, out_i32: Optional[torch.Tensor] = None,
               out_f32: Optional[torch.Tensor] = None, cfg: Optional[int] = None, lean: Optional[int] = None):
    """Returns (out_i32 or None, out_f32 or None), both NCHW.
    cfg / lean (tests only): the same call through bnn_testing_conv2d."""
    _dev(x, torch.float32, "x")
    _dev(w_packed, torch.int64, "w_packed")
    assert x.dim() == 4 and x.is_contiguous() and w_packed.is_contiguous()
    N, C, H, W = x.shape
    OH, OW = conv_out_dim(H, kH, stride[0], pad[0]), conv_out_dim(W, kW, stride[1], pad[1])
    nbytes = conv2d_workspace_bytes(x.shape, kH, kW, stride, pad)
    if workspace is None:
        workspace = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=x.device)
    if want_int and out_i32 is None:
        out_i32 = torch.empty((N, D, OH, OW), dtype=torch.int32, device=x.device)
    if scale is not None and out_f32 is None:
        out_f32 = torch.empty((N, D, OH, OW), dtype=torch.float32, device=x.device)
    if cfg is None and lean is None:
        _check(lib().bnn_conv2d(_ptr(x), _ptr(w_packed), N, C, H, W, D, kH, kW, stride[0], stride[1], pad[0], pad[1],
                                _ptr(out_i32), _ptr(out_f32), _ptr(scale), _ptr(bias), _ptr(workspace),
                                workspace.numel(), _stream()), "bnn_conv2d")
    else:
        _check(lib().bnn_testing_conv2d(_ptr(x), _ptr(w_packed), N, C, H, W, D, kH, kW, stride[0], stride[1], pad[0],
                                        pad[1], _ptr(out_i32), _ptr(out_f32), _ptr(scale), _ptr(bias),
                                        _ptr(workspace), workspace.numel(), -1 if cfg is None else cfg,
                                        1 if lean is None else lean, _stream()), "bnn_testing_conv2d")
    return out_i32, out_f32


def bnn_conv2d_noalloc(x: torch.Tensor, w_packed: torch.Tensor, D: int, kH: int, kW: int, stride, pad,
                       out_i32: Optional[torch.Tensor], out_f32: Optional[torch.Tensor] = None,
                       scale: Optional[torch.Tensor] = None, bias: Optional[torch.Tensor] = None) -> None:
    """bnn_conv2d without a workspace argument; the caller passes every output buffer, so the call
    allocates nothing on either side of the ABI."""
    _dev(x, torch.float32, "x")
    _dev(w_packed, torch.int64, "w_packed")
    assert x.dim() == 4 and x.is_contiguous() and w_packed.is_contiguous()
    N, C, H, W = x.shape
    _check(lib().bnn_conv2d_noalloc(_ptr(x), _ptr(w_packed), N, C, H, W, D, kH, kW, stride[0], stride[1], pad[0],
                                    pad[1], _ptr(out_i32), _ptr(out_f32), _ptr(scale), _ptr(bias), _stream()),
           "bnn_conv2d_noalloc")


def bnn_conv2d_packed(xp: torch.Tensor, w_packed: torch.Tensor, C: int, D: int, kH: int, kW: int, stride=(1, 1),
                      pad=(0, 0), pool: int = 0, scale: Optional[torch.Tensor] = None,
                      bias: Optional[torch.Tensor] = None, out: str = "packed", out_buf: Optional[torch.Tensor] = None,
                      cfg: Optional[int] = None, lean: Optional[int] = None):
    """xp: packed NHWC [N, H, W, Cw] (int64-typed).  out = "packed" | "i32" | "f32".
    cfg / lean (tests only): the same call through bnn_testing_conv2d_packed."""
    _dev(xp, torch.int64, "x_packed")
    _dev(w_packed, torch.int64, "w_packed")
    assert xp.dim() == 4 and xp.is_contiguous() and w_packed.is_contiguous()
    N, H, W, Cw = xp.shape
    assert Cw == packed_words(C)
    OH, OW = conv_out_dim(H, kH, stride[0], pad[0]), conv_out_dim(W, kW, stride[1], pad[1])
    oi = of = op = None
    if out == "packed":
        op = out_buf if out_buf is not None else torch.empty(
            (N, OH // 2 if pool else OH, OW // 2 if pool else OW, packed_words(D)), dtype=torch.int64, device=xp.device)
    elif out == "i32":
        oi = out_buf if out_buf is not None else torch.empty((N, D, OH, OW), dtype=torch.int32, device=xp.device)
    elif out == "f32":
        of = out_buf if out_buf is not None else torch.empty((N, D, OH, OW), dtype=torch.float32, device=xp.device)
    else:
        raise ValueError(out)
    if cfg is None and lean is None:
        _check(lib().bnn_conv2d_packed(_ptr(xp), _ptr(w_packed), N, C, H, W, D, kH, kW, stride[0], stride[1], pad[0],
                                       pad[1], pool, _ptr(oi), _ptr(of), _ptr(op), _ptr(scale), _ptr(bias), _stream()),
               "bnn_conv2d_packed")
    else:
        _check(lib().bnn_testing_conv2d_packed(_ptr(xp), _ptr(w_packed), N, C, H, W, D, kH, kW, stride[0], stride[1],
                                               pad[0], pad[1], pool, _ptr(oi), _ptr(of), _ptr(op), _ptr(scale),
                                               _ptr(bias), -1 if cfg is None else cfg, 1 if lean is None else lean,
                                               _stream()), "bnn_testing_conv2d_packed")
    return op if op is not None else (oi if oi is not None else of)


def bnn_conv2d_f32_sign(x: torch.Tensor, w: torch.Tensor, scale: torch.Tensor, bias: torch.Tensor, stride=(1, 1),
                        pad=(0, 0), out: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev(x, torch.float32, "x")
    _dev(w, torch.float32, "w")
    N, C, H, W = x.shape
    D, _, kH, kW = w.shape
    OH, OW = conv_out_dim(H, kH, stride[0], pad[0]), conv_out_dim(W, kW, stride[1], pad[1])
    if out is None:
        out = torch.empty((N, OH, OW, packed_words(D)), dtype=torch.int64, device=x.device)
    _check(lib().bnn_conv2d_f32_sign(_ptr(x), _ptr(w), N, C, H, W, D, kH, kW, stride[0], stride[1], pad[0], pad[1],
                                     _ptr(scale), _ptr(bias), _ptr(out), _stream()), "bnn_conv2d_f32_sign")
    return out


def bnn_pack_fc_weight_nhwc(w: torch.Tensor, C: int, H: int, W: int) -> torch.Tensor:
    _dev(w, torch.float32, "w")
    assert w.dim() == 2 and w.is_contiguous() and w.shape[1] == C * H * W
    out = torch.empty((w.shape[0], H * W * packed_words(C)), dtype=torch.int64, device=w.device)
    _check(lib().bnn_pack_fc_weight_nhwc(_ptr(w), w.shape[0], C, H, W, _ptr(out), _stream()),
           "bnn_pack_fc_weight_nhwc")
    return out


def bnn_maxpool2x2(a: torch.Tensor, scale: Optional[torch.Tensor] = None, bias: Optional[torch.Tensor] = None,
                   want_int: bool = True, out_i32=None, out_f32=None):
    _dev(a, torch.int32, "in")
    assert a.dim() == 4 and a.is_contiguous()
    N, D, H, W = a.shape
    if want_int and out_i32 is None:
        out_i32 = torch.empty((N, D, H // 2, W // 2), dtype=torch.int32, device=a.device)
    if scale is not None and out_f32 is None:
        out_f32 = torch.empty((N, D, H // 2, W // 2), dtype=torch.float32, device=a.device)
    _check(lib().bnn_maxpool2x2(_ptr(a), N, D, H, W, _ptr(out_i32), _ptr(out_f32), _ptr(scale), _ptr(bias),
                                _stream()), "bnn_maxpool2x2")
    return out_i32, out_f32


def bnn_conv2d_f32(x: torch.Tensor, w: torch.Tensor, stride=(1, 1), pad=(0, 0), scale=None, bias=None, out=None):
    _dev(x, torch.float32, "x")
    _dev(w, torch.float32, "w")
    N, C, H, W = x.shape
    D, _, kH, kW = w.shape
    OH, OW = conv_out_dim(H, kH, stride[0], pad[0]), conv_out_dim(W, kW, stride[1], pad[1])
    if out is None:
        out = torch.empty((N, D, OH, OW), dtype=torch.float32, device=x.device)
    _check(lib().bnn_conv2d_f32(_ptr(x), _ptr(w), N, C, H, W, D, kH, kW, stride[0], stride[1], pad[0], pad[1],
                                _ptr(scale), _ptr(bias), _ptr(out), _stream()), "bnn_conv2d_f32")
    return out


def bnn_fc_f32(x: torch.Tensor, w: torch.Tensor, bias: Optional[torch.Tensor] = None, sign_input: bool = False,
               out=None):
    _dev(x, torch.float32, "x")
    _dev(w, torch.float32, "w")
    M, K = x.shape
    N = w.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=x.device)
    _check(lib().bnn_fc_f32(_ptr(x), _ptr(w), _ptr(bias), M, K, N, int(sign_input), _ptr(out), _stream()),
           "bnn_fc_f32")
    return out


# ---- measurement helpers (include/bnn_testing.h) -----------------------------------
def prof_enable(on: bool) -> None:
    _check(lib().bnn_prof_enable(int(on)), "bnn_prof_enable")


def prof_reset() -> None:
    _check(lib().bnn_prof_reset(), "bnn_prof_reset")


def prof_records() -> List[Tuple[str, float]]:
    """(kernel name, milliseconds) of every launch recorded since the last reset."""
    L = lib()
    out = []
    kid, ms = _i32(0), ctypes.c_float(0.0)
    for i in range(int(L.bnn_prof_count())):
        _check(L.bnn_prof_get(i, ctypes.byref(kid), ctypes.byref(ms)), "bnn_prof_get")
        out.append((L.bnn_kernel_name(kid.value).decode(), float(ms.value)))
    return out


def bnn_valu_peak_probe(sink: torch.Tensor, blocks: int, iters: int, kind: int = 0) -> None:
    _dev(sink, torch.int32, "sink")
    assert sink.numel() >= blocks * 256
    _check(lib().bnn_valu_peak_probe(_ptr(sink), blocks, iters, kind, _stream()), "bnn_valu_peak_probe")


def bnn_copy_probe(src: torch.Tensor, dst: torch.Tensor) -> None:
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() >= nbytes
    _check(lib().bnn_copy_probe(_ptr(src), _ptr(dst), nbytes, _stream()), "bnn_copy_probe")
