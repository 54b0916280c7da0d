"""ctypes binding over the C ABI of ``include/dlrt.h``: argument marshalling only.

Every function has the name of the C entry point it calls and takes ``torch`` CUDA tensors
(used here purely as owners of device memory) plus the scalar arguments of the C call; the
kernels are enqueued on torch's current stream.  Nothing is computed in Python, and there is
no fallback: if the HIP library has not been built, ``load()`` raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdlrt_hip.so")

OK = 0
UNSIGNED, TWOS, BIPOLAR = 0, 1, 2
SRC_U8, SRC_I8, SRC_F32 = 0, 1, 2

_lib = None


class ConvProblem(ctypes.Structure):
    """Mirror of dlrt_conv_problem."""
    _fields_ = [("X", ctypes.c_void_p), ("Wp", ctypes.c_void_p), ("scale", ctypes.c_void_p), ("bias", ctypes.c_void_p)] + \
               [(n, ctypes.c_int) for n in ("N", "H", "W", "Ci", "Co", "KH", "KW", "stride_h", "stride_w", "pad_h", "pad_w")] + \
               [("out_acc", ctypes.c_void_p), ("out_f32", ctypes.c_void_p), ("out_q", ctypes.c_void_p),
                ("out_packed", ctypes.c_void_p), ("qbits", ctypes.c_int)]


class DlrtError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = _lib.dlrt_status_string(code).decode() if _lib is not None else "?"
        super().__init__(f"{where}: {msg} (status {code})")


def load():
    """Load libdlrt_hip.so (after torch, so that both share one HIP runtime)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2207_08820_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    i64, i32, vp, sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
    lib.dlrt_packed_words.restype = sz
    lib.dlrt_packed_words.argtypes = [i64, i64, i32]
    lib.dlrt_status_string.restype = ctypes.c_char_p
    lib.dlrt_status_string.argtypes = [i32]
    lib.dlrt_pack_bitplanes.restype = i32
    lib.dlrt_pack_bitplanes.argtypes = [vp, i32, i64, i64, i64, i32, i32, vp, i32, vp, vp]
    lib.dlrt_pack_conv_weights.restype = i32
    lib.dlrt_pack_conv_weights.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp]
    lib.dlrt_pack_conv_weights_per_channel.restype = i32
    lib.dlrt_pack_conv_weights_per_channel.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp]
    lib.dlrt_bitserial_gemm.restype = i32
    lib.dlrt_bitserial_gemm.argtypes = [vp, vp, vp, i64, i64, i64, i32, i32, i32, i32, vp]
    lib.dlrt_bitserial_gemm_fused.restype = i32
    lib.dlrt_bitserial_gemm_fused.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, i32, i32, i32, vp, vp, vp, vp, i32, vp]
    lib.dlrt_bitserial_conv2d.restype = i32
    lib.dlrt_bitserial_conv2d.argtypes = [vp, vp, vp] + [i32] * 15 + [vp]
    lib.dlrt_bitserial_conv2d_fused.restype = i32
    lib.dlrt_bitserial_conv2d_fused.argtypes = [vp, vp, vp, vp] + [i32] * 15 + [vp, vp, vp, vp, i32, i32, i32, vp]
    lib.dlrt_bitserial_conv2d_fused_pair.restype = i32
    lib.dlrt_bitserial_conv2d_fused_pair.argtypes = [ctypes.POINTER(ConvProblem), ctypes.POINTER(ConvProblem), i32, i32, i32,
                                                     i32, vp]
    lib.dlrt_query_plan.restype = i32
    lib.dlrt_query_plan.argtypes = [i64, i64, i64, i32, i32] + [ctypes.POINTER(ctypes.c_int)] * 4
    lib.dlrt_unpacked_gemm_i8.restype = i32
    lib.dlrt_unpacked_gemm_i8.argtypes = [vp, vp, vp, i64, i64, i64, vp]
    lib.dlrt_pack_nibbles.restype = i32
    lib.dlrt_pack_nibbles.argtypes = [vp, i64, i64, vp, vp]
    lib.dlrt_unpacked_gemm_i4.restype = i32
    lib.dlrt_unpacked_gemm_i4.argtypes = [vp, vp, vp, i64, i64, i64, vp]
    lib.dlrt_epilogue_f32.restype = i32
    lib.dlrt_epilogue_f32.argtypes = [vp, vp, vp, i64, i32, vp, vp, i32, vp]
    _lib = lib
    return lib


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous CUDA tensor")
    return t.data_ptr()


def _expect(t, dtype, numel: int, name: str):
    """The C ABI sees pointers only; a buffer of the wrong type or size would become an out-of-bounds access
    on the device, so every tensor is checked here against the elements the call reads or writes."""
    if t is None:
        return
    dtypes = dtype if isinstance(dtype, tuple) else (dtype,)
    if t.dtype not in dtypes:
        raise ValueError(f"{name}: expected dtype {' or '.join(str(d) for d in dtypes)}, got {t.dtype}")
    if t.numel() < numel:
        raise ValueError(f"{name}: the call touches {numel} elements, the tensor has {t.numel()}")


def _cw(n: int) -> int:
    return (n + 31) // 32


def _expect_fused(M: int, N: int, qbits: int, scale, bias, out_acc, out_f32, out_q, out_packed):
    _expect(scale, torch.float32, N, "scale")
    _expect(bias, torch.float32, N, "bias")
    _expect(out_acc, torch.int32, M * N, "out_acc")
    _expect(out_f32, torch.float32, M * N, "out_f32")
    _expect(out_q, torch.uint8, M * N, "out_q")
    _expect(out_packed, torch.int32, M * qbits * _cw(N), "out_packed")


def _check(code: int, where: str):
    if code != OK:
        raise DlrtError(code, where)


_SRC_OF = {torch.uint8: SRC_U8, torch.int8: SRC_I8, torch.float32: SRC_F32}


def dlrt_packed_words(rows: int, K: int, bits: int) -> int:
    return int(load().dlrt_packed_words(rows, K, bits))


def dlrt_pack_bitplanes(src: torch.Tensor, bits: int, enc: int, scale: torch.Tensor | None = None,
                        out: torch.Tensor | None = None, K: int | None = None) -> torch.Tensor:
    """src [..., ld] (uint8 / int8 / float32) -> int32 words [rows, bits, ceil(K/32)], rows = prod of the rest.
    K defaults to the row length ld; a smaller K packs the first K elements of every row."""
    lib = load()
    ld = src.shape[-1]
    K = ld if K is None else K
    rows = src.numel() // ld
    Kw = (K + 31) // 32
    if src.dtype not in _SRC_OF:
        raise ValueError(f"src: expected uint8, int8 or float32, got {src.dtype}")
    if out is None:
        out = torch.empty((rows, bits, Kw), dtype=torch.int32, device=src.device)
    per_row = int(scale is not None and scale.numel() != 1)
    _expect(scale, torch.float32, rows if per_row else 1, "scale")
    _expect(out, torch.int32, rows * bits * Kw, "out")
    _check(lib.dlrt_pack_bitplanes(_ptr(src), _SRC_OF[src.dtype], rows, K, ld, bits, enc, _ptr(scale), per_row,
                                   _ptr(out), _stream()), "dlrt_pack_bitplanes")
    return out


def dlrt_pack_conv_weights(w_ohwi: torch.Tensor, bits: int, enc: int, scale: torch.Tensor | None = None,
                           out: torch.Tensor | None = None) -> torch.Tensor:
    """w [Co, KH, KW, Ci] -> int32 words [Co, bits, KH*KW*ceil(Ci/32)]."""
    lib = load()
    Co, KH, KW, Ci = w_ohwi.shape
    if w_ohwi.dtype not in _SRC_OF:
        raise ValueError(f"w_ohwi: expected uint8, int8 or float32, got {w_ohwi.dtype}")
    if out is None:
        out = torch.empty((Co, bits, KH * KW * ((Ci + 31) // 32)), dtype=torch.int32, device=w_ohwi.device)
    _expect(scale, torch.float32, 1, "scale")
    _expect(out, torch.int32, Co * bits * KH * KW * _cw(Ci), "out")
    _check(lib.dlrt_pack_conv_weights(_ptr(w_ohwi), _SRC_OF[w_ohwi.dtype], Co, KH, KW, Ci, bits, enc, _ptr(scale),
                                      _ptr(out), _stream()), "dlrt_pack_conv_weights")
    return out


def dlrt_pack_conv_weights_per_channel(w_ohwi: torch.Tensor, bits: int, enc: int, scale: torch.Tensor | None = None,
                                       out: torch.Tensor | None = None) -> torch.Tensor:
    """As dlrt_pack_conv_weights with one quantizer scale per output channel (scale [Co], float32 source)."""
    lib = load()
    Co, KH, KW, Ci = w_ohwi.shape
    if scale is not None:
        _expect(scale, torch.float32, Co, "scale")
    if w_ohwi.dtype not in _SRC_OF:
        raise ValueError(f"w_ohwi: expected uint8, int8 or float32, got {w_ohwi.dtype}")
    if out is None:
        out = torch.empty((Co, bits, KH * KW * ((Ci + 31) // 32)), dtype=torch.int32, device=w_ohwi.device)
    _expect(out, torch.int32, Co * bits * KH * KW * _cw(Ci), "out")
    _check(lib.dlrt_pack_conv_weights_per_channel(_ptr(w_ohwi), _SRC_OF[w_ohwi.dtype], Co, KH, KW, Ci, bits, enc,
                                                  _ptr(scale), _ptr(out), _stream()), "dlrt_pack_conv_weights_per_channel")
    return out


def dlrt_bitserial_gemm(A: torch.Tensor, W: torch.Tensor, M: int, N: int, K: int, abits: int, wbits: int,
                        enc_a: int, enc_w: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """Packed A [M, abits, Kw] and W [N, wbits, Kw] -> int32 C [M, N]."""
    lib = load()
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=A.device)
    _expect(A, torch.int32, M * abits * _cw(K), "A")
    _expect(W, torch.int32, N * wbits * _cw(K), "W")
    _expect(out, torch.int32, M * N, "out")
    _check(lib.dlrt_bitserial_gemm(_ptr(A), _ptr(W), _ptr(out), M, N, K, abits, wbits, enc_a, enc_w, _stream()),
           "dlrt_bitserial_gemm")
    return out


def dlrt_bitserial_gemm_fused(A: torch.Tensor, W: torch.Tensor, scale: torch.Tensor | None, bias: torch.Tensor | None,
                              M: int, N: int, K: int, abits: int, wbits: int, enc_a: int, enc_w: int, qbits: int = 2,
                              out_acc: torch.Tensor | None = None, out_f32: torch.Tensor | None = None,
                              out_q: torch.Tensor | None = None, out_packed: torch.Tensor | None = None):
    """One launch: GEMM -> scale/bias -> requant -> bitplanes.  Only the outputs whose buffers are passed are written."""
    _expect(A, torch.int32, M * abits * _cw(K), "A")
    _expect(W, torch.int32, N * wbits * _cw(K), "W")
    _expect_fused(M, N, qbits, scale, bias, out_acc, out_f32, out_q, out_packed)
    _check(load().dlrt_bitserial_gemm_fused(_ptr(A), _ptr(W), _ptr(scale), _ptr(bias), M, N, K, abits, wbits, enc_a, enc_w,
                                            _ptr(out_acc), _ptr(out_f32), _ptr(out_q), _ptr(out_packed), qbits, _stream()),
           "dlrt_bitserial_gemm_fused")


def dlrt_bitserial_conv2d(X: torch.Tensor, Wp: torch.Tensor, N: int, H: int, W: int, Ci: int, Co: int, KH: int,
                          KW: int, stride, pad, abits: int, wbits: int, enc_a: int, enc_w: int,
                          out: torch.Tensor | None = None) -> torch.Tensor:
    """Packed X [N, H, W, abits, Cw] and Wp [Co, wbits, KH*KW*Cw] -> int32 Y [N, Ho, Wo, Co]."""
    lib = load()
    sh, sw = stride
    ph, pw = pad
    Ho = (H + 2 * ph - KH) // sh + 1
    Wo = (W + 2 * pw - KW) // sw + 1
    if out is None:
        out = torch.empty((N, max(Ho, 0), max(Wo, 0), Co), dtype=torch.int32, device=X.device)
    _expect(X, torch.int32, N * H * W * abits * _cw(Ci), "X")
    _expect(Wp, torch.int32, Co * wbits * KH * KW * _cw(Ci), "Wp")
    _expect(out, torch.int32, N * max(Ho, 0) * max(Wo, 0) * Co, "out")
    _check(lib.dlrt_bitserial_conv2d(_ptr(X), _ptr(Wp), _ptr(out), N, H, W, Ci, Co, KH, KW, sh, sw, ph, pw,
                                     abits, wbits, enc_a, enc_w, _stream()), "dlrt_bitserial_conv2d")
    return out


def dlrt_bitserial_conv2d_fused(X: torch.Tensor, Wp: torch.Tensor, scale: torch.Tensor | None,
                                bias: torch.Tensor | None, N: int, H: int, W: int, Ci: int, Co: int, KH: int, KW: int,
                                stride, pad, abits: int, wbits: int, enc_a: int, enc_w: int, qbits: int = 2,
                                out_acc: torch.Tensor | None = None, out_f32: torch.Tensor | None = None,
                                out_q: torch.Tensor | None = None, out_packed: torch.Tensor | None = None,
                                tile_rows: int = 0, ksplit: int = 0):
    """One launch: conv -> scale/bias -> requant -> bitplanes of the result.  Only the outputs whose
    buffers are passed are written; returns nothing."""
    lib = load()
    sh, sw = stride
    ph, pw = pad
    Mo = N * max((H + 2 * ph - KH) // sh + 1, 0) * max((W + 2 * pw - KW) // sw + 1, 0)
    _expect(X, torch.int32, N * H * W * abits * _cw(Ci), "X")
    _expect(Wp, torch.int32, Co * wbits * KH * KW * _cw(Ci), "Wp")
    _expect_fused(Mo, Co, qbits, scale, bias, out_acc, out_f32, out_q, out_packed)
    _check(lib.dlrt_bitserial_conv2d_fused(_ptr(X), _ptr(Wp), _ptr(scale), _ptr(bias), N, H, W, Ci, Co, KH, KW,
                                           sh, sw, ph, pw, abits, wbits, enc_a, enc_w, _ptr(out_acc), _ptr(out_f32),
                                           _ptr(out_q), _ptr(out_packed), qbits, tile_rows, ksplit, _stream()),
           "dlrt_bitserial_conv2d_fused")


def conv_problem(X, Wp, scale, bias, N, H, W, Ci, Co, KH, KW, stride, pad, abits, wbits, qbits=2, out_acc=None,
                 out_f32=None, out_q=None, out_packed=None) -> ConvProblem:
    """Fill a dlrt_conv_problem from tensors (None = NULL); abits / wbits are those the pair call will be
    given, needed here to check the operand sizes."""
    Mo = N * max((H + 2 * pad[0] - KH) // stride[0] + 1, 0) * max((W + 2 * pad[1] - KW) // stride[1] + 1, 0)
    _expect(X, torch.int32, N * H * W * abits * _cw(Ci), "X")
    _expect(Wp, torch.int32, Co * wbits * KH * KW * _cw(Ci), "Wp")
    _expect_fused(Mo, Co, qbits, scale, bias, out_acc, out_f32, out_q, out_packed)
    return ConvProblem(_ptr(X), _ptr(Wp), _ptr(scale), _ptr(bias), N, H, W, Ci, Co, KH, KW, stride[0], stride[1], pad[0],
                       pad[1], _ptr(out_acc), _ptr(out_f32), _ptr(out_q), _ptr(out_packed), qbits)


def dlrt_bitserial_conv2d_fused_pair(first: ConvProblem, second: ConvProblem, abits: int, wbits: int, enc_a: int,
                                     enc_w: int):
    """Two independent fused convolutions of the same bit widths in one launch."""
    _check(load().dlrt_bitserial_conv2d_fused_pair(ctypes.byref(first), ctypes.byref(second), abits, wbits, enc_a, enc_w,
                                                   _stream()), "dlrt_bitserial_conv2d_fused_pair")


def dlrt_query_plan(M: int, N: int, K: int, abits: int, wbits: int) -> dict:
    """Kernel and tile the library would use for an M x N x K contraction (host only)."""
    out = [ctypes.c_int() for _ in range(4)]
    _check(load().dlrt_query_plan(M, N, K, abits, wbits, *[ctypes.byref(o) for o in out]), "dlrt_query_plan")
    kind = ("wave", "block", "rows", "panels")[out[0].value]
    return dict(kernel=kind, block_kernel=kind == "block", tile_rows=out[1].value, tile_cols=out[2].value,
                ksplit=out[3].value)


def dlrt_unpacked_gemm_i8(A: torch.Tensor, W: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """Comparison variant: int8 values A [M, K], W [N, K] (uint8 values below 128 are reinterpreted) -> int32 [M, N]."""
    lib = load()
    M, K = A.shape
    N = W.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=A.device)
    _expect(A, (torch.int8, torch.uint8), M * K, "A")
    _expect(W, (torch.int8, torch.uint8), N * K, "W")
    if W.shape[1] != K:
        raise ValueError(f"W: reduction length {W.shape[1]} differs from A's {K}")
    _expect(out, torch.int32, M * N, "out")
    _check(lib.dlrt_unpacked_gemm_i8(_ptr(A), _ptr(W), _ptr(out), M, N, K, _stream()), "dlrt_unpacked_gemm_i8")
    return out


def dlrt_pack_nibbles(src: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """Comparison variant: int8 values in [-8, 7], [rows, K] -> int32 words [rows, K / 8], one signed nibble per element."""
    lib = load()
    rows, K = src.shape
    if out is None:
        out = torch.empty((rows, K // 8), dtype=torch.int32, device=src.device)
    _expect(src, (torch.int8, torch.uint8), rows * K, "src")
    _expect(out, torch.int32, rows * (K // 8), "out")
    _check(lib.dlrt_pack_nibbles(_ptr(src), rows, K, _ptr(out), _stream()), "dlrt_pack_nibbles")
    return out


def dlrt_unpacked_gemm_i4(A: torch.Tensor, W: torch.Tensor, K: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """Comparison variant: nibble-packed A [M, K / 8], W [N, K / 8] (dlrt_pack_nibbles) -> int32 [M, N]."""
    lib = load()
    M, N = A.shape[0], W.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=A.device)
    _expect(A, torch.int32, M * (K // 8), "A")
    _expect(W, torch.int32, N * (K // 8), "W")
    _expect(out, torch.int32, M * N, "out")
    _check(lib.dlrt_unpacked_gemm_i4(_ptr(A), _ptr(W), _ptr(out), M, N, K, _stream()), "dlrt_unpacked_gemm_i4")
    return out


def dlrt_epilogue_f32(acc: torch.Tensor, scale: torch.Tensor, bias: torch.Tensor | None = None,
                      want_f32: bool = True, qbits: int | None = None, out_f32: torch.Tensor | None = None,
                      out_q: torch.Tensor | None = None):
    """acc [..., C] int32 -> (float32 y or None, uint8 q or None)."""
    lib = load()
    C = acc.shape[-1]
    rows = acc.numel() // C
    if want_f32 and out_f32 is None:
        out_f32 = torch.empty(acc.shape, dtype=torch.float32, device=acc.device)
    if qbits is not None and out_q is None:
        out_q = torch.empty(acc.shape, dtype=torch.uint8, device=acc.device)
    _expect(acc, torch.int32, rows * C, "acc")
    _expect(scale, torch.float32, C, "scale")
    _expect(bias, torch.float32, C, "bias")
    _expect(out_f32, torch.float32, rows * C, "out_f32")
    _expect(out_q, torch.uint8, rows * C, "out_q")
    _check(lib.dlrt_epilogue_f32(_ptr(acc), _ptr(scale), _ptr(bias), rows, C, _ptr(out_f32), _ptr(out_q),
                                 int(qbits or 0), _stream()), "dlrt_epilogue_f32")
    return out_f32, out_q
