"""Host-only checks of the C ABI: the library loads, exports what the header declares, and
rejects bad arguments before any launch (so these run without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2207_08820_amd", "libdlrt_hip.so")
HEADER = os.path.join(ROOT, "include", "dlrt.h")

OK, ERR_NULL, ERR_BITS, ERR_SHAPE, ERR_ENCODING, ERR_ALIGN = 0, 1, 2, 3, 4, 5
UNSIGNED, TWOS, BIPOLAR = 0, 1, 2
FAKE = 0x10000  # 16-byte aligned, never dereferenced: every call below fails validation first
NULL = None


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2207_08820_amd.build import build_library
        build_library()
    lib = ctypes.CDLL(LIB)
    i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
    lib.dlrt_packed_words.restype = ctypes.c_size_t
    lib.dlrt_packed_words.argtypes = [i64, i64, i32]
    lib.dlrt_status_string.restype = ctypes.c_char_p
    lib.dlrt_pack_bitplanes.argtypes = [vp, i32, i64, i64, i64, i32, i32, vp, i32, vp, vp]
    lib.dlrt_pack_conv_weights.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp]
    lib.dlrt_bitserial_gemm.argtypes = [vp, vp, vp, i64, i64, i64, i32, i32, i32, i32, vp]
    lib.dlrt_bitserial_conv2d.argtypes = [vp, vp, vp] + [i32] * 15 + [vp]
    lib.dlrt_epilogue_f32.argtypes = [vp, vp, vp, i64, i32, vp, vp, i32, vp]
    lib.dlrt_bitserial_conv2d_fused.argtypes = [vp, vp, vp, vp] + [i32] * 15 + [vp, vp, vp, vp, i32, i32, i32, vp]
    return lib


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dlrt_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert names == ["dlrt_bitserial_conv2d", "dlrt_bitserial_conv2d_fused", "dlrt_bitserial_conv2d_fused_pair", "dlrt_bitserial_gemm", "dlrt_bitserial_gemm_fused", "dlrt_epilogue_f32", "dlrt_pack_bitplanes",
                     "dlrt_pack_conv_weights", "dlrt_pack_conv_weights_per_channel", "dlrt_pack_nibbles", "dlrt_packed_words", "dlrt_query_plan", "dlrt_status_string",
                     "dlrt_unpacked_gemm_i4", "dlrt_unpacked_gemm_i8"]
    for n in names:
        assert getattr(lib, n) is not None


def test_packed_words_and_status_strings(lib):
    assert lib.dlrt_packed_words(64, 576, 2) == 64 * 2 * 18
    assert lib.dlrt_packed_words(1, 33, 4) == 8
    assert lib.dlrt_packed_words(4096, 4096, 2) * 4 * 16 == 4096 * 4096 * 4  # 2 bits instead of 32
    assert lib.dlrt_packed_words(0, 5, 2) == 0 and lib.dlrt_packed_words(5, 5, 5) == 0
    seen = {lib.dlrt_status_string(c) for c in range(7)}
    assert len(seen) == 7 and lib.dlrt_status_string(0) == b"ok"


def test_gemm_rejects_bad_arguments_before_launch(lib):
    g = lib.dlrt_bitserial_gemm
    assert g(NULL, FAKE, FAKE, 4, 4, 32, 2, 2, UNSIGNED, TWOS, NULL) == ERR_NULL
    assert g(FAKE, FAKE, NULL, 4, 4, 32, 2, 2, UNSIGNED, TWOS, NULL) == ERR_NULL
    assert g(FAKE, FAKE, FAKE, 4, 4, 32, 0, 2, UNSIGNED, TWOS, NULL) == ERR_BITS
    assert g(FAKE, FAKE, FAKE, 4, 4, 32, 2, 5, UNSIGNED, TWOS, NULL) == ERR_BITS
    assert g(FAKE, FAKE, FAKE, 0, 4, 32, 2, 2, UNSIGNED, TWOS, NULL) == ERR_SHAPE
    assert g(FAKE, FAKE, FAKE, 4, 4, -1, 2, 2, UNSIGNED, TWOS, NULL) == ERR_SHAPE
    assert g(FAKE, FAKE, FAKE, 4, 4, 32, 2, 2, BIPOLAR, TWOS, NULL) == ERR_ENCODING  # activations
    assert g(FAKE, FAKE, FAKE, 4, 4, 32, 2, 2, UNSIGNED, BIPOLAR, NULL) == ERR_ENCODING  # wbits != 1
    assert g(FAKE, FAKE, FAKE, 4, 4, 32, 2, 2, UNSIGNED, 7, NULL) == ERR_ENCODING
    assert g(FAKE + 4, FAKE, FAKE, 4, 4, 32, 2, 2, UNSIGNED, TWOS, NULL) == ERR_ALIGN


def test_conv_rejects_bad_arguments_before_launch(lib):
    c = lib.dlrt_bitserial_conv2d
    ok_shape = [1, 8, 8, 32, 16, 3, 3, 1, 1, 1, 1]
    assert c(NULL, FAKE, FAKE, *ok_shape, 2, 2, UNSIGNED, TWOS, NULL) == ERR_NULL
    assert c(FAKE, FAKE, FAKE, *ok_shape, 2, 9, UNSIGNED, TWOS, NULL) == ERR_BITS
    assert c(FAKE, FAKE, FAKE, 1, 8, 8, 32, 16, 3, 3, 0, 1, 1, 1, 2, 2, UNSIGNED, TWOS, NULL) == ERR_SHAPE  # stride 0
    assert c(FAKE, FAKE, FAKE, 1, 2, 2, 32, 16, 5, 5, 1, 1, 0, 0, 2, 2, UNSIGNED, TWOS, NULL) == ERR_SHAPE  # kernel > image
    assert c(FAKE, FAKE, FAKE, *ok_shape, 2, 2, UNSIGNED, BIPOLAR, NULL) == ERR_ENCODING
    assert c(FAKE, FAKE + 8, FAKE, *ok_shape, 2, 2, UNSIGNED, TWOS, NULL) == ERR_ALIGN


def test_fused_conv_rejects_bad_arguments_before_launch(lib):
    f = lib.dlrt_bitserial_conv2d_fused
    shape = [1, 8, 8, 32, 16, 3, 3, 1, 1, 1, 1]
    enc = [2, 2, UNSIGNED, TWOS]
    assert f(FAKE, FAKE, FAKE, NULL, *shape, *enc, NULL, NULL, NULL, NULL, 2, 0, 0, NULL) == ERR_NULL  # no output
    assert f(FAKE, FAKE, NULL, NULL, *shape, *enc, NULL, NULL, FAKE, NULL, 2, 0, 0, NULL) == ERR_NULL  # q without scale
    assert f(FAKE, FAKE, FAKE, NULL, *shape, *enc, NULL, NULL, NULL, FAKE, 5, 0, 0, NULL) == ERR_BITS
    assert f(FAKE, FAKE, FAKE, NULL, *shape, *enc, NULL, NULL, NULL, FAKE + 4, 2, 0, 0, NULL) == ERR_ALIGN
    assert f(FAKE, FAKE, FAKE, NULL, *shape, *enc, FAKE, NULL, NULL, NULL, 2, 24, 0, NULL) == ERR_SHAPE  # no such tile
    assert f(FAKE, FAKE, FAKE, NULL, *shape, *enc, FAKE, NULL, NULL, NULL, 2, 0, 3, NULL) == ERR_SHAPE
    assert f(FAKE, FAKE, FAKE, NULL, *shape, *enc, FAKE, NULL, NULL, NULL, 2, -1, 0, NULL) == ERR_SHAPE
    assert f(FAKE, FAKE, FAKE, NULL, *shape, 2, 2, UNSIGNED, BIPOLAR, FAKE, NULL, NULL, NULL, 2, 0, 0, NULL) == ERR_ENCODING


def test_fused_gemm_rejects_bad_arguments_before_launch(lib):
    i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
    lib.dlrt_bitserial_gemm_fused.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, i32, i32, i32, vp, vp, vp, vp, i32, vp]
    f = lib.dlrt_bitserial_gemm_fused
    assert f(FAKE, FAKE, FAKE, NULL, 4, 4, 32, 2, 2, UNSIGNED, TWOS, NULL, NULL, NULL, NULL, 2, NULL) == ERR_NULL
    assert f(FAKE, FAKE, NULL, NULL, 4, 4, 32, 2, 2, UNSIGNED, TWOS, NULL, FAKE, NULL, NULL, 2, NULL) == ERR_NULL
    assert f(FAKE, FAKE, FAKE, NULL, 4, 4, 32, 2, 2, UNSIGNED, TWOS, NULL, NULL, FAKE, NULL, 0, NULL) == ERR_BITS
    assert f(FAKE, FAKE, FAKE, NULL, 4, 0, 32, 2, 2, UNSIGNED, TWOS, FAKE, NULL, NULL, NULL, 2, NULL) == ERR_SHAPE
    assert f(FAKE, FAKE, FAKE, NULL, 4, 4, 32, 2, 2, UNSIGNED, TWOS, NULL, NULL, NULL, FAKE + 4, 2, NULL) == ERR_ALIGN
    assert f(FAKE, FAKE, FAKE, NULL, 4, 4, 32, 2, 2, TWOS, BIPOLAR, FAKE, NULL, NULL, NULL, 2, NULL) == ERR_ENCODING


def test_unpacked_gemm_rejects_bad_arguments_before_launch(lib):
    lib.dlrt_unpacked_gemm_i8.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int64] * 3 + [ctypes.c_void_p]
    u = lib.dlrt_unpacked_gemm_i8
    assert u(NULL, FAKE, FAKE, 4, 4, 64, NULL) == ERR_NULL
    assert u(FAKE, FAKE, FAKE, 4, 4, 40, NULL) == ERR_SHAPE  # K not a multiple of 16
    assert u(FAKE, FAKE, FAKE, 0, 4, 64, NULL) == ERR_SHAPE
    assert u(FAKE + 8, FAKE, FAKE, 4, 4, 64, NULL) == ERR_ALIGN
    lib.dlrt_unpacked_gemm_i4.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int64] * 3 + [ctypes.c_void_p]
    u4 = lib.dlrt_unpacked_gemm_i4
    assert u4(FAKE, NULL, FAKE, 4, 4, 64, NULL) == ERR_NULL
    assert u4(FAKE, FAKE, FAKE, 4, 4, 48, NULL) == ERR_SHAPE  # K not a multiple of 32
    assert u4(FAKE, FAKE + 8, FAKE, 4, 4, 64, NULL) == ERR_ALIGN
    lib.dlrt_pack_nibbles.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
    pn = lib.dlrt_pack_nibbles
    assert pn(NULL, 4, 64, FAKE, NULL) == ERR_NULL
    assert pn(FAKE, 4, 40, FAKE, NULL) == ERR_SHAPE
    assert pn(FAKE, 0, 64, FAKE, NULL) == ERR_SHAPE
    assert pn(FAKE + 4, 4, 64, FAKE, NULL) == ERR_ALIGN


def test_pack_and_epilogue_reject_bad_arguments_before_launch(lib):
    p = lib.dlrt_pack_bitplanes
    assert p(NULL, 0, 4, 32, 32, 2, UNSIGNED, NULL, 0, FAKE, NULL) == ERR_NULL
    assert p(FAKE, 0, 4, 32, 32, 6, UNSIGNED, NULL, 0, FAKE, NULL) == ERR_BITS
    assert p(FAKE, 0, 4, 32, 16, 2, UNSIGNED, NULL, 0, FAKE, NULL) == ERR_SHAPE  # ld < K
    assert p(FAKE, 0, 4, 32, 32, 2, BIPOLAR, NULL, 0, FAKE, NULL) == ERR_ENCODING  # bipolar needs 1 bit
    assert p(FAKE, 2, 4, 32, 32, 2, TWOS, NULL, 0, FAKE, NULL) == ERR_NULL  # float source without scale
    assert p(FAKE, 9, 4, 32, 32, 2, TWOS, NULL, 0, FAKE, NULL) == ERR_SHAPE  # unknown source type
    assert p(FAKE, 0, 4, 32, 32, 2, UNSIGNED, NULL, 0, FAKE + 4, NULL) == ERR_ALIGN
    w = lib.dlrt_pack_conv_weights
    assert w(FAKE, 1, 0, 3, 3, 8, 2, TWOS, NULL, FAKE, NULL) == ERR_SHAPE
    assert w(FAKE, 1, 4, 3, 3, 8, 1, 5, NULL, FAKE, NULL) == ERR_ENCODING
    lib.dlrt_pack_conv_weights_per_channel.argtypes = lib.dlrt_pack_conv_weights.argtypes
    wc = lib.dlrt_pack_conv_weights_per_channel
    assert wc(FAKE, 2, 4, 3, 3, 8, 2, TWOS, NULL, FAKE, NULL) == ERR_NULL  # float source without scales
    assert wc(FAKE, 1, 4, 3, 0, 8, 2, TWOS, NULL, FAKE, NULL) == ERR_SHAPE
    assert wc(FAKE, 1, 4, 3, 3, 8, 2, BIPOLAR, NULL, FAKE, NULL) == ERR_ENCODING
    e = lib.dlrt_epilogue_f32
    assert e(FAKE, FAKE, NULL, 4, 4, NULL, NULL, 2, NULL) == ERR_NULL  # no output at all
    assert e(FAKE, NULL, NULL, 4, 4, FAKE, NULL, 2, NULL) == ERR_NULL
    assert e(FAKE, FAKE, NULL, 0, 4, FAKE, NULL, 2, NULL) == ERR_SHAPE
    assert e(FAKE, FAKE, NULL, 4, 4, NULL, FAKE, 0, NULL) == ERR_BITS
    assert e(FAKE, FAKE, NULL, 4, 4, NULL, FAKE, 9, NULL) == ERR_BITS


def query(lib, M, N, K, a, w):
    out = [ctypes.c_int() for _ in range(4)]
    lib.dlrt_query_plan.argtypes = [ctypes.c_int64] * 3 + [ctypes.c_int] * 2 + [ctypes.POINTER(ctypes.c_int)] * 4
    assert lib.dlrt_query_plan(M, N, K, a, w, *[ctypes.byref(o) for o in out]) == OK
    return tuple(o.value for o in out)


WAVE, BLOCK, ROWS, PANELS = 0, 1, 2, 3


def test_planner_choices_for_the_benchmark_workloads(lib):
    """Which kernel the workloads of bench.py get (a record of the plan the published numbers were measured
    with, not of the planner's thresholds)."""
    # the 4096^3 sweep: the throughput kernel with tiles of 16 * {4,4,2,2}[bits]
    assert query(lib, 4096, 4096, 4096, 2, 2) == (BLOCK, 64, 64, 1)
    assert query(lib, 4096, 4096, 4096, 1, 1) == (BLOCK, 64, 64, 1)
    assert query(lib, 4096, 4096, 4096, 2, 4) == (BLOCK, 64, 32, 1)
    assert query(lib, 4096, 4096, 4096, 3, 3) == (BLOCK, 32, 32, 1)
    assert query(lib, 4096, 4096, 4096, 4, 4)[0] == BLOCK
    # every layer of the two stacks at batch 1 except the largest YOLO-style ones: the per-wave kernel
    assert query(lib, 64, 64, 576, 2, 2)[0] == WAVE
    assert query(lib, 3136, 64, 576, 2, 2)[:3] == (WAVE, 8, 32)
    assert query(lib, 49, 512, 4608, 2, 2)[0] == WAVE and query(lib, 49, 512, 4608, 2, 2)[3] >= 4  # deep reduction: split over waves
    assert query(lib, 784, 128, 64, 2, 2) == (WAVE, 8, 32, 1)
    # batch 16 / 64: short reductions with many rows take the row kernel, long ones with many rows the panel kernel
    assert query(lib, 409600, 32, 32, 2, 1)[0] == ROWS
    assert query(lib, 409600, 64, 288, 2, 1)[0] == ROWS
    assert query(lib, 200704, 64, 576, 2, 2)[0] == ROWS
    assert query(lib, 50176, 128, 1152, 2, 2) == (PANELS, 64, 8, 1)
    assert query(lib, 12544, 256, 2304, 2, 2) == (PANELS, 64, 8, 2)   # 6.1 tiles per SIMD: two waves share each
    assert query(lib, 3136, 512, 4608, 2, 2)[:3] == (PANELS, 64, 8) and query(lib, 3136, 512, 4608, 2, 2)[3] >= 2
    assert query(lib, 200704, 64, 576, 2, 2) == (ROWS, 64, 16, 1)     # 6.1 waves per SIMD: half-word waves
    assert lib.dlrt_query_plan(0, 4, 32, 2, 2, None, None, None, None) == ERR_SHAPE
    assert lib.dlrt_query_plan(4, 4, 32, 2, 7, None, None, None, None) == ERR_BITS


def test_planner_always_returns_a_tile_the_kernels_have(lib):
    """Properties of any plan, whatever the thresholds are: the tile it names exists in the kernel it names and
    fits that kernel's registers and LDS, and kernels built for many rows are never given few."""
    import random
    r = random.Random(3)
    seen = set()
    for _ in range(3000):
        a, w = r.randint(1, 4), r.randint(1, 4)
        M, N = r.choice([1, 7, 49, 196, 784, 3136, 12544, 25600, 100000, 3000000]), r.choice([1, 16, 32, 64, 100, 256, 512, 4096])
        K = r.choice([1, 32, 64, 100, 288, 500, 544, 576, 1152, 2304, 4608, 40000])
        kind, rows, cols, ks = query(lib, M, N, K, a, w)
        seen.add(kind)
        Kw = -(-K // 32)
        tn = 4 if w <= 2 else 2
        assert kind in (WAVE, BLOCK, ROWS, PANELS)
        if kind == ROWS:    # the whole reduction in a lane's registers; whole output words per wave, or halves
            assert Kw <= 16 or (Kw == 18 and (w <= 2 or a * w <= 8))   # of them where N fills whole words and waves are few
            assert rows == 64 and ks == 1 and (cols in (32, 64, 128) or (cols in (8, 16) and N % 32 == 0))
        elif kind == PANELS:  # accumulators per lane, the wave's weights in LDS, whole 16-byte groups
            assert rows == 64 and 1 <= ks <= 4 and cols in (8, 16, 32)   # ks waves share a tile's reduction
            assert cols * a * w <= 64 and Kw % 4 == 0 and cols * w * (Kw + 15) // 16 * 16 * 4 <= 65536
        elif kind == BLOCK:
            full = 16 * [4, 4, 2, 2][a - 1]
            assert (cols, ks) == (16 * [4, 4, 2, 2][w - 1], 1) and rows in (full, full // 2)
            # a tile is never mostly padding, unless an operand is too large for the per-wave kernel's 32-bit offsets
            assert 2 * N > cols or M * a * Kw * 4 > 2 ** 31 or N * w * Kw * 4 > 2 ** 31
        else:
            if rows == 4 and w <= 2:   # the half tile of narrow weights: two columns per lane, for few-row layers
                tn, tm = 2, 1
                assert -(-M // 8) * -(-N // 32) <= 128
            else:
                tm = rows // (2 * tn)
            assert cols == 32 and rows == 2 * tn * tm and tm in (1, 2, 4) and ks in (1, 2, 4, 8)
            assert tm * tn * a * w <= 72                                     # accumulators per lane
            assert ks * (4 * a * rows + 4 * w * 32) * 16 <= 65536           # LDS of the ks staging regions
            assert ks == 1 or ks <= -(-Kw // 4)                              # no more slices than 4-word steps
        if kind in (ROWS, PANELS):
            assert M >= 1024                                                # one row per lane: lanes would idle
        if M * N <= 64 * 64:
            assert kind == WAVE                                             # a handful of tiles: the latency kernel
    assert seen == {WAVE, BLOCK, ROWS, PANELS}


def test_hints_override_the_plan_or_are_refused(lib):
    """A tile hint selects that kernel whatever the planner would pick; a hint the kernels do not have is an error."""
    f = lib.dlrt_bitserial_conv2d_fused
    enc = [2, 2, UNSIGNED, TWOS]
    big = [64, 28, 28, 128, 128, 3, 3, 1, 1, 1, 1]     # the planner's choice here is the panel kernel
    small = [1, 8, 8, 32, 16, 3, 3, 1, 1, 1, 1]
    for shape, hint, expect in ((small, (8, 1), None), (small, (64, 0), None), (small, (64, 10000), ERR_SHAPE), (small, (64, 3), ERR_SHAPE),
                                (small, (64, 2), ERR_SHAPE),       # 16 columns per wave need whole output words,
                                (small, (128, 0), ERR_SHAPE),     # 32 channels: not whole 16-byte groups per tap
                                (big, (128, 3), ERR_SHAPE), (big, (128, 4), ERR_SHAPE), (big, (12, 1), ERR_SHAPE),
                                (big, (256, 1), ERR_SHAPE),       # 36 words are 3 panels of 12: two waves cannot share them
                                (big, (640, 1), ERR_SHAPE),       # at most four waves share a tile
                                (big, (200, 1), ERR_SHAPE),
                                # 14 GB of activations: beyond the 32-bit offsets of the per-wave kernel
                                ([1, 30000, 30000, 64, 16, 3, 3, 1, 1, 1, 1], (8, 1), ERR_SHAPE),
                                (big, (64, 1), ERR_SHAPE)):       # 36 words do not fit a lane's registers
        if expect is not None:  # refused on the host: nothing is launched, so fake pointers are safe
            assert f(FAKE, FAKE, FAKE, NULL, *shape, *enc, FAKE, NULL, NULL, NULL, 2, hint[0], hint[1], NULL) == expect


def test_binding_exposes_the_same_names():
    from paper_2207_08820_amd import binding
    for n in declared_functions():
        if n != "dlrt_status_string":
            assert callable(getattr(binding, n))


def test_binding_rejects_wrong_sized_or_typed_tensors_before_calling_the_library():
    """The ctypes layer knows the tensors' sizes, the C ABI does not: a buffer that is too small or of the
    wrong type must be refused on the host (on CPU tensors the size check comes before the device check)."""
    import torch
    from paper_2207_08820_amd import binding

    i32 = lambda *shape: torch.zeros(shape, dtype=torch.int32)
    f32 = lambda *shape: torch.zeros(shape, dtype=torch.float32)
    A, W = i32(8, 2, 2), i32(4, 2, 2)   # M = 8, N = 4, K = 64, two planes each
    with pytest.raises(ValueError, match="out"):
        binding.dlrt_bitserial_gemm(A, W, 8, 4, 64, 2, 2, UNSIGNED, TWOS, out=i32(8, 3))
    with pytest.raises(ValueError, match="A"):
        binding.dlrt_bitserial_gemm(A, W, 8, 4, 64, 4, 2, UNSIGNED, TWOS, out=i32(8, 4))      # A packed for 2 bits
    with pytest.raises(ValueError, match="W"):
        binding.dlrt_bitserial_gemm(A, W.to(torch.int64), 8, 4, 64, 2, 2, UNSIGNED, TWOS, out=i32(8, 4))
    with pytest.raises(ValueError, match="out_packed"):
        binding.dlrt_bitserial_gemm_fused(A, W, f32(4), None, 8, 4, 64, 2, 2, UNSIGNED, TWOS, qbits=4, out_packed=i32(8, 2, 1))
    with pytest.raises(ValueError, match="scale"):
        binding.dlrt_bitserial_gemm_fused(A, W, f32(3), None, 8, 4, 64, 2, 2, UNSIGNED, TWOS, out_f32=f32(8, 4))
    with pytest.raises(ValueError, match="out_q"):
        binding.dlrt_bitserial_gemm_fused(A, W, f32(4), None, 8, 4, 64, 2, 2, UNSIGNED, TWOS, out_q=i32(8, 4))
    X, Wp = i32(1 * 6 * 6, 2, 1), i32(16, 2, 9)   # 6 x 6 x 32 image, 16 filters of 3 x 3 x 32
    geom = (1, 6, 6, 32, 16, 3, 3, (1, 1), (1, 1))
    with pytest.raises(ValueError, match="out"):
        binding.dlrt_bitserial_conv2d(X, Wp, *geom, 2, 2, UNSIGNED, TWOS, out=i32(1, 6, 6, 8))
    with pytest.raises(ValueError, match="Wp"):
        binding.dlrt_bitserial_conv2d(X, i32(16, 2, 8), *geom, 2, 2, UNSIGNED, TWOS, out=i32(1, 6, 6, 16))
    with pytest.raises(ValueError, match="out_packed"):
        binding.dlrt_bitserial_conv2d_fused(X, Wp, f32(16), f32(16), *geom, 2, 2, UNSIGNED, TWOS, qbits=2, out_packed=i32(35, 2, 1))
    with pytest.raises(ValueError, match="bias"):
        binding.dlrt_bitserial_conv2d_fused(X, Wp, f32(16), f32(15), *geom, 2, 2, UNSIGNED, TWOS, qbits=2, out_packed=i32(36, 2, 1))
    with pytest.raises(ValueError, match="X"):
        binding.conv_problem(i32(35, 2, 1), Wp, f32(16), None, *geom, 2, 2, out_packed=i32(36, 2, 1))
    with pytest.raises(ValueError, match="out"):
        binding.dlrt_pack_bitplanes(torch.zeros((4, 70), dtype=torch.uint8), 2, UNSIGNED, out=i32(4, 2, 2))  # needs 3 words
    with pytest.raises(ValueError, match="scale"):
        binding.dlrt_pack_bitplanes(f32(4, 64), 2, TWOS, scale=f32(3), out=i32(4, 2, 2))
    with pytest.raises(ValueError, match="src"):
        binding.dlrt_pack_bitplanes(torch.zeros((4, 64), dtype=torch.int16), 2, UNSIGNED)
    with pytest.raises(ValueError, match="scale"):
        binding.dlrt_pack_conv_weights_per_channel(f32(16, 3, 3, 32), 2, TWOS, scale=f32(15))
    with pytest.raises(ValueError, match="out"):
        binding.dlrt_unpacked_gemm_i8(torch.zeros((4, 32), dtype=torch.int8), torch.zeros((6, 32), dtype=torch.int8), out=i32(4, 5))
    with pytest.raises(ValueError, match="scale"):
        binding.dlrt_epilogue_f32(i32(5, 8), f32(7))
    with pytest.raises(ValueError, match="out_q"):
        binding.dlrt_epilogue_f32(i32(5, 8), f32(8), want_f32=False, qbits=2, out_q=torch.zeros((5, 7), dtype=torch.uint8))
