"""GPU parity: every C-ABI call against the CPU oracle on the same seeded inputs.

int32 accumulators, packed words and requantized uint8 must be bit-exact; the fp32 epilogue must
agree within 1e-6 relative (it is expected to be bit-equal: one fused multiply-add on an exactly
converted integer on both sides).
"""
import itertools

import numpy as np
import pytest
import torch

from paper_2207_08820_amd import inputs

pytestmark = pytest.mark.gpu

UNSIGNED, TWOS, BIPOLAR = 0, 1, 2
DEV = "cuda:0"


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def dev(a):
    return torch.as_tensor(np.ascontiguousarray(a), device=DEV)


def words(t):
    """int32 device words -> uint32 numpy."""
    return t.cpu().numpy().view(np.uint32)


def src_tensor(q, enc):
    """Values as the integer source type the packer accepts: uint8 for unsigned, int8 otherwise."""
    return dev(q.astype(np.uint8)) if enc == UNSIGNED else dev(q.astype(np.int8))


def gpu_gemm(dlrt, a, w, abits, wbits, enc_a, enc_w):
    M, K = a.shape
    N = w.shape[0]
    A = dlrt.dlrt_pack_bitplanes(src_tensor(a, enc_a), abits, enc_a)
    W = dlrt.dlrt_pack_bitplanes(src_tensor(w, enc_w), wbits, enc_w)
    C = dlrt.dlrt_bitserial_gemm(A, W, M, N, K, abits, wbits, enc_a, enc_w)
    torch.cuda.synchronize()
    return C.cpu().numpy()


def gpu_conv(dlrt, x, w, stride, pad, abits, wbits, enc_a, enc_w):
    N, H, W_, Ci = x.shape
    Co, KH, KW, _ = w.shape
    X = dlrt.dlrt_pack_bitplanes(src_tensor(x, enc_a), abits, enc_a)
    Wp = dlrt.dlrt_pack_conv_weights(src_tensor(w, enc_w), wbits, enc_w)
    Y = dlrt.dlrt_bitserial_conv2d(X, Wp, N, H, W_, Ci, Co, KH, KW, stride, pad, abits, wbits, enc_a, enc_w)
    torch.cuda.synchronize()
    return Y.cpu().numpy()


# ---- A2: packing ---------------------------------------------------------------------------------
@pytest.mark.parametrize("K", [1, 31, 32, 33, 64, 100, 576, 1000, 4096])
def test_pack_bitplanes_matches_oracle_bit_for_bit(dlrt, oracle, K):
    r = rng(7000 + K)
    for bits, enc in [(1, UNSIGNED), (2, UNSIGNED), (2, TWOS), (3, TWOS), (4, UNSIGNED), (4, TWOS), (1, BIPOLAR), (1, TWOS)]:
        rows = int(r.integers(1, 70))
        q = inputs.uniform_values((rows, K), bits, enc, int(r.integers(1 << 30)))
        got = dlrt.dlrt_pack_bitplanes(src_tensor(q, enc), bits, enc)
        assert got.shape == (rows, bits, (K + 31) // 32)
        assert np.array_equal(words(got), oracle.pack_bitplanes(q, bits, enc)), (bits, enc, rows)


def test_pack_bitplanes_row_stride_larger_than_K_and_unaligned_rows(dlrt, oracle):
    r = rng(71)
    for ld, K in [(70, 64), (67, 33), (130, 129), (96, 40)]:
        buf = r.integers(0, 4, size=(9, ld)).astype(np.uint8)
        got = dlrt.dlrt_pack_bitplanes(dev(buf), 2, UNSIGNED, K=K)
        assert np.array_equal(words(got), oracle.pack_bitplanes(buf[:, :K].astype(np.int8), 2, UNSIGNED))


def test_pack_bitplanes_nhwc_activations_config2(dlrt, oracle):
    L, x, _, _ = inputs.config2()
    got = dlrt.dlrt_pack_bitplanes(dev(x.astype(np.uint8)), 2, UNSIGNED)
    assert np.array_equal(words(got), oracle.pack_bitplanes(x.reshape(-1, L.Ci), 2, UNSIGNED))


@pytest.mark.parametrize("bits,enc", [(1, TWOS), (2, TWOS), (3, TWOS), (4, TWOS), (2, UNSIGNED), (4, UNSIGNED), (1, BIPOLAR)])
def test_pack_float_source_quantizes_like_the_oracle(dlrt, oracle, bits, enc):
    r = rng(900 + bits * 10 + enc)
    rows, K = 37, 203
    x = r.normal(0, 1.5, size=(rows, K)).astype(np.float32)
    x[0, :8] = [0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 1e9, -1e9]  # ties and saturation
    for scale in (np.array([0.37], np.float32), r.uniform(0.1, 1.0, rows).astype(np.float32)):
        if scale.size == 1:
            x[0, :8] *= scale[0]
        q = oracle.quantize(x, scale, bits, enc)
        if enc == BIPOLAR:
            q = np.where(q > 0, 1, -1).astype(np.int8)
        got = dlrt.dlrt_pack_bitplanes(dev(x), bits, enc, scale=dev(scale))
        assert np.array_equal(words(got), oracle.pack_bitplanes(q, bits, enc))


@pytest.mark.parametrize("Co,k,Ci", [(3, 3, 40), (64, 3, 64), (16, 1, 32), (5, 5, 7), (8, 1, 256)])
def test_pack_conv_weights_matches_oracle(dlrt, oracle, Co, k, Ci):
    for bits, enc in [(2, TWOS), (1, BIPOLAR), (4, TWOS), (3, UNSIGNED)]:
        w = inputs.uniform_values((Co, k, k, Ci), bits, enc, 1234 + Co + Ci)
        got = dlrt.dlrt_pack_conv_weights(src_tensor(w, enc), bits, enc)
        assert np.array_equal(words(got), oracle.pack_conv_weights(w, bits, enc))


# ---- A3: GEMM --------------------------------------------------------------------------------------
def test_gemm_config1(dlrt, oracle):
    c, a, w = inputs.config1()
    got = gpu_gemm(dlrt, a, w, c.abits, c.wbits, c.enc_a, c.enc_w)
    assert got.dtype == np.int32 and np.array_equal(got, oracle.gemm_i32(a, w))


ENC_CASES = [(a, w, ea, ew) for a, w in itertools.product(range(1, 5), repeat=2)
             for ea, ew in ((UNSIGNED, TWOS), (UNSIGNED, UNSIGNED), (TWOS, TWOS), (TWOS, UNSIGNED))] + \
            [(a, 1, ea, BIPOLAR) for a in range(1, 5) for ea in (UNSIGNED, TWOS)]


@pytest.mark.parametrize("M,N,K", [(70, 45, 100), (1, 1, 1), (130, 131, 1056), (33, 257, 576), (200, 40, 2080)])
def test_gemm_all_bit_widths_and_encodings_ragged_shapes(dlrt, oracle, M, N, K):
    """Shapes that are not multiples of any tile, K words not a multiple of 4 or 2, several K chunks."""
    for idx, (abits, wbits, ea, ew) in enumerate(ENC_CASES):
        a = inputs.uniform_values((M, K), abits, ea, 5000 + idx)
        w = inputs.uniform_values((N, K), wbits, ew, 6000 + idx)
        got = gpu_gemm(dlrt, a, w, abits, wbits, ea, ew)
        assert np.array_equal(got, oracle.gemm_i32(a, w)), (abits, wbits, ea, ew)


def test_gemm_closed_forms_on_gpu(dlrt):
    """All-max operands give K * amax * wmax, all-min two's-complement weights -K * amax * 2^(w-1)."""
    M, N, K = 96, 80, 1111
    for abits, wbits in ((1, 1), (2, 2), (3, 3), (4, 4), (2, 4)):
        amax = (1 << abits) - 1
        a = np.full((M, K), amax, np.int8)
        got = gpu_gemm(dlrt, a, np.full((N, K), (1 << wbits) - 1, np.int8), abits, wbits, UNSIGNED, UNSIGNED)
        assert np.all(got == K * amax * ((1 << wbits) - 1))
        got = gpu_gemm(dlrt, a, np.full((N, K), -(1 << (wbits - 1)), np.int8), abits, wbits, UNSIGNED, TWOS)
        assert np.all(got == -K * amax * (1 << (wbits - 1)))


@pytest.mark.parametrize("abits,wbits", inputs.CONFIG5_PAIRS)
def test_gemm_config5_reduced_size_full_compare(dlrt, oracle, abits, wbits):
    c, a, w = inputs.config5(abits, wbits, size=512)
    got = gpu_gemm(dlrt, a, w, abits, wbits, c.enc_a, c.enc_w)
    assert np.array_equal(got, oracle.gemm_i32(a, w))


@pytest.mark.parametrize("abits,wbits,enc_w", [p + (TWOS,) for p in inputs.CONFIG5_PAIRS] + [(1, 1, BIPOLAR)])
def test_gemm_config5_full_size_sampled_rows_and_sum_invariants(dlrt, oracle, abits, wbits, enc_w):
    """4096^3 in the configuration the benchmark times.  The oracle computes 48 sampled rows one by
    one; every other output is covered by the row-sum / column-sum identities, which hold at any size:
    sum_n C[m,n] = a[m,:] . (sum_n w[n,:]) and sum_m C[m,n] = (sum_m a[m,:]) . w[n,:]."""
    c, a, w = inputs.config5(abits, wbits)
    if enc_w == BIPOLAR:
        w = inputs.uniform_values(w.shape, 1, BIPOLAR, inputs.seed_for(5, 1) + 7)
    got = gpu_gemm(dlrt, a, w, abits, wbits, c.enc_a, enc_w)
    rows = rng(55).choice(c.M, size=48, replace=False)
    assert np.array_equal(got[rows], oracle.gemm_i32(a[rows], w))
    a64, w64, g64 = a.astype(np.int64), w.astype(np.int64), got.astype(np.int64)
    assert np.array_equal(g64.sum(axis=1), a64 @ w64.sum(axis=0))
    assert np.array_equal(g64.sum(axis=0), w64 @ a64.sum(axis=0))


# ---- A3: convolution ---------------------------------------------------------------------------------
def test_conv_config2_with_scale_epilogue(dlrt, oracle):
    L, x, w, scale = inputs.config2()
    got = gpu_conv(dlrt, x, w, (1, 1), (1, 1), 2, 2, UNSIGNED, TWOS)
    ref = oracle.conv2d_i32(x, w, (1, 1), (1, 1))
    assert got.shape == (1, 56, 56, 64) and np.array_equal(got, ref)
    y, _ = dlrt.dlrt_epilogue_f32(dev(got), dev(scale))
    y_ref, _ = oracle.epilogue_f32(ref, scale)
    y = y.cpu().numpy()
    assert np.all(np.abs(y - y_ref) <= 1e-6 * np.abs(y_ref))
    assert np.array_equal(y, y_ref)  # expected bit-equal: one correctly rounded fma on each side


CONV_SHAPES = [
    # N, H, W, Ci, Co, k, stride, pad
    (1, 9, 7, 32, 16, 3, 1, 1),     # one word per pixel
    (2, 10, 10, 33, 20, 3, 2, 1),   # ragged channels, batch 2, even size stride 2
    (1, 9, 9, 64, 70, 3, 2, 1),     # odd size stride 2, two words
    (1, 8, 6, 128, 64, 1, 2, 0),    # 1x1 stride 2, four words (16-byte loads)
    (1, 6, 6, 96, 33, 1, 1, 0),     # three words per pixel
    (1, 7, 7, 20, 9, 5, 1, 2),      # 5x5
    (1, 5, 8, 256, 40, 3, 1, 0),    # no padding, eight words
    (3, 4, 4, 512, 130, 3, 1, 1),   # tiny image, deep reduction (several chunks), batch 3
]


@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_conv_edge_shapes_all_encodings(dlrt, oracle, shape):
    N, H, W, Ci, Co, k, stride, pad = shape
    cases = [(2, 2, UNSIGNED, TWOS), (2, 1, UNSIGNED, BIPOLAR), (1, 1, UNSIGNED, TWOS), (4, 4, UNSIGNED, TWOS),
             (3, 2, TWOS, UNSIGNED), (1, 2, UNSIGNED, TWOS), (2, 4, UNSIGNED, TWOS), (3, 3, TWOS, TWOS)]
    for idx, (abits, wbits, ea, ew) in enumerate(cases):
        x = inputs.uniform_values((N, H, W, Ci), abits, ea, 8000 + idx + H)
        w = inputs.uniform_values((Co, k, k, Ci), wbits, ew, 9000 + idx + Ci)
        got = gpu_conv(dlrt, x, w, (stride, stride), (pad, pad), abits, wbits, ea, ew)
        assert np.array_equal(got, oracle.conv2d_i32(x, w, (stride, stride), (pad, pad))), (abits, wbits, ea, ew)


def test_conv_rectangular_stride_and_padding(dlrt, oracle):
    x = inputs.uniform_values((1, 11, 9, 64), 2, UNSIGNED, 4242)
    w = inputs.uniform_values((24, 3, 3, 64), 2, TWOS, 4243)
    got = gpu_conv(dlrt, x, w, (2, 1), (0, 1), 2, 2, UNSIGNED, TWOS)
    assert np.array_equal(got, oracle.conv2d_i32(x, w, (2, 1), (0, 1)))


# ---- A4: epilogue ------------------------------------------------------------------------------------
@pytest.mark.parametrize("rows,C", [(17, 13), (64, 64), (1, 1), (300, 128), (5, 6)])
def test_epilogue_dequant_and_requant(dlrt, oracle, rows, C):
    r = rng(rows * 1000 + C)
    acc = r.integers(-491520, 491520, size=(rows, C)).astype(np.int32)
    scale = r.uniform(1e-4, 1e-1, C).astype(np.float32)
    bias = r.uniform(-3, 3, C).astype(np.float32)
    for b in (None, bias):
        for qbits in (1, 2, 4, 8):
            y, q = dlrt.dlrt_epilogue_f32(dev(acc), dev(scale), None if b is None else dev(b), qbits=qbits)
            y_ref, q_ref = oracle.epilogue_f32(acc, scale, b, qbits=qbits)
            y = y.cpu().numpy()
            assert np.all(np.abs(y - y_ref) <= 1e-6 * np.abs(y_ref))
            assert np.array_equal(y, y_ref)
            assert np.array_equal(q.cpu().numpy(), q_ref)


def test_epilogue_requant_ties_and_single_outputs(dlrt, oracle):
    acc = np.array([[1, 3, 5, 7, -3, 9, 100, 0]], np.int32)
    scale = np.full(8, 0.5, np.float32)
    _, q = dlrt.dlrt_epilogue_f32(dev(acc), dev(scale), want_f32=False, qbits=2)
    assert q.cpu().numpy().tolist() == [[0, 2, 2, 3, 0, 3, 3, 0]]
    y, q = dlrt.dlrt_epilogue_f32(dev(acc), dev(scale))
    assert q is None and y.cpu().numpy().tolist() == [[0.5, 1.5, 2.5, 3.5, -1.5, 4.5, 50.0, 0.0]]


# ---- whole path: chained stacks (configs 3 and 4) -------------------------------------------------------
def calibrate(acc):
    """Per-channel scale and bias that spread a layer's accumulators over the four 2-bit levels (a
    frozen, BN-like affine; computed in float64 from the oracle's accumulators, stored as fp32)."""
    flat = acc.reshape(-1, acc.shape[-1]).astype(np.float64)
    mu, sigma = flat.mean(axis=0), flat.std(axis=0)
    sigma = np.where(sigma > 0, sigma, 1.0)
    scale = (1.0 / sigma).astype(np.float32)
    bias = (1.5 - mu / sigma).astype(np.float32)
    return scale, bias


def run_stack_against_oracle(dlrt, oracle, config, layers, wbits, enc_w):
    from paper_2207_08820_amd.stack import ConvStack

    x0 = inputs.stack_input(config, layers)
    weights = inputs.stack_weights(config, layers, wbits, enc_w)
    # oracle pass, layer by layer, producing the frozen scale / bias arrays both sides use
    ref_acc, ref_q, scales, biases = [], [], [], []
    for i, L in enumerate(layers):
        xin = x0 if L.src < 0 else ref_q[L.src]
        acc = oracle.conv2d_i32(xin.astype(np.int8), weights[i], (L.stride, L.stride), (L.pad, L.pad))
        s, b = calibrate(acc)
        _, q = oracle.epilogue_f32(acc, s, b, qbits=2)
        hist = np.bincount(q.ravel(), minlength=4) / q.size
        assert hist.min() >= 0.05, (L.name, hist)  # the chain must not degenerate to a constant
        ref_acc.append(acc), ref_q.append(q), scales.append(s), biases.append(b)
    stack = ConvStack(layers, weights, scales, biases, 2, wbits, enc_w, device=DEV)
    stack.run(dev(x0.astype(np.uint8)))
    torch.cuda.synchronize()
    for i, L in enumerate(layers):
        assert np.array_equal(stack.layers[i].acc.cpu().numpy(), ref_acc[i]), L.name
        assert np.array_equal(stack.layers[i].q.cpu().numpy(), ref_q[i]), L.name


def test_config3_resnet18_stack_every_layer_bit_exact(dlrt, oracle):
    run_stack_against_oracle(dlrt, oracle, 3, inputs.resnet18_stack(), 2, TWOS)


def test_config4_yolo_style_stack_bipolar_weights_every_layer_bit_exact(dlrt, oracle):
    run_stack_against_oracle(dlrt, oracle, 4, inputs.yolo_style_stack(), 1, BIPOLAR)


# ---- error handling with real buffers ------------------------------------------------------------------
def test_errors_raise_and_launch_nothing(dlrt):
    a = torch.zeros((4, 2, 1), dtype=torch.int32, device=DEV)
    out = torch.full((4, 4), 77, dtype=torch.int32, device=DEV)
    with pytest.raises(dlrt.DlrtError) as e:
        dlrt.dlrt_bitserial_gemm(a, a, 4, 4, 32, 2, 2, BIPOLAR, TWOS, out=out)
    assert e.value.code == 4
    with pytest.raises(dlrt.DlrtError):
        dlrt.dlrt_bitserial_gemm(a, a, 4, 4, 32, 2, 7, UNSIGNED, TWOS, out=out)
    torch.cuda.synchronize()
    assert torch.all(out == 77)
